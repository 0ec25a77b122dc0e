// Internal helpers shared by the translation units of libbda (not part of the public ABI).
#pragma once
#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <functional>
#include <string>

#include "bda.h"

namespace bda {

// Records the message returned by bda_last_error() on this thread and hands back `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// Runs fn(i) for i in [0, n) on up to `max_threads` host threads (0 = hardware concurrency).
void parallel_for(int64_t n, const std::function<void(int64_t)>& fn, int max_threads = 0);

inline size_t dtype_size(int dt)
{
    switch (dt) {
    case BDA_F32: return 4;
    case BDA_F16: return 2;
    case BDA_BF16: return 2;
    case BDA_F64: return 8;
    default: return 0;
    }
}

// Tile policy of the call in progress on this thread (0 = automatic).  The *_ex entry points set it
// for the duration of their call through a PolicyScope; nothing outlives the call.
int tile_policy();
int check_policy(const char* fn, int policy);
class PolicyScope {
public:
    explicit PolicyScope(int policy);
    ~PolicyScope();
    PolicyScope(const PolicyScope&) = delete;
    PolicyScope& operator=(const PolicyScope&) = delete;
private:
    int prev_;
};

// Per-device "the dynamic LDS limit of this kernel has been raised" flags (see set_max_lds).
struct LdsLimitState {
    static constexpr int kMaxDevices = 64;
    std::atomic<bool> done[kMaxDevices] = {};
};

// Byte range [lo, hi) of a rows x cols matrix with leading dimension ld (elements of esz bytes).
struct Span {
    const char* lo;
    const char* hi;
};

inline Span span_of(const void* p, int64_t rows, int64_t cols, int64_t ld, size_t esz)
{
    const char* b = (const char*)p;
    if (!p || rows <= 0 || cols <= 0) return {b, b};
    return {b, b + ((rows - 1) * ld + cols) * (int64_t)esz};
}

inline bool overlaps(Span a, Span b) { return a.lo < b.hi && b.lo < a.hi; }

inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

}  // namespace bda
