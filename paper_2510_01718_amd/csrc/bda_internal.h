// Internal helpers shared by the translation units of libbda (not part of the public ABI).
#pragma once
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

}  // namespace bda
