// Yardsticks for bench.py: what this GPU reaches on the simplest possible kernels, measured in the
// same process and launch mode as the library's kernels, so that a roofline fraction can be read
// against the machine as it runs and not only against the published peak.  No library calls, no
// part of the method: an empty kernel (dispatch floor), a register-resident MFMA loop (matrix-core
// rate under its own power state), and streaming read / write / copy kernels (HBM rate).
// Built into its own shared object (libbda_yardsticks.so); libbda.so does not contain or use it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ void empty_kernel() {}

// Each wave keeps four independent 32x32 accumulators and issues `iters` rounds of four
// v_mfma_f32_32x32x16 on operands that never leave registers.  Nothing else competes for the pipe.
// RANDOM: every lane holds different pseudo-random operand values of magnitude 0.5 .. 2 (the datapath
// then switches as it does on real data; the board lowers the clock to stay inside its power limit),
// otherwise (nearly) the same value in every lane.
template <bool BF16, bool RANDOM>
__global__ __launch_bounds__(256) void mfma_loop_kernel(int iters, float* sink)
{
    const int lane = threadIdx.x & 63;
    u32x4 a = {0x3C003C00u + lane, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    u32x4 b = {0x38003800u, 0x38003800u + lane, 0x38003800u, 0x38003800u};
    if constexpr (RANDOM) {
        uint32_t x = 0x9E3779B9u * (uint32_t)(blockIdx.x * 256 + threadIdx.x + 1);
        auto next = [&]() {                        // two 16-bit floats: random sign and mantissa, exponent of 0.5 .. 2
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            const uint32_t keep = BF16 ? 0x807F807Fu : 0x83FF83FFu, expo = BF16 ? 0x3F003F00u : 0x38003800u;
            const uint32_t bump = BF16 ? ((x >> 7) & 0x00800080u) : ((x >> 5) & 0x04000400u);
            return ((x & keep) | expo) + bump;
        };
        for (int i = 0; i < 4; ++i) { a[i] = next(); b[i] = next(); }
    }
    f32x16 acc0 = {}, acc1 = {}, acc2 = {}, acc3 = {};
#pragma unroll 1
    for (int i = 0; i < iters; ++i) {
        if constexpr (BF16) {
            const bf16x8 av = __builtin_bit_cast(bf16x8, a), bv = __builtin_bit_cast(bf16x8, b);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc1, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc2, 0, 0, 0);
            acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc3, 0, 0, 0);
        } else {
            const f16x8 av = __builtin_bit_cast(f16x8, a), bv = __builtin_bit_cast(f16x8, b);
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc1, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc2, 0, 0, 0);
            acc3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc3, 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc0[r] + acc1[r] + acc2[r] + acc3[r];
    if (s == 12345.678f) sink[0] = s;          // never true: keeps the loop alive without a store
}

// Streaming kernels: every thread moves 16 bytes per step, the grid strides over the buffer.
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* sink)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t x = 0;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        x ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (x == 0x12345679u) sink[0] = x;         // (the buffers hold other values)
}

template <bool NT>
__global__ __launch_bounds__(256) void write_kernel(u32x4* __restrict__ dst, size_t n16, uint32_t value)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const u32x4 v = {value, value, value, value};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        if constexpr (NT) __builtin_nontemporal_store(v, dst + i);
        else dst[i] = v;
    }
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

int status() { return hipGetLastError() == hipSuccess ? 0 : -1; }

}  // namespace

// All calls: device pointers owned by the caller, asynchronous on `stream`, nothing allocated.
// Return 0, or -1 if the launch was refused.

// grid x threads empty workgroups (the dispatch floor of a launch of that shape)
extern "C" int bdy_empty(int grid, int threads, void* stream)
{
    if (grid <= 0 || threads <= 0 || threads > 1024) return -1;
    hipLaunchKernelGGL(empty_kernel, dim3(grid), dim3(threads), 0, (hipStream_t)stream);
    return status();
}

// workgroups x 4 waves, each `iters` x 4 MFMAs of 32x32x16 (32768 flop each).  bf16 != 0: bf16 operands;
// random_data != 0: pseudo-random operand values instead of one value in every lane.
extern "C" int bdy_mfma_loop(int workgroups, int iters, int bf16, int random_data, float* sink, void* stream)
{
    if (workgroups <= 0 || iters <= 0 || !sink) return -1;
    const dim3 g(workgroups), b(256);
    hipStream_t st = (hipStream_t)stream;
    if (bf16 && random_data) hipLaunchKernelGGL((mfma_loop_kernel<true, true>), g, b, 0, st, iters, sink);
    else if (bf16) hipLaunchKernelGGL((mfma_loop_kernel<true, false>), g, b, 0, st, iters, sink);
    else if (random_data) hipLaunchKernelGGL((mfma_loop_kernel<false, true>), g, b, 0, st, iters, sink);
    else hipLaunchKernelGGL((mfma_loop_kernel<false, false>), g, b, 0, st, iters, sink);
    return status();
}

// bytes must be a multiple of 16 and the pointers 16-byte aligned
extern "C" int bdy_read(const void* src, uint64_t bytes, uint32_t* sink, int workgroups, void* stream)
{
    if (!src || !sink || bytes % 16 || workgroups <= 0) return -1;
    hipLaunchKernelGGL(read_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (size_t)(bytes / 16), sink);
    return status();
}

// nontemporal != 0: streaming stores (the cache policy of the library's result stores); 0: plain stores
extern "C" int bdy_write(void* dst, uint64_t bytes, uint32_t value, int workgroups, int nontemporal, void* stream)
{
    if (!dst || bytes % 16 || workgroups <= 0) return -1;
    if (nontemporal) hipLaunchKernelGGL(write_kernel<true>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst, (size_t)(bytes / 16), value);
    else hipLaunchKernelGGL(write_kernel<false>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst, (size_t)(bytes / 16), value);
    return status();
}

extern "C" int bdy_copy(const void* src, void* dst, uint64_t bytes, int workgroups, void* stream)
{
    if (!src || !dst || bytes % 16 || workgroups <= 0) return -1;
    hipLaunchKernelGGL(copy_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src, (u32x4*)dst, (size_t)(bytes / 16));
    return status();
}
