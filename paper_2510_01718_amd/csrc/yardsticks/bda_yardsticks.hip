// Yardsticks for bench.py: what this GPU reaches on the simplest possible kernels, measured in the
// same process and launch mode as the library's kernels, so that a roofline fraction can be read
// against the machine as it runs and not only against the published peak.  No library calls, no
// part of the method: an empty kernel (dispatch floor), a register-resident MFMA loop (matrix-core
// rate under its own power state), and streaming read / write / copy kernels (HBM rate).
// And one model of the large-T kernels' inner loop (stage_model_kernel): the MFMAs, LDS fragment reads,
// global -> LDS DMA loads, load wait and barrier of a 256 x 256 x 64 stage at the lean streaming kernel's
// ratios, with no tile set-up, no epilogue and every load an L2 hit: what the stage structure itself
// reaches on this chip, on operand data of the caller's choice.
// Built into its own shared object (libbda_yardsticks.so); libbda.so does not contain or use it.
// (The stage model borrows the library's inline helpers for buffer descriptors, DMA loads and LDS
// swizzles from bda_gemm_stream.hpp; none of the library's kernels.)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../bda_gemm_stream.hpp"

namespace {

using bda::f32x16;
using bda::u32x4;
using bda::u32x2;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

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

// One workgroup of eight waves (2 x 4, 128 tokens x 64 columns each) per compute unit loops over
// `stages` stages out of two 64 KiB LDS slots: per stage and wave 32 MFMAs of 32x32x16 in four k-steps,
// the 16 + 16 fragment reads that feed them (double-buffered by k-step, the lean kernel's addresses and
// swizzles) and - FULL - eight 1 KiB DMA loads into the other slot spread over the MFMAs of the
// second half, a wait for them and a barrier.  The slots are filled once from `src`, so the operands
// are whatever the caller put there; the loads walk an L2-resident window of `src`.
template <bool FULL>
__global__ __launch_bounds__(512) void stage_model_kernel(const unsigned char* src, uint32_t window, int stages, float* sink)
{
    using namespace bda;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    typedef __attribute__((address_space(3))) unsigned char* lds_u8;
    typedef __attribute__((address_space(3))) const u32x4* lds_u32x4;
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4* lds_s16x4;
    constexpr int SK = 64, RB = 128, TOK_BYTES = 256 * RB, SLOT = 65536;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wt = wave >> 2, wn = wave & 3;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_u8)smem;
    const unsigned char* base = src + (size_t)(blockIdx.x % 8) * window;
    for (int i = threadIdx.x; i < 2 * SLOT / 16; i += 512) ((u32x4*)smem)[i] = ((const u32x4*)base)[i];
    __syncthreads();
    const int l31 = lane & 31, lhi = lane >> 5;
    uint32_t a_tok = lds0 + (uint32_t)((wt * 128 + l31) * RB + ((lhi ^ tok_swz<SK>(l31 & 15)) << 4));
    uint32_t a_wgt[2];
    {
        const int c_s = lane & 15, c_gq = lane >> 4;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int col = wn * 64 + ni * 32 + 16 * (c_gq & 1) + 4 * (c_s & 3);
            const int pc = (col >> 3) ^ wgt_swz(c_s >> 2);
            a_wgt[ni] = lds0 + (uint32_t)(TOK_BYTES + (8 * lhi + (c_s >> 2)) * 512 + (pc << 4) + ((col & 4) << 1));
        }
    }
    auto read_w = [&](int ks, u32x4 (&fw)[2]) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(uintptr_t)(a_wgt[ni] + (16 * ks) * 512));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4)(uintptr_t)(a_wgt[ni] + (16 * ks + 4) * 512));
            const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
            fw[ni] = (u32x4){lo2[0], lo2[1], hi2[0], hi2[1]};
        }
    };
    auto read_t = [&](int ks, u32x4 (&ft)[4]) {
        const uint32_t a = a_tok ^ (uint32_t)(ks << 5);
#pragma unroll
        for (int ti = 0; ti < 4; ++ti) ft[ti] = *(lds_u32x4)(uintptr_t)(a + ti * (32 * RB));
    };
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    u32x4 fw0[2], ft0[4], fw1[2], ft1[4];
    const u32x4 rsrc = make_rsrc_words(base, (int64_t)window);
    uint32_t goff = (uint32_t)((blockIdx.x / 8) * SLOT + wave * 8192);
    const uint32_t voff = (uint32_t)lane * 16u;
    uint32_t slot = 0;
    auto mm8 = [&](u32x4 (&fw)[2], u32x4 (&ft)[4], auto between) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int ti = 0; ti < 4; ti += 2) {
                acc[ni][ti] = BF16::mfma(fw[ni], ft[ti], acc[ni][ti]);
                acc[ni][ti + 1] = BF16::mfma(fw[ni], ft[ti + 1], acc[ni][ti + 1]);
                __builtin_amdgcn_sched_barrier(0);
                between(ni * 2 + ti / 2);
                __builtin_amdgcn_sched_barrier(0);
            }
    };
    auto nothing = [&](int) {};
    read_w(0, fw0);
    read_t(0, ft0);
#pragma unroll 1
    for (int s = 0; s < stages; ++s) {
        const uint32_t so = __builtin_amdgcn_readfirstlane(goff % (window - 2u * SLOT));
        const uint32_t dst = lds0 + ((uint32_t)SLOT - slot) + (uint32_t)wave * 8192u;   // the slot not being read
        read_w(1, fw1); read_t(1, ft1);
        mm8(fw0, ft0, nothing);
        read_w(2, fw0); read_t(2, ft0);
        mm8(fw1, ft1, nothing);
        read_w(3, fw1); read_t(3, ft1);
        a_tok ^= (uint32_t)SLOT; a_wgt[0] ^= (uint32_t)SLOT; a_wgt[1] ^= (uint32_t)SLOT;
        if constexpr (FULL) {
            wait_vmcnt<0>();
            __syncthreads();
        }
        mm8(fw0, ft0, [&](int j) { if constexpr (FULL) lds_dma1s(rsrc, dst + 1024u * j, voff, so + 1024u * j); });
        read_w(0, fw0); read_t(0, ft0);
        mm8(fw1, ft1, [&](int j) { if constexpr (FULL) lds_dma1s(rsrc, dst + 1024u * (4 + j), voff, so + 1024u * (4 + j)); });
        slot = (uint32_t)SLOT - slot;
        goff += (uint32_t)SLOT * 32u;
    }
    wait_vmcnt<0>();                                   // nothing on its way into LDS when the workgroup ends
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
    if (sum == 12345.678f) sink[0] = sum;              // keeps the loop alive without a store
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

// The stage model: 256 workgroups x 8 waves, `stages` stages of 32 MFMAs per wave (256 x 8 x 32 x
// 32768 x stages flop per launch).  `src` holds eight windows of `window_bytes` each (a multiple of
// 16, 256 KiB .. 3 MiB so that they stay in L2): the operand values and the data the loads fetch.
// full != 0: with DMA loads, load wait and barrier; 0: MFMAs and LDS reads only.
extern "C" int bdy_stage_model(const void* src, uint64_t window_bytes, int stages, int full, float* sink, void* stream)
{
    if (!src || !sink || stages <= 0 || window_bytes % 16 || window_bytes < (256u << 10) || window_bytes > (3u << 20)) return -1;
    const int lds = 131072;
    const void* kern = full ? (const void*)stage_model_kernel<true> : (const void*)stage_model_kernel<false>;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return -1;
    if (full) hipLaunchKernelGGL(stage_model_kernel<true>, dim3(256), dim3(512), lds, (hipStream_t)stream, (const unsigned char*)src, (uint32_t)window_bytes, stages, sink);
    else hipLaunchKernelGGL(stage_model_kernel<false>, dim3(256), dim3(512), lds, (hipStream_t)stream, (const unsigned char*)src, (uint32_t)window_bytes, stages, sink);
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
