// Device entry point for the gradients of the BD K/V projection: validation, tile grids, launches.
#include <hip/hip_runtime.h>

#include "bda_bwd_kernels.hpp"
#include "bda_internal.h"

namespace bda {
namespace {

// (same contract as set_max_lds of the forward launchers: per device, retried after a failure)
template <typename K>
int allow_lds(K kernel, int bytes, LdsLimitState& state)
{
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return fail(BDA_EHIP, "hipGetDevice: %s", hipGetErrorString(err));
    const bool tracked = dev >= 0 && dev < LdsLimitState::kMaxDevices;
    if (tracked && state.done[dev].load(std::memory_order_acquire)) return BDA_OK;
    err = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (err != hipSuccess) return fail(BDA_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(err));
    if (tracked) state.done[dev].store(true, std::memory_order_release);
    return BDA_OK;
}

int launched()
{
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

template <typename X, typename OutT, int TT, int TN, bool WEIGHT>
int launch_mfma(const BwdArgs& a, hipStream_t st)
{
    static LdsLimitState once;
    constexpr int lds = WEIGHT ? BwdWeightLds<TT, TN>::BYTES : BwdLds<TT, TN>::BYTES;
    const int total = a.m_tiles * a.n_tiles;
    const int grid = kNumXcd * ((total + kNumXcd - 1) / kNumXcd);
    if constexpr (WEIGHT) {
        auto kern = bwd_weight_kernel<X, OutT, TT, TN>;
        if (int rc = allow_lds(kern, lds, once)) return rc;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, st, a);
    } else {
        auto kern = bwd_latent_kernel<X, OutT, TT, TN>;
        if (int rc = allow_lds(kern, lds, once)) return rc;
        hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, st, a);
    }
    return launched();
}

// The largest tile that still gives every compute unit a workgroup; rows x cols = extent of the output.
template <typename X, typename OutT, bool WEIGHT>
int launch_sized(BwdArgs& a, int64_t rows, const int64_t* group_cols, int G, hipStream_t st)
{
    auto grid = [&](int bt, int bn) {
        a.tile_start[0] = 0;
        for (int g = 0; g < G; ++g) a.tile_start[g + 1] = a.tile_start[g] + (int)((group_cols[g] + bn - 1) / bn);
        a.n_tiles = a.tile_start[G];
        a.m_tiles = (int)((rows + bt - 1) / bt);
        return (int64_t)a.m_tiles * a.n_tiles;
    };
    const int policy = tile_policy();   // 1 forces the 128 x 128 tile (testing hook)
    // (64 x 128 tiles were measured too: never faster than 64 x 64, which keeps two workgroups on a
    // compute unit)
    if (grid(128, 128) >= 256 || policy == 1) return launch_mfma<X, OutT, 2, 2, WEIGHT>(a, st);
    grid(64, 64);
    return launch_mfma<X, OutT, 1, 1, WEIGHT>(a, st);
}

template <bool WEIGHT>
int launch_fast(BwdArgs& a, int64_t rows, const int64_t* group_cols, int G, int dtype, int out_dtype, hipStream_t st)
{
    if (dtype == BDA_F16 && out_dtype == BDA_F16) return launch_sized<F16, uint16_t, WEIGHT>(a, rows, group_cols, G, st);
    if (dtype == BDA_F16 && out_dtype == BDA_F32) return launch_sized<F16, float, WEIGHT>(a, rows, group_cols, G, st);
    if (dtype == BDA_BF16 && out_dtype == BDA_BF16) return launch_sized<BF16, uint16_t, WEIGHT>(a, rows, group_cols, G, st);
    if (dtype == BDA_BF16 && out_dtype == BDA_F32) return launch_sized<BF16, float, WEIGHT>(a, rows, group_cols, G, st);
    return fail(BDA_EDTYPE, "unsupported dtype/grad_dtype pair %d/%d", dtype, out_dtype);
}

template <typename InT, typename OutT, bool WEIGHT>
int launch_general_typed(const BwdArgs& a, hipStream_t st)
{
    if constexpr (WEIGHT) hipLaunchKernelGGL((bwd_weight_general_kernel<InT, OutT>), dim3(a.n_tiles, a.m_tiles), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((bwd_latent_general_kernel<InT, OutT>), dim3(a.n_tiles, a.m_tiles), dim3(256), 0, st, a);
    return launched();
}

template <bool WEIGHT>
int launch_general(const BwdArgs& a, int dtype, int out_dtype, hipStream_t st)
{
    if (a.m_tiles > 65535) return fail(BDA_EINVAL, "general kernel: too many row tiles (%d)", a.m_tiles);
    if (dtype == BDA_F32 && out_dtype == BDA_F32) return launch_general_typed<float, float, WEIGHT>(a, st);
    if (dtype == BDA_F16 && out_dtype == BDA_F16) return launch_general_typed<RawF16, RawF16, WEIGHT>(a, st);
    if (dtype == BDA_F16 && out_dtype == BDA_F32) return launch_general_typed<RawF16, float, WEIGHT>(a, st);
    if (dtype == BDA_BF16 && out_dtype == BDA_BF16) return launch_general_typed<RawBF16, RawBF16, WEIGHT>(a, st);
    if (dtype == BDA_BF16 && out_dtype == BDA_F32) return launch_general_typed<RawBF16, float, WEIGHT>(a, st);
    return fail(BDA_EDTYPE, "unsupported dtype/grad_dtype pair %d/%d", dtype, out_dtype);
}

}  // namespace
}  // namespace bda

using namespace bda;

extern "C" int bda_kv_project_backward_ex(const void* c, int64_t ldc, const void* d_out, int64_t ld_dout,
                                          const void* C, int64_t ldC, int64_t T, int d_c, int d_h, int G,
                                          const int* H, const int* basis_offset, void* grad_c, int64_t ld_gc,
                                          void* grad_C, int64_t ld_gC, bda_dtype dtype, bda_dtype grad_dtype,
                                          void* stream, int tile_policy)
{
    clear_error();
    if (int rc = check_policy("bda_kv_project_backward_ex", tile_policy)) return rc;
    PolicyScope scope(tile_policy);
    return bda_kv_project_backward(c, ldc, d_out, ld_dout, C, ldC, T, d_c, d_h, G, H, basis_offset, grad_c, ld_gc,
                                   grad_C, ld_gC, dtype, grad_dtype, stream);
}

extern "C" int bda_kv_project_backward(const void* c, int64_t ldc, const void* d_out, int64_t ld_dout,
                                       const void* C, int64_t ldC, int64_t T, int d_c, int d_h, int G,
                                       const int* H, const int* basis_offset, void* grad_c, int64_t ld_gc,
                                       void* grad_C, int64_t ld_gC, bda_dtype dtype, bda_dtype grad_dtype,
                                       void* stream)
{
    clear_error();
    const char* fn = "bda_kv_project_backward";
    if (dtype != BDA_F32 && dtype != BDA_F16 && dtype != BDA_BF16) return fail(BDA_EDTYPE, "%s: bad dtype %d", fn, dtype);
    if (grad_dtype != dtype && grad_dtype != BDA_F32) return fail(BDA_EDTYPE, "%s: grad_dtype must equal dtype or be BDA_F32 (got %d/%d)", fn, dtype, grad_dtype);
    if (T < 0 || d_c <= 0 || d_h <= 0 || d_h >= d_c) return fail(BDA_EINVAL, "%s: need T >= 0 and 0 < d_h < d_c (T=%lld d_c=%d d_h=%d)", fn, (long long)T, d_c, d_h);
    if (G <= 0 || G > BDA_MAX_GROUPS || !H || !basis_offset) return fail(BDA_EINVAL, "%s: need 1 <= G <= %d and non-NULL H, basis_offset", fn, BDA_MAX_GROUPS);
    int64_t N = 0;
    int64_t cols[BDA_MAX_GROUPS];
    for (int g = 0; g < G; ++g) {
        if (H[g] <= 0) return fail(BDA_EINVAL, "%s: H[%d]=%d", fn, g, H[g]);
        if (basis_offset[g] < 0 || basis_offset[g] > d_c - d_h) return fail(BDA_EINVAL, "%s: basis_offset[%d]=%d outside [0, %d]", fn, g, basis_offset[g], d_c - d_h);
        cols[g] = (int64_t)H[g] * d_h;
        N += cols[g];
    }
    if (!grad_c && !grad_C) return BDA_OK;
    const int K = d_c - d_h;
    if (T > 0 && !d_out) return fail(BDA_EINVAL, "%s: NULL d_out", fn);
    if (ld_dout < N) return fail(BDA_EINVAL, "%s: ld_dout=%lld < N=%lld", fn, (long long)ld_dout, (long long)N);
    if (grad_c && T > 0 && !C) return fail(BDA_EINVAL, "%s: grad_c needs C", fn);
    if (grad_c && (ldC < N || ld_gc < d_c)) return fail(BDA_EINVAL, "%s: leading dimension too small (ldC=%lld ld_gc=%lld, N=%lld d_c=%d)", fn, (long long)ldC, (long long)ld_gc, (long long)N, d_c);
    if (grad_C && T > 0 && !c) return fail(BDA_EINVAL, "%s: grad_C needs c", fn);
    if (grad_C && (ldc < d_c || ld_gC < N)) return fail(BDA_EINVAL, "%s: leading dimension too small (ldc=%lld ld_gC=%lld, d_c=%d N=%lld)", fn, (long long)ldc, (long long)ld_gC, d_c, (long long)N);
    const size_t esz = dtype_size(dtype), gsz = dtype_size(grad_dtype);
    const Span s_c = span_of(grad_C ? c : nullptr, T, d_c, ldc, esz), s_g = span_of(d_out, T, N, ld_dout, esz);
    const Span s_C = span_of(grad_c ? C : nullptr, K, N, ldC, esz);
    const Span s_gc = span_of(grad_c, T, d_c, ld_gc, gsz), s_gC = span_of(grad_C, K, N, ld_gC, gsz);
    if (overlaps(s_gc, s_c) || overlaps(s_gc, s_g) || overlaps(s_gc, s_C) || overlaps(s_gC, s_c) ||
        overlaps(s_gC, s_g) || overlaps(s_gC, s_C) || overlaps(s_gc, s_gC))
        return fail(BDA_EINVAL, "%s: a gradient overlaps an input or the other gradient", fn);

    BwdArgs a{};
    a.c = c; a.g = d_out; a.C = C;
    a.ldc = ldc; a.ldg = ld_dout; a.ldC = ldC;
    a.T = T; a.d_c = d_c; a.d_h = d_h; a.K = K; a.n_groups = G;
    a.col_start[0] = 0;
    for (int g = 0; g < G; ++g) {
        a.col_start[g + 1] = a.col_start[g] + cols[g];
        a.a_off[g] = basis_offset[g];
    }
    hipStream_t st = (hipStream_t)stream;

    const int64_t max_ld = (int64_t)1 << 21;   // 32-bit buffer offsets inside one tile
    bool fast = (dtype == BDA_F16 || dtype == BDA_BF16) && aligned(d_out, 16) && ld_dout % 8 == 0 && ld_dout < max_ld &&
                d_c % 8 == 0 && d_h % 32 == 0 && N < ((int64_t)1 << 30);
    for (int g = 0; g < G; ++g) fast = fast && basis_offset[g] % 8 == 0;

    if (grad_c && T > 0) {
        a.out = grad_c; a.ldo = ld_gc;
        const bool f = fast && aligned(C, 16) && aligned(grad_c, gsz == 4 ? 16 : 8) && ldC % 8 == 0 && ld_gc % 8 == 0 &&
                       ld_gc < max_ld && (int64_t)K * ldC * 2 < ((int64_t)1 << 31);
        int rc;
        if (f) {
            const int64_t latent_cols[1] = {d_c};
            rc = launch_fast<false>(a, T, latent_cols, 1, dtype, grad_dtype, st);
        } else {
            a.n_tiles = (d_c + 63) / 64;
            a.m_tiles = (int)((T + 63) / 64);
            rc = launch_general<false>(a, dtype, grad_dtype, st);
        }
        if (rc) return rc;
    }
    if (grad_C) {
        a.out = grad_C; a.ldo = ld_gC;
        const bool f = fast && (T == 0 || aligned(c, 16)) && aligned(grad_C, gsz == 4 ? 16 : 8) && ldc % 8 == 0 &&
                       ldc < max_ld && ld_gC % 8 == 0 && ld_gC < max_ld;
        if (f) return launch_fast<true>(a, K, cols, G, dtype, grad_dtype, st);
        a.tile_start[0] = 0;
        for (int g = 0; g < G; ++g) a.tile_start[g + 1] = a.tile_start[g] + (int)((cols[g] + 63) / 64);
        a.n_tiles = a.tile_start[G];
        a.m_tiles = (K + 63) / 64;
        return launch_general<true>(a, dtype, grad_dtype, st);
    }
    return BDA_OK;
}
