// Device entry points of libbda: argument validation, tile-grid construction and kernel launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>

#include "bda_gemm_kernels.hpp"
#include "bda_decode.hpp"
#include "bda_gemm_stream.hpp"
#include "bda_gemm_plain.hpp"
#include "bda_gemm_duo.hpp"
#include "bda_internal.h"

namespace bda {
namespace {

// Tile policy of the call in progress on this thread (0 = automatic; set by the *_ex entry points).
thread_local int t_policy = 0;

// Set by the *_plan entry points: the launchers then describe the launch instead of making it.
thread_local bda_launch_plan* t_plan = nullptr;

bool plan_only(const GemmArgs& a, int kernel, int bt, int bn, int workgroups, int threads, int lds, int rounds)
{
    if (!t_plan) return false;
    *t_plan = bda_launch_plan{kernel, bt, bn, a.m_tiles, a.n_tiles, workgroups, threads, lds, rounds,
                              a.lin_slots > 0 ? 1 : 0, a.sm, a.sn};
    return true;
}

// Raises a kernel's dynamic LDS limit on the current device.  `state` remembers, per device, that
// the attribute is set; a failed attempt is reported to its caller and tried again by the next call
// (the attribute is idempotent, so two threads racing through here do no harm).
template <typename K>
int set_max_lds(K kernel, int bytes, LdsLimitState& state)
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

template <typename X, typename OutT, int TT, int TN>
int launch_mfma(GemmArgs& a, hipStream_t st)
{
    static LdsLimitState once;
    constexpr int lds = 2 * (64 * TT + 64 * TN) * kRowBytes;
    auto kern = gemm_mfma_kernel<X, OutT, TT, TN>;
    {
        const int64_t supers = (int64_t)((a.m_tiles + a.sm - 1) / a.sm) * ((a.n_tiles + a.sn - 1) / a.sn);
        if (plan_only(a, BDA_KERNEL_MFMA, 64 * TT, 64 * TN, kNumXcd * a.sm * a.sn, 256, lds, (int)((supers + kNumXcd - 1) / kNumXcd))) return BDA_OK;
    }
    if (int rc = set_max_lds(kern, lds, once)) return rc;
    hipLaunchKernelGGL(kern, dim3(kNumXcd * a.sm * a.sn), dim3(256), lds, st, a);
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

// Streaming kernel: 8 waves, stages of 64, two LDS stages (+ 4 KiB of epilogue staging per wave).
constexpr int kStreamSK = 64, kStreamNS = 2;

// Streaming kernel; `plain` selects its lean variant (every stage of every tile free of per-lane
// decisions: see bda_gemm_plain.hpp), `tok_tile` = 128 or 64 the lean variant with tiles of that many
// tokens (256: the full tile).
template <typename X, typename OutT>
int launch_stream(GemmArgs& a, bool plain, int tok_tile, hipStream_t st)
{
    static LdsLimitState once, once_plain, once_half, once_quarter;
    const bool half_tokens = tok_tile == 128, quarter_tokens = tok_tile == 64;
    constexpr int lds = kStreamNS * (256 * 2 * kStreamSK + kStreamSK * 512) + 8 * 4096;
    constexpr int lds_half = kStreamNS * (128 * 2 * kStreamSK + kStreamSK * 512) + 8 * 4096;
    constexpr int lds_quarter = kStreamNS * (64 * 2 * kStreamSK + kStreamSK * 512) + 8 * 4096;
    auto kern = gemm_stream_kernel<X, OutT, 2, 4, kStreamSK, kStreamNS>;
    auto kern_plain = gemm_plain_kernel<X, OutT, 4>;
    auto kern_half = gemm_plain_kernel<X, OutT, 2>;
    auto kern_quarter = gemm_plain_kernel<X, OutT, 1>;
    a.n_super_m = (a.m_tiles + a.sm - 1) / a.sm;
    a.n_super_n = (a.n_tiles + a.sn - 1) / a.sn;
    a.dh_magic = a.d_h > 0 ? (((uint64_t)1 << 40) + a.d_h - 1) / a.d_h : 0;
    a.lin_slots = 0;
    int64_t total = (int64_t)a.n_super_m * a.n_super_n;      // super-tiles
    int64_t per_die = (total + kNumXcd - 1) / kNumXcd;
    a.rounds = (int)per_die;
    if (plain || half_tokens || quarter_tokens) {
        // Tile-by-tile order (lean kernel only) where it needs fewer rounds than whole super-tiles:
        // small grids whose shape does not factor into 8 dies x (sm x sn) slots.
        const int64_t tiles = (int64_t)a.m_tiles * a.n_tiles;
        const int64_t run = (tiles + kNumXcd - 1) / kNumXcd;                  // tiles per die
        const int slots = (int)std::min<int64_t>(kSlotsPerXcd, run);
        const int64_t lin_rounds = (run + slots - 1) / slots;
        // ... or as many, when the tile grid does not fill whole super-tiles (no idle slots inside a round then)
        const bool ragged = a.m_tiles % a.sm != 0 || a.n_tiles % a.sn != 0;
        if (lin_rounds < a.rounds || (lin_rounds == a.rounds && ragged)) {
            a.sm = a.sn = 1;
            a.n_super_m = a.m_tiles;
            a.n_super_n = a.n_tiles;
            a.lin_slots = slots;
            a.rounds = (int)lin_rounds;
            total = tiles;
            per_die = run;
        }
    }
    a.sn_shift = 0;
    while ((1 << a.sn_shift) < a.sn) ++a.sn_shift;
    for (int x = 0; x < kNumXcd; ++x) {
        const int64_t first = std::min<int64_t>((int64_t)x * per_die, total);
        a.xcd_q0[x] = (int)(first % a.n_super_m);
        a.xcd_r0[x] = (int)(first / a.n_super_m);
        a.xcd_count[x] = (int)std::min<int64_t>(per_die, total - first);
    }
    const int wgs_per_die = a.lin_slots ? a.lin_slots : a.sm * a.sn;
    if (plan_only(a, plain || half_tokens || quarter_tokens ? BDA_KERNEL_LEAN : BDA_KERNEL_STREAM, quarter_tokens ? 64 : half_tokens ? 128 : 256, 256,
                  kNumXcd * wgs_per_die, 512, quarter_tokens ? lds_quarter : half_tokens ? lds_half : lds, a.rounds)) return BDA_OK;
    if (int rc = quarter_tokens ? set_max_lds(kern_quarter, lds_quarter, once_quarter)
                 : half_tokens ? set_max_lds(kern_half, lds_half, once_half)
                 : plain ? set_max_lds(kern_plain, lds, once_plain) : set_max_lds(kern, lds, once)) return rc;
    if (quarter_tokens) hipLaunchKernelGGL(kern_quarter, dim3(kNumXcd * wgs_per_die), dim3(512), lds_quarter, st, a);
    else if (half_tokens) hipLaunchKernelGGL(kern_half, dim3(kNumXcd * wgs_per_die), dim3(512), lds_half, st, a);
    else if (plain) hipLaunchKernelGGL(kern_plain, dim3(kNumXcd * wgs_per_die), dim3(512), lds, st, a);
    else hipLaunchKernelGGL(kern, dim3(kNumXcd * wgs_per_die), dim3(512), lds, st, a);
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

// Two-workgroups-per-compute-unit kernel (bda_gemm_duo.hpp); a's tile grid is 128 x 256.  The eight
// dies split the grid into dn column ranges x dm token ranges (dn dm = 8): the split with the fewest
// rounds of tiles wins, then the one whose dies read the fewest bytes.
template <typename X, typename OutT>
int launch_duo(const GemmArgs& a, hipStream_t st)
{
    static LdsLimitState once_id, once_plain;
    DuoArgs d{};
    d.A = a.A; d.B = a.B; d.D = a.D;
    d.lda = a.lda; d.ldb = a.ldb; d.ldd = a.ldd;
    d.M = a.M; d.K = a.K; d.n_groups = a.n_groups; d.d_h = a.d_h; d.a_skip = a.a_skip;
    for (int g = 0; g <= kMaxGroups; ++g) { d.tile_start[g] = a.tile_start[g]; d.col_start[g] = a.col_start[g]; }
    for (int g = 0; g < kMaxGroups; ++g) d.a_off[g] = a.a_off[g];
    const double tok_tile = 128.0 * (a.K + a.a_skip) * 2.0, wgt_tile = 256.0 * a.K * 2.0;
    const double l2_budget = 3.0 * 1024 * 1024;            // of the die's 4 MiB
    int best_dn = 0;
    int64_t best_rounds = 0;
    double best_cost = 0.0;
    for (int dn = kNumXcd; dn >= 1; dn /= 2) {
        const int dm = kNumXcd / dn;
        const int64_t cx = (a.n_tiles + dn - 1) / dn, mx = (a.m_tiles + dm - 1) / dm;
        const int64_t rounds = (cx * mx + kDuoSlotsPerXcd - 1) / kDuoSlotsPerXcd;
        // a die streams its token tiles once; its column range of the weights once if that stays in
        // its L2, else once per round
        const double w_reads = cx * wgt_tile <= l2_budget ? (double)cx : (double)rounds * std::min<int64_t>(cx, kDuoSlotsPerXcd);
        const double cost = mx * tok_tile + w_reads * wgt_tile;
        if (!best_dn || rounds < best_rounds || (rounds == best_rounds && cost < best_cost * 0.999)) {
            best_dn = dn; best_rounds = rounds; best_cost = cost;
        }
    }
    const int dn = best_dn, dm = kNumXcd / dn;
    for (int x = 0; x < kNumXcd; ++x) {
        const int xn = x % dn, xm = x / dn;
        // nearly equal ranges: the first (tiles % parts) ranges are one longer
        auto range = [](int tiles, int parts, int i, int& first, int& count) {
            const int base = tiles / parts, extra = tiles % parts;
            first = i * base + std::min(i, extra);
            count = base + (i < extra ? 1 : 0);
        };
        range(a.n_tiles, dn, xn, d.die_c0[x], d.die_cx[x]);
        range(a.m_tiles, dm, xm, d.die_m0[x], d.die_mx[x]);
        const int cx = std::max(d.die_cx[x], 1);
        d.die_magic[x] = (((uint64_t)1 << 40) + cx - 1) / cx;
    }
    d.rounds = (int)best_rounds;
    if (t_plan) {
        *t_plan = bda_launch_plan{BDA_KERNEL_DUO, 128, 256, a.m_tiles, a.n_tiles, kNumXcd * kDuoSlotsPerXcd, kDuoThreads,
                                  kDuoLdsBytes, d.rounds, 1, dm, dn};
        return BDA_OK;
    }
    if (a.ident) {
        auto kern = gemm_duo_kernel<X, OutT, true>;
        if (int rc = set_max_lds(kern, kDuoLdsBytes, once_id)) return rc;
        hipLaunchKernelGGL(kern, dim3(kNumXcd * kDuoSlotsPerXcd), dim3(kDuoThreads), kDuoLdsBytes, st, d);
    } else {
        auto kern = gemm_duo_kernel<X, OutT, false>;
        if (int rc = set_max_lds(kern, kDuoLdsBytes, once_plain)) return rc;
        hipLaunchKernelGGL(kern, dim3(kNumXcd * kDuoSlotsPerXcd), dim3(kDuoThreads), kDuoLdsBytes, st, d);
    }
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

// LDS of the 32-column small-T kernel: slice of C, token rows (TOK_LDS), float32 partial sums of the
// four waves (in the token rows' space when there are two token blocks).
template <int NTB, bool TOK_LDS>
int decode_lds_bytes(int K)
{
    const int wgt = ((K + 15) / 16) * 1024, part = NTB * 16384;
    const int tok = TOK_LDS ? ((K + 63) / 64) * NTB * 4096 : 0;
    return (TOK_LDS && NTB == 2) ? wgt + std::max(tok, part) : wgt + tok + part;
}

template <typename X, typename OutT, int NTB, bool TOK_LDS>
int launch_decode_blocks(GemmArgs& a, hipStream_t st)
{
    static LdsLimitState once;
    auto kern = kv_decode_kernel<X, OutT, NTB, TOK_LDS>;
    const int lds = decode_lds_bytes<NTB, TOK_LDS>(a.K);
    const int per_xcd = (a.n_tiles + kNumXcd - 1) / kNumXcd;
    if (plan_only(a, BDA_KERNEL_DECODE, 32 * NTB, 32, kNumXcd * per_xcd * a.m_tiles, 256, lds, 1)) return BDA_OK;
    if (int rc = set_max_lds(kern, decode_lds_bytes<NTB, TOK_LDS>(TOK_LDS ? kDecodeTokLdsMaxK : kDecodeMaxK), once)) return rc;
    hipLaunchKernelGGL(kern, dim3(kNumXcd * per_xcd * a.m_tiles), dim3(256), lds, st, a);
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

template <typename X, typename OutT, int NTB, int CW>
int launch_decode_wide_blocks(GemmArgs& a, hipStream_t st)
{
    static LdsLimitState once;
    auto kern = kv_decode_wide_kernel<X, OutT, NTB, CW>;
    constexpr int kspr = CW == 128 ? 1 : 2;                 // k-steps per request round
    const int nks = (a.K + 15) / 16;
    const int lds = ((nks + kspr - 1) / kspr) * 4096 + ((a.K + 63) / 64) * NTB * 4096;   // slice of C, token rows
    const int per_xcd = (a.n_tiles + kNumXcd - 1) / kNumXcd;
    if (plan_only(a, BDA_KERNEL_DECODE, 32 * NTB, CW, kNumXcd * per_xcd * a.m_tiles, 256, lds, 1)) return BDA_OK;
    if (int rc = set_max_lds(kern, (kDecodeWideMaxKS / kspr) * 4096 + (kDecodeWideMaxKS / 4) * NTB * 4096, once)) return rc;
    hipLaunchKernelGGL(kern, dim3(kNumXcd * per_xcd * a.m_tiles), dim3(256), lds, st, a);
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

// 128-column slices up to 64 tokens, 64-column slices (four token blocks) up to 128.
template <typename X, typename OutT>
int launch_decode_wide(GemmArgs& a, hipStream_t st)
{
    if (a.M <= 32) return launch_decode_wide_blocks<X, OutT, 1, 128>(a, st);
    if (a.M <= 64) return launch_decode_wide_blocks<X, OutT, 2, 128>(a, st);
    return launch_decode_wide_blocks<X, OutT, 4, 64>(a, st);
}

// One block of 32 token rows per workgroup up to 32 tokens, two up to 64, four up to 128.
template <typename X, typename OutT>
int launch_decode(GemmArgs& a, hipStream_t st)
{
    // Token rows through LDS for 33 .. 64 tokens (measured, V2-Lite shape, us: 64 tokens 5.2 against 5.6
    // with fragments from global memory; 32 tokens level; 1 .. 8 tokens 4.4-4.5 against 4.0-4.1: there
    // the extra wait-for-everything costs more than the cheaper loads save).
    if (a.M <= 32) return launch_decode_blocks<X, OutT, 1, false>(a, st);
    if (a.M <= 64) return a.K <= kDecodeTokLdsMaxK ? launch_decode_blocks<X, OutT, 2, true>(a, st) : launch_decode_blocks<X, OutT, 2, false>(a, st);
    return launch_decode_blocks<X, OutT, 4, false>(a, st);
}

template <typename InT, typename OutT>
int launch_general(GemmArgs& a, int64_t N_total, hipStream_t st)
{
    if (plan_only(a, BDA_KERNEL_GENERAL, 64, 64, a.n_tiles * a.m_tiles, 256, 2 * 16 * 65 * 4, 1)) return BDA_OK;
    hipLaunchKernelGGL((gemm_general_kernel<InT, OutT>), dim3(a.n_tiles, a.m_tiles), dim3(256), 0, st, a, N_total);
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "kernel launch: %s", hipGetErrorString(err));
}

// Fills the per-group tile tables for column tiles of width bn and token tiles of height bt.
void build_tiles(GemmArgs& a, int G, const int64_t* group_cols, int bt, int bn)
{
    a.n_groups = G;
    a.tile_start[0] = 0;
    a.col_start[0] = 0;
    for (int g = 0; g < G; ++g) {
        a.tile_start[g + 1] = a.tile_start[g] + (int)((group_cols[g] + bn - 1) / bn);
        a.col_start[g + 1] = a.col_start[g] + group_cols[g];
    }
    a.n_tiles = a.tile_start[G];
    a.m_tiles = (int)((a.M + bt - 1) / bt);
}

// Shape of the block of tiles one die works on at a time: sm x sn = slots (workgroups per die).  A die
// takes a contiguous run of super-tiles, numbered down the token dimension first, so within a run
// every super-tile brings sm new token tiles, and the sn weight tiles of a column of super-tiles
// stay in the die's L2 while they fit.  Among the shapes that fit the tile grid, the one that makes
// a die read the fewest bytes wins (for the V3 shape 2 x 16: a die then owns one 4096-column block
// of the weights, 3 MiB, and reads the latent once instead of twice).  A small tile grid gets fewer
// slots, so that there are at least as many super-tiles as dies and every die (and its share of
// the memory channels) takes part.
void choose_super(GemmArgs& a, int max_slots, int bt, int bn)
{
    auto pow2ceil = [](int v) { int p = 1; while (p < v) p *= 2; return p; };
    const int mcap = pow2ceil(a.m_tiles), ncap = pow2ceil(a.n_tiles);
    const double tok_tile = (double)bt * (a.K + a.a_skip) * 2.0, wgt_tile = (double)bn * a.K * 2.0;
    const double l2_budget = 3.0 * 1024 * 1024;            // of the die's 4 MiB
    for (int slots = max_slots;; slots /= 2) {
        int best_sm = 0;
        double best_cost = 0.0;
        for (int sm = 1; sm <= slots; sm *= 2) {
            const int sn = slots / sm;
            if ((sm > mcap && sm > 1) || (sn > ncap && sn > 1)) continue;   // no slots for tiles that do not exist
            const int64_t nsm = (a.m_tiles + sm - 1) / sm, nsn = (a.n_tiles + sn - 1) / sn;
            const int64_t total = nsm * nsn;
            if (total < kNumXcd && slots > 1) continue;
            const int64_t per_die = (total + kNumXcd - 1) / kNumXcd;
            const int64_t passes = (per_die + nsm - 1) / nsm;              // columns of super-tiles a die touches
            const double w_reads = sn * wgt_tile <= l2_budget ? (double)passes * sn : (double)per_die * sn;
            const double cost = (double)per_die * sm * tok_tile + w_reads * wgt_tile;
            if (best_sm == 0 || cost < best_cost * 0.999) { best_sm = sm; best_cost = cost; }
        }
        if (best_sm || slots == 1) {
            a.sm = best_sm ? best_sm : 1;
            a.sn = slots / a.sm;
            return;
        }
    }
}

// Common launcher.  a.A/B/D, lda/ldb/ldd, M, K, d_h, a_skip, ident and a_off[] are set by the caller.
// Shape conditions of the lean streaming kernel (nothing in any stage depends on the lane: see
// bda_gemm_plain.hpp) beyond those of the fast path: stages of 64 along K and along the window, whole
// 256-column tiles, at least three stages per tile, sizes within the kernel's 24-bit column arithmetic.
bool lean_kernel_applies(const GemmArgs& a, int G, const int64_t* group_cols)
{
    bool ok = a.K % 64 == 0 && a.K >= 64 && (!a.ident || a.d_h % 64 == 0) && a.d_h < (1 << 16);
    for (int g = 0; g < G; ++g) ok = ok && group_cols[g] % 256 == 0 && group_cols[g] < (1 << 24);
    const int id_width = (a.d_h % 256) == 0 ? 256 : a.d_h;                      // window columns a 256-column tile needs
    const int id_stages = a.ident ? (id_width + 127) / 128 : 0;                 // double-width identity stages
    return ok && a.K / 64 + id_stages >= 3;
}

int run_gemm(GemmArgs& a, int G, const int64_t* group_cols, int dtype, int out_dtype, hipStream_t st)
{
    int64_t N_total = 0;
    for (int g = 0; g < G; ++g) N_total += group_cols[g];
    if (a.M == 0 || N_total == 0) return BDA_OK;

    bool fast = (dtype == BDA_F16 || dtype == BDA_BF16) && a.K > 0;
    const size_t out_sz = dtype_size(out_dtype);
    fast = fast && aligned(a.A, 16) && aligned(a.B, 16) && aligned(a.D, out_sz == 4 ? 16 : 8);
    const bool packed = a.ldb == 0;                          // C in the layout of bda_pack_weights: small-T kernels only
    fast = fast && a.lda % 8 == 0 && a.ldb % 8 == 0 && a.ldd % 8 == 0 && a.K % 8 == 0 && a.a_skip % 8 == 0;
    const bool ident_tiles = !a.ident || a.d_h % 32 == 0;   // one 32-column MFMA tile never straddles two heads
    const bool ident_vec = !a.ident || a.d_h % 8 == 0;
    // 32-bit buffer offsets: a 256-row tile must span less than 2 GiB in each operand
    const int64_t max_ld = (int64_t)1 << 21;
    fast = fast && a.lda < max_ld && a.ldd < max_ld && a.ldb < max_ld && (int64_t)a.K * a.ldb * 2 < ((int64_t)1 << 31);
    for (int g = 0; g < G; ++g) fast = fast && a.a_off[g] % 8 == 0 && group_cols[g] % 8 == 0;

    // Small-T kernels (policy 5 forces the wide-slice one wherever it applies and otherwise acts as 0).
    // Measured on cold weights, K = 384, us.  Up to 64 tokens: with 32-column slices the time grows
    // with the number of workgroups per compute unit, so beyond about 20 k columns one workgroup per
    // 128 columns wins (N = 32768: 9.1-10.4 against 12.5-17), below it loses to the finer split
    // (N = 4096: 6.4-7.4 against 4.0-5.4).  65 .. 128 tokens: the 32-column kernel with four token
    // blocks while every slice has a compute unit of its own (N = 4096: 5.8-7.3 against 10.6 with
    // 128-token tiles), then 64-column slices while those have (N = 12288 .. 16384: 8.4-9.4 against
    // 10.7-11.0), the tiles beyond (N = 24576: 11.3 against 15-16).
    // Can the two-workgroups-per-compute-unit kernel take this launch (the lean kernel's preconditions
    // with stages of 32 and identity slices of 64- or 128-wide heads)?  Policy 6 asks for it wherever
    // it can and otherwise acts as 0.
    bool duo_ok = fast && a.K % 32 == 0 && a.K >= 64 && (!a.ident || a.d_h == 64 || a.d_h == 128);
    {
        int64_t nt256 = 0;
        for (int g = 0; g < G; ++g) { duo_ok = duo_ok && group_cols[g] % 256 == 0; nt256 += (group_cols[g] + 255) / 256; }
        duo_ok = duo_ok && ((a.M + 127) / 128) * nt256 < ((int64_t)1 << 24);
    }
    const int policy0 = (t_policy == 6 && !duo_ok) ? 0 : t_policy;
    const bool small_policy = policy0 == 0 || policy0 == 5;
    int64_t n_slices128 = 0, n_slices64 = 0, n_slices32 = 0;
    for (int g = 0; g < G; ++g) {
        n_slices128 += (group_cols[g] + 127) / 128;
        n_slices64 += (group_cols[g] + 63) / 64;
        n_slices32 += (group_cols[g] + 31) / 32;
    }
    // More than 128 tokens are cut into token tiles of 128 while all the workgroups still fit the chip at once
    // (T = 256, N = 4096: 256 workgroups).
    const int64_t tok_tiles = (a.M + kDecodeMaxT - 1) / kDecodeMaxT;
    const bool fits32 = n_slices32 * tok_tiles <= 256, fits64 = n_slices64 * tok_tiles <= 256;
    // More than 128 tokens where the 32-column slices no longer fit: one round of the lean kernel's 64-token
    // tiles, where that kernel applies, beats 64-column slices with token tiles (N = 4096, 384 / 512 tokens:
    // 8.6 / 8.8 against 8.9 / 9.3 us).
    bool lean64 = policy0 == 0 && !packed && a.M > kDecodeMaxT && fast && ident_tiles && lean_kernel_applies(a, G, group_cols);
    {
        int64_t nt256 = 0;
        for (int g = 0; g < G; ++g) nt256 += (group_cols[g] + 255) / 256;
        lean64 = lean64 && ((a.M + 63) / 64) * nt256 <= kNumXcd * kSlotsPerXcd;
    }
    const bool wide_auto = a.M <= 64 ? n_slices128 >= 160 : (!fits32 && fits64 && !lean64);
    const bool small_T = a.M <= 64 || (!packed && a.M <= kDecodeMaxT * 8 && (fits32 || (fits64 && !lean64) || (policy0 == 5 && a.M <= kDecodeMaxT)));
    if (fast && ident_vec && small_T && a.K <= 16 * kDecodeWideMaxKS && (policy0 == 5 || (policy0 == 0 && wide_auto))) {
        // a few tokens, wide output: stream the weights once, 128 (64) output columns per workgroup
        build_tiles(a, G, group_cols, a.M <= 64 ? 64 : kDecodeMaxT, a.M <= 64 ? 128 : 64);
        a.sm = a.sn = 1;
        if (dtype == BDA_F16 && out_dtype == BDA_F16) return launch_decode_wide<F16, uint16_t>(a, st);
        if (dtype == BDA_F16 && out_dtype == BDA_F32) return launch_decode_wide<F16, float>(a, st);
        if (dtype == BDA_BF16 && out_dtype == BDA_BF16) return launch_decode_wide<BF16, uint16_t>(a, st);
        if (dtype == BDA_BF16 && out_dtype == BDA_F32) return launch_decode_wide<BF16, float>(a, st);
    }
    if (fast && ident_vec && small_policy && a.K <= kDecodeMaxK && (a.M <= 64 || (!packed && a.M <= kDecodeMaxT * 8 && fits32))) {
        // a few tokens: stream the weights once, 32 output columns per workgroup
        build_tiles(a, G, group_cols, a.M <= 64 ? 64 : kDecodeMaxT, 32);
        a.sm = a.sn = 1;
        if (dtype == BDA_F16 && out_dtype == BDA_F16) return launch_decode<F16, uint16_t>(a, st);
        if (dtype == BDA_F16 && out_dtype == BDA_F32) return launch_decode<F16, float>(a, st);
        if (dtype == BDA_BF16 && out_dtype == BDA_BF16) return launch_decode<BF16, uint16_t>(a, st);
        if (dtype == BDA_BF16 && out_dtype == BDA_F32) return launch_decode<BF16, float>(a, st);
    }
    if (packed)
        return fail(BDA_EINVAL, "bda_kv_project_packed: packed weights serve the few-token kernels only (up to 64 tokens, 16-bit types, "
                                "16-byte aligned buffers, pitches and d_c - d_h multiples of 8, d_c - d_h <= %d); use bda_kv_project with the canonical C", kDecodeMaxK);
    if (fast && ident_tiles) {
        const int64_t mt256 = (a.M + 255) / 256, mt128 = (a.M + 127) / 128;
        int64_t nt256 = 0;
        for (int g = 0; g < G; ++g) nt256 += (group_cols[g] + 255) / 256;
        const int policy = policy0 == 5 ? 0 : policy0;
        const int id_width = (a.d_h % 256) == 0 ? 256 : a.d_h;          // window columns a 256-column tile needs
        const int n_stage_id = a.ident ? (id_width + kStreamSK - 1) / kStreamSK : 0;
        const int n_stage_id_lean = a.ident ? (id_width + 2 * kStreamSK - 1) / (2 * kStreamSK) : 0;   // double-width identity stages
        // Can the streaming kernels take this launch at all, and its lean variant (nothing in any
        // stage depends on the lane: see bda_gemm_plain.hpp)?
        bool stream_ok = (a.K + kStreamSK - 1) / kStreamSK + n_stage_id >= kStreamNS && a.d_h < (1 << 16);
        for (int g = 0; g < G; ++g) stream_ok = stream_ok && group_cols[g] < (1 << 24);   // exact x % d_h by multiplication
        const bool plain = stream_ok && kStreamSK == 64 && kStreamNS == 2 && lean_kernel_applies(a, G, group_cols)   // (window starts: multiples of 8, checked above)
                           && policy != 3 && policy != 1;
        // Tile choice.  The lean kernel serves every tile count; its 128-token tile costs 0.53-0.56 of
        // its 256-token tile per round of tiles (measured), so the smaller tile is taken where it
        // needs less than 1 / 0.56 times the rounds.  Without the lean kernel: 256 x 256 streaming
        // tiles from 96 tiles up (measured crossover), else 128 x 128 register-staged tiles.
        auto rounds_of = [&](int64_t tiles) {
            const int64_t run = (tiles + kNumXcd - 1) / kNumXcd;
            return (run + kSlotsPerXcd - 1) / kSlotsPerXcd;
        };
        if (policy == 6) {
            build_tiles(a, G, group_cols, 128, 256);
            a.sm = a.sn = 1;
            if (dtype == BDA_F16 && out_dtype == BDA_F16) return launch_duo<F16, uint16_t>(a, st);
            if (dtype == BDA_F16 && out_dtype == BDA_F32) return launch_duo<F16, float>(a, st);
            if (dtype == BDA_BF16 && out_dtype == BDA_BF16) return launch_duo<BF16, uint16_t>(a, st);
            if (dtype == BDA_BF16 && out_dtype == BDA_F32) return launch_duo<BF16, float>(a, st);
        }
        // Its 64-token tile costs 0.47-0.5 of the 256-token tile per round, less than the 128-token tile, but
        // two rounds of it cost more than one of either: it is taken where one round of it covers the launch.
        const int64_t mt64 = (a.M + 63) / 64;
        const bool quarter_tokens = plain && (policy == 7 || (policy == 0 && rounds_of(mt64 * nt256) == 1));
        const bool half_tokens = plain && !quarter_tokens && (policy == 4 || (policy == 0 && 0.56 * (double)rounds_of(mt128 * nt256) < (double)rounds_of(mt256 * nt256)));
        const int tok_tile = quarter_tokens ? 64 : half_tokens ? 128 : 256;
        const bool big = plain || policy == 2 || policy == 3 || policy == 4 || ((policy == 0 || policy == 7) && mt256 * nt256 >= 96);
        const bool stream = big && stream_ok;
        if (big) {
            build_tiles(a, G, group_cols, tok_tile, 256);
            choose_super(a, kSlotsPerXcd, tok_tile, 256);
            // identity slice: stages of the streaming kernel (the slice of a 256-column tile is the
            // whole window, or the tile's own 256 columns of it when d_h is a multiple of 256)
            a.n_stage_id = plain ? n_stage_id_lean : n_stage_id;
        } else {
            build_tiles(a, G, group_cols, 128, 128);
            choose_super(a, 2 * kSlotsPerXcd, 128, 128);
        }
#define BDA_LAUNCH(X, O)                                      \
    return stream ? launch_stream<X, O>(a, plain, plain ? tok_tile : 256, st) : big ? launch_mfma<X, O, 4, 4>(a, st) : launch_mfma<X, O, 2, 2>(a, st)
        if (dtype == BDA_F16 && out_dtype == BDA_F16) { BDA_LAUNCH(F16, uint16_t); }
        if (dtype == BDA_F16 && out_dtype == BDA_F32) { BDA_LAUNCH(F16, float); }
        if (dtype == BDA_BF16 && out_dtype == BDA_BF16) { BDA_LAUNCH(BF16, uint16_t); }
        if (dtype == BDA_BF16 && out_dtype == BDA_F32) { BDA_LAUNCH(BF16, float); }
#undef BDA_LAUNCH
        return fail(BDA_EDTYPE, "unsupported dtype/out_dtype pair %d/%d", dtype, out_dtype);
    }
    build_tiles(a, G, group_cols, 64, 64);
    a.sm = a.sn = 1;
    if (a.m_tiles > 65535) return fail(BDA_EINVAL, "general kernel: T too large (%lld)", (long long)a.M);
    if (dtype == BDA_F32 && out_dtype == BDA_F32) return launch_general<float, float>(a, N_total, st);
    if (dtype == BDA_F16 && out_dtype == BDA_F16) return launch_general<RawF16, RawF16>(a, N_total, st);
    if (dtype == BDA_F16 && out_dtype == BDA_F32) return launch_general<RawF16, float>(a, N_total, st);
    if (dtype == BDA_BF16 && out_dtype == BDA_BF16) return launch_general<RawBF16, RawBF16>(a, N_total, st);
    if (dtype == BDA_BF16 && out_dtype == BDA_F32) return launch_general<RawBF16, float>(a, N_total, st);
    return fail(BDA_EDTYPE, "unsupported dtype/out_dtype pair %d/%d", dtype, out_dtype);
}

int check_dtypes(const char* fn, int dtype, int out_dtype)
{
    if (dtype != BDA_F32 && dtype != BDA_F16 && dtype != BDA_BF16) return fail(BDA_EDTYPE, "%s: bad dtype %d", fn, dtype);
    if (out_dtype != dtype && out_dtype != BDA_F32) return fail(BDA_EDTYPE, "%s: out_dtype must equal dtype or be BDA_F32 (got %d/%d)", fn, dtype, out_dtype);
    return BDA_OK;
}

}  // namespace

int tile_policy() { return t_policy; }

PolicyScope::PolicyScope(int policy) : prev_(t_policy) { t_policy = policy; }
PolicyScope::~PolicyScope() { t_policy = prev_; }

int check_policy(const char* fn, int policy)
{
    return policy >= 0 && policy <= 7 ? BDA_OK : fail(BDA_EINVAL, "%s: tile_policy must be 0 .. 7 (got %d)", fn, policy);
}

}  // namespace bda

using namespace bda;

extern "C" int bda_kv_project_ex(const void* c, int64_t ldc, int64_t T, int d_c, int d_h, int G,
                                 const int* H, const int* basis_offset, const void* C, int64_t ldC,
                                 void* out, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype,
                                 void* stream, int tile_policy)
{
    clear_error();
    if (int rc = check_policy("bda_kv_project_ex", tile_policy)) return rc;
    PolicyScope scope(tile_policy);
    return bda_kv_project(c, ldc, T, d_c, d_h, G, H, basis_offset, C, ldC, out, ld_out, dtype, out_dtype, stream);
}

extern "C" int bda_kv_project(const void* c, int64_t ldc, int64_t T, int d_c, int d_h, int G,
                              const int* H, const int* basis_offset, const void* C, int64_t ldC,
                              void* out, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype,
                              void* stream)
{
    clear_error();
    if (int rc = check_dtypes("bda_kv_project", dtype, out_dtype)) return rc;
    if (T < 0 || d_c <= 0 || d_h <= 0 || d_h >= d_c) return fail(BDA_EINVAL, "bda_kv_project: need T >= 0 and 0 < d_h < d_c (T=%lld d_c=%d d_h=%d)", (long long)T, d_c, d_h);
    if (G <= 0 || G > BDA_MAX_GROUPS || !H || !basis_offset) return fail(BDA_EINVAL, "bda_kv_project: need 1 <= G <= %d and non-NULL H, basis_offset", BDA_MAX_GROUPS);
    int64_t N = 0;
    int64_t cols[BDA_MAX_GROUPS];
    for (int g = 0; g < G; ++g) {
        if (H[g] <= 0) return fail(BDA_EINVAL, "bda_kv_project: H[%d]=%d", g, H[g]);
        if (basis_offset[g] < 0 || basis_offset[g] > d_c - d_h) return fail(BDA_EINVAL, "bda_kv_project: basis_offset[%d]=%d outside [0, %d]", g, basis_offset[g], d_c - d_h);
        cols[g] = (int64_t)H[g] * d_h;
        N += cols[g];
    }
    if (T == 0) return BDA_OK;
    if (!c || !C || !out) return fail(BDA_EINVAL, "bda_kv_project: NULL device pointer");
    if (ldc < d_c || ldC < N || ld_out < N) return fail(BDA_EINVAL, "bda_kv_project: leading dimension too small (ldc=%lld ldC=%lld ld_out=%lld, d_c=%d N=%lld)", (long long)ldc, (long long)ldC, (long long)ld_out, d_c, (long long)N);
    const size_t esz = dtype_size(dtype), osz = dtype_size(out_dtype);
    const int K = d_c - d_h;
    Span so = span_of(out, T, N, ld_out, osz);
    if (overlaps(so, span_of(c, T, d_c, ldc, esz)) || overlaps(so, span_of(C, K, N, ldC, esz)))
        return fail(BDA_EINVAL, "bda_kv_project: out overlaps an input");
    GemmArgs a{};
    a.A = c; a.B = C; a.D = out;
    a.lda = ldc; a.ldb = ldC; a.ldd = ld_out;
    a.M = T; a.K = K; a.d_h = d_h; a.a_skip = d_h; a.ident = 1;
    for (int g = 0; g < G; ++g) a.a_off[g] = basis_offset[g];
    return run_gemm(a, G, cols, dtype, out_dtype, (hipStream_t)stream);
}

namespace bda {
namespace {

// One 16-byte piece (8 columns of one row) per thread: C[k][n .. n + 7] -> slice n / 32, row k, columns n % 32.
__global__ __launch_bounds__(256) void pack_weights_kernel(const u32x4* __restrict__ C, int64_t ldC8, int K, int64_t N8, u32x4* __restrict__ packed)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)K * N8) return;
    const int64_t k = i / N8, p8 = i % N8;
    packed[((p8 >> 2) * K + k) * 4 + (p8 & 3)] = C[k * ldC8 + p8];
}

int packed_shape(const char* fn, int d_c, int d_h, int G, const int* H, int dtype, int64_t& N)
{
    if (dtype != BDA_F16 && dtype != BDA_BF16) return fail(BDA_EDTYPE, "%s: packed weights are 16-bit (got dtype %d)", fn, dtype);
    if (d_c <= 0 || d_h <= 0 || d_h >= d_c) return fail(BDA_EINVAL, "%s: need 0 < d_h < d_c", fn);
    if (G <= 0 || G > BDA_MAX_GROUPS || !H) return fail(BDA_EINVAL, "%s: need 1 <= G <= %d and non-NULL H", fn, BDA_MAX_GROUPS);
    N = 0;
    for (int g = 0; g < G; ++g) {
        if (H[g] <= 0) return fail(BDA_EINVAL, "%s: H[%d]=%d", fn, g, H[g]);
        if (((int64_t)H[g] * d_h) % 32) return fail(BDA_EINVAL, "%s: every group's width H[g] d_h must be a multiple of 32 (group %d: %lld)", fn, g, (long long)H[g] * d_h);
        N += (int64_t)H[g] * d_h;
    }
    return BDA_OK;
}

}  // namespace
}  // namespace bda

extern "C" size_t bda_packed_weights_bytes(int d_c, int d_h, int G, const int* H, bda_dtype dtype)
{
    clear_error();
    int64_t N = 0;
    if (packed_shape("bda_packed_weights_bytes", d_c, d_h, G, H, (int)dtype, N)) return 0;
    return (size_t)(d_c - d_h) * (size_t)N * 2;
}

extern "C" int bda_pack_weights(const void* C, int64_t ldC, int d_c, int d_h, int G, const int* H, bda_dtype dtype,
                                void* packed, void* stream)
{
    clear_error();
    int64_t N = 0;
    if (int rc = packed_shape("bda_pack_weights", d_c, d_h, G, H, (int)dtype, N)) return rc;
    if (!C || !packed) return fail(BDA_EINVAL, "bda_pack_weights: NULL device pointer");
    if (ldC < N || ldC % 8 || !aligned(C, 16) || !aligned(packed, 16)) return fail(BDA_EINVAL, "bda_pack_weights: need ldC >= N, ldC a multiple of 8 and 16-byte aligned buffers");
    const int K = d_c - d_h;
    if (overlaps(span_of(packed, 1, (int64_t)K * N, (int64_t)K * N, 2), span_of(C, K, N, ldC, 2))) return fail(BDA_EINVAL, "bda_pack_weights: packed overlaps C");
    const int64_t pieces = (int64_t)K * (N / 8);
    if (pieces > ((int64_t)1 << 31) * 256) return fail(BDA_EINVAL, "bda_pack_weights: too large");
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4*)C, ldC / 8, K, N / 8, (u32x4*)packed);
    hipError_t err = hipGetLastError();
    return err == hipSuccess ? BDA_OK : fail(BDA_EHIP, "bda_pack_weights: kernel launch: %s", hipGetErrorString(err));
}

extern "C" int bda_kv_project_packed(const void* c, int64_t ldc, int64_t T, int d_c, int d_h, int G,
                                     const int* H, const int* basis_offset, const void* packed,
                                     void* out, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype, void* stream)
{
    clear_error();
    const char* fn = "bda_kv_project_packed";
    if (int rc = check_dtypes(fn, dtype, out_dtype)) return rc;
    int64_t N = 0;
    if (int rc = packed_shape(fn, d_c, d_h, G, H, (int)dtype, N)) return rc;
    if (T < 0 || !basis_offset) return fail(BDA_EINVAL, "%s: need T >= 0 and non-NULL basis_offset", fn);
    int64_t cols[BDA_MAX_GROUPS];
    for (int g = 0; g < G; ++g) {
        if (basis_offset[g] < 0 || basis_offset[g] > d_c - d_h) return fail(BDA_EINVAL, "%s: basis_offset[%d]=%d outside [0, %d]", fn, g, basis_offset[g], d_c - d_h);
        cols[g] = (int64_t)H[g] * d_h;
    }
    if (T == 0) return BDA_OK;
    if (T > 64) return fail(BDA_EINVAL, "%s: packed weights serve up to 64 tokens (T=%lld); use bda_kv_project with the canonical C", fn, (long long)T);
    if (!c || !packed || !out) return fail(BDA_EINVAL, "%s: NULL device pointer", fn);
    if (ldc < d_c || ld_out < N) return fail(BDA_EINVAL, "%s: leading dimension too small", fn);
    if (!aligned(packed, 16)) return fail(BDA_EINVAL, "%s: packed not 16-byte aligned", fn);
    const int K = d_c - d_h;
    const size_t esz = dtype_size(dtype), osz = dtype_size(out_dtype);
    Span so = span_of(out, T, N, ld_out, osz);
    if (overlaps(so, span_of(c, T, d_c, ldc, esz)) || overlaps(so, span_of(packed, 1, (int64_t)K * N, (int64_t)K * N, esz)))
        return fail(BDA_EINVAL, "%s: out overlaps an input", fn);
    GemmArgs a{};
    a.A = c; a.B = packed; a.D = out;
    a.lda = ldc; a.ldb = 0; a.ldd = ld_out;              // ldb = 0: C in the packed layout
    a.M = T; a.K = K; a.d_h = d_h; a.a_skip = d_h; a.ident = 1;
    for (int g = 0; g < G; ++g) a.a_off[g] = basis_offset[g];
    return run_gemm(a, G, cols, dtype, out_dtype, (hipStream_t)stream);
}

extern "C" int bda_dense_project_ex(const void* c, int64_t ldc, int64_t T, int d_c, const void* W,
                                    int64_t ldW, int64_t N, void* out, int64_t ld_out, bda_dtype dtype,
                                    bda_dtype out_dtype, void* stream, int tile_policy)
{
    clear_error();
    if (int rc = check_policy("bda_dense_project_ex", tile_policy)) return rc;
    PolicyScope scope(tile_policy);
    return bda_dense_project(c, ldc, T, d_c, W, ldW, N, out, ld_out, dtype, out_dtype, stream);
}

extern "C" int bda_dense_project(const void* c, int64_t ldc, int64_t T, int d_c, const void* W,
                                 int64_t ldW, int64_t N, void* out, int64_t ld_out, bda_dtype dtype,
                                 bda_dtype out_dtype, void* stream)
{
    clear_error();
    if (int rc = check_dtypes("bda_dense_project", dtype, out_dtype)) return rc;
    if (T < 0 || d_c <= 0 || N <= 0) return fail(BDA_EINVAL, "bda_dense_project: need T >= 0, d_c > 0, N > 0");
    if (T == 0) return BDA_OK;
    if (!c || !W || !out) return fail(BDA_EINVAL, "bda_dense_project: NULL device pointer");
    if (ldc < d_c || ldW < N || ld_out < N) return fail(BDA_EINVAL, "bda_dense_project: leading dimension too small");
    const size_t esz = dtype_size(dtype), osz = dtype_size(out_dtype);
    Span so = span_of(out, T, N, ld_out, osz);
    if (overlaps(so, span_of(c, T, d_c, ldc, esz)) || overlaps(so, span_of(W, d_c, N, ldW, esz)))
        return fail(BDA_EINVAL, "bda_dense_project: out overlaps an input");
    GemmArgs a{};
    a.A = c; a.B = W; a.D = out;
    a.lda = ldc; a.ldb = ldW; a.ldd = ld_out;
    a.M = T; a.K = d_c; a.d_h = 0; a.a_skip = 0; a.ident = 0;
    a.a_off[0] = d_c;
    int64_t cols[1] = {N};
    return run_gemm(a, 1, cols, dtype, out_dtype, (hipStream_t)stream);
}

extern "C" int bda_lowrank_linear(const void* x, int64_t ldx, int64_t T, int d_in, int r, int d_out,
                                  int basis_offset, const void* Uprime, const void* C, void* out,
                                  int64_t ld_out, bda_dtype dtype, void* stream)
{
    clear_error();
    if (int rc = check_dtypes("bda_lowrank_linear", dtype, dtype)) return rc;
    if (T < 0 || d_in <= 0 || r <= 0 || d_out <= r) return fail(BDA_EINVAL, "bda_lowrank_linear: need T >= 0, d_in > 0, 0 < r < d_out");
    if (basis_offset != 0 && basis_offset != d_out - r) return fail(BDA_EINVAL, "bda_lowrank_linear: basis_offset must be 0 or d_out - r");
    if (T == 0) return BDA_OK;
    if (!x || !Uprime || !C || !out) return fail(BDA_EINVAL, "bda_lowrank_linear: NULL device pointer");
    if (ldx < d_in || ld_out < d_out) return fail(BDA_EINVAL, "bda_lowrank_linear: leading dimension too small");
    const size_t esz = dtype_size(dtype);
    const int nc = d_out - r;
    Span so = span_of(out, T, d_out, ld_out, esz);
    if (overlaps(so, span_of(x, T, d_in, ldx, esz)) || overlaps(so, span_of(Uprime, d_in, r, r, esz)) ||
        overlaps(so, span_of(C, r, nc, nc, esz)))
        return fail(BDA_EINVAL, "bda_lowrank_linear: out overlaps an input");
    char* ob = (char*)out;
    void* h_cols = ob + (size_t)basis_offset * esz;                    // where h lives inside out
    void* c_cols = ob + (size_t)(basis_offset == 0 ? r : 0) * esz;     // where h C goes
    {   // h = x Uprime
        GemmArgs a{};
        a.A = x; a.B = Uprime; a.D = h_cols;
        a.lda = ldx; a.ldb = r; a.ldd = ld_out;
        a.M = T; a.K = d_in; a.a_off[0] = d_in;
        int64_t cols[1] = {r};
        if (int rc = run_gemm(a, 1, cols, dtype, dtype, (hipStream_t)stream)) return rc;
    }
    {   // [.., h C]: reads h back from its columns of out (same stream, so ordered after the first)
        GemmArgs a{};
        a.A = h_cols; a.B = C; a.D = c_cols;
        a.lda = ld_out; a.ldb = nc; a.ldd = ld_out;
        a.M = T; a.K = r; a.a_off[0] = r;
        int64_t cols[1] = {nc};
        return run_gemm(a, 1, cols, dtype, dtype, (hipStream_t)stream);
    }
}

namespace {
// Stand-ins for device pointers (16-byte aligned, far apart): the plan entry points run the same
// validation and tile choice as the real calls and stop before any HIP call.
void* const kFakeA = (void*)((uintptr_t)1 << 40);
void* const kFakeB = (void*)((uintptr_t)2 << 40);
void* const kFakeD = (void*)((uintptr_t)3 << 40);
}  // namespace

extern "C" int bda_kv_project_plan(int64_t T, int d_c, int d_h, int G, const int* H, const int* basis_offset,
                                   int64_t ldc, int64_t ldC, int64_t ld_out, bda_dtype dtype, bda_dtype out_dtype,
                                   int tile_policy, bda_launch_plan* plan)
{
    clear_error();
    if (!plan) return fail(BDA_EINVAL, "bda_kv_project_plan: NULL plan");
    if (int rc = check_policy("bda_kv_project_plan", tile_policy)) return rc;
    PolicyScope scope(tile_policy);
    *plan = bda_launch_plan{BDA_KERNEL_NONE, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    t_plan = plan;
    const int rc = bda_kv_project(kFakeA, ldc, T, d_c, d_h, G, H, basis_offset, kFakeB, ldC, kFakeD, ld_out, dtype, out_dtype, nullptr);
    t_plan = nullptr;
    return rc;
}

extern "C" int bda_dense_project_plan(int64_t T, int d_c, int64_t N, int64_t ldc, int64_t ldW, int64_t ld_out,
                                      bda_dtype dtype, bda_dtype out_dtype, int tile_policy, bda_launch_plan* plan)
{
    clear_error();
    if (!plan) return fail(BDA_EINVAL, "bda_dense_project_plan: NULL plan");
    if (int rc = check_policy("bda_dense_project_plan", tile_policy)) return rc;
    PolicyScope scope(tile_policy);
    *plan = bda_launch_plan{BDA_KERNEL_NONE, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    t_plan = plan;
    const int rc = bda_dense_project(kFakeA, ldc, T, d_c, kFakeB, ldW, N, kFakeD, ld_out, dtype, out_dtype, nullptr);
    t_plan = nullptr;
    return rc;
}
