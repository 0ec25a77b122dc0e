// Host-side (float64) offline preparation for BD Attention and the BD linear layer.
//
// Per head h and basis window B = [off, off + d_h):   C_h = W_h[Bbar,:] W_h[B,:]^{-1}.
// This is what the column-first BD of W_q^h (W_k^h)^T (Eq. qk_bd_single) and the row-first BD of
// W_v^h W_o^h (Appendix "BD for VO in MHA") reduce to when the product matrices are written out:
// the basis factor W_h[B,:] is square, so the coefficient block is a square solve and the inverse
// moves into the companion weight (B_qk^h = W_q^h W_h[B,:]^T, B_vo^h = W_h[B,:] W_o^h).
//
// The square systems x A = y are solved through a Householder LQ factorisation of A (no explicit
// inverse, no pivot search -- the paper's premise is that any contiguous window is a valid basis;
// a window that is not is reported as BDA_ESINGULAR).  The window is chosen as in Algorithm "BD
// Decomposition (Row)" / "BD Attention Preparation (QK)": smallest mean Frobenius residual over
// heads, ties to the earlier candidate.
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>
#include <mutex>
#include <thread>
#include <vector>

#include "bda_internal.h"

namespace bda {

namespace {
thread_local std::string g_last_error;
}

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return code;
}

void clear_error() { g_last_error.clear(); }

void parallel_for(int64_t n, const std::function<void(int64_t)>& fn, int max_threads)
{
    if (n <= 0) return;
    unsigned hw = std::thread::hardware_concurrency();
    int64_t nt = hw ? hw : 4;
    if (nt > 64) nt = 64;
    if (max_threads > 0 && nt > max_threads) nt = max_threads;
    if (nt > n) nt = n;
    if (nt <= 1) {
        for (int64_t i = 0; i < n; ++i) fn(i);
        return;
    }
    std::atomic<int64_t> next{0};
    std::vector<std::thread> pool;
    pool.reserve(nt);
    for (int64_t t = 0; t < nt; ++t)
        pool.emplace_back([&] {
            for (;;) {
                int64_t i = next.fetch_add(1);
                if (i >= n) break;
                fn(i);
            }
        });
    for (auto& th : pool) th.join();
}

namespace {

// One round-to-nearest-even step from double to a format with `sig` significant bits.
double round_sig(double x, int sig, int min_step_exp, double max_finite)
{
    if (!std::isfinite(x) || x == 0.0) return x;
    int e;
    std::frexp(x, &e);
    int s = e - sig;
    if (s < min_step_exp) s = min_step_exp;
    double q = std::ldexp(std::nearbyint(std::ldexp(x, -s)), s);
    if (std::fabs(q) > max_finite) q = std::copysign(std::numeric_limits<double>::infinity(), x);
    return q;
}

double round_store(double x, int dt)
{
    switch (dt) {
    case BDA_F32: return (double)(float)x;
    case BDA_F16: return round_sig(x, 11, -24, 65504.0);
    case BDA_BF16: return round_sig(x, 8, -133, 3.3895313892515355e38);
    default: return x;
    }
}

// In-place Householder LQ of the n x n row-major matrix A: A = L Q with Q = H_{n-1} ... H_0,
// H_k = I - tau_k v_k v_k^T acting on columns k..n-1, v_k[0] = 1 and v_k[1:] stored in A[k][k+1:].
// Returns the index of the first negligible diagonal entry of L, or -1.
int lq_factor(double* A, int n, double* tau)
{
    double fro2 = 0.0;
    for (int64_t i = 0; i < (int64_t)n * n; ++i) fro2 += A[i] * A[i];
    const double tiny = std::sqrt(fro2) * n * std::numeric_limits<double>::epsilon();
    int bad = -1;
    for (int k = 0; k < n; ++k) {
        double* a = A + (int64_t)k * n + k;
        const int m = n - k;
        double sigma = 0.0;
        for (int j = 1; j < m; ++j) sigma += a[j] * a[j];
        const double alpha = a[0];
        double beta, t;
        if (sigma == 0.0) {
            beta = alpha;
            t = 0.0;
        } else {
            beta = -std::copysign(std::sqrt(alpha * alpha + sigma), alpha);
            t = (beta - alpha) / beta;
            const double inv = 1.0 / (alpha - beta);
            for (int j = 1; j < m; ++j) a[j] *= inv;
        }
        a[0] = beta;
        tau[k] = t;
        if (!(std::fabs(beta) > tiny) && bad < 0) bad = k;
        if (t != 0.0) {
            for (int i = k + 1; i < n; ++i) {
                double* z = A + (int64_t)i * n + k;
                double s = z[0];
                for (int j = 1; j < m; ++j) s += z[j] * a[j];
                s *= t;
                z[0] -= s;
                for (int j = 1; j < m; ++j) z[j] -= s * a[j];
            }
        }
    }
    return bad;
}

// Solves x A = y in place (y of length n becomes x), A given by its LQ factors.
void lq_solve_row(const double* LQ, const double* tau, int n, double* y)
{
    for (int k = 0; k < n; ++k) {           // y <- y H_0 H_1 ... H_{n-1}
        const double t = tau[k];
        if (t == 0.0) continue;
        const double* v = LQ + (int64_t)k * n + k;
        double* z = y + k;
        const int m = n - k;
        double s = z[0];
        for (int j = 1; j < m; ++j) s += z[j] * v[j];
        s *= t;
        z[0] -= s;
        for (int j = 1; j < m; ++j) z[j] -= s * v[j];
    }
    for (int i = n - 1; i >= 0; --i) {       // x L = y, L lower triangular
        const double* Li = LQ + (int64_t)i * n;
        const double xi = y[i] / Li[i];
        y[i] = xi;
        for (int j = 0; j < i; ++j) y[j] -= xi * Li[j];
    }
}

std::vector<int> candidate_offsets(int mode, int d, int w, int explicit_offset)
{
    const int last = d - w;
    std::vector<int> o;
    switch (mode) {
    case BDA_BASIS_FIRST: o = {0}; break;
    case BDA_BASIS_LAST: o = {last}; break;
    case BDA_BASIS_RESIDUAL_MIN:
        o = {0};
        if (last != 0) o.push_back(last);
        break;
    case BDA_BASIS_OFFSET_SEARCH:
        // windows starting at multiples of 16 (Appendix "Residual-Min with Offset Search"), no
        // wrap-around, plus the last window so that the search never does worse than first/last
        for (int s = 0; s <= last; s += 16) o.push_back(s);
        if (o.back() != last) o.push_back(last);
        break;
    case BDA_BASIS_EXPLICIT: o = {explicit_offset}; break;
    default: break;
    }
    return o;
}

struct HeadJob {
    const double* W;
    int64_t ldw;
    int d_c, d_h, off;
    const double* side;
    int64_t ld_side;
    int d_side;
    int side_kind;
    int store_dtype;
    bool want_resid;
};

// Processes head h for window job.off.  Writes C (K x d_h block of C_all with row stride ldc_all)
// and the companion block; returns the residual (0 if not wanted) or -1 on a singular block.
double prepare_head(const HeadJob& jb, int h, double* C_all, int64_t ldc_all, double* side_all,
                    int64_t ld_side_all, int* singular_at)
{
    const int n = jb.d_h, d_c = jb.d_c, K = d_c - n, off = jb.off;
    const double* Wh = jb.W + (int64_t)h * n;
    std::vector<double> A((size_t)n * n), LQ, tau(n), Cblk((size_t)K * n);
    for (int i = 0; i < n; ++i)
        std::memcpy(&A[(size_t)i * n], Wh + (int64_t)(off + i) * jb.ldw, sizeof(double) * n);
    LQ = A;
    const int bad = lq_factor(LQ.data(), n, tau.data());
    if (bad >= 0) {
        *singular_at = bad;
        return -1.0;
    }
    auto bbar = [&](int kk) { return kk < off ? kk : kk + n; };
    for (int kk = 0; kk < K; ++kk) {
        double* y = &Cblk[(size_t)kk * n];
        std::memcpy(y, Wh + (int64_t)bbar(kk) * jb.ldw, sizeof(double) * n);
        lq_solve_row(LQ.data(), tau.data(), n, y);
        std::memcpy(C_all + (int64_t)kk * ldc_all + (int64_t)h * n, y, sizeof(double) * n);
    }
    double r2 = 0.0;
    std::vector<double> Chat;
    if (jb.want_resid) {
        Chat.resize(Cblk.size());
        for (size_t i = 0; i < Cblk.size(); ++i) Chat[i] = round_store(Cblk[i], jb.store_dtype);
    }
    if (jb.side_kind == BDA_SIDE_Q) {
        // B_qk^h = W_q^h A^T  (d_side x d_h)
        const int ds = jb.d_side;
        std::vector<double> Bq((size_t)ds * n);
        for (int s = 0; s < ds; ++s) {
            const double* q = jb.side + (int64_t)s * jb.ld_side + (int64_t)h * n;
            for (int i = 0; i < n; ++i) {
                const double* ai = &A[(size_t)i * n];
                double acc = 0.0;
                for (int j = 0; j < n; ++j) acc += q[j] * ai[j];
                Bq[(size_t)s * n + i] = acc;
            }
            std::memcpy(side_all + (int64_t)s * ld_side_all + (int64_t)h * n, &Bq[(size_t)s * n],
                        sizeof(double) * n);
        }
        if (jb.want_resid) {
            std::vector<double> bh(n);
            for (int s = 0; s < ds; ++s) {
                const double* q = jb.side + (int64_t)s * jb.ld_side + (int64_t)h * n;
                for (int i = 0; i < n; ++i) bh[i] = round_store(Bq[(size_t)s * n + i], jb.store_dtype);
                for (int k = 0; k < d_c; ++k) {
                    const double* wk = Wh + (int64_t)k * jb.ldw;
                    double m = 0.0;
                    for (int j = 0; j < n; ++j) m += q[j] * wk[j];       // (W_q^h W_h^T)[s][k]
                    double rec;
                    if (k >= off && k < off + n) {
                        rec = bh[k - off];
                    } else {
                        const double* ck = &Chat[(size_t)(k < off ? k : k - n) * n];
                        rec = 0.0;
                        for (int i = 0; i < n; ++i) rec += bh[i] * ck[i];
                    }
                    const double d = m - rec;
                    r2 += d * d;
                }
            }
        }
    } else if (jb.side_kind == BDA_SIDE_O) {
        // B_vo^h = A W_o^h  (d_h x d_side)
        const int dm = jb.d_side;
        std::vector<double> Bo((size_t)n * dm, 0.0);
        for (int i = 0; i < n; ++i) {
            double* bo = &Bo[(size_t)i * dm];
            for (int j = 0; j < n; ++j) {
                const double a = A[(size_t)i * n + j];
                const double* wo = jb.side + (int64_t)((int64_t)h * n + j) * jb.ld_side;
                for (int m = 0; m < dm; ++m) bo[m] += a * wo[m];
            }
            std::memcpy(side_all + ((int64_t)h * n + i) * ld_side_all, bo, sizeof(double) * dm);
        }
        if (jb.want_resid) {
            std::vector<double> Bh(Bo.size()), mrow(dm), rrow(dm);
            for (size_t i = 0; i < Bo.size(); ++i) Bh[i] = round_store(Bo[i], jb.store_dtype);
            for (int k = 0; k < d_c; ++k) {
                const double* wk = Wh + (int64_t)k * jb.ldw;
                std::fill(mrow.begin(), mrow.end(), 0.0);
                for (int j = 0; j < n; ++j) {
                    const double* wo = jb.side + (int64_t)((int64_t)h * n + j) * jb.ld_side;
                    for (int m = 0; m < dm; ++m) mrow[m] += wk[j] * wo[m];   // (W_h W_o^h)[k][:]
                }
                if (k >= off && k < off + n) {
                    const double* b = &Bh[(size_t)(k - off) * dm];
                    for (int m = 0; m < dm; ++m) rrow[m] = b[m];
                } else {
                    const double* ck = &Chat[(size_t)(k < off ? k : k - n) * n];
                    std::fill(rrow.begin(), rrow.end(), 0.0);
                    for (int i = 0; i < n; ++i) {
                        const double* b = &Bh[(size_t)i * dm];
                        for (int m = 0; m < dm; ++m) rrow[m] += ck[i] * b[m];
                    }
                }
                for (int m = 0; m < dm; ++m) {
                    const double d = mrow[m] - rrow[m];
                    r2 += d * d;
                }
            }
        }
    } else if (jb.want_resid) {
        // row BD of W_h itself: basis rows reproduce themselves, the others are Chat A
        std::vector<double> rec(n);
        for (int kk = 0; kk < K; ++kk) {
            std::fill(rec.begin(), rec.end(), 0.0);
            const double* ck = &Chat[(size_t)kk * n];
            for (int i = 0; i < n; ++i) {
                const double* ai = &A[(size_t)i * n];
                for (int j = 0; j < n; ++j) rec[j] += ck[i] * ai[j];
            }
            const double* w = Wh + (int64_t)bbar(kk) * jb.ldw;
            for (int j = 0; j < n; ++j) {
                const double d = w[j] - rec[j];
                r2 += d * d;
            }
        }
    }
    return std::sqrt(r2);
}

double nan_to_inf(double r) { return std::isnan(r) ? std::numeric_limits<double>::infinity() : r; }

}  // namespace
}  // namespace bda

using namespace bda;

extern "C" const char* bda_last_error(void) { return g_last_error.c_str(); }

extern "C" int bda_version(void) { return 100; }

extern "C" int bda_prepare(const double* W, int64_t ldw, int d_c, int H, int d_h,
                           const double* side, int64_t ld_side, int d_side, bda_side side_kind,
                           bda_basis_mode mode, int explicit_offset, bda_dtype store_dtype,
                           double* C_out, double* side_out, int* basis_offset_out,
                           double* resid_out)
{
    clear_error();
    if (!W || !C_out || !basis_offset_out) return fail(BDA_EINVAL, "bda_prepare: NULL W, C_out or basis_offset_out");
    if (d_c <= 0 || H <= 0 || d_h <= 0 || d_h >= d_c)
        return fail(BDA_EINVAL, "bda_prepare: need 0 < d_h < d_c and H > 0 (d_c=%d H=%d d_h=%d)", d_c, H, d_h);
    const int64_t N = (int64_t)H * d_h;
    if (ldw < N) return fail(BDA_EINVAL, "bda_prepare: ldw=%lld < H*d_h=%lld", (long long)ldw, (long long)N);
    if (store_dtype < BDA_F32 || store_dtype > BDA_F64) return fail(BDA_EDTYPE, "bda_prepare: bad store_dtype %d", (int)store_dtype);
    int sk = side ? (int)side_kind : BDA_SIDE_NONE;
    if (sk != BDA_SIDE_NONE) {
        if (sk != BDA_SIDE_Q && sk != BDA_SIDE_O) return fail(BDA_EINVAL, "bda_prepare: bad side_kind %d", sk);
        if (!side_out || d_side <= 0) return fail(BDA_EINVAL, "bda_prepare: companion given but side_out NULL or d_side <= 0");
        const int64_t need = sk == BDA_SIDE_Q ? N : d_side;
        if (ld_side < need) return fail(BDA_EINVAL, "bda_prepare: ld_side=%lld too small (need %lld)", (long long)ld_side, (long long)need);
    }
    std::vector<int> offs = candidate_offsets((int)mode, d_c, d_h, explicit_offset);
    if (offs.empty()) return fail(BDA_EINVAL, "bda_prepare: bad basis mode %d", (int)mode);
    for (int o : offs)
        if (o < 0 || o > d_c - d_h) return fail(BDA_EINVAL, "bda_prepare: basis offset %d outside [0, %d]", o, d_c - d_h);

    const int K = d_c - d_h;
    const bool want_resid = offs.size() > 1 || resid_out != nullptr;
    const int64_t side_rows = sk == BDA_SIDE_Q ? d_side : N;
    const int64_t side_cols = sk == BDA_SIDE_Q ? N : d_side;
    std::vector<double> C_try, side_try;
    const bool multi = offs.size() > 1;
    if (multi) {
        C_try.resize((size_t)K * N);
        if (sk != BDA_SIDE_NONE) side_try.resize((size_t)side_rows * side_cols);
    }
    double best = std::numeric_limits<double>::infinity();
    int best_off = -1;
    double r_first = std::nan(""), r_last = std::nan("");
    for (size_t ci = 0; ci < offs.size(); ++ci) {
        HeadJob jb{W, ldw, d_c, d_h, offs[ci], side, ld_side, d_side, sk, (int)store_dtype, want_resid};
        double* Cdst = multi ? C_try.data() : C_out;
        double* Sdst = multi ? side_try.data() : side_out;
        std::vector<double> resid(H, 0.0);
        std::vector<int> sing(H, -1);
        parallel_for(H, [&](int64_t h) {
            resid[h] = prepare_head(jb, (int)h, Cdst, N, Sdst, side_cols, &sing[h]);
        });
        double mean = 0.0;
        bool singular = false;
        int sing_head = -1;
        for (int h = 0; h < H; ++h) {
            if (sing[h] >= 0) {
                singular = true;
                if (sing_head < 0) sing_head = h;
            }
            mean += resid[h];
        }
        mean = singular ? std::numeric_limits<double>::infinity() : nan_to_inf(mean / H);
        if (singular && !multi)
            return fail(BDA_ESINGULAR, "bda_prepare: basis block of head %d (window offset %d) is singular at pivot %d",
                        sing_head, offs[ci], sing[sing_head]);
        if (offs[ci] == 0) r_first = mean;
        if (offs[ci] == d_c - d_h) r_last = mean;
        const bool take = best_off < 0 ? !singular : mean < best;
        if (take) {
            best = mean;
            best_off = offs[ci];
            if (multi) {
                std::memcpy(C_out, C_try.data(), sizeof(double) * C_try.size());
                if (sk != BDA_SIDE_NONE) std::memcpy(side_out, side_try.data(), sizeof(double) * side_try.size());
            }
        }
    }
    if (best_off < 0) return fail(BDA_ESINGULAR, "bda_prepare: every candidate basis window is singular");
    *basis_offset_out = best_off;
    if (resid_out) {
        resid_out[0] = r_first;
        resid_out[1] = r_last;
        resid_out[2] = best;
    }
    return BDA_OK;
}

extern "C" int bda_prepare_lowrank(const double* U, const double* V, int d_in, int r, int d_out,
                                   bda_basis_mode mode, bda_dtype store_dtype, double* Uprime_out,
                                   double* C_out, int* basis_offset_out, double* resid_out)
{
    clear_error();
    if (!U || !V || !Uprime_out || !C_out || !basis_offset_out) return fail(BDA_EINVAL, "bda_prepare_lowrank: NULL argument");
    if (d_in <= 0 || r <= 0 || d_out <= r) return fail(BDA_EINVAL, "bda_prepare_lowrank: need d_in > 0 and 0 < r < d_out");
    if (mode != BDA_BASIS_FIRST && mode != BDA_BASIS_LAST && mode != BDA_BASIS_RESIDUAL_MIN)
        return fail(BDA_EINVAL, "bda_prepare_lowrank: mode must be FIRST, LAST or RESIDUAL_MIN");
    if (store_dtype < BDA_F32 || store_dtype > BDA_F64) return fail(BDA_EDTYPE, "bda_prepare_lowrank: bad store_dtype");
    std::vector<int> offs = candidate_offsets((int)mode, d_out, r, 0);
    const int nc = d_out - r;
    const bool multi = offs.size() > 1;
    const bool want_resid = multi || resid_out;
    std::vector<double> Up_try, C_try;
    if (multi) {
        Up_try.resize((size_t)d_in * r);
        C_try.resize((size_t)r * nc);
    }
    double best = std::numeric_limits<double>::infinity();
    int best_off = -1;
    double r_first = std::nan(""), r_last = std::nan("");
    for (size_t ci = 0; ci < offs.size(); ++ci) {
        const int off = offs[ci];
        double* Up = multi ? Up_try.data() : Uprime_out;
        double* Cd = multi ? C_try.data() : C_out;
        auto rest = [&](int m) { return m < off ? m : m + r; };
        // C = Vb^{-1} V[:, rest]  <=>  (column j of C)^T Vb^T = (column j of V_rest)^T
        std::vector<double> At((size_t)r * r), tau(r);
        for (int i = 0; i < r; ++i)
            for (int j = 0; j < r; ++j) At[(size_t)i * r + j] = V[(int64_t)j * d_out + off + i];
        const int bad = lq_factor(At.data(), r, tau.data());
        double res = 0.0;
        if (bad >= 0) {
            if (!multi) return fail(BDA_ESINGULAR, "bda_prepare_lowrank: basis block (window offset %d) is singular at pivot %d", off, bad);
            res = std::numeric_limits<double>::infinity();
        } else {
            parallel_for(nc, [&](int64_t m) {
                std::vector<double> y(r);
                const int col = rest((int)m);
                for (int j = 0; j < r; ++j) y[j] = V[(int64_t)j * d_out + col];
                lq_solve_row(At.data(), tau.data(), r, y.data());
                for (int j = 0; j < r; ++j) Cd[(int64_t)j * nc + m] = y[j];
            });
            parallel_for(d_in, [&](int64_t i) {          // Uprime = U V[:, window]
                double* up = Up + i * r;
                for (int j = 0; j < r; ++j) up[j] = 0.0;
                for (int k = 0; k < r; ++k) {
                    const double u = U[i * r + k];
                    const double* vb = V + (int64_t)k * d_out + off;
                    for (int j = 0; j < r; ++j) up[j] += u * vb[j];
                }
            });
            if (want_resid) {
                std::vector<double> Ch((size_t)r * nc);
                for (size_t i = 0; i < Ch.size(); ++i) Ch[i] = round_store(Cd[i], (int)store_dtype);
                std::vector<double> part(d_in, 0.0);
                parallel_for(d_in, [&](int64_t i) {
                    std::vector<double> w(d_out, 0.0), rec(nc, 0.0), uh(r);
                    for (int k = 0; k < r; ++k) {
                        const double u = U[i * r + k];
                        const double* v = V + (int64_t)k * d_out;
                        for (int j = 0; j < d_out; ++j) w[j] += u * v[j];
                    }
                    for (int j = 0; j < r; ++j) uh[j] = round_store(Up[i * r + j], (int)store_dtype);
                    for (int j = 0; j < r; ++j) {
                        const double* c = &Ch[(size_t)j * nc];
                        for (int m = 0; m < nc; ++m) rec[m] += uh[j] * c[m];
                    }
                    double s = 0.0;
                    for (int j = 0; j < r; ++j) { const double d = w[off + j] - uh[j]; s += d * d; }
                    for (int m = 0; m < nc; ++m) { const double d = w[rest(m)] - rec[m]; s += d * d; }
                    part[i] = s;
                });
                for (double p : part) res += p;
                res = nan_to_inf(std::sqrt(res));
            }
        }
        if (off == 0) r_first = res;
        if (off == d_out - r) r_last = res;
        const bool take = best_off < 0 ? bad < 0 : res < best;
        if (take) {
            best = res;
            best_off = off;
            if (multi) {
                std::memcpy(Uprime_out, Up_try.data(), sizeof(double) * Up_try.size());
                std::memcpy(C_out, C_try.data(), sizeof(double) * C_try.size());
            }
        }
    }
    if (best_off < 0) return fail(BDA_ESINGULAR, "bda_prepare_lowrank: every candidate basis window is singular");
    *basis_offset_out = best_off;
    if (resid_out) {
        resid_out[0] = r_first;
        resid_out[1] = r_last;
        resid_out[2] = best;
    }
    return BDA_OK;
}
