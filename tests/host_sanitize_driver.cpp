// Host-only driver for the sanitizer build (tests/test_host_sanitizers.py): the library's host
// preparation (bda_prepare.cpp) and the oracle's C loops (oracle/bd_project.c), compiled with
// -fsanitize=address,undefined and run on small problems that reach every mode, side, storage
// type, window position and error path.  It is a test program: it links the two sources side by
// side only to run both under the sanitizers, and cross-checks them through the identity
// out_h W_h[B,:] = c W_h (the BD projection is the dense projection in another basis).
// Exit status 0 = no sanitizer report and every check held.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "bda.h"

extern "C" {
int oracle_num_threads(void);
void oracle_kv_project(const double* c, int64_t ldc, int64_t T, int d_c, int d_h, int G, const int* H,
                       const int* basis_offset, const double* C, int64_t ldC, double* out, int64_t ld_out);
void oracle_dense_project(const double* c, int64_t ldc, int64_t T, int d_c, const double* W, int64_t ldW,
                          int64_t N, double* out, int64_t ld_out);
void oracle_lowrank_linear(const double* x, int64_t ldx, int64_t T, int d_in, int r, int d_out, int basis_offset,
                           const double* Bm, const double* C, double* out, int64_t ld_out, double* hbuf);
}

namespace {

uint64_t g_state = 0x9E3779B97F4A7C15ull;
double rnd()   // uniform in (-1, 1), a fixed sequence
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)((g_state >> 11) & ((1ull << 52) - 1)) / (double)(1ull << 51) - 1.0;
}
std::vector<double> randv(size_t n)
{
    std::vector<double> v(n);
    for (auto& x : v) x = rnd();
    return v;
}

int g_failed = 0;
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::fprintf(stderr, "CHECK failed line %d: %s\n", __LINE__, #cond); \
            ++g_failed;                                                      \
        }                                                                    \
    } while (0)

// one projection, every mode / side / storage type; then the projection identity through the oracle
void prepare_cases()
{
    const int d_c = 40, H = 3, d_h = 8, N = H * d_h, K = d_c - d_h, d_side = 12, T = 7;
    const std::vector<double> W = randv((size_t)d_c * N), Wq = randv((size_t)d_side * N), Wo = randv((size_t)N * d_side);
    const std::vector<double> c = randv((size_t)T * d_c);
    std::vector<double> dense((size_t)T * N);
    oracle_dense_project(c.data(), d_c, T, d_c, W.data(), N, N, dense.data(), N);
    const bda_basis_mode modes[] = {BDA_BASIS_FIRST, BDA_BASIS_LAST, BDA_BASIS_RESIDUAL_MIN, BDA_BASIS_OFFSET_SEARCH, BDA_BASIS_EXPLICIT};
    const bda_dtype stores[] = {BDA_F64, BDA_F32, BDA_F16, BDA_BF16};
    for (bda_basis_mode mode : modes)
        for (bda_dtype st : stores)
            for (int side = 0; side < 3; ++side) {
                std::vector<double> C((size_t)K * N), side_out((size_t)d_side * N);
                double resid[3];
                int off = -1;
                const double* sp = side == 1 ? Wq.data() : side == 2 ? Wo.data() : nullptr;
                const int rc = bda_prepare(W.data(), N, d_c, H, d_h, sp, side == 1 ? N : d_side, d_side, (bda_side)side, mode, 16, st,
                                           C.data(), sp ? side_out.data() : nullptr, &off, resid);
                CHECK(rc == BDA_OK);
                CHECK(off >= 0 && off <= K);
                if (mode == BDA_BASIS_EXPLICIT) CHECK(off == 16);
                // out_h A_h = c W_h with A_h = W_h[B, :]
                std::vector<double> out((size_t)T * N);
                const int Hs[1] = {H}, offs[1] = {off};
                oracle_kv_project(c.data(), d_c, T, d_c, d_h, 1, Hs, offs, C.data(), N, out.data(), N);
                double worst = 0;
                for (int t = 0; t < T; ++t)
                    for (int h = 0; h < H; ++h)
                        for (int j = 0; j < d_h; ++j) {
                            double s = 0;
                            for (int i = 0; i < d_h; ++i) s += out[(size_t)t * N + h * d_h + i] * W[(size_t)(off + i) * N + h * d_h + j];
                            worst = std::fmax(worst, std::fabs(s - dense[(size_t)t * N + h * d_h + j]));
                        }
                CHECK(worst < 1e-9);
            }
    // error paths: NULL, bad sizes, singular window (two equal basis rows in head 1)
    std::vector<double> C((size_t)K * N);
    int off = 0;
    CHECK(bda_prepare(nullptr, N, d_c, H, d_h, nullptr, 0, 0, BDA_SIDE_NONE, BDA_BASIS_FIRST, 0, BDA_F64, C.data(), nullptr, &off, nullptr) == BDA_EINVAL);
    CHECK(bda_prepare(W.data(), N, d_c, H, d_c, nullptr, 0, 0, BDA_SIDE_NONE, BDA_BASIS_FIRST, 0, BDA_F64, C.data(), nullptr, &off, nullptr) == BDA_EINVAL);
    CHECK(bda_prepare(W.data(), N, d_c, H, d_h, nullptr, 0, 0, BDA_SIDE_NONE, BDA_BASIS_EXPLICIT, K + 1, BDA_F64, C.data(), nullptr, &off, nullptr) == BDA_EINVAL);
    std::vector<double> Ws = W;
    for (int j = 0; j < d_h; ++j) Ws[(size_t)3 * N + d_h + j] = Ws[(size_t)5 * N + d_h + j];
    CHECK(bda_prepare(Ws.data(), N, d_c, H, d_h, nullptr, 0, 0, BDA_SIDE_NONE, BDA_BASIS_FIRST, 0, BDA_F64, C.data(), nullptr, &off, nullptr) == BDA_ESINGULAR);
    CHECK(bda_last_error()[0] != 0);
    // a strided weight matrix (ldw > N) and two groups with different windows through the oracle
    const int ldw = N + 5;
    std::vector<double> Wp((size_t)d_c * ldw, 1e300);
    for (int i = 0; i < d_c; ++i)
        for (int j = 0; j < N; ++j) Wp[(size_t)i * ldw + j] = W[(size_t)i * N + j];
    std::vector<double> C2((size_t)K * N);
    CHECK(bda_prepare(Wp.data(), ldw, d_c, H, d_h, nullptr, 0, 0, BDA_SIDE_NONE, BDA_BASIS_LAST, 0, BDA_F64, C2.data(), nullptr, &off, nullptr) == BDA_OK);
    CHECK(off == K);
    const int H2[2] = {2, 1}, off2[2] = {K, K};
    std::vector<double> out((size_t)T * (N + 3), -7.0);
    oracle_kv_project(c.data(), d_c, T, d_c, d_h, 2, H2, off2, C2.data(), N, out.data(), N + 3);
    for (int t = 0; t < T; ++t) CHECK(out[(size_t)t * (N + 3) + N] == -7.0);
    oracle_kv_project(c.data(), d_c, 0, d_c, d_h, 2, H2, off2, C2.data(), N, out.data(), N + 3);   // no tokens
}

void lowrank_cases()
{
    const int d_in = 14, r = 5, d_out = 17, T = 6;
    const std::vector<double> U = randv((size_t)d_in * r), V = randv((size_t)r * d_out), x = randv((size_t)T * d_in);
    std::vector<double> xu((size_t)T * r), ref((size_t)T * d_out);
    oracle_dense_project(x.data(), d_in, T, d_in, U.data(), r, r, xu.data(), r);
    oracle_dense_project(xu.data(), r, T, r, V.data(), d_out, d_out, ref.data(), d_out);
    const bda_basis_mode modes[] = {BDA_BASIS_FIRST, BDA_BASIS_LAST, BDA_BASIS_RESIDUAL_MIN};
    for (bda_basis_mode mode : modes)
        for (bda_dtype st : {BDA_F64, BDA_F16, BDA_BF16}) {
            std::vector<double> Up((size_t)d_in * r), C((size_t)r * (d_out - r)), out((size_t)T * d_out), h((size_t)T * r);
            double resid[3];
            int off = -1;
            CHECK(bda_prepare_lowrank(U.data(), V.data(), d_in, r, d_out, mode, st, Up.data(), C.data(), &off, resid) == BDA_OK);
            CHECK(off == 0 || off == d_out - r);
            oracle_lowrank_linear(x.data(), d_in, T, d_in, r, d_out, off, Up.data(), C.data(), out.data(), d_out, h.data());
            double worst = 0;
            for (size_t i = 0; i < out.size(); ++i) worst = std::fmax(worst, std::fabs(out[i] - ref[i]));
            CHECK(worst < 1e-9);
        }
    std::vector<double> Up((size_t)d_in * r), C((size_t)r * (d_out - r));
    int off = 0;
    CHECK(bda_prepare_lowrank(U.data(), V.data(), d_in, r, r, BDA_BASIS_FIRST, BDA_F64, Up.data(), C.data(), &off, nullptr) == BDA_EINVAL);
    CHECK(bda_prepare_lowrank(nullptr, V.data(), d_in, r, d_out, BDA_BASIS_FIRST, BDA_F64, Up.data(), C.data(), &off, nullptr) == BDA_EINVAL);
}

}  // namespace

int main()
{
    CHECK(oracle_num_threads() >= 1);
    CHECK(bda_version() > 0);
    prepare_cases();
    lowrank_cases();
    if (g_failed) {
        std::fprintf(stderr, "%d checks failed\n", g_failed);
        return 1;
    }
    std::puts("host sanitizer driver: all checks passed");
    return 0;
}
