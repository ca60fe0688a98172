// Host-side sanitizer driver (AddressSanitizer + UndefinedBehaviorSanitizer): exercises the
// oracle's C functions on small inputs and every host-only path of the C ABI (shape / workspace /
// plan queries over many descriptors, and the entry points' validation, which fails before
// anything is launched).  No GPU is touched.  Prints "san ok" and exits 0 when nothing fired.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "cac.h"

extern "C" {
void oracle_pooled_shape(int64_t, int64_t, int64_t, int64_t, int, int64_t *, int64_t *);
void oracle_avgpool(const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int, double *);
void oracle_maxpool(const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int, double *);
int oracle_inflate(const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int, double *);
void oracle_conv_fwd(const double *, const double *, const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                     int64_t, int64_t, int64_t, int64_t, double *);
void oracle_conv_dw(const double *, const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                    int64_t, int64_t, double *);
void oracle_conv_dx(const double *, const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                    int64_t, int64_t, double *);
void oracle_tile_sums(const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t,
                      int64_t, int64_t, int64_t, int64_t, double *);
void oracle_bias_grad(const double *, int64_t, int64_t, int64_t, int64_t, double *);
double oracle_cosine(const double *, const double *, int64_t);
}

static int fails = 0;
#define CHECK(c)                                                        \
    do {                                                                \
        if (!(c)) {                                                     \
            fprintf(stderr, "%s:%d: CHECK(%s) failed\n", __FILE__, __LINE__, #c); \
            ++fails;                                                    \
        }                                                               \
    } while (0)

static void oracle_cases()
{
    struct G { int64_t N, C, K, H, W, R, S, sh, sw, ph, pw, kh, kw; };
    const G gs[] = {{2, 3, 4, 7, 9, 3, 3, 1, 1, 1, 1, 2, 2}, {1, 2, 3, 8, 5, 3, 2, 2, 1, 1, 0, 2, 4}, {2, 1, 2, 5, 5, 1, 1, 2, 2, 0, 0, 4, 4},
                    {1, 2, 2, 6, 6, 5, 5, 1, 1, 2, 2, 3, 2}, {1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 2, 2}};
    for (const G &g : gs) {
        const int64_t P = (g.H + 2 * g.ph - g.R) / g.sh + 1, Q = (g.W + 2 * g.pw - g.S) / g.sw + 1;
        int64_t Hp, Wp;
        oracle_pooled_shape(g.H, g.W, g.kh, g.kw, 0, &Hp, &Wp);
        std::vector<double> X(g.N * g.C * g.H * g.W), Wt(g.K * g.C * g.R * g.S), b(g.K), dY(g.N * g.K * P * Q);
        uint32_t s = 12345u;
        auto rnd = [&]() { s = s * 1664525u + 1013904223u; return (double)(int)(s >> 8) / (1 << 23) - 1.0; };
        for (auto &v : X) v = rnd() > 0 ? rnd() : 0.0;
        for (auto &v : Wt) v = rnd();
        for (auto &v : b) v = rnd();
        for (auto &v : dY) v = rnd();
        std::vector<double> Z(g.N * g.C * Hp * Wp), Zm(Z.size()), Xh(X.size()), Y(dY.size()), dW(Wt.size()), dW2(Wt.size()), dX(X.size()),
            db(g.K), T(g.N * g.K * Hp * Wp);
        oracle_avgpool(X.data(), g.N, g.C, g.H, g.W, g.kh, g.kw, 0, Z.data());
        oracle_maxpool(X.data(), g.N, g.C, g.H, g.W, g.kh, g.kw, 0, Zm.data());
        CHECK(oracle_inflate(Z.data(), g.N, g.C, g.H, g.W, g.kh, g.kw, 0, Xh.data()) == 0);
        oracle_conv_fwd(X.data(), Wt.data(), b.data(), g.N, g.C, g.K, g.H, g.W, g.R, g.S, g.sh, g.sw, g.ph, g.pw, Y.data());
        oracle_conv_dw(Xh.data(), dY.data(), g.N, g.C, g.K, g.H, g.W, g.R, g.S, g.sh, g.sw, g.ph, g.pw, dW.data());
        oracle_conv_dx(Wt.data(), dY.data(), g.N, g.C, g.K, g.H, g.W, g.R, g.S, g.sh, g.sw, g.ph, g.pw, dX.data());
        oracle_bias_grad(dY.data(), g.N, g.K, P, Q, db.data());
        // the regrouped form, tap by tap, against the inflated form
        for (int64_t r = 0; r < g.R; ++r)
            for (int64_t t = 0; t < g.S; ++t) {
                oracle_tile_sums(dY.data(), g.N, g.C, g.K, g.H, g.W, g.R, g.S, g.sh, g.sw, g.ph, g.pw, g.kh, g.kw, r, t, T.data());
                for (int64_t o = 0; o < g.K; ++o)
                    for (int64_t c = 0; c < g.C; ++c) {
                        double a = 0;
                        for (int64_t n = 0; n < g.N; ++n)
                            for (int64_t i = 0; i < Hp * Wp; ++i) a += Z[(n * g.C + c) * Hp * Wp + i] * T[(n * g.K + o) * Hp * Wp + i];
                        dW2[((o * g.C + c) * g.R + r) * g.S + t] = a;
                    }
            }
        for (size_t i = 0; i < dW.size(); ++i) CHECK(dW[i] - dW2[i] < 1e-9 && dW2[i] - dW[i] < 1e-9);
        double nrm = 0;
        for (double v : dW) nrm += v * v;
        CHECK(nrm == 0 || oracle_cosine(dW.data(), dW2.data(), (int64_t)dW.size()) > 0.999999);
        for (size_t i = 0; i < Z.size(); ++i) CHECK(Zm[i] >= Z[i] - 1e-12);
    }
    double z[6] = {0}, xh[7 * 8];
    CHECK(oracle_inflate(z, 1, 1, 7, 8, 2, 4, 1, xh) == -1); // floor/drop with a remainder: refused, nothing written
}

static cac_desc desc(int N, int C, int K, int H, int W, int R, int st, int pad, int kh, int kw, int dtype, int algo)
{
    cac_desc d;
    memset(&d, 0, sizeof d);
    d.size = sizeof d;
    d.N = N; d.C_in = C; d.C_out = K; d.H = H; d.W = W; d.R = R; d.S = R; d.stride_h = st; d.stride_w = st; d.pad_h = pad; d.pad_w = pad;
    d.pool_kh = kh; d.pool_kw = kw; d.edge_mode = CAC_EDGE_CEIL_VALID; d.dtype = dtype; d.has_bias = 1; d.pool_mode = CAC_POOL_MEAN;
    d.dw_algo = algo;
    return d;
}

static void abi_cases()
{
    char buf[512];
    const int Hs[] = {1, 2, 4, 7, 8, 14, 16, 28, 30, 32, 56}, Cs[] = {1, 16, 33, 64, 96, 128, 200, 512, 2048}, Ks[] = {1, 2, 3, 4, 8};
    long queried = 0;
    for (int H : Hs)
        for (int C : Cs)
            for (int R : {1, 3, 5, 7})
                for (int st : {1, 2})
                    for (int k : Ks)
                        for (int dt : {CAC_F32, CAC_BF16})
                            for (int algo : {CAC_DW_INFLATE, CAC_DW_REDUCED_K}) {
                                cac_desc d = desc(H > 28 ? 3 : 9, C, C > 512 ? 64 : C + 31, H, H + (k == 3), R, st, R / 2, k, k == 3 ? 2 : k, dt, algo);
                                int32_t P, Q, Hp, Wp;
                                size_t zb, xb, ws;
                                uint64_t fl;
                                if (cac_out_shape(&d, &P, &Q) != CAC_OK) continue;
                                CHECK(cac_pooled_shape(&d, &Hp, &Wp, &zb, &xb) == CAC_OK);
                                CHECK(zb <= xb || k == 1);
                                for (int op = CAC_OP_FWD_AND_COMPRESS; op <= CAC_OP_BN_BWD; ++op) {
                                    CHECK(cac_workspace_size(&d, op, &ws) == CAC_OK);
                                    CHECK(cac_describe_plan(&d, op, buf, sizeof buf) == CAC_OK);
                                    CHECK(strlen(buf) < sizeof buf);
                                }
                                CHECK(cac_describe_plan(&d, CAC_OP_BWD_WEIGHT_COMPRESSED, buf, 8) == CAC_OK && strlen(buf) < 8);
                                CHECK(cac_dw_executed_flops(&d, &fl) == CAC_OK && fl > 0);
                                ++queried;
                            }
    CHECK(queried > 1000);
    // validation of the entry points: every one of these fails before anything is launched
    cac_desc d = desc(2, 4, 4, 8, 8, 3, 1, 1, 2, 2, CAC_BF16, 0);
    alignas(16) static char mem[64];
    CHECK(conv_fwd_and_compress(&d, nullptr, mem, mem, mem, mem, nullptr, 0, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(conv_fwd_and_compress(&d, mem + 2, mem, mem, mem, mem, nullptr, 0, nullptr) == CAC_ERR_ALIGNMENT);
    CHECK(conv_bwd_weight_compressed(&d, mem, mem, nullptr, nullptr, 0, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(conv_bwd_weight_compressed_noalloc(&d, mem, nullptr, mem, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(conv_bwd_data(&d, mem, mem, mem + 8, nullptr, 0, nullptr) == CAC_ERR_ALIGNMENT);
    CHECK(conv_bwd_weight_and_data(&d, mem, mem, mem, mem, nullptr, nullptr, 0, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(cac_compress(&d, mem, nullptr, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(conv_bwd_bias(&d, nullptr, mem, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(cac_grad_cosine(&d, mem, mem, nullptr, nullptr, 0, nullptr) == CAC_ERR_INVALID_ARG);
    CHECK(strlen(cac_last_error()) > 0);
    cac_desc big = desc(1 << 15, 1 << 20, 4, 1 << 15, 1 << 14, 3, 1, 1, 2, 2, CAC_BF16, 0); // extents whose product wraps 64 bits
    size_t ws;
    CHECK(cac_workspace_size(&big, CAC_OP_BWD_DATA, &ws) == CAC_ERR_UNSUPPORTED);
    big = desc(2, 4, 4, 8, 8, 3, 1, 0x7fffffff, 2, 2, CAC_BF16, 0); // padding that overflows int arithmetic
    CHECK(cac_workspace_size(&big, CAC_OP_BWD_DATA, &ws) != CAC_OK);
    d.size = 12;
    CHECK(cac_workspace_size(&d, CAC_OP_BWD_DATA, &ws) == CAC_ERR_INVALID_ARG);
    CHECK(cac_pooled_shape(nullptr, nullptr, nullptr, nullptr, nullptr) == CAC_ERR_INVALID_ARG);
}

int main()
{
    oracle_cases();
    abi_cases();
    if (fails) {
        fprintf(stderr, "%d checks failed\n", fails);
        return 1;
    }
    printf("san ok\n");
    return 0;
}
