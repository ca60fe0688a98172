/*
 * cac_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * Plain, slow, fp64 CPU statement of what the compressed-activation convolution
 * training step computes ("Compressing Activation Maps" section and its figure of
 * the compression scheme).  It exists so that the HIP library can be checked
 * against something that can be verified against the paper by eye.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it; the product
 * path never does.  It shares no code with the HIP path.
 *
 * All tensors are dense row-major fp64:
 *   X  [N][C][H][W]      layer input (activation)
 *   Wt [K][C][R][S]      filter
 *   b  [K]               bias (may be NULL)
 *   Y  [N][K][P][Q]      layer output,  P = (H + 2*ph - R)/sh + 1 (floor), same for Q
 *   Z  [N][C][Hp][Wp]    pooled activation
 *   dY [N][K][P][Q], dW [K][C][R][S], dX [N][C][H][W], db [K]
 *
 * Readings of the paper taken here (it leaves them open):
 *   - inflation replicates each pooled value over the tile it was averaged from
 *     (the compression figure colours a tile of X and its mean alike);
 *   - tiles are kh x kw, start at the origin, do not overlap, and cover single
 *     channel maps only (same figure);
 *   - edge mode 0 ("ceil/valid"): Hp = ceil(H/kh); a ragged last tile is averaged
 *     over the elements it really has.  Edge mode 1 ("floor/drop"): Hp =
 *     floor(H/kh), remainder rows/columns are not pooled (this is what the
 *     per-layer memory table's byte counts imply).  The paper does not say what
 *     dropped rows inflate to, so oracle_inflate refuses that case (returns -1)
 *     instead of inventing a value; floor/drop with tiles that divide the map is
 *     the same as ceil/valid;
 *   - the cosine of the layer-sensitivity equation is undefined for a zero
 *     gradient; oracle_cosine returns 0 there (reading: "no agreement").
 *
 * OpenMP is used only over independent outputs; every output element is still a
 * single sequential sum in the order written here.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_EDGE_CEIL_VALID 0
#define ORACLE_EDGE_FLOOR_DROP 1

static int64_t out_extent(int64_t in, int64_t pad, int64_t filt, int64_t stride)
{
    int64_t span = in + 2 * pad - filt;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* Book-keeping of the saved record: pooled extents and byte counts
 * (memory-footprint table; compression section: the record holds nothing but
 * Z, the original shape and the tile size). */
void oracle_pooled_shape(int64_t H, int64_t W, int64_t kh, int64_t kw, int edge_mode,
                         int64_t *Hp, int64_t *Wp)
{
    if (edge_mode == ORACLE_EDGE_FLOOR_DROP) {
        *Hp = H / kh;
        *Wp = W / kw;
    } else {
        *Hp = (H + kh - 1) / kh;
        *Wp = (W + kw - 1) / kw;
    }
}

void oracle_out_shape(int64_t H, int64_t W, int64_t R, int64_t S, int64_t sh, int64_t sw,
                      int64_t ph, int64_t pw, int64_t *P, int64_t *Q)
{
    *P = out_extent(H, ph, R, sh);
    *Q = out_extent(W, pw, S, sw);
}

/* Compression: Z = block means of X (compression section; compression figure). */
void oracle_avgpool(const double *X, int64_t N, int64_t C, int64_t H, int64_t W,
                    int64_t kh, int64_t kw, int edge_mode, double *Z)
{
    int64_t Hp, Wp;
    oracle_pooled_shape(H, W, kh, kw, edge_mode, &Hp, &Wp);
    int64_t planes = N * C;
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        const double *x = X + pl * H * W;
        double *z = Z + pl * Hp * Wp;
        for (int64_t i = 0; i < Hp; ++i) {
            for (int64_t j = 0; j < Wp; ++j) {
                double sum = 0.0;
                int64_t count = 0;
                for (int64_t a = 0; a < kh; ++a) {
                    int64_t h = i * kh + a;
                    if (h >= H) continue;
                    for (int64_t bcol = 0; bcol < kw; ++bcol) {
                        int64_t w = j * kw + bcol;
                        if (w >= W) continue;
                        sum += x[h * W + w];
                        ++count;
                    }
                }
                z[i * Wp + j] = sum / (double)count;
            }
        }
    }
}

/* Compression with the tile maximum instead of the mean.  The compression section
 * says other forms of pooling are feasible without defining one; the reading taken
 * here: same tiles, same edge modes, Z = the largest of the elements a tile really
 * has; inflation is oracle_inflate unchanged (the maximum repeated over its tile). */
void oracle_maxpool(const double *X, int64_t N, int64_t C, int64_t H, int64_t W,
                    int64_t kh, int64_t kw, int edge_mode, double *Z)
{
    int64_t Hp, Wp;
    oracle_pooled_shape(H, W, kh, kw, edge_mode, &Hp, &Wp);
    int64_t planes = N * C;
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        const double *x = X + pl * H * W;
        double *z = Z + pl * Hp * Wp;
        for (int64_t i = 0; i < Hp; ++i) {
            for (int64_t j = 0; j < Wp; ++j) {
                double best = x[i * kh * W + j * kw]; /* a tile's first element always exists */
                for (int64_t a = 0; a < kh; ++a) {
                    int64_t h = i * kh + a;
                    if (h >= H) continue;
                    for (int64_t bcol = 0; bcol < kw; ++bcol) {
                        int64_t w = j * kw + bcol;
                        if (w >= W) continue;
                        if (x[h * W + w] > best) best = x[h * W + w];
                    }
                }
                z[i * Wp + j] = best;
            }
        }
    }
}

/* Decompression (compression figure, caption): Z is brought back to H x W by
 * replicating every pooled value over its tile.  Returns 0, or -1 without
 * writing anything when the tiles do not cover the map (floor/drop with a
 * remainder): the paper defines no value for the uncovered pixels. */
int oracle_inflate(const double *Z, int64_t N, int64_t C, int64_t H, int64_t W,
                    int64_t kh, int64_t kw, int edge_mode, double *Xhat)
{
    int64_t Hp, Wp;
    oracle_pooled_shape(H, W, kh, kw, edge_mode, &Hp, &Wp);
    if (Hp * kh < H || Wp * kw < W) return -1;
    int64_t planes = N * C;
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        const double *z = Z + pl * Hp * Wp;
        double *xh = Xhat + pl * H * W;
        for (int64_t h = 0; h < H; ++h) {
            int64_t i = h / kh;
            for (int64_t w = 0; w < W; ++w) {
                int64_t j = w / kw;
                xh[h * W + w] = z[i * Wp + j];
            }
        }
    }
    return 0;
}

/* Forward convolution Y = X * W + b, zero padding (compression figure). */
void oracle_conv_fwd(const double *X, const double *Wt, const double *b,
                     int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                     int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                     double *Y)
{
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t o = 0; o < K; ++o) {
            for (int64_t p = 0; p < P; ++p) {
                for (int64_t q = 0; q < Q; ++q) {
                    double acc = b ? b[o] : 0.0;
                    for (int64_t c = 0; c < C; ++c) {
                        for (int64_t r = 0; r < R; ++r) {
                            int64_t h = p * sh + r - ph;
                            if (h < 0 || h >= H) continue;
                            for (int64_t s = 0; s < S; ++s) {
                                int64_t w = q * sw + s - pw;
                                if (w < 0 || w >= W) continue;
                                acc += Wt[((o * C + c) * R + r) * S + s] *
                                       X[((n * C + c) * H + h) * W + w];
                            }
                        }
                    }
                    Y[((n * K + o) * P + p) * Q + q] = acc;
                }
            }
        }
    }
}

/* One weight-gradient entry: dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] *
 * A[n,c,p*sh+r-ph,q*sw+s-pw], out-of-range terms are zero.  A is the activation
 * the backward pass has: the inflated Z for the compressed step, X itself for
 * the exact gradient (weight-gradient formula in the compression figure). */
static double dw_entry(const double *A, const double *dY,
                       int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                       int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                       int64_t P, int64_t Q, int64_t o, int64_t c, int64_t r, int64_t s)
{
    (void)R; (void)S;
    double acc = 0.0;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t p = 0; p < P; ++p) {
            int64_t h = p * sh + r - ph;
            if (h < 0 || h >= H) continue;
            for (int64_t q = 0; q < Q; ++q) {
                int64_t w = q * sw + s - pw;
                if (w < 0 || w >= W) continue;
                acc += dY[((n * K + o) * P + p) * Q + q] * A[((n * C + c) * H + h) * W + w];
            }
        }
    }
    return acc;
}

void oracle_conv_dw(const double *A, const double *dY,
                    int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                    int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                    double *dW)
{
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
    int64_t total = K * C * R * S;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t e = 0; e < total; ++e) {
        int64_t s = e % S, r = (e / S) % R, c = (e / (S * R)) % C, o = e / (S * R * C);
        dW[e] = dw_entry(A, dY, N, C, K, H, W, R, S, sh, sw, ph, pw, P, Q, o, c, r, s);
    }
}

/* Same sums, only for the listed flat indices into dW[K][C][R][S] (each entry is
 * an independent dot product, so a sample is as good a check as the whole). */
void oracle_conv_dw_entries(const double *A, const double *dY,
                            int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                            int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                            const int64_t *flat_index, int64_t n_index, double *out)
{
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_index; ++i) {
        int64_t e = flat_index[i];
        int64_t s = e % S, r = (e / S) % R, c = (e / (S * R)) % C, o = e / (S * R * C);
        out[i] = dw_entry(A, dY, N, C, K, H, W, R, S, sh, sw, ph, pw, P, Q, o, c, r, s);
    }
}

/* Tile sums of dY for one filter tap (r, s): the inflated activation is constant on a pooling
 * tile, so in the weight-gradient formula of the compression figure all pixels (p, q) whose tap
 * lands in tile (i, j) meet the same value Z[n,c,i,j]; collecting them first gives
 *   dW[o,c,r,s] = sum_{n,i,j} Z[n,c,i,j] * T[n,o,i,j],
 *   T[n,o,i,j]  = sum of dY[n,o,p,q] over the (p, q) with
 *                 h = p*sh + r - ph inside [0,H), w = q*sw + s - pw inside [0,W), h/kh = i, w/kw = j.
 * (The same real number as the formula applied to the inflated Z: a regrouping of its terms.)
 * T [N][K][Hp][Wp], ceil/valid tiles. */
void oracle_tile_sums(const double *dY,
                      int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                      int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                      int64_t kh, int64_t kw, int64_t r, int64_t s, double *T)
{
    (void)C;
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
    int64_t Hp = (H + kh - 1) / kh, Wp = (W + kw - 1) / kw;
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < N * K; ++pl) {
        double *t = T + pl * Hp * Wp;
        const double *g = dY + pl * P * Q;
        for (int64_t i = 0; i < Hp * Wp; ++i) t[i] = 0.0;
        for (int64_t p = 0; p < P; ++p) {
            int64_t h = p * sh + r - ph;
            if (h < 0 || h >= H) continue;
            for (int64_t q = 0; q < Q; ++q) {
                int64_t w = q * sw + s - pw;
                if (w < 0 || w >= W) continue;
                t[(h / kh) * Wp + (w / kw)] += g[p * Q + q];
            }
        }
    }
}

/* Data gradient dX = W^T * dY, written as the adjoint scatter of the forward sum
 * (data-gradient formula in the compression figure).  It never sees X or Z. */
void oracle_conv_dx(const double *Wt, const double *dY,
                    int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                    int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                    double *dX)
{
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *dx = dX + n * C * H * W;
        for (int64_t i = 0; i < C * H * W; ++i) dx[i] = 0.0;
        for (int64_t o = 0; o < K; ++o) {
            for (int64_t p = 0; p < P; ++p) {
                for (int64_t q = 0; q < Q; ++q) {
                    double g = dY[((n * K + o) * P + p) * Q + q];
                    for (int64_t c = 0; c < C; ++c) {
                        for (int64_t r = 0; r < R; ++r) {
                            int64_t h = p * sh + r - ph;
                            if (h < 0 || h >= H) continue;
                            for (int64_t s = 0; s < S; ++s) {
                                int64_t w = q * sw + s - pw;
                                if (w < 0 || w >= W) continue;
                                dx[(c * H + h) * W + w] += Wt[((o * C + c) * R + r) * S + s] * g;
                            }
                        }
                    }
                }
            }
        }
    }
}

/* Same sums for listed flat indices into dX[N][C][H][W], gather form. */
void oracle_conv_dx_entries(const double *Wt, const double *dY,
                            int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                            int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                            const int64_t *flat_index, int64_t n_index, double *out)
{
    (void)N;
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_index; ++i) {
        int64_t e = flat_index[i];
        int64_t w = e % W, h = (e / W) % H, c = (e / (W * H)) % C, n = e / (W * H * C);
        double acc = 0.0;
        for (int64_t o = 0; o < K; ++o) {
            for (int64_t p = 0; p < P; ++p) {
                int64_t r = h + ph - p * sh;
                if (r < 0 || r >= R) continue;
                for (int64_t q = 0; q < Q; ++q) {
                    int64_t s = w + pw - q * sw;
                    if (s < 0 || s >= S) continue;
                    acc += Wt[((o * C + c) * R + r) * S + s] * dY[((n * K + o) * P + p) * Q + q];
                }
            }
        }
        out[i] = acc;
    }
}

/* Forward outputs for listed flat indices into Y[N][K][P][Q]. */
void oracle_conv_fwd_entries(const double *X, const double *Wt, const double *b,
                             int64_t N, int64_t C, int64_t K, int64_t H, int64_t W,
                             int64_t R, int64_t S, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                             const int64_t *flat_index, int64_t n_index, double *out)
{
    (void)N;
    int64_t P = out_extent(H, ph, R, sh), Q = out_extent(W, pw, S, sw);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_index; ++i) {
        int64_t e = flat_index[i];
        int64_t q = e % Q, p = (e / Q) % P, o = (e / (Q * P)) % K, n = e / (Q * P * K);
        double acc = b ? b[o] : 0.0;
        for (int64_t c = 0; c < C; ++c) {
            for (int64_t r = 0; r < R; ++r) {
                int64_t h = p * sh + r - ph;
                if (h < 0 || h >= H) continue;
                for (int64_t s = 0; s < S; ++s) {
                    int64_t w = q * sw + s - pw;
                    if (w < 0 || w >= W) continue;
                    acc += Wt[((o * C + c) * R + r) * S + s] * X[((n * C + c) * H + h) * W + w];
                }
            }
        }
        out[i] = acc;
    }
}

/* Bias gradient db[o] = sum over n,p,q of dY (bias-gradient formula, same figure). */
void oracle_bias_grad(const double *dY, int64_t N, int64_t K, int64_t P, int64_t Q, double *db)
{
    for (int64_t o = 0; o < K; ++o) {
        double acc = 0.0;
        for (int64_t n = 0; n < N; ++n)
            for (int64_t i = 0; i < P * Q; ++i) acc += dY[(n * K + o) * P * Q + i];
        db[o] = acc;
    }
}

/* Cosine similarity of two gradients (layer-sensitivity equation). */
double oracle_cosine(const double *a, const double *b, int64_t n)
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        ab += a[i] * b[i];
        aa += a[i] * a[i];
        bb += b[i] * b[i];
    }
    if (aa == 0.0 || bb == 0.0) return 0.0;
    return ab / (sqrt(aa) * sqrt(bb));
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    n = omp_get_max_threads();
#endif
    return n;
}
