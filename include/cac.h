/*
 * cac.h -- C ABI of the compressed-activation convolution training step for
 * AMD MI355X (gfx950).
 *
 * The method (paper section "Compressing Activation Maps" and its figure of the
 * compression scheme): a convolution layer computes its forward output from the
 * full-resolution input X; what it keeps for the backward pass is not X but
 * Z = k x k average pooling of X.  In the backward pass the weight gradient is
 * computed from Z inflated back to the shape of X (every pooled value repeated
 * over the tile it came from); the data gradient and the bias gradient do not
 * depend on the activation and stay exact.
 *
 * This library never writes the inflated activation to memory: the weight
 * gradient kernel reads Z and expands it in registers / LDS.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers (HIP global memory) owned by the
 *     caller, dense, NCHW / KCRS row-major, at least 16-byte aligned.  (NCHW is the
 *     only layout: the pixel sum of the weight gradient wants pixels contiguous.)
 *   - The weight gradient's pixel slices are always summed in a fixed order: results
 *     are reproducible bit for bit; there is no atomic mode.
 *   - dtype CAC_F32 : X, W, b, Y, Z, dY, dX are float;  dW is float.
 *     dtype CAC_BF16: X, W, b, Y, Z, dY, dX are bfloat16 (round to nearest even
 *     on every store), arithmetic accumulates in float; dW is float.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     work is enqueued on it; no entry point synchronises, allocates device
 *     memory, or keeps state between calls.
 *   - `ws` is caller-owned device scratch of at least cac_workspace_size()
 *     bytes (may be NULL when that size is 0).  Its contents are undefined
 *     after a call.
 *   - Return value: CAC_OK (0) or a negative cac_status.  Validation happens
 *     before anything is launched, so a failing call has touched no buffer.
 *     cac_last_error() gives a thread-local message for the last failing call.
 *   - The first launch of a kernel variant in a process sets that kernel's attributes (once,
 *     thread-safe).  Under HIP stream capture, run the same calls once eagerly before
 *     capturing them.
 *   - Extents: N, C_in, C_out, H, W <= 2^24; filter, stride, padding, pooling tile <= 2^15;
 *     every tensor below 2^31 elements (CAC_ERR_UNSUPPORTED otherwise).
 *   - No C++ exception crosses this boundary.
 */
#ifndef CAC_H
#define CAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CAC_VERSION 303 /* major*10000 + minor*100 + patch */

typedef enum cac_status {
    CAC_OK = 0,
    CAC_ERR_INVALID_ARG = -1,      /* NULL pointer, non-positive extent, bad enum, bad desc.size */
    CAC_ERR_UNSUPPORTED = -2,      /* valid request this build has no kernel for */
    CAC_ERR_WORKSPACE_TOO_SMALL = -3,
    CAC_ERR_ALIGNMENT = -4,        /* a tensor pointer is not 16-byte aligned */
    CAC_ERR_LAUNCH_FAILED = -5     /* HIP reported an error at launch */
} cac_status;

typedef enum cac_dtype { CAC_F32 = 0, CAC_BF16 = 1 } cac_dtype;

/* How a pooling tile that sticks out over the edge is treated (the paper is
 * silent; its memory table implies FLOOR_DROP, every stated invariant needs
 * CEIL_VALID):
 *   CEIL_VALID : Hp = ceil(H/kh); a ragged tile is averaged over the elements it
 *                really has; every pixel of X is covered.            (default)
 *   FLOOR_DROP : Hp = floor(H/kh); only shape/byte queries accept it when kh
 *                does not divide H (or kw W); the kernels then return
 *                CAC_ERR_UNSUPPORTED because the paper does not define what the
 *                dropped rows inflate to. */
typedef enum cac_edge_mode { CAC_EDGE_CEIL_VALID = 0, CAC_EDGE_FLOOR_DROP = 1 } cac_edge_mode;

/* What a pooling tile is reduced to.  The paper's experiments use the mean; its
 * compression section names other forms of pooling as feasible without defining
 * one.  MAX is this library's reading of that remark: Z = the largest element the
 * tile really has (same tiles and edge modes as the mean; stored exactly, a
 * maximum needs no rounding), and the backward pass inflates Z in the same way.
 * Inputs are taken to be free of NaN. */
typedef enum cac_pool_mode { CAC_POOL_MEAN = 0, CAC_POOL_MAX = 1 } cac_pool_mode;

/* How the weight gradient is evaluated.  Both give the same real number (the weight-gradient
 * formula of the compression figure applied to the inflated Z); they differ in the work done
 * and in rounding.
 *   INFLATE   : Z is expanded in LDS and multiplied with dY pixel by pixel (the fused kernel the
 *               compression section names as its goal).                               (default)
 *   REDUCED_K : the inflated activation is constant on a tile, so the sum over the pixels of a
 *               tile is Z times the sum of the dY values that meet it there:
 *                 dW[o,c,r,s] = sum_{n,i,j} Z[n,c,i,j] * S_rs[n,o,i,j],
 *                 S_rs[n,o,i,j] = sum of dY[n,o,p,q] over the (p,q) with
 *                                 floor((p*stride_h+r-pad_h)/kh) = i, floor((q*stride_w+s-pad_w)/kw) = j.
 *               kh*kw times fewer multiply-adds.  S is formed in float and rounded to bfloat16
 *               once (one more storage rounding of the same size as Z's own).  Layers this
 *               version has no such kernel for (cac_describe_plan tells) run as INFLATE.
 *   AUTO      : REDUCED_K where that kernel exists for the layer and the layer is large enough
 *               for it to be the faster one (about 24 GFLOP of nominal work per call), else
 *               INFLATE.  cac_describe_plan tells which. */
typedef enum cac_dw_algo { CAC_DW_INFLATE = 0, CAC_DW_REDUCED_K = 1, CAC_DW_AUTO = 2 } cac_dw_algo;

typedef enum cac_op {
    CAC_OP_FWD_AND_COMPRESS = 0,
    CAC_OP_BWD_WEIGHT_COMPRESSED = 1,
    CAC_OP_BWD_DATA = 2,
    CAC_OP_COMPRESS = 3,
    CAC_OP_BWD_BIAS = 4,
    CAC_OP_GRAD_COSINE = 5,
    CAC_OP_BWD_WEIGHT_AND_DATA = 6,
    CAC_OP_BN_BWD = 7
} cac_op;

/* One convolution layer with a compressed saved input.  Plain data, filled by
 * the caller.  `size` must be sizeof(cac_desc) (guards against a mismatched
 * header).  Dilation 1 and groups 1 only. */
typedef struct cac_desc {
    uint32_t size;
    int32_t N;                   /* mini-batch */
    int32_t C_in, C_out;
    int32_t H, W;                /* input extent */
    int32_t R, S;                /* filter extent */
    int32_t stride_h, stride_w;
    int32_t pad_h, pad_w;        /* zero padding on each side */
    int32_t pool_kh, pool_kw;    /* pooling tile, any positive extents (the tiled kernels cover
                                    1, 2, 4 and 8; others run on the plain ones); 1,1 = keep X */
    int32_t edge_mode;           /* cac_edge_mode */
    int32_t dtype;               /* cac_dtype */
    int32_t has_bias;            /* forward adds b[C_out] when non-zero */
    int32_t pool_mode;           /* cac_pool_mode */
    int32_t dw_algo;             /* cac_dw_algo */
} cac_desc;

int cac_version(void);
const char *cac_last_error(void);

/* Host only.  Output extent of the convolution: P = floor((H+2*pad_h-R)/stride_h)+1. */
int cac_out_shape(const cac_desc *d, int32_t *P, int32_t *Q);

/* Host only.  The saved record's book-keeping (compression section: the record is
 * Z plus the original shape and the tile size, nothing else; byte counts as in the
 * per-layer memory table):
 * pooled extent and the bytes of X and of Z in the descriptor's dtype. */
int cac_pooled_shape(const cac_desc *d, int32_t *Hp, int32_t *Wp, size_t *z_bytes, size_t *x_bytes);

/* Host only.  Device scratch bytes the given cac_op needs for this descriptor. */
int cac_workspace_size(const cac_desc *d, int op, size_t *bytes);

/* Host only.  Floating-point operations (2 x multiply-adds, padding of tiles not counted) that
 * conv_bwd_weight_compressed executes for this descriptor: 2*N*P*Q*C_out*C_in*R*S for the
 * inflating form, the pooled count for the reduced-K form where it applies. */
int cac_dw_executed_flops(const cac_desc *d, uint64_t *flops);

/* Host only.  Writes a one-line, human-readable description of the kernel and
 * launch shape the given cac_op would use for this descriptor into buf (always
 * NUL-terminated, truncated to buf_len).  For logs and benchmarks. */
int cac_describe_plan(const cac_desc *d, int op, char *buf, size_t buf_len);

/* Forward pass of the layer plus compression of its input (compression
 * section: the forward convolution is computed from the uncompressed X, and
 * only afterwards X is pooled into Z, the tensor that is kept).
 *   X [N][C_in][H][W], W [C_out][C_in][R][S], b [C_out] or NULL when !has_bias
 *   Y [N][C_out][P][Q]  = X * W + b           (written)
 *   Z [N][C_in][Hp][Wp] = block means of X    (written)
 * After the stream work of this call completes the caller may release X. */
int conv_fwd_and_compress(const cac_desc *d, const void *X, const void *W, const void *b,
                          void *Y, void *Z, void *ws, size_t ws_bytes, void *stream);

/* Compression alone (same section): Z = block means of X, for callers whose
 * producer of X is not this library's forward convolution. */
int cac_compress(const cac_desc *d, const void *X, void *Z, void *stream);

/* Weight gradient from the compressed activation (weight-gradient formula in
 * the compression figure): with xhat[n,c,h,w] = Z[n,c,h/kh,w/kw],
 *   dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] * xhat[n,c,p*stride_h+r-pad_h,q*stride_w+s-pad_w]
 * (terms outside the image are zero).  dW [C_out][C_in][R][S] float is
 * OVERWRITTEN, not accumulated into.  xhat is never stored. */
int conv_bwd_weight_compressed(const cac_desc *d, const void *Z, const void *dY, void *dW,
                               void *ws, size_t ws_bytes, void *stream);

/* conv_bwd_weight_compressed for callers that cannot allocate or hand over device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without the workspace, same kernels, bit-identical dW.  The scratch the kernels
 * need (the float partial sums of the pixel slices) lives in a buffer of
 * CAC_NOALLOC_SCRATCH_BYTES that is part of the library itself: every GPU the library is used
 * on holds one copy of it until the process ends.  The call allocates and frees nothing.
 *   - A layer whose weight gradient needs more scratch than that
 *     (cac_workspace_size(CAC_OP_BWD_WEIGHT_COMPRESSED) tells) is refused with
 *     CAC_ERR_UNSUPPORTED before anything is launched.  (The launch plans of this version keep
 *     the partial sums to one 64 x 64 x 9 float tile per workgroup of a 256-workgroup grid,
 *     36 MiB, so none is.)
 *   - The first call on a GPU looks the buffer's address up once (hipGetSymbolAddress); make
 *     that call outside stream capture.
 *   - All calls on one GPU share that GPU's buffer: calls that may overlap on one GPU
 *     (different streams, several host threads) race; serialise them on one stream.
 *   - The device current at the call must be the one Z, dY and dW live on. */
#define CAC_NOALLOC_SCRATCH_BYTES ((size_t)40 << 20)
int conv_bwd_weight_compressed_noalloc(const cac_desc *d, const void *Z, const void *dY, void *dW, void *stream);

/* Data gradient (data-gradient formula in the same figure), independent of the
 * activation and therefore exact:
 *   dX[n,c,h,w] = sum_{o,r,s} W[o,c,r,s] * dY[n,o,p,q],  p*stride_h+r-pad_h = h, q*stride_w+s-pad_w = w
 * dX [N][C_in][H][W] is overwritten. */
int conv_bwd_data(const cac_desc *d, const void *W, const void *dY, void *dX,
                  void *ws, size_t ws_bytes, void *stream);

/* Both gradients of a layer in one call: exactly the results of
 * conv_bwd_weight_compressed followed by conv_bwd_data (same kernels, same
 * summation orders, bit-identical outputs), with the small launches of the two
 * shared where they are independent -- the sum over the weight gradient's pixel
 * slices runs in the launch that repacks the data gradient's operands.  A
 * backward pass that needs both (the usual case; the gradient formulas of the
 * compression figure) saves a launch per layer.  `ws` needs
 * cac_workspace_size(CAC_OP_BWD_WEIGHT_AND_DATA) bytes. */
int conv_bwd_weight_and_data(const cac_desc *d, const void *Z, const void *W, const void *dY, void *dW,
                             void *dX, void *ws, size_t ws_bytes, void *stream);

/* Compression at the producer of the activation (conclusion: the pooled map is to come from the
 * operation that makes the activation, and batch normalisation's saved activation is to be
 * compressed as well).  `d` describes the convolution that CONSUMES the activation: its input
 * extent N x C_in x H x W, pooling tile, edge and pooling mode, dtype.  From one read of
 *   Y      [N][C_in][H][W]   the input of the normalisation that precedes that convolution
 * the call writes
 *   X_next [N][C_in][H][W]   = relu(scale[c] * Y + shift[c]), the convolution's input
 *   Z_next [N][C_in][Hp][Wp] = pooling of X_next as stored: the convolution's saved record,
 *                              bit for bit what cac_compress(X_next) gives
 *   Z_in   [N][C_in][Hp][Wp] = pooling of Y: the normalisation's own saved record (NULL: not kept)
 * scale, shift: float [C_in] on the device (batch normalisation in training mode:
 * scale = gamma * invstd, shift = beta - mean * scale; the statistics are the caller's).
 * X_next must not alias Y. */
int cac_bn_relu_fwd_compress(const cac_desc *d, const void *Y, const float *scale, const float *shift, void *X_next, void *Z_next,
                             void *Z_in, void *stream);

/* Batch normalisation's backward pass from its compressed saved input (same passage: a reading,
 * the paper gives no formulas for it).  With x~ = Z_in inflated (every pooled value repeated over
 * its tile), xhat~ = (x~ - mean[c]) * invstd[c], M = N*H*W:
 *   dbeta[c]  = sum dY            dgamma[c] = sum dY * xhat~
 *   dX        = gamma[c] * invstd[c] * (dY - dbeta[c] / M - xhat~ * dgamma[c] / M)
 * i.e. the exact formulas with the saved activation replaced by its inflated record; dbeta is
 * exact.  mean, invstd, gamma: float [C_in], read; dgamma, dbeta: float [C_in], written; dX
 * [N][C_in][H][W] in the tensors' type, written.  Sums are taken in a fixed order.
 * ws: cac_workspace_size(d, CAC_OP_BN_BWD) bytes (partial sums of the channels' slices; 0 for many
 * channels or plain kernels). */
int cac_bn_bwd_compressed(const cac_desc *d, const void *Z_in, const void *dY, const float *mean, const float *invstd,
                          const float *gamma, float *dgamma, float *dbeta, void *dX, void *ws, size_t ws_bytes, void *stream);

/* Yardsticks for benchmarks (no part of the method): what this machine attains on a bare
 * matrix-core loop and on a bare stream, to set a kernel's rate against.
 *   CAC_PROBE_MFMA: a grid of 2048 waves, each issuing iters * 16 independent 32x32x16 bfloat16
 *                   MFMAs on fragments read once from src (at least 16 KiB; its VALUES matter: the
 *                   chip clocks lower on random numbers than on zeros); 2*32*32*16 flops each.
 *   CAC_PROBE_COPY: dst = src over `bytes` (a multiple of 16).   CAC_PROBE_READ: reads src.
 *   CAC_PROBE_MFMA_16X16: as CAC_PROBE_MFMA with 16x16x32 MFMAs, iters * 32 of them per wave (the same
 *                   flops).   CAC_PROBE_MFMA_1WAVE: as CAC_PROBE_MFMA with 1024 waves, one per SIMD.
 * dst: at least 8 KiB for every kind but the copy. */
typedef enum cac_probe_kind {
    CAC_PROBE_MFMA = 0, CAC_PROBE_COPY = 1, CAC_PROBE_READ = 2, CAC_PROBE_MFMA_16X16 = 3, CAC_PROBE_MFMA_1WAVE = 4
} cac_probe_kind;
int cac_probe(int kind, const void *src, void *dst, size_t bytes, int iters, void *stream);

/* Bias gradient (bias-gradient formula in the same figure): db[o] = sum_{n,p,q} dY.
 * db [C_out] float is overwritten. */
int conv_bwd_bias(const cac_desc *d, const void *dY, void *db, void *stream);

/* Layer sensitivity metric (the equation of the section "Layer sensitivity"): cosine
 * similarity cos(a, b) = a.b / (|a| |b|) of two weight gradients of this layer, e.g. the one
 * computed from the compressed activation against the exact one (pooling factor 1).
 * dW_a, dW_b: [C_out][C_in][R][S] float, read only.  out: 4 floats on the device, written:
 * {cos, a.b, |a|^2, |b|^2}; cos is 0 when either norm is 0.  Sums are taken in double
 * precision in a fixed order.  ws: cac_workspace_size(d, CAC_OP_GRAD_COSINE) bytes. */
int cac_grad_cosine(const cac_desc *d, const void *dW_a, const void *dW_b, void *out,
                    void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CAC_H */
