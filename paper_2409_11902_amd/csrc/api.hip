// C ABI of the library: descriptor validation, shape/workspace queries (host
// only) and dispatch to the kernels.  Every check runs before anything is
// launched, so all error paths can be exercised without a GPU.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "common.h"
#include "conv_mfma.h"
#include "dw_mfma.h"
#include "dw_rk.h"
#include "dw_tiled.h"

namespace cac {

static thread_local char g_err[256] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static const long kMaxElems = (1L << 31) - 1; // every tensor is indexed with int-sized extents

// a * b * c * e without wrapping, and at most `limit`
static bool product_fits(long a, long b, long c, long e, long limit)
{
    long r;
    return !__builtin_mul_overflow(a, b, &r) && !__builtin_mul_overflow(r, c, &r) && !__builtin_mul_overflow(r, e, &r) && r <= limit;
}

// Validates the descriptor and fills the kernel geometry.  `for_kernel`: also
// reject what only the shape queries accept.
static int make_geom(const cac_desc *d, Geom *g, bool for_kernel)
{
    if (!d) return fail(CAC_ERR_INVALID_ARG, "descriptor is NULL");
    if (d->size != sizeof(cac_desc))
        return fail(CAC_ERR_INVALID_ARG, "desc.size is %u, this library expects %zu", d->size, sizeof(cac_desc));
    if (d->N <= 0 || d->C_in <= 0 || d->C_out <= 0 || d->H <= 0 || d->W <= 0)
        return fail(CAC_ERR_INVALID_ARG, "N, C_in, C_out, H, W must be positive");
    if (d->R <= 0 || d->S <= 0 || d->stride_h <= 0 || d->stride_w <= 0)
        return fail(CAC_ERR_INVALID_ARG, "R, S and strides must be positive");
    if (d->pad_h < 0 || d->pad_w < 0) return fail(CAC_ERR_INVALID_ARG, "padding must be non-negative");
    if (d->pool_kh <= 0 || d->pool_kw <= 0) return fail(CAC_ERR_INVALID_ARG, "pooling tile must be positive");
    if (d->dtype != CAC_F32 && d->dtype != CAC_BF16) return fail(CAC_ERR_INVALID_ARG, "unknown dtype %d", d->dtype);
    if (d->dw_algo != CAC_DW_INFLATE && d->dw_algo != CAC_DW_REDUCED_K && d->dw_algo != CAC_DW_AUTO)
        return fail(CAC_ERR_INVALID_ARG, "unknown dw_algo %d", d->dw_algo);
    if (d->edge_mode != CAC_EDGE_CEIL_VALID && d->edge_mode != CAC_EDGE_FLOOR_DROP)
        return fail(CAC_ERR_INVALID_ARG, "unknown edge_mode %d", d->edge_mode);
    if (d->pool_mode != CAC_POOL_MEAN && d->pool_mode != CAC_POOL_MAX)
        return fail(CAC_ERR_INVALID_ARG, "unknown pool_mode %d", d->pool_mode);
    // bounds that keep every derived extent inside int arithmetic
    const int kMaxExtent = 1 << 24, kMaxSmall = 1 << 15;
    if (d->N > kMaxExtent || d->C_in > kMaxExtent || d->C_out > kMaxExtent || d->H > kMaxExtent || d->W > kMaxExtent)
        return fail(CAC_ERR_UNSUPPORTED, "an extent above 2^24");
    if (d->R > kMaxSmall || d->S > kMaxSmall || d->stride_h > kMaxSmall || d->stride_w > kMaxSmall || d->pad_h > kMaxSmall ||
        d->pad_w > kMaxSmall || d->pool_kh > kMaxSmall || d->pool_kw > kMaxSmall)
        return fail(CAC_ERR_UNSUPPORTED, "filter, stride, padding or pooling tile above 2^15");
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S)
        return fail(CAC_ERR_INVALID_ARG, "filter larger than the padded input");
    bool floor_mode = d->edge_mode == CAC_EDGE_FLOOR_DROP;
    if (floor_mode && (d->H < d->pool_kh || d->W < d->pool_kw))
        return fail(CAC_ERR_INVALID_ARG, "floor/drop pooling tile larger than the input");

    g->N = d->N; g->C = d->C_in; g->K = d->C_out; g->H = d->H; g->W = d->W;
    g->R = d->R; g->S = d->S; g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
    g->P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
    g->Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    g->kh = d->pool_kh; g->kw = d->pool_kw;
    g->pmax = d->pool_mode == CAC_POOL_MAX;
    g->dw_algo = d->dw_algo;
    g->Hp = floor_mode ? d->H / d->pool_kh : (d->H + d->pool_kh - 1) / d->pool_kh;
    g->Wp = floor_mode ? d->W / d->pool_kw : (d->W + d->pool_kw - 1) / d->pool_kw;

    if (!for_kernel) return CAC_OK;
    if (floor_mode && (d->H % d->pool_kh || d->W % d->pool_kw))
        return fail(CAC_ERR_UNSUPPORTED,
                    "floor/drop edge mode with a tile that does not divide the input: inflation of the dropped "
                    "rows is undefined; use CAC_EDGE_CEIL_VALID");
    if (!product_fits(g->N, g->C, g->H, g->W, kMaxElems) || !product_fits(g->N, g->K, g->P, g->Q, kMaxElems) ||
        !product_fits(g->K, g->C, g->R, g->S, kMaxElems))
        return fail(CAC_ERR_UNSUPPORTED, "a tensor has more than 2^31-1 elements");
    if (g->N > 65535) return fail(CAC_ERR_UNSUPPORTED, "N above 65535");
    return CAC_OK;
}

static int check_ptr(const void *p, const char *name)
{
    if (!p) return fail(CAC_ERR_INVALID_ARG, "%s is NULL", name);
    if (((uintptr_t)p) & 15) return fail(CAC_ERR_ALIGNMENT, "%s is not 16-byte aligned", name);
    return CAC_OK;
}

static int check_ws(const Geom &g, int dtype, int op, const void *ws, size_t ws_bytes, size_t *need_out);

static int launched(hipError_t e, const char *what)
{
    if (e != hipSuccess) return fail(CAC_ERR_LAUNCH_FAILED, "%s: %s", what, hipGetErrorString(e));
    return CAC_OK;
}

static size_t workspace_bytes(const Geom &g, int dtype, int op);

// Part of the combined backward call's workspace that the weight gradient uses (the data
// gradient's part starts behind it, 256-byte aligned).
// The reduced-K kernel's plan when the descriptor asks for that form and the kernel covers the
// geometry.  AUTO asks for it only where it has measured faster than the inflating kernel: from
// about 24 GFLOP of nominal work per call on.  Below that the two finish within a few microseconds
// of each other or the inflating kernel wins (a workgroup of the reduced-K kernel forms the tile
// sums of its 32 output channels for only 128 input channels, and its partial sums are larger).
static bool reduced_k_plan(const Geom &g, int dtype, DwRkPlan *rk)
{
    if (g.dw_algo != CAC_DW_REDUCED_K && g.dw_algo != CAC_DW_AUTO) return false;
    if (!dw_rk_plan(g, dtype, rk)) return false;
    if (g.dw_algo == CAC_DW_AUTO) {
        const double nominal = 2.0 * g.N * g.P * g.Q * (double)g.K * g.C * g.R * g.S;
        if (nominal < 24e9) return false;
    }
    return true;
}

static size_t both_dw_bytes(const Geom &g, int dtype)
{
    return (workspace_bytes(g, dtype, CAC_OP_BWD_WEIGHT_COMPRESSED) + 255) & ~(size_t)255;
}

static size_t workspace_bytes(const Geom &g, int dtype, int op)
{
    if (op == CAC_OP_BWD_WEIGHT_COMPRESSED) {
        DwRkPlan rk;
        if (reduced_k_plan(g, dtype, &rk)) return rk.partial_bytes;
        DwMfmaPlan plan;
        if (dw_mfma_plan(g, dtype, &plan)) return plan.partial_bytes; // partial sums of the pixel slices
        DwTiledPlan tl;
        if (dw_tiled_plan(g, dtype, &tl)) return tl.partial_bytes;
    }
    // channels-last copy of the input and the repacked filter
    if (op == CAC_OP_FWD_AND_COMPRESS) return conv_mfma_workspace(g, dtype, false);
    if (op == CAC_OP_BWD_DATA) return conv_mfma_workspace(g, dtype, true);
    if (op == CAC_OP_GRAD_COSINE) return cosine_workspace((long)g.K * g.C * g.R * g.S);
    // both gradients in one call: the partial sums are still being read when the repacks are written
    if (op == CAC_OP_BWD_WEIGHT_AND_DATA)
        return both_dw_bytes(g, dtype) + workspace_bytes(g, dtype, CAC_OP_BWD_DATA);
    if (op == CAC_OP_BN_BWD) return bn_bwd_workspace_bytes(g, dtype);
    return 0;
}

static int check_ws(const Geom &g, int dtype, int op, const void *ws, size_t ws_bytes, size_t *need_out)
{
    size_t need = workspace_bytes(g, dtype, op);
    if (need_out) *need_out = need;
    if (need == 0) return CAC_OK;
    if (!ws) return fail(CAC_ERR_WORKSPACE_TOO_SMALL, "workspace is NULL, %zu bytes needed", need);
    if (((uintptr_t)ws) & 15) return fail(CAC_ERR_ALIGNMENT, "workspace is not 16-byte aligned");
    if (ws_bytes < need) return fail(CAC_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return CAC_OK;
}

static hipError_t do_compress(const Geom &g, int dtype, const void *X, void *Z, hipStream_t st)
{
    hipError_t e = hipSuccess;
    if (launch_compress_fast(g, dtype, X, Z, st, &e)) return e;
    return launch_compress_generic(g, dtype, X, Z, st);
}

// The weight gradient with the kernel the descriptor asks for (the reduced-K form where this
// version has one for the geometry, else the inflating MFMA kernel, else the plain one).
static int launch_weight_gradient(const Geom &g, int dtype, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                                  DwReduceTail *defer)
{
    if (defer) defer->blocks = 0;
    DwRkPlan rk;
    if (reduced_k_plan(g, dtype, &rk))
        return launched(launch_dw_rk(rk, Z, dY, dW, ws, st, defer), "weight gradient (reduced K)");
    DwMfmaPlan plan;
    if (dw_mfma_plan(g, dtype, &plan)) return launched(launch_dw_mfma(plan, Z, dY, dW, ws, st, defer), "weight gradient (MFMA)");
    DwTiledPlan tl;
    if (dw_tiled_plan(g, dtype, &tl)) return launched(launch_dw_tiled(tl, dtype, Z, dY, dW, ws, st, defer), "weight gradient (tiled)");
    return launched(launch_dw_generic(g, dtype, Z, dY, dW, st), "weight gradient");
}

// ---- scratch of the entry point that allocates nothing ------------------------------------
// Device memory that belongs to the library's code object: every GPU the library runs on holds
// its own copy, at its own address, until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and copies get the address looked up below.
constexpr size_t kScratchBytes = CAC_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch` (looked up once per device, with that device current).
static int scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(CAC_ERR_LAUNCH_FAILED, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(CAC_ERR_UNSUPPORTED, "device ordinal %d above %d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(CAC_ERR_LAUNCH_FAILED, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CAC_OK;
}

} // namespace cac

using namespace cac;

extern "C" {

int cac_version(void) { return CAC_VERSION; }

const char *cac_last_error(void) { return g_err; }

int cac_out_shape(const cac_desc *d, int32_t *P, int32_t *Q)
{
    Geom g;
    int rc = make_geom(d, &g, false);
    if (rc) return rc;
    if (!P || !Q) return fail(CAC_ERR_INVALID_ARG, "output pointer is NULL");
    *P = g.P;
    *Q = g.Q;
    return CAC_OK;
}

int cac_pooled_shape(const cac_desc *d, int32_t *Hp, int32_t *Wp, size_t *z_bytes, size_t *x_bytes)
{
    Geom g;
    int rc = make_geom(d, &g, false);
    if (rc) return rc;
    size_t eb = d->dtype == CAC_F32 ? 4 : 2;
    if (!product_fits(g.N, g.C, g.H, g.W, (1L << 60)))
        return fail(CAC_ERR_UNSUPPORTED, "the byte count of X does not fit 64 bits");
    if (Hp) *Hp = g.Hp;
    if (Wp) *Wp = g.Wp;
    if (z_bytes) *z_bytes = (size_t)g.N * g.C * g.Hp * g.Wp * eb;
    if (x_bytes) *x_bytes = (size_t)g.N * g.C * g.H * g.W * eb;
    return CAC_OK;
}

int cac_workspace_size(const cac_desc *d, int op, size_t *bytes)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if (op < CAC_OP_FWD_AND_COMPRESS || op > CAC_OP_BN_BWD) return fail(CAC_ERR_INVALID_ARG, "unknown op %d", op);
    if (!bytes) return fail(CAC_ERR_INVALID_ARG, "bytes is NULL");
    *bytes = workspace_bytes(g, d->dtype, op);
    return CAC_OK;
}

int cac_dw_executed_flops(const cac_desc *d, uint64_t *flops)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if (!flops) return fail(CAC_ERR_INVALID_ARG, "flops is NULL");
    DwRkPlan rk;
    if (reduced_k_plan(g, d->dtype, &rk))
        *flops = rk.executed_flops;
    else
        *flops = 2ull * g.N * g.P * g.Q * (uint64_t)g.K * g.C * g.R * g.S;
    return CAC_OK;
}

int cac_describe_plan(const cac_desc *d, int op, char *buf, size_t buf_len)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if (!buf || buf_len == 0) return fail(CAC_ERR_INVALID_ARG, "buf is NULL or empty");
    if (op < CAC_OP_FWD_AND_COMPRESS || op > CAC_OP_BN_BWD) return fail(CAC_ERR_INVALID_ARG, "unknown op %d", op);
    DwMfmaPlan plan;
    DwRkPlan rk;
    if (op == CAC_OP_BWD_WEIGHT_COMPRESSED && reduced_k_plan(g, d->dtype, &rk)) {
        const DwRkParams &p = rk.p;
        snprintf(buf, buf_len,
                 "dw_rk tile=32x128 unit=%dimg x %dpooled rows (Z rows %d, tile-sum rows %d, blocks %d/%d) chunk=2 units "
                 "lds=%dB units=%d slices=%d x %d tiles grid=%u partial=%zuB",
                 p.NBIu, p.PRp, p.UZ, p.US, p.SEGS, p.SEGS_S, p.lds_bytes, p.nunits, p.nslices, p.tiles_o * p.tiles_c, rk.grid,
                 rk.partial_bytes);
    } else if (op == CAC_OP_BWD_WEIGHT_COMPRESSED && dw_mfma_plan(g, d->dtype, &plan)) {
        const DwMfmaParams &p = plan.p;
        snprintf(buf, buf_len,
                 "dw_mfma variant=%d tile=%dx%d chunk=%dimg x %drows (LR=%d/%d SEGS=%d NZ=%d XW=%d) items dy=%d z=%d "
                 "passes dy=%d z=%d lds=%dB chunks=%d slices=%d x %d tiles grid=%u partial=%zuB%s",
                 plan.variant, p.tile_o, p.tile_c, p.NBI, p.PR, p.LR, p.LRpad, p.SEGS, p.NZ, p.XW, p.rowitems, p.citems, p.dy_passes,
                 p.z_passes, p.lds_bytes, p.nchunks, p.nslices, p.tiles_o * p.tiles_c, plan.grid,
                 plan.partial_bytes, p.dy_direct ? " dY straight into LDS" : "");
    } else if (DwTiledPlan tl; op == CAC_OP_BWD_WEIGHT_COMPRESSED && dw_tiled_plan(g, d->dtype, &tl)) {
        snprintf(buf, buf_len, "dw_tiled tile=16x16 unit=%d rows (LDS rows %d x %d floats) lds=%dB units=%d slices=%d x %d tiles grid=%u partial=%zuB",
                 tl.p.PR, tl.p.XR, tl.p.XW, tl.p.lds_bytes, tl.p.nunits, tl.p.nslices, tl.p.tiles_o * tl.p.tiles_c, tl.grid,
                 tl.partial_bytes);
    } else if ((op == CAC_OP_FWD_AND_COMPRESS || op == CAC_OP_BWD_DATA) &&
               describe_conv_mfma(g, d->dtype, op == CAC_OP_BWD_DATA, buf, buf_len)) {
    } else if (op == CAC_OP_COMPRESS || op == CAC_OP_GRAD_COSINE) {
        snprintf(buf, buf_len, "streaming kernel");
    } else if (op == CAC_OP_BN_BWD) {
        const size_t n = bn_bwd_workspace_bytes(g, d->dtype);
        snprintf(buf, buf_len, "sums and element-wise pass (%zu slices per channel where the chunk kernels take the tile)",
                 n ? n / (2 * sizeof(float) * (size_t)g.C) : (size_t)1);
    } else if (op == CAC_OP_BWD_WEIGHT_AND_DATA) {
        char dx[64];
        const bool split = (reduced_k_plan(g, d->dtype, &rk)) ? !rk.p.direct
                                                                                           : (dw_mfma_plan(g, d->dtype, &plan) && !plan.p.direct);
        const bool merged = split && describe_conv_mfma(g, d->dtype, true, dx, sizeof dx);
        snprintf(buf, buf_len, merged ? "weight gradient, then its slice sum in the launch of the data gradient's repack, then the data gradient"
                                      : "weight gradient, then data gradient, as in the separate calls");
    } else {
        snprintf(buf, buf_len, "generic kernel");
    }
    return CAC_OK;
}

int conv_fwd_and_compress(const cac_desc *d, const void *X, const void *W, const void *b, void *Y, void *Z,
                          void *ws, size_t ws_bytes, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(X, "X")) || (rc = check_ptr(W, "W")) || (rc = check_ptr(Y, "Y")) || (rc = check_ptr(Z, "Z")))
        return rc;
    if (d->has_bias && (rc = check_ptr(b, "b"))) return rc;
    if ((rc = check_ws(g, d->dtype, CAC_OP_FWD_AND_COMPRESS, ws, ws_bytes, nullptr))) return rc;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    bool pooled = false;
    if (!launch_fwd_mfma(g, d->dtype, X, W, d->has_bias ? b : nullptr, Y, Z, ws, st, &e, &pooled))
        e = launch_fwd_generic(g, d->dtype, X, W, d->has_bias ? b : nullptr, Y, st);
    if ((rc = launched(e, "forward convolution"))) return rc;
    if (pooled) return CAC_OK;
    return launched(do_compress(g, d->dtype, X, Z, st), "compress");
}

int cac_compress(const cac_desc *d, const void *X, void *Z, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(X, "X")) || (rc = check_ptr(Z, "Z"))) return rc;
    return launched(do_compress(g, d->dtype, X, Z, (hipStream_t)stream), "compress");
}

int conv_bwd_weight_compressed(const cac_desc *d, const void *Z, const void *dY, void *dW, void *ws,
                               size_t ws_bytes, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(Z, "Z")) || (rc = check_ptr(dY, "dY")) || (rc = check_ptr(dW, "dW"))) return rc;
    if ((rc = check_ws(g, d->dtype, CAC_OP_BWD_WEIGHT_COMPRESSED, ws, ws_bytes, nullptr))) return rc;
    return launch_weight_gradient(g, d->dtype, Z, dY, (float *)dW, ws, (hipStream_t)stream, nullptr);
}

int conv_bwd_weight_compressed_noalloc(const cac_desc *d, const void *Z, const void *dY, void *dW, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(Z, "Z")) || (rc = check_ptr(dY, "dY")) || (rc = check_ptr(dW, "dW"))) return rc;
    const size_t need = workspace_bytes(g, d->dtype, CAC_OP_BWD_WEIGHT_COMPRESSED);
    if (need > kScratchBytes)
        return fail(CAC_ERR_UNSUPPORTED,
                    "this layer's weight gradient needs %zu bytes of scratch, the built-in buffer has %zu: "
                    "use conv_bwd_weight_compressed with a workspace of the caller's",
                    need, kScratchBytes);
    void *ws = nullptr;
    if (need && (rc = scratch_of_current_device(&ws))) return rc;
    // (nothing in the buffer has to start as zero: every pixel slice writes the whole of its
    // partial sums before the slice sum reads them)
    return launch_weight_gradient(g, d->dtype, Z, dY, (float *)dW, ws, (hipStream_t)stream, nullptr);
}

int conv_bwd_data(const cac_desc *d, const void *W, const void *dY, void *dX, void *ws, size_t ws_bytes,
                  void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(W, "W")) || (rc = check_ptr(dY, "dY")) || (rc = check_ptr(dX, "dX"))) return rc;
    if ((rc = check_ws(g, d->dtype, CAC_OP_BWD_DATA, ws, ws_bytes, nullptr))) return rc;
    hipError_t e = hipSuccess;
    if (!launch_dx_mfma(g, d->dtype, W, dY, dX, ws, (hipStream_t)stream, &e))
        e = launch_dx_generic(g, d->dtype, W, dY, dX, (hipStream_t)stream);
    return launched(e, "data gradient");
}

int conv_bwd_weight_and_data(const cac_desc *d, const void *Z, const void *W, const void *dY, void *dW, void *dX, void *ws,
                             size_t ws_bytes, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(Z, "Z")) || (rc = check_ptr(W, "W")) || (rc = check_ptr(dY, "dY")) || (rc = check_ptr(dW, "dW")) ||
        (rc = check_ptr(dX, "dX")))
        return rc;
    if ((rc = check_ws(g, d->dtype, CAC_OP_BWD_WEIGHT_AND_DATA, ws, ws_bytes, nullptr))) return rc;
    hipStream_t st = (hipStream_t)stream;
    void *ws_dx = ws ? (char *)ws + both_dw_bytes(g, d->dtype) : nullptr;
    DwReduceTail tail{};
    if ((rc = launch_weight_gradient(g, d->dtype, Z, dY, (float *)dW, ws, st, &tail))) return rc;
    hipError_t e = hipSuccess;
    if (!launch_dx_mfma(g, d->dtype, W, dY, dX, ws_dx, st, &e, &tail)) {
        if ((rc = launched(launch_dw_reduce(tail, st), "weight gradient (slice sum)"))) return rc;
        e = launch_dx_generic(g, d->dtype, W, dY, dX, st);
    }
    return launched(e, "data gradient");
}

int cac_bn_relu_fwd_compress(const cac_desc *d, const void *Y, const float *scale, const float *shift, void *X_next, void *Z_next,
                             void *Z_in, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(Y, "Y")) || (rc = check_ptr(scale, "scale")) || (rc = check_ptr(shift, "shift")) ||
        (rc = check_ptr(X_next, "X_next")) || (rc = check_ptr(Z_next, "Z_next")))
        return rc;
    if (Z_in && (rc = check_ptr(Z_in, "Z_in"))) return rc;
    if (Y == X_next) return fail(CAC_ERR_INVALID_ARG, "X_next must not alias Y (tiles are read after their neighbours are written)");
    hipError_t e = hipSuccess;
    if (!launch_producer_fast(g, d->dtype, Y, scale, shift, X_next, Z_next, Z_in, (hipStream_t)stream, &e))
        e = launch_producer_generic(g, d->dtype, Y, scale, shift, X_next, Z_next, Z_in, (hipStream_t)stream);
    return launched(e, "normalise + activate + compress");
}

int cac_bn_bwd_compressed(const cac_desc *d, const void *Z_in, const void *dY, const float *mean, const float *invstd,
                          const float *gamma, float *dgamma, float *dbeta, void *dX, void *ws, size_t ws_bytes, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(Z_in, "Z_in")) || (rc = check_ptr(dY, "dY")) || (rc = check_ptr(mean, "mean")) ||
        (rc = check_ptr(invstd, "invstd")) || (rc = check_ptr(gamma, "gamma")) || (rc = check_ptr(dgamma, "dgamma")) ||
        (rc = check_ptr(dbeta, "dbeta")) || (rc = check_ptr(dX, "dX")))
        return rc;
    if ((rc = check_ws(g, d->dtype, CAC_OP_BN_BWD, ws, ws_bytes, nullptr))) return rc;
    hipError_t e = hipSuccess;
    if (launch_bn_bwd_fast(g, d->dtype, Z_in, dY, mean, invstd, gamma, dgamma, dbeta, dX, ws, (hipStream_t)stream, &e))
        return launched(e, "batch normalisation backward");
    if ((long)g.N * g.C > 65535L * 32767L) return fail(CAC_ERR_UNSUPPORTED, "N * C_in too large for this kernel's grid");
    return launched(launch_bn_bwd(g, d->dtype, Z_in, dY, mean, invstd, gamma, dgamma, dbeta, dX, (hipStream_t)stream),
                    "batch normalisation backward");
}

int cac_probe(int kind, const void *src, void *dst, size_t bytes, int iters, void *stream)
{
    int rc;
    if (kind < CAC_PROBE_MFMA || kind > CAC_PROBE_MFMA_1WAVE) return fail(CAC_ERR_INVALID_ARG, "unknown probe kind %d", kind);
    if ((rc = check_ptr(src, "src")) || (rc = check_ptr(dst, "dst"))) return rc;
    if (bytes < 16384 || (bytes & 15)) return fail(CAC_ERR_INVALID_ARG, "bytes must be a multiple of 16, at least 16384");
    if (iters < 0 || iters > (1 << 24)) return fail(CAC_ERR_INVALID_ARG, "iters out of range");
    return launched(launch_probe(kind, src, dst, bytes, iters, (hipStream_t)stream), "probe");
}

int conv_bwd_bias(const cac_desc *d, const void *dY, void *db, void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(dY, "dY")) || (rc = check_ptr(db, "db"))) return rc;
    hipError_t e = hipSuccess;
    if (launch_db_fast(g, d->dtype, dY, (float *)db, (hipStream_t)stream, &e)) return launched(e, "bias gradient");
    return launched(launch_db(g, d->dtype, dY, (float *)db, (hipStream_t)stream), "bias gradient");
}

int cac_grad_cosine(const cac_desc *d, const void *dW_a, const void *dW_b, void *out, void *ws, size_t ws_bytes,
                    void *stream)
{
    Geom g;
    int rc = make_geom(d, &g, true);
    if (rc) return rc;
    if ((rc = check_ptr(dW_a, "dW_a")) || (rc = check_ptr(dW_b, "dW_b")) || (rc = check_ptr(out, "out"))) return rc;
    if ((rc = check_ws(g, d->dtype, CAC_OP_GRAD_COSINE, ws, ws_bytes, nullptr))) return rc;
    return launched(launch_cosine((const float *)dW_a, (const float *)dW_b, (long)g.K * g.C * g.R * g.S, (float *)out, ws,
                                  (hipStream_t)stream),
                    "gradient cosine");
}

} // extern "C"
