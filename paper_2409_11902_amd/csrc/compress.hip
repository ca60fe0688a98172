// Activation compression: Z = average pooling of X over non-overlapping,
// origin-aligned kh x kw tiles (compression section; the compression figure
// shows the tiling); on request the tile maximum instead (the same section names
// other poolings as feasible).  Bandwidth-bound: every element of X is read once with
// 16-byte loads, every element of Z written once; no LDS, except in the kernel for rows of 10 to
// 14 elements further down (compress_narrow_kernel).
//
// A thread owns one "chunk": 16 bytes of kh consecutive input rows (8 bfloat16
// or 4 float columns) and the 16/(kw*elem) pooled values below them.  Chunks of
// a row are handed to consecutive threads, so a wave reads whole rows.
// Ragged edges follow the ceil/valid rule: a tile that sticks out is averaged
// over the elements it really has.
#include "chunk.h"

namespace cac {

namespace {

// What the producer form of the kernel does on top of compression (see launch_producer_fast).
struct Producer {
    const float *scale, *shift; // per channel
    void *Xn;                   // relu(scale * X + shift), the next layer's input
    void *Zin;                  // pooled X itself (the normalisation's own saved record), or null
    double inv_c;               // 1 / channels
};

// One chunk's pooled values: sums in row-then-column order; whole tiles multiply by the exact
// reciprocal of their power-of-two count, ragged ones divide by the elements they really have.
template <typename T, int EPC, int KH, int KW>
__device__ __forceinline__ void pool_and_store(const Geom &g, const float (&v)[KH][EPC], int rows, int w0, int j0, T *zrow)
{
    constexpr int OPC = EPC / KW;
    const float inv_full = 1.0f / (float)(rows * KW); // exact for the power-of-two counts of whole tiles
    float res[OPC];
#pragma unroll
    for (int o = 0; o < OPC; ++o) {
        const int cols = min(KW, g.W - (w0 + o * KW)); // < 1 for pooled columns that do not exist
        float sum = 0.f, best = v[0][o * KW]; // (a pooled column that exists has its first element)
#pragma unroll
        for (int a = 0; a < KH; ++a)
#pragma unroll
            for (int b = 0; b < KW; ++b)
                if (a < rows && b < cols) {
                    sum += v[a][o * KW + b];
                    best = fmaxf(best, v[a][o * KW + b]);
                }
        res[o] = g.pmax ? best : cols == KW ? sum * inv_full : sum / (float)(rows * max(cols, 1));
    }
    if (g.Wp % OPC == 0) {
        // whole chunks only, and the row of Z starts on a multiple of OPC elements: one store
        if constexpr (sizeof(T) == 4) {
            typedef __attribute__((ext_vector_type(OPC))) float fvec;
            fvec out;
#pragma unroll
            for (int o = 0; o < OPC; ++o) out[o] = res[o];
            *(fvec *)(zrow + j0) = out;
        } else if constexpr (OPC >= 2) {
            typedef __attribute__((ext_vector_type(OPC / 2))) uint32_t uvec;
            uvec out;
#pragma unroll
            for (int o = 0; o < OPC / 2; ++o)
                out[o] = (uint32_t)f32_to_bf16(res[2 * o]) | ((uint32_t)f32_to_bf16(res[2 * o + 1]) << 16);
            *(uvec *)(zrow + j0) = out;
        } else {
            Elem<T>::store(zrow + j0, res[0]);
        }
    } else if (sizeof(T) == 2 && OPC >= 2 && g.Wp % 2 == 0) {
        // a row of Z ends inside the last chunk (pooled rows of 14): every row still starts on a
        // dword and the chunks on even elements, so pairs of neighbours leave as dword stores
        if constexpr (sizeof(T) == 2 && OPC >= 2) {
            uint32_t *dst = (uint32_t *)((bf16_t *)zrow + j0);
#pragma unroll
            for (int o = 0; o < OPC / 2; ++o)
                if (j0 + 2 * o < g.Wp) dst[o] = (uint32_t)f32_to_bf16(res[2 * o]) | ((uint32_t)f32_to_bf16(res[2 * o + 1]) << 16);
        }
    } else {
#pragma unroll
        for (int o = 0; o < OPC; ++o)
            if (j0 + o < g.Wp) Elem<T>::store(zrow + j0 + o, res[o]);
    }
}

template <typename T, int EPC, int KH, int KW, bool PROD>
__global__ void __launch_bounds__(256) compress_kernel(Geom g, const T *__restrict__ X, T *__restrict__ Z, int cpr,
                                                       uint32_t total, double inv_cpr, double inv_hp, Producer pr)
{
    constexpr int OPC = EPC / KW; // pooled values per chunk
    static_assert(OPC >= 1, "");
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x;
    if (idx >= total) return;
    // idx -> (plane, pooled row i, chunk c), chunk fastest
    const uint32_t rowi = udiv(idx, inv_cpr);
    const uint32_t c = idx - rowi * cpr;
    const uint32_t plane = udiv(rowi, inv_hp);
    const uint32_t i = rowi - plane * g.Hp;

    const rsrc_t rs = make_rsrc(X, (uint32_t)g.N * g.C * g.H * g.W * (uint32_t)sizeof(T));
    const int h0 = i * KH;
    const int rows = min(KH, g.H - h0);
    float v[KH][EPC];
#pragma unroll
    for (int a = 0; a < KH; ++a)
        Chunk<T, EPC>::load(rs, (plane * g.H + h0 + a) * g.W + c * EPC, a < rows, g.W & 1, v[a]);

    const int w0 = c * EPC;       // first input column of the chunk
    const int j0 = c * OPC;       // first pooled column
    const long zoff = ((long)plane * g.Hp + i) * g.Wp;
    if constexpr (PROD) {
        // the producer's own saved record: X pooled as it is
        if (pr.Zin) pool_and_store<T, EPC, KH, KW>(g, v, rows, w0, j0, (T *)pr.Zin + zoff);
        // the next layer's input, rounded to its storage type, and from those rounded values the
        // next layer's pooled map (bit for bit what compressing the stored tensor would give)
        const uint32_t ch = plane - udiv(plane, pr.inv_c) * (uint32_t)g.C;
        const float sc = pr.scale[ch], sh = pr.shift[ch];
        T *xn = (T *)pr.Xn;
        typedef u32x4 __attribute__((aligned(4))) u32x4_u;
#pragma unroll
        for (int a = 0; a < KH; ++a) {
            if (a >= rows) continue;
            const long e = ((long)plane * g.H + h0 + a) * g.W + w0;
            const int left = g.W - w0;
            if constexpr (sizeof(T) == 4) {
#pragma unroll
                for (int b = 0; b < EPC; ++b) v[a][b] = fmaxf(fmaf(sc, v[a][b], sh), 0.f);
                if (left >= EPC) { // (float rows start on dwords: a 16-byte global store only needs that)
                    *(u32x4_u *)(xn + e) = u32x4{__float_as_uint(v[a][0]), __float_as_uint(v[a][1]), __float_as_uint(v[a][2]), __float_as_uint(v[a][3])};
                } else {
#pragma unroll
                    for (int b = 0; b < EPC; ++b)
                        if (b < left) xn[e + b] = v[a][b];
                }
            } else {
                // pairs rounded by the hardware conversion (round to nearest even); the pooled map is
                // formed from the rounded values
                uint32_t o[EPC / 2];
#pragma unroll
                for (int b = 0; b < EPC / 2; ++b) {
                    o[b] = f32x2_to_bf16x2(fmaxf(fmaf(sc, v[a][2 * b], sh), 0.f), fmaxf(fmaf(sc, v[a][2 * b + 1], sh), 0.f));
                    v[a][2 * b] = __uint_as_float(o[b] << 16);
                    v[a][2 * b + 1] = __uint_as_float(o[b] & 0xffff0000u);
                }
                if ((e & 1) == 0) {
                    // the chunk starts on a dword (every row of an even W does): global stores of several
                    // dwords only need that alignment
                    if (EPC == 8 && left >= 8) {
                        *(u32x4_u *)(xn + e) = u32x4{o[0], o[1], o[EPC / 4], o[EPC / 2 - 1]};
                    } else {
#pragma unroll
                        for (int b = 0; b < EPC / 2; ++b) {
                            if (2 * b + 1 < left)
                                *(uint32_t *)(xn + e + 2 * b) = o[b];
                            else if (2 * b < left)
                                xn[e + 2 * b] = (bf16_t)(o[b] & 0xffffu);
                        }
                    }
                } else {
#pragma unroll
                    for (int b = 0; b < EPC; ++b)
                        if (b < left) xn[e + b] = (bf16_t)((b & 1) ? o[b / 2] >> 16 : o[b / 2] & 0xffffu);
                }
            }
        }
    }
    pool_and_store<T, EPC, KH, KW>(g, v, rows, w0, j0, Z + zoff);
}

// ---- rows of 10, 12 or 14 elements (bfloat16, 2 x 2 tiles, an even number of rows) --------------
// With the chunk kernel such a row is one and a half chunks, its pooled row five to seven 2-byte
// stores at odd offsets.  Here a thread owns a pair of rows: they are 4*W contiguous bytes of X
// (row pairs of all planes follow one another without a gap), its pooled row W/2 contiguous values
// of Z, so both tensors are plain arrays of per-thread records.  The records of a wave are
// contiguous and start on a multiple of 16 bytes: they are written to a wave-private piece of LDS
// and leave as whole 16-byte stores.  Sums and rounding as in the chunk kernel (bit-identical).
template <int W, bool PROD>
__global__ void __launch_bounds__(256) compress_narrow_kernel(Geom g, const bf16_t *__restrict__ X, bf16_t *__restrict__ Z,
                                                              uint32_t total, double inv_hp, Producer pr)
{
    constexpr int WP = W / 2;          // pooled values per thread = dwords per input row
    constexpr int XB = 4 * W;          // bytes of a thread's two rows
    constexpr int ZB = 2 * WP;         // bytes of its pooled row
    __shared__ __align__(16) unsigned char lds[4 * 64 * (PROD ? XB + 2 * ZB : ZB)];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char *zbuf = lds + wave * 64 * (PROD ? XB + 2 * ZB : ZB);
    const uint32_t idx = blockIdx.x * 256u + threadIdx.x, first = idx - lane;
    const bool live = idx < total;
    const bool whole = first + 64 <= total; // every lane of the wave has a record

    const rsrc_t rs = make_rsrc(X, total * (uint32_t)XB);
    constexpr int NL = (XB + 15) / 16; // 16-byte loads that cover a record (the last may reach into the next one)
    uint32_t d[4 * NL];
#pragma unroll
    for (int k = 0; k < NL; ++k) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, live ? idx * (uint32_t)XB + 16u * k : kNoLoad, 0, 0);
        d[4 * k] = v[0]; d[4 * k + 1] = v[1]; d[4 * k + 2] = v[2]; d[4 * k + 3] = v[3];
    }
    auto lo = [](uint32_t w) { return __uint_as_float(w << 16); };
    auto hi = [](uint32_t w) { return __uint_as_float(w & 0xffff0000u); };
    // pooled row of the two rows in d (dwords [0, WP) and [WP, 2*WP)): row-then-column sums
    auto pool = [&](const uint32_t (&x)[4 * NL], bf16_t (&out)[WP]) {
#pragma unroll
        for (int j = 0; j < WP; ++j) {
            const float a = lo(x[j]), b = hi(x[j]), c = lo(x[WP + j]), e = hi(x[WP + j]);
            float sum = 0.f;
            sum += a; sum += b; sum += c; sum += e;
            out[j] = f32_to_bf16(g.pmax ? fmaxf(fmaxf(fmaxf(a, b), c), e) : sum * 0.25f);
        }
    };
    bf16_t zr[WP];
    if constexpr (PROD) {
        unsigned char *xbuf = zbuf + 64 * 2 * ZB;
        if (pr.Zin) {
            // the producer's own saved record: its input pooled as it is
            pool(d, zr);
#pragma unroll
            for (int j = 0; j < WP; ++j) ((bf16_t *)(zbuf + 64 * ZB))[lane * WP + j] = zr[j];
            flush_records<ZB>(zbuf + 64 * ZB, (unsigned char *)pr.Zin, first, lane, whole, live);
        }
        // the next layer's input, rounded to its storage type; its pooled map from the rounded values
        const uint32_t plane = udiv(min(idx, total - 1), inv_hp);
        const uint32_t ch = plane - udiv(plane, pr.inv_c) * (uint32_t)g.C;
        const float sc = pr.scale[ch], sh = pr.shift[ch];
#pragma unroll
        for (int k = 0; k < W; ++k)
            d[k] = f32x2_to_bf16x2(fmaxf(fmaf(sc, lo(d[k]), sh), 0.f), fmaxf(fmaf(sc, hi(d[k]), sh), 0.f));
        typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
#pragma unroll
        for (int k = 0; k < W / 2; ++k) *(u32x2 *)(xbuf + lane * XB + 8 * k) = u32x2{d[2 * k], d[2 * k + 1]};
        flush_records<XB>(xbuf, (unsigned char *)pr.Xn, first, lane, whole, live);
    }
    pool(d, zr);
#pragma unroll
    for (int j = 0; j < WP; ++j) ((bf16_t *)zbuf)[lane * WP + j] = zr[j];
    flush_records<ZB>(zbuf, (unsigned char *)Z, first, lane, whole, live);
}

template <typename T, int EPC> bool launch_epc(const Geom &g, const void *X, void *Z, hipStream_t st, const Producer *prod = nullptr)
{
    const int cpr = (g.W + EPC - 1) / EPC;
    const long total = (long)g.N * g.C * g.Hp * cpr;
    if (total >= (1L << 31) || cpr >= (1 << 16) || g.Hp >= (1 << 16)) return false; // udiv's range
    const dim3 grid((unsigned)((total + 255) / 256));
#define CAC_LAUNCH(KH, KW)                                                                                            \
    if (prod)                                                                                                         \
        hipLaunchKernelGGL((compress_kernel<T, EPC, KH, KW, true>), grid, dim3(256), 0, st, g, (const T *)X, (T *)Z, cpr, \
                           (uint32_t)total, 1.0 / cpr, 1.0 / g.Hp, *prod);                                            \
    else                                                                                                              \
        hipLaunchKernelGGL((compress_kernel<T, EPC, KH, KW, false>), grid, dim3(256), 0, st, g, (const T *)X, (T *)Z, cpr, \
                           (uint32_t)total, 1.0 / cpr, 1.0 / g.Hp, Producer{})
    if (g.kh == 2 && g.kw == 2) { CAC_LAUNCH(2, 2); }
    else if (g.kh == 4 && g.kw == 4) { CAC_LAUNCH(4, 4); }
    else if (g.kh == 1 && g.kw == 1) { CAC_LAUNCH(1, 1); }
    else if (g.kh == 2 && g.kw == 4) { CAC_LAUNCH(2, 4); }
    else if (g.kh == 4 && g.kw == 2) { CAC_LAUNCH(4, 2); }
    else return false;
#undef CAC_LAUNCH
    return true;
}

} // namespace

static bool launch_fast(const Geom &g, int dtype, const void *X, void *Z, hipStream_t st, hipError_t *err, const Producer *prod)
{
    if ((long)g.N * g.C * g.H * g.W * 4 >= (1L << 31)) return false; // 32-bit buffer offsets
    bool ok;
    if (dtype == CAC_BF16 && g.kh == 2 && g.kw == 2 && g.H % 2 == 0 && (g.W == 10 || g.W == 12 || g.W == 14 || (prod && g.W == 28))) {
        // narrow rows: a thread per pair of rows (see compress_narrow_kernel).  Rows of 28: only the
        // producer form, whose stores of the activation gain more than its strided cold loads lose
        // (plain compression measured 4.05 TB/s this way against 4.9 with the chunk kernel)
        const long total = (long)g.N * g.C * g.Hp;
        const dim3 grid((unsigned)((total + 255) / 256));
#define CAC_NARROW(WW)                                                                                                   \
    if (g.W == WW) {                                                                                                     \
        if (prod)                                                                                                        \
            hipLaunchKernelGGL((compress_narrow_kernel<WW, true>), grid, dim3(256), 0, st, g, (const bf16_t *)X, (bf16_t *)Z,  \
                               (uint32_t)total, 1.0 / g.Hp, *prod);                                                      \
        else                                                                                                             \
            hipLaunchKernelGGL((compress_narrow_kernel<WW, false>), grid, dim3(256), 0, st, g, (const bf16_t *)X, (bf16_t *)Z, \
                               (uint32_t)total, 1.0 / g.Hp, Producer{});                                                 \
    }
        CAC_NARROW(10) CAC_NARROW(12) CAC_NARROW(14) CAC_NARROW(28)
#undef CAC_NARROW
        *err = hipGetLastError();
        return true;
    }
    if (dtype == CAC_F32) {
        if (g.kw > 4) return false;
        ok = launch_epc<float, 4>(g, X, Z, st, prod);
    } else {
        // narrow maps: 8-byte chunks so that a chunk does not span more than one row's worth
        ok = g.W >= 8 ? launch_epc<bf16_t, 8>(g, X, Z, st, prod) : (g.kw <= 4 ? launch_epc<bf16_t, 4>(g, X, Z, st, prod) : false);
    }
    if (ok) *err = hipGetLastError();
    return ok;
}

// True when the fast kernel covers the geometry (and has been launched).
bool launch_compress_fast(const Geom &g, int dtype, const void *X, void *Z, hipStream_t st, hipError_t *err)
{
    return launch_fast(g, dtype, X, Z, st, err, nullptr);
}

// The producer form: Xn = relu(scale[c] * Y + shift[c]) stored in the tensors' type, Zn = pooled Xn,
// Zin (optional) = pooled Y, all from one read of Y.
bool launch_producer_fast(const Geom &g, int dtype, const void *Y, const float *scale, const float *shift, void *Xn, void *Zn, void *Zin,
                          hipStream_t st, hipError_t *err)
{
    const Producer prod{scale, shift, Xn, Zin, 1.0 / g.C};
    return launch_fast(g, dtype, Y, Zn, st, err, &prod);
}

} // namespace cac
