// Weight gradient from the compressed activation as an MFMA implicit GEMM
// (bfloat16 operands, float accumulation), gfx950.
//
//   dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] * xhat[n,c,p*SG+r-PAD,q*SG+s-PAD],
//   xhat[n,c,h,w] = Z[n,c,h/kh,w/kw]        (weight-gradient formula of the
//                                             compression figure; inflation by
//                                             replication)
//
// GEMM view: M = output channels o, N = (input channel c, filter tap), K = pixels.
// A workgroup (4 waves, 2x2) owns a 64 (o) x 64 (c) x all-taps tile and a slice
// of the pixels; each wave a 32 x 32 x taps tile, i.e. one 32x32 accumulator
// block per tap.  The pixel dimension is walked in "segments" of 8 consecutive
// output pixels of one output row: a 32x32x16 MFMA consumes two segments, one in
// lanes 0-31 and one in lanes 32-63 (rows rho and rho+1 of the staged chunk).
//
// Staging per chunk (NBI images x PR output rows):
//   sDY [64 o][LR rows][Qpad]      dY, rows padded with zeros to a multiple of 8
//   sX  [64 c][slots][XW]          the needed rows of Z, expanded along the row
//                                  to full input width (xhat rows), zeros past W;
//                                  the last slot is an all-zero row
// The inflated activation exists only here: expanded horizontally when written
// to LDS, expanded vertically by mapping an input row h to the slot of Z row
// h/kh.  The filter taps along the row are produced in registers by shifting a
// sliding window of xhat blocks with v_perm.
#include "common.h"
#include "dw_mfma.h"

namespace cac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ uint32_t fdiv(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

__device__ __forceinline__ uint32_t pack16(uint32_t lo, uint32_t hi) { return (lo & 0xffffu) | (hi << 16); }

// Result: low half = half `ha` of a, high half = half `hb` of b.
template <int ha, int hb> __device__ __forceinline__ uint32_t halves(uint32_t a, uint32_t b)
{
    constexpr uint32_t sel = (2 * ha) | ((2 * ha + 1) << 8) | ((4 + 2 * hb) << 16) | ((5 + 2 * hb) << 24);
    return __builtin_amdgcn_perm(b, a, sel);
}

constexpr int kMaxDy = 4; // 16-byte dY items a thread moves per chunk
constexpr int kMaxZ = 8;  // 8-byte Z items a thread moves per chunk

// A window of one xhat row held in registers: the last dword of the block left
// of the current position and NB blocks starting at it.
template <int NB> struct Window {
    uint32_t prev3;
    u32x4 blk[NB];
};

// Element `e` (relative to the first element of blk[0]; -2 <= e < 8*NB) as
// (register, half).
template <int NB, int e> __device__ __forceinline__ uint32_t win_reg(const Window<NB> &w)
{
    static_assert(e >= -2 && e < 8 * NB, "window too small");
    if constexpr (e < 0)
        return w.prev3;
    else
        return w.blk[e / 8][(e % 8) / 2];
}
template <int e> constexpr int win_half() { return ((e % 2) + 2) % 2; }

// B fragment for filter column s: pixel j of the segment needs element
// SG*j + s - PAD of the window.
template <int NB, int SG, int PAD, int s> __device__ __forceinline__ bf16x8 make_frag(const Window<NB> &w)
{
    union { u32x4 u; bf16x8 v; } f;
#define CAC_FRAG_DWORD(i)                                                                        \
    {                                                                                            \
        constexpr int e0 = SG * (2 * i) + s - PAD, e1 = SG * (2 * i + 1) + s - PAD;              \
        f.u[i] = halves<win_half<e0>(), win_half<e1>()>(win_reg<NB, e0>(w), win_reg<NB, e1>(w)); \
    }
    CAC_FRAG_DWORD(0) CAC_FRAG_DWORD(1) CAC_FRAG_DWORD(2) CAC_FRAG_DWORD(3)
#undef CAC_FRAG_DWORD
    return f.v;
}

// 8 consecutive bf16 starting at src, of which only the first `left` exist;
// VEC = widest vector the address is aligned for.
template <int VEC> __device__ __forceinline__ u32x4 load8(const bf16_t *src, int left)
{
    u32x4 v = {0, 0, 0, 0};
    if constexpr (VEC == 8) {
        v = *(const u32x4 *)src;
    } else if constexpr (VEC == 4) {
        u32x2 a = *(const u32x2 *)src, b = {0, 0};
        if (left > 4) b = *(const u32x2 *)(src + 4);
        v = u32x4{a[0], a[1], b[0], b[1]};
    } else if constexpr (VEC == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (left > 2 * j) v[j] = *(const uint32_t *)(src + 2 * j);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t lo = left > 2 * j ? src[2 * j] : 0, hi = left > 2 * j + 1 ? src[2 * j + 1] : 0;
            v[j] = pack16(lo, hi);
        }
    }
    return v;
}

template <int VEC> __device__ __forceinline__ u32x2 load4(const bf16_t *src, int left)
{
    u32x2 v = {0, 0};
    if constexpr (VEC == 4) {
        v = *(const u32x2 *)src;
    } else if constexpr (VEC == 2) {
        v[0] = *(const uint32_t *)src;
        if (left > 2) v[1] = *(const uint32_t *)(src + 2);
    } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            uint32_t lo = left > 2 * j ? src[2 * j] : 0, hi = left > 2 * j + 1 ? src[2 * j + 1] : 0;
            v[j] = pack16(lo, hi);
        }
    }
    return v;
}

template <int R, int S, int SG, int PAD>
__global__ void __launch_bounds__(256, 2) dw_mfma_kernel(DwMfmaParams p)
{
    constexpr int T = R * S;
    // blocks of 8 xhat elements a segment touches, counted from block SG*seg
    constexpr int NB = (7 * SG + S - 1 - PAD) / 8 + 1;
    static_assert(PAD <= 2 && SG <= NB, "unsupported filter geometry");

    extern __shared__ __align__(16) unsigned char smem[];
    // [zero row][buffer 0: sDY, sX][buffer 1: sDY, sX]
    const bf16_t *sZero = (const bf16_t *)smem;
    bf16_t *sBuf = (bf16_t *)smem + p.XW;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1, half = lane >> 5, l32 = lane & 31;

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that each
    // XCD works on consecutive (slice, o-tile, c-tile) triples and re-reads of dY
    // and Z hit its own L2.
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= p.total_wg) return;
    const int ntiles = p.tiles_o * p.tiles_c;
    const int slice = v / ntiles, tile = v - slice * ntiles;
    const int ot = tile / p.tiles_c, ct = tile - ot * p.tiles_c;
    const int o0 = ot * 64, c0 = ct * 64;

    // Everything in LDS starts finite (zero): pad columns, the spare row of an odd
    // chunk and the zero row are multiplied with something in every MFMA.
    for (int i = tid; i < p.lds_bytes / 16; i += 256) ((u32x4 *)smem)[i] = u32x4{0, 0, 0, 0};

    const int ci_begin = slice * p.chunks_per_slice;
    const int ci_end = min(ci_begin + p.chunks_per_slice, p.nchunks);

    // ---- what this thread copies, fixed for the whole kernel ----------------------
    // dY: LDY lanes share one output channel's rows; item j = (row rho, segment sg)
    const uint32_t dyj = tid & (p.LDY - 1), dyo = tid >> p.ldy_log2;
    const uint32_t dy_rho = fdiv(dyj, p.m_segs), dy_sg = dyj - dy_rho * p.SEGS;
    const uint32_t dy_ni = fdiv(dy_rho, p.m_pr), dy_pr = dy_rho - dy_ni * p.PR;
    const bool dy_write = dyj < (uint32_t)p.rowitems;             // lanes past the row's items idle
    const bool dy_real = dy_write && dy_rho < (uint32_t)p.LR;     // the spare row stays zero
    const int dy_left = p.Q - (int)dy_sg * 8;
    const uint32_t dy_rel = ((dy_ni * p.K + dyo) * p.P + dy_pr) * p.Q + dy_sg * 8;
    const uint32_t dy_gstep = (256u >> p.ldy_log2) * p.P * p.Q;   // next pass: 256/LDY channels on
    const uint32_t dy_lds = dyo * p.dy_ostride + dyj * 8;
    const uint32_t dy_lstep = (256u >> p.ldy_log2) * p.dy_ostride;
    // Z: LPC lanes share one input channel; item j = (image ni, slot sl, vector zv)
    const uint32_t zj = tid & (p.LPC - 1), zc = tid >> p.lpc_log2;
    const uint32_t z_row = fdiv(zj, p.m_zv), z_zv = zj - z_row * p.ZV;
    const uint32_t z_ni = fdiv(z_row, p.m_nz), z_sl = z_row - z_ni * p.NZ;
    const bool z_write = zj < (uint32_t)p.citems;
    const int z_left = p.Wp - (int)z_zv * 4;
    const uint32_t z_rel = ((z_ni * p.C + zc) * p.Hp + z_sl) * p.Wp + z_zv * 4;
    const uint32_t z_gstep = (256u >> p.lpc_log2) * p.Hp * p.Wp;
    const uint32_t z_lds = zc * p.x_cstride + z_row * p.XW + ((z_zv * 4) << p.kw_log2);
    const uint32_t z_lstep = (256u >> p.lpc_log2) * p.x_cstride;
    const int z_col0 = (int)(z_zv * 4) << p.kw_log2;              // first xhat column of the item

    u32x4 pre_dy[kMaxDy];
    u32x2 pre_z[kMaxZ];

    // ---- global -> registers for one chunk ----------------------------------------
    auto prefetch = [&](int ci) {
        const int ig = ci / p.RB, rb = ci - ig * p.RB;
        const int n0 = ig * p.NBI, p0 = rb * p.PR;
        const int zbase = max(0, (p0 * SG - PAD) >> p.kh_log2);
        {
            const bool ok = dy_real && n0 + (int)dy_ni < p.N && p0 + (int)dy_pr < p.P;
            const bf16_t *src = p.dY + ((uint32_t)(n0 * p.K + o0) * p.P + p0) * p.Q + dy_rel;
            const int olim = p.K - o0 - (int)dyo; // passes with i*OPP < olim are real channels
#define CAC_DY_PASSES(VEC)                                                                        \
    _Pragma("unroll") for (int i = 0; i < kMaxDy; ++i)                                            \
    {                                                                                             \
        u32x4 val = {0, 0, 0, 0};                                                                 \
        if (i < p.dy_passes && ok && (i << (8 - p.ldy_log2)) < olim) val = load8<VEC>(src + i * dy_gstep, dy_left); \
        pre_dy[i] = val;                                                                          \
    }
            if (p.dy_vec == 8) { CAC_DY_PASSES(8) }
            else if (p.dy_vec == 4) { CAC_DY_PASSES(4) }
            else if (p.dy_vec == 2) { CAC_DY_PASSES(2) }
            else { CAC_DY_PASSES(1) }
#undef CAC_DY_PASSES
        }
        {
            const bool ok = z_write && n0 + (int)z_ni < p.N && zbase + (int)z_sl < p.Hp;
            const bf16_t *src = p.Z + ((uint32_t)(n0 * p.C + c0) * p.Hp + zbase) * p.Wp + z_rel;
            const int clim = p.C - c0 - (int)zc;
#define CAC_Z_PASSES(VEC)                                                                         \
    _Pragma("unroll") for (int i = 0; i < kMaxZ; ++i)                                             \
    {                                                                                             \
        u32x2 val = {0, 0};                                                                       \
        if (i < p.z_passes && ok && (i << (8 - p.lpc_log2)) < clim) val = load4<VEC>(src + i * z_gstep, z_left); \
        pre_z[i] = val;                                                                           \
    }
            if (p.z_vec == 4) { CAC_Z_PASSES(4) }
            else if (p.z_vec == 2) { CAC_Z_PASSES(2) }
            else { CAC_Z_PASSES(1) }
#undef CAC_Z_PASSES
        }
    };

    // ---- registers -> LDS buffer (with the horizontal inflation) --------------------
    auto stage = [&](bf16_t *sDY, bf16_t *sX) {
        if (dy_write) {
#pragma unroll
            for (int i = 0; i < kMaxDy; ++i)
                if (i < p.dy_passes) *(u32x4 *)(sDY + dy_lds + i * dy_lstep) = pre_dy[i];
        }
        if (z_write) {
#pragma unroll
            for (int i = 0; i < kMaxZ; ++i) {
                if (i < p.z_passes) {
                    const u32x2 z = pre_z[i];
                    bf16_t *dst = sX + z_lds + i * z_lstep;
                    // pooled value e of the vector, in both halves of a dword
                    const uint32_t d0 = halves<0, 0>(z[0], z[0]), d1 = halves<1, 1>(z[0], z[0]);
                    const uint32_t d2 = halves<0, 0>(z[1], z[1]), d3 = halves<1, 1>(z[1], z[1]);
                    // columns at or beyond W are zero (a ragged last pooling tile reaches past W)
                    auto put = [&](int off, u32x4 x) {
                        const int left = p.W - z_col0 - off;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (left <= 2 * j) x[j] = 0;
                            else if (left == 2 * j + 1) x[j] &= 0xffffu;
                        }
                        *(u32x4 *)(dst + off) = x;
                    };
                    if (p.kw_log2 == 0) {
                        *(u32x2 *)dst = z; // no horizontal inflation; zeros past W come from the load
                    } else if (p.kw_log2 == 1) {
                        put(0, u32x4{d0, d1, d2, d3});
                    } else if (p.kw_log2 == 2) {
                        put(0, u32x4{d0, d0, d1, d1});
                        put(8, u32x4{d2, d2, d3, d3});
                    } else {
                        put(0, u32x4{d0, d0, d0, d0});
                        put(8, u32x4{d1, d1, d1, d1});
                        put(16, u32x4{d2, d2, d2, d2});
                        put(24, u32x4{d3, d3, d3, d3});
                    }
                }
            }
        }
    };

    f32x16 acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][j] = 0.f;

    // ---- MFMA over one staged chunk --------------------------------------------------
    auto compute = [&](int ci, const bf16_t *sDY, const bf16_t *sX) {
        const int ig = ci / p.RB, rb = ci - ig * p.RB;
        const int n0 = ig * p.NBI, p0 = rb * p.PR;
        const int zbase = max(0, (p0 * SG - PAD) >> p.kh_log2);
        const bf16_t *xc = sX + (wn * 32 + l32) * p.x_cstride;
        const bf16_t *ac = sDY + (wm * 32 + l32) * p.dy_ostride;
        for (int rp = 0; rp < p.LRpad / 2; ++rp) {
            const uint32_t rho = 2 * rp + half;
            const uint32_t ni = fdiv(rho, p.m_pr);
            const int pp = p0 + (int)(rho - ni * p.PR);
            const bool row_ok = rho < (uint32_t)p.LR && pp < p.P && n0 + (int)ni < p.N;
            const bf16_t *xrow[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int h = pp * SG + r - PAD;
                const bool ok = row_ok && h >= 0 && h < p.H;
                xrow[r] = ok ? xc + ((int)ni * p.NZ + (h >> p.kh_log2) - zbase) * p.XW : sZero;
            }
            const bf16_t *arow = ac + rho * p.Qpad;
            Window<NB> win[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                win[r].prev3 = 0;
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    win[r].blk[b] = b < p.XB ? *(const u32x4 *)(xrow[r] + 8 * b) : u32x4{0, 0, 0, 0};
            }
            for (int seg = 0; seg < p.SEGS; ++seg) {
                union { u32x4 u; bf16x8 v; } a;
                a.u = *(const u32x4 *)(arow + seg * 8);
#pragma unroll
                for (int r = 0; r < R; ++r) {
#define CAC_TAP(s)                                                                                       \
    if constexpr (s < S)                                                                                 \
        acc[r * S + s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, make_frag<NB, SG, PAD, s>(win[r]), \
                                                                 acc[r * S + s], 0, 0, 0);
                    CAC_TAP(0) CAC_TAP(1) CAC_TAP(2)
#undef CAC_TAP
                }
                // slide every window SG blocks to the right
                const int nxt = (seg + 1) * SG; // block index of the new blk[0]
                const bool more = seg + 1 < p.SEGS;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    win[r].prev3 = win[r].blk[SG - 1][3];
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        if (b + SG < NB)
                            win[r].blk[b] = win[r].blk[b + SG];
                        else
                            win[r].blk[b] = (more && nxt + b < p.XB) ? *(const u32x4 *)(xrow[r] + 8 * (nxt + b))
                                                                    : u32x4{0, 0, 0, 0};
                    }
                }
            }
        }
    };

    // Double-buffered: while the MFMAs run on buffer b, the next chunk's global
    // loads are in flight and are written to buffer b^1 afterwards; one barrier
    // per chunk separates "all waves done reading b^1's previous content" from
    // its refill and the refill from its use.
    bf16_t *const sDY0 = sBuf, *const sX0 = sDY0 + 64 * p.dy_ostride;
    bf16_t *const sDY1 = sX0 + 64 * p.x_cstride, *const sX1 = sDY1 + 64 * p.dy_ostride;
    __syncthreads(); // zero fill done
    if (ci_begin < ci_end) {
        prefetch(ci_begin);
        stage(sDY0, sX0);
    }
    __syncthreads();
    int buf = 0;
    for (int ci = ci_begin; ci < ci_end; ++ci, buf ^= 1) {
        const bool more = ci + 1 < ci_end;
        if (more) prefetch(ci + 1);
        compute(ci, buf ? sDY1 : sDY0, buf ? sX1 : sX0);
        if (more) stage(buf ? sDY0 : sDY1, buf ? sX0 : sX1);
        __syncthreads();
    }

    // ---- epilogue --------------------------------------------------------------------
    // accumulator register j of lane l holds row 8*(j/4) + 4*(l/32) + j%4, column l%32
    if (p.direct) {
        const int c = c0 + wn * 32 + l32;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int o = o0 + wm * 32 + 8 * (j / 4) + 4 * half + (j % 4);
            if (o < p.K && c < p.C) {
                float *dst = p.out + ((long)o * p.C + c) * T;
#pragma unroll
                for (int t = 0; t < T; ++t) dst[t] = acc[t][j];
            }
        }
    } else {
        // partial sums in fragment order: [slice][tile][wave][tap][register][lane]
        float *dst = p.out + ((((long)slice * ntiles + tile) * 4 + wave) * T) * 16 * 64 + lane;
#pragma unroll
        for (int t = 0; t < T; ++t)
#pragma unroll
            for (int j = 0; j < 16; ++j) dst[(t * 16 + j) * 64] = acc[t][j];
    }
}

// Sums the slices' partial tiles in slice order and writes dW in its own layout.
__global__ void __launch_bounds__(256) dw_reduce_kernel(const float *__restrict__ part, float *__restrict__ dW, int nslices,
                                                        int tiles_o, int tiles_c, int T, int K, int C)
{
    const long per_slice = (long)tiles_o * tiles_c * 4 * T * 16 * 64;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= per_slice) return;
    float s = 0.f;
    for (int sl = 0; sl < nslices; ++sl) s += part[sl * per_slice + idx];
    const int lane = idx & 63;
    long t1 = idx >> 6;
    const int j = t1 & 15;
    t1 >>= 4;
    const int tap = t1 % T;
    t1 /= T;
    const int wave = t1 & 3;
    const int tile = t1 >> 2;
    const int ot = tile / tiles_c, ct = tile - ot * tiles_c;
    const int o = ot * 64 + (wave & 1) * 32 + 8 * (j / 4) + 4 * (lane >> 5) + (j % 4);
    const int c = ct * 64 + (wave >> 1) * 32 + (lane & 31);
    if (o < K && c < C) dW[((long)o * C + c) * T + tap] = s;
}

uint32_t magic_of(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }

int largest_vec(int extent, int cap)
{
    int v = 1;
    while (v < cap && extent % (2 * v) == 0) v *= 2;
    return v;
}

template <int R, int S, int SG, int PAD> hipError_t launch_variant(const DwMfmaParams &p, dim3 grid, hipStream_t st)
{
    auto kern = dw_mfma_kernel<R, S, SG, PAD>;
    static bool attr_set = false; // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), p.lds_bytes, st, p);
    return hipGetLastError();
}

} // namespace

bool dw_mfma_plan(const Geom &g, int dtype, DwMfmaPlan *plan)
{
    if (dtype != CAC_BF16) return false;
    if (g.R != g.S || g.sh != g.sw || g.ph != g.pw) return false;
    const bool f3 = g.R == 3 && g.ph == 1, f1 = g.R == 1 && g.ph == 0;
    if (!(f3 || f1) || (g.sh != 1 && g.sh != 2)) return false;
    auto log2_of = [](int k) { return k == 1 ? 0 : k == 2 ? 1 : k == 4 ? 2 : k == 8 ? 3 : -1; };
    const int khl = log2_of(g.kh), kwl = log2_of(g.kw);
    if (khl < 0 || kwl < 0) return false;
    if (g.Q > 256 || g.W > 1024) return false;
    const int T = g.R * g.S;

    DwMfmaParams base{};
    base.N = g.N; base.C = g.C; base.K = g.K; base.H = g.H; base.W = g.W; base.P = g.P; base.Q = g.Q;
    base.Hp = g.Hp; base.Wp = g.Wp;
    base.kh_log2 = khl; base.kw_log2 = kwl;
    base.SEGS = (g.Q + 7) / 8;
    base.Qpad = base.SEGS * 8;
    base.XB = (g.W + 7) / 8;
    base.ZV = (g.Wp + 3) / 4;
    base.XW = 8 * ((max(g.W, base.ZV * 4 * g.kw) + 7) / 8);

    // Fills the chunk-dependent fields; false when the chunk does not fit the
    // per-thread copy registers or the LDS budget of two workgroups per CU
    // (two buffers each).
    auto shape = [&](int nbi, int pr, DwMfmaParams &q) {
        q = base;
        q.NBI = nbi; q.PR = pr;
        q.RB = (g.P + pr - 1) / pr;
        q.LR = nbi * pr;
        q.LRpad = (q.LR + 1) & ~1;
        int nz = 1;
        for (int rb = 0; rb < q.RB; ++rb) {
            const int p0 = rb * pr, p1 = min(p0 + pr, g.P) - 1;
            const int zlo = max(0, (p0 * g.sh - g.ph) >> khl);
            const int hhi = min(g.H - 1, p1 * g.sh + g.R - 1 - g.ph);
            nz = max(nz, (hhi >> khl) - zlo + 1);
        }
        q.NZ = nz;
        q.rowitems = q.LRpad * q.SEGS;
        q.citems = nbi * nz * q.ZV;
        if (q.rowitems > 4 * kMaxDy || q.citems > 4 * kMaxZ) return false;
        auto pow2_at_least = [](int x) { int v = 4, l = 2; while (v < x) { v *= 2; ++l; } return l; };
        q.ldy_log2 = pow2_at_least(q.rowitems); q.LDY = 1 << q.ldy_log2; q.dy_passes = q.LDY / 4;
        q.lpc_log2 = pow2_at_least(q.citems);   q.LPC = 1 << q.lpc_log2; q.z_passes = q.LPC / 4;
        // strides: an odd number of 16-byte units so that the 32 lanes of a half
        // wave (one output channel / input channel each) read distinct LDS banks
        q.dy_ostride = 8 * (q.rowitems | 1);
        q.x_cstride = 8 * ((nbi * nz * (q.XW / 8)) | 1);
        q.lds_bytes = (q.XW + 2 * (64 * q.dy_ostride + 64 * q.x_cstride)) * 2;
        return q.lds_bytes <= 78 * 1024;
    };
    // Candidates: part of one image (nbi = 1, pr <= P) or several whole images.
    // Cost = MFMA steps spent per useful pixel row, then prefer longer chunks.
    DwMfmaParams best{};
    double best_cost = 1e30;
    auto consider = [&](int nbi, int pr) {
        DwMfmaParams q;
        if (!shape(nbi, pr, q)) return;
        const double steps = (double)q.RB * (q.LRpad / 2) * q.SEGS;      // per group of nbi images
        const double useful = (double)nbi * g.P * g.Q / 16.0;
        const double per_chunk = (q.LRpad / 2) * q.SEGS;
        const double cost = steps / useful * (1.0 + 2.5 / per_chunk);     // barrier + epilogue share
        if (cost < best_cost) { best_cost = cost; best = q; }
    };
    for (int pr = 1; pr <= g.P; ++pr) consider(1, pr);
    for (int nbi = 2; nbi <= min(g.N, 64); ++nbi) consider(nbi, g.P);
    if (best_cost > 1e29) return false;

    DwMfmaParams &p = plan->p;
    p = best;
    p.m_rowitems = magic_of(p.rowitems);
    p.m_segs = magic_of(p.SEGS);
    p.m_pr = magic_of(p.PR);
    p.m_citems = magic_of(p.citems);
    p.m_zv = magic_of(p.ZV);
    p.m_nz = magic_of(p.NZ);
    // widest aligned vector for the global reads (tensor bases are 16-byte aligned)
    p.dy_vec = largest_vec(g.Q, 8);
    p.z_vec = largest_vec(g.Wp, 4);

    p.tiles_o = (g.K + 63) / 64;
    p.tiles_c = (g.C + 63) / 64;
    const int ntiles = p.tiles_o * p.tiles_c;
    p.nchunks = ((g.N + p.NBI - 1) / p.NBI) * p.RB;
    // enough workgroups for two per CU on 256 CUs, each with at least two chunks
    int want = max(1, (512 + ntiles - 1) / ntiles);
    want = min(want, max(1, p.nchunks / 2));
    p.chunks_per_slice = (p.nchunks + want - 1) / want;
    p.nslices = (p.nchunks + p.chunks_per_slice - 1) / p.chunks_per_slice;
    p.total_wg = p.nslices * ntiles;
    p.direct = p.nslices == 1;
    plan->grid = ((p.total_wg + 7) / 8) * 8;
    plan->partial_bytes = p.direct ? 0 : (size_t)p.nslices * ntiles * 4 * T * 16 * 64 * sizeof(float);
    plan->variant = (f3 ? 0 : 2) + (g.sh == 2 ? 1 : 0);
    return true;
}

hipError_t launch_dw_mfma(const DwMfmaPlan &plan, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st)
{
    DwMfmaParams p = plan.p;
    p.Z = (const bf16_t *)Z;
    p.dY = (const bf16_t *)dY;
    p.out = p.direct ? dW : (float *)ws;
    dim3 grid(plan.grid);
    hipError_t e;
    switch (plan.variant) {
    case 0: e = launch_variant<3, 3, 1, 1>(p, grid, st); break;
    case 1: e = launch_variant<3, 3, 2, 1>(p, grid, st); break;
    case 2: e = launch_variant<1, 1, 1, 0>(p, grid, st); break;
    default: e = launch_variant<1, 1, 2, 0>(p, grid, st); break;
    }
    if (e != hipSuccess || p.direct) return e;
    const int T = plan.variant < 2 ? 9 : 1;
    const long per_slice = (long)p.tiles_o * p.tiles_c * 4 * T * 16 * 64;
    hipLaunchKernelGGL(dw_reduce_kernel, dim3((unsigned)((per_slice + 255) / 256)), dim3(256), 0, st,
                       (const float *)ws, dW, p.nslices, p.tiles_o, p.tiles_c, T, p.K, p.C);
    return hipGetLastError();
}

} // namespace cac
