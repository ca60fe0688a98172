// Weight gradient from the compressed activation for the float path and for every geometry the
// MFMA kernels do not take (5x5 and 7x7 filters, pooling tiles that are not powers of two, ...):
// an LDS-tiled multiply-add kernel in float arithmetic, gfx950.
//
//   dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] * xhat[n,c,p*SG+r-ph,q*SG+s-pw],
//   xhat[n,c,h,w] = Z[n,c,h/kh,w/kw]      (weight-gradient formula of the compression figure;
//                                           inflation by replication)
//
// A workgroup of 256 threads owns a 16 (o) x 16 (c) patch of dW, all R*S taps (a thread keeps the
// taps of one (o, c) pair in registers), and a slice of the pixels.  Per unit (PR output rows of
// one image) it stages the dY rows and the input rows they meet -- inflated from Z and zero-padded
// on the way, so the inflated activation exists only there -- in LDS as floats, then every thread
// walks the rows four output pixels at a time: one 16-byte read of dY and two or three of the
// xhat row feed 4*S multiply-adds per filter row.  Lanes that share an output channel (or an
// input channel) read the same LDS address, which is a broadcast.
// Pixel slices write partial sums to the workspace; dw_reduce adds them in a fixed order.
#include "common.h"
#include "dw_tiled.h"

namespace cac {

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ uint32_t fdiv(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

template <typename T, int R, int S, int SG>
__global__ void __launch_bounds__(256) dw_tiled_kernel(DwTiledParams p)
{
    constexpr int TO = 16, TC = 16;
    constexpr int NX = (3 * SG + S + 3) / 4; // 16-byte pieces of an xhat row that four output pixels meet
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float *sDY = (float *)smem_raw;                  // [TO][PR][QW] (+ 4 per output channel)
    float *sX = sDY + TO * p.dy_stride;              // [TC][XR][XW] (+ 4 per input channel)
    const Geom &g = p.g;
    const T *Z = (const T *)p.Z, *dY = (const T *)p.dY;

    const int ntiles = p.tiles_o * p.tiles_c;
    const int slice = blockIdx.x / ntiles, tile = blockIdx.x - slice * ntiles;
    const int o0 = (tile / p.tiles_c) * TO, c0 = (tile % p.tiles_c) * TC;
    const int tid = threadIdx.x, to = tid >> 4, tc = tid & 15;

    float acc[R][S];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int s = 0; s < S; ++s) acc[r][s] = 0.f;

    const int u_begin = slice * p.units_per_slice, u_end = min(u_begin + p.units_per_slice, p.nunits);
    for (int u = u_begin; u < u_end; ++u) {
        const int n = fdiv(u, p.m_rb), p0 = (u - n * p.RB) * p.PR;
        // ---- stage dY: [to][pr][q], zero beyond K, P, Q
        for (int i = tid; i < TO * p.PR * p.QW; i += 256) {
            const int t = fdiv(i, p.m_qw), q = i - t * p.QW, a = fdiv(t, p.m_pr), pr = t - a * p.PR;
            const int o = o0 + a, pp = p0 + pr;
            float v = 0.f;
            if (o < g.K && pp < g.P && q < g.Q) v = Elem<T>::load(dY + (((long)n * g.K + o) * g.P + pp) * g.Q + q);
            sDY[a * p.dy_stride + pr * p.QW + q] = v;
        }
        // ---- stage xhat: [tc][xr][xc] = Z[n][c][h/kh][w/kw] with h = p0*SG - ph + xr, w = xc - pw
        for (int i = tid; i < TC * p.XR * p.XW; i += 256) {
            const int t = fdiv(i, p.m_xw), xc = i - t * p.XW, e = fdiv(t, p.m_xr), xr = t - e * p.XR;
            const int c = c0 + e, h = p0 * SG - g.ph + xr, w = xc - g.pw;
            float v = 0.f;
            if (c < g.C && h >= 0 && h < g.H && w >= 0 && w < g.W)
                v = Elem<T>::load(Z + (((long)n * g.C + c) * g.Hp + fdiv(h, p.m_kh)) * g.Wp + fdiv(w, p.m_kw));
            sX[e * p.x_stride + xr * p.XW + xc] = v;
        }
        __syncthreads();
        // ---- multiply-add: four output pixels of a row per step
        const float *gy = sDY + to * p.dy_stride;
        const float *xh = sX + tc * p.x_stride;
        for (int pr = 0; pr < p.PR; ++pr) {
            for (int q4 = 0; q4 < p.QW; q4 += 4) {
                const f32x4 gv = *(const f32x4 *)(gy + pr * p.QW + q4);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const float *row = xh + (pr * SG + r) * p.XW + q4 * SG;
                    float x[4 * NX];
#pragma unroll
                    for (int k = 0; k < NX; ++k) {
                        const f32x4 v = *(const f32x4 *)(row + 4 * k);
                        x[4 * k] = v[0]; x[4 * k + 1] = v[1]; x[4 * k + 2] = v[2]; x[4 * k + 3] = v[3];
                    }
#pragma unroll
                    for (int s = 0; s < S; ++s)
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc[r][s] += gv[j] * x[j * SG + s];
                }
            }
        }
        __syncthreads();
    }
    const int o = o0 + to, c = c0 + tc;
    if (o < g.K && c < g.C) {
        float *out = (p.direct ? p.out : p.out + (long)slice * g.K * g.C * R * S) + ((long)o * g.C + c) * R * S;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int s = 0; s < S; ++s) out[r * S + s] = acc[r][s];
    }
}

uint32_t magic_of(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }

template <typename T, int R, int SG> hipError_t launch_rs(const DwTiledParams &p, dim3 grid, hipStream_t st)
{
    hipLaunchKernelGGL((dw_tiled_kernel<T, R, R, SG>), grid, dim3(256), p.lds_bytes, st, p);
    return hipGetLastError();
}
template <typename T> hipError_t launch_t(const DwTiledParams &p, dim3 grid, hipStream_t st)
{
    const int R = p.g.R, SG = p.g.sh;
#define CAC_TILED(RR)                                  \
    if (R == RR) {                                     \
        if (SG == 1) return launch_rs<T, RR, 1>(p, grid, st); \
        return launch_rs<T, RR, 2>(p, grid, st);       \
    }
    CAC_TILED(1) CAC_TILED(3) CAC_TILED(5) CAC_TILED(7)
#undef CAC_TILED
    return hipErrorInvalidValue;
}

} // namespace

bool dw_tiled_plan(const Geom &g, int dtype, DwTiledPlan *plan)
{
    (void)dtype;
    if (g.R != g.S || (g.R != 1 && g.R != 3 && g.R != 5 && g.R != 7)) return false;
    if (g.sh != g.sw || (g.sh != 1 && g.sh != 2)) return false;
    if ((long)g.N * g.K * g.P * g.Q >= (1L << 31) || (long)g.N * g.C * g.Hp * g.Wp >= (1L << 31)) return false;
    DwTiledParams p{};
    p.g = g;
    p.QW = (g.Q + 3) & ~3;
    p.XW = ((p.QW - 1) * g.sh + g.S + 3 + 3) & ~3; // what the last step's widest read reaches, in whole pieces
    p.XW = max(p.XW, ((p.QW - 4) * g.sh + 4 * ((3 * g.sh + g.S + 3) / 4) + 3) & ~3);
    p.tiles_o = (g.K + 15) / 16;
    p.tiles_c = (g.C + 15) / 16;
    const int ntiles = p.tiles_o * p.tiles_c;
    // rows per unit: as many as LDS takes (48 KB) while the launch still has a few hundred workgroups
    int best = 0;
    const long min_wg = 256; // (measured on the single 16-channel float layer: 11.5 us with 256 workgroups, 28 us with 32)
    for (int pr = 8; pr >= 1; pr >>= 1) {
        if (pr > g.P && pr > 1) continue;
        const int xr = (pr - 1) * g.sh + g.R;
        const long lds = 4L * (16 * (pr * p.QW + 4) + 16 * (xr * p.XW + 4));
        if (lds > 48 * 1024) continue;
        if (!best) best = pr;
        if ((long)ntiles * g.N * ((g.P + pr - 1) / pr) >= min_wg) { best = pr; break; }
        best = pr; // fewer rows per unit: more units to share out
    }
    if (!best) return false;
    p.PR = best;
    p.XR = (p.PR - 1) * g.sh + g.R;
    p.dy_stride = p.PR * p.QW + 4;
    p.x_stride = p.XR * p.XW + 4;
    p.lds_bytes = 4 * (16 * p.dy_stride + 16 * p.x_stride);
    p.RB = (g.P + p.PR - 1) / p.PR;
    p.nunits = g.N * p.RB;
    const int want = max(1, min(p.nunits, 1024 / ntiles));
    p.units_per_slice = (p.nunits + want - 1) / want;
    p.nslices = (p.nunits + p.units_per_slice - 1) / p.units_per_slice;
    p.direct = p.nslices == 1;
    p.m_rb = magic_of(p.RB);
    p.m_kh = magic_of(g.kh);
    p.m_kw = magic_of(g.kw);
    p.m_qw = magic_of(p.QW);
    p.m_pr = magic_of(p.PR);
    p.m_xw = magic_of(p.XW);
    p.m_xr = magic_of(p.XR);
    plan->p = p;
    plan->grid = (unsigned)(ntiles * p.nslices);
    plan->partial_bytes = p.direct ? 0 : (size_t)p.nslices * g.K * g.C * g.R * g.S * sizeof(float);
    return true;
}

hipError_t launch_dw_tiled(const DwTiledPlan &plan, int dtype, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                           DwReduceTail *defer)
{
    DwTiledParams p = plan.p;
    p.Z = Z;
    p.dY = dY;
    p.out = p.direct ? dW : (float *)ws;
    if (defer) defer->blocks = 0;
    hipError_t e = dtype == CAC_F32 ? launch_t<float>(p, dim3(plan.grid), st) : launch_t<bf16_t>(p, dim3(plan.grid), st);
    if (e != hipSuccess || p.direct) return e;
    const DwReduceTail t = make_reduce_tail((const float *)ws, dW, (long)p.g.K * p.g.C * p.g.R * p.g.S, p.nslices);
    if (defer) {
        *defer = t;
        return hipSuccess;
    }
    return launch_dw_reduce(t, st);
}

} // namespace cac
