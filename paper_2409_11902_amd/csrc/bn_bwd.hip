// Batch normalisation's backward pass from the pooled record of its input (the paper's conclusion
// names compressing what batch normalisation saves as a next step; the formulas are the textbook
// ones with the saved input replaced by its inflated record):
//   xhat~ = (Zin[n,c,h/kh,w/kw] - mean[c]) * invstd[c],  M = N*H*W
//   dbeta[c] = sum dy      dgamma[c] = sum dy * xhat~
//   dx = gamma[c] * invstd[c] * (dy - dbeta[c] / M - xhat~ * dgamma[c] / M)
// Bandwidth-bound, gfx950.  Three launches over the chunks of compress.hip (16 bytes of kh rows
// of dY and the pooled values under them, so that a pooled value is read once per tile):
//   1. partial sums: a block per (channel, slice of the channel's chunks over all images); a
//      channel is shared out over as many slices as it takes to have about 2048 blocks;
//   2. the slices of a channel added in a fixed order (skipped when a channel is one slice);
//   3. the element-wise pass, one thread per chunk, 16-byte stores.
// Everything is summed in an order that depends on the shape only: results are reproducible.
// Also here, for the helpers it shares: the bias gradient db = sum of dY over n, p, q (db_kernel).
#include "chunk.h"

namespace cac {

namespace {

constexpr int kT = 256;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

struct BnPlan {
    int cpr;               // chunks per row
    uint32_t ipp;          // chunks per plane (pooled rows x chunks per row)
    uint32_t per_channel;  // chunks of a channel: N * ipp
    uint32_t per_slice;    // chunks a block of the first launch goes through
    int S;                 // slices per channel
    uint32_t total;        // chunks of the tensor
    double inv_cpr, inv_ipp, inv_hp, inv_c;
};

// The chunk's dY values (rows past the plane read as zero) and what the pooled values under it say
// about the normalised input: xh[o] = (Z - mean) * invstd, 0 where the pooled column does not exist.
template <typename T, int EPC, int KH, int KW>
__device__ __forceinline__ void load_chunk(const Geom &g, rsrc_t rs_dy, const T *__restrict__ Zin, uint32_t plane, int i, int ch, float mu,
                                           float is, float (&v)[KH][EPC], float (&xh)[EPC / KW], int &rows)
{
    constexpr int OPC = EPC / KW;
    const int h0 = i * KH;
    rows = min(KH, g.H - h0);
#pragma unroll
    for (int a = 0; a < KH; ++a)
        Chunk<T, EPC>::load(rs_dy, (plane * g.H + h0 + a) * g.W + ch * EPC, a < rows, g.W & 1, v[a]);
    const T *z = Zin + ((long)plane * g.Hp + i) * g.Wp + ch * OPC;
#pragma unroll
    for (int o = 0; o < OPC; ++o) xh[o] = ch * OPC + o < g.Wp ? (Elem<T>::load(z + o) - mu) * is : 0.f;
}

template <typename T, int EPC, int KH, int KW>
__global__ void __launch_bounds__(kT) bn_partial_kernel(Geom g, BnPlan q, const T *__restrict__ Zin, const T *__restrict__ dY,
                                                        const float *__restrict__ mean, const float *__restrict__ invstd,
                                                        float *__restrict__ o_dy, float *__restrict__ o_dx)
{
    constexpr int OPC = EPC / KW;
    __shared__ float red[2][kT / 64];
    const int c = blockIdx.x / q.S, s = blockIdx.x - c * q.S;
    const float mu = mean[c], is = invstd[c];
    const rsrc_t rs = make_rsrc(dY, (uint32_t)g.N * g.C * g.H * g.W * (uint32_t)sizeof(T));
    const uint32_t end = min((uint32_t)(s + 1) * q.per_slice, q.per_channel);
    float sdy = 0.f, sdx = 0.f;
    for (uint32_t it = (uint32_t)s * q.per_slice + threadIdx.x; it < end; it += kT) {
        const uint32_t n = udiv(it, q.inv_ipp), rem = it - n * q.ipp;
        const uint32_t i = udiv(rem, q.inv_cpr), ch = rem - i * q.cpr;
        float v[KH][EPC], xh[OPC];
        int rows;
        load_chunk<T, EPC, KH, KW>(g, rs, Zin, n * g.C + c, (int)i, (int)ch, mu, is, v, xh, rows);
        const int left = g.W - (int)ch * EPC; // columns of the chunk inside the row
#pragma unroll
        for (int o = 0; o < OPC; ++o) {
            float t = 0.f; // the tile's dY, row by row (rows past the plane are zeros already)
#pragma unroll
            for (int a = 0; a < KH; ++a)
#pragma unroll
                for (int b = 0; b < KW; ++b)
                    if (o * KW + b < left) t += v[a][o * KW + b];
            sdy += t;
            sdx += t * xh[o];
        }
    }
    sdy = wave_sum(sdy);
    sdx = wave_sum(sdx);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) {
        red[0][wave] = sdy;
        red[1][wave] = sdx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        o_dy[blockIdx.x] = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
        o_dx[blockIdx.x] = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
    }
}

// One wave per channel: its S <= 64 slices, one per lane, added by the wave's fixed tree.
__global__ void __launch_bounds__(64) bn_finish_kernel(int S, const float *__restrict__ p_dy, const float *__restrict__ p_dx,
                                                       float *__restrict__ dgamma, float *__restrict__ dbeta)
{
    const int c = blockIdx.x, lane = threadIdx.x;
    const float a = lane < S ? p_dy[c * S + lane] : 0.f, b = lane < S ? p_dx[c * S + lane] : 0.f;
    const float sa = wave_sum(a), sb = wave_sum(b);
    if (lane == 0) {
        dbeta[c] = sa;
        dgamma[c] = sb;
    }
}

template <typename T, int EPC, int KH, int KW>
__global__ void __launch_bounds__(kT) bn_dx_kernel(Geom g, BnPlan q, const T *__restrict__ Zin, const T *__restrict__ dY,
                                                   const float *__restrict__ mean, const float *__restrict__ invstd,
                                                   const float *__restrict__ gamma, const float *__restrict__ dgamma,
                                                   const float *__restrict__ dbeta, T *__restrict__ dX)
{
    constexpr int OPC = EPC / KW;
    const uint32_t idx = blockIdx.x * (uint32_t)kT + threadIdx.x;
    if (idx >= q.total) return;
    const uint32_t rowi = udiv(idx, q.inv_cpr), ch = idx - rowi * q.cpr;
    const uint32_t plane = udiv(rowi, q.inv_hp), i = rowi - plane * g.Hp;
    const uint32_t c = plane - udiv(plane, q.inv_c) * (uint32_t)g.C;
    const float inv_m = 1.0f / ((float)g.N * (float)(g.H * g.W));
    const float mu = mean[c], is = invstd[c], k = gamma[c] * is;
    const float mdy = dbeta[c] * inv_m, mdx = dgamma[c] * inv_m;
    const rsrc_t rs = make_rsrc(dY, (uint32_t)g.N * g.C * g.H * g.W * (uint32_t)sizeof(T));
    float v[KH][EPC], xh[OPC];
    int rows;
    load_chunk<T, EPC, KH, KW>(g, rs, Zin, plane, (int)i, (int)ch, mu, is, v, xh, rows);
    const int w0 = (int)ch * EPC, left = g.W - w0;
#pragma unroll
    for (int a = 0; a < KH; ++a) {
        if (a >= rows) continue;
        float out[EPC];
#pragma unroll
        for (int b = 0; b < EPC; ++b) out[b] = k * (v[a][b] - mdy - xh[b / KW] * mdx);
        store_chunk<T, EPC>(dX, ((long)plane * g.H + (int)i * KH + a) * g.W + w0, left, out);
    }
}

// ---- rows of 10, 12 or 14 elements (bfloat16, 2 x 2 tiles, an even number of rows): the row-pair
// records of compress.hip's narrow kernel.  Record r = (plane, pooled row) is 4*W contiguous bytes of
// dY and dX and W contiguous bytes of Zin.
template <int W> struct Narrow {
    static constexpr int WP = W / 2, XB = 4 * W, NL = (XB + 15) / 16, NZ = (WP + 7) / 8;
    // the record's dY dwords (row 0: [0, WP), row 1: [WP, 2*WP)) and xh[j] = (Z[j] - mean) * invstd
    static __device__ __forceinline__ void load(rsrc_t rs_dy, rsrc_t rs_z, uint32_t rec, bool live, float mu, float is, uint32_t (&d)[4 * NL],
                                                float (&xh)[8 * NZ])
    {
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, live ? rec * (uint32_t)XB + 16u * k : kNoLoad, 0, 0);
            d[4 * k] = v[0]; d[4 * k + 1] = v[1]; d[4 * k + 2] = v[2]; d[4 * k + 3] = v[3];
        }
#pragma unroll
        for (int k = 0; k < NZ; ++k) {
            float z[8];
            Chunk<bf16_t, 8>::load(rs_z, rec * (uint32_t)WP + 8u * k, live, true, z); // (a pooled row can start on an odd element)
#pragma unroll
            for (int j = 0; j < 8; ++j) xh[8 * k + j] = (z[j] - mu) * is;
        }
    }
};
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

template <int W>
__global__ void __launch_bounds__(kT) bn_partial_narrow_kernel(Geom g, BnPlan q, const bf16_t *__restrict__ Zin, const bf16_t *__restrict__ dY,
                                                               const float *__restrict__ mean, const float *__restrict__ invstd,
                                                               float *__restrict__ o_dy, float *__restrict__ o_dx)
{
    typedef Narrow<W> R;
    __shared__ float red[2][kT / 64];
    const int c = blockIdx.x / q.S, s = blockIdx.x - c * q.S;
    const float mu = mean[c], is = invstd[c];
    const rsrc_t rs = make_rsrc(dY, q.total * (uint32_t)R::XB), rs_z = make_rsrc(Zin, q.total * (uint32_t)(2 * R::WP));
    const uint32_t end = min((uint32_t)(s + 1) * q.per_slice, q.per_channel);
    float sdy = 0.f, sdx = 0.f;
    for (uint32_t it = (uint32_t)s * q.per_slice + threadIdx.x; it < end; it += kT) {
        const uint32_t n = udiv(it, q.inv_hp), i = it - n * g.Hp; // the channel's records: image by image
        uint32_t d[4 * R::NL];
        float xh[8 * R::NZ];
        R::load(rs, rs_z, (n * g.C + c) * g.Hp + i, true, mu, is, d, xh);
#pragma unroll
        for (int j = 0; j < R::WP; ++j) {
            float t = 0.f;
            t += bf_lo(d[j]); t += bf_hi(d[j]); t += bf_lo(d[R::WP + j]); t += bf_hi(d[R::WP + j]);
            sdy += t;
            sdx += t * xh[j];
        }
    }
    sdy = wave_sum(sdy);
    sdx = wave_sum(sdx);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) {
        red[0][wave] = sdy;
        red[1][wave] = sdx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        o_dy[blockIdx.x] = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
        o_dx[blockIdx.x] = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
    }
}

template <int W>
__global__ void __launch_bounds__(kT) bn_dx_narrow_kernel(Geom g, BnPlan q, const bf16_t *__restrict__ Zin, const bf16_t *__restrict__ dY,
                                                          const float *__restrict__ mean, const float *__restrict__ invstd,
                                                          const float *__restrict__ gamma, const float *__restrict__ dgamma,
                                                          const float *__restrict__ dbeta, bf16_t *__restrict__ dX)
{
    typedef Narrow<W> R;
    __shared__ __align__(16) unsigned char lds[4 * 64 * R::XB];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned char *buf = lds + wave * 64 * R::XB;
    const uint32_t rec = blockIdx.x * (uint32_t)kT + threadIdx.x, first = rec - lane;
    const bool live = rec < q.total, whole = first + 64 <= q.total;
    const uint32_t plane = udiv(min(rec, q.total - 1), q.inv_hp);
    const uint32_t c = plane - udiv(plane, q.inv_c) * (uint32_t)g.C;
    const float inv_m = 1.0f / ((float)g.N * (float)(g.H * g.W));
    const float mu = mean[c], is = invstd[c], k = gamma[c] * is;
    const float mdy = dbeta[c] * inv_m, mdx = dgamma[c] * inv_m;
    const rsrc_t rs = make_rsrc(dY, q.total * (uint32_t)R::XB), rs_z = make_rsrc(Zin, q.total * (uint32_t)(2 * R::WP));
    uint32_t d[4 * R::NL];
    float xh[8 * R::NZ];
    R::load(rs, rs_z, rec, live, mu, is, d, xh);
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    uint32_t o[W];
#pragma unroll
    for (int t = 0; t < W; ++t) {
        const float x = xh[t < R::WP ? t : t - R::WP] * mdx;
        o[t] = f32x2_to_bf16x2(k * (bf_lo(d[t]) - mdy - x), k * (bf_hi(d[t]) - mdy - x));
    }
#pragma unroll
    for (int t = 0; t < W / 2; ++t) *(u32x2 *)(buf + lane * R::XB + 8 * t) = u32x2{o[2 * t], o[2 * t + 1]};
    flush_records<R::XB>(buf, (unsigned char *)dX, first, lane, whole, live);
}

// db[o] = sum over n, p, q of dY[n,o,p,q] (bias-gradient formula of the compression figure): a block of
// 1024 threads per output channel streams the channel's N planes (each a contiguous run) in 16-byte
// chunks, two in flight per thread; fixed order, no scratch.
template <typename T, int EPC>
__global__ void __launch_bounds__(1024) db_kernel(int N, int K, int pq, uint32_t cpp, double inv_cpp, const T *__restrict__ dY,
                                                  float *__restrict__ db)
{
    __shared__ float red[16];
    const int o = blockIdx.x;
    const rsrc_t rs = make_rsrc(dY, (uint32_t)N * K * pq * (uint32_t)sizeof(T));
    const uint32_t total = (uint32_t)N * cpp;
    auto chunk = [&](uint32_t it, float (&v)[EPC], int &left) {
        const uint32_t n = udiv(min(it, total - 1), inv_cpp), ch = min(it, total - 1) - n * cpp;
        Chunk<T, EPC>::load(rs, (n * K + o) * pq + ch * EPC, it < total, pq & 1, v);
        left = pq - (int)ch * EPC;
    };
    float acc = 0.f;
    for (uint32_t it = threadIdx.x; it < total; it += 2048) {
        float v0[EPC], v1[EPC];
        int l0, l1;
        chunk(it, v0, l0);
        chunk(it + 1024, v1, l1);
#pragma unroll
        for (int b = 0; b < EPC; ++b) acc += b < l0 ? v0[b] : 0.f;
#pragma unroll
        for (int b = 0; b < EPC; ++b) acc += b < l1 ? v1[b] : 0.f; // (a chunk past the end was not loaded: zeros)
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w];
        db[o] = t;
    }
}

inline unsigned cdiv(long a, long b) { return (unsigned)((a + b - 1) / b); }

template <int EPC> bool make_plan(const Geom &g, BnPlan *q)
{
    q->cpr = (g.W + EPC - 1) / EPC;
    const long ipp = (long)g.Hp * q->cpr, per_channel = (long)g.N * ipp, total = per_channel * g.C;
    if (total >= (1L << 31) || q->cpr >= (1 << 16) || ipp >= (1 << 16) || g.Hp >= (1 << 16) || g.C >= (1 << 16)) return false; // udiv's range
    q->ipp = (uint32_t)ipp;
    q->per_channel = (uint32_t)per_channel;
    q->total = (uint32_t)total;
    int S = (int)std::max(1L, std::min(64L, 2048L / g.C));
    S = (int)std::max(1L, std::min((long)S, (per_channel + kT - 1) / kT)); // no slice without a chunk per thread
    q->per_slice = (uint32_t)((per_channel + S - 1) / S);
    q->S = (int)((per_channel + q->per_slice - 1) / q->per_slice);
    q->inv_cpr = 1.0 / q->cpr;
    q->inv_ipp = 1.0 / (double)ipp;
    q->inv_hp = 1.0 / g.Hp;
    q->inv_c = 1.0 / g.C;
    return true;
}

// false: a pooling tile the chunk kernels do not take
template <typename T, int EPC>
bool launch_t(const Geom &g, const BnPlan &q, const void *Zin, const void *dY, const float *mean, const float *invstd, const float *gamma,
              float *dgamma, float *dbeta, void *dX, float *ws, hipStream_t st)
{
    const bool one = q.S == 1; // a channel is one slice: the first launch writes the sums themselves
    float *o_dy = one ? dbeta : ws, *o_dx = one ? dgamma : ws + (size_t)g.C * q.S;
#define CAC_BN(KH, KW)                                                                                                              \
    {                                                                                                                               \
        hipLaunchKernelGGL((bn_partial_kernel<T, EPC, KH, KW>), dim3((unsigned)(g.C * q.S)), dim3(kT), 0, st, g, q, (const T *)Zin,  \
                           (const T *)dY, mean, invstd, o_dy, o_dx);                                                                \
        if (!one) hipLaunchKernelGGL(bn_finish_kernel, dim3((unsigned)g.C), dim3(64), 0, st, q.S, o_dy, o_dx, dgamma, dbeta);       \
        hipLaunchKernelGGL((bn_dx_kernel<T, EPC, KH, KW>), dim3(cdiv(q.total, kT)), dim3(kT), 0, st, g, q, (const T *)Zin,           \
                           (const T *)dY, mean, invstd, gamma, dgamma, dbeta, (T *)dX);                                             \
        return true;                                                                                                                \
    }
    if (g.kh == 2 && g.kw == 2) CAC_BN(2, 2)
    if (g.kh == 4 && g.kw == 4) CAC_BN(4, 4)
    if (g.kh == 1 && g.kw == 1) CAC_BN(1, 1)
    if (g.kh == 2 && g.kw == 4) CAC_BN(2, 4)
    if (g.kh == 4 && g.kw == 2) CAC_BN(4, 2)
#undef CAC_BN
    return false;
}

// The chunk width for a geometry (0: no chunk kernel) and its plan.
int plan_of(const Geom &g, int dtype, BnPlan *q)
{
    if ((long)g.N * g.C * g.H * g.W * 4 >= (1L << 31)) return 0; // 32-bit buffer offsets
    const bool tile_ok = (g.kh == g.kw && (g.kh == 1 || g.kh == 2 || g.kh == 4)) || (g.kh == 2 && g.kw == 4) || (g.kh == 4 && g.kw == 2);
    if (!tile_ok) return 0;
    const int epc = dtype == CAC_F32 ? 4 : (g.W >= 8 ? 8 : 4);
    if (g.kw > epc) return 0;
    const bool ok = epc == 8 ? make_plan<8>(g, q) : make_plan<4>(g, q);
    return ok ? epc : 0;
}

// Rows of 10, 12 or 14 bfloat16 under 2 x 2 tiles with an even number of rows: the record kernels.
bool narrow_plan(const Geom &g, int dtype, BnPlan *q)
{
    if (dtype != CAC_BF16 || g.kh != 2 || g.kw != 2 || g.H % 2 || !(g.W == 10 || g.W == 12 || g.W == 14)) return false;
    const long per_channel = (long)g.N * g.Hp, total = per_channel * g.C;
    if (total * 4 * g.W >= (1L << 31) || g.Hp >= (1 << 16) || g.C >= (1 << 16)) return false; // 32-bit offsets, udiv's range
    q->cpr = 1;
    q->ipp = (uint32_t)g.Hp;
    q->per_channel = (uint32_t)per_channel;
    q->total = (uint32_t)total;
    int S = (int)std::max(1L, std::min(64L, 2048L / g.C));
    S = (int)std::max(1L, std::min((long)S, (per_channel + kT - 1) / kT));
    q->per_slice = (uint32_t)((per_channel + S - 1) / S);
    q->S = (int)((per_channel + q->per_slice - 1) / q->per_slice);
    q->inv_cpr = 1.0;
    q->inv_ipp = 1.0 / g.Hp;
    q->inv_hp = 1.0 / g.Hp;
    q->inv_c = 1.0 / g.C;
    return true;
}

template <int W>
void launch_narrow(const Geom &g, const BnPlan &q, const void *Zin, const void *dY, const float *mean, const float *invstd, const float *gamma,
                   float *dgamma, float *dbeta, void *dX, float *ws, hipStream_t st)
{
    const bool one = q.S == 1;
    float *o_dy = one ? dbeta : ws, *o_dx = one ? dgamma : ws + (size_t)g.C * q.S;
    hipLaunchKernelGGL((bn_partial_narrow_kernel<W>), dim3((unsigned)(g.C * q.S)), dim3(kT), 0, st, g, q, (const bf16_t *)Zin, (const bf16_t *)dY,
                       mean, invstd, o_dy, o_dx);
    if (!one) hipLaunchKernelGGL(bn_finish_kernel, dim3((unsigned)g.C), dim3(64), 0, st, q.S, o_dy, o_dx, dgamma, dbeta);
    hipLaunchKernelGGL((bn_dx_narrow_kernel<W>), dim3(cdiv(q.total, kT)), dim3(kT), 0, st, g, q, (const bf16_t *)Zin, (const bf16_t *)dY, mean,
                       invstd, gamma, dgamma, dbeta, (bf16_t *)dX);
}

} // namespace

// Bytes of device scratch launch_bn_bwd_fast needs (the slices' partial sums); 0 when a channel is
// one slice or the geometry runs on the plain kernels.
size_t bn_bwd_workspace_bytes(const Geom &g, int dtype)
{
    BnPlan q;
    if (!narrow_plan(g, dtype, &q) && !plan_of(g, dtype, &q)) return 0;
    return q.S == 1 ? 0 : (size_t)2 * g.C * q.S * sizeof(float);
}

// True when the chunk kernels cover the geometry (and have been launched).
bool launch_bn_bwd_fast(const Geom &g, int dtype, const void *Zin, const void *dY, const float *mean, const float *invstd,
                        const float *gamma, float *dgamma, float *dbeta, void *dX, void *ws, hipStream_t st, hipError_t *err)
{
    BnPlan q;
    if (narrow_plan(g, dtype, &q)) {
        if (g.W == 10) launch_narrow<10>(g, q, Zin, dY, mean, invstd, gamma, dgamma, dbeta, dX, (float *)ws, st);
        else if (g.W == 12) launch_narrow<12>(g, q, Zin, dY, mean, invstd, gamma, dgamma, dbeta, dX, (float *)ws, st);
        else launch_narrow<14>(g, q, Zin, dY, mean, invstd, gamma, dgamma, dbeta, dX, (float *)ws, st);
        *err = hipGetLastError();
        return true;
    }
    const int epc = plan_of(g, dtype, &q);
    if (!epc) return false;
    if (dtype == CAC_BF16 && g.kh == 2 && g.kw == 2 && g.H % 2 == 0 && g.W == 28 && (long)g.N * g.C * g.Hp * 4 * g.W < (1L << 31)) {
        // rows of 28: the sums with the chunk kernel (the records' strided cold loads lose there, as
        // in plain compression), the element-wise pass with the row-pair records (its stores gain)
        const bool one = q.S == 1;
        float *o_dy = one ? dbeta : (float *)ws, *o_dx = one ? dgamma : (float *)ws + (size_t)g.C * q.S;
        hipLaunchKernelGGL((bn_partial_kernel<bf16_t, 8, 2, 2>), dim3((unsigned)(g.C * q.S)), dim3(kT), 0, st, g, q, (const bf16_t *)Zin,
                           (const bf16_t *)dY, mean, invstd, o_dy, o_dx);
        if (!one) hipLaunchKernelGGL(bn_finish_kernel, dim3((unsigned)g.C), dim3(64), 0, st, q.S, o_dy, o_dx, dgamma, dbeta);
        BnPlan r = q;
        r.total = (uint32_t)((long)g.N * g.C * g.Hp);
        hipLaunchKernelGGL((bn_dx_narrow_kernel<28>), dim3(cdiv(r.total, kT)), dim3(kT), 0, st, g, r, (const bf16_t *)Zin, (const bf16_t *)dY,
                           mean, invstd, gamma, dgamma, dbeta, (bf16_t *)dX);
        *err = hipGetLastError();
        return true;
    }
    bool ok;
    if (dtype == CAC_F32)
        ok = launch_t<float, 4>(g, q, Zin, dY, mean, invstd, gamma, dgamma, dbeta, dX, (float *)ws, st);
    else if (epc == 8)
        ok = launch_t<bf16_t, 8>(g, q, Zin, dY, mean, invstd, gamma, dgamma, dbeta, dX, (float *)ws, st);
    else
        ok = launch_t<bf16_t, 4>(g, q, Zin, dY, mean, invstd, gamma, dgamma, dbeta, dX, (float *)ws, st);
    if (ok) *err = hipGetLastError();
    return ok;
}

// True when the streaming kernel takes the shape (and has been launched).
bool launch_db_fast(const Geom &g, int dtype, const void *dY, float *db, hipStream_t st, hipError_t *err)
{
    const long pq = (long)g.P * g.Q;
    if ((long)g.N * g.K * pq * 4 >= (1L << 31)) return false; // 32-bit buffer offsets
    const int epc = dtype == CAC_F32 ? 4 : 8;
    const long cpp = (pq + epc - 1) / epc;
    if (cpp >= (1 << 16) || (long)g.N * cpp >= (1L << 31)) return false; // udiv's range
    if (dtype == CAC_F32)
        hipLaunchKernelGGL((db_kernel<float, 4>), dim3((unsigned)g.K), dim3(1024), 0, st, g.N, g.K, (int)pq, (uint32_t)cpp, 1.0 / (double)cpp,
                           (const float *)dY, db);
    else
        hipLaunchKernelGGL((db_kernel<bf16_t, 8>), dim3((unsigned)g.K), dim3(1024), 0, st, g.N, g.K, (int)pq, (uint32_t)cpp, 1.0 / (double)cpp,
                           (const bf16_t *)dY, db);
    *err = hipGetLastError();
    return true;
}

} // namespace cac
