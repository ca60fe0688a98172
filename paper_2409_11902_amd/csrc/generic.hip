// Shape-generic kernels of the step: any filter extent, stride, padding and pooling
// tile, float or bfloat16 storage, float accumulation.  They are the float path
// and the fallback for geometries the MFMA kernels do not cover.  Plain FMA, one
// output (or a small block of outputs) per thread; no tiling through LDS.
#include "common.h"

namespace cac {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// Sum of v over the 256 threads of a block, valid in thread 0.
__device__ __forceinline__ float block_sum(float v, float *lds4)
{
    v = wave_sum(v);
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) lds4[wave] = v;
    __syncthreads();
    return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

// Z[n,c,i,j] = mean (or, for the maximum reading of "other forms of pooling", the largest
// element) over the valid part of tile (i,j) of X[n,c] (compression section).
template <typename T>
__global__ void __launch_bounds__(kThreads) compress_generic(Geom g, const T *__restrict__ X, T *__restrict__ Z)
{
    long total = (long)g.N * g.C * g.Hp * g.Wp;
    long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    int j = (int)(idx % g.Wp);
    long t = idx / g.Wp;
    int i = (int)(t % g.Hp);
    long plane = t / g.Hp;
    const T *x = X + plane * g.H * g.W;
    int h0 = i * g.kh, w0 = j * g.kw;
    int h1 = min(h0 + g.kh, g.H), w1 = min(w0 + g.kw, g.W);
    float sum = 0.f, best = Elem<T>::load(x + h0 * g.W + w0);
    for (int h = h0; h < h1; ++h)
        for (int w = w0; w < w1; ++w) {
            const float v = Elem<T>::load(x + h * g.W + w);
            sum += v;
            best = fmaxf(best, v);
        }
    float cnt = (float)((h1 - h0) * (w1 - w0));
    Elem<T>::store(Z + idx, g.pmax ? best : sum / cnt);
}

// Y = X * W + b (forward formula of the compression figure).
template <typename T, int OT>
__global__ void __launch_bounds__(kThreads)
fwd_generic(Geom g, const T *__restrict__ X, const T *__restrict__ Wt, const T *__restrict__ b, T *__restrict__ Y)
{
    int pix = blockIdx.x * kThreads + threadIdx.x;
    int o0 = blockIdx.y * OT;
    int n = blockIdx.z;
    if (pix >= g.P * g.Q) return;
    int p = pix / g.Q, q = pix - p * g.Q;
    float acc[OT];
#pragma unroll
    for (int j = 0; j < OT; ++j) acc[j] = b ? Elem<T>::load(b + min(o0 + j, g.K - 1)) : 0.f;
    const T *xn = X + (long)n * g.C * g.H * g.W;
    for (int c = 0; c < g.C; ++c) {
        for (int r = 0; r < g.R; ++r) {
            int h = p * g.sh + r - g.ph;
            if (h < 0 || h >= g.H) continue;
            for (int s = 0; s < g.S; ++s) {
                int w = q * g.sw + s - g.pw;
                if (w < 0 || w >= g.W) continue;
                float x = Elem<T>::load(xn + ((long)c * g.H + h) * g.W + w);
#pragma unroll
                for (int j = 0; j < OT; ++j) {
                    int o = min(o0 + j, g.K - 1);
                    acc[j] += x * Elem<T>::load(Wt + (((long)o * g.C + c) * g.R + r) * g.S + s);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < OT; ++j)
        if (o0 + j < g.K) Elem<T>::store(Y + (((long)n * g.K + o0 + j) * g.P + p) * g.Q + q, acc[j]);
}

// dX = W^T * dY, gather form (data-gradient formula of the compression figure).
template <typename T, int CT>
__global__ void __launch_bounds__(kThreads)
dx_generic(Geom g, const T *__restrict__ Wt, const T *__restrict__ dY, T *__restrict__ dX)
{
    int pix = blockIdx.x * kThreads + threadIdx.x;
    int c0 = blockIdx.y * CT;
    int n = blockIdx.z;
    if (pix >= g.H * g.W) return;
    int h = pix / g.W, w = pix - h * g.W;
    float acc[CT];
#pragma unroll
    for (int j = 0; j < CT; ++j) acc[j] = 0.f;
    const T *gn = dY + (long)n * g.K * g.P * g.Q;
    for (int r = 0; r < g.R; ++r) {
        int th = h + g.ph - r;
        if (th < 0 || th % g.sh) continue;
        int p = th / g.sh;
        if (p >= g.P) continue;
        for (int s = 0; s < g.S; ++s) {
            int tw = w + g.pw - s;
            if (tw < 0 || tw % g.sw) continue;
            int q = tw / g.sw;
            if (q >= g.Q) continue;
            for (int o = 0; o < g.K; ++o) {
                float gy = Elem<T>::load(gn + ((long)o * g.P + p) * g.Q + q);
#pragma unroll
                for (int j = 0; j < CT; ++j) {
                    int c = min(c0 + j, g.C - 1);
                    acc[j] += gy * Elem<T>::load(Wt + (((long)o * g.C + c) * g.R + r) * g.S + s);
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < CT; ++j)
        if (c0 + j < g.C) Elem<T>::store(dX + (((long)n * g.C + c0 + j) * g.H + h) * g.W + w, acc[j]);
}

// dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] * Z[n,c,(p*sh+r-ph)/kh,(q*sw+s-pw)/kw]
// (weight-gradient formula of the compression figure, inflation by index only).
// One block owns an OT x CT patch of (o,c) pairs and walks the filter taps; its
// threads stride over the pixels and the sums are reduced in a fixed order.
template <typename T, int OT, int CT>
__global__ void __launch_bounds__(kThreads)
dw_generic(Geom g, const T *__restrict__ Z, const T *__restrict__ dY, float *__restrict__ dW)
{
    __shared__ float red[4];
    int o0 = blockIdx.x * OT, c0 = blockIdx.y * CT;
    long npix = (long)g.N * g.P * g.Q;
    for (int r = 0; r < g.R; ++r) {
        for (int s = 0; s < g.S; ++s) {
            float acc[OT][CT];
#pragma unroll
            for (int a = 0; a < OT; ++a)
#pragma unroll
                for (int e = 0; e < CT; ++e) acc[a][e] = 0.f;
            for (long i = threadIdx.x; i < npix; i += kThreads) {
                int q = (int)(i % g.Q);
                long t = i / g.Q;
                int p = (int)(t % g.P);
                int n = (int)(t / g.P);
                int h = p * g.sh + r - g.ph, w = q * g.sw + s - g.pw;
                if (h < 0 || h >= g.H || w < 0 || w >= g.W) continue;
                int zi = h / g.kh, zj = w / g.kw;
                float gy[OT], xz[CT];
#pragma unroll
                for (int a = 0; a < OT; ++a)
                    gy[a] = Elem<T>::load(dY + (((long)n * g.K + min(o0 + a, g.K - 1)) * g.P + p) * g.Q + q);
#pragma unroll
                for (int e = 0; e < CT; ++e)
                    xz[e] = Elem<T>::load(Z + (((long)n * g.C + min(c0 + e, g.C - 1)) * g.Hp + zi) * g.Wp + zj);
#pragma unroll
                for (int a = 0; a < OT; ++a)
#pragma unroll
                    for (int e = 0; e < CT; ++e) acc[a][e] += gy[a] * xz[e];
            }
#pragma unroll
            for (int a = 0; a < OT; ++a)
#pragma unroll
                for (int e = 0; e < CT; ++e) {
                    float v = block_sum(acc[a][e], red);
                    if (threadIdx.x == 0 && o0 + a < g.K && c0 + e < g.C)
                        dW[(((long)(o0 + a) * g.C + c0 + e) * g.R + r) * g.S + s] = v;
                }
        }
    }
}

// db[o] = sum_{n,p,q} dY[n,o,p,q] (bias-gradient formula of the compression figure).
template <typename T>
__global__ void __launch_bounds__(kThreads) db_generic(Geom g, const T *__restrict__ dY, float *__restrict__ db)
{
    __shared__ float red[4];
    int o = blockIdx.x;
    int pq = g.P * g.Q;
    float acc = 0.f;
    for (int n = 0; n < g.N; ++n) {
        const T *row = dY + ((long)n * g.K + o) * pq;
        for (int i = threadIdx.x; i < pq; i += kThreads) acc += Elem<T>::load(row + i);
    }
    float v = block_sum(acc, red);
    if (threadIdx.x == 0) db[o] = v;
}

inline unsigned cdiv(long a, long b) { return (unsigned)((a + b - 1) / b); }

} // namespace

hipError_t launch_compress_generic(const Geom &g, int dtype, const void *X, void *Z, hipStream_t st)
{
    long total = (long)g.N * g.C * g.Hp * g.Wp;
    dim3 grid(cdiv(total, kThreads));
    if (dtype == CAC_F32)
        hipLaunchKernelGGL(compress_generic<float>, grid, dim3(kThreads), 0, st, g, (const float *)X, (float *)Z);
    else
        hipLaunchKernelGGL(compress_generic<bf16_t>, grid, dim3(kThreads), 0, st, g, (const bf16_t *)X, (bf16_t *)Z);
    return hipGetLastError();
}

hipError_t launch_fwd_generic(const Geom &g, int dtype, const void *X, const void *W, const void *b, void *Y,
                              hipStream_t st)
{
    constexpr int OT = 8;
    dim3 grid(cdiv((long)g.P * g.Q, kThreads), cdiv(g.K, OT), g.N);
    if (dtype == CAC_F32)
        hipLaunchKernelGGL((fwd_generic<float, OT>), grid, dim3(kThreads), 0, st, g, (const float *)X,
                           (const float *)W, (const float *)b, (float *)Y);
    else
        hipLaunchKernelGGL((fwd_generic<bf16_t, OT>), grid, dim3(kThreads), 0, st, g, (const bf16_t *)X,
                           (const bf16_t *)W, (const bf16_t *)b, (bf16_t *)Y);
    return hipGetLastError();
}

hipError_t launch_dx_generic(const Geom &g, int dtype, const void *W, const void *dY, void *dX, hipStream_t st)
{
    constexpr int CT = 8;
    dim3 grid(cdiv((long)g.H * g.W, kThreads), cdiv(g.C, CT), g.N);
    if (dtype == CAC_F32)
        hipLaunchKernelGGL((dx_generic<float, CT>), grid, dim3(kThreads), 0, st, g, (const float *)W,
                           (const float *)dY, (float *)dX);
    else
        hipLaunchKernelGGL((dx_generic<bf16_t, CT>), grid, dim3(kThreads), 0, st, g, (const bf16_t *)W,
                           (const bf16_t *)dY, (bf16_t *)dX);
    return hipGetLastError();
}

hipError_t launch_dw_generic(const Geom &g, int dtype, const void *Z, const void *dY, float *dW, hipStream_t st)
{
    constexpr int OT = 4, CT = 4;
    dim3 grid(cdiv(g.K, OT), cdiv(g.C, CT));
    if (dtype == CAC_F32)
        hipLaunchKernelGGL((dw_generic<float, OT, CT>), grid, dim3(kThreads), 0, st, g, (const float *)Z,
                           (const float *)dY, dW);
    else
        hipLaunchKernelGGL((dw_generic<bf16_t, OT, CT>), grid, dim3(kThreads), 0, st, g, (const bf16_t *)Z,
                           (const bf16_t *)dY, dW);
    return hipGetLastError();
}

hipError_t launch_db(const Geom &g, int dtype, const void *dY, float *db, hipStream_t st)
{
    dim3 grid(g.K);
    if (dtype == CAC_F32)
        hipLaunchKernelGGL(db_generic<float>, grid, dim3(kThreads), 0, st, g, (const float *)dY, db);
    else
        hipLaunchKernelGGL(db_generic<bf16_t>, grid, dim3(kThreads), 0, st, g, (const bf16_t *)dY, db);
    return hipGetLastError();
}

} // namespace cac
