// Compression at the producer of an activation, and batch normalisation's backward pass from
// its compressed saved input (the paper's conclusion names both as the next steps: emitting the
// pooled map where the activation is made, so that it is never read again just to be pooled,
// and compressing what batch normalisation saves).  gfx950, bandwidth-bound kernels.
//
// Forward (one read of Y, the normalisation's input):
//   Xn = relu(scale[c] * Y + shift[c])      the next convolution's input, stored in the tensors' type
//   Zn = pooling of the stored Xn           the next convolution's saved record
//   Zin = pooling of Y                      the normalisation's own saved record (optional)
// (scale = gamma * invstd, shift = beta - mean * scale for batch normalisation in training mode;
// the statistics are the caller's.)  The fast form is compress.hip's kernel with a prologue; the
// kernel here takes every other pooling tile.
//
// Backward of y = gamma * xhat + beta, xhat = (x - mean) * invstd, over M = N*H*W elements per
// channel, with x replaced by the inflated record (x~ = Zin repeated over its tiles):
//   dbeta[c]  = sum dy            dgamma[c] = sum dy * xhat~
//   dx        = gamma * invstd * (dy - dbeta / M - xhat~ * dgamma / M)
// Here: the plain form for pooling tiles the chunk kernels of bn_bwd.hip do not take -- two launches,
// per-channel sums in a fixed order (one block per channel), then the element-wise pass.  The sums
// are exact in the same sense as the weight gradient: only xhat~ is approximate.
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

// One thread per pooled tile: transforms and stores the tile's elements, pools the stored values
// (and, on request, the raw ones) in row-then-column order.
template <typename T>
__global__ void __launch_bounds__(kThreads) producer_generic(Geom g, const T *__restrict__ Y, const float *__restrict__ scale,
                                                             const float *__restrict__ shift, T *__restrict__ Xn, T *__restrict__ Zn,
                                                             T *__restrict__ Zin)
{
    const long total = (long)g.N * g.C * g.Hp * g.Wp;
    const long idx = (long)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx % g.Wp);
    const long t = idx / g.Wp;
    const int i = (int)(t % g.Hp);
    const long plane = t / g.Hp;
    const int c = (int)(plane % g.C);
    const float sc = scale[c], sh = shift[c];
    const T *y = Y + plane * g.H * g.W;
    T *x = Xn + plane * g.H * g.W;
    const int h0 = i * g.kh, w0 = j * g.kw;
    const int h1 = min(h0 + g.kh, g.H), w1 = min(w0 + g.kw, g.W);
    float sum = 0.f, best = 0.f, rsum = 0.f, rbest = 0.f;
    bool first = true;
    for (int h = h0; h < h1; ++h)
        for (int w = w0; w < w1; ++w) {
            const float raw = Elem<T>::load(y + h * g.W + w);
            Elem<T>::store(x + h * g.W + w, fmaxf(fmaf(sc, raw, sh), 0.f));
            const float v = Elem<T>::load(x + h * g.W + w); // the stored (rounded) value
            sum += v;
            rsum += raw;
            best = first ? v : fmaxf(best, v);
            rbest = first ? raw : fmaxf(rbest, raw);
            first = false;
        }
    const float cnt = (float)((h1 - h0) * (w1 - w0));
    Elem<T>::store(Zn + idx, g.pmax ? best : sum / cnt);
    if (Zin) Elem<T>::store(Zin + idx, g.pmax ? rbest : rsum / cnt);
}

// Per-channel sums over n, h, w of dy and dy * xhat~; one block per channel, fixed order.
template <typename T>
__global__ void __launch_bounds__(kThreads) bn_bwd_sums(Geom g, const T *__restrict__ Zin, const T *__restrict__ dY,
                                                        const float *__restrict__ mean, const float *__restrict__ invstd,
                                                        float *__restrict__ dgamma, float *__restrict__ dbeta)
{
    __shared__ float red[2][4];
    const int c = blockIdx.x;
    const float mu = mean[c], is = invstd[c];
    const int hw = g.H * g.W;
    float sdy = 0.f, sdx = 0.f;
    for (int n = 0; n < g.N; ++n) {
        const T *dy = dY + ((long)n * g.C + c) * hw;
        const T *z = Zin + ((long)n * g.C + c) * g.Hp * g.Wp;
        for (int i = threadIdx.x; i < hw; i += kThreads) {
            const int h = i / g.W, w = i - h * g.W;
            const float d = Elem<T>::load(dy + i);
            const float xh = (Elem<T>::load(z + (h / g.kh) * g.Wp + w / g.kw) - mu) * is;
            sdy += d;
            sdx += d * xh;
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
        dbeta[c] = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
        dgamma[c] = ((red[1][0] + red[1][1]) + red[1][2]) + red[1][3];
    }
}

template <typename T>
__global__ void __launch_bounds__(kThreads) bn_bwd_dx(Geom g, const T *__restrict__ Zin, const T *__restrict__ dY,
                                                      const float *__restrict__ mean, const float *__restrict__ invstd,
                                                      const float *__restrict__ gamma, const float *__restrict__ dgamma,
                                                      const float *__restrict__ dbeta, T *__restrict__ dX)
{
    const int hw = g.H * g.W;
    const long plane = blockIdx.y; // (n, c)
    const int c = (int)(plane % g.C);
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= hw) return;
    const float inv_m = 1.0f / ((float)g.N * (float)hw);
    const float mu = mean[c], is = invstd[c], k = gamma[c] * is;
    const float mdy = dbeta[c] * inv_m, mdx = dgamma[c] * inv_m;
    const int h = i / g.W, w = i - h * g.W;
    const float xh = (Elem<T>::load(Zin + plane * g.Hp * g.Wp + (h / g.kh) * g.Wp + w / g.kw) - mu) * is;
    const float d = Elem<T>::load(dY + plane * hw + i);
    Elem<T>::store(dX + plane * hw + i, k * (d - mdy - xh * mdx));
}

inline unsigned cdiv(long a, long b) { return (unsigned)((a + b - 1) / b); }

} // namespace

hipError_t launch_producer_generic(const Geom &g, int dtype, const void *Y, const float *scale, const float *shift, void *Xn, void *Zn,
                                   void *Zin, hipStream_t st)
{
    const long total = (long)g.N * g.C * g.Hp * g.Wp;
    const dim3 grid(cdiv(total, kThreads));
    if (dtype == CAC_F32)
        hipLaunchKernelGGL(producer_generic<float>, grid, dim3(kThreads), 0, st, g, (const float *)Y, scale, shift, (float *)Xn,
                           (float *)Zn, (float *)Zin);
    else
        hipLaunchKernelGGL(producer_generic<bf16_t>, grid, dim3(kThreads), 0, st, g, (const bf16_t *)Y, scale, shift, (bf16_t *)Xn,
                           (bf16_t *)Zn, (bf16_t *)Zin);
    return hipGetLastError();
}

hipError_t launch_bn_bwd(const Geom &g, int dtype, const void *Zin, const void *dY, const float *mean, const float *invstd,
                         const float *gamma, float *dgamma, float *dbeta, void *dX, hipStream_t st)
{
    const dim3 grid2(cdiv((long)g.H * g.W, kThreads), (unsigned)(g.N * g.C));
    if (dtype == CAC_F32) {
        hipLaunchKernelGGL(bn_bwd_sums<float>, dim3(g.C), dim3(kThreads), 0, st, g, (const float *)Zin, (const float *)dY, mean, invstd,
                           dgamma, dbeta);
        hipLaunchKernelGGL(bn_bwd_dx<float>, grid2, dim3(kThreads), 0, st, g, (const float *)Zin, (const float *)dY, mean, invstd, gamma,
                           dgamma, dbeta, (float *)dX);
    } else {
        hipLaunchKernelGGL(bn_bwd_sums<bf16_t>, dim3(g.C), dim3(kThreads), 0, st, g, (const bf16_t *)Zin, (const bf16_t *)dY, mean,
                           invstd, dgamma, dbeta);
        hipLaunchKernelGGL(bn_bwd_dx<bf16_t>, grid2, dim3(kThreads), 0, st, g, (const bf16_t *)Zin, (const bf16_t *)dY, mean, invstd,
                           gamma, dgamma, dbeta, (bf16_t *)dX);
    }
    return hipGetLastError();
}

} // namespace cac
