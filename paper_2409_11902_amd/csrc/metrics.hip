// Layer sensitivity metric (equation 1 of the paper's section on layer sensitivity): cosine
// similarity of two weight gradients, cos(a, b) = a.b / (|a| |b|).  Two launches, both with a
// fixed summation order: per-block partial sums of a.b, a.a, b.b in double precision, then one
// block adds the partials in index order.
#include "common.h"

namespace cac {

namespace {

constexpr int kCosBlocks = 512; // upper bound of the first launch's grid (sizes the workspace)

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

__global__ void __launch_bounds__(256) cosine_partial_kernel(const float *__restrict__ a, const float *__restrict__ b, long n,
                                                             double *__restrict__ part)
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    const long stride = (long)gridDim.x * 256;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const double x = a[i], y = b[i];
        ab += x * y;
        aa += x * x;
        bb += y * y;
    }
    __shared__ double red[3][4];
    ab = wave_sum(ab);
    aa = wave_sum(aa);
    bb = wave_sum(bb);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        red[0][wave] = ab;
        red[1][wave] = aa;
        red[2][wave] = bb;
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const double *r = red[threadIdx.x];
        part[blockIdx.x * 3 + threadIdx.x] = ((r[0] + r[1]) + r[2]) + r[3];
    }
}

__global__ void __launch_bounds__(64) cosine_final_kernel(const double *__restrict__ part, int nblocks, float *__restrict__ out)
{
    // every lane adds the partial sums k = lane, lane + 64, ... in that order, then lanes 0..2 add the
    // 64 lane sums of one quantity each, lane by lane: a fixed order, and a chain of loads 64 times shorter
    // than one thread walking all partial sums
    __shared__ double lane_sum[3][64];
    __shared__ double tot[3];
    double s[3] = {0.0, 0.0, 0.0};
    for (int k = threadIdx.x; k < nblocks; k += 64)
#pragma unroll
        for (int q = 0; q < 3; ++q) s[q] += part[k * 3 + q];
#pragma unroll
    for (int q = 0; q < 3; ++q) lane_sum[q][threadIdx.x] = s[q];
    __syncthreads();
    if (threadIdx.x < 3) {
        double t = 0.0;
        for (int l = 0; l < 64; ++l) t += lane_sum[threadIdx.x][l];
        tot[threadIdx.x] = t;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const double ab = tot[0], aa = tot[1], bb = tot[2];
        out[0] = (aa == 0.0 || bb == 0.0) ? 0.f : (float)(ab / (sqrt(aa) * sqrt(bb)));
        out[1] = (float)ab;
        out[2] = (float)aa;
        out[3] = (float)bb;
    }
}

} // namespace

size_t cosine_workspace(long n) { (void)n; return (size_t)kCosBlocks * 3 * sizeof(double); }

hipError_t launch_cosine(const float *a, const float *b, long n, float *out, void *ws, hipStream_t st)
{
    const int nblocks = (int)max(1L, min((long)kCosBlocks, (n + 1023) / 1024));
    hipLaunchKernelGGL(cosine_partial_kernel, dim3(nblocks), dim3(256), 0, st, a, b, n, (double *)ws);
    hipLaunchKernelGGL(cosine_final_kernel, dim3(1), dim3(64), 0, st, (const double *)ws, nblocks, out);
    return hipGetLastError();
}

} // namespace cac
