// Sum of the weight gradient's partial sums over the pixel slices (second step of the split
// weight-gradient kernel, see dw_mfma.hip), as a device function so that the launch can be shared
// with other small work of a backward pass.
#pragma once
#include "common.h"

namespace cac {

// What is left to do after the main weight-gradient kernel when its reduction is deferred.
struct DwReduceTail {
    const float *part; // [nslices][total] partial sums
    float *dW;
    long total;        // elements of dW
    int nslices;
    int SY, V;         // thread rows over the slices; floats per vector
    unsigned blocks;   // blocks of 256 threads; 0: nothing to do
};

// Vectors of 4 floats when a slice is a whole number of them (every slice then starts aligned);
// thread rows over the slices when there are many of them.
inline DwReduceTail make_reduce_tail(const float *part, float *dW, long total, int nslices)
{
    DwReduceTail t{part, dW, total, nslices, 1, 1, 0};
    t.V = total % 4 == 0 ? 4 : 1;
    t.SY = nslices >= 32 ? 16 : nslices >= 8 ? 4 : 1;
    t.blocks = (unsigned)((total / t.V + 256 / t.SY - 1) / (256 / t.SY));
    return t;
}

// dW = sum over the slices of their partial sums, in slice order.  A block of 256 threads owns
// 256/SY vectors of V floats; its SY thread rows take every SY-th slice each and are combined
// through LDS in a fixed order, so the result does not depend on scheduling.
template <int SY, int V>
__device__ __forceinline__ void dw_reduce_body(const float *__restrict__ part, float *__restrict__ dW, long total, int nslices,
                                               unsigned block)
{
    typedef float vec __attribute__((ext_vector_type(V)));
    constexpr int CX = 256 / SY;
    __shared__ vec red[SY > 1 ? SY : 1][CX];
    const int cx = threadIdx.x % CX, sy = threadIdx.x / CX;
    const long nvec = total / V, col = (long)block * CX + cx;
    const bool valid = col < nvec;
    const vec *src = (const vec *)part + (valid ? col : 0);
    vec sum = 0.f;
    int sl = sy;
    for (; sl + 3 * SY < nslices; sl += 4 * SY) {
        const vec a = src[(long)sl * nvec], b = src[(long)(sl + SY) * nvec];
        const vec c = src[(long)(sl + 2 * SY) * nvec], d = src[(long)(sl + 3 * SY) * nvec];
        sum += a;
        sum += b;
        sum += c;
        sum += d;
    }
    for (; sl < nslices; sl += SY) sum += src[(long)sl * nvec];
    if (SY > 1) {
        red[sy][cx] = sum;
        __syncthreads();
        if (sy != 0) return;
#pragma unroll
        for (int k = 1; k < SY; ++k) sum += red[k][cx];
    }
    if (valid) ((vec *)dW)[col] = sum;
}

// dw_mfma.hip: the reduction as a launch of its own.
hipError_t launch_dw_reduce(const DwReduceTail &t, hipStream_t st);

} // namespace cac
