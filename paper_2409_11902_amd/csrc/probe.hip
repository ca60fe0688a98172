// Yardstick kernels for the benchmark: what this machine attains on a bare matrix-core loop and
// on a bare stream, so that a kernel's rate can be set against the attainable rate as well as
// against the data-sheet peak (the measurement plan asks for both).  gfx950.
//   CAC_PROBE_MFMA : every wave keeps four A and four B fragments read from `src` in registers and
//                    issues `iters` rounds of 16 independent 32x32x16 bfloat16 MFMAs on them (no
//                    LDS, no memory traffic in the loop); 2 * 32*32*16 flops per MFMA.  The rate
//                    depends on the DATA: the chip lowers its clock under sustained matrix load,
//                    and an MFMA on zeros draws less power than one on random numbers.
//   CAC_PROBE_MFMA_16X16 : the same with 16x16x32 MFMAs (32 per round: as many flops).
//   CAC_PROBE_MFMA_1WAVE : the first kind with one wave per SIMD instead of two (1024 waves).
//   CAC_PROBE_COPY : dst = src, 16 bytes per lane, grid-stride.
//   CAC_PROBE_READ : sums src (16-byte loads), one float per workgroup to dst.
#include "common.h"

namespace cac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ void __launch_bounds__(256) probe_mfma_kernel(const u32x4 *__restrict__ src, float *__restrict__ dst, int iters)
{
    union { u32x4 u; bf16x8 v; } a[4], b[4];
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = src[(i * 64 + lane) & 1023];
        b[i].u = src[((i + 4) * 64 + lane) & 1023];
    }
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3].v, b[i >> 2].v, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][lane & 15];
    if (s == 123.456f) dst[0] = s; // (keeps the loop alive; practically never true)
}

__global__ void __launch_bounds__(256) probe_mfma16_kernel(const u32x4 *__restrict__ src, float *__restrict__ dst, int iters)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    union { u32x4 u; bf16x8 v; } a[4], b[4];
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i].u = src[(i * 64 + lane) & 1023];
        b[i].u = src[((i + 4) * 64 + lane) & 1023];
    }
    f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3].v, b[i >> 2].v, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][lane & 3];
    if (s == 123.456f) dst[0] = s; // (keeps the loop alive; practically never true)
}

__global__ void __launch_bounds__(256) probe_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, long n16)
{
    const long stride = (long)gridDim.x * 256;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ void __launch_bounds__(256) probe_read_kernel(const u32x4 *__restrict__ src, float *__restrict__ dst, long n16)
{
    const long stride = (long)gridDim.x * 256;
    uint32_t s = 0;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = src[i];
        s ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (s == 0x12345678u) dst[blockIdx.x] = 1.f; // (keeps the loads alive)
}

} // namespace

hipError_t launch_probe(int kind, const void *src, void *dst, size_t bytes, int iters, hipStream_t st)
{
    if (kind == CAC_PROBE_MFMA) {
        // one wave per SIMD of every compute unit, twice over
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(512), dim3(256), 0, st, (const u32x4 *)src, (float *)dst, iters);
    } else if (kind == CAC_PROBE_MFMA_16X16) {
        hipLaunchKernelGGL(probe_mfma16_kernel, dim3(512), dim3(256), 0, st, (const u32x4 *)src, (float *)dst, iters);
    } else if (kind == CAC_PROBE_MFMA_1WAVE) {
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(256), dim3(256), 0, st, (const u32x4 *)src, (float *)dst, iters);
    } else if (kind == CAC_PROBE_COPY) {
        hipLaunchKernelGGL(probe_copy_kernel, dim3(256 * 8), dim3(256), 0, st, (const u32x4 *)src, (u32x4 *)dst, (long)(bytes / 16));
    } else {
        hipLaunchKernelGGL(probe_read_kernel, dim3(256 * 8), dim3(256), 0, st, (const u32x4 *)src, (float *)dst, (long)(bytes / 16));
    }
    return hipGetLastError();
}

} // namespace cac
