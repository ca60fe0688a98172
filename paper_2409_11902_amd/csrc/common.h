// Shared device/host definitions of the HIP path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cac.h"

namespace cac {

// Geometry handed to every kernel by value.
struct Geom {
    int N, C, K;        // batch, input channels, output channels
    int H, W;           // input extent
    int R, S;           // filter extent
    int sh, sw, ph, pw; // stride, zero padding
    int P, Q;           // output extent
    int kh, kw;         // pooling tile
    int Hp, Wp;         // pooled extent (ceil)
    int pmax;           // non-zero: a tile is reduced to its maximum instead of its mean
    int dw_algo;        // cac_dw_algo: how the weight gradient is evaluated
};

typedef uint16_t bf16_t; // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Two floats to a pair of bfloat16 (lo in bits 15:0) with the hardware conversion
// (v_cvt_pk_bf16_f32: round to nearest even).
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    union { bf16x2_t v; uint32_t u; } r;
    r.v = __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t);
    return r.u;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float *p) { return *p; }
    static __device__ __forceinline__ void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t *p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t *p, float v) { *p = f32_to_bf16(v); }
};

// ---- launchers implemented in the .hip files.  All enqueue on `st` and return the
// launch status; operand shapes have been validated by the caller (api.hip).
// compress.hip: true when the fast kernel covers the geometry and was launched (status in *err)
bool launch_compress_fast(const Geom &g, int dtype, const void *X, void *Z, hipStream_t st, hipError_t *err);
hipError_t launch_compress_generic(const Geom &g, int dtype, const void *X, void *Z, hipStream_t st);
hipError_t launch_fwd_generic(const Geom &g, int dtype, const void *X, const void *W, const void *b, void *Y,
                              hipStream_t st);
hipError_t launch_dx_generic(const Geom &g, int dtype, const void *W, const void *dY, void *dX, hipStream_t st);
hipError_t launch_dw_generic(const Geom &g, int dtype, const void *Z, const void *dY, float *dW, hipStream_t st);
hipError_t launch_db(const Geom &g, int dtype, const void *dY, float *db, hipStream_t st);
// compress.hip / producer.hip: compression at the producer of the activation, and batch
// normalisation's backward pass from its compressed saved input
bool launch_producer_fast(const Geom &g, int dtype, const void *Y, const float *scale, const float *shift, void *Xn, void *Zn, void *Zin,
                          hipStream_t st, hipError_t *err);
hipError_t launch_producer_generic(const Geom &g, int dtype, const void *Y, const float *scale, const float *shift, void *Xn, void *Zn,
                                   void *Zin, hipStream_t st);
bool launch_db_fast(const Geom &g, int dtype, const void *dY, float *db, hipStream_t st, hipError_t *err);
size_t bn_bwd_workspace_bytes(const Geom &g, int dtype);
bool launch_bn_bwd_fast(const Geom &g, int dtype, const void *Zin, const void *dY, const float *mean, const float *invstd,
                        const float *gamma, float *dgamma, float *dbeta, void *dX, void *ws, hipStream_t st, hipError_t *err);
hipError_t launch_bn_bwd(const Geom &g, int dtype, const void *Zin, const void *dY, const float *mean, const float *invstd,
                         const float *gamma, float *dgamma, float *dbeta, void *dX, hipStream_t st);
// Buffer descriptor over a dense tensor of `bytes` bytes (raw, 32-bit elements): loads through
// it return zero for every dword that does not lie entirely below the size, without touching
// memory.  The size is rounded up to whole dwords: a tensor with an odd number of 2-byte
// elements ends in the middle of a dword, which would otherwise read as zero as a whole; the
// two bytes past the tensor share that aligned dword, so they are mapped (and never used).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (bytes + 3u) & ~3u, 0x00020000);
}

// probe.hip: the benchmark's yardstick kernels
hipError_t launch_probe(int kind, const void *src, void *dst, size_t bytes, int iters, hipStream_t st);

size_t cosine_workspace(long n);
hipError_t launch_cosine(const float *a, const float *b, long n, float *out, void *ws, hipStream_t st);

} // namespace cac
