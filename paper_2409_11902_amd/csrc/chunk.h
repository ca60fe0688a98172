// What the streaming kernels share (compression, its producer form, batch normalisation's backward
// pass): a thread's "chunk" -- 16 bytes of a row as floats, whatever the row's alignment -- and the
// division by a run-time constant they index with.  Included into an unnamed namespace's worth of
// device code per translation unit (everything here is static or inline).
#pragma once
#include "common.h"

namespace cac {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr uint32_t kNoLoad = 0x80000000u;

// EPC consecutive elements starting at element e (any alignment the type
// allows) as floats; elements past the tensor read as zero.
template <typename T, int EPC> struct Chunk;
template <int EPC> struct Chunk<bf16_t, EPC> {
    static_assert(EPC == 8 || EPC == 4, "");
    // odd: rows can start on odd elements (odd W); only then the extra dword is fetched
    static __device__ __forceinline__ void load(rsrc_t rs, uint32_t e, bool live, bool odd, float (&out)[EPC])
    {
        // dword-aligned address at or below the element; an odd start is shifted out afterwards
        const uint32_t byte = live ? (e & ~1u) * 2u : kNoLoad;
        uint32_t d[EPC / 2 + 1];
        d[EPC / 2] = 0;
        if constexpr (EPC == 8) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, byte, 0, 0);
            d[0] = v[0]; d[1] = v[1]; d[2] = v[2]; d[3] = v[3];
            if (odd) d[4] = __builtin_amdgcn_raw_buffer_load_b32(rs, byte == kNoLoad ? kNoLoad : byte + 16, 0, 0);
        } else {
            typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs, byte, 0, 0);
            d[0] = v[0]; d[1] = v[1];
            if (odd) d[2] = __builtin_amdgcn_raw_buffer_load_b32(rs, byte == kNoLoad ? kNoLoad : byte + 8, 0, 0);
        }
        const uint32_t sh = (e & 1u) * 16u;
#pragma unroll
        for (int j = 0; j < EPC / 2; ++j) {
            const uint32_t w = __builtin_amdgcn_alignbit(d[j + 1], d[j], sh);
            out[2 * j] = __uint_as_float(w << 16);
            out[2 * j + 1] = __uint_as_float(w & 0xffff0000u);
        }
    }
};
template <> struct Chunk<float, 4> {
    static __device__ __forceinline__ void load(rsrc_t rs, uint32_t e, bool live, bool, float (&out)[4])
    {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, live ? e * 4u : kNoLoad, 0, 0);
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = __uint_as_float(v[j]);
    }
};

// floor(x / d) for x < 2^31 and d < 2^16, given inv = 1.0 / d: the quotient's
// fractional part is a multiple of 1/d >= 2^-16, so adding 2^-18 before
// truncating absorbs the rounding of x * inv without ever reaching the next integer.
__device__ __forceinline__ uint32_t udiv(uint32_t x, double inv) { return (uint32_t)((double)x * inv + 0x1p-18); }


// EPC floats of a row to memory in the tensors' type, starting at element e of `base`, of which
// `left` lie inside the row (the others are dropped).  16-byte stores where the whole chunk is
// inside (global stores of several dwords only need dword alignment), dwords and single elements at
// the end of a row; bfloat16 is rounded by the hardware conversion (round to nearest even).
template <typename T, int EPC> __device__ __forceinline__ void store_chunk(T *base, long e, int left, const float (&v)[EPC])
{
    typedef u32x4 __attribute__((aligned(4))) u32x4_u;
    if constexpr (sizeof(T) == 4) {
        static_assert(EPC == 4, "");
        if (left >= EPC) {
            *(u32x4_u *)(base + e) = u32x4{__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        } else {
#pragma unroll
            for (int b = 0; b < EPC; ++b)
                if (b < left) base[e + b] = v[b];
        }
    } else {
        uint32_t o[EPC / 2];
#pragma unroll
        for (int b = 0; b < EPC / 2; ++b) o[b] = f32x2_to_bf16x2(v[2 * b], v[2 * b + 1]);
        if ((e & 1) == 0) {
            if (EPC == 8 && left >= 8) {
                *(u32x4_u *)(base + e) = u32x4{o[0], o[1], o[EPC / 4], o[EPC / 2 - 1]};
            } else {
#pragma unroll
                for (int b = 0; b < EPC / 2; ++b) {
                    if (2 * b + 1 < left)
                        *(uint32_t *)(base + e + 2 * b) = o[b];
                    else if (2 * b < left)
                        base[e + 2 * b] = (bf16_t)(o[b] & 0xffffu);
                }
            }
        } else {
#pragma unroll
            for (int b = 0; b < EPC; ++b)
                if (b < left) base[e + b] = (bf16_t)((b & 1) ? o[b / 2] >> 16 : o[b / 2] & 0xffffu);
        }
    }
}

// A wave's 64 records of BYTES bytes each, written by its lanes to the wave-private LDS region
// `buf` (lane l at l * BYTES), to memory at dst + idx * BYTES: the records of a wave are contiguous
// and start on a multiple of 16 bytes (first = index of lane 0's record, a multiple of 64), so they
// leave as whole 16-byte pieces; the last wave of a tensor, when it is not full (`whole` false),
// stores its live lanes' records two bytes at a time.
template <int BYTES>
__device__ __forceinline__ void flush_records(const unsigned char *buf, unsigned char *dst, uint32_t first, int lane, bool whole, bool live)
{
    static_assert(BYTES % 2 == 0, "");
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (whole) {
        unsigned char *base = dst + (size_t)first * BYTES;
#pragma unroll
        for (int k = 0; k < (4 * BYTES + 63) / 64; ++k) {
            const int piece = lane + 64 * k;
            if (piece < 4 * BYTES) *(u32x4 *)(base + 16 * piece) = *(const u32x4 *)(buf + 16 * piece);
        }
    } else if (live) {
        const uint16_t *src = (const uint16_t *)(buf + lane * BYTES);
        uint16_t *o = (uint16_t *)(dst + (size_t)(first + lane) * BYTES);
#pragma unroll
        for (int k = 0; k < BYTES / 2; ++k) o[k] = src[k];
    }
}

} // namespace
} // namespace cac
