// Forward convolution and data gradient (forward / data-gradient formulas of the
// compression figure; neither depends on the compressed activation) as one MFMA
// implicit GEMM.
//
// Both are the same "gather" sum
//   out[n, m, h, w] = bias[m] + sum_t sum_kc Wt[t][m][kc] * in[n, i*is + dh_t, j*is + dw_t, kc]
// over a list of taps t, for the output pixels (h, w) = (i*os + a0, j*os + b0):
//   forward:            in = X,  m = o, kc = c, os = 1, is = stride, (dh, dw) = (r - pad, s - pad)
//   data gradient, s=1: in = dY, m = c, kc = o, os = 1, is = 1,      (dh, dw) = (pad - r, pad - s)
//   data gradient, s=2: one launch per output parity class (a0, b0) with the
//                       taps whose (a0 + pad - r) and (b0 + pad - s) are even.
// The reduction index kc must be contiguous per pixel for the MFMA operand
// layout.  In LDS it always is; on the way there the input takes one of two
// routes: a channels-last copy in the workspace (repack_kernel) that the GEMM's
// copy waves move in 16-byte pieces, or -- where that copy would be the larger
// part of the repack launch -- no copy at all: the copy waves read 8 channel x
// 8 pixel blocks of the tensor as it lies and transpose them in registers.  The
// filter is always repacked into MFMA fragment order, padded with zeros to
// multiples of 16 channels (same launch; the forward pass forms the 2 x 2 pooled
// map there too where the tiles are whole).  The GEMM is conv_gather_kernel.
#include <stdio.h>
#include <stdlib.h>

#include <mutex>

#include "common.h"
#include "conv_mfma.h"
#include "dw_reduce.h"

namespace cac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr uint32_t kNoLoad = 0x80000000u;
constexpr int KC = 32;       // channels staged per pass
constexpr int KCS = KC + 8;  // LDS elements per patch pixel: 80 bytes, an odd number of 16-byte units

// ---- repacks ---------------------------------------------------------------------

// Both repacks of a call in one launch.
//
// Input: in [N][C][HW] -> out [N][HW][Cp], zeros for c >= C.
//   HW even (every plane starts at a multiple of 4 bytes): a thread moves an 8 channel x 8 pixel
//   block: eight 16-byte loads along the pixels (consecutive lanes = consecutive pixel groups of
//   a channel row), an 8 x 8 transpose in registers (v_perm), eight 16-byte stores of 8 channels
//   each; the last block of a plane may be partial (it reads on into the next plane, or zeros
//   past the tensor, and stores only its own pixels).
//   Otherwise: 64 x 64 tiles through LDS, element by element.
// Filter: W [O][C][R][S] -> Wt in MFMA fragment order [R*S][KCp/16][Mp/32][lane 64][8]: lane l of
//   a wave holds row m = 32*mblk + l%32 and the 8 channels kc = 16*kblk + 8*(l/32) ..., so a wave
//   reads the A fragment of a (tap, 16-channel block, 32-row block) as one contiguous KiB.
//   Forward: m = o, kc = c; data gradient: m = c, kc = o.
// Blocks [0, in_blocks) do the input, the rest the filter.
struct RepackParams {
    const bf16_t *in;
    bf16_t *out;        // null: no channels-last copy, the input blocks only form Z
    int N, C, HW, Cp, in_blocks, fast;
    int in_wpb;         // waves of an input block that take items (fast path): fewer than 4 spread a small
                        // input over more compute units, one block each
    bf16_t *Z;          // pooled copy of `in` written on the way (2 x 2 means), or null
    int Wimg;           // image width (only with Z)
    int decim;          // with Z: `out` takes pixel (2h, 2w) of every 2 x 2 tile only, as an image of half the extent
    const bf16_t *W;
    bf16_t *Wt;
    int O, Cw, RS, Mp, KCp, transpose;
};

__device__ __forceinline__ void repack_body(const RepackParams &p, const int bid)
{
    constexpr int kFilterElems = 32 * (16 * 9 + 2); // a 32 x 16 block of (o, c) pairs, 9 taps, padded rows
    __shared__ bf16_t sm[kFilterElems > 64 * 66 ? kFilterElems : 64 * 66];
    if (bid >= p.in_blocks) {
        // One block per (32-row block, 16-channel block): its part of W -- for every o a contiguous
        // run of (c, tap) -- goes through LDS as it lies in memory; then every thread gathers the
        // 8 channels of one lane of one tap's fragment and writes them as 16 bytes, a wave one
        // contiguous KiB.  Rows are padded to an odd number of dwords against bank conflicts.
        const int b = bid - p.in_blocks;
        const int mblks = p.Mp / 32, kblks = p.KCp / 16, mblk = b % mblks, kblk = b / mblks;
        const int rows = p.transpose ? 16 : 32, cols = p.transpose ? 32 : 16; // o rows, c columns
        const int o0 = p.transpose ? kblk * 16 : mblk * 32, c0 = p.transpose ? mblk * 32 : kblk * 16;
        const int L = cols * p.RS, Lp = L + 2;
        const int wv = threadIdx.x >> 6, ln = threadIdx.x & 63;
        // a wave takes every fourth row; all of a thread's loads are issued before the first is
        // used (at most 8 rows of 3 x 64 elements, or 4 rows of 5 x 64)
        constexpr int kRowsPerWave = 8, kMaxX = 5;
        const rsrc_t rs = make_rsrc(p.W, (uint32_t)p.O * p.Cw * p.RS * 2u);
        // Whole blocks whose runs are multiples of 16 bytes and start on such (every row of W does
        // when Cw * RS is a multiple of 8): 16-byte loads, at most 3 per thread, instead of up to 40
        // loads of one element each.
        const int segs = L >> 3;
        if ((L & 7) == 0 && ((p.Cw * p.RS) & 7) == 0 && c0 + cols <= p.Cw) {
            u32x4 t4[3];
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int it = threadIdx.x + 256 * q, r = it / segs, sg = it - r * segs, o = o0 + r;
                const bool ok = it < rows * segs && o < p.O;
                t4[q] = __builtin_amdgcn_raw_buffer_load_b128(rs, ok ? ((uint32_t)(o * p.Cw + c0) * p.RS) * 2u + sg * 16u : kNoLoad, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int it = threadIdx.x + 256 * q, r = it / segs, sg = it - r * segs;
                if (it < rows * segs) {
                    uint32_t *d = (uint32_t *)(sm + r * Lp + sg * 8); // (Lp is even: 4-byte aligned)
#pragma unroll
                    for (int k = 0; k < 4; ++k) d[k] = t4[q][k];
                }
            }
        } else {
        uint16_t tmp[kRowsPerWave][kMaxX];
#pragma unroll
        for (int j = 0; j < kRowsPerWave; ++j) {
            const int r = wv + 4 * j, o = o0 + r;
            const int lim = (r < rows && o < p.O) ? min(L, (p.Cw - c0) * p.RS) : 0; // elements of the run inside the tensor
            const uint32_t base = ((uint32_t)(o * p.Cw + c0) * p.RS) * 2u;
#pragma unroll
            for (int k = 0; k < kMaxX; ++k) {
                const int x = ln + 64 * k;
                tmp[j][k] = __builtin_amdgcn_raw_buffer_load_b16(rs, x < lim ? base + 2u * x : kNoLoad, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < kRowsPerWave; ++j) {
            const int r = wv + 4 * j;
#pragma unroll
            for (int k = 0; k < kMaxX; ++k) {
                const int x = ln + 64 * k;
                if (r < rows && x < L) sm[r * Lp + x] = tmp[j][k];
            }
        }
        }
        __syncthreads();
        for (int it = threadIdx.x; it < p.RS * 64; it += 256) {
            const int tap = it >> 6, lane = it & 63, m = lane & 31, k8 = 8 * (lane >> 5);
            u32x4 v;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t h[2];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int kc = k8 + 2 * k + e;
                    h[e] = p.transpose ? sm[kc * Lp + m * p.RS + tap] : sm[m * Lp + kc * p.RS + tap];
                }
                v[k] = h[0] | (h[1] << 16);
            }
            ((u32x4 *)p.Wt)[((long)(tap * kblks + kblk) * mblks + mblk) * 64 + lane] = v;
        }
        return;
    }
    bf16_t (*tile)[66] = (bf16_t (*)[66])sm;
    if (p.fast) {
        // item -> (image n, block of up to 8 channel groups, pixel group pg of 8, channel group
        // within the block), the last fastest: 8 neighbouring lanes read 8 channel rows and
        // write the 128 contiguous bytes of 64 channels of one pixel; the next lanes move along
        // the pixels, so every row is read in 128-byte runs too.  With Z, an item is the same 8
        // pixels of TWO image rows (2h, 2h+1), from which it also forms the 2 x 2 means.
        const bool pool = p.Z != nullptr && p.Wimg != 4;
        const bool pool4 = p.Z != nullptr && p.Wimg == 4; // rows of 4 pixels: an item is already two whole rows
        const int wgs = pool ? p.Wimg / 8 : 1;                 // pixel groups per image row
        const int pgs = pool ? p.HW / 16 : (p.HW + 7) / 8;     // items along the pixels (the last may be partial)
        const int cgs = p.Cp / 8, cgw = min(cgs, 8), cgb = (cgs + cgw - 1) / cgw;
        if ((int)(threadIdx.x >> 6) >= p.in_wpb) return;
        // (fewer than 2^31 items: 32-bit divisions)
        const uint32_t item = ((uint32_t)bid * p.in_wpb + (threadIdx.x >> 6)) * 64u + (threadIdx.x & 63);
        if (item >= (uint32_t)p.N * cgb * pgs * cgw) return;
        const int cl = item % (uint32_t)cgw;
        uint32_t t1 = item / (uint32_t)cgw;
        const int pi = t1 % (uint32_t)pgs;
        t1 /= (uint32_t)pgs;
        const int cg = (int)(t1 % (uint32_t)cgb) * cgw + cl, n = t1 / (uint32_t)cgb;
        if (cg >= cgs) return;
        // first pixel of the item's (first) row segment
        const int hh = pool ? pi / wgs : 0, wg = pool ? pi - hh * wgs : 0;
        const int px0 = pool ? (2 * hh * wgs + wg) * 8 : pi * 8;
        const rsrc_t rs = make_rsrc(p.in, (uint32_t)p.N * p.C * p.HW * 2u);
        u32x4 r[2][8];
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            if (a == 1 && !pool) break;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = cg * 8 + i;
                const uint32_t e = ((uint32_t)(n * p.C + c) * p.HW + px0 + a * p.Wimg) * 2u;
                r[a][i] = __builtin_amdgcn_raw_buffer_load_b128(rs, c < p.C ? e : kNoLoad, 0, 0);
            }
        }
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            if (a == 1 && !pool) break;
            if (!p.out) break; // only the pooled map is wanted
            if (p.decim && a == 1) break; // (odd rows are not kept)
            bf16_t *dst = p.decim ? p.out + ((long)n * (p.HW / 4) + hh * (p.Wimg / 2) + wg * 4) * p.Cp + cg * 8
                                  : p.out + ((long)n * p.HW + px0 + a * p.Wimg) * p.Cp + cg * 8;
#pragma unroll
            for (int px = 0; px < 8; ++px) {
                // pixel px of the 8 channels: half px%2 of dword px/2 of every row
                u32x4 v;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t lo = r[a][2 * k][px / 2], hi = r[a][2 * k + 1][px / 2];
                    v[k] = (px & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                }
                if (p.decim) {
                    if (!(px & 1)) *(u32x4 *)(dst + (long)(px / 2) * p.Cp) = v;
                } else if (px0 + px < p.HW) {
                    *(u32x4 *)(dst + (long)px * p.Cp) = v; // (a plane's last item may reach past it)
                }
            }
        }
        if (pool4) {
            // Z[n][c][pi][0..1] from pixels (0, 1, 4, 5) and (2, 3, 6, 7) of the item, summed row by
            // row like the stand-alone kernel does
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = cg * 8 + i;
                if (c >= p.C) break;
                uint32_t h2[2];
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const uint32_t t0 = r[0][i][jj], t1r = r[0][i][2 + jj];
                    float sum = 0.f;
                    sum += __uint_as_float(t0 << 16);
                    sum += __uint_as_float(t0 & 0xffff0000u);
                    sum += __uint_as_float(t1r << 16);
                    sum += __uint_as_float(t1r & 0xffff0000u);
                    h2[jj] = f32_to_bf16(sum * 0.25f);
                }
                *(uint32_t *)(p.Z + (((long)n * p.C + c) * (p.HW / 8) + pi) * 2) = h2[0] | (h2[1] << 16);
            }
        }
        if (pool) {
            // Z[n][c][hh][4*wg .. +3]: the same sum order and rounding as the stand-alone kernel
            const int Hp = p.HW / p.Wimg / 2, Wp = p.Wimg / 2;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int c = cg * 8 + i;
                if (c >= p.C) break;
                uint32_t o[2];
#pragma unroll
                for (int j2 = 0; j2 < 2; ++j2) {
                    uint32_t h2[2];
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        const uint32_t t0 = r[0][i][2 * j2 + jj], t1r = r[1][i][2 * j2 + jj];
                        float sum = 0.f;
                        sum += __uint_as_float(t0 << 16);
                        sum += __uint_as_float(t0 & 0xffff0000u);
                        sum += __uint_as_float(t1r << 16);
                        sum += __uint_as_float(t1r & 0xffff0000u);
                        h2[jj] = f32_to_bf16(sum * 0.25f);
                    }
                    o[j2] = h2[0] | (h2[1] << 16);
                }
                typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                *(u32x2 *)(p.Z + (((long)n * p.C + c) * Hp + hh) * Wp + wg * 4) = u32x2{o[0], o[1]};
            }
        }
        return;
    }
    // block -> (image, 64-channel block, 64-pixel block)
    const int pbs = (p.HW + 63) / 64, cbs = (p.Cp + 63) / 64;
    const int pb = bid % pbs, t1 = bid / pbs;
    const int cb = t1 % cbs, n = t1 / cbs;
    const int c0 = cb * 64, p0 = pb * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int k = ty; k < 64; k += 4) {
        const int c = c0 + k, px = p0 + tx;
        tile[k][tx] = (c < p.C && px < p.HW) ? p.in[((long)n * p.C + c) * p.HW + px] : (bf16_t)0;
    }
    __syncthreads();
    for (int k = ty; k < 64; k += 4) {
        const int px = p0 + k, c = c0 + tx;
        if (px < p.HW && c < p.Cp) p.out[((long)n * p.HW + px) * p.Cp + c] = tile[tx][k];
    }
}

__global__ void __launch_bounds__(256) repack_kernel(RepackParams p) { repack_body(p, blockIdx.x); }

// The repacks of a data-gradient call and, in the blocks after them, the slice sum that the
// weight gradient of the same layer has left over: two small, independent pieces of a backward
// pass that would otherwise each pay for a launch.
template <int SY, int V>
__global__ void __launch_bounds__(256) repack_reduce_kernel(RepackParams p, unsigned nrep, DwReduceTail t)
{
    if (blockIdx.x < nrep)
        repack_body(p, blockIdx.x);
    else
        dw_reduce_body<SY, V>(t.part, t.dW, t.total, t.nslices, blockIdx.x - nrep);
}

// Launches the input and filter repacks of one call.
// Z, Wimg: see RepackParams (Z null: no pooling; else HW must be a multiple of 2*Wimg and Wimg 4 or a multiple of 8).
// tail: a deferred weight-gradient slice sum to run in the same launch, or null.
hipError_t launch_repack(const bf16_t *in, bf16_t *out, int N, int C, int HW, int Cp, const bf16_t *W, bf16_t *Wt, int O,
                         int Cw, int RS, int Mp, int KCp, int transpose, bf16_t *Z, int Wimg, hipStream_t st,
                         const DwReduceTail *tail = nullptr, int decim = 0)
{
    RepackParams p{};
    p.in = in; p.out = out; p.N = N; p.C = C; p.HW = HW; p.Cp = Cp;
    p.Z = Z; p.Wimg = Wimg; p.decim = decim;
    p.fast = HW % 2 == 0; // planes start at multiples of 4 bytes: 16-byte loads need no more
    if (!in) N = 0;       // filter only
    const int cgs = Cp / 8, cgw = cgs < 8 ? cgs : 8;
    const long items = p.fast ? (long)N * ((cgs + cgw - 1) / cgw) * cgw * (Z && Wimg != 4 ? HW / 16 : (HW + 7) / 8) : 0;
    // (a thread's loads are all in flight at once, so a small input is bound by latency, not by
    // the number of waves per compute unit: give every unit a wave before any gets a second)
    p.in_wpb = items > 64 * 256 ? 4 : 1; // (measured: two waves per block are slower than either)
    p.in_blocks = p.fast ? (int)((items + 64 * p.in_wpb - 1) / (64 * p.in_wpb)) : N * ((Cp + 63) / 64) * ((HW + 63) / 64);
    p.W = W; p.Wt = Wt; p.O = O; p.Cw = Cw; p.RS = RS; p.Mp = Mp; p.KCp = KCp; p.transpose = transpose;
    const unsigned nrep = (unsigned)(p.in_blocks + (Mp / 32) * (KCp / 16));
    if (tail && tail->blocks) {
        const DwReduceTail &t = *tail;
#define CAC_RR(SY, V) hipLaunchKernelGGL((repack_reduce_kernel<SY, V>), dim3(nrep + t.blocks), dim3(256), 0, st, p, nrep, t)
        if (t.V == 4) {
            if (t.SY == 16) CAC_RR(16, 4);
            else if (t.SY == 4) CAC_RR(4, 4);
            else CAC_RR(1, 4);
        } else {
            if (t.SY == 16) CAC_RR(16, 1);
            else if (t.SY == 4) CAC_RR(4, 1);
            else CAC_RR(1, 1);
        }
#undef CAC_RR
        return hipGetLastError();
    }
    hipLaunchKernelGGL(repack_kernel, dim3(nrep), dim3(256), 0, st, p);
    return hipGetLastError();
}

// Clears n bfloat16 elements: whole 16-byte units, then the (up to 7) elements that remain --
// not a byte past the tensor.
__global__ void __launch_bounds__(256) zero_fill_kernel(bf16_t *dst, long n)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x, n16 = n / 8;
    if (i < n16) ((u32x4 *)dst)[i] = u32x4{0, 0, 0, 0};
    if (i < n - n16 * 8) dst[n16 * 8 + i] = (bf16_t)0;
}

// ---- the gather GEMM ----------------------------------------------------------------
//
// Workgroup: 4 MFMA waves (WM x WN, a wave owns 64 (m) x 32*NI (pixels)) and 4 copy waves.
// A pixel tile is PT = WN*NI*32 pixels of one image, or IPT whole images when an image has at
// most PT/2 pixels.  The work of a workgroup is a run of "units" (the same tile position in
// consecutive image groups), each unit kbs "stages" of KC input channels (all nkb channel blocks,
// or this workgroup's share of them when several workgroups -- grid z -- share a tile: then the
// epilogue writes float sums for gather_finish_kernel); the stages of the whole run form one
// software pipeline: the copy waves keep two stages of global loads in flight and write the patch
// of stage s+1 into the LDS buffer the MFMA waves are not reading (one barrier per stage).
// Filter fragments come straight from global memory (fragment order, cache resident), fetched
// ahead by the MFMA waves themselves -- six steps with nine taps, eight where taps x channel groups of
// a pass is 4 or 8 (NTT), else two -- whose only
// other memory traffic is LDS reads, so their load counter never waits on the long-latency
// patch loads.
constexpr int kMaxItems = 12; // 16-byte patch items a copy thread moves per stage, at most (kernel parameter ITEMS: 6 or 12)
// floor(x / d) for small x (x * d < 2^32) with magic = ceil(2^32 / d), 0 standing for d = 1
__device__ __forceinline__ uint32_t fdiv(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }
constexpr uint32_t kNoElem = 0x40000000u;

// TR: the accumulators hold the transposed tile (lanes = output channels, registers = pixels):
// a lane then owns runs of 4 consecutive pixels.  Used when consecutive pixels of the launch are
// consecutive and 8-byte aligned in memory; the runs leave as 8-byte stores, or, with
// p.wide_store, through LDS as 16-byte stores that cover whole rows.
// NTT: taps x 32-channel groups of a pass when that is 9 (nine taps, one group), 8 or 4: the operand
// rings described at their declaration; 0: any number of taps, one group, a shallow prefetch.
template <int NI, int WM, int WN, bool TR, int NTT, int ITEMS, bool NCHW>
__global__ void __launch_bounds__(512) conv_gather_kernel(GatherParams p)
{
    constexpr int MI = 2;
    constexpr int PT = WN * NI * 32; // pixel lanes per workgroup
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr bool DEEP = NTT != 0;
    // several groups per pass only in the kernels made for it (constants everywhere else)
    const int t_log2 = (NTT == 4 || NTT == 8) ? p.t_log2 : 0, kcs = (NTT == 4 || NTT == 8) ? p.kcs : KCS;
    const int KCT = KC << t_log2;                   // channels staged per pass
    const uint32_t buf_bytes = (uint32_t)p.patch_px * kcs * 2;

    const int wave_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tau = blockIdx.x % p.tiles_per_img, run = blockIdx.x / p.tiles_per_img;
    const int g_begin = run * p.gpw, g_end = min(g_begin + p.gpw, p.ngrp);
    const int kb0 = blockIdx.z * p.kbs;             // this workgroup's share of the channel blocks
    const int nstages = (g_end - g_begin) * p.kbs;
    const int ppi = p.Hc * p.Wc;
    const int pix0 = p.IPT > 1 ? 0 : tau * PT;      // first class-grid pixel of the tile
    const int i0 = fdiv(pix0, p.m_wc);               // its row
    // input patch: rows i0*is + dhmin ..., all columns dwmin ... (Wc-1)*is + dwmax
    const int hin0 = i0 * p.is + p.dhmin, win0 = p.dwmin;

    if (wave_id >= 4) {
        // =========================== copy waves ===========================================
        const int tid = threadIdx.x - 256;
        if constexpr (NCHW) {
            // The input in its own layout [N][Cin][Hin][Win] (Win even): an item is 8 channels x 8
            // pixels of one patch row, as in the repack kernel: eight 16-byte loads along the
            // row (4-byte aligned at least), an 8 x 8 transpose in registers, eight 16-byte
            // LDS writes of one pixel's 8 channels each.  Items exist for the image's own
            // columns only; what lies outside the image is zero in both buffers from the start
            // and is never written.  ITEMS here: items per thread (1 or 2).
            const int GX = (p.Win + 7) >> 3;           // 8-pixel groups of an image row
            const int nitems = (p.IPT * p.PH * GX * (KC / 8)) << t_log2;
            uint32_t e0[ITEMS], l0[ITEMS], m8[ITEMS], gq[ITEMS];
            const int co = tid & ((4 << t_log2) - 1);  // channel octet of the stage (256 is a multiple of their number)
#pragma unroll
            for (int q = 0; q < ITEMS; ++q) {
                const int it = tid + 256 * q;
                const int rest = it >> (2 + t_log2);
                const int rows = fdiv(rest, p.m_gx), gx = rest - rows * GX; // (g, pr) as one index
                const int g = fdiv(rows, p.m_ph), pr = rows - g * p.PH;
                const int hin = hin0 + pr, w0 = gx * 8;
                const bool ok = it < nitems && hin >= 0 && hin < p.Hin;
                uint32_t m = 0;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int w = w0 + k;               // written: inside the image and inside the patch
                    if (ok && w < p.Win && w >= win0 && w < win0 + p.PWd) m |= 1u << k;
                }
                m8[q] = m;
                gq[q] = g;
                e0[q] = ok ? (uint32_t)((g * p.KCin + co * 8) * p.Hin + hin) * p.Win + w0 : kNoElem;
                l0[q] = (uint32_t)(((g * p.PH + pr) * p.PWd + (w0 - win0)) * kcs + co * 8) * 2u; // (used under the mask only)
            }
            const rsrc_t rs_in = make_rsrc(p.in, (uint32_t)p.N * p.KCin * p.Hin * p.Win * 2u);
            const uint32_t plane = (uint32_t)p.Hin * p.Win;
            auto fetch = [&](int s, u32x4 (&r)[ITEMS][8]) {
                const int u = fdiv(s, p.m_kbs), kb = kb0 + s - u * p.kbs;
                const int n_base = (g_begin + u) * p.IPT;
                const uint32_t sbase = (uint32_t)(n_base * p.KCin + kb * KCT) * plane;
                const int c_first = kb * KCT + co * 8;   // the item's first channel
                const uint32_t lim = s < nstages ? (uint32_t)max(p.N - n_base, 0) : 0u;
#pragma unroll
                for (int q = 0; q < ITEMS; ++q)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const uint32_t e = (gq[q] < lim && c_first + i < p.KCin) ? e0[q] + sbase + i * plane : kNoElem;
                        r[q][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, e * 2u, 0, 0);
                    }
            };
            auto put = [&](uint32_t buf, const u32x4 (&r)[ITEMS][8]) {
#pragma unroll
                for (int q = 0; q < ITEMS; ++q)
#pragma unroll
                    for (int px = 0; px < 8; ++px) {
                        u32x4 v; // pixel px of the 8 channels: half px%2 of dword px/2 of every row
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const uint32_t lo = r[q][2 * k][px / 2], hi = r[q][2 * k + 1][px / 2];
                            v[k] = (px & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                        }
                        if (m8[q] & (1u << px)) *(u32x4 *)(smem + buf + l0[q] + px * (kcs * 2)) = v;
                    }
            };
            u32x4 ra[ITEMS][8], rb[ITEMS][8];
            fetch(0, ra);
            fetch(1, rb);
            for (uint32_t i = tid; i < 2 * buf_bytes / 16; i += 256) ((u32x4 *)smem)[i] = u32x4{0, 0, 0, 0};
            __syncthreads(); // (the zeros of one thread lie where another writes pixels)
            put(0, ra);
            __syncthreads();
            for (int s = 0; s < nstages; s += 2) {
                fetch(s + 2, ra);
                put(buf_bytes, rb);
                __syncthreads();
                if (s + 1 >= nstages) break;
                fetch(s + 3, rb);
                put(0, ra);
                __syncthreads();
            }
            return;
        }
        const int items = (p.patch_px * (KC / 8)) << t_log2;
        const int v8 = (tid & ((4 << t_log2) - 1)) * 8; // channel offset of this lane's items in the stage
        uint32_t eq[ITEMS], gq[ITEMS], lq[ITEMS];
#pragma unroll
        for (int q = 0; q < ITEMS; ++q) {
            const int it = tid + 256 * q;
            const int pp = it >> (2 + t_log2);
            const int g = fdiv(pp, p.m_img), rem = pp - g * (p.PH * p.PWd);
            const int pr = fdiv(rem, p.m_pwd), pc = rem - pr * p.PWd;
            const int hin = hin0 + pr, win = win0 + pc;
            const bool ok = it < items && hin >= 0 && hin < p.Hin && win >= 0 && win < p.Win;
            eq[q] = ok ? (uint32_t)((g * p.Hin + hin) * p.Win + win) * p.KCp + v8 : kNoElem;
            gq[q] = g;
            lq[q] = it < items ? (uint32_t)(pp * kcs + v8) * 2u : 0xffffffffu;
        }
        const rsrc_t rs_in = make_rsrc(p.in, (uint32_t)p.N * p.Hin * p.Win * p.KCp * 2u);
        // global -> registers for stage s (dead stages load nothing but are issued all the same:
        // the number of loads in flight is then the same on every path)
        auto fetch = [&](int s, u32x4 (&r)[ITEMS]) {
            const int u = fdiv(s, p.m_kbs), kb = kb0 + s - u * p.kbs;
            const int n_base = (g_begin + u) * p.IPT;
            const uint32_t sbase = (uint32_t)n_base * p.Hin * p.Win * p.KCp + kb * KCT;
            const bool lane_ok = s < nstages && kb * KCT + v8 < p.KCp;
            const uint32_t lim = lane_ok ? (uint32_t)max(p.N - n_base, 0) : 0u;
#pragma unroll
            for (int q = 0; q < ITEMS; ++q) {
                const uint32_t e = gq[q] < lim ? eq[q] + sbase : kNoElem;
                r[q] = __builtin_amdgcn_raw_buffer_load_b128(rs_in, e * 2u, 0, 0);
            }
        };
        auto put = [&](uint32_t buf, const u32x4 (&r)[ITEMS]) {
#pragma unroll
            for (int q = 0; q < ITEMS; ++q)
                if (lq[q] != 0xffffffffu) *(u32x4 *)(smem + buf + lq[q]) = r[q];
        };
        u32x4 ra[ITEMS], rb[ITEMS];
        fetch(0, ra);
        fetch(1, rb);
        put(0, ra);
        __syncthreads();
        for (int s = 0; s < nstages; s += 2) {
            // (a stage past the end is written all the same -- zeros into a buffer nobody reads
            // any more -- so that every path consumes every load)
            fetch(s + 2, ra);
            put(buf_bytes, rb);
            __syncthreads();
            if (s + 1 >= nstages) break;
            fetch(s + 3, rb);
            put(0, ra);
            __syncthreads();
        }
        return;
    }

    // =============================== MFMA waves ===========================================
    const int tid = threadIdx.x, lane = tid & 63, wave = wave_id;
    const int wm = wave % WM, wn = wave / WM, half = lane >> 5, l32 = lane & 31;
    const int m0 = (blockIdx.y * WM + wm) * 64;    // this wave's first output channel
    const bool wave_live = m0 < p.Mp;              // waves past the (padded) output channels only keep the barriers

    // this lane's pixels: image within the tile, class-grid coordinates, LDS byte offset of their
    // tap-(dhmin,dwmin) input pixel
    uint32_t pbase[NI];
    int pi[NI], pj[NI], pg[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int idx = (wn * NI + ni) * 32 + l32;
        int g = 0, px = pix0 + idx;
        bool ok = px < ppi;
        if (p.IPT > 1) {
            g = fdiv(idx, p.m_ppi);
            px = idx - g * ppi;
            ok = g < p.IPT;
        }
        const int i = fdiv(px, p.m_wc), j = px - i * p.Wc;
        pi[ni] = ok ? i : -1;
        pj[ni] = j;
        pg[ni] = g;
        pbase[ni] = ok ? (uint32_t)(((g * p.PH + (i - i0) * p.is) * p.PWd + j * p.is) * kcs * 2) : 0u;
    }

    f32x16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[mi][ni][j] = 0.f;

    const rsrc_t rs_w = make_rsrc(p.wt, (uint32_t)p.ntaps_total * p.Mp * p.KCp * 2u);
    const uint32_t kblks = p.KCp / 16, mblks = p.Mp / 32;
    // Per-tap constants in vector registers (uniform values; with constant indices after
    // unrolling they never have to be reloaded inside the loop): byte offset of the tap's
    // filter fragments and LDS byte offset of the tap within the patch (with this half-wave's
    // 8 channels).
    constexpr uint32_t kFrag = 64 * 16; // bytes of one fragment of the repacked filter
    // With T groups of 32 channels per pass, entry tt stands for (tap tt / T, group tt % T): the
    // loops below run over these "taps" and do not know the difference.
    uint32_t wofs[9], toff[9];
    const int ksteps = (KC / 16) << t_log2;         // 16-channel steps of a pass per tap
#pragma unroll
    for (int tt = 0; tt < 9; ++tt) {
        const int t = tt >> t_log2, tb = tt & ((1 << t_log2) - 1);
        wofs[tt] = ((uint32_t)p.wtap[t] * kblks + tb * (KC / 16)) * mblks * kFrag;
        toff[tt] = (uint32_t)(((p.dh[t] - p.dhmin) * p.PWd + (p.dw[t] - p.dwmin)) * kcs + tb * KC + 8 * half) * 2u;
    }
    // this lane's part of a fragment address; a dead wave reads nothing
    const uint32_t wlane = wave_live ? (uint32_t)(m0 >> 5) * kFrag + lane * 16u : kNoLoad;
    // filter fragment of (tap offset wo, 16-channel block kblk) for output channel block mi
    auto wfrag = [&](uint32_t wo, int kblk, int mi) {
        return __builtin_amdgcn_raw_buffer_load_b128(rs_w, wlane + wo + (uint32_t)(kblk * mblks + mi) * kFrag, 0, 0);
    };
    // Fragments are fetched two steps ahead: a tap is KC/16 = 2 steps, so while step (t, kk) runs,
    // the fragment of (t+1, kk) -- or of the next stage's first tap -- is requested.  The pixel
    // operands (LDS) are requested one step ahead.
    static_assert(KC / 16 == 2, "the prefetch distance below is one tap");
    u32x4 wcur[MI], wnxt[MI], wnn[MI];
    // DEEP (NTT = 9, 8 or 4 "taps" a pass): a ring of D steps of fragments instead, enough to cover a miss
    // in the vector cache at full MFMA rate.  A stage is 2 * NTT steps, a multiple of D, so that step q of
    // every stage uses ring slot q % D and, once the steps are unrolled, every slot is a fixed
    // register.  The uniform part of a fragment's address goes into the load's scalar offset.
    constexpr int NTTS = DEEP ? NTT : 9;            // (the ring code is compiled, never run, in the kernels without it)
    constexpr int D = NTTS == 9 ? (NI >= 4 ? 3 : 6) : 8, STEPS = NTTS * (KC / 16); // (a step of NI = 4 is twice as long)
    static_assert(STEPS % D == 0, "ring slots must not move from stage to stage");
    u32x4 wr[DEEP ? D : 1][MI];
    uint32_t wl[9];
    if constexpr (DEEP) {
#pragma unroll
        for (int t = 0; t < 9; ++t) wl[t] = wlane + wofs[t];
#pragma unroll
        for (int q = 0; q < D; ++q)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                wr[q][mi] = __builtin_amdgcn_raw_buffer_load_b128(
                    rs_w, wl[q >> 1], (uint32_t)((kb0 * ksteps + (q & 1)) * mblks + mi) * kFrag, 0);
    } else {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            wcur[mi] = wfrag(wofs[0], kb0 * ksteps, mi);
            wnxt[mi] = wfrag(wofs[0], kb0 * ksteps + 1, mi);
        }
    }

    // TR epilogues: a lane's output channels are fixed, so their bias is fetched here, once, and
    // not in the epilogue, where the load's latency would lie bare
    float bias_tr[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + mi * 32 + l32;
        bias_tr[mi] = (TR && p.bias && m < p.M) ? bf16_to_f32(p.bias[m]) : 0.f;
    }

    if constexpr (NCHW) __syncthreads(); // the copy waves have zeroed both buffers
    __syncthreads(); // buffer 0 holds stage 0
    int kb = 0, unit = 0;
    for (int s = 0; s < nstages; ++s) {
        if (wave_live) {
            const uint32_t buf = (s & 1) ? buf_bytes : 0u;
            const int kb_next = kb + 1 == p.kbs ? 0 : kb + 1;
            u32x4 bcur[NI], bnxt[NI];
            if constexpr (!DEEP) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) bcur[ni] = *(const u32x4 *)(smem + buf + pbase[ni] + toff[0]);
            }
            if constexpr (DEEP) {
                const uint32_t so_cur = (uint32_t)((kb0 + kb) * ksteps * mblks) * kFrag;
                const uint32_t so_nxt = (uint32_t)((kb0 + kb_next) * ksteps * mblks) * kFrag;
                // pixel operands: a ring of DB steps in registers of their own (a copy from a
                // "next" to a "current" set lets the compiler merge the two and issue the LDS read
                // only after the current value's last use, a fraction of a step ahead)
                constexpr int DB = (NI >= 4 || NTTS != 9) ? 2 : 3;
                static_assert(STEPS % DB == 0, "ring slots must not move from stage to stage");
                u32x4 bq[DB][NI];
                auto pixels = [&](int q, int ni) { return *(const u32x4 *)(smem + buf + pbase[ni] + toff[q >> 1] + 32 * (q & 1)); };
#pragma unroll
                for (int q = 0; q < DB - 1; ++q)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) bq[q][ni] = pixels(q, ni);
#pragma unroll
                for (int q = 0; q < STEPS; ++q) {
                    // pixels of step q + DB - 1 (nothing past the stage's last step: the other
                    // buffer is not ready yet)
                    if (q + DB - 1 < STEPS) {
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) bq[(q + DB - 1) % DB][ni] = pixels(q + DB - 1, ni);
                    }
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi) {
                            union { u32x4 u; bf16x8 v; } af, bf;
                            af.u = wr[q % D][mi];
                            bf.u = bq[q % DB][ni];
                            acc[mi][ni] = TR ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf.v, af.v, acc[mi][ni], 0, 0, 0)
                                             : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bf.v, acc[mi][ni], 0, 0, 0);
                        }
                    // refill the slot with the fragments of step q + D (of this stage or the next;
                    // after the last stage: of the first again, never used)
                    const int q2 = q + D < STEPS ? q + D : q + D - STEPS;
                    const uint32_t so = (q + D < STEPS ? so_cur : so_nxt) + (uint32_t)((q2 & 1) * mblks) * kFrag;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
                        wr[q % D][mi] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, wl[q2 >> 1], so + mi * kFrag, 0);
                    // Pin the order LDS reads, MFMAs, refill, and keep the instruction scheduler from
                    // moving anything to another step (it would sink the loads towards their uses).
                    // one LDS read or one filter load after each MFMA, in its shadow
                    if (q + DB - 1 < STEPS) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, NI - 1, 0);
                    } else {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - 3, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, MI - 1, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                if (t >= p.ntaps) break;
                const bool last = t + 1 >= p.ntaps;
                const uint32_t wo_n = last ? wofs[0] : wofs[t + 1 < 9 ? t + 1 : 0];
                const uint32_t to_n = toff[t + 1 < 9 ? t + 1 : 0];
                const int kblk_n = (kb0 + (last ? kb_next : kb)) * ksteps;
#pragma unroll
                for (int kk = 0; kk < KC / 16; ++kk) {
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) wnn[mi] = wfrag(wo_n, kblk_n + kk, mi);
                    // next step's pixels: the second channel half of this tap, or the next tap
                    // (nothing after the stage's last step: the other buffer is not ready yet)
                    if (kk == 0) {
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) bnxt[ni] = *(const u32x4 *)(smem + buf + pbase[ni] + toff[t] + 32);
                    } else if (!last) {
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) bnxt[ni] = *(const u32x4 *)(smem + buf + pbase[ni] + to_n);
                    }
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi) {
                            union { u32x4 u; bf16x8 v; } af, bf;
                            af.u = wcur[mi];
                            bf.u = bcur[ni];
                            acc[mi][ni] = TR ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf.v, af.v, acc[mi][ni], 0, 0, 0)
                                             : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bf.v, acc[mi][ni], 0, 0, 0);
                        }
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) {
                        wcur[mi] = wnxt[mi];
                        wnxt[mi] = wnn[mi];
                    }
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) bcur[ni] = bnxt[ni];
                }
            }
            if (kb == p.kbs - 1) {
                // ---- epilogue of the unit: bias, bfloat16, NCHW
                const int n_base = (g_begin + unit) * p.IPT;
                if (TR && p.wide_store) {
                    // Through LDS (a region of the wave's own, past the staging buffers), so that
                    // the lanes of a store cover whole rows: the wave's 64 channels x NI*32 pixels
                    // as [channel][pixel] bfloat16, rows padded by 16 bytes; then 8 pixels (16 bytes)
                    // per lane, NI*4 neighbouring lanes one channel's run.
                    // Two pixel blocks (64 pixels) per pass, so that the region stays at 9 KB per wave.
                    constexpr int NIB = NI < 2 ? NI : 2, ROWB = NIB * 64 + 16, LPR = NIB * 4;
                    unsigned char *ep = smem + 2 * buf_bytes + wave * (64 * ROWB);
                    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
#pragma unroll
                    for (int pass = 0; pass < NI / NIB; ++pass) {
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi) {
                            const float bias = bias_tr[mi];
#pragma unroll
                            for (int nb = 0; nb < NIB; ++nb)
#pragma unroll
                                for (int jq = 0; jq < 4; ++jq) {
                                    const f32x16 &a = acc[mi][pass * NIB + nb];
                                    *(u32x2 *)(ep + (mi * 32 + l32) * ROWB + (nb * 32 + 8 * jq + 4 * half) * 2) =
                                        u32x2{f32x2_to_bf16x2(a[4 * jq] + bias, a[4 * jq + 1] + bias), f32x2_to_bf16x2(a[4 * jq + 2] + bias, a[4 * jq + 3] + bias)};
                                }
                        }
                        // (the wave reads what it wrote itself: LDS serves a wave's requests in order)
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        const int seg = lane % LPR, idx = (wn * NI + pass * NIB) * 32 + seg * 8; // pixel of the tile
                        int g = 0, px = pix0 + idx;
                        if (p.IPT > 1) {
                            g = fdiv(idx, p.m_ppi);
                            px = idx - g * ppi;
                        }
                        const int n = n_base + g;
                        const bool px_ok = px < ppi && g < p.IPT && n < p.N;
#pragma unroll
                        for (int it = 0; it < LPR; ++it) {
                            const int row = it * (64 / LPR) + lane / LPR, m = m0 + row;
                            const u32x4 v = *(const u32x4 *)(ep + row * ROWB + seg * 16);
                            if (px_ok && m < p.M) *(u32x4 *)(p.out + ((long)n * p.M + m) * ppi + px) = v;
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                    }
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int j = 0; j < 16; ++j) acc[mi][ni][j] = 0.f;
                } else if constexpr (TR) {
                    // register j of lane l: pixel 8*(j/4) + 4*(l/32) + j%4 of the block, channel l%32
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) {
                        const int m = m0 + mi * 32 + l32;
                        const float bias = bias_tr[mi];
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int jq = 0; jq < 4; ++jq) {
                                // the 4 pixels idx .. idx+3 of the tile (same image: an image's pixel
                                // count is a multiple of 4 on this path)
                                const int idx = (wn * NI + ni) * 32 + 8 * jq + 4 * half;
                                int g = 0, px = pix0 + idx;
                                if (p.IPT > 1) {
                                    g = fdiv(idx, p.m_ppi);
                                    px = idx - g * ppi;
                                }
                                const int n = n_base + g;
                                if (m < p.M && px < ppi && g < p.IPT && n < p.N) {
                                    const f32x16 &a = acc[mi][ni];
                                    if (p.part) { // a share of the channels: float sums, finished by gather_finish_kernel
                                        typedef __attribute__((ext_vector_type(4))) float f32x4;
                                        *(f32x4 *)(p.part + (((long)blockIdx.z * p.N + n) * p.M + m) * ppi + px) =
                                            f32x4{a[4 * jq], a[4 * jq + 1], a[4 * jq + 2], a[4 * jq + 3]};
                                        continue;
                                    }
                                    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
                                    const u32x2 v = {f32x2_to_bf16x2(a[4 * jq] + bias, a[4 * jq + 1] + bias), f32x2_to_bf16x2(a[4 * jq + 2] + bias, a[4 * jq + 3] + bias)};
                                    *(u32x2 *)(p.out + ((long)n * p.M + m) * ppi + px) = v;
                                }
                            }
                    }
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int j = 0; j < 16; ++j) acc[mi][ni][j] = 0.f;
                } else {
                    // register j of lane l: channel 8*(j/4) + 4*(l/32) + j%4, pixel l%32 of the block
                    // Stores through a buffer descriptor over the whole output (less than 2^31 bytes on this
                    // path): 32-bit offsets, split into the pixel's part (per block) and the channel's, and
                    // an offset past the tensor instead of a branch for lanes that own no output.
                    const rsrc_t rs_out = make_rsrc(p.out, (uint32_t)p.N * p.M * p.Hout * p.Wout * 2u);
                    const uint32_t plane_out = (uint32_t)p.Hout * p.Wout;
                    uint32_t obase[NI];
                    bool oky[NI];
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) {
                        const int n = n_base + pg[ni];
                        const int h = pi[ni] * p.os + p.a0, w = pj[ni] * p.os + p.b0;
                        oky[ni] = pi[ni] >= 0 && n < p.N;
                        obase[ni] = oky[ni] ? ((uint32_t)n * p.M * plane_out + h * p.Wout + w) * 2u : 0u;
                    }
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const int m = m0 + mi * 32 + 8 * (j / 4) + 4 * half + (j % 4);
                            const float bias = (p.bias && m < p.M) ? bf16_to_f32(p.bias[m]) : 0.f;
                            const uint32_t moff = (uint32_t)min(m, p.M) * plane_out * 2u;
#pragma unroll
                            for (int ni = 0; ni < NI; ++ni) {
                                const uint32_t off = (m < p.M && oky[ni]) ? obase[ni] + moff : kNoLoad;
                                __builtin_amdgcn_raw_buffer_store_b16(f32_to_bf16(acc[mi][ni][j] + bias), rs_out, off, 0, 0);
                                acc[mi][ni][j] = 0.f;
                            }
                        }
                }
            }
        }
        if (++kb == p.kbs) {
            kb = 0;
            ++unit;
        }
        __syncthreads();
    }
}

// out = bfloat16(bias + sum over the channel shares of their float sums), 4 pixels per thread.
__global__ void __launch_bounds__(256) gather_finish_kernel(const float *__restrict__ part, const bf16_t *__restrict__ bias,
                                                            bf16_t *__restrict__ out, long quads, int nsplit, int ppi, int M)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    const long q = (long)blockIdx.x * 256 + threadIdx.x;
    if (q >= quads) return;
    const f32x4 *src = (const f32x4 *)part + q;
    f32x4 sum = src[0];
    for (int k = 1; k < nsplit; ++k) sum += src[k * quads];
    if (bias) sum += bf16_to_f32(bias[((uint32_t)q * 4u / (uint32_t)ppi) % (uint32_t)M]); // (fewer than 2^30 quads)
    const u32x2 v = {f32x2_to_bf16x2(sum[0], sum[1]), f32x2_to_bf16x2(sum[2], sum[3])};
    *((u32x2 *)out + q) = v;
}

template <int NI, int WM, int WN, bool TR, int NTT, int ITEMS, bool NCHW> hipError_t launch_gather_items(const GatherParams &p, hipStream_t st)
{
    auto kern = conv_gather_kernel<NI, WM, WN, TR, NTT, ITEMS, NCHW>;
    // (per instantiation; once per process, whichever host thread comes first)
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] { attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); });
    if (attr_err != hipSuccess) return attr_err;
    const int runs = (p.ngrp + p.gpw - 1) / p.gpw;
    dim3 grid(p.tiles_per_img * runs, (p.Mp / 64 + WM - 1) / WM, p.ksplit);
    const size_t lds = (size_t)2 * p.patch_px * p.kcs * 2 + (p.wide_store ? 4 * 64 * ((NI < 2 ? NI : 2) * 64 + 16) : 0);
    hipLaunchKernelGGL(kern, grid, dim3(512), lds, st, p);
    if (p.ksplit > 1) {
        const long quads = (long)p.N * p.M * p.Hc * p.Wc / 4;
        hipLaunchKernelGGL(gather_finish_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, (const float *)p.part,
                           p.bias, p.out, quads, p.ksplit, p.Hc * p.Wc, p.M);
    }
    return hipGetLastError();
}

// (small patches: half the items, half the loads per stage and a shorter start-up)
template <int NI, int WM, int WN, bool TR, int NTT> hipError_t launch_gather_shape(const GatherParams &p, hipStream_t st)
{
    if (p.nchw) // items of 8 x 8 elements, one or two per copy thread
        return p.IPT * p.PH * ((p.Win + 7) / 8) * (KC / 8) * p.T <= 256 ? launch_gather_items<NI, WM, WN, TR, NTT, 1, true>(p, st)
                                                                         : launch_gather_items<NI, WM, WN, TR, NTT, 2, true>(p, st);
    return p.patch_px * (KC / 8) * p.T <= 256 * 6 ? launch_gather_items<NI, WM, WN, TR, NTT, 6, false>(p, st)
                                                  : launch_gather_items<NI, WM, WN, TR, NTT, kMaxItems, false>(p, st);
}

template <int NI, int WM, int WN> hipError_t launch_gather(const GatherParams &p, hipStream_t st)
{
    // runs of 4 pixels are contiguous and 8-byte aligned: the class grid is the whole output
    // plane and a plane is a multiple of 4 pixels
    const bool packed = p.os == 1 && p.Hc == p.Hout && p.Wc == p.Wout && (p.Hc * p.Wc) % 4 == 0;
    // (the planner gives T > 1 only where taps x T is 4 or 8)
    const int ntt = p.ntaps * p.T;
    if (ntt == 9 && p.T == 1) return packed ? launch_gather_shape<NI, WM, WN, true, 9>(p, st) : launch_gather_shape<NI, WM, WN, false, 9>(p, st);
    if (ntt == 8) return packed ? launch_gather_shape<NI, WM, WN, true, 8>(p, st) : launch_gather_shape<NI, WM, WN, false, 8>(p, st);
    if (ntt == 4) return packed ? launch_gather_shape<NI, WM, WN, true, 4>(p, st) : launch_gather_shape<NI, WM, WN, false, 4>(p, st);
    if (p.T != 1) return hipErrorInvalidValue; // (never planned)
    return packed ? launch_gather_shape<NI, WM, WN, true, 0>(p, st) : launch_gather_shape<NI, WM, WN, false, 0>(p, st);
}

int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Chooses the workgroup shape and fills the tiling; false if no shape fits.
//
// Candidates: waves along m (wm) x pixel blocks per wave (ni), and, where the output is written
// in whole planes, the number of workgroups that share a tile's channel blocks (their float sums
// go to the workspace and gather_finish_kernel adds them up).  Each is priced with a rough model
// in clock cycles: a step (one tap, 16 channels) costs a wave 32 cycles per MFMA but at least the
// time the CU's vector cache needs for the four waves' filter fragments; a workgroup pays a fixed
// start-up and epilogue; the chip runs 256 workgroups at a time; all filter and input bytes have
// to come through L2; shared-out channels cost a second kernel and the traffic of the sums.
bool shape_gather(GatherParams &p, int *variant)
{
    p.dhmin = p.dwmin = 1 << 30;
    int dhmax = -(1 << 30), dwmax = -(1 << 30);
    for (int t = 0; t < p.ntaps; ++t) {
        p.dhmin = min(p.dhmin, p.dh[t]); dhmax = max(dhmax, p.dh[t]);
        p.dwmin = min(p.dwmin, p.dw[t]); dwmax = max(dwmax, p.dw[t]);
    }
    p.PWd = (p.Wc - 1) * p.is + (dwmax - p.dwmin) + 1;
    p.nkb = (p.KCp + KC - 1) / KC;
    p.part = nullptr;
    const int ppi = p.Hc * p.Wc;
    auto magic = [](uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); };
    p.m_wc = magic(p.Wc); p.m_ppi = magic(ppi); p.m_pwd = magic(p.PWd);
    const bool whole_planes = p.os == 1 && p.Hc == p.Hout && p.Wc == p.Wout && ppi % 4 == 0;
    const char *force = nullptr;
    int f_wm = 0, f_ni = 0, f_ks = 0;
#ifdef CAC_TUNING // development builds: CAC_GATHER_SHAPE="wm,ni,ksplit" overrides the model
    force = getenv("CAC_GATHER_SHAPE");
    if (force) sscanf(force, "%d,%d,%d", &f_wm, &f_ni, &f_ks);
#endif
    GatherParams best{};
    double best_cost = 1e300;
    int best_variant = 0;
    for (int wm : {4, 2, 1}) {
        if (wm * 64 > p.Mp && wm > 1) continue;
        const int wn = 4 / wm;
        for (int ni : {2, 1}) { // (NI = 4 fits the register file only with spills and measured slower)
            GatherParams q = p;
            const int pt = wn * ni * 32;
            q.IPT = 2 * ppi <= pt ? pt / ppi : 1;
            if (q.IPT > 1) {
                q.tiles_per_img = 1;
                q.PH = (q.Hc - 1) * q.is + (dhmax - q.dhmin) + 1;
            } else {
                q.tiles_per_img = (ppi + pt - 1) / pt;
                const int rows = min(q.Hc, (pt + q.Wc - 2) / q.Wc + 1); // class-grid rows a tile can touch
                q.PH = (rows - 1) * q.is + (dhmax - q.dhmin) + 1;
            }
            q.patch_px = q.IPT * q.PH * q.PWd;
            if (q.patch_px * (KC / 8) > 256 * kMaxItems) continue;
            if ((long)2 * q.patch_px * KCS * 2 > 110 * 1024) continue; // (leaves room for the epilogue's transpose)
            // Few taps: several 32-channel groups per pass, which the kernel treats as further taps,
            // so that taps x groups is 4 or 8 and the kernels with the deep operand rings apply
            // (with one or two taps a pass is otherwise a handful of MFMAs, and the filter
            // fragments, requested two steps ahead, arrive long after they are wanted).  As many
            // groups as the channels, LDS and the copy threads' registers allow -- and, where the
            // input could be read in place with one group, only as many as still allow that.
            q.T = 1;
            const int items_in_place = q.IPT * q.PH * ((q.Win + 7) / 8) * (KC / 8);
            for (int t : {4, 2}) {
                if ((q.ntaps * t != 8 && q.ntaps * t != 4) || KC * (t - 1) >= q.KCp) continue;
                if (q.patch_px * (KC / 8) * t > 256 * kMaxItems) continue;
                if ((long)2 * q.patch_px * (KC * t + 8) * 2 > 124 * 1024) continue; // (with the wide stores' 36 KB still inside the CU's 160 KB)
                if (items_in_place <= 512 && items_in_place * t > 512) continue;
                q.T = t;
                break;
            }
            q.t_log2 = q.T == 4 ? 2 : q.T == 2 ? 1 : 0;
            q.kcs = KC * q.T + 8;
            q.nkb = (q.KCp + KC * q.T - 1) / (KC * q.T);
            q.m_img = magic(q.PH * q.PWd);
            q.m_gx = magic((q.Win + 7) / 8); q.m_ph = magic(q.PH);
            q.ngrp = (q.N + q.IPT - 1) / q.IPT;
            const int mtiles = (q.Mp / 64 + wm - 1) / wm;
            const long wgs1 = (long)q.tiles_per_img * q.ngrp * mtiles;
            for (int ks = 1; ks <= (whole_planes ? q.nkb : 1); ++ks) {
                if (q.nkb % ks) continue;
                if (force && (wm != f_wm || ni != f_ni || ks != f_ks)) continue;
                q.ksplit = ks;
                q.wide_store = whole_planes && ks == 1 && ppi % 8 == 0; // 16-byte runs of pixels, aligned
                q.kbs = q.nkb / ks;
                q.m_kbs = magic(q.kbs);
                // a few units per workgroup (a longer pipeline) as long as every CU still gets a workgroup
                q.gpw = (int)max(1L, min((long)((8 + q.kbs - 1) / q.kbs), wgs1 * ks / 256));
                const long runs = (q.ngrp + q.gpw - 1) / q.gpw;
                const long wgs = (long)q.tiles_per_img * runs * mtiles * ks;
                // cycles per step as measured (vector-cache bound below NI = 4), two-step prefetch 1.35 x
                // (without the deep rings a step waits for its filter fragments: measured 700-1000 cycles;
                // with them on few taps, where every fragment is used once, 500-600)
                const int ntt = q.ntaps * q.T;
                const double step = ntt == 9 ? (ni == 1 ? 150.0 : 235.0) : (ntt == 4 || ntt == 8) ? (ni == 1 ? 500.0 : 600.0) : 800.0;
                const double t_wg = (double)q.gpw * q.kbs * 2 * q.ntaps * q.T * step + 8000.0;
                const double l2_bytes = (double)wgs * q.gpw * q.kbs * KC * q.T * 2.0 * (q.ntaps * 64.0 * wm + q.patch_px);
                double cost = max((double)((wgs + 255) / 256) * t_wg, l2_bytes / 6000.0 + 8000.0);
                cost += l2_bytes / 6000.0 * 0.01; // between equals, the one that moves less
                if (ks > 1) cost += 6000.0 + (double)ks * q.N * q.M * ppi * 8.0 / 2500.0;
                if (cost < best_cost) {
                    best_cost = cost;
                    best = q;
                    best_variant = (ni == 2 ? 0 : 3) + (wm == 1 ? 0 : wm == 2 ? 1 : 2);
                }
            }
        }
    }
    if (best_cost > 1e299) return false;
    p = best;
    *variant = best_variant;
    return true;
}

hipError_t run_gather(const GatherParams &p, int variant, hipStream_t st)
{
    switch (variant) {
    case 0: return launch_gather<2, 1, 4>(p, st);
    case 1: return launch_gather<2, 2, 2>(p, st);
    case 2: return launch_gather<2, 4, 1>(p, st);
    case 3: return launch_gather<1, 1, 4>(p, st);
    case 4: return launch_gather<1, 2, 2>(p, st);
    default: return launch_gather<1, 4, 1>(p, st);
    }
}

bool supported(const Geom &g, int dtype)
{
    if (dtype != CAC_BF16) return false;
    if (g.R * g.S > 9) return false;
    if (g.sh != g.sw || (g.sh != 1 && g.sh != 2)) return false;
    // 32-bit byte offsets with 2^31 reserved for "no load"
    const long lim = 1L << 30;
    if ((long)g.N * g.H * g.W * round_up(g.C, 16) >= lim || (long)g.N * g.P * g.Q * round_up(g.K, 16) >= lim) return false;
    if ((long)g.R * g.S * round_up(g.K, 64) * round_up(g.C, 64) >= lim) return false;
    return true;
}

// Forward pass as a gather GEMM: output channels x output pixels, taps (r - ph, s - pw).
bool plan_fwd(const Geom &g, int dtype, GatherParams &p, int *variant)
{
    if (!supported(g, dtype)) return false;
    p = GatherParams{};
    p.N = g.N; p.M = g.K; p.Mp = round_up(g.K, 64); p.KCp = round_up(g.C, 16);
    p.Hin = g.H; p.Win = g.W; p.Hout = g.P; p.Wout = g.Q; p.Hc = g.P; p.Wc = g.Q;
    p.os = 1; p.a0 = p.b0 = 0; p.is = g.sh;
    p.ntaps = p.ntaps_total = g.R * g.S;
    for (int r = 0; r < g.R; ++r)
        for (int s = 0; s < g.S; ++s) {
            const int t = r * g.S + s;
            p.dh[t] = r - g.ph; p.dw[t] = s - g.pw; p.wtap[t] = t;
        }
    // A 1 x 1 filter with stride 2 reaches one pixel of every 2 x 2 tile.  Where the repack launch goes
    // over those tiles anyway (it forms the 2 x 2 pooled map: rows a multiple of 8 pixels, an even
    // number of them), its channels-last copy keeps just that pixel: a quarter of the bytes to write
    // and to stage, and the GEMM sees a stride-1 layer on an image of half the extent.
    p.decim = g.R == 1 && g.S == 1 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 && g.kh == 2 && g.kw == 2 &&
              !g.pmax && g.H % 2 == 0 && g.W % 8 == 0;
    if (p.decim) {
        p.Hin = g.H / 2; p.Win = g.W / 2; p.is = 1;
    }
    return shape_gather(p, variant);
}

// Data gradient: one gather GEMM (input channels x input pixels) per parity class of the input
// pixel, each with the taps that reach that class.  Every class is planned before anything is
// launched.  *empty_class: some class has no tap at all (stride > filter) and stays zero.
bool plan_dx(const Geom &g, int dtype, GatherParams &base, GatherParams (&cls)[4], int (&variant)[4], int *ncls, bool *empty_class)
{
    if (!supported(g, dtype)) return false;
    base = GatherParams{};
    base.N = g.N; base.M = g.C; base.Mp = round_up(g.C, 64); base.KCp = round_up(g.K, 16);
    base.Hin = g.P; base.Win = g.Q; base.Hout = g.H; base.Wout = g.W;
    base.os = g.sh; base.is = 1; base.ntaps_total = g.R * g.S;
    *ncls = 0;
    *empty_class = false;
    for (int a0 = 0; a0 < g.sh; ++a0)
        for (int b0 = 0; b0 < g.sw; ++b0) {
            GatherParams p = base;
            p.a0 = a0; p.b0 = b0;
            p.Hc = (g.H - a0 + g.sh - 1) / g.sh;
            p.Wc = (g.W - b0 + g.sw - 1) / g.sw;
            if (p.Hc <= 0 || p.Wc <= 0) continue;
            p.ntaps = 0;
            for (int r = 0; r < g.R; ++r)
                for (int s = 0; s < g.S; ++s) {
                    const int th = a0 + g.ph - r, tw = b0 + g.pw - s;
                    if (th % g.sh || tw % g.sw) continue; // C++ remainder: zero iff divisible, also for negatives
                    p.dh[p.ntaps] = th / g.sh; p.dw[p.ntaps] = tw / g.sw; p.wtap[p.ntaps] = r * g.S + s;
                    ++p.ntaps;
                }
            if (p.ntaps == 0) { *empty_class = true; continue; }
            if (!shape_gather(p, &variant[*ncls])) return false;
            cls[(*ncls)++] = p;
        }
    return true;
}

// The data gradient reads dY where it lies when every class's patch splits into at most 512
// items of 8 x 8 elements (rows of an even number of pixels): no channels-last copy, only the
// filter repack.  It pays where the copy is the larger part of the repack launch (measured:
// 3.8 us gained per call at 230 input elements per filter element, 1.5 us lost at 3.5).
bool dx_reads_in_place(const Geom &g, const GatherParams (&cls)[4], int ncls)
{
    bool direct = g.Q % 2 == 0 && (long)g.N * g.K * g.P * g.Q >= 8L * g.R * g.S * g.K * g.C;
    for (int k = 0; k < ncls; ++k) direct = direct && cls[k].IPT * cls[k].PH * ((g.Q + 7) / 8) * (KC / 8) * cls[k].T <= 512;
    return direct;
}

int describe_one(const GatherParams &p, int variant, char *buf, size_t len)
{
    static const int shape[6][3] = {{2, 1, 4}, {2, 2, 2}, {2, 4, 1}, {1, 1, 4}, {1, 2, 2}, {1, 4, 1}}; // NI, WM, WN
    const int *v = shape[variant];
    const int runs = (p.ngrp + p.gpw - 1) / p.gpw, mt = (p.Mp / 64 + v[1] - 1) / v[1];
    return snprintf(buf, len, "gather tile=%dch x %dpx (NI=%d WM=%d WN=%d) taps=%d ch/pass=%d img/tile=%d patch=%dx%d units/wg=%d grid=%dx%dx%d lds=%dB",
                    64 * v[1], 32 * v[0] * v[2], v[0], v[1], v[2], p.ntaps, KC * p.T, p.IPT, p.PH, p.PWd, p.gpw, p.tiles_per_img * runs, mt,
                    p.ksplit, 2 * p.patch_px * p.kcs * 2 + (p.wide_store ? 4 * 64 * ((v[0] < 2 ? v[0] : 2) * 64 + 16) : 0));
}

// Workspace: [channels-last input][repacked filter][float sums of shared-out channels], each
// part starting at a multiple of 256 bytes.
struct WsLayout { size_t in, wt, part; };
WsLayout ws_layout(size_t in_elems, size_t wt_elems, const GatherParams &p)
{
    auto up = [](size_t n) { return (n + 255) / 256 * 256; };
    WsLayout l;
    l.in = up(in_elems * 2);
    l.wt = up(wt_elems * 2);
    l.part = p.ksplit > 1 ? (size_t)p.ksplit * p.N * p.M * p.Hc * p.Wc * sizeof(float) : 0;
    return l;
}

} // namespace

bool describe_conv_mfma(const Geom &g, int dtype, bool data_grad, char *buf, size_t len)
{
    GatherParams p{}, cls[4];
    int variant[4], ncls = 0;
    bool empty = false;
    if (!data_grad) {
        if (!plan_fwd(g, dtype, p, &variant[0])) return false;
        const int n = describe_one(p, variant[0], buf, len);
        if (p.decim && n > 0 && (size_t)n + 1 < len) snprintf(buf + n, len - n, "; the copy of the input keeps one pixel of every 2 x 2 tile");
        return true;
    }
    if (!plan_dx(g, dtype, p, cls, variant, &ncls, &empty)) return false;
    size_t at = 0;
    for (int k = 0; k < ncls && at + 1 < len; ++k) {
        int n = snprintf(buf + at, len - at, "%sclass(%d,%d): ", k ? "; " : "", cls[k].a0, cls[k].b0);
        at += (size_t)max(n, 0);
        if (at + 1 >= len) break;
        n = describe_one(cls[k], variant[k], buf + at, len - at);
        at += (size_t)max(n, 0);
    }
    if (at + 1 < len && dx_reads_in_place(g, cls, ncls)) snprintf(buf + at, len - at, "; dY read in place");
    return true;
}

size_t conv_mfma_workspace(const Geom &g, int dtype, bool data_grad)
{
    GatherParams p{}, cls[4];
    int variant[4], ncls = 0;
    bool empty = false;
    const size_t RS = (size_t)g.R * g.S;
    if (!data_grad) {
        if (!plan_fwd(g, dtype, p, &variant[0])) return 0;
        const WsLayout l = ws_layout((size_t)g.N * g.H * g.W * p.KCp, RS * p.Mp * p.KCp, p);
        return l.in + l.wt + l.part;
    }
    if (!plan_dx(g, dtype, p, cls, variant, &ncls, &empty)) return 0;
    // (only a stride-1 data gradient, a single class, ever shares out its channels)
    const WsLayout l = ws_layout((size_t)g.N * g.P * g.Q * p.KCp, RS * p.Mp * p.KCp, ncls == 1 ? cls[0] : p);
    return l.in + l.wt + l.part;
}

// Forward: Y = X * W + b.  False when the geometry is not covered.
// *pooled: Z has been written on the way (the channels-last repack reads X anyway); otherwise
// the caller runs the compress kernel.
bool launch_fwd_mfma(const Geom &g, int dtype, const void *X, const void *W, const void *b, void *Y, void *Z, void *ws,
                     hipStream_t st, hipError_t *err, bool *pooled)
{
    *pooled = false;
    GatherParams p{};
    int variant;
    if (!plan_fwd(g, dtype, p, &variant)) return false;
    const WsLayout l = ws_layout((size_t)g.N * g.H * g.W * p.KCp, (size_t)g.R * g.S * p.Mp * p.KCp, p);
    bf16_t *in = (bf16_t *)ws, *wt = (bf16_t *)((char *)ws + l.in);
    p.part = l.part ? (float *)((char *)ws + l.in + l.wt) : nullptr;
    // whole 2 x 2 tiles, rows a multiple of 8 pixels: the pooled map falls out of the repack
    const bool fuse0 = Z && !g.pmax && g.kh == 2 && g.kw == 2 && g.H % 2 == 0 && (g.W % 8 == 0 || g.W == 4);
    // Where the pooled map cannot come out of the repack anyway, X is read where it lies under the
    // same conditions as dY in the data gradient (no channels-last copy, only the filter repack).
    const bool direct = !p.decim && g.W % 2 == 0 && (long)g.N * g.C * g.H * g.W >= 8L * g.R * g.S * g.K * g.C &&
                        p.IPT * p.PH * ((g.W + 7) / 8) * (KC / 8) * p.T <= 512;
    const bool fuse = fuse0; // (with `direct` the repack launch forms Z without writing the channels-last copy)
    *err = launch_repack(direct && !fuse ? nullptr : (const bf16_t *)X, direct ? nullptr : in, g.N, g.C, g.H * g.W, p.KCp,
                         (const bf16_t *)W, wt, g.K, g.C, p.ntaps_total, p.Mp, p.KCp, 0, fuse ? (bf16_t *)Z : nullptr, g.W, st, nullptr,
                         p.decim);
    *pooled = fuse;
    if (*err != hipSuccess) return true;
    p.in = direct ? (const bf16_t *)X : in;
    p.nchw = direct;
    p.KCin = g.C;
    p.wt = wt; p.bias = (const bf16_t *)b; p.out = (bf16_t *)Y;
    *err = run_gather(p, variant, st);
    return true;
}

// Data gradient: dX = W^T * dY.  False when the geometry is not covered.
// tail: a weight-gradient slice sum to run in the repack launch (see repack_reduce_kernel); when
// this returns false nothing has been launched and the tail is still the caller's to run.
bool launch_dx_mfma(const Geom &g, int dtype, const void *W, const void *dY, void *dX, void *ws, hipStream_t st,
                    hipError_t *err, const DwReduceTail *tail)
{
    GatherParams base{}, cls[4];
    int variant[4], ncls = 0;
    bool empty_class = false;
    if (!plan_dx(g, dtype, base, cls, variant, &ncls, &empty_class)) return false;
    const WsLayout l = ws_layout((size_t)g.N * g.P * g.Q * base.KCp, (size_t)g.R * g.S * base.Mp * base.KCp, ncls == 1 ? cls[0] : base);
    bf16_t *in = (bf16_t *)ws, *wt = (bf16_t *)((char *)ws + l.in);
    for (int k = 0; k < ncls; ++k) cls[k].part = cls[k].ksplit > 1 ? (float *)((char *)ws + l.in + l.wt) : nullptr;
    // pixels no output pixel's tap reaches (possible when stride > filter) stay zero
    if (empty_class) {
        // (a fill kernel, not a memset node: callers may capture this call in a HIP graph)
        const long n = (long)g.N * g.C * g.H * g.W;
        hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)((n / 8 + 256) / 256)), dim3(256), 0, st, (bf16_t *)dX, n);
    }
    const bool direct = dx_reads_in_place(g, cls, ncls);
    *err = launch_repack(direct ? nullptr : (const bf16_t *)dY, in, g.N, g.K, g.P * g.Q, base.KCp, (const bf16_t *)W, wt, g.K, g.C,
                         base.ntaps_total, base.Mp, base.KCp, 1, nullptr, 0, st, tail);
    for (int k = 0; k < ncls && *err == hipSuccess; ++k) {
        cls[k].in = direct ? (const bf16_t *)dY : in;
        cls[k].nchw = direct;
        cls[k].KCin = g.K;
        cls[k].wt = wt; cls[k].bias = nullptr; cls[k].out = (bf16_t *)dX;
        *err = run_gather(cls[k], variant[k], st);
    }
    return true;
}

} // namespace cac
