// Weight gradient from the compressed activation as an MFMA implicit GEMM
// (bfloat16 operands, float accumulation), gfx950.
//
//   dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] * xhat[n,c,p*SG+r-PAD,q*SG+s-PAD],
//   xhat[n,c,h,w] = Z[n,c,h/kh,w/kw]        (weight-gradient formula of the
//                                             compression figure; inflation by
//                                             replication)
//
// GEMM view: M = output channels o, N = (input channel c, filter tap), K = pixels.
// A workgroup owns a (32*MI*WM) x (32*NI*WN) x all-taps tile and a slice of the
// pixels.  It has WM*WN*KS MFMA waves -- each holding MI x NI x taps accumulator
// blocks of 32x32; the KS waves that share a block split the rows of every chunk
// and add up through LDS at the end -- and as many copy waves, which bring the
// operands from global memory into LDS (one MFMA and one copy wave per SIMD).
//
// The pixel sum is re-indexed by the xhat column instead of the output column:
// with s - PAD = SG*a_s + b_s (0 <= b_s < SG),
//   dW[o,c,r,s] = sum_{n,p,j} dY[n,o,p,j-a_s] * xhat[n,c,p*SG+r-PAD, SG*j+b_s]
// so the xhat operand is always an ALIGNED block of 8 columns of "phase" b_s of
// an xhat row (phase b holds columns b, b+SG, ...), and only the dY operand is
// shifted (by a_s = -1, 0 or +1 columns).  One shifted dY fragment serves all
// filter rows and input-channel blocks; it is made in registers with v_perm from
// a sliding window over the dY row.  Zero padding needs no halo: columns outside
// the image simply do not occur, pixels outside the row are zero in the window.
// A 32x32x16 MFMA consumes two such blocks of 8, one in lanes 0-31 and one in
// lanes 32-63 (rows rho and rho+1 of the staged chunk).
//
// Staging per chunk (NBI images x PR output rows), double buffered in LDS:
//   rows [LR]                      per row: LDS offsets of its dY row and of the
//                                  xhat rows feeding each filter row
//   sDY  [tile_o][LR rows][Qpad]   dY, rows padded with zeros to a multiple of 8
//   sX   [tile_c][slots][phase][Qpad]  the needed rows of Z, expanded along the
//                                  row to full input width, zeros past W
// plus one shared all-zero row.  The inflated activation exists only here:
// expanded horizontally when written to LDS, expanded vertically by mapping an
// input row h to the slot of Z row h/kh.

#include <mutex>

#include "common.h"
#include "dw_mfma.h"
#include "dw_reduce.h"

namespace cac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ uint32_t fdiv(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

__device__ __forceinline__ uint32_t pack16(uint32_t lo, uint32_t hi) { return (lo & 0xffffu) | (hi << 16); }

// Result: low half = half `ha` of a, high half = half `hb` of b.
template <int ha, int hb> __device__ __forceinline__ uint32_t halves(uint32_t a, uint32_t b)
{
    constexpr uint32_t sel = (2 * ha) | ((2 * ha + 1) << 8) | ((4 + 2 * hb) << 16) | ((5 + 2 * hb) << 24);
    return __builtin_amdgcn_perm(b, a, sel);
}

// 16 bytes of LDS at an absolute LDS byte address (saves the compiler adding the
// base of the dynamic LDS block, unknown until link time, to every access).
typedef __attribute__((address_space(3))) const u32x4 *lds_u32x4_ptr;
__device__ __forceinline__ u32x4 lds16(uint32_t addr) { return *(lds_u32x4_ptr)(uintptr_t)addr; }

constexpr int kMaxDy = 8; // 16-byte dY items a thread moves per chunk
constexpr int kMaxZ = 4;  // 16-byte Z items a thread moves per chunk

// A window of one xhat row held in registers: the last dword of the block left
// of the current position and NB blocks starting at it.
template <int NB> struct Window {
    uint32_t prev3;
    u32x4 blk[NB];
};

// Element `e` (relative to the first element of blk[0]; -2 <= e < 8*NB): its register.
template <int NB, int e> __device__ __forceinline__ uint32_t win_reg(const Window<NB> &w)
{
    static_assert(e >= -2 && e < 8 * NB, "window too small");
    if constexpr (e < 0)
        return w.prev3;
    else
        return w.blk[e / 8][(e % 8) / 2];
}
template <int e> constexpr int win_half() { return ((e % 2) + 2) % 2; }

// B fragment for filter column s: pixel j of the segment needs element
// SG*j + s - PAD of the window.
template <int NB, int SG, int PAD, int s> __device__ __forceinline__ bf16x8 make_frag(const Window<NB> &w)
{
    union { u32x4 u; bf16x8 v; } f;
#define CAC_FRAG_DWORD(i)                                                                            \
    {                                                                                                \
        constexpr int e0 = SG * (2 * i) + s - PAD, e1 = SG * (2 * i + 1) + s - PAD;                  \
        if constexpr (e0 >= 0 && e0 % 2 == 0 && e1 == e0 + 1)                                        \
            f.u[i] = win_reg<NB, e0>(w); /* both halves of one dword, in place */                    \
        else                                                                                         \
            f.u[i] = halves<win_half<e0>(), win_half<e1>()>(win_reg<NB, e0>(w), win_reg<NB, e1>(w)); \
    }
    CAC_FRAG_DWORD(0) CAC_FRAG_DWORD(1) CAC_FRAG_DWORD(2) CAC_FRAG_DWORD(3)
#undef CAC_FRAG_DWORD
    return f.v;
}

// Global reads go through buffer loads: a lane whose byte offset lies at or beyond
// the tensor's size gets zeros back without touching memory and without a branch,
// so every load of a chunk can be in flight at once (tensors on this path are
// smaller than 2 GiB; offsets from 2^31 on mean "no load").
// Items are read with one 16-byte load each from the dword-aligned address at or below
// their first element (rows of odd length start on odd elements).
// The 8 elements themselves.  After an odd start everything moves down by one
// element and the last one comes from the first dword of the next item of the
// same row, which the next lane holds (the copy maps consecutive items of a row
// to consecutive lanes; the last item of a row never needs it: a row of odd
// length ends before its 8th element).  Then ANDed with `mask`: zero from the
// row's end on, what follows belongs to another row.
__device__ __forceinline__ u32x4 fix8(const u32x4 &d, uint32_t e, const u32x4 &mask, bool odd_possible)
{
    u32x4 v = d;
    if (odd_possible) {
        const uint32_t next0 = __shfl_down(d[0], 1, 64);
        const uint32_t sh = (e & 1u) * 16u;
        v[0] = __builtin_amdgcn_alignbit(d[1], d[0], sh);
        v[1] = __builtin_amdgcn_alignbit(d[2], d[1], sh);
        v[2] = __builtin_amdgcn_alignbit(d[3], d[2], sh);
        v[3] = __builtin_amdgcn_alignbit(next0, d[3], sh);
    }
    return v & mask;
}
// Dword j of the mask keeps the elements 2j, 2j+1 that lie below `left`.
__device__ __forceinline__ u32x4 mask8(int left)
{
    u32x4 m;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int l2 = left - 2 * j;
        m[j] = l2 >= 2 ? 0xffffffffu : (l2 == 1 ? 0xffffu : 0u);
    }
    return m;
}

// SC: the number of 8-pixel segments per output row when it is known at compile
// time (0: read from the plan).  With SC the walk along a row is unrolled and the
// segment offsets become immediates of the LDS reads.
template <int R, int S, int SG, int PAD, int MI, int NI, int WM, int WN, int KS, int SC, bool DYL>
__global__ void __launch_bounds__(128 * WM * WN * KS) dw_mfma_kernel(DwMfmaParams p)
{
    constexpr int T = R * S;
    constexpr int NT = 64 * WM * WN * KS; // threads of each kind: MFMA waves, then as many copy waves
    constexpr int TILE_O = 32 * MI * WM, TILE_C = 32 * NI * WN;
    // floor division / remainder of (s - PAD) by SG for every filter column
    constexpr auto a_of = [](int s) { int d = s - PAD; return d >= 0 ? d / SG : -((-d + SG - 1) / SG); };
    constexpr auto b_of = [](int s) { int d = s - PAD; return d - SG * (d >= 0 ? d / SG : -((-d + SG - 1) / SG)); };
    constexpr int NPH = (S == 1) ? 1 : SG; // xhat column phases in use
    static_assert(S <= 3 && SG <= 2 && a_of(0) >= -1 && a_of(S - 1) <= 1, "unsupported filter geometry");

    extern __shared__ __align__(16) unsigned char smem[];
    // [zero row][buffer 0: rows, sDY, sX][buffer 1: rows, sDY, sX]; offsets below are in
    // bf16 elements from the start of LDS, so offset 0 is the zero row
    bf16_t *sW = (bf16_t *)smem;
    const uint32_t rows_elems = p.LRpad * 8;                   // one 16-byte entry per row
    const uint32_t buf_elems = rows_elems + TILE_O * p.dy_ostride + TILE_C * p.x_cstride;
    const uint32_t slot_w = NPH * p.PW;                        // one xhat row: all phases
    const uint32_t base0 = slot_w, base1 = base0 + buf_elems;  // the buffers follow the zero row

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that each
    // XCD works on consecutive (slice, o-tile, c-tile) triples and re-reads of dY
    // and Z hit its own L2.
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= p.total_wg) return;
    const int ntiles = p.tiles_o * p.tiles_c;
    const int slice = v / ntiles, tile = v - slice * ntiles;
    const int ot = tile / p.tiles_c, ct = tile - ot * p.tiles_c;
    const int o0 = ot * TILE_O, c0 = ct * TILE_C;

    // What is read without ever being staged must start as zero: the shared zero row and,
    // in both buffers, the xhat part (every channel ends with an all-zero slot).  The row
    // table and the dY part are rewritten in full for every chunk.
    auto zero_fill = [&]() {
        const uint32_t x_elems = TILE_C * p.x_cstride, x_off = rows_elems + TILE_O * p.dy_ostride;
        u32x4 *l = (u32x4 *)smem;
        for (uint32_t i = threadIdx.x; i < slot_w / 8; i += 2 * NT) l[i] = u32x4{0, 0, 0, 0};
        for (uint32_t i = threadIdx.x; i < x_elems / 8; i += 2 * NT) {
            l[(base0 + x_off) / 8 + i] = u32x4{0, 0, 0, 0};
            l[(base1 + x_off) / 8 + i] = u32x4{0, 0, 0, 0};
        }
    };

    const int ci_begin = slice * p.chunks_per_slice;
    const int ci_end = min(ci_begin + p.chunks_per_slice, p.nchunks);

    // the role of a wave is uniform over the wave: tell the compiler so
    const int wave_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave_id >= NT / 64) {
        // =========================== copy waves ===========================================
        // They keep two chunks of global loads in flight and fill the LDS buffer the
        // MFMA waves are not reading; the only hand-over is one barrier per chunk.
        const int tid = threadIdx.x - NT;
        // dY: LDY lanes share one output channel's rows; item j = (row rho, segment sg)
        const uint32_t dyj = tid & (p.LDY - 1), dyo = tid >> p.ldy_log2;
        const uint32_t dy_rho = fdiv(dyj, p.m_segs), dy_sg = dyj - dy_rho * p.SEGS;
        const uint32_t dy_ni = fdiv(dy_rho, p.m_pr), dy_pr = dy_rho - dy_ni * p.PR;
        const bool dy_write = dyj < (uint32_t)p.rowitems;         // lanes past the row's items idle
        const bool dy_real = dy_write && dy_rho < (uint32_t)p.LR; // the spare row stays zero
        u32x4 dy_mask, z_mask, rag[2][2]; // (filled after the first loads are on their way)
        const uint32_t dy_rel = ((dy_ni * p.K + dyo) * p.P + dy_pr) * p.Q + dy_sg * 8;
        const uint32_t dy_opp = (uint32_t)NT >> p.ldy_log2;       // output channels per pass
        const uint32_t dy_gstep = dy_opp * p.P * p.Q;
        const uint32_t dy_lds = rows_elems + dyo * p.dy_ostride + dyj * 8;
        const uint32_t dy_lstep = dy_opp * p.dy_ostride;
        // Z: LPC lanes share one input channel; item j = (image ni, slot sl, vector zv of 8 pooled values)
        const uint32_t zj = tid & (p.LPC - 1), zc = tid >> p.lpc_log2;
        const uint32_t z_row = fdiv(zj, p.m_zv), z_zv = zj - z_row * p.ZV;
        const uint32_t z_ni = fdiv(z_row, p.m_nz), z_sl = z_row - z_ni * p.NZ;
        const bool z_write = zj < (uint32_t)p.citems;
        const uint32_t z_rel = ((z_ni * p.C + zc) * p.Hp + z_sl) * p.Wp + z_zv * 8;
        const uint32_t z_cpp = (uint32_t)NT >> p.lpc_log2;        // input channels per pass
        const uint32_t z_gstep = z_cpp * p.Hp * p.Wp;
        const uint32_t z_lds = rows_elems + TILE_O * p.dy_ostride + zc * p.x_cstride + z_row * slot_w;
        const uint32_t z_lstep = z_cpp * p.x_cstride;
        const bool dy_odd = p.Q & 1, z_odd = p.Wp & 1;
        const int f_log2 = p.kw_log2 - (SG == 2 ? 1 : 0);        // columns of one phase per pooled value, log2
        const bool ragged = (p.W & ((1 << p.kw_log2) - 1)) != 0; // the last pooling tile reaches past W
        const rsrc_t rs_dy = make_rsrc(p.dY, (uint32_t)p.N * p.K * p.P * p.Q * 2u);
        const rsrc_t rs_z = make_rsrc(p.Z, (uint32_t)p.N * p.C * p.Hp * p.Wp * 2u);
        // Output channels past K and input channels past C of an edge tile are read like any
        // other (from whatever follows in the tensor, zeros past its end): they only reach
        // accumulators that are never written out.

        // What depends on the chunk is uniform over the workgroup: the first image and output
        // row, the first Z row kept, and the element offsets of the tile's first dY / Z element.
        struct Src { uint32_t dy, z; int zbase, n0, p0; };
        auto src_of = [&](int ci) {
            Src s;
            const int ig = fdiv(ci, p.m_rb), rb = ci - ig * p.RB;
            s.n0 = ig * p.NBI;
            s.p0 = rb * p.PR;
            s.zbase = max(0, (s.p0 * SG - PAD) >> p.kh_log2);
            s.dy = ((uint32_t)(s.n0 * p.K + o0) * p.P + s.p0) * p.Q;
            s.z = ((uint32_t)(s.n0 * p.C + c0) * p.Hp + s.zbase) * p.Wp;
            return s;
        };
        // Element offset of this lane's item within the chunk, or far outside the tensor
        // (2^30 elements: the byte offset stays in [2^31, 2^32) after every addition below)
        // for a lane without an item.
        constexpr uint32_t kNoElem = 0x40000000u;
        const uint32_t dy_lane = dy_real ? dy_rel : kNoElem, z_lane = z_write ? z_rel : kNoElem;
        const uint32_t dy_istep = dy_gstep, z_istep = z_gstep;
        // ---- global -> registers for one chunk: one add per item, no branch
        // `live` false (uniform): the chunk does not exist; the loads are issued all the same,
        // past the tensors, so that the number of loads in flight is the same on every path and
        // a wait for the older chunk never has to include the younger one.
        auto fetch = [&](int ci, bool live, u32x4 (&rdy)[kMaxDy], u32x4 (&rz)[kMaxZ]) {
            const Src s = src_of(ci);
            // rows past P and images past N of an edge chunk must read as zeros: their pixels
            // meet real xhat rows in the shifted windows of their neighbours
            const bool dy_in = live && s.n0 + (int)dy_ni < p.N && s.p0 + (int)dy_pr < p.P;
            const uint32_t e_dy = dy_in ? s.dy + dy_lane : kNoElem;
            const uint32_t e_z = live ? s.z + z_lane : kNoElem; // rows past Hp are never looked at
            if constexpr (!DYL) {
#pragma unroll
                for (int i = 0; i < kMaxDy; ++i) {
                    // items past the last pass: offset 2^30 elements as well (uniform select)
                    const uint32_t e = e_dy + (i < p.dy_passes ? i * dy_istep : kNoElem);
                    rdy[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, (e & ~1u) * 2u, 0, 0);
                }
            }
#pragma unroll
            for (int i = 0; i < kMaxZ; ++i) {
                const uint32_t e = e_z + (i < p.z_passes ? i * z_istep : kNoElem);
                rz[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_z, (e & ~1u) * 2u, 0, 0);
            }
        };
        const int cw = __builtin_amdgcn_readfirstlane(tid >> 6); // index among the copy waves
        // DYL: dY goes from global memory straight into the LDS buffer (no registers, no LDS
        // store instructions).  A load of this kind writes the 64 lanes' 16 bytes side by side
        // from a uniform LDS address on, which is this kernel's dY layout when a wave's 64
        // lanes are the 64 items of one output channel and no item needs a mask (the plan sets
        // dy_direct then); lanes without a row, and chunks that do not exist, load zeros.
        auto load_dy = [&](int ci, bool live, uint32_t base) {
            const Src s = src_of(ci);
            const bool dy_in = live && s.n0 + (int)dy_ni < p.N && s.p0 + (int)dy_pr < p.P;
            const uint32_t e_dy = dy_in ? s.dy + dy_lane : kNoElem;
            __attribute__((address_space(3))) unsigned char *l3 = (__attribute__((address_space(3))) unsigned char *)smem;
#pragma unroll
            for (int i = 0; i < kMaxDy; ++i) {
                const uint32_t off = __builtin_amdgcn_readfirstlane((base + rows_elems + (cw + i * dy_opp) * p.dy_ostride) * 2u);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_dy, (__attribute__((address_space(3))) void *)(l3 + off), 16,
                                                         (e_dy + i * dy_istep) * 2u, 0, 0, 0);
            }
        };
        // DYL: everything but the Z loads of the youngest fetch has arrived, this chunk's dY too
        auto dy_landed = [&]() { __builtin_amdgcn_s_waitcnt((kMaxZ & 0xF) | ((kMaxZ >> 4) << 14) | 0x0F70); };
        // ---- registers -> LDS buffer at element offset `base` (with the horizontal inflation)
        auto stage = [&](int ci, uint32_t base, const u32x4 (&rdy)[kMaxDy], const u32x4 (&rz)[kMaxZ]) {
            // Everything but the kMaxDy + kMaxZ loads of the younger chunk has arrived.  Said
            // explicitly: items past the last pass are loaded but never looked at, and the
            // compiler, seeing loads nobody waited for, would otherwise drain the whole queue
            // before reusing their registers.  (s_waitcnt operand: vmcnt in bits 3:0 and 15:14,
            // the other counters left at their maximum.)
            constexpr int kYounger = kMaxDy + kMaxZ;
            __builtin_amdgcn_s_waitcnt((kYounger & 0xF) | ((kYounger >> 4) << 14) | 0x0F70);
            const Src s = src_of(ci);
            // row table: entry rho = {dY row offset, xhat row offset per filter row (the zero
            // slot for rows outside the image)}, in elements from the lane's channel base
            if (cw == 0 && tid < p.LRpad) {
                const uint32_t rho = tid;
                const uint32_t ni = fdiv(rho, p.m_pr);
                const int pp = s.p0 + (int)(rho - ni * p.PR);
                const bool row_ok = rho < (uint32_t)p.LR && pp < p.P && s.n0 + (int)ni < p.N;
                const uint32_t zero_slot = p.NBI * p.NZ * slot_w; // each channel ends with an all-zero xhat row
                u32x4 e = {rho * (uint32_t)p.Qpad, zero_slot, zero_slot, zero_slot};
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int h = pp * SG + r - PAD;
                    const bool ok = row_ok && h >= 0 && h < p.H;
                    e[1 + r] = ok ? ((int)ni * p.NZ + (h >> p.kh_log2) - s.zbase) * slot_w : zero_slot;
                }
                *(u32x4 *)(sW + base + rho * 8) = e;
            }
            // dY: fix-ups for all items first (they exchange data between lanes), then one
            // predicated run of stores
            u32x4 val[kMaxDy];
            if constexpr (DYL) {
            } else if (dy_odd) {
#pragma unroll
                for (int i = 0; i < kMaxDy; ++i) val[i] = fix8(rdy[i], s.dy + dy_rel + i * dy_istep, dy_mask, true);
            } else {
#pragma unroll
                for (int i = 0; i < kMaxDy; ++i) val[i] = rdy[i] & dy_mask;
            }
            if (!DYL && dy_write) {
                bf16_t *d = sW + base + dy_lds;
#pragma unroll
                for (int i = 0; i < kMaxDy; ++i)
                    if (i < p.dy_passes) *(u32x4 *)(d + i * dy_lstep) = val[i];
            }
            // Z
            u32x4 zz[kMaxZ];
            if (z_odd) {
#pragma unroll
                for (int i = 0; i < kMaxZ; ++i) zz[i] = fix8(rz[i], s.z + z_rel + i * z_istep, z_mask, true);
            } else {
#pragma unroll
                for (int i = 0; i < kMaxZ; ++i) zz[i] = rz[i] & z_mask;
            }
            if (z_write) {
                bf16_t *zd = sW + base + z_lds;
                // Writes 8 elements of phase ph starting at element j; in the ragged case the
                // elements whose xhat column SG*j+ph is at or beyond W are zeroed.
                auto put8 = [&](bf16_t *dst, int ph, int j, u32x4 x) {
                    if (ragged) x &= mask8((p.W - ph + SG - 1) / SG - j);
                    *(u32x4 *)(dst + ph * p.PW + j) = x;
                };
#define CAC_Z_ITEMS(...)                                                                           \
    _Pragma("unroll") for (int i = 0; i < kMaxZ; ++i) if (i < p.z_passes)                          \
    {                                                                                              \
        const u32x4 z = zz[i];                                                                     \
        bf16_t *dst = zd + i * z_lstep;                                                            \
        /* pooled value k of the item in both halves of a dword */                                 \
        auto dup = [&](int k) { return (k & 1) ? halves<1, 1>(z[k >> 1], z[k >> 1]) : halves<0, 0>(z[k >> 1], z[k >> 1]); }; \
        (void)dup;                                                                                 \
        __VA_ARGS__                                                                                \
    }
                if (f_log2 < 0) {
                    // kw = 1, stride 2: even columns to phase 0, odd ones to phase 1
                    // (zeros past W come from the load)
                    const int j0 = z_zv * 4;
                    CAC_Z_ITEMS({
                        *(u32x2 *)(dst + j0) = u32x2{halves<0, 0>(z[0], z[1]), halves<0, 0>(z[2], z[3])};
                        if (NPH > 1) *(u32x2 *)(dst + p.PW + j0) = u32x2{halves<1, 1>(z[0], z[1]), halves<1, 1>(z[2], z[3])};
                    })
                } else if (f_log2 == 0) {
                    const int j0 = z_zv * 8;
                    CAC_Z_ITEMS({
                        _Pragma("unroll") for (int ph = 0; ph < NPH; ++ph)
                            *(u32x4 *)(dst + ph * p.PW + j0) = ragged ? z & rag[ph][0] : z;
                    })
                } else if (f_log2 == 1) {
                    const int j0 = z_zv * 16;
                    CAC_Z_ITEMS({
                        const u32x4 lo = {dup(0), dup(1), dup(2), dup(3)}, hi = {dup(4), dup(5), dup(6), dup(7)};
                        _Pragma("unroll") for (int ph = 0; ph < NPH; ++ph) {
                            *(u32x4 *)(dst + ph * p.PW + j0) = ragged ? lo & rag[ph][0] : lo;
                            *(u32x4 *)(dst + ph * p.PW + j0 + 8) = ragged ? hi & rag[ph][1] : hi;
                        }
                    })
                } else if (f_log2 == 2) {
                    const int j0 = z_zv * 32;
                    CAC_Z_ITEMS({
                        _Pragma("unroll") for (int g = 0; g < 4; ++g) {
                            const u32x4 x = {dup(2 * g), dup(2 * g), dup(2 * g + 1), dup(2 * g + 1)};
                            _Pragma("unroll") for (int ph = 0; ph < NPH; ++ph) put8(dst, ph, j0 + 8 * g, x);
                        }
                    })
                } else {
                    const int j0 = z_zv * 64;
                    CAC_Z_ITEMS({
                        _Pragma("unroll") for (int g = 0; g < 8; ++g) {
                            const u32x4 x = {dup(g), dup(g), dup(g), dup(g)};
                            _Pragma("unroll") for (int ph = 0; ph < NPH; ++ph) put8(dst, ph, j0 + 8 * g, x);
                        }
                    })
                }
#undef CAC_Z_ITEMS
            }
        };

        u32x4 dyA[kMaxDy], zA[kMaxZ], dyB[kMaxDy], zB[kMaxZ];
        // Two chunks of loads are in flight.  A register set is refilled right after it has been
        // staged, in the same straight-line code, so that the compiler sees every load consumed
        // before its register is reused and never has to drain the other set's loads.
        fetch(ci_begin, true, dyA, zA); // (every workgroup has at least one chunk)
        fetch(ci_begin + 1, ci_begin + 1 < ci_end, dyB, zB);
        // what only the staging needs: the masks that cut an item at the end of its row, and,
        // for the ragged case, the two blocks an item expands to when f_log2 <= 1
        dy_mask = mask8(p.Q - (int)dy_sg * 8);
        z_mask = mask8(p.Wp - (int)z_zv * 8);
#pragma unroll
        for (int ph = 0; ph < 2; ++ph)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                rag[ph][h] = mask8((p.W - ph + SG - 1) / SG - (int)(z_zv << (3 + max(f_log2, 0))) - 8 * h);
        if constexpr (DYL) load_dy(ci_begin, true, base0);
        zero_fill(); // in the shadow of the first loads
        __syncthreads();
        stage(ci_begin, base0, dyA, zA);
        fetch(ci_begin + 2, ci_begin + 2 < ci_end, dyA, zA);
        if constexpr (DYL) dy_landed();
        __syncthreads(); // buffer 0 holds the first chunk
        for (int ci = ci_begin; ci < ci_end; ci += 2) {
            // MFMA waves are on buffer 0 (chunk ci); set B holds chunk ci+1, set A chunk ci+2.
            // (A chunk past the end is staged all the same -- zeros into a buffer nobody reads
            // any more -- so that every path consumes every load.)
            if constexpr (DYL) load_dy(ci + 1, ci + 1 < ci_end, base1); // (buffer 1 is free since the last barrier)
            stage(ci + 1, base1, dyB, zB);
            fetch(ci + 3, ci + 3 < ci_end, dyB, zB);
            if constexpr (DYL) dy_landed();
            __syncthreads();
            if (ci + 1 >= ci_end) break;
            // MFMA waves are on buffer 1 (chunk ci+1); set A holds chunk ci+2, set B chunk ci+3
            if constexpr (DYL) load_dy(ci + 2, ci + 2 < ci_end, base0);
            stage(ci + 2, base0, dyA, zA);
            fetch(ci + 4, ci + 4 < ci_end, dyA, zA);
            if constexpr (DYL) dy_landed();
            __syncthreads();
        }
        if constexpr (KS > 1) __syncthreads(); // the barrier inside the MFMA waves' cross-wave sum
        return;
    }

    // =============================== MFMA waves ===========================================
    const int tid = threadIdx.x, lane = tid & 63, wave = wave_id;
    const int wm = wave % WM, wn = (wave / WM) % WN, ks = wave / (WM * WN), half = lane >> 5, l32 = lane & 31;

    zero_fill();
    __syncthreads();

    f32x16 acc[MI][NI][T];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int j = 0; j < 16; ++j) acc[mi][ni][t][j] = 0.f;

    // ---- MFMA over one staged chunk --------------------------------------------------
    // Operands of one step: the window over the dY row(s) and the xhat blocks.
    struct Ops {
        Window<2> aw[MI];
        u32x4 b[R][NI][NPH];
    };
    // all MFMAs of one step: the window supplies the shifted dY fragments
    auto mfma_step = [&](const Ops &o) {
#define CAC_COL(s)                                                                                          \
    if constexpr (s < S) {                                                                                  \
        bf16x8 af[MI];                                                                                      \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi) af[mi] = make_frag<2, 1, a_of(s), 0>(o.aw[mi]);   \
        _Pragma("unroll") for (int r = 0; r < R; ++r)                                                       \
        _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                                   \
        {                                                                                                   \
            union { u32x4 u; bf16x8 v; } bf;                                                                \
            bf.u = o.b[r][ni][b_of(s)];                                                                     \
            _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                                               \
                acc[mi][ni][r * S + s] =                                                                    \
                    __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bf.v, acc[mi][ni][r * S + s], 0, 0, 0); \
        }                                                                                                   \
    }
        CAC_COL(1) CAC_COL(0) CAC_COL(2)
#undef CAC_COL
    };
    // Interleaving hint for one step: after every MFMA one LDS read (while any are
    // left) and a few VALU instructions, so that the next step's operand requests,
    // the address arithmetic and the v_perm of the shifted fragments issue in the
    // shadow of the MFMAs instead of between two steps (one MFMA wave per SIMD:
    // nothing else would fill the gap).
    auto interleave = [&]() {
        constexpr int kMfma = MI * NI * T, kReads = MI * (S > 1 ? 2 : 1) + R * NI * NPH + 1;
#pragma unroll
        for (int i = 0; i < kMfma; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // MFMA
            if (i < kReads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0); // DS read
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);                 // VALU
        }
    };
    // Requests the operands of segment `seg` of the rows at byte addresses ra / rx[]
    // into `o`.  `tail`: the segment is the last of its row, nothing lies right of it.
    const uint32_t astep = 64 * p.dy_ostride, xstep = 64 * p.x_cstride, pw = 2 * p.PW;
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    // have_blk0: the caller has filled blk[0] already (the block a step looks at to its right is
    // the next step's own block)
    auto request = [&](Ops &o, uint32_t ra, const uint32_t (&rx)[R], int seg, bool tail, bool have_blk0 = false) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            if (!(have_blk0 && S > 1)) o.aw[mi].blk[0] = lds16(ra + mi * astep + 16 * seg);
            if constexpr (S > 1) {
                // nothing lies right of a row's last segment.  Where the caller knows at compile
                // time that this is one, the block is a constant; otherwise it is read from the
                // zero row the dynamic LDS block starts with.
                if (__builtin_constant_p(tail) && tail) o.aw[mi].blk[1] = u32x4{0, 0, 0, 0};
                else o.aw[mi].blk[1] = lds16(tail ? lds0 : ra + mi * astep + 16 * seg + 16);
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int ph = 0; ph < NPH; ++ph) o.b[r][ni][ph] = lds16(rx[r] + ni * xstep + ph * pw + 16 * seg);
    };
    auto compute = [&](uint32_t base) {
        // byte addresses in LDS of this lane's output channel / input channel
        const uint32_t ac = lds0 + 2 * (base + rows_elems + (wm * 32 * MI + l32) * p.dy_ostride);
        const uint32_t xc = lds0 + 2 * (base + rows_elems + TILE_O * p.dy_ostride + (wn * 32 * NI + l32) * p.x_cstride);
        const uint32_t tab = lds0 + 2 * base + half * 16; // row table, this half-wave's entries
        // the KS waves that share a tile take every KS-th row pair each
        const int nrp = p.LRpad / 2, segs = SC > 0 ? SC : p.SEGS;
        if constexpr (R == 1 && S == 1) {
            // One tap: a step is MI*NI MFMAs, far too short to hide the two LDS round trips behind
            // it (row table, then operands) when operands are asked for one step ahead -- counters
            // and timings showed the MFMA waves of these layers waiting on LDS four fifths of the
            // time.  Without a window no step depends on its neighbour, so: the KS waves take
            // every KS-th (row pair, segment) step, whatever the row (rows per chunk need not be a
            // multiple of 2*KS for all of them to work); operands are requested two steps ahead
            // into a ring of three sets, the row table three steps ahead.
            const int total = nrp * segs;
            if (ks >= total) return;
            const int n = (total - ks + KS - 1) / KS;
            // step index of this wave's i-th step, clamped: requests past the end re-read the last step
            auto entry_of = [&](int i) {
                const int t = min(ks + i * KS, total - 1);
                return lds16(tab + 32 * (int)fdiv(t, p.m_segs));
            };
            auto ask = [&](Ops &o, int i, const u32x4 &e) {
                const int t = min(ks + i * KS, total - 1);
                const int seg = t - (int)fdiv(t, p.m_segs) * segs;
                const uint32_t rxx[R] = {xc + 2 * e[1]};
                request(o, ac + 2 * e[0], rxx, seg, true);
            };
            Ops O0, O1, O2;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) O0.aw[mi].prev3 = O1.aw[mi].prev3 = O2.aw[mi].prev3 = 0;
            u32x4 e0 = entry_of(0), e1 = entry_of(1), e_ahead = entry_of(2);
            ask(O0, 0, e0);
            ask(O1, 1, e1);
            int i = 0;
#define CAC_PW_PHASE(USE, GET)                    \
    {                                             \
        const u32x4 e_now = e_ahead;              \
        e_ahead = entry_of(i + 3);                \
        ask(GET, i + 2, e_now);                   \
        mfma_step(USE);                           \
        interleave();                             \
        if (++i == n) break;                      \
    }
            for (;;) {
                CAC_PW_PHASE(O0, O2)
                CAC_PW_PHASE(O1, O0)
                CAC_PW_PHASE(O2, O1)
            }
#undef CAC_PW_PHASE
            return;
        }
        const int nsteps = ((nrp - ks + KS - 1) / KS) * segs;
        if (KS > 1 && nsteps == 0) return;

        // current rows of this lane and the raw table entry of the next row pair
        u32x4 e = lds16(tab + 32 * ks);
        uint32_t ra = ac + 2 * e[0], rx[R];
#pragma unroll
        for (int r = 0; r < R; ++r) rx[r] = xc + 2 * e[1 + r];
        u32x4 e_next = lds16(tab + 32 * min(ks + KS, nrp - 1));

        Ops X, Y;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) X.aw[mi].prev3 = 0;
        request(X, ra, rx, 0, segs == 1);

        if constexpr (SC > 0 && NPH == 1) {
            // Row pairs as an outer loop, the SC segments of a row unrolled.  The operand sets
            // alternate from step to step; an odd SC swaps their roles from one row to the next.
            int rp = ks;
            // step SGI of a row pair: MFMAs on USE while GET receives the operands of the next
            // step (one segment to the right, or the first segment of the wave's next row pair)
#define CAC_ROWSTEP(USE, GET, SGI)                                                                  \
    if constexpr (SGI < SC) {                                                                       \
        if constexpr (SGI + 1 < SC) {                                                               \
            _Pragma("unroll") for (int mi = 0; mi < MI; ++mi) {                                     \
                GET.aw[mi].prev3 = USE.aw[mi].blk[0][3];                                            \
                GET.aw[mi].blk[0] = USE.aw[mi].blk[1];                                              \
            }                                                                                       \
            request(GET, ra, rx, SGI + 1, SGI + 2 == SC, true);                                     \
        } else {                                                                                    \
            ra = ac + 2 * e_next[0];                                                                \
            _Pragma("unroll") for (int r = 0; r < R; ++r) rx[r] = xc + 2 * e_next[1 + r];           \
            e_next = lds16(tab + 32 * min(rp + 2 * KS, nrp - 1));                                   \
            _Pragma("unroll") for (int mi = 0; mi < MI; ++mi) GET.aw[mi].prev3 = 0;                 \
            request(GET, ra, rx, 0, SC == 1);                                                       \
            rp += KS;                                                                               \
        }                                                                                           \
        mfma_step(USE);                                                                             \
        interleave();                                                                               \
    }
#define CAC_ROW(A, B)                                                                              \
    CAC_ROWSTEP(A, B, 0) CAC_ROWSTEP(B, A, 1) CAC_ROWSTEP(A, B, 2) CAC_ROWSTEP(B, A, 3)            \
    CAC_ROWSTEP(A, B, 4) CAC_ROWSTEP(B, A, 5) CAC_ROWSTEP(A, B, 6) CAC_ROWSTEP(B, A, 7)
            static_assert(SC <= 8, "row steps are written out up to 8");
            const int nrows = nsteps / SC;
            if constexpr (SC % 2 == 0) {
                for (int i = 0; i < nrows; ++i) { CAC_ROW(X, Y) }
            } else {
                for (int i = 0;;) {
                    CAC_ROW(X, Y)
                    if (++i == nrows) break;
                    CAC_ROW(Y, X)
                    if (++i == nrows) break;
                }
            }
#undef CAC_ROW
#undef CAC_ROWSTEP
            return;
        }
        int seg = 0, rp = ks;
        // One step: MFMAs on USE, operands of the following step requested into GET
        // (same rows one segment to the right, or the next row pair, whose table
        // entry was requested a row pair ago).
#define CAC_STEP(USE, GET)                                                                        \
    if (seg + 1 < segs) {                                                                         \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi) GET.aw[mi].prev3 = USE.aw[mi].blk[0][3]; \
        request(GET, ra, rx, seg + 1, seg + 2 == segs);                                           \
        mfma_step(USE);                                                                           \
        interleave();                                                                             \
        ++seg;                                                                                    \
    } else {                                                                                      \
        ra = ac + 2 * e_next[0];                                                                  \
        _Pragma("unroll") for (int r = 0; r < R; ++r) rx[r] = xc + 2 * e_next[1 + r];             \
        e_next = lds16(tab + 32 * min(rp + 2 * KS, nrp - 1));                   \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi) GET.aw[mi].prev3 = 0;                   \
        request(GET, ra, rx, 0, segs == 1);                                                       \
        mfma_step(USE);                                                                           \
        interleave();                                                                             \
        seg = 0;                                                                                  \
        rp += KS;                                                                                 \
    }
        if constexpr (NPH == 1) {
            for (int t = 0;;) {
                CAC_STEP(X, Y)
                if (++t == nsteps) break;
                CAC_STEP(Y, X)
                if (++t == nsteps) break;
            }
        } else {
            // two column phases double the xhat operands: a second operand set does not
            // fit the register file next to the accumulators, so these (few) layers
            // request each step's operands right before using them
            for (int t = 0; t < nsteps; ++t) {
                mfma_step(X);
                if (t + 1 == nsteps) break;
                if (seg + 1 < segs) {
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) X.aw[mi].prev3 = X.aw[mi].blk[0][3];
                    request(X, ra, rx, seg + 1, seg + 2 == segs);
                    ++seg;
                } else {
                    ra = ac + 2 * e_next[0];
#pragma unroll
                    for (int r = 0; r < R; ++r) rx[r] = xc + 2 * e_next[1 + r];
                    e_next = lds16(tab + 32 * min(rp + 2 * KS, nrp - 1));
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) X.aw[mi].prev3 = 0;
                    request(X, ra, rx, 0, segs == 1);
                    seg = 0;
                    rp += KS;
                }
            }
        }
#undef CAC_STEP
    };

    __syncthreads(); // buffer 0 holds the first chunk
    for (int ci = ci_begin; ci < ci_end; ci += 2) {
        compute(base0);
        __syncthreads();
        if (ci + 1 >= ci_end) break;
        compute(base1);
        __syncthreads();
    }

    // ---- epilogue --------------------------------------------------------------------
    // accumulator register j of lane l holds row 8*(j/4) + 4*(l/32) + j%4, column l%32.
    // The accumulators are handled as G groups of 4 registers: g = (j/4)*(G/4) + (mi*NI + ni)*T + tap.
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    typedef f32x4 __attribute__((aligned(4))) f32x4_u;
    constexpr int G = MI * NI * T * 4;
    static_assert(KS == 1 || KS == 2 || KS == 4, "the K-split waves share the four row groups");
    // The KS waves of a tile hold sums over different pixels.  Wave ks keeps the groups with
    // j/4 in [ks*4/KS, (ks+1)*4/KS) and hands the others over through LDS (the staging buffers
    // are dead: the loop above ends with a barrier), then adds what the other waves hand it, in
    // wave order.  red[wm, wn][source wave][g][lane].
    f32x4 *red = (f32x4 *)smem + ((wn * WM + wm) * KS) * (G * 64) + lane;
#define CAC_G(mi, ni, t, jq) ((jq) * (G / 4) + ((mi) * NI + (ni)) * T + (t))
#define CAC_GROUP(mi, ni, t, jq) \
    f32x4 { acc[mi][ni][t][4 * (jq)], acc[mi][ni][t][4 * (jq) + 1], acc[mi][ni][t][4 * (jq) + 2], acc[mi][ni][t][4 * (jq) + 3] }
    if constexpr (KS > 1) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int t = 0; t < T; ++t)
#pragma unroll
                    for (int jq = 0; jq < 4; ++jq)
                        if (jq * KS / 4 != ks) red[(ks * G + CAC_G(mi, ni, t, jq)) * 64] = CAC_GROUP(mi, ni, t, jq);
        __syncthreads();
    }
    // Output: dW itself (one slice), or this slice's partial sums in the workspace, in the same
    // [o][c][tap] order, so that the sum over the slices is a plain stream.
    float *out = p.direct ? p.out : p.out + (long)slice * p.K * p.C * T;
    const bool inside = o0 + TILE_O <= p.K && c0 + TILE_C <= p.C; // no edge of dW crosses the tile
    // Nine taps, a tile inside dW, rows of dW a multiple of 16 bytes: a group (8 output channels x
    // 32 input channels x 9 taps) is 8 contiguous runs of 1152 bytes in memory.  It goes through
    // a wave-private 9 KB of LDS, [row][c][tap], and leaves as 16-byte stores in which the lanes
    // of a wave cover whole runs (a lane's own 36-byte runs, unaligned and 36 bytes apart, cost
    // the store unit 1.5 us per group).  The 9 KB: with the pixels split over the waves, the part
    // of `red` reserved for the groups the wave keeps from itself, which nobody writes or reads;
    // otherwise the dead staging buffers.
    const bool runs16 = T == 9 && inside && (p.C & 3) == 0;
    float *tb = KS > 1 ? (float *)((f32x4 *)smem + (((wn * WM + wm) * KS + ks) * G + (ks * 4 / KS) * (G / 4)) * 64)
                       : (float *)smem + wave * (8 * 32 * 9);
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                if (KS > 1 && jq * KS / 4 != ks) continue;
                f32x4 v[T];
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    v[t] = CAC_GROUP(mi, ni, t, jq);
                    if constexpr (KS > 1) {
#pragma unroll
                        for (int k2 = 0; k2 < KS; ++k2)
                            if (k2 != ks) v[t] += red[(k2 * G + CAC_G(mi, ni, t, jq)) * 64];
                    }
                }
                if (T == 9 && runs16) {
#pragma unroll
                    for (int t = 0; t < T; ++t)
#pragma unroll
                        for (int e = 0; e < 4; ++e) tb[half * 1152 + l32 * 9 + e * 288 + t] = v[t][e];
                    // (the wave reads what it wrote itself: LDS serves a wave's requests in order)
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    const long row0 = (long)(o0 + (wm * MI + mi) * 32 + 8 * jq) * p.C + c0 + (wn * NI + ni) * 32;
#pragma unroll
                    for (int k = 0; k < 9; ++k) {
                        const int q4 = k * 64 + lane, rr = q4 / 72, w4 = q4 - rr * 72; // row, 16-byte unit of its run
                        *(f32x4 *)(out + (row0 + (long)rr * p.C) * 9 + 4 * w4) = ((const f32x4 *)tb)[q4];
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    continue;
                }
                // the T taps of one (o, c) are consecutive floats
                const int c = c0 + (wn * NI + ni) * 32 + l32;
                const int ob = o0 + (wm * MI + mi) * 32 + 8 * jq + 4 * half;
                float *dst = out + ((long)ob * p.C + c) * T;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (inside || (ob + e < p.K && c < p.C)) {
                        float *d = dst + (long)e * p.C * T;
                        if constexpr (T == 9) {
                            *(f32x4_u *)d = f32x4{v[0][e], v[1][e], v[2][e], v[3][e]};
                            *(f32x4_u *)(d + 4) = f32x4{v[4][e], v[5][e], v[6][e], v[7][e]};
                            d[8] = v[8][e];
                        } else {
#pragma unroll
                            for (int t = 0; t < T; ++t) d[t] = v[t][e];
                        }
                    }
                }
            }
#undef CAC_GROUP
#undef CAC_G
}

// The slice sum as a launch of its own (body and description: dw_reduce.h).
template <int SY, int V>
__global__ void __launch_bounds__(256) dw_reduce_kernel(const float *__restrict__ part, float *__restrict__ dW, long total, int nslices)
{
    dw_reduce_body<SY, V>(part, dW, total, nslices, blockIdx.x);
}

uint32_t magic_of(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }

// Kernel table: filter/stride family x workgroup shape.
struct Variant {
    int R, SG, MI, NI, WM, WN, KS;
    hipError_t (*launch)(const DwMfmaParams &, dim3, hipStream_t);
};

template <int R, int S, int SG, int PAD, int MI, int NI, int WM, int WN, int KS, int SC, bool DYL = false>
hipError_t launch_fixed(const DwMfmaParams &p, dim3 grid, hipStream_t st)
{
    auto kern = dw_mfma_kernel<R, S, SG, PAD, MI, NI, WM, WN, KS, SC, DYL>;
    // (per instantiation; once per process, whichever host thread comes first)
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] { attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); });
    if (attr_err != hipSuccess) return attr_err;
    hipLaunchKernelGGL(kern, grid, dim3(128 * WM * WN * KS), p.lds_bytes, st, p);
    return hipGetLastError();
}
// Picks the instantiation with the row length built in when there is one.
template <int R, int S, int SG, int PAD, int MI, int NI, int WM, int WN, int KS>
hipError_t launch_variant(const DwMfmaParams &p, dim3 grid, hipStream_t st)
{
    if constexpr (S == 3 && SG == 1 && KS == 4) {
        if (p.dy_direct) {
            switch (p.SEGS) {
            case 1: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 1, true>(p, grid, st);
            case 2: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 2, true>(p, grid, st);
            case 4: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 4, true>(p, grid, st);
            default: break;
            }
        }
    }
    if constexpr (S == 3 && SG == 1) {
        switch (p.SEGS) {
        case 1: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 1>(p, grid, st);
        case 2: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 2>(p, grid, st);
        case 4: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 4>(p, grid, st);
        case 7: return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 7>(p, grid, st);
        default: break;
        }
    }
    return launch_fixed<R, S, SG, PAD, MI, NI, WM, WN, KS, 0>(p, grid, st);
}

const Variant kVariants[] = {
    {3, 1, 1, 1, 2, 2, 1, launch_variant<3, 3, 1, 1, 1, 1, 2, 2, 1>}, // 3x3: 64 x 64 tile, 144 accumulators per wave
    {3, 1, 1, 1, 1, 1, 4, launch_variant<3, 3, 1, 1, 1, 1, 1, 1, 4>}, // 3x3: 32 x 32 tile, the pixels split over 4 waves
    {3, 2, 1, 1, 2, 2, 1, launch_variant<3, 3, 2, 1, 1, 1, 2, 2, 1>},
    {3, 2, 1, 1, 1, 1, 4, launch_variant<3, 3, 2, 1, 1, 1, 1, 1, 4>},
    {1, 1, 2, 2, 2, 2, 1, launch_variant<1, 1, 1, 0, 2, 2, 2, 2, 1>}, // 1x1: 128 x 128 tile
    {1, 1, 2, 2, 1, 1, 4, launch_variant<1, 1, 1, 0, 2, 2, 1, 1, 4>}, // 1x1:  64 x 64 tile, the pixels split over 4 waves
    {1, 1, 2, 2, 1, 1, 1, launch_variant<1, 1, 1, 0, 2, 2, 1, 1, 1>}, // 1x1:  64 x 64 tile, one wave
    {1, 2, 2, 2, 2, 2, 1, launch_variant<1, 1, 2, 0, 2, 2, 2, 2, 1>},
    {1, 2, 2, 2, 1, 1, 4, launch_variant<1, 1, 2, 0, 2, 2, 1, 1, 4>},
    {1, 2, 2, 2, 1, 1, 1, launch_variant<1, 1, 2, 0, 2, 2, 1, 1, 1>},
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

} // namespace

namespace {

// The plan for one entry of the kernel table; false when the geometry does not fit it.
bool plan_with(const Geom &g, int vi, DwMfmaPlan *plan)
{
    auto log2_of = [](int k) { return k == 1 ? 0 : k == 2 ? 1 : k == 4 ? 2 : k == 8 ? 3 : -1; };
    const int khl = log2_of(g.kh), kwl = log2_of(g.kw);
    const int T = g.R * g.S;
    const Variant &var = kVariants[vi];
    const int KS = var.KS;
    const int NT = 64 * var.WM * var.WN * KS;
    const int tile_o = 32 * var.MI * var.WM, tile_c = 32 * var.NI * var.WN;
    const int lds_budget = (NT == 256 ? 156 : NT == 128 ? 78 : 39) * 1024; // whole CU / half / quarter
    const int groups = var.MI * var.NI * T * 4;                             // accumulator groups of 4 per wave
    const int red_bytes = KS > 1 ? var.WM * var.WN * KS * groups * 64 * 16 : 0;

    DwMfmaParams base{};
    base.N = g.N; base.C = g.C; base.K = g.K; base.H = g.H; base.W = g.W; base.P = g.P; base.Q = g.Q;
    base.Hp = g.Hp; base.Wp = g.Wp;
    base.kh_log2 = khl; base.kw_log2 = kwl;
    base.SEGS = (g.Q + 7) / 8;
    base.Qpad = base.SEGS * 8;
    base.ZV = (g.Wp + 7) / 8;
    const int NPH = g.S == 1 ? 1 : g.sh;  // xhat column phases kept per row
    // width of one phase of an xhat row in LDS: the padded output row, or what the
    // staging of whole 8-value items writes if that is more
    const int f_log2 = kwl - (g.sh == 2 ? 1 : 0);
    base.PW = max(base.Qpad, f_log2 >= 0 ? (8 * base.ZV) << f_log2 : 4 * base.ZV);
    base.XW = NPH * base.PW;              // one xhat row in LDS: all phases
    base.tile_o = tile_o; base.tile_c = tile_c;

    // Fills the chunk-dependent fields; false when the chunk does not fit the
    // per-thread copy registers or the LDS budget (two buffers).
    auto shape = [&](int nbi, int pr, DwMfmaParams &q) {
        q = base;
        q.NBI = nbi; q.PR = pr;
        q.RB = (g.P + pr - 1) / pr;
        q.LR = nbi * pr;
        q.LRpad = (q.LR + 1) & ~1;
        int nz = 1;
        for (int rb = 0; rb < q.RB; ++rb) {
            const int p0 = rb * pr, p1 = min(p0 + pr, g.P) - 1;
            const int zlo = max(0, (p0 * g.sh - g.ph) >> khl);
            const int hhi = min(g.H - 1, p1 * g.sh + g.R - 1 - g.ph);
            nz = max(nz, (hhi >> khl) - zlo + 1);
        }
        q.NZ = nz;
        q.rowitems = q.LRpad * q.SEGS;
        q.citems = nbi * nz * q.ZV;
        auto pow2_at_least = [](int x) { int l = 2; while ((1 << l) < x) ++l; return l; };
        q.ldy_log2 = pow2_at_least(q.rowitems); q.LDY = 1 << q.ldy_log2;
        q.lpc_log2 = pow2_at_least(q.citems);   q.LPC = 1 << q.lpc_log2;
        if (q.LDY > NT || q.LPC > NT) return false;
        q.dy_passes = (tile_o * q.LDY + NT - 1) / NT;
        q.z_passes = (tile_c * q.LPC + NT - 1) / NT;
        if (q.dy_passes > kMaxDy || q.z_passes > kMaxZ) return false;
        if ((tile_o * q.LDY) % NT || (tile_c * q.LPC) % NT) return false; // passes cover the tile exactly
        // strides: an odd number of 16-byte units so that the 32 lanes of a half
        // wave (one output channel / input channel each) read distinct LDS banks
        q.dy_ostride = 8 * ((q.rowitems + 1) | 1); // + one block: the dY window looks one block past a row
        q.x_cstride = 8 * (((nbi * nz + 1) * (q.XW / 8)) | 1); // + the zero slot
        q.dy_direct = var.R == 3 && var.SG == 1 && var.KS == 4 && // (the kernels that exist with it: see launch_variant)
                      g.Q % 8 == 0 && q.rowitems == 64 && q.LDY == 64 && q.dy_passes == 8 && (q.SEGS == 1 || q.SEGS == 2 || q.SEGS == 4);
        q.lds_bytes = (q.XW + 2 * (q.LRpad * 8 + tile_o * q.dy_ostride + tile_c * q.x_cstride)) * 2;
        if (q.lds_bytes > lds_budget) return false;
        q.lds_bytes = max(q.lds_bytes, red_bytes); // the cross-wave sum reuses the staging space
        q.lds_bytes = max(q.lds_bytes, var.WM * var.WN * 8 * 32 * 9 * 4); // so does the epilogue's transpose (9 KB per wave)
        return true;
    };
    // Candidates: part of one image (nbi = 1, pr <= P) or several whole images.
    // Cost = MFMA steps spent per useful pixel row, then prefer longer chunks.
    DwMfmaParams best{};
    double best_cost = 1e30;
    auto consider = [&](int nbi, int pr) {
        DwMfmaParams q;
        if (!shape(nbi, pr, q)) return;
        const int rp_wave = (q.LRpad / 2 + KS - 1) / KS;                 // row pairs of the busiest wave
        const double steps = (double)q.RB * rp_wave * KS * q.SEGS;       // per group of nbi images
        const double useful = (double)nbi * g.P * g.Q / 16.0;
        const double per_chunk = rp_wave * q.SEGS;
        const double cost = steps / useful * (1.0 + 1.5 / per_chunk);     // barrier + refill share
        if (cost < best_cost) { best_cost = cost; best = q; }
    };
    for (int pr = 1; pr <= g.P; ++pr) consider(1, pr);
    for (int nbi = 2; nbi <= min(g.N, 64); ++nbi) consider(nbi, g.P);
    if (best_cost > 1e29) return false;

    DwMfmaParams &p = plan->p;
    p = best;
    p.m_segs = magic_of(p.SEGS);
    p.m_pr = magic_of(p.PR);
    p.m_zv = magic_of(p.ZV);
    p.m_nz = magic_of(p.NZ);
    p.m_rb = magic_of(p.RB);

    p.tiles_o = (g.K + tile_o - 1) / tile_o;
    p.tiles_c = (g.C + tile_c - 1) / tile_c;
    const int ntiles = p.tiles_o * p.tiles_c;
    p.nchunks = ((g.N + p.NBI - 1) / p.NBI) * p.RB;
    // one workgroup per 256 threads of the 256 CUs, each with at least two chunks
    const int wg_target = 256 * (256 / NT);
    int want = max(1, wg_target / ntiles);
    want = min(want, max(1, p.nchunks / 2));
    p.chunks_per_slice = (p.nchunks + want - 1) / want;
    p.nslices = (p.nchunks + p.chunks_per_slice - 1) / p.chunks_per_slice;
    p.total_wg = p.nslices * ntiles;
    p.direct = p.nslices == 1;
    plan->grid = ((p.total_wg + 7) / 8) * 8;
    plan->threads = NT;
    plan->partial_bytes = p.direct ? 0 : (size_t)p.nslices * g.K * g.C * T * sizeof(float);
    plan->variant = vi;
    return true;
}

} // namespace

bool dw_mfma_plan(const Geom &g, int dtype, DwMfmaPlan *plan)
{
    if (dtype != CAC_BF16) return false;
    if (g.R != g.S || g.sh != g.sw || g.ph != g.pw) return false;
    const bool f3 = g.R == 3 && g.ph == 1, f1 = g.R == 1 && g.ph == 0;
    if (!(f3 || f1) || (g.sh != 1 && g.sh != 2)) return false;
    auto log2_of = [](int k) { return k == 1 ? 0 : k == 2 ? 1 : k == 4 ? 2 : k == 8 ? 3 : -1; };
    const int khl = log2_of(g.kh), kwl = log2_of(g.kw);
    if (khl < 0 || kwl < 0) return false;
    if (g.Q > 256 || g.W > 1024) return false;
    // buffer loads address with 32-bit byte offsets and use 2^31 as "no load"
    if ((long)g.N * g.K * g.P * g.Q >= (1L << 30) || (long)g.N * g.C * g.Hp * g.Wp >= (1L << 30)) return false;

    // Workgroup shape.  Splitting the pixels over the waves of a workgroup (KS > 1) cuts the
    // partial sums a workgroup writes by KS at the price of shorter runs between barriers and
    // twice the staging work per MFMA; it pays when a workgroup has only a few chunks to go
    // through.  Among the others: the large tile unless it would be mostly padding.
    DwMfmaPlan whole, split;
    bool have_whole = false, have_split = false;
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant &v = kVariants[i];
        if (v.R != g.R || v.SG != g.sh) continue;
        const int to = 32 * v.MI * v.WM, tc = 32 * v.NI * v.WN;
        if (to > 64 && (g.K <= to / 2 || g.C <= tc / 2)) continue;
        if (v.KS > 1) {
            if (!have_split) have_split = plan_with(g, i, &split);
        } else {
            if (!have_whole) have_whole = plan_with(g, i, &whole);
        }
    }
    if (!have_whole && !have_split) return false;
    const int thr = g.R == 1 ? 12 : 24; // measured break-even (chunks per workgroup: split wins at 16, loses at 32)
    bool use_split = have_split && (!have_whole || split.p.chunks_per_slice <= thr);
#ifdef CAC_TUNING // development builds: CAC_DW_SHAPE=whole|split overrides the rule
    if (const char *f = getenv("CAC_DW_SHAPE")) {
        if (f[0] == 'w' && have_whole) use_split = false;
        if (f[0] == 's' && have_split) use_split = true;
    }
#endif
    *plan = use_split ? split : whole;
    return true;
}

hipError_t launch_dw_reduce(const DwReduceTail &t, hipStream_t st)
{
    if (!t.blocks) return hipSuccess;
#define CAC_REDUCE(SY, V) \
    hipLaunchKernelGGL((dw_reduce_kernel<SY, V>), dim3(t.blocks), dim3(256), 0, st, t.part, t.dW, t.total, t.nslices)
    if (t.V == 4) {
        if (t.SY == 16) CAC_REDUCE(16, 4);
        else if (t.SY == 4) CAC_REDUCE(4, 4);
        else CAC_REDUCE(1, 4);
    } else {
        if (t.SY == 16) CAC_REDUCE(16, 1);
        else if (t.SY == 4) CAC_REDUCE(4, 1);
        else CAC_REDUCE(1, 1);
    }
#undef CAC_REDUCE
    return hipGetLastError();
}

// `defer`: when given, the slice sum is not launched; what it has to do is written there instead
// (blocks = 0 when the main kernel has written dW itself) and the caller sees to it.
hipError_t launch_dw_mfma(const DwMfmaPlan &plan, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                          DwReduceTail *defer)
{
    DwMfmaParams p = plan.p;
    p.Z = (const bf16_t *)Z;
    p.dY = (const bf16_t *)dY;
    p.out = p.direct ? dW : (float *)ws;
    if (defer) defer->blocks = 0;
    const Variant &var = kVariants[plan.variant];
    hipError_t e = var.launch(p, dim3(plan.grid), st);
    if (e != hipSuccess || p.direct) return e;
    const DwReduceTail t = make_reduce_tail((const float *)ws, dW, (long)p.K * p.C * var.R * var.R, p.nslices);
    if (defer) {
        *defer = t;
        return hipSuccess;
    }
    return launch_dw_reduce(t, st);
}

} // namespace cac
