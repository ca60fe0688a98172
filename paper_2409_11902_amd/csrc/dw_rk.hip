// Weight gradient from the compressed activation in its reduced-K form, gfx950
// (bfloat16 operands, float accumulation; 3x3 filter, stride 1, padding 1, 2x2 tiles,
// even maps).
//
// The inflated activation xhat[n,c,h,w] = Z[n,c,h/2,w/2] is constant on a pooling tile, so in
//   dW[o,c,r,s] = sum_{n,p,q} dY[n,o,p,q] * xhat[n,c,p+r-1,q+s-1]
// (weight-gradient formula of the compression figure, applied to the inflated Z) all pixels
// whose tap lands in tile (i,j) meet the same Z[n,c,i,j]:
//   dW[o,c,r,s] = sum_{n,i,j} Z[n,c,i,j] * T_rs[n,o,i,j],
//   T_rs[n,o,i,j] = sum of dY[n,o,p,q] over p+r-1 in {2i,2i+1}, q+s-1 in {2j,2j+1}.
// The GEMM runs over pooled pixels: a quarter of the multiply-adds, and Z is used as it is
// stored -- nothing is inflated anywhere.  The rows p that feed tile row i are
//   r = 1: {2i, 2i+1}          "even pairs"   E[i]
//   r = 0: {2i+1, 2i+2}        "odd pairs"    O[i]
//   r = 2: {2i-1, 2i}                       = O[i-1]
// and the same for columns, so four maps (E or O rows) x (E or O columns) of dY pair sums serve
// all nine taps; O maps are stored from index -1 on, which turns r = 2 / s = 2 into the aligned
// read and r = 0 / s = 0 into the read one row down / one element to the right.  (With an odd
// extent the last, ragged tile would need different sums for r = 0 and r = 2; such layers stay
// on the inflating kernel.)
//
// A workgroup owns a 32 (o) x 128 (c) x 9 taps tile of dW and a slice of the images: 4 MFMA
// waves (32 x 32 x 9 accumulator blocks each) and 4 copy waves, one of each per SIMD.  The copy
// waves form the four maps from dY in float, round them to bfloat16 once and write them to LDS
// next to the rows of Z; a 32x32x16 MFMA consumes one 8-column block of two pooled rows.  The
// tile sums are the only place where this form rounds differently from the inflating one.
//
// LDS (bfloat16 elements): [zero block][buffer 0][buffer 1], a buffer = one chunk = two units:
//   table [LRZpad]                           per Z row: byte offsets of its Z row and tile-sum row
//   sS    [32 o][2*US rows][4 maps][SW]      maps: 0 = E rows, E cols; 1 = E rows, O cols;
//                                                  2 = O rows, E cols; 3 = O rows, O cols
//   sZ    [128 c][LRZpad rows + zero row][ZW]
// A unit is what one set of copy registers holds (NBIu images x PRp pooled rows).
#include <mutex>

#include "common.h"
#include "dw_rk.h"

namespace cac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ uint32_t fdiv(uint32_t x, uint32_t magic) { return magic ? __umulhi(x, magic) : x; }

typedef __attribute__((address_space(3))) const u32x4 *lds_u32x4_ptr;
__device__ __forceinline__ u32x4 lds16(uint32_t addr) { return *(lds_u32x4_ptr)(uintptr_t)addr; }

__device__ __forceinline__ bf16x8 as_frag(const u32x4 &u)
{
    union { u32x4 u; bf16x8 v; } f;
    f.u = u;
    return f.v;
}
// Elements 1..8 of the 16 elements (lo, hi).
__device__ __forceinline__ bf16x8 shifted_frag(const u32x4 &lo, const u32x4 &hi)
{
    u32x4 r;
    r[0] = __builtin_amdgcn_alignbit(lo[1], lo[0], 16);
    r[1] = __builtin_amdgcn_alignbit(lo[2], lo[1], 16);
    r[2] = __builtin_amdgcn_alignbit(lo[3], lo[2], 16);
    r[3] = __builtin_amdgcn_alignbit(hi[0], lo[3], 16);
    return as_frag(r);
}

constexpr int kMaxZ = 4;               // 16-byte Z items a thread moves per unit
constexpr uint32_t kNoByte = 0x80000000u; // buffer offset of a load that must return zeros

// SS: 8-column blocks per tile-sum row (1 or 2); PART: a unit is part of an image
template <int SS, bool PART>
__global__ void __launch_bounds__(512) dw_rk_kernel(DwRkParams p)
{
    constexpr int T = 9, NTM = 256, TILE_O = 32, TILE_C = 128;
    constexpr int SW = 8 * SS;                 // tile-sum row, elements
    constexpr uint32_t MAPB = SW * 2;          // bytes from one map of a row to the next
    constexpr uint32_t ROWB = 4 * SW * 2;      // bytes from one tile-sum row to the next
    constexpr bool NEXT = SS > 1;

    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t *sW = (bf16_t *)smem;
    const uint32_t tab_elems = p.LRZpad * 8;
    const uint32_t buf_elems = tab_elems + TILE_O * p.o_stride + TILE_C * p.c_stride;
    const uint32_t base0 = 8, base1 = base0 + buf_elems; // the buffers follow the zero block

    // XCD-aware numbering: each XCD works on consecutive (slice, o-tile, c-tile) triples
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= p.total_wg) return;
    const int ntiles = p.tiles_o * p.tiles_c;
    const int slice = v / ntiles, tile = v - slice * ntiles;
    const int ot = tile / p.tiles_c, ct = tile - ot * p.tiles_c;
    const int o0 = ot * TILE_O, c0 = ct * TILE_C;

    const int u_begin = slice * p.units_per_slice;
    const int u_end = min(u_begin + p.units_per_slice, p.nunits);
    const int nck = (u_end - u_begin + 1) >> 1; // chunks of this slice

    auto zero_fill = [&]() {
        u32x4 *l = (u32x4 *)smem;
        const uint32_t n16 = (8 + 2 * buf_elems) / 8;
        for (uint32_t i = threadIdx.x; i < n16; i += 2 * NTM) l[i] = u32x4{0, 0, 0, 0};
    };

    const int wave_id = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave_id >= NTM / 64) {
        // =========================== copy waves ===========================================
        const int tid = threadIdx.x - NTM;
        const int cw = __builtin_amdgcn_readfirstlane(tid >> 6);
        // ---- tile sums: one task per lane and unit = (output channel, tile-sum row, block)
        const uint32_t slot = tid & 7, s_o = tid >> 3;
        const uint32_t s_sr = slot >> p.segp2_log2, s_t = slot & ((1u << p.segp2_log2) - 1);
        const bool s_task = s_sr < (uint32_t)p.US && s_t < (uint32_t)SS;
        const uint32_t s_ni = fdiv(s_sr, p.m_pr1), s_e = s_sr - s_ni * (p.PRp + 1);
        // Dword k of a loaded row holds columns 16t-2+2k and the next one: inside the row or not as
        // a whole (Q is even).  The dword in front of a row's first block (columns -2, -1) is not
        // loaded at all; the others are cut with lane-constant masks where any lane needs it.
        u32x4 s_ma, s_mb;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            s_ma[k] = 16 * (int)s_t + 2 * k < p.Q ? 0xffffffffu : 0u;
            s_mb[k] = 16 * (int)s_t + 8 + 2 * k < p.Q ? 0xffffffffu : 0u;
        }
        const bool cut_a = p.Q < 16 * (SS - 1) + 8, cut_b = p.Q < 16 * SS; // (uniform)
        const uint32_t s_lds = tab_elems + s_o * p.o_stride + s_sr * (4 * SW) + s_t * 8;
        // A task owns the dY row pair (2e, 2e+1) of its unit-relative tile-sum row e and takes the
        // row above (2e-1) from the task of row e-1 -- the lane SEGP2 places below -- with a DPP
        // move; element offset of the pair's first row relative to the unit's first image and row pair
        const int s_rel = (((int)s_ni * p.K + o0 + (int)s_o) * p.P + 2 * (int)s_e) * p.Q + 16 * (int)s_t - 2;
        const int s_p = 2 * (int)s_e;                     // that row, relative to the unit's first row pair
        const int s_nmax = s_task ? p.N - (int)s_ni : 0;  // the unit's first image must lie below this
        // Units that are part of an image: the row above the unit's first pair belongs to no task of
        // the unit; the tasks of tile-sum row 0 load it themselves.
        constexpr bool partial = PART;
        const bool s_first = partial && s_task && s_e == 0;
        // ---- Z: LPCZ lanes share one input channel; item j = (Z row of the unit, block)
        const uint32_t zj = tid & ((1u << p.lpcz_log2) - 1), zc = tid >> p.lpcz_log2;
        const uint32_t z_zr = fdiv(zj, p.m_segs), z_t = zj - z_zr * p.SEGS;
        const uint32_t z_ni = fdiv(z_zr, p.m_pr), z_il = z_zr - z_ni * p.PRp;
        const bool z_item = zj < (uint32_t)p.z_items;
        const uint32_t z_cpp = (uint32_t)NTM >> p.lpcz_log2; // input channels per pass
        const uint32_t z_lds = tab_elems + TILE_O * p.o_stride + zc * p.c_stride + z_zr * p.ZW + z_t * 8;
        const bool z_odd = p.Wp & 1;
        u32x4 z_mask;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int l2 = p.Wp - (int)z_t * 8 - 2 * j;
            z_mask[j] = l2 >= 2 ? 0xffffffffu : (l2 == 1 ? 0xffffu : 0u);
        }
        const uint32_t z_rel = (((z_ni * p.C + c0 + zc) * p.Hp + z_il) * p.Wp) + z_t * 8;
        const uint32_t z_step = z_cpp * p.Hp * p.Wp;            // elements from one pass to the next
        const int z_nmax = z_item ? p.N - (int)z_ni : 0, z_imax = p.Hp - (int)z_il;
        const rsrc_t rs_dy = make_rsrc(p.dY, (uint32_t)p.N * p.K * p.P * p.Q * 2u);
        const rsrc_t rs_z = make_rsrc(p.Z, (uint32_t)p.N * p.C * p.Hp * p.Wp * 2u);

        // One set of copy registers: two dY rows of 18 elements (columns 16t-2 .. 16t+15: one
        // dword, then two 16-byte pieces; row 0 is the extra row above of a partial unit) and the
        // unit's Z items.
        struct Set {
            uint32_t h[3];
            u32x4 a[3], b[3];
            u32x4 z[kMaxZ];
            uint32_t zx[kMaxZ];
            uint32_t zsh; // bit i: item i starts on an odd element
        };
        // the 9th element of an item that starts on an odd element is only needed when the row goes on
        const bool z_tail = z_odd && p.Wp > 8;            // (uniform)
        // ---- global -> registers for one unit; every load is issued on every path (a lane or a
        // unit without work loads from beyond the tensors and gets zeros).  What depends on the
        // unit is uniform: its first image n0 and first pooled row i0.
        auto fetch = [&](int u, Set &s) {
            const int ig = fdiv(u, p.m_rb), rb = u - ig * p.RB;
            const int n0 = u < u_end ? ig * p.NBIu : p.N, i0 = rb * p.PRp; // (a unit past the end: no image is valid)
            const int ubase = (n0 * p.K * p.P + 2 * i0) * p.Q;              // (uniform)
            const bool n_ok = n0 < s_nmax;
            const int e0 = ubase + s_rel;
#pragma unroll
            for (int r = 1; r < 3; ++r) {
                const bool row_ok = n_ok && (uint32_t)(2 * i0 + s_p + r - 1) < (uint32_t)p.P;
                const uint32_t off = row_ok ? (uint32_t)(e0 + (r - 1) * p.Q) * 2u : kNoByte;
                // (the dword in front of a row's first block would be columns -2, -1: never loaded)
                if constexpr (SS > 1) s.h[r] = __builtin_amdgcn_raw_buffer_load_b32(rs_dy, s_t ? off : kNoByte, 0, 0);
                s.a[r] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, off + 4u, 0, 0);
                s.b[r] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, off + 20u, 0, 0);
            }
            if constexpr (partial) {
                const bool row_ok = n_ok && s_first && i0 > 0;
                const uint32_t off = row_ok ? (uint32_t)(e0 - p.Q) * 2u : kNoByte;
                if constexpr (SS > 1) s.h[0] = __builtin_amdgcn_raw_buffer_load_b32(rs_dy, s_t ? off : kNoByte, 0, 0);
                s.a[0] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, off + 4u, 0, 0);
                s.b[0] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, off + 20u, 0, 0);
            }
            const bool zok = n0 < z_nmax && i0 < z_imax;
            const uint32_t ez = (uint32_t)((n0 * p.C * p.Hp + i0) * p.Wp) + z_rel;
            s.zsh = 0;
#pragma unroll
            for (int i = 0; i < kMaxZ; ++i) {
                const uint32_t e = ez + i * z_step;
                const uint32_t off = (zok && i < p.z_passes) ? (e & ~1u) * 2u : kNoByte;
                s.z[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_z, off, 0, 0);
                if (z_tail) s.zx[i] = __builtin_amdgcn_raw_buffer_load_b32(rs_z, off + 16u, 0, 0);
                s.zsh |= (e & 1u) << i;
            }
        };
        // ---- registers -> LDS (unit `half` of the buffer at element offset `base`)
        auto stage = [&](int half, uint32_t base, const Set &s) {
            // tile sums.  Element m of a row (column 16t-2+m) as a float; m = 1..17 are used.
            // f1, f2: the task's own rows (2e, 2e+1).  The row above (2e-1) is the lower row of the
            // task SEGP2 lanes below: it comes in as the DPP operand of the add itself (zero where
            // that lane lies outside the 16-lane DPP row); the first tasks of a partial unit have
            // loaded it instead.
            float ra[18], rb[18]; // E pair sums (rows 2e, 2e+1) and O pair sums (rows 2e-1, 2e), per column
            auto above = [&](float lower) {
                const int v = __builtin_bit_cast(int, lower);
                return __builtin_bit_cast(float, SS > 1 ? __builtin_amdgcn_mov_dpp(v, 0x112, 0xf, 0xf, true)
                                                        : __builtin_amdgcn_mov_dpp(v, 0x111, 0xf, 0xf, true));
            };
#pragma unroll
            for (int k = SS > 1 ? 0 : 1; k < 9; ++k) {
                uint32_t w[3];
#pragma unroll
                for (int r = 1; r < 3; ++r) {
                    if (k == 0)
                        w[r] = s.h[r];
                    else if (k < 5)
                        w[r] = cut_a ? s.a[r][k - 1] & s_ma[k - 1] : s.a[r][k - 1];
                    else
                        w[r] = cut_b ? s.b[r][k - 5] & s_mb[k - 5] : s.b[r][k - 5];
                }
                const float h1 = __uint_as_float(w[1] & 0xffff0000u), h2 = __uint_as_float(w[2] & 0xffff0000u);
                const float l1 = __uint_as_float(w[1] << 16), l2 = __uint_as_float(w[2] << 16);
                float h0 = above(h2), l0 = above(l2);
                if constexpr (partial) {
                    const uint32_t x = k == 0 ? s.h[0] : k < 5 ? s.a[0][k - 1] & s_ma[k - 1] : s.b[0][k - 5] & s_mb[k - 5];
                    h0 = s_first ? __uint_as_float(x & 0xffff0000u) : h0;
                    l0 = s_first ? __uint_as_float(x << 16) : l0;
                }
                rb[2 * k + 1] = h0 + h1;
                ra[2 * k + 1] = h1 + h2;
                if (k > 0) { // (element 0 is not used)
                    rb[2 * k] = l0 + l1;
                    ra[2 * k] = l1 + l2;
                }
            }
            if constexpr (SS == 1) ra[1] = rb[1] = 0.f; // (column -1)
            if (s_task) {
                bf16_t *d = sW + base + s_lds + half * (p.US * 4 * SW);
                u32x4 m0, m1, m2, m3;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // E columns: elements (2+4j, 3+4j) and (4+4j, 5+4j); O columns: (1+4j, 2+4j) and (3+4j, 4+4j)
                    m0[j] = f32x2_to_bf16x2(ra[2 + 4 * j] + ra[3 + 4 * j], ra[4 + 4 * j] + ra[5 + 4 * j]);
                    m1[j] = f32x2_to_bf16x2(ra[1 + 4 * j] + ra[2 + 4 * j], ra[3 + 4 * j] + ra[4 + 4 * j]);
                    m2[j] = f32x2_to_bf16x2(rb[2 + 4 * j] + rb[3 + 4 * j], rb[4 + 4 * j] + rb[5 + 4 * j]);
                    m3[j] = f32x2_to_bf16x2(rb[1 + 4 * j] + rb[2 + 4 * j], rb[3 + 4 * j] + rb[4 + 4 * j]);
                }
                *(u32x4 *)(d) = m0;
                *(u32x4 *)(d + SW) = m1;
                *(u32x4 *)(d + 2 * SW) = m2;
                *(u32x4 *)(d + 3 * SW) = m3;
            }
            // Z: one element down after an odd start (rows of odd length), cut at the row's end
            if (z_item) {
                bf16_t *zd = sW + base + z_lds + half * (p.UZ * p.ZW);
#pragma unroll
                for (int i = 0; i < kMaxZ; ++i) {
                    if (i < p.z_passes) {
                        u32x4 x = s.z[i];
                        if (z_odd) {
                            const uint32_t sh = ((s.zsh >> i) & 1u) * 16u;
                            x[0] = __builtin_amdgcn_alignbit(s.z[i][1], s.z[i][0], sh);
                            x[1] = __builtin_amdgcn_alignbit(s.z[i][2], s.z[i][1], sh);
                            x[2] = __builtin_amdgcn_alignbit(s.z[i][3], s.z[i][2], sh);
                            x[3] = __builtin_amdgcn_alignbit(z_tail ? s.zx[i] : 0u, s.z[i][3], sh);
                        }
                        *(u32x4 *)(zd + i * z_cpp * p.c_stride) = x & z_mask;
                    }
                }
            }
        };
        // ---- row table of the chunk whose first unit is u: entry rho = {Z row offset, tile-sum
        // row offset} in bytes from the lane's channel base; rows that do not exist point at the
        // all-zero Z row
        struct Unit { int n0, i0; bool live; };
        auto unit_of = [&](int u) {
            Unit t;
            const int ig = fdiv(u, p.m_rb), rb = u - ig * p.RB;
            t.n0 = ig * p.NBIu;
            t.i0 = rb * p.PRp;
            t.live = u < u_end;
            return t;
        };
        auto stage_table = [&](int u, uint32_t base) {
            if (cw == 0 && tid < p.LRZpad) {
                const uint32_t rho = tid;
                const uint32_t h = rho >= (uint32_t)p.UZ ? 1u : 0u, zr = rho - h * p.UZ;
                const uint32_t ni = fdiv(zr, p.m_pr), il = zr - ni * p.PRp;
                const Unit t = unit_of(u + (int)h);
                const bool ok = t.live && t.n0 + (int)ni < p.N && t.i0 + (int)il < p.Hp;
                u32x4 e = {ok ? rho * p.ZW * 2u : (uint32_t)p.LRZpad * p.ZW * 2u,
                           ok ? (h * p.US + ni * (p.PRp + 1) + il) * ROWB : 0u, 0u, 0u};
                *(u32x4 *)(sW + base + rho * 8) = e;
            }
        };

        Set A, B;
        fetch(u_begin, A); // (every workgroup has at least one unit)
        fetch(u_begin + 1, B);
        zero_fill();
        __syncthreads();
        stage_table(u_begin, base0);
        stage(0, base0, A);
        fetch(u_begin + 2, A);
        stage(1, base0, B);
        fetch(u_begin + 3, B);
        __syncthreads(); // buffer 0 holds the first chunk
        for (int ck = 0; ck < nck; ck += 2) {
            // MFMA waves are on buffer 0 (chunk ck); the sets hold chunk ck+1.  A chunk past the
            // end is staged all the same (zeros into a buffer nobody reads any more).
            const int u1 = u_begin + 2 * (ck + 1);
            stage_table(u1, base1);
            stage(0, base1, A);
            fetch(u1 + 2, A);
            stage(1, base1, B);
            fetch(u1 + 3, B);
            __syncthreads();
            if (ck + 1 >= nck) break;
            // MFMA waves are on buffer 1 (chunk ck+1); the sets hold chunk ck+2
            const int u2 = u1 + 2;
            stage_table(u2, base0);
            stage(0, base0, A);
            fetch(u2 + 2, A);
            stage(1, base0, B);
            fetch(u2 + 3, B);
            __syncthreads();
        }
        return;
    }

    // =============================== MFMA waves ===========================================
    const int lane = threadIdx.x & 63, wn = wave_id, half = lane >> 5, l32 = lane & 31;

    zero_fill();
    __syncthreads();

    f32x16 acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][j] = 0.f;

    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    // Operands of one step (one block of two pooled rows): the Z block and, for the three row
    // kinds (E rows; O rows one down; O rows), the E-column block and the O-column block with
    // its right-hand neighbour.
    struct Ops {
        u32x4 z;
        u32x4 e[3], o0[3], o1[3];
    };
    auto request = [&](Ops &x, uint32_t za, uint32_t sa, int seg) {
        x.z = lds16(za + 16 * seg);
        const uint32_t a = sa + 16 * seg;
        // row kind 0: E rows (r = 1); 1: O rows, one row down (r = 0); 2: O rows (r = 2)
        x.e[0] = lds16(a);
        x.o0[0] = lds16(a + MAPB);
        x.e[1] = lds16(a + ROWB + 2 * MAPB);
        x.o0[1] = lds16(a + ROWB + 3 * MAPB);
        x.e[2] = lds16(a + 2 * MAPB);
        x.o0[2] = lds16(a + 3 * MAPB);
        if constexpr (NEXT) {
            // the block to the right; beyond the last one lies nothing: the zero block at LDS offset 0
            const bool last = seg + 1 >= SS;
            x.o1[0] = lds16(last ? lds0 : a + MAPB + 16);
            x.o1[1] = lds16(last ? lds0 : a + ROWB + 3 * MAPB + 16);
            x.o1[2] = lds16(last ? lds0 : a + 3 * MAPB + 16);
        } else {
#pragma unroll
            for (int k = 0; k < 3; ++k) x.o1[k] = u32x4{0, 0, 0, 0};
        }
    };
    auto mfma_step = [&](const Ops &x) {
        const bf16x8 zf = as_frag(x.z);
        // filter row of row kind k: 1, 0, 2
#define CAC_RK_ROW(k, r)                                                                                            \
    acc[r * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(x.e[k]), zf, acc[r * 3 + 1], 0, 0, 0);         \
    acc[r * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(x.o0[k]), zf, acc[r * 3 + 2], 0, 0, 0);        \
    acc[r * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(shifted_frag(x.o0[k], x.o1[k]), zf, acc[r * 3 + 0], 0, 0, 0);
        CAC_RK_ROW(0, 1) CAC_RK_ROW(1, 0) CAC_RK_ROW(2, 2)
#undef CAC_RK_ROW
    };
    auto interleave = [&]() {
        constexpr int kReads = NEXT ? 11 : 8, kPer = NEXT ? 2 : 1;
#pragma unroll
        for (int i = 0; i < T; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                            // MFMA
            if (i * kPer < kReads) __builtin_amdgcn_sched_group_barrier(0x100, kPer, 0);  // DS read
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);                            // VALU
        }
    };
    auto compute = [&](uint32_t base) {
        const uint32_t tab = lds0 + 2 * base + half * 16;
        const uint32_t oc = lds0 + 2 * (base + tab_elems + l32 * p.o_stride);
        const uint32_t zc = lds0 + 2 * (base + tab_elems + TILE_O * p.o_stride + (wn * 32 + l32) * p.c_stride);
        const int nrp = p.LRZpad / 2, segs = p.SEGS;
        const int nsteps = nrp * segs;
        u32x4 e = lds16(tab);
        uint32_t za = zc + e[0], sa = oc + e[1];
        u32x4 e_next = lds16(tab + 32 * min(1, nrp - 1));
        Ops X, Y;
        request(X, za, sa, 0);
        int seg = 0, rp = 0;
#define CAC_RK_STEP(USE, GET)                                        \
    if (seg + 1 < segs) {                                            \
        ++seg;                                                       \
    } else {                                                         \
        za = zc + e_next[0];                                         \
        sa = oc + e_next[1];                                         \
        ++rp;                                                        \
        e_next = lds16(tab + 32 * min(rp + 1, nrp - 1));             \
        seg = 0;                                                     \
    }                                                                \
    request(GET, za, sa, seg);                                       \
    mfma_step(USE);                                                  \
    interleave();
        for (int t = 0;;) {
            CAC_RK_STEP(X, Y)
            if (++t == nsteps) break;
            CAC_RK_STEP(Y, X)
            if (++t == nsteps) break;
        }
#undef CAC_RK_STEP
    };

    __syncthreads(); // buffer 0 holds the first chunk
    for (int ck = 0; ck < nck; ck += 2) {
        compute(base0);
        __syncthreads();
        if (ck + 1 >= nck) break;
        compute(base1);
        __syncthreads();
    }

    // ---- epilogue --------------------------------------------------------------------
    // accumulator register j of lane l holds row 8*(j/4) + 4*(l/32) + j%4 (o), column l%32 (c).
    // Output: dW itself (one slice), or this slice's partial sums in the workspace, in the same
    // [o][c][tap] order, so that the sum over the slices is a plain stream.
    float *out = p.direct ? p.out : p.out + (long)slice * p.K * p.C * T;
    const bool inside = o0 + TILE_O <= p.K && c0 + TILE_C <= p.C;
    // A tile inside dW whose rows are a multiple of 16 bytes: 8 output channels x 32 input
    // channels x 9 taps are 8 contiguous runs of 1152 bytes.  They go through a wave-private 9 KB
    // of LDS (the staging buffers are dead: the loop ends with a barrier), [row][c][tap], and
    // leave as 16-byte stores in which the lanes of a wave cover whole runs.
    const bool runs16 = inside && (p.C & 3) == 0;
    float *tb = (float *)smem + wn * (8 * 32 * 9);
#pragma unroll
    for (int jq = 0; jq < 4; ++jq) {
        f32x4 val[T];
#pragma unroll
        for (int t = 0; t < T; ++t) val[t] = f32x4{acc[t][4 * jq], acc[t][4 * jq + 1], acc[t][4 * jq + 2], acc[t][4 * jq + 3]};
        if (runs16) {
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) tb[half * 1152 + l32 * 9 + e * 288 + t] = val[t][e];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            const long row0 = (long)(o0 + 8 * jq) * p.C + c0 + wn * 32;
#pragma unroll
            for (int k = 0; k < 9; ++k) {
                const int q4 = k * 64 + lane, rr = q4 / 72, w4 = q4 - rr * 72; // row, 16-byte unit of its run
                *(f32x4 *)(out + (row0 + (long)rr * p.C) * 9 + 4 * w4) = ((const f32x4 *)tb)[q4];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            continue;
        }
        const int c = c0 + wn * 32 + l32;
        const int ob = o0 + 8 * jq + 4 * half;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (ob + e < p.K && c < p.C) {
                float *d = out + ((long)(ob + e) * p.C + c) * T;
#pragma unroll
                for (int t = 0; t < T; ++t) d[t] = val[t][e];
            }
        }
    }
}

uint32_t magic_of(uint32_t d) { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }

template <int SS, bool PART> hipError_t launch_ss(const DwRkParams &p, dim3 grid, hipStream_t st)
{
    auto kern = dw_rk_kernel<SS, PART>;
    // (per instantiation; once per process, whichever host thread comes first)
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [&] { attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024); });
    if (attr_err != hipSuccess) return attr_err;
    hipLaunchKernelGGL(kern, grid, dim3(512), p.lds_bytes, st, p);
    return hipGetLastError();
}

} // namespace

bool dw_rk_plan(const Geom &g, int dtype, DwRkPlan *plan)
{
    if (dtype != CAC_BF16) return false;
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1) return false;
    if (g.kh != 2 || g.kw != 2) return false;
    if ((g.H & 1) || (g.W & 1)) return false; // a ragged last tile needs other sums for r = 0 than for r = 2
    if (g.C < 96 || g.K < 16) return false;   // the 32 x 128 tile would be mostly padding
    if ((long)g.N * g.K * g.P * g.Q >= (1L << 29) || (long)g.N * g.C * g.Hp * g.Wp >= (1L << 29)) return false;

    DwRkParams p{};
    p.N = g.N; p.C = g.C; p.K = g.K; p.P = g.P; p.Q = g.Q; p.Hp = g.Hp; p.Wp = g.Wp;
    p.SEGS = (g.Wp + 7) / 8;
    p.SEGS_S = (g.Wp + 1 + 7) / 8;
    if (p.SEGS_S > 2) return false;
    p.segp2_log2 = p.SEGS_S == 1 ? 0 : 1;
    const int segp2 = 1 << p.segp2_log2;
    p.ZW = 8 * p.SEGS;
    p.SW = 8 * p.SEGS_S;
    // unit: 8 tile-sum tasks per output channel, at most 8 Z items per input channel
    if ((g.Hp + 1) * segp2 <= 8) {
        p.PRp = g.Hp;
        p.NBIu = 8 / ((g.Hp + 1) * segp2);
        while (p.NBIu > 1 && p.NBIu * g.Hp * p.SEGS > 8) --p.NBIu;
        p.NBIu = min(p.NBIu, g.N);
    } else {
        p.NBIu = 1;
        p.PRp = 8 / segp2 - 1;
    }
    if (p.PRp < 1 || p.NBIu * p.PRp * p.SEGS > 8) return false;
    p.RB = (g.Hp + p.PRp - 1) / p.PRp;
    p.UZ = p.NBIu * p.PRp;
    p.US = p.NBIu * (p.PRp + 1);
    if (p.US * segp2 > 8) return false;
    p.LRZpad = 2 * p.UZ;
    p.z_items = p.UZ * p.SEGS;
    p.lpcz_log2 = 1;
    while ((1 << p.lpcz_log2) < p.z_items) ++p.lpcz_log2;
    p.z_passes = (128 << p.lpcz_log2) / 256;
    if (p.z_passes > kMaxZ) return false;
    // strides: an odd number of 16-byte units, so that the 32 lanes of a half wave (one channel
    // each) read distinct LDS banks
    p.o_stride = 8 * ((2 * p.US * 4 * p.SEGS_S) | 1);
    p.c_stride = 8 * (((p.LRZpad + 1) * p.SEGS) | 1); // + the all-zero row
    p.map_stride = p.SW;
    p.lds_bytes = (8 + 2 * (p.LRZpad * 8 + 32 * p.o_stride + 128 * p.c_stride)) * 2;
    if (p.lds_bytes > 158 * 1024) return false;
    p.lds_bytes = max(p.lds_bytes, 4 * 8 * 32 * 9 * 4); // the epilogue's transpose (9 KB per wave)
    p.m_pr1 = magic_of(p.PRp + 1);
    p.m_pr = magic_of(p.PRp);
    p.m_segs = magic_of(p.SEGS);
    p.m_rb = magic_of(p.RB);

    p.tiles_o = (g.K + 31) / 32;
    p.tiles_c = (g.C + 127) / 128;
    const int ntiles = p.tiles_o * p.tiles_c;
    p.nunits = ((g.N + p.NBIu - 1) / p.NBIu) * p.RB;
    const int nchunks = (p.nunits + 1) / 2;
    int want = max(1, 256 / ntiles);              // one workgroup per compute unit ...
    want = min(want, max(1, nchunks / 2));        // ... each with at least two chunks
    p.units_per_slice = 2 * ((nchunks + want - 1) / want);
    p.nslices = (p.nunits + p.units_per_slice - 1) / p.units_per_slice;
    p.total_wg = p.nslices * ntiles;
    p.direct = p.nslices == 1;
    plan->p = p;
    plan->grid = ((p.total_wg + 7) / 8) * 8;
    plan->partial_bytes = p.direct ? 0 : (size_t)p.nslices * g.K * g.C * 9 * sizeof(float);
    plan->next = p.SEGS_S > 1;
    plan->executed_flops = 2ull * 9 * g.K * g.C * (uint64_t)g.N * g.Hp * g.Wp;
    return true;
}

hipError_t launch_dw_rk(const DwRkPlan &plan, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                        DwReduceTail *defer)
{
    DwRkParams p = plan.p;
    p.Z = (const bf16_t *)Z;
    p.dY = (const bf16_t *)dY;
    p.out = p.direct ? dW : (float *)ws;
    if (defer) defer->blocks = 0;
    const bool part = p.PRp < p.Hp;
    hipError_t e = p.SEGS_S == 1 ? (part ? launch_ss<1, true>(p, dim3(plan.grid), st) : launch_ss<1, false>(p, dim3(plan.grid), st))
                                 : (part ? launch_ss<2, true>(p, dim3(plan.grid), st) : launch_ss<2, false>(p, dim3(plan.grid), st));
    if (e != hipSuccess || p.direct) return e;
    const DwReduceTail t = make_reduce_tail((const float *)ws, dW, (long)p.K * p.C * 9, p.nslices);
    if (defer) {
        *defer = t;
        return hipSuccess;
    }
    return launch_dw_reduce(t, st);
}

} // namespace cac
