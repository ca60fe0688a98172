// Launch plan of the reduced-K weight-gradient kernel (see dw_rk.hip).
#pragma once
#include "common.h"
#include "dw_reduce.h"

namespace cac {

struct DwRkParams {
    const bf16_t *Z;
    const bf16_t *dY;
    float *out; // dW (direct) or the partial-sum workspace
    int N, C, K, P, Q, Hp, Wp;
    // unit = NBIu images x PRp pooled rows (what one set of copy registers holds); chunk = 2 units
    int NBIu, PRp, RB;          // RB = row blocks per image
    int UZ, US;                 // Z rows / tile-sum rows per unit
    int LRZpad;                 // Z rows per chunk (2 * UZ, even)
    int SEGS, SEGS_S;           // 8-column blocks per Z row / per tile-sum row
    int segp2_log2;             // log2 of SEGS_S rounded up to a power of two
    int ZW, SW;                 // LDS width of a Z row / of a tile-sum row, elements
    int map_stride;             // LDS elements of one of the four tile-sum maps of an output channel
    int o_stride, c_stride;     // LDS elements per output channel / per input channel
    int lpcz_log2, z_items, z_passes; // lanes per input channel in the Z copy, 16-byte items per channel and unit
    uint32_t m_pr1, m_pr, m_segs, m_rb;
    int nunits, units_per_slice, nslices;
    int tiles_o, tiles_c, total_wg;
    int direct;
    int lds_bytes;
};

struct DwRkPlan {
    DwRkParams p;
    unsigned grid;
    size_t partial_bytes;
    int next;                   // kernel variant: tile-sum rows wider than one block
    uint64_t executed_flops;    // 2 x multiply-adds over real pooled pixels
};

// False when the geometry is not covered (the caller then uses the inflating kernel).
bool dw_rk_plan(const Geom &g, int dtype, DwRkPlan *plan);
hipError_t launch_dw_rk(const DwRkPlan &plan, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                        DwReduceTail *defer = nullptr);

} // namespace cac
