// Launch plan of the LDS-tiled float weight-gradient kernel (see dw_tiled.hip).
#pragma once
#include "common.h"
#include "dw_reduce.h"

namespace cac {

struct DwTiledParams {
    const void *Z;
    const void *dY;
    float *out;          // dW (direct) or the partial-sum workspace
    Geom g;
    int PR, RB;          // output rows per unit; units per image
    int XR;              // input rows a unit meets
    int QW, XW;          // LDS widths of a dY row and of an input row, floats (multiples of 4)
    int dy_stride, x_stride; // LDS floats per output channel / per input channel
    int nunits, units_per_slice, nslices;
    int tiles_o, tiles_c;
    int direct;
    int lds_bytes;
    uint32_t m_rb, m_kh, m_kw, m_qw, m_pr, m_xw, m_xr;
};

struct DwTiledPlan {
    DwTiledParams p;
    unsigned grid;
    size_t partial_bytes;
};

// False when the geometry is not covered (the caller then uses the plain kernel).
bool dw_tiled_plan(const Geom &g, int dtype, DwTiledPlan *plan);
hipError_t launch_dw_tiled(const DwTiledPlan &plan, int dtype, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                           DwReduceTail *defer = nullptr);

} // namespace cac
