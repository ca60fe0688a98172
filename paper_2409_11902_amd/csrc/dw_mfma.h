// Launch plan of the MFMA weight-gradient kernel (see dw_mfma.hip).
#pragma once
#include "common.h"
#include "dw_reduce.h"

namespace cac {

struct DwMfmaParams {
    const bf16_t *Z;
    const bf16_t *dY;
    float *out; // dW (direct) or the partial-sum workspace
    int N, C, K, H, W, P, Q, Hp, Wp;
    int kh_log2, kw_log2;
    // chunk = NBI images x PR output rows
    int NBI, PR, RB;     // RB = row blocks per image
    int LR, LRpad;       // rows per chunk, rounded up to even
    int SEGS, Qpad;      // 8-pixel segments per output row
    int NZ;              // Z-row slots per image and chunk
    int XW, PW;          // LDS width of an xhat row (all phases) and of one phase
    int ZV;              // 4-element vectors per Z row
    int rowitems, citems;         // 16-byte dY items per output channel; 8-byte Z items per input channel
    int LDY, ldy_log2, dy_passes; // lanes sharing an output channel in the dY copy; passes per chunk
    int LPC, lpc_log2, z_passes;  // same for the Z copy
    int dy_ostride, x_cstride;    // LDS elements per output channel / per input channel
    int dy_direct;       // dY can go from global memory straight into LDS (see the kernel)
    int lds_bytes;
    uint32_t m_segs, m_pr, m_zv, m_nz, m_rb;
    int nchunks, chunks_per_slice, nslices;
    int tile_o, tile_c;  // workgroup tile
    int tiles_o, tiles_c, total_wg;
    int direct;
};

struct DwMfmaPlan {
    DwMfmaParams p;
    unsigned grid, threads;
    size_t partial_bytes;
    int variant;        // index into the kernel table
};

// False when the geometry is not covered (the caller then uses the generic kernel).
bool dw_mfma_plan(const Geom &g, int dtype, DwMfmaPlan *plan);
hipError_t launch_dw_mfma(const DwMfmaPlan &plan, const void *Z, const void *dY, float *dW, void *ws, hipStream_t st,
                          DwReduceTail *defer = nullptr);

} // namespace cac
