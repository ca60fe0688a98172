// Forward convolution / data gradient as an MFMA gather GEMM (see conv_mfma.hip).
#pragma once
#include "common.h"
#include "dw_reduce.h"

namespace cac {

struct GatherParams {
    const bf16_t *in;   // [N][Hin][Win][KCp], channels last; with nchw: the caller's tensor itself, [N][KCin][Hin][Win]
    const bf16_t *wt;   // [ntaps_total][KCp/16][Mp/32][64][8], MFMA fragment order
    const bf16_t *bias; // [M] or null
    bf16_t *out;        // [N][M][Hout][Wout]
    float *part;        // [ksplit][N][M][Hout*Wout] float sums when the channels are shared out, else null
    int N, M, Mp, KCp;
    int Hin, Win, Hout, Wout;
    int Hc, Wc;         // grid of output pixels of this launch: (h, w) = (i*os + a0, j*os + b0)
    int os, a0, b0, is; // input pixel of tap t: (i*is + dh[t], j*is + dw[t])
    int ntaps, ntaps_total;
    int dh[9], dw[9], wtap[9];
    int dhmin, dwmin;
    int PH, PWd;        // input patch of one image staged per workgroup (rows, columns)
    int IPT, patch_px;  // images per pixel tile; patch pixels of the whole tile
    int tiles_per_img, ngrp, gpw, nkb; // tiles per image; image groups; groups per workgroup; channel blocks
    int ksplit, kbs;    // workgroups sharing one tile's channel blocks (grid z); channel blocks of each
    int T, t_log2, kcs; // 32-channel groups staged per pass (1, 2 or 4; more than one only where taps * T is 4 or 8);
                        // LDS elements per patch pixel (32 * T + 8); a "channel block" above is 32 * T channels
    int nchw, KCin;     // the kernel reads the input in its own layout (KCin channels) instead of a channels-last copy
    int wide_store;     // the epilogue writes 16-byte runs of 8 pixels (whole planes, a multiple of 8 pixels each)
    int decim;          // forward, 1 x 1 filter, stride 2: `in` holds only the pixels the filter reaches (every second
                        // one of every second row), as an image of half the extent read with stride 1
    uint32_t m_wc, m_ppi, m_pwd, m_kbs, m_img; // division magics of Wc, Hc*Wc, PWd, kbs, PH*PWd
    uint32_t m_gx, m_ph;                       // ... of the 8-pixel groups of an input row and of PH (in-place copy)
};

size_t conv_mfma_workspace(const Geom &g, int dtype, bool data_grad);
// Text description of the launch shape(s) chosen; false when the geometry is not covered.
bool describe_conv_mfma(const Geom &g, int dtype, bool data_grad, char *buf, size_t len);
bool launch_fwd_mfma(const Geom &g, int dtype, const void *X, const void *W, const void *b, void *Y, void *Z, void *ws,
                     hipStream_t st, hipError_t *err, bool *pooled);
bool launch_dx_mfma(const Geom &g, int dtype, const void *W, const void *dY, void *dX, void *ws, hipStream_t st,
                    hipError_t *err, const DwReduceTail *tail = nullptr);

} // namespace cac
