// Wave-level W4A8 contraction on the int8 MFMA units (gfx950).
//
// A wavefront owns MT row tiles (16 weight rows each) times NT column tiles (16
// activation rows each).  Weights come from the TILED blob: one 128-bit load per
// lane per (row tile, 128-column chunk), split by qr_unpack into the operands of
// two MFMAs.  Activations are int8 rows in memory; lane l reads the 16 bytes of
// activation row (tile base + l%16) at column 16*(l/16) of each 64-column half.
// Accumulators hold 16x the true sums (see qr_unpack).
#pragma once

#include "qrnnt_common.h"

template <int MT, int NT>
__device__ __forceinline__ void qr_mma_range(const v4i *__restrict__ wblk, int nkc, int n_row_tiles, int rt0, int lane,
                                             const int8_t *const (&aptr)[NT], int K, v4i (&acc)[MT][NT])
{
    const int grp = lane >> 4;
    const v4i zero = {0, 0, 0, 0};
    const v4i *wrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int rt = rt0 + mt;
        rt = rt < n_row_tiles ? rt : n_row_tiles - 1;
        wrow[mt] = wblk + (size_t)rt * nkc * 64 + lane;
    }

    for (int kc = 0; kc < nkc; ++kc) {
        v4i p[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) p[mt] = wrow[mt][(size_t)kc * 64];
        const int k0 = kc * QRNNT_KCHUNK + grp * 16;
        v4i b0[NT], b1[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            b0[nt] = (k0 < K) ? *(const v4i *)(aptr[nt] + kc * QRNNT_KCHUNK) : zero;
            b1[nt] = (k0 + 64 < K) ? *(const v4i *)(aptr[nt] + kc * QRNNT_KCHUNK + 64) : zero;
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            v4i lo, hi;
            qr_unpack(p[mt], lo, hi);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                acc[mt][nt] = qr_mfma(lo, b0[nt], acc[mt][nt]);
                acc[mt][nt] = qr_mfma(hi, b1[nt], acc[mt][nt]);
            }
        }
    }
}
