// Block-level W4A8 contraction for the compute-bound shapes (many activation
// rows): 256 threads = 2 x 2 waves, each wave owns MT x NT 16x16 MFMA tiles, so a
// block covers BM = 32*MT weight rows x BN = 32*NT activation rows.
//
//  - Weights never touch LDS: the TILED blob is already in operand order, each
//    wave streams its own row tiles with one 128-bit load per lane per 128
//    columns and unpacks them in registers (qr_unpack), reusing every fragment
//    for NT column tiles.
//  - Activations are shared by the two waves of a block column, so a block stages
//    its BN x 128-byte activation panel in LDS (double buffered, rows padded to
//    144 bytes so that 128-bit reads of 8 consecutive rows hit distinct banks).
//  - The next panel and the next weight fragments are fetched while the current
//    chunk's MFMAs run; one barrier per 128-column chunk.
#pragma once

#include "qrnnt_common.h"

#define QR_LDS_ROW 144   // bytes per staged activation row (128 + 16 padding)

template <int MT, int NT>
struct QrBlockTile {
    static constexpr int BM = 32 * MT;          // weight rows per block
    static constexpr int BN = 32 * NT;          // activation rows per block
    static constexpr int ROWS_PER_PASS = 32;    // 256 threads x 16 B = 32 rows of 128 B
    static constexpr int PASSES = BN / ROWS_PER_PASS;
    static constexpr int STAGE_BYTES = BN * QR_LDS_ROW;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

// rowptr[i]: global address of the activation row this thread stages in pass i
// (already offset by the thread's 16-byte segment), K: valid columns.
// acc[mt][nt] accumulates 16x the true sums.
template <int MT, int NT>
__device__ __forceinline__ void qr_block_mma(const v4i *__restrict__ wblk, int nkc, int n_row_tiles, int rt0,
                                             const int8_t *const (&rowptr)[QrBlockTile<MT, NT>::PASSES], int K,
                                             char *lds, int wn, v4i (&acc)[MT][NT])
{
    using Cfg = QrBlockTile<MT, NT>;
    const int tid = threadIdx.x, lane = tid & 63;
    const int col = lane & 15, grp = lane >> 4;
    const int seg = tid & 7, srow = tid >> 3;
    const v4i zero = {0, 0, 0, 0};

    const v4i *wrow[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int rt = rt0 + mt;
        rt = rt < n_row_tiles ? rt : n_row_tiles - 1;
        wrow[mt] = wblk + (size_t)rt * nkc * 64 + lane;
    }
    char *st_base = lds + srow * QR_LDS_ROW + seg * 16;                       // where this thread stores
    const char *ld_base = lds + (wn * NT * 16 + col) * QR_LDS_ROW + grp * 16; // where this lane reads tile 0

    v4i pa[MT], pb[Cfg::PASSES];
    // prologue: chunk 0
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) pa[mt] = wrow[mt][0];
#pragma unroll
    for (int i = 0; i < Cfg::PASSES; ++i) pb[i] = (seg * 16 < K) ? *(const v4i *)(rowptr[i]) : zero;
#pragma unroll
    for (int i = 0; i < Cfg::PASSES; ++i) *(v4i *)(st_base + i * Cfg::ROWS_PER_PASS * QR_LDS_ROW) = pb[i];
    __syncthreads();

    for (int kc = 0; kc < nkc; ++kc) {
        const int cur = kc & 1;
        const bool more = kc + 1 < nkc;
        v4i na[MT];
        if (more) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) na[mt] = wrow[mt][(size_t)(kc + 1) * 64];
            const int k0 = (kc + 1) * QRNNT_KCHUNK + seg * 16;
#pragma unroll
            for (int i = 0; i < Cfg::PASSES; ++i)
                pb[i] = (k0 < K) ? *(const v4i *)(rowptr[i] + (kc + 1) * QRNNT_KCHUNK) : zero;
        }
        const char *rb = ld_base + cur * Cfg::STAGE_BYTES;
        v4i b0[NT], b1[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            b0[nt] = *(const v4i *)(rb + nt * 16 * QR_LDS_ROW);
            b1[nt] = *(const v4i *)(rb + nt * 16 * QR_LDS_ROW + 64);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            v4i lo, hi;
            qr_unpack(pa[mt], lo, hi);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                acc[mt][nt] = qr_mfma(lo, b0[nt], acc[mt][nt]);
                acc[mt][nt] = qr_mfma(hi, b1[nt], acc[mt][nt]);
            }
        }
        if (more) {
            char *wb = st_base + (cur ^ 1) * Cfg::STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < Cfg::PASSES; ++i) *(v4i *)(wb + i * Cfg::ROWS_PER_PASS * QR_LDS_ROW) = pb[i];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) pa[mt] = na[mt];
        }
        __syncthreads();
    }
}
