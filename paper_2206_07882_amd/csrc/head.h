// Split-K contraction for "head" layers: few weight rows (a block owns 64 of them),
// 16 activation rows per block, the 64-column K blocks dealt round-robin to the 4
// waves, partial sums reduced through LDS into wave 0.  All loads of a wave are
// issued before its first MFMA, so a block exposes one memory latency.
#pragma once

#include "qrnnt_common.h"

#define QR_HEAD_BATCH 4   // K blocks per wave per batch (registers: 4 x (4+1) fragments)

// bload(kb) issues the loads of this lane's 16 activation values of K block kb and returns them raw;
// bmake(raw, kb) turns them into the 16 codes (zero beyond K).  after_issue() runs once, after the first
// batch of loads has been issued and before anything waits for it: the place for loads that only the
// caller's epilogue needs (issued earlier they would sit in front of the operands in the in-order
// memory counter and the contraction would wait for them too).
// w8 (uniform): the weights are 8-bit (two blocks per chunk, operands as stored).
template <int BATCH, class BLoad, class BMake, class AfterIssue>
__device__ __forceinline__ void qr_head_mma(const v4i *__restrict__ w, int nkc, int n_row_tiles, int rt0, int K,
                                            BLoad &&bload, BMake &&bmake, AfterIssue &&after_issue, v4i (&acc)[4],
                                            v4i *lds /* [4][4][64] */, bool w8 = false)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: MFMAs below sit under wave-uniform branches
    const int nkb = (K + 63) >> 6;
    const v4i zero = {0, 0, 0, 0};
    const int m = (int)0xF0F0F0F0u;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt] = zero;
    for (int kb0 = wave; kb0 == wave || kb0 < nkb; kb0 += 4 * BATCH) {   // at least once: after_issue must run
        v4i pa[BATCH][4], pb[BATCH];
        decltype(bload(0)) raw[BATCH];
#pragma unroll
        for (int it = 0; it < BATCH; ++it) {
            const int kb = kb0 + 4 * it;
            const bool ok = kb < nkb;
            const int kc = ok ? (kb >> 1) : 0;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                int rt = rt0 + mt;
                rt = rt < n_row_tiles ? rt : n_row_tiles - 1;
                pa[it][mt] = w8 ? w[(((size_t)rt * nkc + kc) * 2 + (kb & 1)) * 64 + lane] : w[((size_t)rt * nkc + kc) * 64 + lane];
            }
            raw[it] = bload(ok ? kb : 0);
        }
        if (kb0 == wave) after_issue();
#pragma unroll
        for (int it = 0; it < BATCH; ++it) {
            const int kb = kb0 + 4 * it;
            pb[it] = kb < nkb ? bmake(raw[it], kb) : zero;
        }
#pragma unroll
        for (int it = 0; it < BATCH; ++it) {
            const int kb = kb0 + 4 * it;
            if (kb < nkb) {
                const bool hi = kb & 1;
#pragma unroll
                for (int mt = 0; mt < 4; ++mt) {
                    const v4i a = w8 ? pa[it][mt] : (hi ? (pa[it][mt] & m) : ((pa[it][mt] << 4) & m));
                    acc[mt] = qr_mfma(a, pb[it], acc[mt]);
                }
            }
        }
    }
    // reduce the four partial sums into wave 0
    if (wave != 0) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) lds[(wave * 4 + mt) * 64 + lane] = acc[mt];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int wv = 1; wv < 4; ++wv)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) acc[mt] += lds[(wv * 4 + mt) * 64 + lane];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) acc[mt] = w8 ? acc[mt] : (acc[mt] >> 4);   // 4-bit operands carry a factor 16
    }
}
