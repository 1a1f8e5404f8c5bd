// Block-level W4A8 contraction with a multi-stage LDS ring fed by direct
// global->LDS loads (gfx950 global_load_lds_dwordx4), for the compute-bound shapes.
//
// 256 threads = 2 x 2 waves; a wave owns MT x NT 16x16 MFMA tiles, a block
// BM = 32*MT weight rows x BN = 32*NT activation rows.  Per 128-column chunk a
// stage of the ring holds
//   A: 2*MT weight blocks of 1 KiB, copied verbatim from the TILED blob (the blob
//      is already in operand order, so lane l later reads bytes [16l, 16l+16));
//   B: 4*NT activation blocks of 1 KiB, each 8 activation rows x the chunk's 128
//      bytes.  Lane l of the loading wave fetches row l/8, 16-byte piece
//      (l%8) ^ (l/8): every load instruction covers 8 whole 128-byte lines (half
//      lines cost the vector-memory path as much as whole ones, measured: twice
//      the time per byte), and the XOR spreads the 8 rows that the lanes of one
//      MFMA operand read at the same piece index over all LDS banks.
// Every LDS read is a conflict-free 128-bit read, and the data never passes
// through registers on its way in, so S-1 chunks can be in flight per block
// (what hides the ~1 us L2/HBM latency at this consumption rate).
//
// The direct loads are issued from inline asm (the compiler would otherwise wait
// for all of them before any LDS read); their completion is tracked by hand with
// s_waitcnt vmcnt(n) + s_barrier.  Between the first issue and the end of
// qr_pipe_mma no other vector-memory instruction may be issued by the caller.
// Activation columns >= K inside the last chunk are fetched from column 0 of the
// same row: they meet the zero padding of the weight blob.
#pragma once

#include "qrnnt_common.h"

template <int NT>
struct QrPhase {
    const v4i *w;            // TILED blob
    int nkc;                 // 128-column chunks
    int K;                   // valid activation columns
    const int8_t *row[NT];   // this thread's activation rows (one per B block it loads)
};

// W8: 8-bit weights, two blocks per row tile and chunk (the two operands as stored) instead of one.
template <int MT, int NT, int S, bool W8 = false>
struct QrPipe {
    static_assert(MT % 2 == 0 && NT % 2 == 0, "tiles per wave must be even");
    static constexpr int BM = 32 * MT, BN = 32 * NT;
    static constexpr int A_BLOCKS = (W8 ? 4 : 2) * MT, B_BLOCKS = 4 * NT;
    static constexpr int A_PER_WAVE = A_BLOCKS / 4, B_PER_WAVE = NT;
    static constexpr int LOADS = A_PER_WAVE + B_PER_WAVE;   // vector-memory loads per thread per chunk
    static constexpr int STAGE_BYTES = (A_BLOCKS + B_BLOCKS) * 1024;
    static constexpr int LDS_BYTES = S * STAGE_BYTES;
    static constexpr int DIST = S - 1;                       // chunks in flight
};

__device__ __forceinline__ void qr_load_lds16(const void *gptr, unsigned lds_addr)
{
    // M0 carries the wave-uniform LDS base; each lane's 16 bytes land at base + 16*lane.
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory");
}

template <int N>
__device__ __forceinline__ void qr_wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Which 1 KiB activation block (8 rows) load `i` of a wave's B loads stages.  All 4*NT blocks, NT per wave; or, with
// NTV < NT, only the blocks of the first NTV column tiles of each of the two wave columns, NTV per wave.
template <int NT, int NTV = NT>
__device__ __forceinline__ int qr_pipe_b_block(int wave, int i)
{
    if (NTV == NT) return wave * NT + i;
    const int k = wave * NTV + i, tv = k >> 1;   // tv: which of the 2 * NTV staged tiles (two blocks each)
    return 2 * ((tv / NTV) * NT + tv % NTV) + (k & 1);
}

// Which activation row load `i` of this thread's B loads fetches, relative to the block's first row.
template <int NT, int NTV = NT>
__device__ __forceinline__ int qr_pipe_b_row(int wave, int i, int lane)
{
    return qr_pipe_b_block<NT, NTV>(wave, i) * 8 + (lane >> 3);
}

// NTV: only the wave's first NTV column tiles are staged (ph[].row[0 .. NTV), see qr_pipe_b_block) and contracted.
template <int MT, int NT, int S, int NPH, bool TAIL, bool W8 = false, int NTV = NT, class PhaseEnd>
__device__ __forceinline__ void qr_pipe_mma(const QrPhase<NT> (&ph)[NPH], int n_row_tiles, int block_rt0, char *lds,
                                            v4i (&acc)[MT][NT], PhaseEnd &&on_phase_end)
{
    using P = QrPipe<MT, NT, S, W8>;
    constexpr int LOADS = P::A_PER_WAVE + NTV;   // vector-memory loads per thread per chunk
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = lane >> 4, col = lane & 15;
    const int wm = wave & 1, wn = wave >> 1;
    const int p0 = (grp ^ (col & 7)) * 16, p1 = ((4 + grp) ^ (col & 7)) * 16;   // swizzled pieces of the two K halves
    const unsigned lds_base = (unsigned)(size_t)lds;
    const int nk0 = ph[0].nkc;
    const int total = nk0 + (NPH == 2 ? ph[NPH - 1].nkc : 0);

    // Issue stream: running source pointers, advanced by one chunk per call and
    // re-based when the stream crosses from phase 0 to phase 1.
    const int boff = ((lane & 7) ^ (lane >> 3)) * 16;   // this lane's 16-byte piece of a chunk row
    const v4i *cur_a[P::A_PER_WAVE];
    const int8_t *cur_b[NTV];
    int cur_p = 0, cur_kc = 0, cur_nkc = 0, cur_K = 0;
    auto rebase = [&](int p) {
        const QrPhase<NT> &ps = ph[p];
        cur_nkc = ps.nkc;
        cur_K = ps.K;
#pragma unroll
        for (int a = 0; a < P::A_PER_WAVE; ++a) {
            const int ab = wave * P::A_PER_WAVE + a;   // block of the stage: row tile ab (4-bit) or (row tile ab/2, K half ab%2)
            int rt = block_rt0 + (W8 ? ab >> 1 : ab);
            rt = rt < n_row_tiles ? rt : n_row_tiles - 1;
            cur_a[a] = W8 ? ps.w + ((size_t)rt * ps.nkc * 2 + (ab & 1)) * 64 + lane : ps.w + (size_t)rt * ps.nkc * 64 + lane;
        }
#pragma unroll
        for (int i = 0; i < NTV; ++i) cur_b[i] = ps.row[i] + boff;
    };
    rebase(0);
    // One chunk = LOADS loads per thread; issue_one(q) is load q of the chunk at the head of
    // the issue stream, issue_done() moves the stream to the next chunk.
    auto chunk_tail = [&]() { return TAIL && (cur_kc == cur_nkc - 1) && (cur_K & (QRNNT_KCHUNK - 1)); };   // uniform
    auto issue_one = [&](int q, unsigned sbase, bool tail) {
        if (q < P::A_PER_WAVE) {
            qr_load_lds16(cur_a[q], sbase + (wave * P::A_PER_WAVE + q) * 1024);
            cur_a[q] += W8 ? 128 : 64;
        } else {
            const int i = q - P::A_PER_WAVE;
            const int8_t *src = cur_b[i];
            if (TAIL && tail) {
                const int k = cur_kc * QRNNT_KCHUNK + boff;
                if (k >= cur_K) src = cur_b[i] - k;   // row start: any valid bytes do, they meet zero weights
            }
            qr_load_lds16(src, sbase + (P::A_BLOCKS + qr_pipe_b_block<NT, NTV>(wave, i)) * 1024);
            cur_b[i] += QRNNT_KCHUNK;
        }
    };
    auto issue_done = [&]() {
        if (++cur_kc == cur_nkc && NPH == 2 && cur_p == 0) {
            cur_p = 1;
            cur_kc = 0;
            rebase(1);
        }
    };
    auto issue = [&](int stage) {
        const unsigned sbase = lds_base + stage * P::STAGE_BYTES;
        const bool tail = chunk_tail();
#pragma unroll
        for (int q = 0; q < LOADS; ++q) issue_one(q, sbase, tail);
        issue_done();
    };

    // prologue: fill DIST stages
#pragma unroll
    for (int v = 0; v < P::DIST; ++v)
        if (v < total) issue(v);

    int stage = 0, istage = P::DIST % S;
    for (int c = 0; c < total; ++c) {
        const int after = total - 1 - c;   // chunks after c; min(DIST-1, after) of them are already in flight
        static_assert(P::DIST >= 1 && P::DIST <= 3, "ring depth 2..4");
        if (P::DIST >= 3 && after >= 2) qr_wait_vmcnt<2 * LOADS>();
        else if (P::DIST >= 2 && after >= 1) qr_wait_vmcnt<LOADS>();
        else qr_wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        // The refill of the stage that was read in the previous iteration is issued in
        // shares between the row tiles' MFMAs: a wave issues in order, and a burst of
        // direct loads would keep it away from the matrix unit for their whole issue time.
        const bool do_issue = c + P::DIST < total;
        const unsigned isbase = lds_base + istage * P::STAGE_BYTES;
        const bool itail = chunk_tail();
        istage = (istage + 1 == S) ? 0 : istage + 1;

        const char *sb = lds + stage * P::STAGE_BYTES + lane * 16;
        const char *sbb = lds + stage * P::STAGE_BYTES + (P::A_BLOCKS + (col >> 3)) * 1024 + (col & 7) * 128;
        stage = (stage + 1 == S) ? 0 : stage + 1;
        v4i pa[MT], pa_hi[W8 ? MT : 1], b0[NT], b1[NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (W8) {
                pa[mt] = *(const v4i *)(sb + ((wm * MT + mt) * 2) * 1024);
                pa_hi[mt] = *(const v4i *)(sb + ((wm * MT + mt) * 2 + 1) * 1024);
            } else {
                pa[mt] = *(const v4i *)(sb + (wm * MT + mt) * 1024);
            }
        }
#pragma unroll
        for (int nt = 0; nt < NTV; ++nt) {
            b0[nt] = *(const v4i *)(sbb + (wn * NT + nt) * 2048 + p0);
            b1[nt] = *(const v4i *)(sbb + (wn * NT + nt) * 2048 + p1);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            v4i lo, hi;
            if (W8) { lo = pa[mt]; hi = pa_hi[mt]; }
            else qr_unpack(pa[mt], lo, hi);
#pragma unroll
            for (int nt = 0; nt < NTV; ++nt) {
                acc[mt][nt] = qr_mfma(lo, b0[nt], acc[mt][nt]);
                acc[mt][nt] = qr_mfma(hi, b1[nt], acc[mt][nt]);
            }
            constexpr int SHARE = (LOADS + MT - 1) / MT;
            __builtin_amdgcn_sched_barrier(0);
            if (do_issue) {
#pragma unroll
                for (int q = mt * SHARE; q < (mt + 1) * SHARE && q < LOADS; ++q) issue_one(q, isbase, itail);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (do_issue) issue_done();
        if (NPH == 2 && c == nk0 - 1) on_phase_end();
    }
}
