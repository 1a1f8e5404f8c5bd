// Quantized LSTM cell: INT4 weights x INT4 activations on the int8 MFMA units
// with the whole cell fused behind the contraction (Sec. 3.2: integer MACs for
// W_ih and W_hh, fp bias and cell state; Sec. 3.4: the hidden state is
// quantized once, at the cell output).
#include <atomic>
#include <mutex>
#include <type_traits>

#include "kernels.h"
#include "mma_pipe.h"

namespace {

// Bandwidth-bound variant (few hypotheses, e.g. one utterance at beam 16).
// The packed weights are streamed exactly once per 16 hypotheses: a workgroup owns one row
// tile (4 cells) x one column tile (16 hypotheses); its 128-column chunks of W_ih and W_hh are
// dealt round-robin to the 4 waves, every wave issues all of its loads before its first MFMA
// (what keeps the whole matrix in flight across the chip), and the partial sums meet in LDS.
// Wave 0 then finishes the 4 cells, one (cell, hypothesis) per lane.  N = 16 is exactly one
// 16-column MFMA tile, so the matrix cores serve this regime too: the kernel is bound by the
// weight stream and by its chain of dependent loads, which is kept to two links: the weight
// loads (which depend on nothing) go first, then the row indices, then everything that
// depends on them, including what the cell update will need.
// Grid: x = row tiles, y = column tiles, z = problem of a group.
constexpr int SMALL_BATCH = 4;   // chunks per wave per batch (K <= 2048 in one batch)

template <bool USE_GX>
__global__ __launch_bounds__(256) void lstm_step_small_kernel(const QrStepGroup g)
{
    __shared__ v4i part[3][2][64];   // waves 1..3: [x|h][lane]
    if (g.gate && *g.gate == 0) return;   // uniform: a decoding round without any live hypothesis
    const QrStepArgs a = g.p[blockIdx.z];   // a copy: the fields arrive with a few wide scalar loads up front
    const int H = a.H, N = a.N;
    const int rt = blockIdx.x;
    const int n0 = blockIdx.y * 16;
    if (rt >= (H >> 2) || n0 >= N) return;   // uniform
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: MFMAs below sit under wave-uniform branches
    const int col = lane & 15, grp = lane >> 4;
    const v4i zero = {0, 0, 0, 0};
    const int m = (int)0xF0F0F0F0u;
    const int nkx = USE_GX ? 0 : a.nkc_x;
    const int total = nkx + a.nkc_h;

    // ---- first batch of weight fragments: independent of every index
    v4i pa[SMALL_BATCH];
    auto load_weights = [&](int v0) {
#pragma unroll
        for (int it = 0; it < SMALL_BATCH; ++it) {
            const int v = v0 + 4 * it;
            const bool ok = v < total;
            const bool isx = ok && v < nkx;
            const int kc = ok ? (isx ? v : v - nkx) : 0;
            const v4i *w = isx ? a.wih : a.whh;
            const int nkc = isx ? a.nkc_x : a.nkc_h;
            pa[it] = ok ? w[((size_t)rt * nkc + kc) * 64 + lane] : zero;
        }
    };
    load_weights(wave);

    // ---- indices, then everything that hangs on them
    bool n_ok = n0 + col < N;
    int nn = n_ok ? n0 + col : N - 1;
    int s, xr;
    if (g.rows) {   // row j of the problem stands for the hypothesis of entry j (see QrStepGroup.rows)
        const v4i e = g.rows[nn];
        const int n_cnt = *g.n_rows;
        if (n0 >= n_cnt) return;   // uniform
        n_ok = n0 + col < n_cnt;
        nn = e[0] < 0 ? 0 : (e[0] >= N ? N - 1 : e[0]);
        s = a.parent ? e[1] : nn;
        xr = a.x_row ? e[2] : nn;
    } else {
        s = a.parent ? a.parent[nn] : nn;
        xr = a.x_row ? a.x_row[nn] : nn;
    }
    const int n = nn;
    s = s < 0 ? 0 : (s >= a.n_slots ? a.n_slots - 1 : s);
    xr = xr < 0 ? 0 : (xr >= a.n_x_rows ? a.n_x_rows - 1 : xr);
    const int8_t *hrow = a.h_prev + (int64_t)s * a.ld_hp + grp * 16;
    const int8_t *xrow = USE_GX ? nullptr : a.x + (int64_t)xr * a.ld_x + grp * 16;
    // the cell update of wave 0: cell j of (row tile, grp) for hypothesis n
    const int j = qr_gates_cell(rt, grp);
    float sx[4], sh[4], bb[4], cp = 0.0f;
    int act = 1, hp_code = 0;
    v4i gxv = zero;
    if (wave == 0) {
#pragma unroll
        for (int gt = 0; gt < 4; ++gt) {
            sx[gt] = a.x_scale * a.s_wih[gt * H + j];
            sh[gt] = a.h_scale * a.s_whh[gt * H + j];
            bb[gt] = a.bias[gt * H + j];
        }
        cp = a.c_prev[(int64_t)s * H + j];
        if (USE_GX) gxv = *(const v4i *)(a.gx + (int64_t)xr * a.ld_gx + rt * 16 + 4 * grp);
        if (a.active) {
            act = a.active[nn];
            hp_code = a.h_prev[(int64_t)s * a.ld_hp + j];
        }
    }

    v4i accx = zero, acch = zero;
    for (int v0 = wave; v0 < total; v0 += 4 * SMALL_BATCH) {
        if (v0 != wave) load_weights(v0);
        v4i b0[SMALL_BATCH], b1[SMALL_BATCH];
#pragma unroll
        for (int it = 0; it < SMALL_BATCH; ++it) {
            const int v = v0 + 4 * it;
            const bool ok = v < total;
            const bool isx = ok && v < nkx;
            const int kc = ok ? (isx ? v : v - nkx) : 0;
            const int K = isx ? a.I : H;
            const int k0 = kc * QRNNT_KCHUNK + grp * 16;
            const int8_t *row = isx ? xrow : hrow;
            b0[it] = (ok && k0 < K) ? *(const v4i *)(row + kc * QRNNT_KCHUNK) : zero;
            b1[it] = (ok && k0 + 64 < K) ? *(const v4i *)(row + kc * QRNNT_KCHUNK + 64) : zero;
        }
#pragma unroll
        for (int it = 0; it < SMALL_BATCH; ++it) {
            const int v = v0 + 4 * it;
            if (v < total) {   // uniform per wave
                const v4i lo = (pa[it] << 4) & m, hi = pa[it] & m;
                if (v < nkx) {
                    accx = qr_mfma(lo, b0[it], accx);
                    accx = qr_mfma(hi, b1[it], accx);
                } else {
                    acch = qr_mfma(lo, b0[it], acch);
                    acch = qr_mfma(hi, b1[it], acch);
                }
            }
        }
    }
    if (wave != 0) {
        part[wave - 1][0][lane] = accx;
        part[wave - 1][1][lane] = acch;
    }
    __syncthreads();
    if (wave != 0) return;

    v4i ax = accx, ah = acch;
#pragma unroll
    for (int wv = 0; wv < 3; ++wv) { ax += part[wv][0][lane]; ah += part[wv][1][lane]; }
    ax = USE_GX ? gxv : (ax >> 4);
    ah = ah >> 4;
    float p[4];
#pragma unroll
    for (int gt = 0; gt < 4; ++gt) p[gt] = sx[gt] * (float)ax[gt] + (sh[gt] * (float)ah[gt] + bb[gt]);
    const float gi = qr_sigmoid(p[0]), gf = qr_sigmoid(p[1]), gg = qr_tanh(p[2]), go = qr_sigmoid(p[3]);
    float cn = gf * cp + gi * gg;
    const float h = go * qr_tanh(cn);
    int code = qr_quant4(h, a.h_inv);
    const bool on = act != 0;
    cn = on ? cn : cp;
    code = on ? code : hp_code;
    if (n_ok) {
        a.c_next[(int64_t)n * H + j] = cn;
        a.h_next[(int64_t)n * a.ld_hn + j] = (int8_t)code;
        if (a.h_copy) a.h_copy[(int64_t)n * H + j] = (int8_t)code;
        if (a.dbg_accx)
#pragma unroll
            for (int gt = 0; gt < 4; ++gt) a.dbg_accx[(int64_t)n * 4 * H + gt * H + j] = ax[gt];
        if (a.dbg_acch)
#pragma unroll
            for (int gt = 0; gt < 4; ++gt) a.dbg_acch[(int64_t)n * 4 * H + gt * H + j] = ah[gt];
        if (a.dbg_gates && on) {
            float *dg = a.dbg_gates + (int64_t)n * 4 * H + j;
            dg[0] = gi; dg[H] = gf; dg[2 * H] = gg; dg[3 * H] = go;
        }
    }
}

template <bool USE_GX>
void launch_small(const QrStepGroup &g, hipStream_t st)
{
    int max_n = 0, max_rt = 0;
    for (int i = 0; i < g.n; ++i) {
        max_n = g.p[i].N > max_n ? g.p[i].N : max_n;
        max_rt = (g.p[i].H >> 2) > max_rt ? (g.p[i].H >> 2) : max_rt;
    }
    lstm_step_small_kernel<USE_GX><<<dim3(max_rt, (max_n + 15) / 16, g.n), 256, 0, st>>>(g);
}

// Compute-bound variant (many hypotheses): multi-stage LDS ring, see mma_pipe.h.
// Grid: x = blocks of 32*MT gate rows (8*MT cells), z = blocks of 32*NT hypotheses (or of a half or a
// quarter of that: few hypotheses are spread over more workgroups, which then run a narrower instance
// of the kernel's body, see the index section below), y = problem of a group (independent layer-steps
// batched into one launch).
// Every global load outside the ring is issued in a batch ahead of its first use
// and the cell update is branch-free, so a block exposes one memory latency per
// batch instead of one per element.  DBG adds the int32 / gate outputs.
// FAST: every K is a multiple of 128, every tile is full (no bounds checks needed).
// With a precomputed input projection (USE_GX) there is one contraction phase and no fp32 copy
// of the input part to keep alive across it: that variant is held to 168 registers so that three
// workgroups share a CU (with a two-stage ring), which is what lets the 704 workgroups of the
// decoder's first-layer launch run in one round instead of two.
// TAB (with USE_GX): the looked-up input part is an fp32 table that already holds
// gate_k * (x_scale * s_wih[r] * sum + bias[r]) (see qr_launch_gx_table): one fused multiply-add per gate
// is all that is left of the dequantisation.
template <int MT, int NT, int S, bool USE_GX, bool TAB, bool DBG, bool FAST>
__global__ __launch_bounds__(256, (USE_GX && !DBG) ? 3 : 2) void lstm_step_pipe_kernel(const QrStepGroup g)
{
    using P = QrPipe<MT, NT, S>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    if (g.gate && *g.gate == 0) return;   // uniform: a decoding round without any live hypothesis
    // The column block is the slowest grid dimension: the workgroups of a short list's few column blocks are then
    // the first to be dispatched, and those that only look at the count and return follow behind them.
    const int col_block = g.col_block0 + (int)blockIdx.z;
    // A copy, not a reference: the fields then arrive with a few wide scalar loads up front instead of one load (and
    // one wait) at a time wherever the code first needs them.
    const QrStepArgs a = g.p[blockIdx.y];
    const int H = a.H, N = a.N;
    const int n_row_tiles = H >> 2;
    const int block_rt0 = blockIdx.x * 2 * MT;
    const int n0 = col_block * P::BN;
    if (block_rt0 >= n_row_tiles) return;   // uniform per block

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, grp = lane >> 4;
    const int wm = wave & 1, wn = wave >> 1;
    const int rt0 = block_rt0 + wm * MT;

    // Row constants of the input part (two-phase variants): what the hand-over between the phases needs is fetched
    // now, one value per thread, and parked in LDS, so that the hand-over itself issues no vector-memory load (the
    // wave's memory counter is in order: waiting for such a load there would wait for the whole ring as well).
    constexpr int CELLS = 8 * MT;   // cells of a workgroup's row block
    __shared__ __attribute__((aligned(16))) float xc[USE_GX ? 4 : 8 * CELLS];   // [s_wih, bias][gate][cell]
    float xc_val = 0.0f;
    if (!USE_GX) {
        static_assert(USE_GX || 8 * CELLS == 256, "one constant per thread");
        int cell = (block_rt0 >> 2) * 16 + (tid & (CELLS - 1));
        cell = cell < H ? cell : H - 1;
        xc_val = (tid < 4 * CELLS ? a.s_wih : a.bias)[((tid / CELLS) & 3) * H + cell];
    }

    // ---- indices: rows this thread stages (ld_*) and hypotheses this lane finishes (n_of)
    int ld_n[NT], ld_s[NT], ld_x[NT], n_of[NT], src_of[NT], gx_of[NT];
    bool n_ok[NT];   // the column stands for a hypothesis (not for padding of the last block)
    int nt_valid = NT;   // this wave's column tiles from here on are padding (list mode)
    constexpr bool HALF_OK = true;   // every variant has the narrower instances (the debug build of each included)
    // With a list the problem has *n_rows rows, row j standing for the hypothesis of entry j.
    //  * A workgroup takes 32*NT, 16*NT or 8*NT consecutive entries (width 0, 1, 2): the narrowest width at which the
    //    launch's column blocks still cover the list and the working workgroups do not outnumber the compute units
    //    (beyond that, narrower only means fetching the weights more often), so that a short list is spread over
    //    more workgroups, each of which then runs the half- or quarter-width instance of the body below.
    //  * The 16-column tiles of a workgroup's entries are dealt to the two column halves of the wave grid in turn
    //    (logical tile 2*nt + wn sits at wave column wn, position nt), so that every wave holds the same number of
    //    live tiles; a workgroup at full width whose share of the list ends within its first half runs the
    //    half-width instance as well.
    const v4i *rows = g.rows;
    int width = 0;   // log2 of (full width / entries per workgroup)
    if (rows) {
        // The entries are requested before the length of the list is looked at, so the two fetches overlap
        // (columns beyond the end compute on whatever their entry names, clamped into range, and store
        // nothing); an entry brings parent and input row along.  Which entries a thread stages and finishes
        // depends on the width and on the instance, which the count decides.
        // The entries of the workgroup's three possible ranges (full, half and quarter width: 7/4 of a column block in
        // all) go through LDS, one load per thread; every thread then picks the ones it stages and finishes.  (The
        // ring is not in use yet; the second barrier below keeps its first loads behind the last of these reads.)
        // staged row rl of a workgroup's range: tile rl / 16 = wn' * NT + nt' -> logical tile 2 * nt' + wn'
        auto logical = [](int rl) { return (((rl >> 4) % NT) * 2 + (rl >> 4) / NT) * 16 + (rl & 15); };
        const int n0h = col_block * (P::BN / 2), n0q = col_block * (P::BN / 4);
        static_assert(P::BN + P::BN / 2 + P::BN / 4 <= 256, "one entry per thread");
        v4i *se = (v4i *)lds;
        if (tid < P::BN + P::BN / 2 + P::BN / 4) {
            const int j = tid < P::BN ? n0 + tid : (tid < P::BN + P::BN / 2 ? n0h + tid - P::BN : n0q + tid - P::BN - P::BN / 2);
            se[tid] = rows[j < N ? j : N - 1];
        }
        const int n_cnt = *g.n_rows;
        if (HALF_OK) {   // uniform: the narrowest width that covers the list and does not ask for more workgroups than CUs
#pragma unroll
            for (int w = 1; w <= 2; ++w) {
                const int per = P::BN >> w;
                if (per * (g.col_block0 + (int)gridDim.z) >= n_cnt && g.row_blocks * ((n_cnt + per - 1) / per) <= g.n_cu) width = w;
            }
        }
        const int n0w = width == 2 ? n0q : (width == 1 ? n0h : n0);
        if (n0w >= n_cnt) return;   // uniform per block
        __syncthreads();
        const int se0 = width == 2 ? P::BN + P::BN / 2 : (width == 1 ? P::BN : 0);   // where the range of this width starts in se
        nt_valid = NT >> width;
        if (width == 0) {   // tiles that hold entries, per wave column (rounded up); at this width no instance below the half
            nt_valid = (((n_cnt - n0 + 15) >> 4) + 1) >> 1;
            nt_valid = nt_valid < NT / 2 ? NT / 2 : nt_valid;
        }
        const bool half = HALF_OK && width == 0 && nt_valid * 2 <= NT;   // uniform
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int jf = n0w + (i * 2 + wn) * 16 + col;
            const int ih = i < NT / 2 ? i : 0, iq = i < NT / 4 ? i : 0;   // (entries past an instance's tiles are not used)
            int rl = qr_pipe_b_row<NT>(wave, i, lane);                        // the row this thread stages with load i
            if (half || (HALF_OK && width == 1)) rl = qr_pipe_b_row<NT, NT / 2>(wave, ih, lane);
            if (HALF_OK && width == 2) rl = qr_pipe_b_row<NT, NT / 4>(wave, iq, lane);
            int fl = (i * 2 + wn) * 16 + col;                                 // the column this lane finishes in tile i
            fl = fl < (P::BN >> width) ? fl : 0;
            const v4i el_i = se[se0 + logical(rl)], ef_i = se[se0 + fl];
            auto hyp = [&](int r) { return r < 0 ? 0 : (r >= N ? N - 1 : r); };
            ld_n[i] = hyp(el_i[0]);
            ld_s[i] = a.parent ? el_i[1] : ld_n[i];
            ld_x[i] = (!USE_GX && a.x_row) ? el_i[2] : ld_n[i];
            n_of[i] = hyp(ef_i[0]);
            src_of[i] = a.parent ? ef_i[1] : n_of[i];
            n_ok[i] = jf < n_cnt;
            if (USE_GX) {
                const int r = a.x_row ? ef_i[2] : n_of[i];
                gx_of[i] = r < 0 ? 0 : (r >= a.n_x_rows ? a.n_x_rows - 1 : r);
            }
        }
        __syncthreads();
    } else {
        // Without a list the launcher has chosen the width from N by the same rule (g.width); at full width the
        // columns keep their natural order.
        width = HALF_OK ? g.width : 0;   // uniform
        const int n0w = col_block * (P::BN >> width);
        if (n0w >= N) return;   // uniform per block
        nt_valid = NT >> width;
        auto logical = [](int rl) { return (((rl >> 4) % NT) * 2 + (rl >> 4) / NT) * 16 + (rl & 15); };
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            int n = qr_pipe_b_row<NT>(wave, i, lane), m = (wn * NT + i) * 16 + col;
            if (HALF_OK && width == 1) { n = logical(qr_pipe_b_row<NT, NT / 2>(wave, i < NT / 2 ? i : 0, lane)); m = (i * 2 + wn) * 16 + col; }
            if (HALF_OK && width == 2) { n = logical(qr_pipe_b_row<NT, NT / 4>(wave, i < NT / 4 ? i : 0, lane)); m = (i * 2 + wn) * 16 + col; }
            n += n0w;
            m += n0w;
            ld_n[i] = n < N ? n : N - 1;
            n_of[i] = m;
            n_ok[i] = m < N;
            src_of[i] = m < N ? m : N - 1;
        }
        if (a.parent) {
#pragma unroll
            for (int i = 0; i < NT; ++i) { ld_s[i] = a.parent[ld_n[i]]; src_of[i] = a.parent[src_of[i]]; }
        } else {
#pragma unroll
            for (int i = 0; i < NT; ++i) ld_s[i] = ld_n[i];
        }
        if (!USE_GX && a.x_row) {
#pragma unroll
            for (int i = 0; i < NT; ++i) ld_x[i] = a.x_row[ld_n[i]];
        } else {
#pragma unroll
            for (int i = 0; i < NT; ++i) ld_x[i] = ld_n[i];
        }
        if (USE_GX) {   // row of the precomputed input projection for the hypotheses this lane finishes
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const int n = n_of[i] < N ? n_of[i] : N - 1;
                int r = a.x_row ? a.x_row[n] : n;
                gx_of[i] = r < 0 ? 0 : (r >= a.n_x_rows ? a.n_x_rows - 1 : r);
            }
        }
    }
    constexpr int NPH = USE_GX ? 1 : 2;
    QrPhase<NT> ph[NPH];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        int s = ld_s[i];
        s = s < 0 ? 0 : (s >= a.n_slots ? a.n_slots - 1 : s);
        ph[NPH - 1].row[i] = a.h_prev + (int64_t)s * a.ld_hp;
        if (!USE_GX) {
            int xr = ld_x[i];
            xr = xr < 0 ? 0 : (xr >= a.n_x_rows ? a.n_x_rows - 1 : xr);
            ph[0].row[i] = a.x + (int64_t)xr * a.ld_x;
        }
        int q = src_of[i];
        src_of[i] = q < 0 ? 0 : (q >= a.n_slots ? a.n_slots - 1 : q);
    }
    if (!USE_GX) { ph[0].w = a.wih;  ph[0].nkc = a.nkc_x;  ph[0].K = a.I; }
    ph[NPH - 1].w = a.whh;  ph[NPH - 1].nkc = a.nkc_h;  ph[NPH - 1].K = H;

    // Everything from here on exists three times: for all NT column tiles of the wave, for its first NT / 2 and for
    // its first NT / 4 only.
    auto run = [&](auto ntv_tag) {
    constexpr int NTV = decltype(ntv_tag)::value;
    v4i acc[MT][NT];
    float pre[MT][NT][4];
    const v4i zero = {0, 0, 0, 0};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTV; ++nt) acc[mt][nt] = zero;

    // This lane finishes cells jb[q] .. jb[q]+3 (row tiles 4q .. 4q+3 of the wave) for
    // hypotheses n_of[nt]; out-of-range quartets are clamped for loads and skipped at the stores.
    static_assert(MT % 4 == 0, "a wave owns whole 64-row groups");
    constexpr int MQ = MT / 4;
    int jb[MQ];
#pragma unroll
    for (int q = 0; q < MQ; ++q) {
        const int j = qr_gates_cell(rt0 + 4 * q, grp);
        jb[q] = j < H ? j : H - 4;
    }
    auto load4 = [](const float *p) { return *(const v4f *)p; };
    // The pre-activations are formed already multiplied by the constant their activation feeds to
    // exp2 (-log2 e for the sigmoids, -2 log2 e for tanh): folded into the per-row scales and the
    // bias, it costs nothing per element.
    auto gate_k = [](int gt) { return gt == 2 ? -2.885390081777927f : -1.4426950408889634f; };

    // input part -> fp32 (s_x * s_wih[r] * accx); the accumulators restart for the recurrent part
    auto x_done = [&]() {
#pragma unroll
        for (int q = 0; q < MQ; ++q) {
            v4f sx[4], bx[4];
#pragma unroll
            for (int gt = 0; gt < 4; ++gt) {   // accumulators hold 16 x sum; gate_k: see the epilogue
                const float *xq = xc + gt * CELLS + (wm * MQ + q) * 16 + 4 * grp;   // this lane's four cells
                sx[gt] = *(const v4f *)xq * a.x_scale * (0.0625f * gate_k(gt));
                bx[gt] = *(const v4f *)(xq + 4 * CELLS) * gate_k(gt);   // the bias rides with the input part
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int nt = 0; nt < NTV; ++nt) {
                    const int mt = 4 * q + i;
                    if (DBG && a.dbg_accx && jb[q] == qr_gates_cell(rt0 + 4 * q, grp) && n_ok[nt])
#pragma unroll
                        for (int gt = 0; gt < 4; ++gt)
                            a.dbg_accx[(int64_t)n_of[nt] * 4 * H + gt * H + jb[q] + i] = acc[mt][nt][gt] >> 4;
#pragma unroll
                    for (int gt = 0; gt < 4; ++gt) pre[mt][nt][gt] = sx[gt][i] * (float)acc[mt][nt][gt] + bx[gt][i];
                    acc[mt][nt] = zero;
                }
        }
    };
    if (!USE_GX) {
        xc[tid] = xc_val;
        __syncthreads();
    }
    qr_pipe_mma<MT, NT, S, NPH, !FAST, false, NTV>(ph, n_row_tiles, block_rt0, lds, acc, x_done);

    // ---- fused cell: batched 128-bit loads, then branch-free arithmetic, then 128-bit / 32-bit stores
    v4f cp[MQ][NT], sh[MQ][4], bb[MQ][4], sxg[MQ][4];
    int act[NT], hp_code[MQ][NT];
#pragma unroll
    for (int q = 0; q < MQ; ++q) {
#pragma unroll
        for (int gt = 0; gt < 4; ++gt) {
            sh[q][gt] = load4(a.s_whh + gt * H + jb[q]) * a.h_scale * (0.0625f * gate_k(gt));   // accumulators hold 16 x sum
            if (USE_GX && !TAB) bb[q][gt] = load4(a.bias + gt * H + jb[q]) * gate_k(gt);
            if (USE_GX && !TAB) sxg[q][gt] = load4(a.s_wih + gt * H + jb[q]) * a.x_scale * gate_k(gt);
        }
#pragma unroll
        for (int nt = 0; nt < NTV; ++nt) cp[q][nt] = load4(a.c_prev + (int64_t)src_of[nt] * H + jb[q]);
    }
    if (a.active) {
#pragma unroll
        for (int nt = 0; nt < NTV; ++nt) {
            act[nt] = a.active[n_of[nt] < N ? n_of[nt] : N - 1];
#pragma unroll
            for (int q = 0; q < MQ; ++q) hp_code[q][nt] = *(const int *)(a.h_prev + (int64_t)src_of[nt] * a.ld_hp + jb[q]);
        }
    } else {
#pragma unroll
        for (int nt = 0; nt < NTV; ++nt) {
            act[nt] = 1;
#pragma unroll
            for (int q = 0; q < MQ; ++q) hp_code[q][nt] = 0;
        }
    }
    // precomputed input part: the four gate quartets of (q, nt), fetched one column tile ahead of their use
    auto load_gx = [&](int q, int nt, v4i (&dst)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int tr = (rt0 + 4 * q + i) * 16 + 4 * grp;   // gx columns are in tiled-row order
            tr = tr < 4 * H ? tr : 4 * H - 4;
            dst[i] = *(const v4i *)((TAB ? (const int32_t *)a.tabf : a.gx) + (int64_t)gx_of[nt] * a.ld_gx + tr);
        }
    };
    v4i gxv[2][4];
    if (USE_GX) load_gx(0, 0, gxv[0]);
    const float hinv2 = 2.0f * a.h_inv;
#pragma unroll
    for (int q = 0; q < MQ; ++q) {
        const bool jv = FAST || qr_gates_cell(rt0 + 4 * q, grp) < H;
#pragma unroll
        for (int nt = 0; nt < NTV; ++nt) {
            const int n = n_of[nt];
            const bool on = act[nt] != 0;
            const int cur = (q * NTV + nt) & 1;
            if (USE_GX && q * NTV + nt + 1 < MQ * NTV) load_gx((q * NTV + nt + 1) / NTV, (q * NTV + nt + 1) % NTV, gxv[cur ^ 1]);
            v4f cn;
            unsigned codes = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int mt = 4 * q + i;
                float p[4];
#pragma unroll
                for (int gt = 0; gt < 4; ++gt) {
                    if (TAB) p[gt] = sh[q][gt][i] * (float)acc[mt][nt][gt] + __int_as_float(gxv[cur][i][gt]);
                    else if (USE_GX) p[gt] = sxg[q][gt][i] * (float)gxv[cur][i][gt] + (sh[q][gt][i] * (float)acc[mt][nt][gt] + bb[q][gt][i]);
                    else p[gt] = sh[q][gt][i] * (float)acc[mt][nt][gt] + pre[mt][nt][gt];
                }
                const float gi = qr_sigmoid_scaled(p[0]), gf = qr_sigmoid_scaled(p[1]);
                const float gg = 2.0f * qr_sigmoid_scaled(p[2]) - 1.0f, go = qr_sigmoid_scaled(p[3]);
                const float c1 = gf * cp[q][nt][i] + gi * gg;
                // h * h_inv with the factor folded into tanh's last multiply-add: (2r - 1) * h_inv
                const float rc = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.885390081777927f * c1));
                const float hq = go * (hinv2 * rc - a.h_inv);
                cn[i] = on ? c1 : cp[q][nt][i];
                codes |= (unsigned)((int)fminf(fmaxf(__builtin_rintf(hq), -8.0f), 7.0f) & 0xFF) << (8 * i);
                if (DBG && jv && n_ok[nt]) {
                    if (USE_GX && !TAB && a.dbg_accx)
#pragma unroll
                        for (int gt = 0; gt < 4; ++gt) a.dbg_accx[(int64_t)n * 4 * H + gt * H + jb[q] + i] = gxv[cur][i][gt];
                    if (a.dbg_acch)
#pragma unroll
                        for (int gt = 0; gt < 4; ++gt)
                            a.dbg_acch[(int64_t)n * 4 * H + gt * H + jb[q] + i] = acc[mt][nt][gt] >> 4;
                    if (a.dbg_gates && on) {
                        float *dg = a.dbg_gates + (int64_t)n * 4 * H + jb[q] + i;
                        dg[0] = gi; dg[H] = gf; dg[2 * H] = gg; dg[3 * H] = go;
                    }
                }
            }
            codes = on ? codes : (unsigned)hp_code[q][nt];
            if (FAST ? (!rows || n_ok[nt]) : (jv && n_ok[nt])) {
                *(v4f *)(a.c_next + (int64_t)n * H + jb[q]) = cn;
                *(unsigned *)(a.h_next + (int64_t)n * a.ld_hn + jb[q]) = codes;
                if (a.h_copy) *(unsigned *)(a.h_copy + (int64_t)n * H + jb[q]) = codes;
            }
        }
    }
    };
    nt_valid = __builtin_amdgcn_readfirstlane(nt_valid);
    if (HALF_OK && nt_valid * 4 <= NT) run(std::integral_constant<int, NT / 4>{});
    else if (HALF_OK && nt_valid * 2 <= NT) run(std::integral_constant<int, NT / 2>{});
    else run(std::integral_constant<int, NT>{});
}

template <int MT, int NT, int S, bool USE_GX, bool TAB, bool DBG, bool FAST>
void launch_pipe_f(const QrStepGroup &g, hipStream_t st)
{
    using P = QrPipe<MT, NT, S>;
    static std::atomic<int> n_cu_of[QR_MAX_DEVICES];   // 0: not asked yet (also marks "attribute not set yet")
    auto kern = lstm_step_pipe_kernel<MT, NT, S, USE_GX, TAB, DBG, FAST>;
    const int dev = qr_current_device();
    int n_cu = n_cu_of[dev].load(std::memory_order_relaxed);
    if (n_cu == 0) {
        (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, P::LDS_BYTES);
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) n_cu = 1;
        n_cu_of[dev].store(n_cu, std::memory_order_relaxed);
    }
    QrStepGroup gg = g;
    int gx = 0, max_n = 0;
    gg.row_blocks = 0;
    gg.n_cu = n_cu;
    for (int i = 0; i < g.n; ++i) {
        const int rb = ((g.p[i].H >> 2) + 2 * MT - 1) / (2 * MT);
        gx = rb > gx ? rb : gx;
        max_n = g.p[i].N > max_n ? g.p[i].N : max_n;
        gg.row_blocks += rb;
    }
    // Without a list the width is chosen here, by the rule the kernel applies to a list's length: the narrowest
    // share per workgroup at which the working workgroups do not outnumber the compute units.
    gg.width = 0;
    if (!g.rows)
        for (int w = 1; w <= 2; ++w)
            if (gg.row_blocks * ((max_n + (P::BN >> w) - 1) / (P::BN >> w)) <= n_cu) gg.width = w;
    const int per = P::BN >> gg.width;
    const int gz = (max_n + per - 1) / per;
    for (int z0 = 0; z0 < gz; z0 += 65535) {   // a grid's z extent ends at 65535
        gg.col_block0 = z0;
        kern<<<dim3(gx, g.n, gz - z0 < 65535 ? gz - z0 : 65535), 256, P::LDS_BYTES, st>>>(gg);
    }
}

template <int MT, int NT, int S, bool USE_GX>
void launch_pipe(const QrStepGroup &g, hipStream_t st)
{
    using P = QrPipe<MT, NT, S>;
    bool dbg = false, fast = true, tab = USE_GX;
    for (int i = 0; i < g.n; ++i) {
        const QrStepArgs &a = g.p[i];
        dbg = dbg || a.dbg_accx || a.dbg_acch || a.dbg_gates;
        tab = tab && a.tabf != nullptr;
        fast = fast && a.H % (8 * MT) == 0 && a.N % P::BN == 0 && a.H % QRNNT_KCHUNK == 0 &&
               (USE_GX || a.I % QRNNT_KCHUNK == 0);
    }
    // with debug outputs: the debug build of the same variant (same body, same tile walk, same narrow instances)
    if (dbg && USE_GX && tab && fast) launch_pipe_f<MT, NT, S, USE_GX, USE_GX, true, true>(g, st);
    else if (dbg && USE_GX && tab) launch_pipe_f<MT, NT, S, USE_GX, USE_GX, true, false>(g, st);
    else if (dbg && fast) launch_pipe_f<MT, NT, S, USE_GX, false, true, true>(g, st);
    else if (dbg) launch_pipe_f<MT, NT, S, USE_GX, false, true, false>(g, st);
    else if (USE_GX && tab && fast) launch_pipe_f<MT, NT, S, USE_GX, USE_GX, false, true>(g, st);
    else if (USE_GX && tab) launch_pipe_f<MT, NT, S, USE_GX, USE_GX, false, false>(g, st);
    else if (fast) launch_pipe_f<MT, NT, S, USE_GX, false, false, true>(g, st);
    else launch_pipe_f<MT, NT, S, USE_GX, false, false, false>(g, st);
}

// Hypothesis counts up to this go to the weight-streaming kernel.
static int small_n_max()
{
    return 32;   // measured per decoding round: 64 hypotheses 21.4 us here, 19.1 us in the tiled kernel at 32 per
                 // workgroup; 32 hypotheses 13.3 us here, 18.8 us there
}

template <bool USE_GX>
void launch_step_t(const QrStepArgs &a, hipStream_t st)
{
    QrStepGroup g;
    g.p[0] = a;
    g.n = 1;
    g.gate = nullptr;
    if (a.N <= small_n_max()) launch_small<USE_GX>(g, st);
    else launch_pipe<4, 4, USE_GX ? 2 : 3, USE_GX>(g, st);
}

// Input projection of all frames: gx[m, 4j+g] = sum_k Wih[g*H+j, k] * x[m, k].
// Output columns stay in tiled-row (gate-interleaved) order so that the recurrence
// fetches a cell's four gate sums with one 128-bit load.  A true dense contraction:
// the LDS ring of mma_pipe.h with a 32*MT x 32*NT block tile; no second phase, so the
// registers that the step kernel spends on the input part go into a taller tile.
// Grid: 1-D.  Consecutive workgroup ids go to different XCDs (8 of them, each with its own
// L2), so the id is split as (XCD, index within the XCD) and every XCD walks its own frame
// blocks, all row blocks of a frame block in a row: an activation tile is fetched from HBM
// by one L2 only (measured before: 181 MB fetched for 22 MB of operands), while the small
// weight matrix lives in every L2.
template <int MT, int NT, int S, bool TAIL, bool W8>
__global__ __launch_bounds__(256, (S == 2 && !W8) ? 3 : 2) void gx_gemm_pipe_kernel(const v4i *__restrict__ wih, int nkc, int n_row_tiles,
                                                              const int8_t *__restrict__ x, int64_t ld_x, int M, int K,
                                                              int32_t *__restrict__ gx, int H,
                                                              int32_t *__restrict__ dbg_accx)
{
    using P = QrPipe<MT, NT, S, W8>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, grp = lane >> 4;
    const int wm = wave & 1, wn = wave >> 1;
    const int nbx = (n_row_tiles + 2 * MT - 1) / (2 * MT);
    const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int by = (idx / nbx) * 8 + xcd;
    const int block_rt0 = (idx % nbx) * 2 * MT;
    const int m0 = by * P::BN;
    if (m0 >= M) return;   // uniform: padding of the last round of frame blocks
    const int rt0 = block_rt0 + wm * MT;
    QrPhase<NT> ph[1];
    ph[0].w = wih;  ph[0].nkc = nkc;  ph[0].K = K;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        int m = m0 + qr_pipe_b_row<NT>(wave, i, lane);
        m = m < M ? m : M - 1;
        ph[0].row[i] = x + (int64_t)m * ld_x;
    }
    v4i acc[MT][NT];
    const v4i zero = {0, 0, 0, 0};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = zero;
    qr_pipe_mma<MT, NT, S, 1, TAIL, W8>(ph, n_row_tiles, block_rt0, lds, acc, [] {});
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int j = qr_gates_cell(rt0 + mt, grp);
        if (j >= H) continue;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int m = m0 + (wn * NT + nt) * 16 + col;
            if (m >= M) continue;
            const v4i v = W8 ? acc[mt][nt] : (acc[mt][nt] >> 4);   // 4-bit operands carry a factor 16
            *(v4i *)(gx + (int64_t)m * 4 * H + (rt0 + mt) * 16 + 4 * grp) = v;
            if (dbg_accx)
#pragma unroll
                for (int gt = 0; gt < 4; ++gt) dbg_accx[(int64_t)m * 4 * H + gt * H + j] = v[gt];
        }
    }
}

template <int MT, int NT, int S, bool W8>
void launch_gx_pipe(const qrnnt_lstm *L, const int8_t *x_codes, int M, int32_t *gx, int32_t *dbg_accx, hipStream_t st)
{
    using P = QrPipe<MT, NT, S, W8>;
    const int H = L->hidden_size, I = L->input_size;
    const int n_row_tiles = H >> 2;
    const int nkc = qr_round_up(I, QRNNT_KCHUNK) / QRNNT_KCHUNK;
    const int nbx = (n_row_tiles + 2 * MT - 1) / (2 * MT), nby = (M + P::BN - 1) / P::BN;
    dim3 grid((unsigned)(nbx * 8 * ((nby + 7) / 8)));
    static std::atomic<bool> configured[QR_MAX_DEVICES];
    const int dev = qr_current_device();
    if (!configured[dev].load(std::memory_order_relaxed)) {
        (void)hipFuncSetAttribute((const void *)gx_gemm_pipe_kernel<MT, NT, S, true, W8>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, P::LDS_BYTES);
        (void)hipFuncSetAttribute((const void *)gx_gemm_pipe_kernel<MT, NT, S, false, W8>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, P::LDS_BYTES);
        configured[dev].store(true, std::memory_order_relaxed);
    }
    const int64_t ld_x = qr_act_pitch(I);
    if (I % QRNNT_KCHUNK)
        gx_gemm_pipe_kernel<MT, NT, S, true, W8><<<grid, 256, P::LDS_BYTES, st>>>((const v4i *)L->w_ih.packed, nkc, n_row_tiles,
                                                                                 x_codes, ld_x, M, I, gx, H, dbg_accx);
    else
        gx_gemm_pipe_kernel<MT, NT, S, false, W8><<<grid, 256, P::LDS_BYTES, st>>>((const v4i *)L->w_ih.packed, nkc, n_row_tiles,
                                                                                  x_codes, ld_x, M, I, gx, H, dbg_accx);
}

// fp32 form of a precomputed input projection: tab[m, r'] = k * (x_scale * s_wih[r] * gx[m, r'] + bias[r]),
// r' the TILED_GATES position of source row r, k the exp2 constant of the row's gate.
__global__ void gx_table_kernel(const int32_t *__restrict__ gx, const float *__restrict__ s_wih,
                                const float *__restrict__ bias, float x_scale, int H, size_t n, float *__restrict__ tab)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n) return;
    const int tr = (int)(idx % (size_t)(4 * H));
    const int gt = tr & 3, j = qr_gates_cell(tr >> 4, (tr & 15) >> 2);
    const float k = gt == 2 ? -2.885390081777927f : -1.4426950408889634f;
    const int r = gt * H + j;
    tab[idx] = (s_wih[r] * x_scale * k) * (float)gx[idx] + bias[r] * k;
}

__global__ void fill_zero_kernel(uint32_t *p, size_t n_words)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) p[i] = 0u;
}

}  // namespace

qrnnt_status qr_check_lstm(const qrnnt_lstm *L)
{
    QR_REQUIRE(L != nullptr, QRNNT_ERR_NULL);
    qrnnt_status s = qr_check_qmat(&L->w_ih, QRNNT_LAYOUT_TILED_GATES);
    if (s != QRNNT_OK) return s;
    s = qr_check_qmat(&L->w_hh, QRNNT_LAYOUT_TILED_GATES);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(L->bias != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(qr_aligned(L->bias, 16) && qr_aligned(L->w_ih.row_scale, 16) && qr_aligned(L->w_hh.row_scale, 16),
               QRNNT_ERR_ALIGN);
    QR_REQUIRE(L->input_size > 0 && L->hidden_size > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(L->hidden_size % 16 == 0, QRNNT_ERR_SHAPE);   // any input size: its rows are stored with a pitch of qr_act_pitch
    QR_REQUIRE(L->w_ih.rows == 4 * L->hidden_size && L->w_hh.rows == 4 * L->hidden_size, QRNNT_ERR_SHAPE);
    QR_REQUIRE(L->w_ih.cols == L->input_size && L->w_hh.cols == L->hidden_size, QRNNT_ERR_SHAPE);
    QR_REQUIRE(L->x_scale > 0.0f && L->h_scale > 0.0f && L->h_inv_scale > 0.0f, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_bits(&L->w_ih) == qr_bits(&L->w_hh), QRNNT_ERR_RANGE);
    return QRNNT_OK;
}

void qr_launch_gx_table(const qrnnt_lstm *L, const int32_t *gx, int M, float *tab, hipStream_t st)
{
    const size_t n = (size_t)M * 4 * L->hidden_size;
    gx_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(gx, L->w_ih.row_scale, L->bias, L->x_scale, L->hidden_size, n,
                                                                  tab);
}

void qr_fill_lstm_weights(QrStepArgs &a, const qrnnt_lstm *L)
{
    a.wih = (const v4i *)L->w_ih.packed;
    a.whh = (const v4i *)L->w_hh.packed;
    a.s_wih = L->w_ih.row_scale;
    a.s_whh = L->w_hh.row_scale;
    a.bias = L->bias;
    a.I = L->input_size;
    a.H = L->hidden_size;
    a.nkc_x = qr_round_up(L->input_size, QRNNT_KCHUNK) / QRNNT_KCHUNK;
    a.nkc_h = qr_round_up(L->hidden_size, QRNNT_KCHUNK) / QRNNT_KCHUNK;
    a.x_scale = L->x_scale;
    a.h_scale = L->h_scale;
    a.h_inv = L->h_inv_scale;
}

void qr_launch_lstm_step(const QrStepArgs &a, bool use_gx, hipStream_t st)
{
    if (use_gx) launch_step_t<true>(a, st); else launch_step_t<false>(a, st);
}

template <bool USE_GX>
static void launch_group_t(const QrStepGroup &g, hipStream_t st)
{
    // one launch when every member is in the compute-bound regime, else member by member
    bool all_big = true, all_small = true;
    for (int i = 0; i < g.n; ++i) {
        all_big = all_big && g.p[i].N > small_n_max();
        all_small = all_small && g.p[i].N <= small_n_max();
    }
    if (all_big) launch_pipe<4, 4, USE_GX ? 2 : 3, USE_GX>(g, st);
    else if (all_small) launch_small<USE_GX>(g, st);
    else
        for (int i = 0; i < g.n; ++i) launch_step_t<USE_GX>(g.p[i], st);
}

void qr_launch_lstm_step_group(const QrStepGroup &g, bool use_gx, hipStream_t st)
{
    if (use_gx) launch_group_t<true>(g, st); else launch_group_t<false>(g, st);
}

static qrnnt_status make_step_args(QrStepArgs &a, const qrnnt_lstm *L, const int8_t *x_codes, const int32_t *x_row,
                                   int32_t n_x_rows, const int32_t *parent, const int8_t *h_prev, const float *c_prev,
                                   int32_t n_slots, const uint8_t *active, int32_t N, int8_t *h_next, float *c_next)
{
    qrnnt_status s = qr_check_lstm(L);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(qr_bits(&L->w_hh) == 4, QRNNT_ERR_UNSUPPORTED);   // the step kernels unpack nibbles
    QR_REQUIRE(x_codes && h_prev && c_prev && h_next && c_next, QRNNT_ERR_NULL);
    QR_REQUIRE(N > 0 && n_slots > 0 && n_x_rows > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(parent != nullptr || n_slots >= N, QRNNT_ERR_SHAPE);
    QR_REQUIRE(x_row != nullptr || n_x_rows >= N, QRNNT_ERR_SHAPE);
    QR_REQUIRE(qr_aligned(x_codes, 16) && qr_aligned(h_prev, 16), QRNNT_ERR_ALIGN);
    QR_REQUIRE(qr_aligned(c_prev, 16) && qr_aligned(c_next, 16) && qr_aligned(h_next, 4), QRNNT_ERR_ALIGN);
    QR_REQUIRE((const void *)h_next != (const void *)h_prev && c_next != c_prev, QRNNT_ERR_RANGE);
    a = QrStepArgs{};
    qr_fill_lstm_weights(a, L);
    a.x = x_codes;  a.ld_x = qr_act_pitch(L->input_size);  a.x_row = x_row;  a.n_x_rows = n_x_rows;
    a.parent = parent;  a.n_slots = n_slots;
    a.h_prev = h_prev;  a.ld_hp = L->hidden_size;  a.c_prev = c_prev;  a.active = active;
    a.h_next = h_next;  a.ld_hn = L->hidden_size;  a.c_next = c_next;
    a.N = N;
    return QRNNT_OK;
}

extern "C" qrnnt_status qrnnt_lstm_step(const qrnnt_lstm *L, const int8_t *x_codes, const int32_t *x_row,
                                        int32_t n_x_rows, const int32_t *parent, const int8_t *h_prev,
                                        const float *c_prev, int32_t n_slots, const uint8_t *active, int32_t N,
                                        int8_t *h_next, float *c_next, int32_t *dbg_accx, int32_t *dbg_acch,
                                        float *dbg_gates, void *stream)
{
    QrStepArgs a;
    qrnnt_status s = make_step_args(a, L, x_codes, x_row, n_x_rows, parent, h_prev, c_prev, n_slots, active, N, h_next,
                                    c_next);
    if (s != QRNNT_OK) return s;
    a.dbg_accx = dbg_accx;  a.dbg_acch = dbg_acch;  a.dbg_gates = dbg_gates;
    qr_launch_lstm_step(a, false, (hipStream_t)stream);
    return qr_launch_status();
}

namespace {

qrnnt_status step_group(const qrnnt_step_desc *steps, int32_t n_steps, const int32_t *list, const int32_t *n_list,
                        void *stream)
{
    QR_REQUIRE(steps != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(n_steps >= 1 && n_steps <= QR_MAX_GROUP, QRNNT_ERR_RANGE);
    QrStepGroup g;
    g.n = n_steps;
    g.gate = nullptr;
    g.rows = (const v4i *)list;
    g.n_rows = n_list;
    if (list)   // one list serves all members: same number of hypotheses, same use of parent and x_row
        for (int i = 1; i < n_steps; ++i)
            QR_REQUIRE(steps[i].N == steps[0].N && (steps[i].parent != nullptr) == (steps[0].parent != nullptr) &&
                           (steps[i].x_row != nullptr) == (steps[0].x_row != nullptr),
                       QRNNT_ERR_RANGE);
    for (int i = 0; i < n_steps; ++i) {
        const qrnnt_step_desc &d = steps[i];
        qrnnt_status s = make_step_args(g.p[i], d.L, d.x_codes, d.x_row, d.n_x_rows, d.parent, d.h_prev, d.c_prev,
                                        d.n_slots, d.active, d.N, d.h_next, d.c_next);
        if (s != QRNNT_OK) return s;
        QR_REQUIRE((d.gx != nullptr) == (steps[0].gx != nullptr), QRNNT_ERR_RANGE);
        QR_REQUIRE(qr_aligned(d.gx, 16), QRNNT_ERR_ALIGN);
        QR_REQUIRE(d.gx_table == nullptr || d.gx != nullptr, QRNNT_ERR_NULL);
        QR_REQUIRE(qr_aligned(d.gx_table, 16), QRNNT_ERR_ALIGN);
        g.p[i].gx = d.gx;  g.p[i].ld_gx = 4 * (int64_t)d.L->hidden_size;  g.p[i].tabf = d.gx_table;
        g.p[i].dbg_accx = d.dbg_accx;  g.p[i].dbg_acch = d.dbg_acch;  g.p[i].dbg_gates = d.dbg_gates;
    }
    qr_launch_lstm_step_group(g, steps[0].gx != nullptr, (hipStream_t)stream);
    return qr_launch_status();
}

}  // namespace

extern "C" qrnnt_status qrnnt_lstm_step_group(const qrnnt_step_desc *steps, int32_t n_steps, void *stream)
{
    return step_group(steps, n_steps, nullptr, nullptr, stream);
}

extern "C" qrnnt_status qrnnt_lstm_step_group_listed(const qrnnt_step_desc *steps, int32_t n_steps, const int32_t *list,
                                                     const int32_t *n_list, void *stream)
{
    QR_REQUIRE(list != nullptr && n_list != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(qr_aligned(list, 16) && qr_aligned(n_list, 4), QRNNT_ERR_ALIGN);
    return step_group(steps, n_steps, list, n_list, stream);
}

void qr_launch_input_projection(const qrnnt_lstm *L, const int8_t *x_codes, int M, int32_t *gx, int32_t *dbg_accx,
                                hipStream_t st)
{
    // 128 x 128 block tile; two ring stages leave room for a third workgroup per CU, which at many
    // frames is worth more than a deeper ring (measured: 69 vs 74 us at 16000 x 1280 x 2560)
    if (qr_bits(&L->w_ih) == 8) launch_gx_pipe<4, 4, 2, true>(L, x_codes, M, gx, dbg_accx, st);   // 8-bit layer (the encoder's first)
    else if (M <= 256) launch_gx_pipe<4, 4, 3, false>(L, x_codes, M, gx, dbg_accx, st);
    else launch_gx_pipe<4, 4, 2, false>(L, x_codes, M, gx, dbg_accx, st);
}

extern "C" qrnnt_status qrnnt_input_table(const qrnnt_lstm *L, const int32_t *gx, int32_t M, float *table, void *stream)
{
    qrnnt_status s = qr_check_lstm(L);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(gx && table, QRNNT_ERR_NULL);
    QR_REQUIRE(M > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(qr_aligned(gx, 16) && qr_aligned(table, 16), QRNNT_ERR_ALIGN);
    qr_launch_gx_table(L, gx, M, table, (hipStream_t)stream);
    return qr_launch_status();
}

extern "C" qrnnt_status qrnnt_input_projection(const qrnnt_lstm *L, const int8_t *x_codes, int32_t M, int32_t *gx,
                                               int32_t *dbg_accx, void *stream)
{
    qrnnt_status s = qr_check_lstm(L);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(x_codes && gx, QRNNT_ERR_NULL);
    QR_REQUIRE(M > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(qr_aligned(x_codes, 16) && qr_aligned(gx, 16), QRNNT_ERR_ALIGN);
    qr_launch_input_projection(L, x_codes, M, gx, dbg_accx, (hipStream_t)stream);
    return qr_launch_status();
}

// Workspace layout of one layer-direction:
//   int32 gx [T*B, 4H] | h state 2 x [B,H] int8 | c state 2 x [B,H] fp32 |
//   exchange words of the persistent recurrence | error flag
struct LayerWs {
    size_t gx_b, h_b, c_b, x_b, total;
};
static LayerWs layer_ws(const qrnnt_lstm *L, int T, int B)
{
    LayerWs w;
    const size_t H = (size_t)L->hidden_size;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    w.gx_b = up((size_t)T * B * 4 * H * sizeof(int32_t));
    w.h_b = up((size_t)B * H);
    w.c_b = up((size_t)B * H * sizeof(float));
    w.x_b = up(qr_rec_xbuf_bytes((int)H, B));
    w.total = w.gx_b + 2 * w.h_b + 2 * w.c_b + w.x_b + 256;
    return w;
}

extern "C" size_t qrnnt_lstm_layer_workspace(const qrnnt_lstm *L, int32_t T, int32_t B)
{
    if (L == nullptr || T <= 0 || B <= 0 || L->hidden_size <= 0) return 0;
    return layer_ws(L, T, B).total;
}

namespace {

struct LayerCall {
    const qrnnt_lstm *L;
    int reverse;
    const int8_t *h0;  const float *c0;
    int col_off;
    int8_t *h_last;  float *c_last;
    int32_t *dbg_accx;  float *dbg_c_all;
    char *ws;
};

qrnnt_status check_layer_call(const LayerCall &c, const int8_t *x_codes, int T, int B, const int8_t *h_out, int ld_out)
{
    qrnnt_status s = qr_check_lstm(c.L);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(x_codes && h_out && c.ws, QRNNT_ERR_NULL);
    QR_REQUIRE(T > 0 && B > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(c.col_off >= 0 && ld_out >= c.col_off + c.L->hidden_size, QRNNT_ERR_SHAPE);
    QR_REQUIRE(ld_out % 16 == 0 && c.col_off % 16 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(qr_aligned(x_codes, 16) && qr_aligned(h_out, 16) && qr_aligned(c.ws, 256), QRNNT_ERR_ALIGN);
    QR_REQUIRE(c.h0 == nullptr || qr_aligned(c.h0, 16), QRNNT_ERR_ALIGN);
    return QRNNT_OK;
}

// 1 or 2 directions over the same input: projections, then either the persistent
// recurrence (both directions in one launch) or one fused launch per time step.
qrnnt_status run_layer(const LayerCall *calls, int n, const int8_t *x_codes, int T, int B, int8_t *h_out, int ld_out,
                       hipStream_t st)
{
    const int H = calls[0].L->hidden_size;
    bool persist = qr_rec_supported(H, B);
    for (int d = 1; d < n; ++d) persist = persist && calls[d].L->hidden_size == H;
    bool any8 = false;
    for (int d = 0; d < n; ++d) any8 = any8 || qr_bits(&calls[d].L->w_hh) == 8;
    QR_REQUIRE(!any8 || persist, QRNNT_ERR_UNSUPPORTED);   // 8-bit layers run in the persistent recurrence only
    QrRecGroup rg;
    rg.n = n;
    for (int d = 0; d < n; ++d) {
        const LayerCall &c = calls[d];
        const qrnnt_lstm *L = c.L;
        const LayerWs w = layer_ws(L, T, B);
        int32_t *gx = (int32_t *)c.ws;
        qr_launch_input_projection(L, x_codes, T * B, gx, c.dbg_accx, st);
        if (persist) {
            char *xb = c.ws + w.gx_b + 2 * w.h_b + 2 * w.c_b;
            const size_t nw = (w.x_b + 256) / 4;
            fill_zero_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)xb, nw);
            QrRecArgs &a = rg.d[d];
            a = QrRecArgs{};
            a.whh = (const v4i *)L->w_hh.packed;  a.s_wih = L->w_ih.row_scale;  a.s_whh = L->w_hh.row_scale;
            a.bias = L->bias;  a.gx = gx;  a.h0 = c.h0;  a.c0 = c.c0;
            a.h_out = h_out;  a.ld_out = ld_out;  a.col_off = c.col_off;
            a.h_last = c.h_last;  a.c_last = c.c_last;  a.dbg_c_all = c.dbg_c_all;
            a.xbuf = (unsigned long long *)xb;  a.err = (int *)(xb + w.x_b);
            a.T = T;  a.B = B;  a.H = H;  a.nkc_h = qr_round_up(H, QRNNT_KCHUNK) / QRNNT_KCHUNK;
            a.reverse = c.reverse;  a.spin_limit = 1 << 18;
            a.x_scale = L->x_scale;  a.h_scale = L->h_scale;  a.h_inv = L->h_inv_scale;
            a.w8 = qr_bits(&L->w_hh) == 8;
        }
    }
    if (persist && qr_launch_recurrence(rg, st)) return qr_launch_status();
    QR_REQUIRE(!any8, QRNNT_ERR_UNSUPPORTED);
    for (int d = 0; d < n; ++d) {
        const LayerCall &c = calls[d];
        const qrnnt_lstm *L = c.L;
        const LayerWs w = layer_ws(L, T, B);
        int32_t *gx = (int32_t *)c.ws;
        int8_t *hbuf = (int8_t *)(c.ws + w.gx_b);
        float *cbuf[2] = {(float *)(c.ws + w.gx_b + 2 * w.h_b), (float *)(c.ws + w.gx_b + 2 * w.h_b + w.c_b)};
        if (c.h0 == nullptr) {
            const size_t nw = w.h_b / 4;
            fill_zero_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)hbuf, nw);
        }
        if (c.c0 == nullptr) {
            const size_t nw = w.c_b / 4;
            fill_zero_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)cbuf[0], nw);
        }
        QrStepArgs a = {};
        qr_fill_lstm_weights(a, L);
        a.ld_gx = 4 * (int64_t)H;
        a.n_x_rows = B;   // rows of the step's slice of gx (row indices are clamped into [0, n_x_rows))
        a.n_slots = B;
        a.N = B;
        a.ld_hn = ld_out;
        const float *c_prev = c.c0 ? c.c0 : cbuf[0];
        int cur = c.c0 ? 0 : 1;   // next c buffer to write
        for (int step = 0; step < T; ++step) {
            const int t = c.reverse ? T - 1 - step : step;
            a.gx = gx + (int64_t)t * B * 4 * H;
            if (step == 0) {
                a.h_prev = c.h0 ? c.h0 : hbuf;
                a.ld_hp = H;
            } else {
                const int tp = c.reverse ? t + 1 : t - 1;
                a.h_prev = h_out + (int64_t)tp * B * ld_out + c.col_off;
                a.ld_hp = ld_out;
            }
            a.c_prev = c_prev;
            a.c_next = c.dbg_c_all ? c.dbg_c_all + (int64_t)t * B * H : cbuf[cur];
            a.h_next = h_out + (int64_t)t * B * ld_out + c.col_off;
            a.h_copy = (step == T - 1) ? c.h_last : nullptr;
            qr_launch_lstm_step(a, true, st);
            c_prev = a.c_next;
            cur ^= 1;
        }
        if (c.c_last)
            (void)hipMemcpyAsync(c.c_last, c_prev, (size_t)B * H * sizeof(float), hipMemcpyDeviceToDevice, st);
    }
    return qr_launch_status();
}

}  // namespace

extern "C" qrnnt_status qrnnt_lstm_layer(const qrnnt_lstm *L, const int8_t *x_codes, int32_t T, int32_t B,
                                         int32_t reverse, const int8_t *h0, const float *c0, int8_t *h_out,
                                         int32_t ld_out, int32_t col_off, int8_t *h_last, float *c_last,
                                         int32_t *dbg_accx, float *dbg_c_all, void *workspace, size_t workspace_bytes,
                                         void *stream)
{
    LayerCall c = {L, reverse, h0, c0, col_off, h_last, c_last, dbg_accx, dbg_c_all, (char *)workspace};
    qrnnt_status s = check_layer_call(c, x_codes, T, B, h_out, ld_out);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(workspace_bytes >= layer_ws(L, T, B).total, QRNNT_ERR_WORKSPACE);
    return run_layer(&c, 1, x_codes, T, B, h_out, ld_out, (hipStream_t)stream);
}

extern "C" size_t qrnnt_bilstm_layer_workspace(const qrnnt_lstm *fwd, const qrnnt_lstm *bwd, int32_t T, int32_t B)
{
    const size_t a = qrnnt_lstm_layer_workspace(fwd, T, B), b = qrnnt_lstm_layer_workspace(bwd, T, B);
    return (a == 0 || b == 0) ? 0 : a + b;
}

extern "C" qrnnt_status qrnnt_bilstm_layer(const qrnnt_lstm *fwd, const qrnnt_lstm *bwd, const int8_t *x_codes, int32_t T,
                                           int32_t B, int8_t *h_out, void *workspace, size_t workspace_bytes, void *stream)
{
    QR_REQUIRE(fwd && bwd, QRNNT_ERR_NULL);
    QR_REQUIRE(fwd->hidden_size > 0 && fwd->hidden_size == bwd->hidden_size && fwd->input_size == bwd->input_size,
               QRNNT_ERR_SHAPE);
    const int H = fwd->hidden_size;
    LayerCall c[2] = {{fwd, 0, nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, (char *)workspace},
                      {bwd, 1, nullptr, nullptr, H, nullptr, nullptr, nullptr, nullptr, nullptr}};
    if (T > 0 && B > 0 && workspace) c[1].ws = (char *)workspace + layer_ws(fwd, T, B).total;
    for (int d = 0; d < 2; ++d) {
        qrnnt_status s = check_layer_call(c[d], x_codes, T, B, h_out, 2 * H);
        if (s != QRNNT_OK) return s;
    }
    QR_REQUIRE(workspace_bytes >= layer_ws(fwd, T, B).total + layer_ws(bwd, T, B).total, QRNNT_ERR_WORKSPACE);
    return run_layer(c, 2, x_codes, T, B, h_out, 2 * H, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------------------
// qrnnt_lstm_layer for callers that cannot allocate device memory: the workspace of the layer (input projection
// sums, state buffers, exchange words of the persistent recurrence) lives in a file-scope device array.  Every
// device the library runs on holds its own copy of the array at its own address; the host gets that address once
// per device from the runtime and hands it to the same code path that qrnnt_lstm_layer takes with a caller's
// workspace.  The array keeps the previous call's contents: run_layer clears what has to start at zero (exchange
// words and error flag, zero initial state) on the stream before it is read.
#define QR_STATIC_WS_BYTES ((size_t)QRNNT_STATIC_WORKSPACE_BYTES)
static __device__ __align__(256) unsigned char scratch[QR_STATIC_WS_BYTES];

namespace {
std::mutex scratch_mutex;
void *scratch_ptr[QR_MAX_DEVICES];   // per device: address of `scratch` on that device (nullptr: not asked yet)

// Device address of the scratch array on the device that is current on the calling thread.
qrnnt_status static_scratch(char **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= QR_MAX_DEVICES) return QRNNT_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[dev] == nullptr) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return QRNNT_ERR_HIP;
        scratch_ptr[dev] = p;
    }
    *out = (char *)scratch_ptr[dev];
    return QRNNT_OK;
}
}  // namespace

extern "C" qrnnt_status qrnnt_lstm_layer_static(const qrnnt_lstm *L, const int8_t *x_codes, int32_t T, int32_t B,
                                                int32_t reverse, const int8_t *h0, const float *c0, int8_t *h_out,
                                                int32_t ld_out, int32_t col_off, int8_t *h_last, float *c_last,
                                                void *stream)
{
    // validation first (needs no GPU): a dummy non-null workspace address stands in until the size is known to fit
    LayerCall c = {L, reverse, h0, c0, col_off, h_last, c_last, nullptr, nullptr, (char *)(uintptr_t)256};
    qrnnt_status s = check_layer_call(c, x_codes, T, B, h_out, ld_out);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(layer_ws(L, T, B).total <= QR_STATIC_WS_BYTES, QRNNT_ERR_WORKSPACE);
    s = static_scratch(&c.ws);
    if (s != QRNNT_OK) return s;
    return run_layer(&c, 1, x_codes, T, B, h_out, ld_out, (hipStream_t)stream);
}
