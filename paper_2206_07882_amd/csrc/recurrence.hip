// The time loop of an LSTM layer as one persistent kernel (Sec. 3.4: the hidden
// state is quantized once at the cell output and that code feeds the next step).
//
// The recurrence is a chain of T dependent steps, each far too small to fill the
// GPU, so its cost is the latency of one step, not arithmetic.  Design:
//   - a workgroup owns 16 cells (64 gate rows = 4 row tiles) x 16 utterances of one
//     direction for all T steps.  Utterances never interact, so hidden codes are
//     exchanged only among the H/16 workgroups of the same utterance group;
//   - the K dimension of W_hh is dealt to the 4 waves in 64-column steps; each wave
//     keeps its share of the workgroup's weight rows in registers, already unpacked
//     to int8 MFMA operands, for the whole sequence.  Partial sums meet in LDS and
//     wave w then finishes row tile w: one cell x one utterance per lane, cell state
//     in a register;
//   - the 4-bit codes of h_t travel through a double-buffered exchange area in 8-byte
//     words {4 codes, step tag}, laid out so that a wave reads each of its K steps
//     as one contiguous 2 KiB run.  A consumer knows a word is current when its tag
//     matches: no grid barrier, no atomic and no fence on the critical path (data and
//     flag arrive in the same store);
//   - both directions of a bidirectional layer run in the same launch.
// All workgroups must be co-resident (checked against the occupancy of the device
// before the launch); a wait is bounded by spin_limit polls, after which the error
// flag is set and the workgroup leaves the loop, so the grid always drains.
#include <hip/hip_runtime.h>

#include <atomic>

#include "kernels.h"

namespace {

typedef unsigned long long u64;

// Two exchange words per 128-bit load, bypassing the non-coherent cache levels.
// p[k] is the lane's address for its k-th K step.
template <int KW>
__device__ __forceinline__ void ll_load_frags(const v4i *const (&p)[KW], v4i (&lo)[KW], v4i (&hi)[KW])
{
#pragma unroll
    for (int k = 0; k < KW; ++k) {
        asm volatile("global_load_dwordx4 %0, %2, off sc0 sc1\n\t"
                     "global_load_dwordx4 %1, %2, off offset:16 sc0 sc1"
                     : "=&v"(lo[k]), "=&v"(hi[k])
                     : "v"(p[k])
                     : "memory");
    }
    // every output is an operand of the wait, so no consumer can be scheduled before it
    if constexpr (KW == 1) asm volatile("s_waitcnt vmcnt(0)" : "+v"(lo[0]), "+v"(hi[0])::"memory");
    if constexpr (KW == 2)
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(lo[0]), "+v"(hi[0]), "+v"(lo[1]), "+v"(hi[1])::"memory");
    if constexpr (KW == 3)
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+v"(lo[0]), "+v"(hi[0]), "+v"(lo[1]), "+v"(hi[1]), "+v"(lo[2]), "+v"(hi[2])::"memory");
    if constexpr (KW == 4)
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+v"(lo[0]), "+v"(hi[0]), "+v"(lo[1]), "+v"(hi[1]), "+v"(lo[2]), "+v"(hi[2]), "+v"(lo[3]),
                       "+v"(hi[3])::"memory");
}

__device__ __forceinline__ void ll_store(u64 *p, u64 v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Exchange layout: [parity][utterance group][K step][lane = 16*grp + col][4 words];
// word q of lane (grp, col) of K step ks holds cells 64*ks + 16*grp + 4*q .. +3 of
// utterance 16*ug + col.
// KW: K steps per wave (H <= 256*KW).
// CT: 16-cell groups per workgroup (1 or 2).  A workgroup of CT = 2 owns 32 cells (8 row tiles, two per wave in the
// epilogue) and so halves the number of workgroups of a launch: used when CT = 1 would ask for more workgroups than
// the device has compute units (two workgroups sharing a CU take turns, and every step then waits for the slower
// ones), e.g. 64 utterances x 640 cells x 2 directions = 320 workgroups on 256 CUs.  H must be a multiple of 16*CT.
template <int KW, int CT>
__global__ __launch_bounds__(256) void lstm_rec_kernel(const QrRecGroup g)
{
    constexpr int RT = 4 * CT;             // row tiles (of 4 cells x 4 gates) per workgroup
    __shared__ v4i part[4][RT][64];    // [wave][row tile][lane] partial sums
    __shared__ __attribute__((aligned(16))) int8_t hc[16][16 * CT]; // [utterance][cell] codes of this step (read back as 32-bit words)
    __shared__ int s_fail;
    const QrRecArgs &a = g.d[blockIdx.z];
    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, grp = lane >> 4;
    const int cg = blockIdx.x, ug = blockIdx.y;
    const int nks = (H + 63) >> 6;              // K steps in total (the layout pads to whole steps)
    const v4i zero = {0, 0, 0, 0};
    const int m = (int)0xF0F0F0F0u;

    // ---- stationary operands: this wave's K steps of the workgroup's row tiles
    v4i A[RT][KW];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int k = 0; k < KW; ++k) {
            const int ks = wave + 4 * k;
            A[rt][k] = zero;
            if (ks < nks) {
                if (a.w8) {   // 8-bit layer: the operand as stored, two blocks per 128-column chunk
                    A[rt][k] = a.whh[(((size_t)(cg * RT + rt) * a.nkc_h + (ks >> 1)) * 2 + (ks & 1)) * 64 + lane];
                } else {
                    const v4i p = a.whh[((size_t)(cg * RT + rt) * a.nkc_h + (ks >> 1)) * 64 + lane];
                    A[rt][k] = (ks & 1) ? (p & m) : ((p << 4) & m);
                }
            }
        }
    // ---- the cells this lane finishes: row tiles 4*c + wave (c < CT), cell j[c], utterance n
    const int n = ug * 16 + col;
    const int nn = n < B ? n : B - 1;
    int j[CT];
    float sx[CT][4], sh[CT][4], bb[CT][4], c[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        j[ct] = qr_gates_cell(cg * RT + 4 * ct + wave, grp);   // = 16*(CT*cg + ct) + 4*grp + wave
#pragma unroll
        for (int gt = 0; gt < 4; ++gt) {
            sx[ct][gt] = a.x_scale * a.s_wih[gt * H + j[ct]];
            sh[ct][gt] = a.h_scale * a.s_whh[gt * H + j[ct]];
            bb[ct][gt] = a.bias[gt * H + j[ct]];
        }
        c[ct] = a.c0 ? a.c0[(int64_t)nn * H + j[ct]] : 0.0f;
    }
    if (tid == 0) s_fail = 0;
    __syncthreads();

    const size_t xgroup = (size_t)nks * 64 * 4;                    // words per (parity, utterance group)
    const size_t xparity = (size_t)((B + 15) >> 4) * xgroup;
    for (int s = 0; s < T; ++s) {
        const int t = a.reverse ? T - 1 - s : s;
        v4i gxv[CT];   // independent of h: first
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
            gxv[ct] = *(const v4i *)(a.gx + ((int64_t)t * B + nn) * 4 * H + (cg * RT + 4 * ct + wave) * 16 + 4 * grp);
        v4i acc[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) acc[rt] = zero;
        bool failed = false;
        if (s > 0 || a.h0) {
            v4i bf[KW];
            if (s == 0) {
                const int8_t *hr = a.h0 + (int64_t)nn * H + grp * 16;
#pragma unroll
                for (int k = 0; k < KW; ++k) {
                    const int ks = wave + 4 * k;
                    bf[k] = (ks * 64 + grp * 16 < H) ? *(const v4i *)(hr + ks * 64) : zero;
                }
            } else {
                // words written at step s-1 carry tag s; this wave's K steps are 4 steps (= 4*64*2 v4i) apart
                const u64 *xw = a.xbuf + (size_t)((s - 1) & 1) * xparity + (size_t)ug * xgroup;
                const v4i *src[KW];
#pragma unroll
                for (int k = 0; k < KW; ++k) {
                    const int ks = wave + 4 * k < nks ? wave + 4 * k : 0;   // absent steps re-read step 0 (ignored)
                    src[k] = (const v4i *)(xw + ((size_t)ks * 64 + lane) * 4);
                }
                const int want = s;
                int spins = 0;
                while (true) {
                    v4i lo[KW], hi[KW];
                    ll_load_frags<KW>(src, lo, hi);
                    bool ok = true;
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        const int ks = wave + 4 * k;
                        if (ks < nks) {
                            const bool in = ks * 64 + grp * 16 < H;
                            ok = ok && (!in || (lo[k][1] == want && lo[k][3] == want && hi[k][1] == want && hi[k][3] == want));
                            bf[k] = in ? v4i{lo[k][0], lo[k][2], hi[k][0], hi[k][2]} : zero;
                        } else {
                            bf[k] = zero;
                        }
                    }
                    if (__all(ok)) break;
                    if (++spins > a.spin_limit) { failed = true; break; }
                }
            }
#pragma unroll
            for (int k = 0; k < KW; ++k)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) acc[rt] = qr_mfma(A[rt][k], bf[k], acc[rt]);
        }
        if (failed && lane == 0) {
            atomicExch(a.err, 1);
            s_fail = 1;
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) part[wave][rt][lane] = acc[rt];
        __syncthreads();
        const int fail_now = s_fail;   // written only before this barrier, read only after it: uniform
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const int rt = 4 * ct + wave;
            const v4i asum = part[0][rt][lane] + part[1][rt][lane] + part[2][rt][lane] + part[3][rt][lane];
            const v4i ah = a.w8 ? asum : (asum >> 4);   // 4-bit operands carry a factor 16
            float p[4];
#pragma unroll
            for (int gt = 0; gt < 4; ++gt) p[gt] = sx[ct][gt] * (float)gxv[ct][gt] + (sh[ct][gt] * (float)ah[gt] + bb[ct][gt]);
            const float gi = qr_sigmoid(p[0]), gf = qr_sigmoid(p[1]), gg = qr_tanh(p[2]), go = qr_sigmoid(p[3]);
            c[ct] = gf * c[ct] + gi * gg;
            const float h = go * qr_tanh(c[ct]);
            hc[col][16 * ct + grp * 4 + wave] = (int8_t)qr_quant(h, a.h_inv, a.w8 ? 8 : 4);
            if (a.dbg_c_all && n < B) a.dbg_c_all[((int64_t)t * B + n) * H + j[ct]] = c[ct];
        }
        __syncthreads();
        // publish: 16 utterances x 4*CT quads, one 8-byte word each, tagged s+1
        if (tid < 64 * CT) {
            const int u = tid & 15, q = tid >> 4;       // quad q of the workgroup's 4*CT: cells 4*q .. 4*q+3 of its 16*CT
            const int Q = cg * RT + q;                  // quad of the layer
            const unsigned data = *(const unsigned *)&hc[u][q * 4];
            u64 *dst = a.xbuf + (size_t)(s & 1) * xparity + (size_t)ug * xgroup +
                       ((size_t)(Q >> 4) * 64 + ((Q & 15) >> 2) * 16 + u) * 4 + (Q & 3);
            ll_store(dst, ((u64)(unsigned)(s + 1) << 32) | data);
            const int nu = ug * 16 + u;
            if (nu < B) {
                *(unsigned *)(a.h_out + ((int64_t)t * B + nu) * a.ld_out + a.col_off + 4 * Q) = data;
                if (s == T - 1 && a.h_last) *(unsigned *)(a.h_last + (int64_t)nu * H + 4 * Q) = data;
            }
        }
        if (fail_now) break;
    }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
        if (a.c_last && n < B) a.c_last[(int64_t)n * H + j[ct]] = c[ct];
}

template <int KW, int CT>
bool launch_rec_ct(const QrRecGroup &g, bool only_if_it_fits_the_cus, hipStream_t st)
{
    const int H = g.d[0].H, B = g.d[0].B;
    if (H % (16 * CT) != 0) return false;
    dim3 grid(H / (16 * CT), (B + 15) / 16, g.n);
    // every workgroup spins on its peers: all of them must fit on the device at once
    static std::atomic<long long> resident_of[QR_MAX_DEVICES];   // workgroups the device holds at once; 0: not asked yet
    static std::atomic<int> n_cu_of[QR_MAX_DEVICES];
    const int dev = qr_current_device();
    long long resident = resident_of[dev].load(std::memory_order_relaxed);
    int n_cu = n_cu_of[dev].load(std::memory_order_relaxed);
    if (resident == 0) {
        int per_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, lstm_rec_kernel<KW, CT>, 256, 0) != hipSuccess) return false;
        resident = (long long)per_cu * n_cu;
        if (resident <= 0 || n_cu <= 0) return false;
        n_cu_of[dev].store(n_cu, std::memory_order_relaxed);
        resident_of[dev].store(resident, std::memory_order_relaxed);
    }
    const long long wgs = (long long)grid.x * grid.y * grid.z;
    if (wgs > resident) return false;
    if (only_if_it_fits_the_cus && wgs > n_cu) return false;
    lstm_rec_kernel<KW, CT><<<grid, 256, 0, st>>>(g);
    return true;
}

// One workgroup per compute unit if either form allows it (16 cells each, else 32 cells each); otherwise whichever
// form is resident at all, fewest workgroups sharing a CU first.
template <int KW>
bool launch_rec_t(const QrRecGroup &g, hipStream_t st)
{
    if (launch_rec_ct<KW, 1>(g, true, st)) return true;
    if (launch_rec_ct<KW, 2>(g, true, st)) return true;
    if (launch_rec_ct<KW, 2>(g, false, st)) return true;
    return launch_rec_ct<KW, 1>(g, false, st);
}

}  // namespace

bool qr_rec_supported(int H, int B) { return H % 16 == 0 && H <= 1024 && B >= 1; }

size_t qr_rec_xbuf_bytes(int H, int B)
{
    return (size_t)2 * ((B + 15) / 16) * ((H + 63) / 64) * 64 * 4 * sizeof(u64);
}

// Launches the recurrence of 1 or 2 directions (same H, B, T).  Returns false if it
// cannot run (size or residency): the caller then takes the step-by-step path.
bool qr_launch_recurrence(const QrRecGroup &g, hipStream_t st)
{
    const int nks = (g.d[0].H + 63) / 64;
    const int kw = (nks + 3) / 4;
    switch (kw) {
    case 1: return launch_rec_t<1>(g, st);
    case 2: return launch_rec_t<2>(g, st);
    case 3: return launch_rec_t<3>(g, st);
    case 4: return launch_rec_t<4>(g, st);
    default: return false;
    }
}
