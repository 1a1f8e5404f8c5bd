// The time loop of an LSTM layer as one persistent kernel (Sec. 3.4: the hidden
// state is quantized once at the cell output and that code feeds the next step).
//
// The recurrence is a chain of T dependent steps, each far too small to fill the
// GPU, so its cost is the latency of one step, not arithmetic.  Design:
//   - a workgroup owns 8 cells (32 gate rows = 2 row tiles) of one direction for
//     all T steps; its slice of W_hh is unpacked once into registers as int8 MFMA
//     operands and never re-read; the cell state of its cells stays in registers;
//   - wave w of the workgroup serves utterances 16*(w + 4*i) .. +15;
//   - the 4-bit codes of h_t travel between workgroups through a double-buffered
//     exchange area in 8-byte words {4 codes, step tag}: a consumer knows a word is
//     current when its tag matches, so there is no grid barrier, no atomic and no
//     fence on the critical path (data and flag arrive in the same store);
//   - both directions of a bidirectional layer run in the same launch.
// All workgroups must be co-resident (cooperative launch guarantees it); a wait is
// bounded by spin_limit polls, after which the error flag is set and every wave
// leaves the loop, so the grid always drains.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace {

__device__ __forceinline__ unsigned long long ll_load(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_store(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// KS: 64-column K steps held in registers (H <= 64*KS); NTW: utterance tiles per wave.
template <int KS, int NTW>
__global__ __launch_bounds__(256, 1) void lstm_rec_kernel(const QrRecGroup g)
{
    __shared__ int8_t hc[64 * NTW][8];   // codes of this workgroup's 8 cells for its utterances
    __shared__ int s_fail;
    const QrRecArgs &a = g.d[blockIdx.y];
    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, grp = lane >> 4;
    const int wg = blockIdx.x;                 // cells 8*wg .. 8*wg+7
    const int n_row_tiles = H >> 2;
    const int nks = (H + 63) >> 6;
    const int HQ = H >> 2;                     // exchange words per utterance
    const v4i zero = {0, 0, 0, 0};
    const int m = (int)0xF0F0F0F0u;

    // ---- stationary operands: W_hh rows of this workgroup, unpacked to int8 (x16)
    v4i A[2][KS];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int rt = 2 * wg + mt < n_row_tiles ? 2 * wg + mt : n_row_tiles - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            A[mt][ks] = zero;
            if (ks < nks) {
                const v4i p = a.whh[((size_t)rt * a.nkc_h + (ks >> 1)) * 64 + lane];
                A[mt][ks] = (ks & 1) ? (p & m) : ((p << 4) & m);
            }
        }
    }
    float sx[2][4], sh[2][4], bb[2][4];
    int jc[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        const int j = (2 * wg + mt) * 4 + grp;
        jc[mt] = j < H ? j : H - 1;
#pragma unroll
        for (int gt = 0; gt < 4; ++gt) {
            sx[mt][gt] = a.x_scale * a.s_wih[gt * H + jc[mt]];
            sh[mt][gt] = a.h_scale * a.s_whh[gt * H + jc[mt]];
            bb[mt][gt] = a.bias[gt * H + jc[mt]];
        }
    }
    // ---- state
    float c[NTW][2];
    int n_of[NTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
        const int n = (wave + 4 * i) * 16 + col;
        n_of[i] = n;
        const int nn = n < B ? n : B - 1;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) c[i][mt] = a.c0 ? a.c0[(int64_t)nn * H + jc[mt]] : 0.0f;
    }
    bool failed = false;
    if (tid == 0) s_fail = 0;
    __syncthreads();

    for (int s = 0; s < T; ++s) {
        const int t = a.reverse ? T - 1 - s : s;
        // input projection of this step (does not depend on h): issue first
        v4i gxv[NTW][2];
#pragma unroll
        for (int i = 0; i < NTW; ++i) {
            const int nn = n_of[i] < B ? n_of[i] : B - 1;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                gxv[i][mt] = *(const v4i *)(a.gx + ((int64_t)t * B + nn) * 4 * H + 4 * jc[mt]);
        }
#pragma unroll
        for (int i = 0; i < NTW; ++i) {
            const int nn = n_of[i] < B ? n_of[i] : B - 1;
            v4i acc[2] = {zero, zero};
            if (s > 0 || a.h0) {
                v4i bf[KS];
                if (s == 0) {
                    const int8_t *hr = a.h0 + (int64_t)nn * H + grp * 16;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) bf[ks] = (ks * 64 + grp * 16 < H) ? *(const v4i *)(hr + ks * 64) : zero;
                } else {
                    // words of utterance nn written at step s-1 carry tag s
                    const unsigned long long *xw = a.xbuf + ((size_t)((s - 1) & 1) * B + nn) * HQ + grp * 4;
                    const unsigned want = (unsigned)s;
                    int spins = 0;
                    while (true) {
                        bool ok = true;
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks) {
                            bf[ks] = zero;
                            if (ks * 64 + grp * 16 < H) {
#pragma unroll
                                for (int q = 0; q < 4; ++q) {
                                    const unsigned long long wv = ll_load(xw + ks * 16 + q);
                                    bf[ks][q] = (int)(unsigned)wv;
                                    ok = ok && ((unsigned)(wv >> 32) == want);
                                }
                            }
                        }
                        if (__all(ok)) break;
                        if (++spins > a.spin_limit) { failed = true; break; }
                    }
                    if (failed && lane == 0) {
                        atomicExch(a.err, 1);
                        s_fail = 1;
                    }
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt) acc[mt] = qr_mfma(A[mt][ks], bf[ks], acc[mt]);
            }
            // fused cell for 2 cells x 1 utterance per lane
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const v4i ah = acc[mt] >> 4;
                float p[4];
#pragma unroll
                for (int gt = 0; gt < 4; ++gt)
                    p[gt] = sx[mt][gt] * (float)gxv[i][mt][gt] + (sh[mt][gt] * (float)ah[gt] + bb[mt][gt]);
                const float gi = qr_sigmoid(p[0]), gf = qr_sigmoid(p[1]), gg = qr_tanh(p[2]), go = qr_sigmoid(p[3]);
                const float cn = gf * c[i][mt] + gi * gg;
                c[i][mt] = cn;
                const float h = go * qr_tanh(cn);
                hc[(wave + 4 * i) * 16 + col][mt * 4 + grp] = (int8_t)qr_quant4(h, a.h_inv);
                if (a.dbg_c_all && n_of[i] < B && (2 * wg + mt) * 4 + grp < H)
                    a.dbg_c_all[((int64_t)t * B + n_of[i]) * H + jc[mt]] = cn;
            }
        }
        __syncthreads();
        const int fail_now = s_fail;   // written only before this barrier, read only after it: uniform
        // publish: one word = 4 consecutive cells of one utterance, tagged s+1
        for (int wd = tid; wd < 128 * NTW; wd += 256) {
            const int n = wd >> 1, mt = wd & 1;
            const int q = 2 * wg + mt;
            if (n < B && q < HQ) {
                const unsigned data = *(const unsigned *)&hc[n][mt * 4];
                ll_store(a.xbuf + ((size_t)(s & 1) * B + n) * HQ + q, ((unsigned long long)(unsigned)(s + 1) << 32) | data);
                *(unsigned *)(a.h_out + ((int64_t)t * B + n) * a.ld_out + a.col_off + 4 * q) = data;
                if (s == T - 1 && a.h_last) *(unsigned *)(a.h_last + (int64_t)n * H + 4 * q) = data;
            }
        }
        __syncthreads();
        if (fail_now) break;
    }
    if (a.c_last) {
#pragma unroll
        for (int i = 0; i < NTW; ++i)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
                if (n_of[i] < B && (2 * wg + mt) * 4 + grp < H) a.c_last[(int64_t)n_of[i] * H + jc[mt]] = c[i][mt];
    }
}

template <int KS, int NTW>
hipError_t launch_rec_t(const QrRecGroup &g, hipStream_t st)
{
    QrRecGroup gg = g;
    void *params[] = {(void *)&gg};
    dim3 grid((g.d[0].H + 7) / 8, g.n);
    return hipLaunchCooperativeKernel((const void *)lstm_rec_kernel<KS, NTW>, grid, dim3(256), params, 0, st);
}

}  // namespace

bool qr_rec_supported(int H, int B) { return H % 8 == 0 && H <= 1024 && B <= 128 && (H / 8) * 2 <= 256; }

size_t qr_rec_xbuf_bytes(int H, int B) { return (size_t)2 * B * (H / 4) * sizeof(unsigned long long); }

// Launches the recurrence of 1 or 2 directions (same H, B, T).  Returns false if the launch failed.
bool qr_launch_recurrence(const QrRecGroup &g, hipStream_t st)
{
    const int H = g.d[0].H, B = g.d[0].B;
    const int ks = (H + 63) / 64;
    const int ntw = (B + 63) / 64;
    hipError_t e = hipErrorInvalidValue;
#define QR_REC_CASE(KS)                                            \
    if (ks <= KS) {                                                \
        e = ntw == 1 ? launch_rec_t<KS, 1>(g, st) : launch_rec_t<KS, 2>(g, st); \
    } else
    QR_REC_CASE(1) QR_REC_CASE(2) QR_REC_CASE(4) QR_REC_CASE(8) QR_REC_CASE(10) QR_REC_CASE(12) QR_REC_CASE(16) {}
#undef QR_REC_CASE
    return e == hipSuccess;
}
