// Quantized linear layer (Sec. 3.2: weights and inputs of linear layers are
// quantized) with an optional fused log-softmax for the LM output layer (Sec. 2).
#include "head.h"
#include "kernels.h"

namespace {

// Grid: x = blocks of 16 activation rows, y = blocks of 64 weight rows, z = problem.
__global__ __launch_bounds__(256) void linear_head_kernel(const QrLinearGroup g)
{
    __shared__ v4i lds[4 * 4 * 64];
    if (g.gate && *g.gate == 0) return;   // uniform: a decoding round without any live hypothesis
    const QrLinearArgs a = g.p[blockIdx.z];   // a copy: the fields arrive with a few wide scalar loads up front
    const int n_row_tiles = (a.rows + 15) >> 4;
    const int rt0 = blockIdx.y * 4;
    if (rt0 >= n_row_tiles || (int)blockIdx.x * 16 >= a.N) return;   // uniform per block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, grp = lane >> 4;
    int n = blockIdx.x * 16 + col;
    bool nv = n < a.N;
    n = nv ? n : a.N - 1;
    if (g.rows) {   // column j stands for the activation row of list entry j; the entry is fetched before the count is looked at
        const v4i e = g.rows[n];
        const int n_cnt = *g.n_rows;
        if ((int)blockIdx.x * 16 >= n_cnt) return;   // uniform per block
        nv = nv && (int)blockIdx.x * 16 + col < n_cnt;
        n = e[0] < 0 ? 0 : (e[0] >= a.N ? a.N - 1 : e[0]);
    }
    const int8_t *arow = a.act + (int64_t)n * a.K + grp * 16;
    const int K = a.K;
    auto bload = [&](int kb) -> v4i {
        const v4i zero = {0, 0, 0, 0};
        return (kb * 64 + grp * 16 < K) ? *(const v4i *)(arow + kb * 64) : zero;
    };
    auto bmake = [](const v4i &raw, int) -> v4i { return raw; };
    // row constants of the lanes that finish the rows (wave 0): fetched behind the operands of the contraction
    float sw[4][4], bs[4][4];
    auto row_constants = [&]() {
        if (wave == 0) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = (rt0 + mt) * 16 + grp * 4 + i;
                    const int rr = r < a.rows ? r : a.rows - 1;
                    sw[mt][i] = a.a_scale * a.s_w[rr];
                    bs[mt][i] = a.bias ? a.bias[rr] : 0.0f;
                }
        }
    };
    v4i acc[4];
    qr_head_mma<QR_HEAD_BATCH>(a.w, a.nkc, n_row_tiles, rt0, K, bload, bmake, row_constants, acc, lds, a.w8 != 0);
    if (wave != 0) return;

    float v[4][4];
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = (rt0 + mt) * 16 + grp * 4 + i;
            if (r < a.rows) {
                v[mt][i] = sw[mt][i] * (float)acc[mt][i] + bs[mt][i];
                if (a.dbg_acc && nv) a.dbg_acc[(int64_t)n * a.rows + r] = acc[mt][i];
                mx = fmaxf(mx, v[mt][i]);
            } else {
                v[mt][i] = -INFINITY;
            }
        }
    float lse = 0.0f;
    if (a.log_softmax) {   // rows <= 64: the whole row set is in this wave (4 lane groups x 16 values)
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float sum = 0.0f;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) sum += (mt * 16 + grp * 4 + i < a.rows) ? qr_exp(v[mt][i] - mx) : 0.0f;
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        lse = mx + qr_log(sum);
    }
    if (!nv) return;
    if (a.q_out) {   // the fp32 result goes straight through the quantizer of the layer that consumes it
        const bool wide_q = (a.rows & 3) == 0 && ((uintptr_t)a.q_out & 3) == 0;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const int r0 = (rt0 + mt) * 16 + grp * 4;
            unsigned word = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) word |= (unsigned)(qr_quant(v[mt][i] - lse, a.q_inv, a.q_bits) & 0xFF) << (8 * i);
            if (wide_q) {
                if (r0 < a.rows) *(unsigned *)(a.q_out + (int64_t)n * a.rows + r0) = word;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (r0 + i < a.rows) a.q_out[(int64_t)n * a.rows + r0 + i] = (int8_t)(word >> (8 * i));
            }
        }
        if (!a.y) return;
    }
    const bool wide = (a.rows & 3) == 0 && ((uintptr_t)a.y & 15) == 0;   // rows of y are 16-byte aligned: one 128-bit store per lane and row tile
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int r0 = (rt0 + mt) * 16 + grp * 4;
        if (wide) {
            if (r0 < a.rows) *(v4f *)(a.y + (int64_t)n * a.rows + r0) = v4f{v[mt][0] - lse, v[mt][1] - lse, v[mt][2] - lse, v[mt][3] - lse};
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (r0 + i < a.rows) a.y[(int64_t)n * a.rows + r0 + i] = v[mt][i] - lse;
        }
    }
}

}  // namespace

void qr_launch_linear_group(const QrLinearGroup &g, hipStream_t st)
{
    int gx = 0, gy = 0;
    for (int i = 0; i < g.n; ++i) {
        const int nb = (g.p[i].N + 15) / 16, rb = ((g.p[i].rows + 15) / 16 + 3) / 4;
        gx = nb > gx ? nb : gx;
        gy = rb > gy ? rb : gy;
    }
    linear_head_kernel<<<dim3(gx, gy, g.n), 256, 0, st>>>(g);
}

void qr_launch_linear(const QrLinearArgs &a, hipStream_t st)
{
    QrLinearGroup g;
    g.p[0] = a;
    g.n = 1;
    g.gate = nullptr;
    g.rows = nullptr;
    g.n_rows = nullptr;
    qr_launch_linear_group(g, st);
}

extern "C" qrnnt_status qrnnt_linear_quant(const qrnnt_qmat *w, const float *bias, float a_scale, const int8_t *a, int32_t N,
                                           float inv_scale, int32_t bits, int8_t *q, void *stream)
{
    QR_REQUIRE(bits == 4 || bits == 8, QRNNT_ERR_RANGE);
    qrnnt_status s = qr_check_qmat(w, QRNNT_LAYOUT_TILED);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(a != nullptr && q != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(N > 0 && w->cols % 16 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(a_scale > 0.0f && inv_scale > 0.0f, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(a, 16), QRNNT_ERR_ALIGN);
    QrLinearArgs la = {};
    la.w = (const v4i *)w->packed;  la.nkc = qr_round_up(w->cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;  la.rows = w->rows;
    la.s_w = w->row_scale;  la.bias = bias;  la.a_scale = a_scale;  la.w8 = qr_bits(w) == 8;
    la.act = a;  la.K = w->cols;  la.N = N;  la.q_out = q;  la.q_inv = inv_scale;  la.q_bits = bits;
    qr_launch_linear(la, (hipStream_t)stream);
    return qr_launch_status();
}

extern "C" qrnnt_status qrnnt_linear(const qrnnt_qmat *w, const float *bias, float a_scale, const int8_t *a, int32_t N,
                                     int32_t log_softmax, float *y, int32_t *dbg_acc, void *stream)
{
    qrnnt_status s = qr_check_qmat(w, QRNNT_LAYOUT_TILED);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(a != nullptr && y != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(N > 0 && w->cols % 16 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(a_scale > 0.0f, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(a, 16) && qr_aligned(y, 4), QRNNT_ERR_ALIGN);
    QR_REQUIRE(!log_softmax || w->rows <= 64, QRNNT_ERR_UNSUPPORTED);
    QrLinearArgs la = {};
    la.w = (const v4i *)w->packed;  la.nkc = qr_round_up(w->cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;  la.rows = w->rows;
    la.s_w = w->row_scale;  la.bias = bias;  la.a_scale = a_scale;  la.w8 = qr_bits(w) == 8;
    la.act = a;  la.K = w->cols;  la.N = N;  la.y = y;  la.dbg_acc = dbg_acc;  la.log_softmax = log_softmax;
    qr_launch_linear(la, (hipStream_t)stream);
    return qr_launch_status();
}
