// Quantized linear layer (Sec. 3.2: weights and inputs of linear layers are
// quantized) with an optional fused log-softmax for the LM output layer (Sec. 2).
#include "kernels.h"
#include "mma_core.h"

namespace {

// Grid: x = groups of 4*MT row tiles, y = groups of NT*16 activation rows.
template <int MT, int NT>
__global__ __launch_bounds__(256) void linear_kernel(const v4i *__restrict__ w, int nkc, int rows, const float *__restrict__ s_w,
                                                      const float *__restrict__ bias, float a_scale,
                                                      const int8_t *__restrict__ act, int K, int N,
                                                      float *__restrict__ y, int32_t *__restrict__ dbg_acc)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, grp = lane >> 4;
    const int n_row_tiles = (rows + 15) >> 4;
    const int rt0 = (blockIdx.x * 4 + wave) * MT;
    if (rt0 >= n_row_tiles) return;
    const int8_t *aptr[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int n = (blockIdx.y * NT + nt) * 16 + col;
        n = n < N ? n : N - 1;
        aptr[nt] = act + (int64_t)n * K + grp * 16;
    }
    v4i acc[MT][NT];
    const v4i zero = {0, 0, 0, 0};
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = zero;
    qr_mma_range<MT, NT>(w, nkc, n_row_tiles, rt0, lane, aptr, K, acc);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r0 = (rt0 + mt) * 16 + grp * 4;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int n = (blockIdx.y * NT + nt) * 16 + col;
            if (n >= N) continue;
            const v4i v = acc[mt][nt] >> 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = r0 + i;
                if (r >= rows) continue;
                y[(int64_t)n * rows + r] = (a_scale * s_w[r]) * (float)v[i] + (bias ? bias[r] : 0.0f);
                if (dbg_acc) dbg_acc[(int64_t)n * rows + r] = v[i];
            }
        }
    }
}

// rows <= 64: one wave owns all rows of 16 activation rows, so the log-softmax
// over the rows is a reduction over the lane's own values and the four lane
// groups (xor 16, 32).
__global__ __launch_bounds__(64) void linear_logsoftmax_kernel(const v4i *__restrict__ w, int nkc, int rows,
                                                                const float *__restrict__ s_w, const float *__restrict__ bias,
                                                                float a_scale, const int8_t *__restrict__ act, int K, int N,
                                                                float *__restrict__ y, int32_t *__restrict__ dbg_acc)
{
    const int lane = threadIdx.x & 63;
    const int col = lane & 15, grp = lane >> 4;
    const int n_row_tiles = (rows + 15) >> 4;
    const int8_t *aptr[1];
    int n = blockIdx.x * 16 + col;
    const bool nv = n < N;
    n = nv ? n : N - 1;
    aptr[0] = act + (int64_t)n * K + grp * 16;
    v4i acc[4][1];
    const v4i zero = {0, 0, 0, 0};
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) acc[mt][0] = zero;
    qr_mma_range<4, 1>(w, nkc, n_row_tiles, 0, lane, aptr, K, acc);
    float v[4][4];
    float m = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = mt * 16 + grp * 4 + i;
            const int a = acc[mt][0][i] >> 4;
            if (r < rows) {
                v[mt][i] = (a_scale * s_w[r]) * (float)a + (bias ? bias[r] : 0.0f);
                if (dbg_acc && nv) dbg_acc[(int64_t)n * rows + r] = a;
                m = fmaxf(m, v[mt][i]);
            } else {
                v[mt][i] = -INFINITY;
            }
        }
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    float sum = 0.0f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) sum += (mt * 16 + grp * 4 + i < rows) ? expf(v[mt][i] - m) : 0.0f;
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    const float lse = m + logf(sum);
    if (!nv) return;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = mt * 16 + grp * 4 + i;
            if (r < rows) y[(int64_t)n * rows + r] = v[mt][i] - lse;
        }
}

}  // namespace

void qr_launch_linear(const QrLinearArgs &a, hipStream_t st)
{
    const int n_row_tiles = (a.rows + 15) / 16;
    if (a.log_softmax) {
        linear_logsoftmax_kernel<<<(a.N + 15) / 16, 64, 0, st>>>(a.w, a.nkc, a.rows, a.s_w, a.bias, a.a_scale, a.act, a.K,
                                                                 a.N, a.y, a.dbg_acc);
    } else if (a.N <= 16) {
        dim3 grid((n_row_tiles + 3) / 4, 1);
        linear_kernel<1, 1><<<grid, 256, 0, st>>>(a.w, a.nkc, a.rows, a.s_w, a.bias, a.a_scale, a.act, a.K, a.N, a.y,
                                                  a.dbg_acc);
    } else {
        dim3 grid((n_row_tiles + 7) / 8, (a.N + 63) / 64);
        linear_kernel<2, 4><<<grid, 256, 0, st>>>(a.w, a.nkc, a.rows, a.s_w, a.bias, a.a_scale, a.act, a.K, a.N, a.y,
                                                  a.dbg_acc);
    }
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
    la.s_w = w->row_scale;  la.bias = bias;  la.a_scale = a_scale;
    la.act = a;  la.K = w->cols;  la.N = N;  la.y = y;  la.dbg_acc = dbg_acc;  la.log_softmax = log_softmax;
    qr_launch_linear(la, (hipStream_t)stream);
    return qr_launch_status();
}
