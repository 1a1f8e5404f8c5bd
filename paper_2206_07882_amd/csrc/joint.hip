// Joint network, log-softmax and density-ratio fusion in one kernel (Sec. 2:
// encoder and prediction outputs are combined multiplicatively, a linear layer
// and a log-softmax follow; Eq. 1 adds the weighted LM log-probabilities).
#include "head.h"
#include "kernels.h"

namespace {

// One block (4 waves) per 16 hypotheses; the J columns are dealt to the waves in
// 64-column blocks.  Lane (col, grp) produces the 16 codes of z that are its own
// MFMA operand for that block, so z never leaves registers; partial sums meet in
// wave 0, which holds all V <= 64 rows of the output layer for the log-softmax.
__global__ __launch_bounds__(256) void joint_fuse_kernel(const QrJointArgs a)
{
    __shared__ v4i lds[4 * 4 * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, grp = lane >> 4;
    int n = blockIdx.x * 16 + col;
    const bool nv = n < a.N;
    n = nv ? n : a.N - 1;
    int fr = a.frame_row ? a.frame_row[n] : a.frame_base + n / a.rows_per_utt;
    fr = fr < 0 ? 0 : (fr >= a.n_enc_rows ? a.n_enc_rows - 1 : fr);
    const float *e = a.enc + (int64_t)fr * a.J + grp * 16;
    const float *p = a.pred + (int64_t)n * a.J + grp * 16;
    int8_t *zq = a.dbg_zq ? a.dbg_zq + (int64_t)n * a.J + grp * 16 : nullptr;
    const int J = a.J;
    const float z_inv = a.z_inv;
    auto bfrag = [&](int kb) -> v4i {
        v4i b = {0, 0, 0, 0};
        if (kb * 64 + grp * 16 < J) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const v4f ev = *(const v4f *)(e + kb * 64 + 4 * d);
                const v4f pv = *(const v4f *)(p + kb * 64 + 4 * d);
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float z = qr_tanh(ev[i] * pv[i]);
                    word |= (uint32_t)(qr_quant4(z, z_inv) & 0xFF) << (8 * i);
                }
                b[d] = (int)word;
            }
            if (zq && nv) *(v4i *)(zq + kb * 64) = b;
        }
        return b;
    };
    const int n_row_tiles = (a.V + 15) >> 4;
    v4i acc[4];
    qr_head_mma(a.w, a.nkc, n_row_tiles, 0, J, bfrag, acc, lds);
    if (wave != 0) return;

    float v[4][4];
    float m = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = mt * 16 + grp * 4 + i;
            if (k < a.V) {
                v[mt][i] = (a.z_scale * a.s_w[k]) * (float)acc[mt][i] + (a.b_out ? a.b_out[k] : 0.0f);
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
        for (int i = 0; i < 4; ++i) sum += (mt * 16 + grp * 4 + i < a.V) ? expf(v[mt][i] - m) : 0.0f;
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    const float lse = m + logf(sum);
    if (!nv) return;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = mt * 16 + grp * 4 + i;
            if (k >= a.V) continue;
            const float lp = v[mt][i] - lse;
            float f = lp;
            if (k != a.blank) {
                if (a.lp_src) f -= a.lambda_src * a.lp_src[(int64_t)n * a.V + k];
                if (a.lp_ext) f += a.lambda_ext * a.lp_ext[(int64_t)n * a.V + k];
                f += a.rho;
            }
            if (a.lp_out) a.lp_out[(int64_t)n * a.V + k] = lp;
            a.fused[(int64_t)n * a.V + k] = f;
        }
}

}  // namespace

void qr_launch_joint(const QrJointArgs &a, hipStream_t st)
{
    joint_fuse_kernel<<<(a.N + 15) / 16, 256, 0, st>>>(a);
}

extern "C" qrnnt_status qrnnt_joint_fuse(const float *enc_proj, int32_t n_enc_rows, const int32_t *frame_row,
                                         const float *pred_proj, const qrnnt_qmat *w_out, const float *b_out,
                                         float z_scale, float z_inv_scale, const float *lp_src, const float *lp_ext,
                                         float lambda_src, float lambda_ext, float rho, int32_t N, int32_t blank,
                                         float *lp_rnnt_out, int8_t *dbg_zq, float *fused_out, void *stream)
{
    qrnnt_status s = qr_check_qmat(w_out, QRNNT_LAYOUT_TILED);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(enc_proj && frame_row && pred_proj && fused_out, QRNNT_ERR_NULL);
    QR_REQUIRE(N > 0 && n_enc_rows > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(w_out->cols % 16 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(w_out->rows <= 64, QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(blank >= 0 && blank < w_out->rows, QRNNT_ERR_RANGE);
    QR_REQUIRE(z_scale > 0.0f && z_inv_scale > 0.0f, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(enc_proj, 16) && qr_aligned(pred_proj, 16), QRNNT_ERR_ALIGN);
    QR_REQUIRE(dbg_zq == nullptr || qr_aligned(dbg_zq, 16), QRNNT_ERR_ALIGN);
    QrJointArgs a = {};
    a.enc = enc_proj;  a.n_enc_rows = n_enc_rows;  a.frame_row = frame_row;  a.pred = pred_proj;
    a.w = (const v4i *)w_out->packed;  a.s_w = w_out->row_scale;  a.b_out = b_out;
    a.z_scale = z_scale;  a.z_inv = z_inv_scale;
    a.lp_src = lp_src;  a.lp_ext = lp_ext;
    a.lambda_src = lambda_src;  a.lambda_ext = lambda_ext;  a.rho = rho;
    a.N = N;  a.J = w_out->cols;  a.V = w_out->rows;  a.blank = blank;
    a.nkc = qr_round_up(w_out->cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
    a.lp_out = lp_rnnt_out;  a.dbg_zq = dbg_zq;  a.fused = fused_out;
    a.rows_per_utt = 1;
    qr_launch_joint(a, (hipStream_t)stream);
    return qr_launch_status();
}
