// Joint network, log-softmax and density-ratio fusion in one kernel (Sec. 2:
// encoder and prediction outputs are combined multiplicatively, a linear layer
// and a log-softmax follow; Eq. 1 adds the weighted LM log-probabilities).
#include "head.h"
#include "kernels.h"
#include "route.h"
#include "select.h"

namespace {

// The 16 encoder and 16 prediction values of one lane's K block, as loaded.
struct QrJointRaw {
    v4f e[4], p[4];
};

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
    const int zbits = a.w8 ? 8 : 4;
    auto bload = [&](int kb) -> QrJointRaw {
        QrJointRaw raw = {};
        if (kb * 64 + grp * 16 < J) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                raw.e[d] = *(const v4f *)(e + kb * 64 + 4 * d);
                raw.p[d] = *(const v4f *)(p + kb * 64 + 4 * d);
            }
        }
        return raw;
    };
    auto bmake = [&](const QrJointRaw &raw, int kb) -> v4i {
        v4i b = {0, 0, 0, 0};
        if (kb * 64 + grp * 16 < J) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t word = 0;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float z = qr_tanh(raw.e[d][i] * raw.p[d][i]);
                    word |= (uint32_t)(qr_quant(z, z_inv, zbits) & 0xFF) << (8 * i);
                }
                b[d] = (int)word;
            }
            if (zq && nv) *(v4i *)(zq + kb * 64) = b;
        }
        return b;
    };
    const int n_row_tiles = (a.V + 15) >> 4;
    v4i acc[4];
    qr_head_mma<1>(a.w, a.nkc, n_row_tiles, 0, J, bload, bmake, [] {}, acc, lds, a.w8 != 0);
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
        for (int i = 0; i < 4; ++i) sum += (mt * 16 + grp * 4 + i < a.V) ? qr_exp(v[mt][i] - m) : 0.0f;
    sum += __shfl_xor(sum, 16);
    sum += __shfl_xor(sum, 32);
    const float lse = m + qr_log(sum);
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

// Decoding-loop variant: one block per utterance does the joint + fusion for its W
// hypotheses (NTW column tiles of 16), and wave 0, which ends up holding every fused
// score of the utterance in registers, goes straight on to select the W best
// (parent, token) extensions and to route them (route.h).  The fused scores never
// touch memory and a decoding round saves a launch.
// Lane (grp, col) of wave 0 holds, in slot s = 16*nt + 4*mt + i, the candidate
// (hypothesis w = 16*nt + col, token k = 16*mt + 4*grp + i); its flat index
// w*V + k grows with s, so the first best slot of a lane is its lowest index.
// ALSD: the same joint + selection inside the alignment-length synchronous search (route.h, qr_alsd_route):
// every hypothesis reads its own encoder frame (iteration - labels so far), a blank at the last frame
// finishes a hypothesis instead of being a candidate, labels beyond the cap are no candidates.
// Workgroups beyond the B utterances (time-synchronous search, first round of a frame) copy the state rows of the
// new beam from their sources into the beam's buffer, four slots of one tensor per wave: that copy only has to be
// done before the next network advance, so it runs here, on the CUs this kernel leaves idle, instead of in a launch
// of its own.  The joint of this round reads its inputs through the same source indices (QrJointArgs.row_idx).
template <int NTW, bool ALSD>
__global__ __launch_bounds__(256) void joint_route_kernel(const QrJointArgs a, const QrRouteArgs r, const QrAlsdArgs s,
                                                          const QrGatherTable gt)
{
    __shared__ v4i lds[4 * 4 * 64];
    __shared__ float cand[16 * NTW * 64];   // the utterance's candidates by flat index (second attempt of the selection)
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (!ALSD && (int)blockIdx.x >= r.B) {   // uniform per workgroup
        // A wave moves the rows of 4 consecutive slots of one tensor.  This kernel's register footprint allows only
        // 8 waves per CU, so what keeps the copy near the memory rate is the amount each wave has in flight: all
        // loads of its (up to) four rows are issued before the first store, 16 KiB per wave for 4 KiB rows.
        const int nq = (gt.N + 3) >> 2;
        const int quad = ((int)blockIdx.x - r.B) * 4 + wave;
        if (quad >= nq * gt.n) return;
        const int t = quad / nq, n0 = (quad - t * nq) * 4;
        const int rb = gt.row_bytes[t];
        const char *sp[4];
        char *dp[4];
        bool ok[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int n = n0 + u;
            const int src = n < gt.N ? gt.beam_src[n] : -1;   // an empty rank keeps whatever the destination holds (its score is -inf)
            ok[u] = src >= 0 && src < gt.src_limit;
            sp[u] = gt.base[t] + (size_t)(ok[u] ? src : 0) * rb;
            dp[u] = gt.base[t] + ((size_t)gt.dst_buf * gt.N + (n < gt.N ? n : 0)) * rb;
        }
        if ((rb & 15) == 0 && ((uintptr_t)gt.base[t] & 15) == 0) {
            const int n16 = rb >> 4;
            for (int i0 = 0; i0 < n16; i0 += 256) {
                v4i tmp[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (ok[u] && i0 + v * 64 + lane < n16) tmp[u][v] = ((const v4i *)sp[u])[i0 + v * 64 + lane];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (ok[u] && i0 + v * 64 + lane < n16) ((v4i *)dp[u])[i0 + v * 64 + lane] = tmp[u][v];
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (ok[u])
                    for (int i = lane; i < rb / 4; i += 64) ((uint32_t *)dp[u])[i] = ((const uint32_t *)sp[u])[i];
        }
        return;
    }
    const int col = lane & 15, grp = lane >> 4;
    const int b = blockIdx.x;
    const int W = r.W, V = a.V, J = a.J;
    if (r.gate && *r.gate == 0) {   // uniform: no utterance carried a label into this round, nothing can be picked
        if (ALSD) return;           // no live hypothesis anywhere: the finals stay as they are
        if (wave == 0) {
            if (lane == 0 && b == 0 && r.live_clear) *r.live_clear = 0;
            if (lane == 0 && b == 0 && r.n_rows_clear) *r.n_rows_clear = 0;
            if (r.last_round) qr_frame_end(r, b, lane, r.nx_count[b], (unsigned *)lds, (int *)lds + 64);
        }
        return;
    }
    int fr = a.frame_base + b;
    fr = fr < 0 ? 0 : (fr >= a.n_enc_rows ? a.n_enc_rows - 1 : fr);
    const float *e_utt = a.enc + (int64_t)fr * J + grp * 16;
    const float z_inv = a.z_inv;
    const int zbits = a.w8 ? 8 : 4;
    const int n_row_tiles = (V + 15) >> 4;
    constexpr int PER = 16 * NTW;
    float val[PER];
    float *fin_new = (float *)lds + 256;   // ALSD: value of hypothesis w finishing now; wave 0's own part of the buffer
    QrAlsdOwn own = {};
    int nx0 = 0;   // length of the utterance's candidate list before this round
    if (ALSD && wave == 0) {
        fin_new[lane] = -INFINITY;
        own = qr_alsd_load_own(r, s, b, lane);
    }
    if (!ALSD && wave == 0) {   // what the routing will need of this lane's hypothesis (its blank picks carry it into the candidate list)
        const int o = b * W + (lane < W ? lane : 0);
        own.node = r.node_src[o];
        own.len = r.len_src[o];
        nx0 = r.nx_count[b];
    }
    // per-token constants of this lane's 16 tokens (fetched behind the first tile's operands, see qr_head_mma)
    float wscale[4][4], wbias[4][4];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const int w = nt * 16 + col;
        const bool wv = w < W;
        const int n = b * W + (wv ? w : W - 1);
        int64_t nrow = n;   // row of the cached network outputs that hypothesis n reads
        if (!ALSD && a.row_idx) {
            const int src = a.row_idx[n];
            nrow = src >= 0 ? (int64_t)src : (int64_t)a.row_idx_buf * a.N + n;
        }
        const float *p = a.pred + nrow * J + grp * 16;
        const float *e = e_utt;
        int len_w = 0, t_w = 0;
        if (ALSD) {   // this hypothesis' own frame
            len_w = r.len_src[n];
            t_w = s.iter - len_w;
            t_w = t_w < 0 ? 0 : (t_w > s.T - 1 ? s.T - 1 : t_w);
            e = a.enc + ((int64_t)t_w * r.B + b) * J + grp * 16;
        }
        auto bload = [&](int kb) -> QrJointRaw {
            QrJointRaw raw = {};
            if (kb * 64 + grp * 16 < J) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    raw.e[d] = *(const v4f *)(e + kb * 64 + 4 * d);
                    raw.p[d] = *(const v4f *)(p + kb * 64 + 4 * d);
                }
            }
            return raw;
        };
        auto bmake = [&](const QrJointRaw &raw, int kb) -> v4i {
            v4i bq = {0, 0, 0, 0};
            if (kb * 64 + grp * 16 < J) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    uint32_t word = 0;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float z = qr_tanh(raw.e[d][i] * raw.p[d][i]);
                        word |= (uint32_t)(qr_quant(z, z_inv, zbits) & 0xFF) << (8 * i);
                    }
                    bq[d] = (int)word;
                }
            }
            return bq;
        };
        // LM log-probabilities, the running score and (first tile) the per-token constants: what only the
        // epilogue of wave 0 needs
        float ls[4][4], le[4][4], sc = 0.0f;
        auto epilogue_loads = [&]() {
            if (wave == 0) {
                sc = r.score_src[(int64_t)b * W + (wv ? w : W - 1)];
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int k = mt * 16 + grp * 4 + i;
                        const int kk = k < V ? k : V - 1;
                        ls[mt][i] = a.lp_src ? a.lp_src[nrow * V + kk] : 0.0f;
                        le[mt][i] = a.lp_ext ? a.lp_ext[nrow * V + kk] : 0.0f;
                        if (nt == 0) {
                            wscale[mt][i] = a.z_scale * a.s_w[kk];
                            wbias[mt][i] = a.b_out ? a.b_out[kk] : 0.0f;
                        }
                    }
            }
        };
        v4i acc[4];
        if (nt > 0) __syncthreads();   // the reduction buffer of the previous tile has been read
        qr_head_mma<1>(a.w, a.nkc, n_row_tiles, 0, J, bload, bmake, epilogue_loads, acc, lds, a.w8 != 0);
        if (wave == 0) {
            float v[4][4];
            float m = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = mt * 16 + grp * 4 + i;
                    v[mt][i] = k < V ? wscale[mt][i] * (float)acc[mt][i] + wbias[mt][i] : -INFINITY;
                    m = fmaxf(m, v[mt][i]);
                }
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            float sum = 0.0f;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) sum += (mt * 16 + grp * 4 + i < V) ? qr_exp(v[mt][i] - m) : 0.0f;
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            const float lse = m + qr_log(sum);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k = mt * 16 + grp * 4 + i;
                    float f = v[mt][i] - lse;
                    if (k != a.blank) {
                        if (a.lp_src) f -= a.lambda_src * ls[mt][i];
                        if (a.lp_ext) f += a.lambda_ext * le[mt][i];
                        f += a.rho;
                    }
                    // an empty slot (score -inf) offers nothing, whatever its rows of the network outputs hold
                    bool ok = wv && k < V && sc > -INFINITY && (ALSD || !r.last_round || k == a.blank);
                    if (ALSD) {
                        if (k != a.blank && len_w >= s.u_max) ok = false;      // label cap
                        if (k == a.blank && t_w == s.T - 1) {                  // a blank at the last frame finishes w
                            if (ok && sc > -INFINITY) fin_new[w] = sc + f;
                            ok = false;
                        }
                    }
                    val[nt * 16 + mt * 4 + i] = ok ? (sc + f) + 0.0f : -INFINITY;   // + 0: one key per value
                }
        }
    }
    if (wave != 0) return;

    // ---- the W best under (value descending, flat index ascending)
    const int cbase = col * V + grp * 4;   // flat index of slot s: cbase + (s>>4)*16*V + ((s>>2)&3)*16 + (s&3)
    auto index_of = [&](int s) { return cbase + (s >> 4) * 16 * V + ((s >> 2) & 3) * 16 + (s & 3); };
    float last_v = INFINITY;
    int last_c = -1, my_c = -1;
    float my_v = -INFINITY;
    bool fast = qr_select_pruned<PER>(val, index_of, W, lane, (unsigned *)lds, (int *)lds + 64, my_c, my_v);
    if (!fast) {   // uniform
        // More than 64 candidates passed the bound: the MFMA layout keeps a hypothesis' tokens in 4 lanes, and when
        // the best candidates of the utterance belong to one or two hypotheses a lane's best says little.  The
        // candidates change places through LDS (lane l takes the flat indices l, l + 64, ...: every hypothesis is
        // then spread over all lanes and the bound is tight) and the pruned selection runs again.
#pragma unroll
        for (int sl = 0; sl < PER; ++sl) {
            const int w = (sl >> 4) * 16 + col, k = ((sl >> 2) & 3) * 16 + grp * 4 + (sl & 3);
            if (w < W && k < V) cand[w * V + k] = val[sl];
        }
        __builtin_amdgcn_wave_barrier();
        const int n_cand = W * V;
#pragma unroll
        for (int sl = 0; sl < PER; ++sl) val[sl] = (lane + 64 * sl < n_cand) ? cand[lane + 64 * sl] : -INFINITY;
        __builtin_amdgcn_wave_barrier();
        auto index_t = [&](int sl) { return lane + 64 * sl; };
        fast = qr_select_pruned<PER>(val, index_t, W, lane, (unsigned *)lds, (int *)lds + 64, my_c, my_v);
        for (int rd = 0; !fast && rd < W; ++rd) {   // general case: W rounds of arg-best
            float bv = -INFINITY;
            int bc = 0x7fffffff;
#pragma unroll
            for (int sl = 0; sl < PER; ++sl) {
                const int c = lane + 64 * sl;
                const float v = val[sl];
                const bool ok = v > -INFINITY && (v < last_v || (v == last_v && c > last_c));
                if (ok && v > bv) { bv = v; bc = c; }   // slots are visited in index order: first best wins
            }
            if (!qr_select_round(bv, bc, rd, lane, last_v, last_c, my_c, my_v)) break;
        }
    }
    if (ALSD) {
        __builtin_amdgcn_wave_barrier();
        qr_alsd_route(r, s, b, lane, my_c, my_v, fin_new[lane], own);
        return;
    }
    const int cnt = qr_route_picks(r, b, lane, my_c, my_v, own.node, own.len, nx0);
    if (r.last_round) {   // the frame is complete for this utterance: prune its candidate list to the new beam
        __threadfence();
        qr_frame_end(r, b, lane, cnt, (unsigned *)lds, (int *)lds + 64);
    }
}

}  // namespace

void qr_launch_joint_route(const QrJointArgs &a, const QrRouteArgs &r, const QrGatherTable &gt, hipStream_t st)
{
    const QrAlsdArgs none = {};
    const unsigned grid = (unsigned)(r.B + (gt.n > 0 ? (((gt.N + 3) / 4) * gt.n + 3) / 4 : 0));   // copy: 4 slots per wave, 4 waves per workgroup
    if (r.W <= 16) joint_route_kernel<1, false><<<grid, 256, 0, st>>>(a, r, none, gt);
    else if (r.W <= 32) joint_route_kernel<2, false><<<grid, 256, 0, st>>>(a, r, none, gt);
    else joint_route_kernel<4, false><<<grid, 256, 0, st>>>(a, r, none, gt);
}

void qr_launch_joint_alsd(const QrJointArgs &a, const QrRouteArgs &r, const QrAlsdArgs &s, hipStream_t st)
{
    const QrGatherTable none = {};
    if (r.W <= 16) joint_route_kernel<1, true><<<r.B, 256, 0, st>>>(a, r, s, none);
    else if (r.W <= 32) joint_route_kernel<2, true><<<r.B, 256, 0, st>>>(a, r, s, none);
    else joint_route_kernel<4, true><<<r.B, 256, 0, st>>>(a, r, s, none);
}

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
    a.w8 = qr_bits(w_out) == 8;
    a.lp_out = lp_rnnt_out;  a.dbg_zq = dbg_zq;  a.fused = fused_out;
    a.rows_per_utt = 1;
    qr_launch_joint(a, (hipStream_t)stream);
    return qr_launch_status();
}
