// The decoding loop, entirely on the device: joint + fusion (Eq. 1), beam
// selection, hypothesis bookkeeping and the advance of the prediction network
// and both language models (Sec. 2).  The paper's simulated system sorts
// hypotheses on an attached CPU and is limited by the link to it (Sec. 4.1);
// here the selection and the bookkeeping are kernels and the host only enqueues
// a data-independent launch sequence.
#include "kernels.h"
#include "select.h"

namespace {


struct NetBuf {
    int8_t *h[QRNNT_MAX_LAYERS];   // [NB][N][H]
    float *c[QRNNT_MAX_LAYERS];    // [NB][N][H]
    float *y;                      // [NB][N][out_rows]
    int32_t *gx0;                  // [V][4*H0]: input projection of layer 0 for every token
    float *tab0;                   // the same as fp32 pre-activation contributions (scales, bias folded in)
    int8_t *mid_q;                 // [N][M]: codes of the bottleneck's output (consumed in the same advance)
};

struct Plan {
    int T, B, W, N, R, NB, V, J, max_sym;
    NetBuf net[3];
    float *score;        // [NB][B][W]
    int32_t *node, *len; // [NB][N]
    int32_t *parent_idx, *token;  uint8_t *active;        // [N]
    float *nx_score;  v4i *nx_info;  int32_t *nx_count; // [B][R*W], [B]
    int32_t *beam_src;   // [N]
    int32_t *node_tok, *node_prev;   // [1 + T*max_sym*N]
    int32_t *live;       // [2][max_sym+2]: utterances that carried a label into round v of the frame (early stop)
    v4i *rows;  int32_t *n_rows;   // [N], [2][max_sym+2]: the slots that carry a label into round v of the frame, and how many
    size_t total;
};

struct Carver {
    char *base;  size_t off;
    template <typename Tp> Tp *take(size_t n)
    {
        off = (off + 255) / 256 * 256;
        Tp *p = base ? (Tp *)(base + off) : nullptr;
        off += n * sizeof(Tp);
        return p;
    }
};

const qrnnt_net *net_of(const qrnnt_model *m, int k) { return k == 0 ? &m->pred : (k == 1 ? &m->lm_src : &m->lm_ext); }
bool net_used(const qrnnt_model *m, int k) { return k == 0 || (k == 1 ? m->use_src != 0 : m->use_ext != 0); }

void make_plan(const qrnnt_model *m, int T, int B, int W, int max_sym, void *ws, Plan &p)
{
    p.T = T; p.B = B; p.W = W; p.N = B * W; p.max_sym = max_sym;
    p.R = max_sym + 1; p.NB = max_sym + 2; p.V = m->V; p.J = m->joint_out.cols;
    Carver cv{(char *)ws, 0};
    const size_t N = (size_t)p.N, NB = (size_t)p.NB;
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        const qrnnt_net *net = net_of(m, k);
        for (int l = 0; l < net->n_layers; ++l) {
            p.net[k].h[l] = cv.take<int8_t>(NB * N * net->layer[l].hidden_size);
            p.net[k].c[l] = cv.take<float>(NB * N * net->layer[l].hidden_size);
        }
        p.net[k].y = cv.take<float>(NB * N * net->out.rows);
        p.net[k].gx0 = cv.take<int32_t>((size_t)m->V * 4 * net->layer[0].hidden_size);
        p.net[k].tab0 = cv.take<float>((size_t)m->V * 4 * net->layer[0].hidden_size);
        p.net[k].mid_q = net->mid.packed ? cv.take<int8_t>(N * net->mid.rows) : nullptr;
    }
    p.score = cv.take<float>(NB * N);
    p.node = cv.take<int32_t>(NB * N);
    p.len = cv.take<int32_t>(NB * N);
    p.parent_idx = cv.take<int32_t>(N);
    p.token = cv.take<int32_t>(N);
    p.active = cv.take<uint8_t>(N);
    p.nx_score = cv.take<float>((size_t)B * p.R * W);
    p.nx_info = cv.take<v4i>((size_t)B * p.R * W);
    p.nx_count = cv.take<int32_t>(B);
    p.beam_src = cv.take<int32_t>(N);
    const size_t pool = 1 + (size_t)T * max_sym * N;
    p.node_tok = cv.take<int32_t>(pool);
    p.node_prev = cv.take<int32_t>(pool);
    p.live = cv.take<int32_t>(2 * (size_t)(max_sym + 2));
    p.rows = cv.take<v4i>(N);
    p.n_rows = cv.take<int32_t>(2 * (size_t)(max_sym + 2));
    p.total = (cv.off + 255) / 256 * 256;
}

__global__ void fill_words_kernel(uint32_t *p, size_t n_words, uint32_t v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_words) p[i] = v;
}

// Start of an utterance: slot 0 holds the empty sequence with score 0, every slot
// is fed the start symbol from the zero state.
__global__ void decode_init_kernel(float *score0, int32_t *node0, int32_t *len0, int32_t *parent_idx, int32_t *token,
                                   uint8_t *active, int32_t *nx_count, int32_t *node_tok, int32_t *node_prev, int N,
                                   int W, int B, int start_symbol)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n == 0) { node_tok[0] = -1; node_prev[0] = 0; }
    if (n < B) nx_count[n] = 0;
    if (n >= N) return;
    score0[n] = (n % W == 0) ? 0.0f : -INFINITY;
    node0[n] = 0;
    len0[n] = 0;
    parent_idx[n] = n;
    token[n] = start_symbol;
    active[n] = 1;
}

__global__ void backtrack_kernel(const float *__restrict__ score, const int32_t *__restrict__ node,
                                 const int32_t *__restrict__ len, const int32_t *__restrict__ node_tok,
                                 const int32_t *__restrict__ node_prev, int N, int max_len,
                                 int32_t *__restrict__ tokens_out, int32_t *__restrict__ len_out, float *__restrict__ score_out)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    const float sc = score[n];
    const bool live = sc > -INFINITY;
    const int L = live ? len[n] : 0;
    int32_t *out = tokens_out + (size_t)n * max_len;
    for (int i = (L < max_len ? L : max_len); i < max_len; ++i) out[i] = -1;
    int id = node[n];
    for (int i = L - 1; i >= 0; --i) {
        if (i < max_len) out[i] = node_tok[id];
        id = node_prev[id];
    }
    len_out[n] = live ? L : -1;
    score_out[n] = sc;
}

qrnnt_status check_net(const qrnnt_net *net, int V, int out_rows)
{
    QR_REQUIRE(net->embed_codes != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(net->n_layers >= 1 && net->n_layers <= QRNNT_MAX_LAYERS, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(net->embed_codes, 16), QRNNT_ERR_ALIGN);
    for (int l = 0; l < net->n_layers; ++l) {
        qrnnt_status s = qr_check_lstm(&net->layer[l]);
        if (s != QRNNT_OK) return s;
        QR_REQUIRE(qr_bits(&net->layer[l].w_hh) == 4, QRNNT_ERR_UNSUPPORTED);   // the step kernels unpack nibbles
        if (l > 0) QR_REQUIRE(net->layer[l].input_size == net->layer[l - 1].hidden_size, QRNNT_ERR_SHAPE);
    }
    qrnnt_status s = qr_check_qmat(&net->out, QRNNT_LAYOUT_TILED);
    if (s != QRNNT_OK) return s;
    if (net->mid.packed) {
        s = qr_check_qmat(&net->mid, QRNNT_LAYOUT_TILED);
        if (s != QRNNT_OK) return s;
        QR_REQUIRE(net->mid.cols == net->layer[net->n_layers - 1].hidden_size, QRNNT_ERR_SHAPE);
        QR_REQUIRE(net->mid.rows % 16 == 0 && net->out.cols == net->mid.rows, QRNNT_ERR_SHAPE);
        QR_REQUIRE(net->mid_scale > 0.0f && net->mid_inv_scale > 0.0f, QRNNT_ERR_RANGE);
    } else {
        QR_REQUIRE(net->out.cols == net->layer[net->n_layers - 1].hidden_size, QRNNT_ERR_SHAPE);
    }
    QR_REQUIRE(net->out.rows == out_rows, QRNNT_ERR_SHAPE);
    QR_REQUIRE(!net->log_softmax || net->out.rows <= 64, QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(net->out_a_scale > 0.0f, QRNNT_ERR_RANGE);
    (void)V;
    return QRNNT_OK;
}

qrnnt_status check_model(const qrnnt_model *m)
{
    QR_REQUIRE(m != nullptr, QRNNT_ERR_NULL);
    qrnnt_status s = qr_check_qmat(&m->joint_out, QRNNT_LAYOUT_TILED);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(m->V > 0 && m->V <= 64 && m->joint_out.rows == m->V, QRNNT_ERR_SHAPE);
    QR_REQUIRE(m->joint_out.cols % 16 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(m->blank >= 0 && m->blank < m->V, QRNNT_ERR_RANGE);
    QR_REQUIRE(m->z_scale > 0.0f && m->z_inv_scale > 0.0f, QRNNT_ERR_RANGE);
    s = check_net(&m->pred, m->V, m->joint_out.cols);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(!m->pred.log_softmax, QRNNT_ERR_RANGE);
    if (m->use_src) { s = check_net(&m->lm_src, m->V, m->V); if (s != QRNNT_OK) return s; }
    if (m->use_ext) { s = check_net(&m->lm_ext, m->V, m->V); if (s != QRNNT_OK) return s; }
    return QRNNT_OK;
}

// All used networks consume `token` and move from buffer src to buffer dst.  Layer l
// of every network goes out as one grouped launch (the networks are independent).
// n_rows (optional): only the hypotheses p.rows[0 .. *n_rows) advance (recurrent and output layers; the rows
// that did not advance are not read afterwards).
void advance_nets(const qrnnt_model *m, const Plan &p, int src, int dst, int n_embed_rows, const int32_t *gate,
                  const int32_t *n_rows, hipStream_t st)
{
    const size_t N = (size_t)p.N;
    int max_layers = 0;
    for (int k = 0; k < 3; ++k)
        if (net_used(m, k) && net_of(m, k)->n_layers > max_layers) max_layers = net_of(m, k)->n_layers;
    for (int l = 0; l < max_layers; ++l) {
        QrStepGroup g;
        g.n = 0;
        g.gate = gate;
        g.rows = n_rows ? p.rows : nullptr;
        g.n_rows = n_rows;
        for (int k = 0; k < 3; ++k) {
            if (!net_used(m, k)) continue;
            const qrnnt_net *net = net_of(m, k);
            if (l >= net->n_layers) continue;
            const qrnnt_lstm *L = &net->layer[l];
            const size_t H = (size_t)L->hidden_size;
            QrStepArgs &a = g.p[g.n++];
            a = QrStepArgs{};
            qr_fill_lstm_weights(a, L);
            if (l == 0) {
                // The input of layer 0 is one of V embedding rows, so its integer input
                // projection is a table lookup (exactly the sums the contraction would give).
                a.x = net->embed_codes;  a.ld_x = qr_act_pitch(L->input_size);  a.x_row = p.token;  a.n_x_rows = n_embed_rows;
                a.gx = p.net[k].gx0;  a.ld_gx = 4 * (int64_t)H;  a.tabf = p.net[k].tab0;
            } else {
                a.x = p.net[k].h[l - 1] + (size_t)dst * N * L->input_size;  a.ld_x = L->input_size;
                a.x_row = nullptr;  a.n_x_rows = p.N;
            }
            a.parent = p.parent_idx;  a.n_slots = p.N;
            a.h_prev = p.net[k].h[l] + (size_t)src * N * H;  a.ld_hp = (int64_t)H;
            a.c_prev = p.net[k].c[l] + (size_t)src * N * H;
            a.active = p.active;
            a.h_next = p.net[k].h[l] + (size_t)dst * N * H;  a.ld_hn = (int64_t)H;
            a.c_next = p.net[k].c[l] + (size_t)dst * N * H;
            a.N = p.N;
        }
        qr_launch_lstm_step_group(g, l == 0, st);
    }
    // Output layers: one grouped launch; a network with a bottleneck sends that layer (fused with the
    // quantizer of its output) in the first launch and its output layer in a second one.
    QrLinearGroup lg, lg2;
    lg.n = lg2.n = 0;
    lg.gate = lg2.gate = gate;
    lg.rows = lg2.rows = n_rows ? p.rows : nullptr;
    lg.n_rows = lg2.n_rows = n_rows;
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        const qrnnt_net *net = net_of(m, k);
        const int top = net->n_layers - 1;
        const bool has_mid = net->mid.packed != nullptr;
        QrLinearArgs out = QrLinearArgs{};
        out.w = (const v4i *)net->out.packed;
        out.nkc = qr_round_up(net->out.cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
        out.rows = net->out.rows;  out.s_w = net->out.row_scale;  out.bias = net->out_bias;
        out.K = net->out.cols;  out.N = p.N;  out.w8 = qr_bits(&net->out) == 8;
        out.y = p.net[k].y + (size_t)dst * N * net->out.rows;  out.log_softmax = net->log_softmax;
        if (has_mid) {
            QrLinearArgs &la = lg.p[lg.n++];
            la = QrLinearArgs{};
            la.w = (const v4i *)net->mid.packed;
            la.nkc = qr_round_up(net->mid.cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
            la.rows = net->mid.rows;  la.s_w = net->mid.row_scale;  la.bias = net->mid_bias;  la.a_scale = net->out_a_scale;
            la.act = p.net[k].h[top] + (size_t)dst * N * net->mid.cols;  la.K = net->mid.cols;  la.N = p.N;
            la.q_out = p.net[k].mid_q;  la.q_inv = net->mid_inv_scale;  la.q_bits = qr_bits(&net->out);  la.w8 = qr_bits(&net->mid) == 8;
            out.a_scale = net->mid_scale;  out.act = p.net[k].mid_q;
            lg2.p[lg2.n++] = out;
        } else {
            out.a_scale = net->out_a_scale;  out.act = p.net[k].h[top] + (size_t)dst * N * net->out.cols;
            lg.p[lg.n++] = out;
        }
    }
    qr_launch_linear_group(lg, st);
    if (lg2.n) qr_launch_linear_group(lg2, st);
}

}  // namespace

extern "C" size_t qrnnt_decode_workspace(const qrnnt_model *m, int32_t T, int32_t B, int32_t W, int32_t max_sym)
{
    if (check_model(m) != QRNNT_OK || T <= 0 || B <= 0 || W <= 0 || W > 64 || max_sym < 0) return 0;
    Plan p;
    make_plan(m, T, B, W, max_sym, nullptr, p);
    return p.total;
}

extern "C" qrnnt_status qrnnt_decode(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                                     int32_t max_sym, int32_t max_len, int32_t *tokens_out, int32_t *len_out,
                                     float *score_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return qrnnt_decode_ex(m, enc_proj, T, B, W, max_sym, max_len, 0u, tokens_out, len_out, score_out, workspace,
                           workspace_bytes, stream);
}

extern "C" qrnnt_status qrnnt_decode_ex(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                                        int32_t max_sym, int32_t max_len, uint32_t flags, int32_t *tokens_out,
                                        int32_t *len_out, float *score_out, void *workspace, size_t workspace_bytes,
                                        void *stream)
{
    qrnnt_status s = check_model(m);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE(enc_proj && tokens_out && len_out && score_out && workspace, QRNNT_ERR_NULL);
    QR_REQUIRE(T > 0 && B > 0 && W > 0 && max_len > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(W <= 64, QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(max_sym >= 0 && max_sym <= 16, QRNNT_ERR_RANGE);
    QR_REQUIRE((flags & ~(uint32_t)QRNNT_DECODE_EARLY_STOP) == 0u, QRNNT_ERR_RANGE);
    const bool early = (flags & QRNNT_DECODE_EARLY_STOP) != 0u;
    QR_REQUIRE((double)T * (max_sym > 0 ? max_sym : 1) * B * W < 2.0e9, QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(qr_aligned(enc_proj, 16) && qr_aligned(workspace, 256), QRNNT_ERR_ALIGN);
    Plan p;
    make_plan(m, T, B, W, max_sym, workspace, p);
    QR_REQUIRE(workspace_bytes >= p.total, QRNNT_ERR_WORKSPACE);
    hipStream_t st = (hipStream_t)stream;
    const int N = p.N, V = p.V;
    const size_t Ns = (size_t)N;
    const int ZB = p.NB - 1;   // second A0 buffer; holds the zero state before the first frame
    const int n_embed_rows = V;

    // zero state in buffer ZB, then every slot consumes the start symbol into buffer 0
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        const qrnnt_net *net = net_of(m, k);
        for (int l = 0; l < net->n_layers; ++l) {
            const size_t H = (size_t)net->layer[l].hidden_size;
            size_t nw = Ns * H / 4;
            fill_words_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)(p.net[k].h[l] + (size_t)ZB * Ns * H), nw, 0u);
            nw = Ns * H;
            fill_words_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)(p.net[k].c[l] + (size_t)ZB * Ns * H), nw, 0u);
        }
    }
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        qr_launch_input_projection(&net_of(m, k)->layer[0], net_of(m, k)->embed_codes, V, p.net[k].gx0, nullptr, st);
        qr_launch_gx_table(&net_of(m, k)->layer[0], p.net[k].gx0, V, p.net[k].tab0, st);
    }
    fill_words_kernel<<<1, 256, 0, st>>>((uint32_t *)p.live, 2 * (size_t)(max_sym + 2), 0u);
    fill_words_kernel<<<1, 256, 0, st>>>((uint32_t *)p.n_rows, 2 * (size_t)(max_sym + 2), 0u);
    decode_init_kernel<<<(N + 255) / 256 + 1, 256, 0, st>>>(p.score, p.node, p.len, p.parent_idx, p.token, p.active,
                                                            p.nx_count, p.node_tok, p.node_prev, N, W, B, m->blank);
    advance_nets(m, p, ZB, 0, n_embed_rows, nullptr, nullptr, st);

    // The state rows a new beam slot takes over from its source (copied by the first joint + selection kernel of
    // the next frame, see joint_route_kernel)
    QrGatherTable tb = {};
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        const qrnnt_net *net = net_of(m, k);
        for (int l = 0; l < net->n_layers; ++l) {
            tb.base[tb.n] = (char *)p.net[k].h[l];  tb.row_bytes[tb.n++] = net->layer[l].hidden_size;
            tb.base[tb.n] = (char *)p.net[k].c[l];  tb.row_bytes[tb.n++] = net->layer[l].hidden_size * 4;
        }
        tb.base[tb.n] = (char *)p.net[k].y;  tb.row_bytes[tb.n++] = net->out.rows * 4;
    }
    tb.beam_src = p.beam_src;  tb.N = N;  tb.src_limit = p.NB * N;
    const QrGatherTable no_copy = {};

    QrJointArgs ja = {};
    ja.enc = enc_proj;  ja.n_enc_rows = T * B;  ja.frame_row = nullptr;  ja.rows_per_utt = W;
    ja.w = (const v4i *)m->joint_out.packed;  ja.s_w = m->joint_out.row_scale;  ja.b_out = m->joint_bias;
    ja.z_scale = m->z_scale;  ja.z_inv = m->z_inv_scale;
    ja.lambda_src = m->lambda_src;  ja.lambda_ext = m->lambda_ext;  ja.rho = m->rho;
    ja.N = N;  ja.J = p.J;  ja.V = V;  ja.blank = m->blank;
    ja.nkc = qr_round_up(p.J, QRNNT_KCHUNK) / QRNNT_KCHUNK;
    ja.w8 = qr_bits(&m->joint_out) == 8;

    int a0 = 0;   // buffer of the beam at the current frame
    for (int t = 0; t < T; ++t) {
        for (int v = 0; v <= max_sym; ++v) {
            const int cur = (v == 0) ? a0 : v;
            const int nxt = v + 1;   // only used when v < max_sym
            ja.frame_base = t * B;
            // first round of a frame after the first: the beam's cached outputs are still where their sources left
            // them (read through beam_src); this kernel's spare workgroups move all state rows into buffer `cur`
            const bool moving = (v == 0 && t > 0);
            const size_t yb = moving ? 0 : (size_t)cur;
            ja.pred = p.net[0].y + yb * Ns * p.J;
            ja.lp_src = m->use_src ? p.net[1].y + yb * Ns * V : nullptr;
            ja.lp_ext = m->use_ext ? p.net[2].y + yb * Ns * V : nullptr;
            ja.row_idx = moving ? p.beam_src : nullptr;
            ja.row_idx_buf = cur;
            tb.dst_buf = cur;
            const int last = (v == max_sym);
            QrRouteArgs ra = {};
            ra.score_src = p.score + (size_t)cur * Ns;
            ra.B = B;  ra.W = W;  ra.V = V;  ra.R = p.R;  ra.blank = m->blank;  ra.src_buf = cur;  ra.last_round = last;
            ra.node_base = 1 + (t * max_sym + v) * N;
            ra.node_src = p.node + (size_t)cur * Ns;  ra.len_src = p.len + (size_t)cur * Ns;
            ra.score_dst = p.score + (size_t)nxt * Ns;  ra.node_dst = p.node + (size_t)nxt * Ns;
            ra.len_dst = p.len + (size_t)nxt * Ns;
            ra.parent_idx = p.parent_idx;  ra.token = p.token;  ra.active = p.active;
            ra.nx_score = p.nx_score;  ra.nx_info = p.nx_info;  ra.nx_count = p.nx_count;
            ra.node_tok = p.node_tok;  ra.node_prev = p.node_prev;
            ra.fe_dst_buf = (a0 == 0) ? ZB : 0;
            ra.fe_score_all = p.score;
            ra.fe_node_all_w = p.node;  ra.fe_len_all_w = p.len;  ra.beam_src = p.beam_src;
            if (early) {   // live[t&1][v] = utterances that carried a label into round v of this frame
                int32_t *lv = p.live + (size_t)(t & 1) * (max_sym + 2), *lo = p.live + (size_t)((t + 1) & 1) * (max_sym + 2);
                ra.gate = v > 0 ? lv + v : nullptr;
                ra.live_next = lv + v + 1;
                ra.live_clear = lo + v + 1;
            }
            // n_rows[t&1][v] = slots that carry a label into round v of this frame, listed in p.rows
            ra.rows_next = p.rows;
            ra.n_rows_next = p.n_rows + (size_t)(t & 1) * (max_sym + 2) + v + 1;
            ra.n_rows_clear = p.n_rows + (size_t)((t + 1) & 1) * (max_sym + 2) + v + 1;
            qr_launch_joint_route(ja, ra, moving ? tb : no_copy, st);
            if (!last) advance_nets(m, p, cur, nxt, n_embed_rows, early ? ra.live_next : nullptr, ra.n_rows_next, st);
        }
        a0 = (a0 == 0) ? ZB : 0;   // the new beam's buffer; its state rows follow in the next frame's first kernel
    }
    backtrack_kernel<<<(N + 63) / 64, 64, 0, st>>>(p.score + (size_t)a0 * Ns, p.node + (size_t)a0 * Ns,
                                                   p.len + (size_t)a0 * Ns, p.node_tok, p.node_prev, N, max_len,
                                                   tokens_out, len_out, score_out);
    return qr_launch_status();
}

// ---------------------------------------------------------------------------------------------------------
// Alignment-length synchronous search with recombination (Sec. 2: the search the paper decodes with).

namespace {

struct AlsdPlan {
    Plan p;                        // network buffers (2 state buffers), parent_idx / token / active, label trie
    unsigned long long *hash;      // [2][N]
    float *fin_score;  int32_t *fin_node, *fin_len;   // [N]
    int n_iter;
};

void make_alsd_plan(const qrnnt_model *m, int T, int B, int W, int u_max, void *ws, AlsdPlan &ap)
{
    Plan &p = ap.p;
    p = Plan{};
    p.T = T; p.B = B; p.W = W; p.N = B * W; p.max_sym = 0;
    p.R = 1; p.NB = 2; p.V = m->V; p.J = m->joint_out.cols;
    ap.n_iter = T + u_max;
    Carver cv{(char *)ws, 0};
    const size_t N = (size_t)p.N, NB = 2;
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        const qrnnt_net *net = net_of(m, k);
        for (int l = 0; l < net->n_layers; ++l) {
            p.net[k].h[l] = cv.take<int8_t>(NB * N * net->layer[l].hidden_size);
            p.net[k].c[l] = cv.take<float>(NB * N * net->layer[l].hidden_size);
        }
        p.net[k].y = cv.take<float>(NB * N * net->out.rows);
        p.net[k].gx0 = cv.take<int32_t>((size_t)m->V * 4 * net->layer[0].hidden_size);
        p.net[k].tab0 = cv.take<float>((size_t)m->V * 4 * net->layer[0].hidden_size);
        p.net[k].mid_q = net->mid.packed ? cv.take<int8_t>(N * net->mid.rows) : nullptr;
    }
    p.score = cv.take<float>(NB * N);
    p.node = cv.take<int32_t>(NB * N);
    p.len = cv.take<int32_t>(NB * N);
    ap.hash = cv.take<unsigned long long>(NB * N);
    p.parent_idx = cv.take<int32_t>(N);
    p.token = cv.take<int32_t>(N);
    p.active = cv.take<uint8_t>(N);
    p.nx_count = cv.take<int32_t>(B);
    ap.fin_score = cv.take<float>(N);
    ap.fin_node = cv.take<int32_t>(N);
    ap.fin_len = cv.take<int32_t>(N);
    const size_t pool = 1 + (size_t)ap.n_iter * N;
    p.node_tok = cv.take<int32_t>(pool);
    p.node_prev = cv.take<int32_t>(pool);
    p.live = cv.take<int32_t>((size_t)ap.n_iter + 2);
    p.rows = nullptr;  p.n_rows = nullptr;
    p.total = (cv.off + 255) / 256 * 256;
}

bool alsd_args_ok(int32_t T, int32_t B, int32_t W, int32_t u_max)
{
    return T > 0 && B > 0 && W > 0 && W <= 64 && u_max >= 0 && (double)(T + (double)u_max) * B * W < 2.0e9;
}

}  // namespace

extern "C" size_t qrnnt_decode_alsd_workspace(const qrnnt_model *m, int32_t T, int32_t B, int32_t W, int32_t u_max)
{
    if (check_model(m) != QRNNT_OK || !alsd_args_ok(T, B, W, u_max)) return 0;
    AlsdPlan ap;
    make_alsd_plan(m, T, B, W, u_max, nullptr, ap);
    return ap.p.total;
}

extern "C" qrnnt_status qrnnt_decode_alsd(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                                          int32_t u_max, int32_t max_len, int32_t *tokens_out, int32_t *len_out,
                                          float *score_out, void *workspace, size_t workspace_bytes, void *stream)
{
    return qrnnt_decode_alsd_ex(m, enc_proj, T, B, W, u_max, max_len, 0u, nullptr, tokens_out, len_out, score_out,
                                workspace, workspace_bytes, stream);
}

extern "C" qrnnt_status qrnnt_decode_alsd_ex(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                                             int32_t u_max, int32_t max_len, uint32_t flags, int32_t *stats,
                                             int32_t *tokens_out, int32_t *len_out, float *score_out, void *workspace,
                                             size_t workspace_bytes, void *stream)
{
    qrnnt_status s = check_model(m);
    if (s != QRNNT_OK) return s;
    QR_REQUIRE((flags & ~(uint32_t)QRNNT_ALSD_REUSE) == 0u, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(stats, 4), QRNNT_ERR_ALIGN);
    QR_REQUIRE(enc_proj && tokens_out && len_out && score_out && workspace, QRNNT_ERR_NULL);
    QR_REQUIRE(T > 0 && B > 0 && W > 0 && max_len > 0 && u_max >= 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(W <= 64, QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(alsd_args_ok(T, B, W, u_max), QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(qr_aligned(enc_proj, 16) && qr_aligned(workspace, 256), QRNNT_ERR_ALIGN);
    AlsdPlan ap;
    make_alsd_plan(m, T, B, W, u_max, workspace, ap);
    const Plan &p = ap.p;
    QR_REQUIRE(workspace_bytes >= p.total, QRNNT_ERR_WORKSPACE);
    hipStream_t st = (hipStream_t)stream;
    const int N = p.N, V = p.V;
    const size_t Ns = (size_t)N;

    // zero state in buffer 1, then every slot consumes the start symbol into buffer 0
    for (int k = 0; k < 3; ++k) {
        if (!net_used(m, k)) continue;
        const qrnnt_net *net = net_of(m, k);
        for (int l = 0; l < net->n_layers; ++l) {
            const size_t H = (size_t)net->layer[l].hidden_size;
            size_t nw = Ns * H / 4;
            fill_words_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)(p.net[k].h[l] + Ns * H), nw, 0u);
            nw = Ns * H;
            fill_words_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)(p.net[k].c[l] + Ns * H), nw, 0u);
        }
        qr_launch_input_projection(&net->layer[0], net->embed_codes, V, p.net[k].gx0, nullptr, st);
        qr_launch_gx_table(&net->layer[0], p.net[k].gx0, V, p.net[k].tab0, st);
    }
    {
        size_t nw = (size_t)ap.n_iter + 2;
        fill_words_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)p.live, nw, 0u);
        nw = 2 * Ns * 2;
        fill_words_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>((uint32_t *)ap.hash, nw, 0u);
        fill_words_kernel<<<(unsigned)((Ns + 255) / 256), 256, 0, st>>>((uint32_t *)ap.fin_score, Ns, 0xFF800000u);   // -inf
        fill_words_kernel<<<(unsigned)((Ns + 255) / 256), 256, 0, st>>>((uint32_t *)ap.fin_node, Ns, 0u);
        fill_words_kernel<<<(unsigned)((Ns + 255) / 256), 256, 0, st>>>((uint32_t *)ap.fin_len, Ns, 0u);
    }
    decode_init_kernel<<<(N + 255) / 256 + 1, 256, 0, st>>>(p.score, p.node, p.len, p.parent_idx, p.token, p.active,
                                                            p.nx_count, p.node_tok, p.node_prev, N, W, B, m->blank);
    advance_nets(m, p, 1, 0, V, nullptr, nullptr, st);

    QrJointArgs ja = {};
    ja.enc = enc_proj;  ja.n_enc_rows = T * B;  ja.frame_row = nullptr;  ja.rows_per_utt = W;  ja.frame_base = 0;
    ja.w = (const v4i *)m->joint_out.packed;  ja.s_w = m->joint_out.row_scale;  ja.b_out = m->joint_bias;
    ja.z_scale = m->z_scale;  ja.z_inv = m->z_inv_scale;
    ja.lambda_src = m->lambda_src;  ja.lambda_ext = m->lambda_ext;  ja.rho = m->rho;
    ja.N = N;  ja.J = p.J;  ja.V = V;  ja.blank = m->blank;
    ja.nkc = qr_round_up(p.J, QRNNT_KCHUNK) / QRNNT_KCHUNK;
    ja.w8 = qr_bits(&m->joint_out) == 8;

    int cur = 0;
    for (int i = 0; i < ap.n_iter; ++i) {
        const int nxt = cur ^ 1;
        ja.pred = p.net[0].y + (size_t)cur * Ns * p.J;
        ja.lp_src = m->use_src ? p.net[1].y + (size_t)cur * Ns * V : nullptr;
        ja.lp_ext = m->use_ext ? p.net[2].y + (size_t)cur * Ns * V : nullptr;
        QrRouteArgs ra = {};
        ra.score_src = p.score + (size_t)cur * Ns;
        ra.B = B;  ra.W = W;  ra.V = V;  ra.R = 1;  ra.blank = m->blank;  ra.src_buf = cur;  ra.last_round = 0;
        ra.node_base = 1 + i * N;
        ra.node_src = p.node + (size_t)cur * Ns;  ra.len_src = p.len + (size_t)cur * Ns;
        ra.score_dst = p.score + (size_t)nxt * Ns;  ra.node_dst = p.node + (size_t)nxt * Ns;
        ra.len_dst = p.len + (size_t)nxt * Ns;
        ra.parent_idx = p.parent_idx;  ra.token = p.token;  ra.active = p.active;
        ra.node_tok = p.node_tok;  ra.node_prev = p.node_prev;
        ra.gate = i > 0 ? p.live + i : nullptr;   // live[i]: utterances with a live hypothesis entering iteration i
        ra.live_next = p.live + i + 1;
        QrAlsdArgs sa = {};
        sa.iter = i;  sa.T = T;  sa.u_max = u_max;
        sa.hash_src = ap.hash + (size_t)cur * Ns;  sa.hash_dst = ap.hash + (size_t)nxt * Ns;
        sa.fin_score = ap.fin_score;  sa.fin_node = ap.fin_node;  sa.fin_len = ap.fin_len;
        sa.reuse = (flags & QRNNT_ALSD_REUSE) ? 1 : 0;  sa.stats = stats;
        qr_launch_joint_alsd(ja, ra, sa, st);
        if (i + 1 < ap.n_iter) advance_nets(m, p, cur, nxt, V, ra.live_next, nullptr, st);
        cur = nxt;
    }
    backtrack_kernel<<<(N + 63) / 64, 64, 0, st>>>(ap.fin_score, ap.fin_node, ap.fin_len, p.node_tok, p.node_prev, N,
                                                   max_len, tokens_out, len_out, score_out);
    return qr_launch_status();
}
