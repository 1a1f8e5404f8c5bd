// Internal launch interface between the translation units of libqrnnt.  The
// public entry points validate and then call these; the decoder calls them
// directly.  Nothing here is exported.
#pragma once

#include "qrnnt_common.h"

#define QR_HIDDEN __attribute__((visibility("hidden")))

struct QrStepArgs {
    const v4i *wih, *whh;             // TILED_GATES blobs
    const float *s_wih, *s_whh, *bias;
    const int8_t *x;  int64_t ld_x;   // input codes, row pitch in bytes
    const int32_t *x_row;  int n_x_rows; // optional row index into x (or into gx) per hypothesis; rows available
    const int32_t *gx;  int64_t ld_gx; // precomputed input projection [rows, 4H], tiled-row order (USE_GX only)
    const float *tabf;                 // optional fp32 form of gx with scales, bias and exp2 constants folded in
    const int32_t *parent;  int n_slots;
    const int8_t *h_prev;  int64_t ld_hp;
    const float *c_prev;
    const uint8_t *active;
    int8_t *h_next;  int64_t ld_hn;
    float *c_next;
    int8_t *h_copy;                    // optional second copy of the output codes [N, H]
    int32_t *dbg_accx, *dbg_acch;
    float *dbg_gates;
    int I, H, N, nkc_x, nkc_h;
    float x_scale, h_scale, h_inv;
};

#define QR_MAX_GROUP 3
struct QrStepGroup {
    QrStepArgs p[QR_MAX_GROUP];
    int n;
    const int32_t *gate;               // optional [device]: the launch does nothing when *gate == 0
    // optional [device] (same N, parent and x_row arrays for all members): the launch advances the hypotheses
    // listed in rows[0 .. *n_rows) and leaves every other row of the outputs untouched.  An entry is
    // (hypothesis n, parent[n], x_row[n], unused): what the kernel would otherwise fetch through n, so that
    // the list adds no link to its chain of dependent loads.  Entries beyond the end may hold anything.
    const v4i *rows = nullptr;
    const int32_t *n_rows = nullptr;
    // filled in by the launcher of the tiled kernel: row blocks of all members together, compute units of the device,
    // and (launches without a list) log2 of how many times narrower than the full column block a workgroup's share is
    int row_blocks = 0, n_cu = 0, width = 0;
    int col_block0 = 0;                // first column block of this launch (a grid's z extent is limited to 65535)
};

struct QrLinearArgs {
    const v4i *w;  int nkc, rows;
    const float *s_w, *bias;
    float a_scale;
    const int8_t *act;  int K, N;
    float *y;  int32_t *dbg_acc;
    int log_softmax;
    int8_t *q_out;  float q_inv;  int q_bits;   // optional: codes of y under the next layer's input quantizer, [N, rows]
    int w8;                            // 8-bit weights
};

struct QrLinearGroup {
    QrLinearArgs p[QR_MAX_GROUP];
    int n;
    const int32_t *gate;               // optional [device]: the launch does nothing when *gate == 0
    // optional [device] (same N for all members), as in QrStepGroup: only the activation rows n listed in
    // rows[0 .. *n_rows) (first word of an entry) are computed, every other row of the outputs stays as it is.
    const v4i *rows = nullptr;
    const int32_t *n_rows = nullptr;
};

// State tensors of the decoder ([buffers][N][row]): what a new beam slot copies from its source (buffer, slot).
#define QR_MAX_GATHER 32
struct QrGatherTable {
    char *base[QR_MAX_GATHER];
    int row_bytes[QR_MAX_GATHER];
    int n;                             // 0: nothing to copy
    const int32_t *beam_src;           // [N] flat source row (buffer * N + slot) of every new beam slot, -1: empty rank
    int N, dst_buf;
    int src_limit;                     // flat source rows are below this (buffers x N); anything else is skipped
};

struct QrJointArgs {
    const float *enc;  int n_enc_rows;
    const int32_t *frame_row;          // per-row encoder row, or null: row = frame_base + n / rows_per_utt
    int frame_base, rows_per_utt;
    const float *pred;
    const v4i *w;  const float *s_w;  const float *b_out;
    float z_scale, z_inv;
    const float *lp_src, *lp_ext;
    float lambda_src, lambda_ext, rho;
    int N, J, V, blank, nkc;
    float *lp_out;  int8_t *dbg_zq;  float *fused;
    int w8;                            // 8-bit output layer: 8-bit weights and an 8-bit quantizer on z
    const int32_t *row_idx;            // optional (decoding loop): hypothesis n reads row row_idx[n] of pred / lp_src / lp_ext
                                       // (which then point at buffer 0 of those arrays); < 0: row n of buffer row_idx_buf
    int row_idx_buf;
};

struct QrRouteArgs {
    const float *score_src;                         // [B,W] of the current round
    int B, W, V, R, blank, src_buf, last_round, node_base;
    const int32_t *node_src, *len_src;              // [N] of the current round
    float *score_dst;  int32_t *node_dst, *len_dst; // [N] of the next round
    int32_t *parent_idx, *token;  uint8_t *active;  // [N] inputs of the next network advance
    float *nx_score;  v4i *nx_info;  int32_t *nx_count;   // the frame's candidate list; info = (flat source (buffer, slot), trie node, length, -)
    int32_t *node_tok, *node_prev;                  // label trie
    // end of the frame (used when last_round): the W best of the candidate list become the beam in buffer fe_dst_buf
    int fe_dst_buf;
    float *fe_score_all;  int32_t *fe_node_all_w, *fe_len_all_w;
    int32_t *beam_src;                              // [N] flat source (buffer, slot) of every new beam slot, or -1
    // early stop (all optional): the round is dead when *gate == 0; an utterance that picked a label
    // adds 1 to *live_next; workgroup 0 clears *live_clear for a later frame
    const int32_t *gate;  int32_t *live_next, *live_clear;
    // list of the slots that carry a label into the next round (optional, see QrStepGroup.rows): every utterance
    // appends its slots at rows_next[old *n_rows_next ...]; workgroup 0 clears *n_rows_clear for a later frame
    v4i *rows_next;  int32_t *n_rows_next, *n_rows_clear;
};

// One direction of the persistent recurrence (see recurrence.hip).
// Alignment-length synchronous search: what one iteration needs beyond QrRouteArgs (of which it uses score/node/len
// src and dst, parent_idx/token/active, the label trie, node_base, gate and live_next).
struct QrAlsdArgs {
    int iter, T, u_max;                              // hypothesis w stands at frame iter - len[w]
    const unsigned long long *hash_src;              // [N] hash of the label sequence (recombination key, with the length)
    unsigned long long *hash_dst;
    float *fin_score;  int32_t *fin_node, *fin_len;  // [B,W] the W best finished hypotheses so far, best first
    int reuse;                                       // a label pick whose sequence a live hypothesis of the beam holds takes over its states
    int32_t *stats;                                  // optional [device] int32[2]: += label picks that kept their slot, += those that reused states
};

struct QrRecArgs {
    const v4i *whh;  const float *s_wih, *s_whh, *bias;
    const int32_t *gx;                 // [T*B, 4H] gate-interleaved input projection
    const int8_t *h0;  const float *c0;
    int8_t *h_out;  int64_t ld_out;  int col_off;
    int8_t *h_last;  float *c_last;  float *dbg_c_all;
    unsigned long long *xbuf;          // [2][B][H/4] exchange words, zeroed before the launch
    int *err;                          // set to 1 when a bounded wait ran out
    int T, B, H, nkc_h, reverse, spin_limit;
    float x_scale, h_scale, h_inv;
    int w8;                            // 8-bit layer: 8-bit W_hh blob and an 8-bit hidden-state quantizer
};
struct QrRecGroup {
    QrRecArgs d[2];
    int n;
};
QR_HIDDEN bool qr_rec_supported(int H, int B);
QR_HIDDEN size_t qr_rec_xbuf_bytes(int H, int B);
QR_HIDDEN bool qr_launch_recurrence(const QrRecGroup &g, hipStream_t st);

QR_HIDDEN void qr_fill_lstm_weights(QrStepArgs &a, const qrnnt_lstm *L);
QR_HIDDEN qrnnt_status qr_check_lstm(const qrnnt_lstm *L);
QR_HIDDEN void qr_launch_lstm_step(const QrStepArgs &a, bool use_gx, hipStream_t st);
QR_HIDDEN void qr_launch_lstm_step_group(const QrStepGroup &g, bool use_gx, hipStream_t st);
QR_HIDDEN void qr_launch_gx_table(const qrnnt_lstm *L, const int32_t *gx, int M, float *tab, hipStream_t st);
QR_HIDDEN void qr_launch_input_projection(const qrnnt_lstm *L, const int8_t *x_codes, int M, int32_t *gx, int32_t *dbg_accx,
                                          hipStream_t st);
QR_HIDDEN void qr_launch_linear_group(const QrLinearGroup &g, hipStream_t st);
QR_HIDDEN void qr_launch_linear(const QrLinearArgs &a, hipStream_t st);
QR_HIDDEN void qr_launch_joint(const QrJointArgs &a, hipStream_t st);
QR_HIDDEN void qr_launch_joint_route(const QrJointArgs &a, const QrRouteArgs &r, const QrGatherTable &gt, hipStream_t st);
QR_HIDDEN void qr_launch_joint_alsd(const QrJointArgs &a, const QrRouteArgs &r, const QrAlsdArgs &s, hipStream_t st);
QR_HIDDEN void qr_launch_beam(const float *score, const float *fused, int B, int W, int V, int blank, int force_blank,
                              int32_t *parent_out, int32_t *token_out, float *score_out, hipStream_t st);
