/*
 * qrnnt.h -- C ABI of libqrnnt: INT4 RNN-T inference with density-ratio LM
 * fusion on one AMD MI355X (gfx950).
 *
 * The calls follow the statement of the method in arXiv 2206.07882: weights
 * are quantized once (Sec. 3.2), activations at every step; LSTM cells take
 * integer inputs and hidden states, keep an unquantized cell state and emit
 * the hidden state as a 4-bit code at the cell output ("Outer" quantization,
 * Sec. 3.4); the joint network combines encoder and prediction outputs
 * multiplicatively and ends in a log-softmax (Sec. 2); scores are fused by
 * Eq. 1; a beam of up to 16 hypotheses is kept per utterance (Sec. 2).
 *
 * Conventions that hold for every entry point
 *   - Pointers marked [device] must be device memory reachable from the GPU
 *     that is current on the calling thread; pointers marked [host] are host
 *     memory.  The caller owns every buffer, including workspaces; the library
 *     allocates no device memory.  The only state it keeps between calls is what
 *     it has learned about each device on first use (number of compute units,
 *     how many workgroups of the persistent recurrence fit at once, kernel
 *     attributes already set), cached per device; no call's result depends on
 *     an earlier call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued asynchronously; nothing synchronises.
 *   - Every call validates its arguments on the host before launching
 *     anything and returns a qrnnt_status; nothing throws across the boundary.
 *     Validation needs no GPU.
 *   - Activation codes travel as int8 containers holding values in [-8, 7].
 *     A matrix of activation codes with C columns ([N, I] inputs of an LSTM
 *     layer, [V, E] embedding tables) is stored with a row pitch of
 *     qrnnt_act_pitch(C) = C rounded up to a multiple of 16 bytes, so that every
 *     row starts on a 16-byte boundary; the bytes behind column C may hold
 *     anything (they meet the zero padding of the packed weights).  Where C is a
 *     multiple of 16, as every hidden size is, this is the plain [N, C] array.
 *     qrnnt_quantize_act_rows writes that form from fp32 rows of any width.
 *     Weights only exist as nibble-packed blobs written by qrnnt_pack_int4.
 *   - Quantizer: q = clamp(rne(x * inv_step), -8, 7), product in fp32, ties to
 *     even; step = alpha/7 (symmetric LQ of Sec. 3.1 on a signed 4-bit grid).
 *   - LSTM gate rows are ordered i, f, g, o (rows [0,H), [H,2H), ...).
 */
#ifndef QRNNT_H
#define QRNNT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    QRNNT_OK = 0,
    QRNNT_ERR_NULL = 1,        /* a required pointer is NULL */
    QRNNT_ERR_SHAPE = 2,       /* a dimension is non-positive or violates a stated multiple */
    QRNNT_ERR_ALIGN = 3,       /* a pointer violates its stated alignment */
    QRNNT_ERR_RANGE = 4,       /* a scalar argument is outside its domain */
    QRNNT_ERR_WORKSPACE = 5,   /* workspace too small */
    QRNNT_ERR_LAYOUT = 6,      /* unknown or unsuitable weight layout */
    QRNNT_ERR_UNSUPPORTED = 7, /* valid but not implemented for this size */
    QRNNT_ERR_HIP = 8          /* the HIP runtime reported an error at launch */
} qrnnt_status;

const char *qrnnt_status_str(qrnnt_status s);
uint32_t qrnnt_abi_version(void);

/* Weight layouts.
 * ROWMAJOR: byte j of row r holds element (r,2j) in bits 0-3 and (r,2j+1) in
 *   bits 4-7 (two's complement); columns are zero-padded to cols_padded.
 *   Exchange/test format; compute kernels do not read it.
 * TILED: rows padded to a multiple of 16 and columns to a multiple of 128,
 *   stored as 1 KiB blocks [row_tile][k_chunk]; inside a block, lane l of a
 *   wavefront owns 16 bytes at offset 16*l whose dword d, byte b holds, in its
 *   low nibble, W[16*row_tile + l%16][128*k_chunk + 16*(l/16) + 4*d + b] and,
 *   in its high nibble, the element 64 columns further.  One 128-bit load per
 *   lane thus yields two int8 MFMA operands after two mask/shift operations.
 * TILED_GATES: TILED applied after permuting the 4H gate rows (source row
 *   g*H + j = gate g of cell j) in groups of 16 cells = 64 tiled rows: cell
 *   j = 16*q + 4*a + b, gate g is tiled row 64*q + 16*b + 4*a + g (rows padded
 *   to a multiple of 64).  The four gates of a cell land in one lane's
 *   accumulator quartet, and over the 4 row tiles of a group a lane owns 4
 *   consecutive cells.  Row scales and biases stay in source order.
 * 8-bit matrices (bits = 8; Sec. 3.2 keeps the first encoder layer and the
 * RNN-T's linear layers at 8 bits) use the same three layouts with one byte per
 * element: ROWMAJOR rows are padded to a multiple of 64 bytes; in TILED and
 * TILED_GATES every [row_tile][k_chunk] position holds two 1 KiB blocks, the
 * first with W[16*row_tile + l%16][128*k_chunk + 16*(l/16) + 4*d + b] at byte
 * 16*l + 4*d + b, the second with the elements 64 columns further: the two
 * MFMA operands of the chunk as they are. */
enum { QRNNT_LAYOUT_ROWMAJOR = 0, QRNNT_LAYOUT_TILED = 1, QRNNT_LAYOUT_TILED_GATES = 2 };
enum { QRNNT_SRC_INT8_CODES = 0, QRNNT_SRC_FP32 = 1 };

/* One quantized matrix: value[r,k] = row_scale[r] * code[r,k]. */
typedef struct {
    const void *packed;     /* [device] written by qrnnt_pack_int4, 16-byte aligned */
    const float *row_scale; /* [device] [rows] fp32 */
    int32_t rows, cols;     /* logical size */
    int32_t layout;         /* QRNNT_LAYOUT_* */
    int32_t bits;           /* 4 (0 is read as 4: qrnnt_pack_int4) or 8 (qrnnt_pack_int8) */
} qrnnt_qmat;

/* One LSTM layer-direction (Sec. 3.2): both matrices in TILED_GATES layout,
 * rows = 4*hidden_size, both of the same width.  The hidden-state quantizer
 * has the width of the weights: codes in [-8,7] for a 4-bit layer, [-128,127]
 * for an 8-bit one (FIX +-1: h_inv_scale 7 resp. 127).  8-bit layers run in
 * qrnnt_input_projection, qrnnt_lstm_layer and qrnnt_bilstm_layer (the encoder's
 * first layer); the single-step entry points take 4-bit layers only. */
typedef struct {
    qrnnt_qmat w_ih;        /* [4H, I] */
    qrnnt_qmat w_hh;        /* [4H, H] */
    const float *bias;      /* [device] [4H] fp32, b_ih + b_hh, not quantized */
    float x_scale;          /* step of the input codes */
    float h_scale;          /* step of the hidden codes (FIX +-1: 1/7) */
    float h_inv_scale;      /* 7/alpha of the hidden quantizer (FIX +-1: 7) */
    int32_t input_size, hidden_size; /* hidden_size a multiple of 16; input_size any (rows of input codes
                                        have the pitch qrnnt_act_pitch(input_size)) */
} qrnnt_lstm;

/* ---- weights: quantize once, pack (Sec. 3.1 MAX per row + symmetric LQ; Sec. 3.2) ---- */

/* Bytes of the packed blob for a rows x cols matrix in `layout`; 0 on bad arguments. */
size_t qrnnt_pack_int4_bytes(int32_t rows, int32_t cols, int32_t layout);

/* src [device]: rows x cols row-major, either int8 codes in [-8,7]
 * (QRNNT_SRC_INT8_CODES; row_scale_out untouched, may be NULL) or fp32 weights
 * (QRNNT_SRC_FP32; each row gets alpha = max|w|, row_scale_out[r] = alpha/7,
 * code = clamp(rne(w * (7/alpha))); an all-zero row gets scale 1, codes 0).
 * packed_out [device]: qrnnt_pack_int4_bytes bytes, 16-byte aligned, fully
 * written (padding included).  TILED_GATES needs rows % 4 == 0. */
qrnnt_status qrnnt_pack_int4(const void *src, int32_t src_dtype, int32_t rows, int32_t cols, int32_t layout,
                             void *packed_out, float *row_scale_out, void *stream);

/* The same at 8 bits (Sec. 3.2: MAX quantizer, 8 bits): codes in [-128,127] are
 * taken as they are; fp32 rows get alpha = max|w|, row_scale_out[r] = alpha/127,
 * code = clamp(rne(w * (127/alpha)), -128, 127).  The caller sets bits = 8 in
 * the qrnnt_qmat that describes the result. */
size_t qrnnt_pack_int8_bytes(int32_t rows, int32_t cols, int32_t layout);
qrnnt_status qrnnt_pack_int8(const void *src, int32_t src_dtype, int32_t rows, int32_t cols, int32_t layout,
                             void *packed_out, float *row_scale_out, void *stream);

/* Inverse of the packing, for tests: codes_out [device] rows x cols int8 in
 * source row order.  Reads m->bits (both widths). */
qrnnt_status qrnnt_unpack_int4(const qrnnt_qmat *m, int8_t *codes_out, void *stream);

/* ---- activations (Sec. 3.1 symmetric LQ with a FIX boundary, Sec. 3.2) ---- */

/* q[i] = clamp(rne(x[i] * inv_scale), -8, 7); x, q [device], n elements. */
qrnnt_status qrnnt_quantize_act(const float *x, int64_t n, float inv_scale, int8_t *q, void *stream);
/* The 8-bit form (input of the encoder's first layer, Sec. 3.2): clamp to [-128, 127]. */
qrnnt_status qrnnt_quantize_act8(const float *x, int64_t n, float inv_scale, int8_t *q, void *stream);

/* Row pitch in bytes of an activation-code matrix with `cols` columns (cols rounded up to a multiple of 16). */
int32_t qrnnt_act_pitch(int32_t cols);

/* The same quantizer for a matrix: x [device] fp32 [rows, cols] contiguous (any cols) -> q [device] int8 with a
 * row pitch of ld_out bytes (ld_out >= cols, a multiple of 16; normally qrnnt_act_pitch(cols)); bits = 4 clamps
 * to [-8, 7], bits = 8 to [-128, 127]; the bytes behind column cols are written as zero.  This is how features of
 * any width (Sec. 2: 340) and embedding tables of any width (Sec. 2: "a small embedding") reach the LSTM entry
 * points. */
qrnnt_status qrnnt_quantize_act_rows(const float *x, int64_t rows, int32_t cols, float inv_scale, int32_t bits,
                                     int8_t *q, int32_t ld_out, void *stream);

/* ---- quantized linear layer (Sec. 3.2: weights and inputs quantized) ---- */

/* y[n,r] = a_scale * row_scale[r] * sum_k w[r,k]*a[n,k] + bias[r]; with
 * log_softmax != 0 each row of y is replaced by its log-softmax (LM output
 * layer, Sec. 2).  w: TILED layout.  a [device] [N, cols] int8, 16-byte aligned,
 * cols % 16 == 0.  bias [device] [rows] or NULL.  y [device] [N, rows] fp32.
 * dbg_acc [device] [N, rows] int32 or NULL.  log_softmax needs rows <= 64.
 * w may be 4- or 8-bit; the codes in a are contracted as they are (any int8). */
qrnnt_status qrnnt_linear(const qrnnt_qmat *w, const float *bias, float a_scale, const int8_t *a, int32_t N,
                          int32_t log_softmax, float *y, int32_t *dbg_acc, void *stream);

/* qrnnt_linear feeding another quantized linear layer (Sec. 3.2: linear layers
 * quantize their inputs): q[n,r] = clamp(rne(y[n,r] * inv_scale), lo, hi) with y
 * as in qrnnt_linear (no log-softmax) and [lo,hi] = [-8,7] for bits = 4,
 * [-128,127] for bits = 8 (the width of the consuming layer); the fp32 y is not
 * stored.  q [device] [N, rows] int8.  This is the bottleneck layer of the
 * external LM (Sec. 2). */
qrnnt_status qrnnt_linear_quant(const qrnnt_qmat *w, const float *bias, float a_scale, const int8_t *a, int32_t N,
                                float inv_scale, int32_t bits, int8_t *q, void *stream);

/* ---- LSTM: one step for a set of hypotheses (Sec. 3.2, Sec. 3.4) ---- */

/* For n in [0,N): input row x_codes[x_row ? x_row[n] : n] (length I, row pitch qrnnt_act_pitch(I)), previous
 * state from slot s = parent ? parent[n] : n of h_prev/c_prev ([n_slots, H]);
 *   pre = x_scale*s_wih[r]*accx + h_scale*s_whh[r]*acch + bias[r]   (fp32)
 *   i,f,o = sigmoid, g = tanh, c' = f*c + i*g, h' = o*tanh(c'),
 *   h_next[n] = Q(h'; h_inv_scale), c_next[n] = c'.
 * Rows with active[n] == 0 copy slot s through unchanged.  h_next/c_next must
 * not overlap h_prev/c_prev.  Optional debug outputs [device]: dbg_accx,
 * dbg_acch int32 [N,4H], dbg_gates fp32 [N,4H] (activated i,f,g,o), all in
 * source row order.  parent values are clamped to [0, n_slots). */
qrnnt_status qrnnt_lstm_step(const qrnnt_lstm *L, const int8_t *x_codes, const int32_t *x_row, int32_t n_x_rows,
                             const int32_t *parent, const int8_t *h_prev, const float *c_prev, int32_t n_slots,
                             const uint8_t *active, int32_t N, int8_t *h_next, float *c_next,
                             int32_t *dbg_accx, int32_t *dbg_acch, float *dbg_gates, void *stream);

/* Up to 3 independent steps (e.g. the first layers of the prediction network and
 * of both LMs) in one launch, so that small problems fill the GPU together.
 * Each descriptor carries the arguments of qrnnt_lstm_step; its debug outputs are
 * optional as there (dbg_accx is not written by a launch that takes the input part
 * from gx_table: the table holds no integers).  A launch with a debug output runs
 * the debug build of the kernel variant the same launch would run without one.
 * gx [device] int32 [n_x_rows, 4H] or NULL: the input projection of the rows of
 * x_codes as written by qrnnt_input_projection.  When given, the input part of
 * the step is looked up in it (row x_row ? x_row[n] : n) instead of contracted:
 * the same integer sums, e.g. one table row per vocabulary entry for a layer fed
 * by an embedding.  Either every step of a group has gx or none has.
 * gx_table [device] fp32 [n_x_rows, 4H] or NULL: the same rows as written by
 * qrnnt_input_table (scales and bias folded in); steps that have gx may add it,
 * and a launch whose steps all have it uses it in place of gx where that is
 * faster (many hypotheses).
 * steps [host] is read during the call only. */
typedef struct {
    const qrnnt_lstm *L;
    const int8_t *x_codes;  const int32_t *x_row;  int32_t n_x_rows;
    const int32_t *parent;  const int8_t *h_prev;  const float *c_prev;  int32_t n_slots;
    const uint8_t *active;  int32_t N;
    int8_t *h_next;  float *c_next;
    const int32_t *gx;
    const float *gx_table;
    int32_t *dbg_accx, *dbg_acch;   /* [device] int32 [N, 4H] in source row order, or NULL */
    float *dbg_gates;               /* [device] fp32 [N, 4H] activated i,f,g,o, or NULL */
} qrnnt_step_desc;

qrnnt_status qrnnt_lstm_step_group(const qrnnt_step_desc *steps, int32_t n_steps, void *stream);

/* The same launch restricted to a list of hypotheses (Sec. 2: in a round of the
 * beam search only the hypotheses that were extended by a label advance the
 * prediction network and the LMs).
 * list [device] int32 [>= N][4], 16-byte aligned: entry j = (n, slot of n's
 *   previous state, input row of n, unused) for the j-th hypothesis to advance,
 *   i.e. n together with the values the step would read from parent[n] and
 *   x_row[n].  Those two arrays are not read; whether a descriptor has them
 *   (non-NULL) still says whether the entry's second / third word is used or n
 *   itself.  Values are clamped like parent and x_row.
 * n_list [device]: the number of entries, read by the kernel, so that a kernel
 *   earlier on the stream can write list and count without a host round trip.
 *   Entries at or beyond *n_list may hold anything: they may be read, are
 *   clamped into range and nothing is stored for them.  *n_list <= N.
 * Rows of h_next / c_next of hypotheses that are not listed are left untouched
 * (active[] still applies to the listed ones).  All steps of the group share N,
 * and all of them or none have parent, likewise x_row. */
qrnnt_status qrnnt_lstm_step_group_listed(const qrnnt_step_desc *steps, int32_t n_steps, const int32_t *list,
                                          const int32_t *n_list, void *stream);

/* ---- LSTM: one layer-direction over whole utterances (Sec. 2 encoder, Sec. 3.4) ---- */

size_t qrnnt_lstm_layer_workspace(const qrnnt_lstm *L, int32_t T, int32_t B);

/* x_codes [device] [T,B,I] int8 (row pitch qrnnt_act_pitch(I)).  The input projection of all T*B frames is
 * one integer GEMM; the recurrence then runs t = 0..T-1 (T-1..0 if reverse).
 * Output codes go to h_out[(t*B + b)*ld_out + col_off + j], so the two
 * directions of a bidirectional layer fill the two halves of [T,B,2H] (both
 * use the FIX +-1 grid, Sec. 3.2).  h0/c0 [device] [B,H] or NULL (zero state,
 * as Sec. 3.4 assumes).  h_last/c_last [device] [B,H] or NULL.  Debug
 * [device] or NULL: dbg_accx int32 [T,B,4H] (source row order), dbg_c_all fp32
 * [T,B,H].  All utterances have length T.
 * The recurrence runs as one persistent kernel (H/16 x ceil(B/16) workgroups per
 * direction, exchanging hidden codes through the workspace) when H <= 1024 and all
 * of those workgroups fit on the device at once (as reported by the runtime's
 * occupancy query for an otherwise idle device); otherwise as one fused launch per
 * time step (4-bit layers only: an 8-bit layer that cannot take the persistent path
 * returns QRNNT_ERR_UNSUPPORTED).  The persistent kernel's waits are bounded: if one
 * ever runs out (e.g. other work keeps part of the device busy), the int32 at
 * workspace + qrnnt_lstm_layer_workspace(L, T, B) - 256 is set to 1 and the outputs
 * are invalid; it is 0 after every other call. */
qrnnt_status qrnnt_lstm_layer(const qrnnt_lstm *L, const int8_t *x_codes, int32_t T, int32_t B, int32_t reverse,
                              const int8_t *h0, const float *c0, int8_t *h_out, int32_t ld_out, int32_t col_off,
                              int8_t *h_last, float *c_last, int32_t *dbg_accx, float *dbg_c_all,
                              void *workspace, size_t workspace_bytes, void *stream);

/* qrnnt_lstm_layer for callers that cannot allocate device memory or supply a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results and error flag semantics as qrnnt_lstm_layer
 * without the debug outputs; the workspace is a device array inside the library of
 * QRNNT_STATIC_WORKSPACE_BYTES bytes (held by every GPU the library runs on until the
 * process ends).  Returns QRNNT_ERR_WORKSPACE when qrnnt_lstm_layer_workspace(L, T, B)
 * exceeds that size (roughly T*B*16*H + 10*B*H bytes: e.g. one utterance of 3000
 * frames at H = 640).  The call allocates nothing.  All calls on one GPU share the
 * array: calls that may overlap on one GPU (different streams, different threads)
 * race; calls on one stream are ordered.  The bounded-wait flag of the persistent
 * recurrence is not visible to the caller here. */
#define QRNNT_STATIC_WORKSPACE_BYTES (32u << 20)
qrnnt_status qrnnt_lstm_layer_static(const qrnnt_lstm *L, const int8_t *x_codes, int32_t T, int32_t B, int32_t reverse,
                                     const int8_t *h0, const float *c0, int8_t *h_out, int32_t ld_out, int32_t col_off,
                                     int8_t *h_last, float *c_last, void *stream);

/* Both directions of a bidirectional layer in one call (zero initial state):
 * forward codes go to columns [0,H) and backward codes to [H,2H) of h_out [device]
 * [T,B,2H].  The two recurrences advance concurrently in one launch.  workspace
 * [device]: qrnnt_bilstm_layer_workspace bytes, 256-byte aligned; it holds the
 * forward direction's workspace followed by the backward direction's, so there are
 * two bounded-wait flags: the int32 at workspace + qrnnt_lstm_layer_workspace(fwd, T, B)
 * - 256 and the int32 at workspace + qrnnt_bilstm_layer_workspace(...) - 256. */
size_t qrnnt_bilstm_layer_workspace(const qrnnt_lstm *fwd, const qrnnt_lstm *bwd, int32_t T, int32_t B);
qrnnt_status qrnnt_bilstm_layer(const qrnnt_lstm *fwd, const qrnnt_lstm *bwd, const int8_t *x_codes, int32_t T,
                                int32_t B, int8_t *h_out, void *workspace, size_t workspace_bytes, void *stream);

/* The input projection alone (first half of qrnnt_lstm_layer): for M rows of
 * input codes x [device] [M, I], gx[m, r'] = sum_k w_ih[g*H + j, k] * x[m, k]
 * as int32 [M, 4H], where r' is the TILED_GATES row of (cell j, gate g) (see the
 * layout note above: the four gate sums of a cell are adjacent), which is the
 * order the recurrence and qrnnt_step_desc.gx consume.  dbg_accx [device] int32
 * [M, 4H] in source row order, or NULL.  hidden_size % 16 == 0. */
qrnnt_status qrnnt_input_projection(const qrnnt_lstm *L, const int8_t *x_codes, int32_t M, int32_t *gx,
                                    int32_t *dbg_accx, void *stream);

/* fp32 form of M rows of an input projection gx (as written by
 * qrnnt_input_projection): table[m, r'] = k * (x_scale * row_scale[r] * gx[m, r']
 * + bias[r]) for the TILED_GATES position r' of row r, with k = -log2(e) for the
 * sigmoid gates and -2 log2(e) for the tanh gate (the constants the cell feeds to
 * exp2).  Consumed through qrnnt_step_desc.gx_table.  table [device] fp32
 * [M, 4H], 16-byte aligned. */
qrnnt_status qrnnt_input_table(const qrnnt_lstm *L, const int32_t *gx, int32_t M, float *table, void *stream);

/* ---- joint network + log-softmax + Eq. 1 ---- */

/* For n in [0,N): e = enc_proj[frame_row[n]], p = pred_proj[n] (length J);
 *   z = tanh(e .* p); zq = Q(z; z_inv_scale);
 *   logit[k] = z_scale*row_scale[k]*sum_j w_out[k,j]*zq[j] + b_out[k];
 *   lp = log_softmax(logit);
 *   fused[n,blank] = lp[blank];
 *   fused[n,k] = lp[k] - lambda_src*lp_src[n,k] + lambda_ext*lp_ext[n,k] + rho  (k != blank).
 * The quantizer of z has the width of w_out (Sec. 3.2: a linear layer's weights
 * and inputs share one precision): codes in [-8,7], or [-128,127] when
 * w_out->bits == 8 (then z_inv_scale is 127/alpha).
 * w_out: TILED layout, rows = V <= 64, cols = J (multiple of 64).  lp_src /
 * lp_ext [device] [N,V] or NULL (term dropped).  Optional outputs [device]:
 * lp_rnnt_out fp32 [N,V], dbg_zq int8 [N,J].  frame_row values are clamped to
 * [0, n_enc_rows). */
qrnnt_status qrnnt_joint_fuse(const float *enc_proj, int32_t n_enc_rows, const int32_t *frame_row,
                              const float *pred_proj, const qrnnt_qmat *w_out, const float *b_out,
                              float z_scale, float z_inv_scale, const float *lp_src, const float *lp_ext,
                              float lambda_src, float lambda_ext, float rho, int32_t N, int32_t blank,
                              float *lp_rnnt_out, int8_t *dbg_zq, float *fused_out, void *stream);

/* ---- beam selection (Sec. 2: up to W hypotheses kept per iteration) ---- */

/* Per utterance b: candidates (w,k) valued score[b,w] + fused[b*W+w,k] (fp32);
 * the W best by (value descending, w*V+k ascending) are written best first to
 * parent_out/token_out/score_out [B,W]; -inf candidates are never taken and
 * unfilled ranks get parent = token = -1, score = -inf.  force_blank != 0
 * restricts the candidates to k == blank.  W <= 64. */
qrnnt_status qrnnt_beam_step(const float *score, const float *fused, int32_t B, int32_t W, int32_t V,
                             int32_t blank, int32_t force_blank, int32_t *parent_out, int32_t *token_out,
                             float *score_out, void *stream);

/* ---- the whole decoding loop on the device (Sec. 2; Eq. 1) ---- */

#define QRNNT_MAX_LAYERS 4

/* Embedding -> quantizer -> stacked LSTM steps -> quantized linear layer: the
 * prediction network (log_softmax = 0, output = the joint's prediction input)
 * or a language model (log_softmax = 1, output = log-probabilities).
 * Optional bottleneck (Sec. 2, the external LM: LSTM stack -> bottleneck ->
 * output layer), present when mid.packed != NULL: the top hidden codes go
 * through mid (qrnnt_linear_quant with a_scale = out_a_scale, quantizer
 * mid_inv_scale at the width of `out`; no activation function, the paper names
 * none) and `out` then reads those codes with step mid_scale. */
typedef struct {
    const int8_t *embed_codes;  /* [device] [V, E] embedding rows already quantized (FIX boundary, Sec. 3.2), row pitch qrnnt_act_pitch(E) */
    int32_t n_layers;           /* 1..QRNNT_MAX_LAYERS; layer[0].input_size = E */
    qrnnt_lstm layer[QRNNT_MAX_LAYERS];
    qrnnt_qmat out;             /* TILED, [out_rows, H_top] ([out_rows, M] behind a bottleneck) */
    const float *out_bias;      /* [device] [out_rows] or NULL */
    float out_a_scale;          /* step of the top layer's hidden codes */
    int32_t log_softmax;
    qrnnt_qmat mid;             /* TILED, [M, H_top], M % 16 == 0; packed == NULL: no bottleneck */
    const float *mid_bias;      /* [device] [M] or NULL */
    float mid_scale, mid_inv_scale; /* alpha/7 and 7/alpha of the quantizer on the bottleneck's output */
} qrnnt_net;

typedef struct {
    qrnnt_net pred, lm_src, lm_ext;
    int32_t use_src, use_ext;   /* 0 drops the LM and its term of Eq. 1 */
    qrnnt_qmat joint_out;       /* TILED, [V, J] */
    const float *joint_bias;    /* [device] [V] or NULL */
    float z_scale, z_inv_scale; /* quantizer of the joint activation */
    float lambda_src, lambda_ext, rho;
    int32_t V, blank;           /* blank doubles as the start symbol fed to all networks */
} qrnnt_model;

size_t qrnnt_decode_workspace(const qrnnt_model *m, int32_t T, int32_t B, int32_t W, int32_t max_sym);

/* Time-synchronous beam search over enc_proj [device] [T,B,J] fp32, every
 * utterance of length T, W hypotheses per utterance, at most max_sym labels per
 * frame.  Per utterance: the beam starts as the empty sequence (score 0, all
 * networks advanced once on the start symbol from the zero state).  Per frame:
 * A <- beam; for round v = 0..max_sym: fused scores of A at this frame
 * (qrnnt_joint_fuse), the W best extensions (qrnnt_beam_step, blank only when
 * v == max_sym); blank picks join the frame's candidate list with their new
 * score, label picks form the next A with all networks advanced from the
 * parent's state (qrnnt_lstm_step with parent gather); after the last round the
 * beam becomes the W best candidates by (score descending, insertion order).
 * Equal label sequences are not merged.  All rounds always run (dead slots carry
 * score -inf), so the launch sequence does not depend on the data and nothing
 * is copied to the host.
 * Outputs [device], best first: tokens_out int32 [B,W,max_len] (padded with
 * -1), len_out int32 [B,W] (-1 for an empty rank), score_out fp32 [B,W].
 * workspace [device]: qrnnt_decode_workspace bytes, 256-byte aligned. */
qrnnt_status qrnnt_decode(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                          int32_t max_sym, int32_t max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/* qrnnt_decode with options.  flags: QRNNT_DECODE_EARLY_STOP makes every kernel
 * of a round start by reading a device-side count of the utterances that carried
 * a label into that round and return at once when it is zero (then no later round
 * of the frame can pick anything either): same results, a few loads more per
 * kernel, and the cost of a frame follows the labels it actually emits.  The host
 * still enqueues the same launch sequence.  flags == 0 is qrnnt_decode. */
#define QRNNT_DECODE_EARLY_STOP 1u
qrnnt_status qrnnt_decode_ex(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                             int32_t max_sym, int32_t max_len, uint32_t flags, int32_t *tokens_out, int32_t *len_out,
                             float *score_out, void *workspace, size_t workspace_bytes, void *stream);

/* Alignment-length synchronous beam search with recombination (Sec. 2: the
 * search the paper decodes with, beam width 1 to 16) over enc_proj [device]
 * [T,B,J] fp32.  All hypotheses of a beam have taken the same number i of
 * alignment steps (labels + blanks): one with u labels stands at frame i - u.
 * Per utterance the beam has W slots and starts as the empty sequence in slot 0.
 * For i = 0 .. T + u_max - 1: fused scores of every hypothesis at its own frame
 * (qrnnt_joint_fuse); candidates (w,k) = score_w + fused[w,k], except labels of
 * a hypothesis that already holds u_max labels; a blank at the last frame
 * finishes the hypothesis (it joins the finished list with that value and is no
 * candidate); the W best candidates in qrnnt_beam_step's order become the next
 * slots in rank order (blank: same sequence and network state, one frame later;
 * label: extended, all networks advanced); picks that stand for the same label
 * sequence are merged into the best-ranked of them with score
 * log(sum exp(scores)), the other slots stay empty; the finished list keeps its
 * W best by (score descending, insertion order; newcomers in slot order).
 * Label sequences are compared through their length and a 64-bit hash.
 * Outputs [device] as for qrnnt_decode, from the finished list (empty ranks:
 * len -1, score -inf).  The launch sequence is fixed (T + u_max iterations);
 * once no hypothesis is alive anywhere the remaining kernels return at once.
 * workspace [device]: qrnnt_decode_alsd_workspace bytes, 256-byte aligned. */
size_t qrnnt_decode_alsd_workspace(const qrnnt_model *m, int32_t T, int32_t B, int32_t W, int32_t u_max);
qrnnt_status qrnnt_decode_alsd(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                               int32_t u_max, int32_t max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                               void *workspace, size_t workspace_bytes, void *stream);

/* qrnnt_decode_alsd with options.  QRNNT_ALSD_REUSE: reuse of cached hypotheses (Sec. 4.1 names it as what
 * makes the decoding time fall sub-linearly at small beams).  The states of the prediction network and of the
 * LMs after a label sequence depend on that sequence alone; with this flag a label pick whose resulting
 * sequence a live hypothesis of the current beam already holds takes over that hypothesis' states (the slot
 * becomes an inactive row of the network advance, copied from that hypothesis) instead of advancing the
 * networks from its own parent.  Results are bit for bit those of qrnnt_decode_alsd; sequences are compared
 * by (length, 64-bit hash) as in the recombination.  The cache is the current beam: a sequence that left the
 * beam is not remembered.  stats [device] int32[2] or NULL: the call adds the number of label picks that kept
 * their slot to stats[0] and the number of those that reused states to stats[1] (the caller zeroes it). */
#define QRNNT_ALSD_REUSE 1u
qrnnt_status qrnnt_decode_alsd_ex(const qrnnt_model *m, const float *enc_proj, int32_t T, int32_t B, int32_t W,
                                  int32_t u_max, int32_t max_len, uint32_t flags, int32_t *stats, int32_t *tokens_out,
                                  int32_t *len_out, float *score_out, void *workspace, size_t workspace_bytes,
                                  void *stream);

/* ---- diagnostics ---- */

/* Register-only issue rate of one of the matrix instructions that can carry the 4-bit x 4-bit contraction
 * exactly or nearly so (codes in [-8, 7] are exact in int8, fp8-E4M3 and fp6-E3M2, [-7, 7] in fp6-E2M3; fp4-E2M1
 * is listed for its rate only; partial sums stay below 2^24; Sec. 3.1 fixes the integer grid only).
 * form in [0, qrnnt_diag_mfma_forms()); qrnnt_diag_mfma_form_name gives its name.
 * Runs `iters` loop iterations on two workgroups per compute unit (two instructions on each of 8 accumulator
 * chains per wave, 4 chains for the 32-row forms; registers only), or, for the forms named "chunk loop ...", on
 * three workgroups per compute unit a loop shaped like the contraction kernels' 128-column chunk without its
 * global loads (barrier, LDS operand reads of a wave's 64 x 64 tile, nibble unpack, matrix instructions), and
 * writes the rate in TOP/s (2 ops per multiply-accumulate) to *tops_out [host].  sink [device]: one float the
 * kernel may write.  Unlike every other call this one waits for its own work (it times it with events). */
int32_t qrnnt_diag_mfma_forms(void);
const char *qrnnt_diag_mfma_form_name(int32_t form);
qrnnt_status qrnnt_diag_mfma_rate(int32_t form, int32_t iters, float *sink, double *tops_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QRNNT_H */
