/*
 * qrnnt_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-pass CPU statement of what the INT4 RNN-T hot path
 * computes (arXiv 2206.07882: Sec. 3.1 quantizers, Sec. 3.2 placement of the
 * quantizers, Sec. 3.4 "Outer" quantization, Sec. 2 network and Eq. 1 fusion).
 * It exists so that the GPU library can be checked against something that was
 * written from the paper and not from the GPU code.  Nothing in the product
 * path may call it; it shares no source, header, table or helper with the HIP
 * library.
 *
 * Arithmetic conventions (each is a reading of the paper, which prints no
 * bit-level definition):
 *   - symmetric b=4 grid: signed codes in [-8,7], step s = alpha/7 (Sec. 3.1,
 *     symmetric LQ has one boundary alpha and no zero point); the 8-bit layers
 *     of Sec. 3.2 use the same grid with 127 steps per side, and a layer's own
 *     quantizer (hidden state; z for the joint's output layer) has the width
 *     of the layer's weights (`bits` of oq_lstm_t / oq_linear_t);
 *   - the rounding operator of Eq. 2 is round-half-to-even;
 *   - a value is quantized as clamp(rne(x * inv_s)) with the product taken in
 *     fp32, because that product decides an integer and the GPU path takes the
 *     same decision in fp32;
 *   - every other floating-point quantity (gate pre-activations, sigmoid,
 *     tanh, log-softmax, Eq. 1) is evaluated in fp64 and rounded to fp32 only
 *     where the method stores fp32 (cell state, projections, scores);
 *   - LSTM: gate rows ordered i,f,g,o; one fp32 bias per gate row; weights and
 *     activations integer, bias and cell state not quantized (Sec. 3.2).
 *
 * Parity status of each function is stated next to it: "pinned by" names the
 * independent check in tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define OQ_MAX_LAYERS 4

/* Counters of activation-quantizer invocations (one per tensor handed to the
 * quantizer), for the Outer-vs-Inner call-count check of Sec. 3.4. */
static long g_quant_tensor_calls = 0;
long oq_quant_calls_get(void) { return g_quant_tensor_calls; }
void oq_quant_calls_reset(void) { g_quant_tensor_calls = 0; }

/* ------------------------------------------------------------------ */
/* Sec. 3.1: linear quantizers                                         */
/* ------------------------------------------------------------------ */

/* Symmetric 4-bit code of one value.  Pinned by: clip range, Q(deq(q))=q on
 * all 16 codes, Q(0)=0, residual <= s/2 in range, monotonicity. */
int8_t oq_quant_sym4(float x, float inv_s)
{
    float t = x * inv_s;
    float r = nearbyintf(t); /* default rounding mode: ties to even */
    if (r < -8.0f) r = -8.0f;
    if (r > 7.0f) r = 7.0f;
    return (int8_t)r;
}

void oq_quantize_sym4(const float *x, int64_t n, float inv_s, int8_t *q)
{
    g_quant_tensor_calls += 1;
    for (int64_t i = 0; i < n; ++i) q[i] = oq_quant_sym4(x[i], inv_s);
}

/* The same symmetric quantizer at b bits (Sec. 3.2 keeps the first encoder layer
 * and the linear layers of the RNN-T at 8 bits): codes in [-2^(b-1), 2^(b-1)-1],
 * step alpha/(2^(b-1)-1).  bits == 0 means 4.  Pinned by: equals oq_quant_sym4 at
 * b = 4, clip range and grid identity on all 256 codes at b = 8, hand values. */
int8_t oq_quant_sym(float x, float inv_s, int bits)
{
    if (bits == 0) bits = 4;
    float lo = -(float)(1 << (bits - 1)), hi = (float)((1 << (bits - 1)) - 1);
    float t = x * inv_s;
    float r = nearbyintf(t);
    if (r < lo) r = lo;
    if (r > hi) r = hi;
    return (int8_t)r;
}

void oq_quantize_sym(const float *x, int64_t n, float inv_s, int bits, int8_t *q)
{
    g_quant_tensor_calls += 1;
    for (int64_t i = 0; i < n; ++i) q[i] = oq_quant_sym(x[i], inv_s, bits);
}

/* Bookkeeping for free-running comparisons (no part of the method): how close
 * the quantizer's decision on x came to a rounding tie.  A value computed in
 * fp32 by another implementation differs from this file's fp64 value by a few
 * units in the last place; when x * inv_s lies that close to k + 1/2 the two
 * round to different codes, both within the accuracy the method has.  Returned
 * in units of 4-bit code steps (the distance on the 8-bit grid times 7/127, so
 * that one bound serves both widths); +inf where the clamp decides the code
 * (no rounding involved).  Pinned by: hand values. */
double oq_tie_distance(float x, float inv_s, int bits)
{
    if (bits == 0) bits = 4;
    const double qmax = (double)((1 << (bits - 1)) - 1);
    const double t = (double)(x * inv_s);           /* the fp32 product that is rounded */
    if (t <= -qmax - 1.5 || t >= qmax + 0.5) return INFINITY;
    const double frac = t - floor(t);
    return fabs(frac - 0.5) * (7.0 / qmax);
}

/* Asymmetric LQ, Eq. 2 and Eq. 3, for b bits and boundaries alpha_-/alpha_+.
 * Not on the integer path (weights are symmetric and every activation range
 * used is +-alpha); carried as a utility.  Pinned by: alpha_- maps to 0,
 * alpha_+ to 2^b-1, residual <= s/2 inside the range. */
void oq_quantize_asym(const float *x, int64_t n, int bits, double a_lo, double a_hi,
                      int32_t *x_int, double *x_q)
{
    double levels = (double)((1 << bits) - 1);
    double s = (a_hi - a_lo) / levels;
    double z = -a_lo / s;
    for (int64_t i = 0; i < n; ++i) {
        double v = nearbyint((double)x[i] / s) + z;
        if (v < 0.0) v = 0.0;
        if (v > levels) v = levels;
        if (x_int) x_int[i] = (int32_t)nearbyint(v);
        if (x_q) x_q[i] = s * (v - z);
    }
}

/* MAX range picker applied per output row, then the symmetric quantizer
 * (Sec. 3.1 MAX; per-row granularity is the measured configuration's choice).
 * scale[r] = alpha_r/7 and the code uses inv = 7/alpha_r, both fp32 divisions.
 * An all-zero row gets scale 1 and codes 0.  Pinned by: |code| reaches 7 on
 * the max-abs element, codes on a hand-made row. */
void oq_quantize_weight_rows(const float *w, int rows, int cols, int8_t *codes, float *scale)
{
    for (int r = 0; r < rows; ++r) {
        const float *wr = w + (int64_t)r * cols;
        float alpha = 0.0f;
        for (int k = 0; k < cols; ++k) {
            float a = fabsf(wr[k]);
            if (a > alpha) alpha = a;
        }
        if (alpha == 0.0f) {
            scale[r] = 1.0f;
            for (int k = 0; k < cols; ++k) codes[(int64_t)r * cols + k] = 0;
            continue;
        }
        float s = alpha / 7.0f;
        float inv = 7.0f / alpha;
        scale[r] = s;
        for (int k = 0; k < cols; ++k) codes[(int64_t)r * cols + k] = oq_quant_sym4(wr[k], inv);
    }
}

/* The same at b bits: scale[r] = alpha_r/qmax, inv = qmax/alpha_r with
 * qmax = 2^(b-1)-1 (the 8-bit MAX quantizer of Sec. 3.2).  Pinned by: |code|
 * reaches qmax on the max-abs element, equals the 4-bit routine at b = 4,
 * dequantization error <= scale/2. */
void oq_quantize_weight_rows_bits(const float *w, int rows, int cols, int bits, int8_t *codes, float *scale)
{
    if (bits == 0) bits = 4;
    const float qmax = (float)((1 << (bits - 1)) - 1);
    for (int r = 0; r < rows; ++r) {
        const float *wr = w + (int64_t)r * cols;
        float alpha = 0.0f;
        for (int k = 0; k < cols; ++k) {
            float a = fabsf(wr[k]);
            if (a > alpha) alpha = a;
        }
        if (alpha == 0.0f) {
            scale[r] = 1.0f;
            for (int k = 0; k < cols; ++k) codes[(int64_t)r * cols + k] = 0;
            continue;
        }
        float inv = qmax / alpha;
        scale[r] = alpha / qmax;
        for (int k = 0; k < cols; ++k) codes[(int64_t)r * cols + k] = oq_quant_sym(wr[k], inv, bits);
    }
}

/* Canonical nibble packing: byte j of row r holds element (r,2j) in bits 0-3
 * and (r,2j+1) in bits 4-7, two's complement; columns >= cols up to
 * cols_padded are zero.  Pinned by: hand-written bytes, unpack(pack)=id over
 * all 256 byte values. */
void oq_pack_rows(const int8_t *codes, int rows, int cols, int cols_padded, uint8_t *packed)
{
    int bpr = cols_padded / 2;
    for (int r = 0; r < rows; ++r)
        for (int j = 0; j < bpr; ++j) {
            int k0 = 2 * j, k1 = 2 * j + 1;
            int lo = k0 < cols ? codes[(int64_t)r * cols + k0] : 0;
            int hi = k1 < cols ? codes[(int64_t)r * cols + k1] : 0;
            packed[(int64_t)r * bpr + j] = (uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));
        }
}

void oq_unpack_rows(const uint8_t *packed, int rows, int cols, int cols_padded, int8_t *codes)
{
    int bpr = cols_padded / 2;
    for (int r = 0; r < rows; ++r)
        for (int k = 0; k < cols; ++k) {
            uint8_t byte = packed[(int64_t)r * bpr + k / 2];
            int nib = (k & 1) ? (byte >> 4) : (byte & 0xF);
            codes[(int64_t)r * cols + k] = (int8_t)(nib >= 8 ? nib - 16 : nib);
        }
}

/* ------------------------------------------------------------------ */
/* Integer contraction (the MAC of Sec. 3.1/3.2)                        */
/* ------------------------------------------------------------------ */

/* acc[n,r] = sum_k w[r,k]*a[n,k], int32.  Pinned by: Python triple loop on
 * tiny shapes, extreme-code closed forms, permutation of k. */
void oq_matmul_i32(const int8_t *w, int rows, int K, const int8_t *a, int N, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const int8_t *an = a + (int64_t)n * K;
        for (int r = 0; r < rows; ++r) {
            const int8_t *wr = w + (int64_t)r * K;
            int32_t s = 0;
            for (int k = 0; k < K; ++k) s += (int32_t)wr[k] * (int32_t)an[k];
            acc[(int64_t)n * rows + r] = s;
        }
    }
}

/* ------------------------------------------------------------------ */
/* Quantized LSTM cell (Sec. 3.2, Sec. 3.4)                             */
/* ------------------------------------------------------------------ */

typedef struct {
    const int8_t *w_ih;   /* [4H, I] codes, gate rows i,f,g,o */
    const int8_t *w_hh;   /* [4H, H] codes */
    const float *s_wih;   /* [4H] row scales */
    const float *s_whh;   /* [4H] */
    const float *bias;    /* [4H] fp32, not quantized */
    int32_t I, H;
    float s_x;            /* step of the input codes  */
    float s_h;            /* step of the hidden codes (FIX +-1: 1/7) */
    float inv_s_h;        /* 7/alpha_h (FIX +-1: 7); 127/alpha_h for an 8-bit layer */
    int32_t bits;         /* width of the layer (weights and hidden-state quantizer, Sec. 3.2): 0 or 4, or 8 */
} oq_lstm_t;

static double sigm(double v) { return 1.0 / (1.0 + exp(-v)); }

/* One time step for N rows.  Row n reads its previous state from slot
 * parent[n] (n itself when parent is NULL).  Rows with active[n]==0 copy the
 * parent's state through unchanged.  The hidden state leaves the cell as a
 * 4-bit code (one quantizer call per cell output: Outer quantization,
 * Sec. 3.4); that code is what the next step and the next layer consume.
 * Optional outputs: accx/acch int32 [N,4H], gates fp64 [N,4H] (activated
 * i,f,g,o), h_real fp64 [N,H] (h before the quantizer).
 * Pinned by: zero-weight closed form, |code|<=7, hand-rolled numpy cell on
 * random small inputs, pass-through of inactive rows. */
static void lstm_step_core(const oq_lstm_t *L, const int8_t *x, const int32_t *parent,
                  const int8_t *h_prev, const float *c_prev, const uint8_t *active, int N,
                  int8_t *h_next, float *c_next,
                  int32_t *accx_out, int32_t *acch_out, double *gates_out, double *h_real_out,
                  double *row_margin /* [N] or NULL: smallest oq_tie_distance among the row's H decisions */)
{
    const int H = L->H, I = L->I, R = 4 * L->H;
    g_quant_tensor_calls += 1; /* the one quantizer at the cell output */
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        int src = parent ? parent[n] : n;
        const int8_t *hp = h_prev + (int64_t)src * H;
        const float *cp = c_prev + (int64_t)src * H;
        if (row_margin) row_margin[n] = INFINITY;
        if (active && !active[n]) {
            memcpy(h_next + (int64_t)n * H, hp, (size_t)H);
            memcpy(c_next + (int64_t)n * H, cp, (size_t)H * sizeof(float));
            continue;
        }
        const int8_t *xn = x + (int64_t)n * I;
        double *pre = (double *)malloc(sizeof(double) * (size_t)R);
        for (int r = 0; r < R; ++r) {
            int32_t ax = 0, ah = 0;
            const int8_t *wi = L->w_ih + (int64_t)r * I;
            const int8_t *wh = L->w_hh + (int64_t)r * H;
            for (int k = 0; k < I; ++k) ax += (int32_t)wi[k] * (int32_t)xn[k];
            for (int k = 0; k < H; ++k) ah += (int32_t)wh[k] * (int32_t)hp[k];
            if (accx_out) accx_out[(int64_t)n * R + r] = ax;
            if (acch_out) acch_out[(int64_t)n * R + r] = ah;
            pre[r] = (double)L->s_x * (double)L->s_wih[r] * (double)ax +
                     (double)L->s_h * (double)L->s_whh[r] * (double)ah + (double)L->bias[r];
        }
        for (int j = 0; j < H; ++j) {
            double gi = sigm(pre[j]);
            double gf = sigm(pre[H + j]);
            double gg = tanh(pre[2 * H + j]);
            double go = sigm(pre[3 * H + j]);
            double c = gf * (double)cp[j] + gi * gg;
            double h = go * tanh(c);
            c_next[(int64_t)n * H + j] = (float)c;
            h_next[(int64_t)n * H + j] = oq_quant_sym((float)h, L->inv_s_h, L->bits);
            if (row_margin) {
                const double d = oq_tie_distance((float)h, L->inv_s_h, L->bits);
                if (d < row_margin[n]) row_margin[n] = d;
            }
            if (gates_out) {
                double *g = gates_out + (int64_t)n * R;
                g[j] = gi; g[H + j] = gf; g[2 * H + j] = gg; g[3 * H + j] = go;
            }
            if (h_real_out) h_real_out[(int64_t)n * H + j] = h;
        }
        free(pre);
    }
}

void oq_lstm_step(const oq_lstm_t *L, const int8_t *x, const int32_t *parent,
                  const int8_t *h_prev, const float *c_prev, const uint8_t *active, int N,
                  int8_t *h_next, float *c_next,
                  int32_t *accx_out, int32_t *acch_out, double *gates_out, double *h_real_out)
{
    lstm_step_core(L, x, parent, h_prev, c_prev, active, N, h_next, c_next, accx_out, acch_out, gates_out, h_real_out, NULL);
}

/* One layer-direction over a whole batch of equal-length utterances.
 * x [T,B,I] codes; output codes written to h_out[t,b,col_off + j] with row
 * pitch ld_out, so that a bidirectional layer is two calls that fill the two
 * halves of [T,B,2H] (both directions share the FIX +-1 step, Sec. 3.2).
 * reverse!=0 walks t = T-1..0.  h0/c0 NULL mean zero (Sec. 3.4 assumes a zero
 * state before the first step).  c_all (optional) receives c_t for every t.
 * Pinned by: reverse == time-flip of forward on flipped input; T=1 == step. */
static void lstm_layer_core(const oq_lstm_t *L, const int8_t *x, int T, int B, int reverse,
                   const int8_t *h0, const float *c0,
                   int8_t *h_out, int ld_out, int col_off,
                   int8_t *h_last, float *c_last, float *c_all,
                   double *utt_margin /* [B] or NULL: lowered to the smallest oq_tie_distance of utterance b's cells */)
{
    const int H = L->H, I = L->I;
    double *rm = utt_margin ? (double *)malloc(sizeof(double) * (size_t)B) : NULL;
    int8_t *h = (int8_t *)calloc((size_t)B * H, 1), *hn = (int8_t *)calloc((size_t)B * H, 1);
    float *c = (float *)calloc((size_t)B * H, sizeof(float)), *cn = (float *)calloc((size_t)B * H, sizeof(float));
    if (h0) memcpy(h, h0, (size_t)B * H);
    if (c0) memcpy(c, c0, (size_t)B * H * sizeof(float));
    for (int s = 0; s < T; ++s) {
        int t = reverse ? T - 1 - s : s;
        lstm_step_core(L, x + (int64_t)t * B * I, NULL, h, c, NULL, B, hn, cn, NULL, NULL, NULL, NULL, rm);
        for (int b = 0; b < B; ++b) {
            memcpy(h_out + ((int64_t)t * B + b) * ld_out + col_off, hn + (int64_t)b * H, (size_t)H);
            if (rm && rm[b] < utt_margin[b]) utt_margin[b] = rm[b];
        }
        if (c_all) memcpy(c_all + (int64_t)t * B * H, cn, (size_t)B * H * sizeof(float));
        int8_t *th = h; h = hn; hn = th;
        float *tc = c; c = cn; cn = tc;
    }
    if (h_last) memcpy(h_last, h, (size_t)B * H);
    if (c_last) memcpy(c_last, c, (size_t)B * H * sizeof(float));
    free(h); free(hn); free(c); free(cn); free(rm);
}

void oq_lstm_layer(const oq_lstm_t *L, const int8_t *x, int T, int B, int reverse,
                   const int8_t *h0, const float *c0,
                   int8_t *h_out, int ld_out, int col_off,
                   int8_t *h_last, float *c_last, float *c_all)
{
    lstm_layer_core(L, x, T, B, reverse, h0, c0, h_out, ld_out, col_off, h_last, c_last, c_all, NULL);
}

/* The same, also lowering utt_margin[b] (caller-initialised, e.g. to +inf) to the smallest
 * oq_tie_distance met by any hidden-state quantizer of utterance b. */
void oq_lstm_layer_margin(const oq_lstm_t *L, const int8_t *x, int T, int B, int reverse,
                          const int8_t *h0, const float *c0,
                          int8_t *h_out, int ld_out, int col_off,
                          int8_t *h_last, float *c_last, float *c_all, double *utt_margin)
{
    lstm_layer_core(L, x, T, B, reverse, h0, c0, h_out, ld_out, col_off, h_last, c_last, c_all, utt_margin);
}

/* ------------------------------------------------------------------ */
/* Quantized linear layer, log-softmax, joint, fusion (Sec. 2, Eq. 1)   */
/* ------------------------------------------------------------------ */

typedef struct {
    const int8_t *w;      /* [rows, cols] codes */
    const float *s_w;     /* [rows] */
    const float *bias;    /* [rows] or NULL */
    int32_t rows, cols;
    float s_a;            /* step of the input codes */
    int32_t bits;         /* width of the layer (weights and its own input quantizer, Sec. 3.2): 0 or 4, or 8 */
} oq_linear_t;

/* y[n,r] = s_a*s_w[r]*acc[n,r] + b[r], fp64, stored fp32.
 * Pinned by: dequantize-then-float-matmul in numpy. */
void oq_linear(const oq_linear_t *P, const int8_t *a, int N, float *y, int32_t *acc_out)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int r = 0; r < P->rows; ++r) {
            int32_t s = 0;
            const int8_t *wr = P->w + (int64_t)r * P->cols, *an = a + (int64_t)n * P->cols;
            for (int k = 0; k < P->cols; ++k) s += (int32_t)wr[k] * (int32_t)an[k];
            if (acc_out) acc_out[(int64_t)n * P->rows + r] = s;
            double v = (double)P->s_a * (double)P->s_w[r] * (double)s + (P->bias ? (double)P->bias[r] : 0.0);
            y[(int64_t)n * P->rows + r] = (float)v;
        }
}

/* lp = x - max - log sum exp(x - max) over V entries, fp64.
 * Pinned by: sum exp(lp) = 1, shift invariance, uniform input -> -log V. */
static void log_softmax_d(const double *x, int V, double *lp)
{
    double m = x[0];
    for (int k = 1; k < V; ++k) if (x[k] > m) m = x[k];
    double s = 0.0;
    for (int k = 0; k < V; ++k) s += exp(x[k] - m);
    double ls = log(s);
    for (int k = 0; k < V; ++k) lp[k] = x[k] - m - ls;
}

void oq_log_softmax(const float *x, int N, int V, float *lp)
{
    double *xd = (double *)malloc(sizeof(double) * 2 * (size_t)V);
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < V; ++k) xd[k] = x[(int64_t)n * V + k];
        log_softmax_d(xd, V, xd + V);
        for (int k = 0; k < V; ++k) lp[(int64_t)n * V + k] = (float)xd[V + k];
    }
    free(xd);
}

/* Joint, first half: z = tanh(e .* p) (multiplicative combination, Sec. 2;
 * the tanh is the measured configuration's), then the 4-bit code of z since z
 * is the input of a quantized linear layer (Sec. 3.2).  Row n uses encoder row
 * frame_row[n].  Pinned by: numpy restatement, |code| <= 7. */
static void joint_z_core(const float *enc_proj, const int32_t *frame_row, const float *pred_proj,
                         int N, int J, float inv_s_z, int bits, int8_t *zq, double *z_real,
                         double *row_margin /* [N] or NULL: smallest oq_tie_distance among the row's J decisions */)
{
    for (int n = 0; n < N; ++n) {
        const float *e = enc_proj + (int64_t)frame_row[n] * J, *p = pred_proj + (int64_t)n * J;
        if (row_margin) row_margin[n] = INFINITY;
        for (int j = 0; j < J; ++j) {
            double z = tanh((double)e[j] * (double)p[j]);
            if (z_real) z_real[(int64_t)n * J + j] = z;
            zq[(int64_t)n * J + j] = oq_quant_sym((float)z, inv_s_z, bits);
            if (row_margin) {
                const double d = oq_tie_distance((float)z, inv_s_z, bits);
                if (d < row_margin[n]) row_margin[n] = d;
            }
        }
    }
}

void oq_joint_z(const float *enc_proj, const int32_t *frame_row, const float *pred_proj,
                int N, int J, float inv_s_z, int bits, int8_t *zq, double *z_real)
{
    joint_z_core(enc_proj, frame_row, pred_proj, N, J, inv_s_z, bits, zq, z_real, NULL);
}

/* Joint, second half + Eq. 1.  logits = Linear_out(zq); lp = log_softmax;
 * fused[blank] = lp[blank]; fused[k] = lp[k] - lambda_src*lp_src[k]
 * + lambda_ext*lp_ext[k] + rho for k != blank (the LMs score label sequences,
 * which hold no blank; rho is the per-label insertion reward of Eq. 1).
 * lp_src/lp_ext may be NULL (term dropped).
 * Pinned by: sum exp(lp)=1, lambda=rho=0 gives lp, affinity in lambda. */
void oq_joint_out(const oq_linear_t *out, const int8_t *zq, const float *lp_src, const float *lp_ext,
                  float lambda_src, float lambda_ext, float rho, int N, int blank,
                  float *lp_rnnt, float *fused)
{
    const int V = out->rows, J = out->cols;
    double *buf = (double *)malloc(sizeof(double) * 2 * (size_t)V);
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < V; ++k) {
            int32_t s = 0;
            for (int j = 0; j < J; ++j) s += (int32_t)out->w[(int64_t)k * J + j] * (int32_t)zq[(int64_t)n * J + j];
            buf[k] = (double)out->s_a * (double)out->s_w[k] * (double)s + (out->bias ? (double)out->bias[k] : 0.0);
        }
        log_softmax_d(buf, V, buf + V);
        for (int k = 0; k < V; ++k) {
            double lp = buf[V + k], f = lp;
            if (k != blank) {
                if (lp_src) f -= (double)lambda_src * (double)lp_src[(int64_t)n * V + k];
                if (lp_ext) f += (double)lambda_ext * (double)lp_ext[(int64_t)n * V + k];
                f += (double)rho;
            }
            if (lp_rnnt) lp_rnnt[(int64_t)n * V + k] = (float)lp;
            fused[(int64_t)n * V + k] = (float)f;
        }
    }
    free(buf);
}

static void joint_fuse_core(const float *enc_proj, const int32_t *frame_row, const float *pred_proj,
                            const oq_linear_t *out, float inv_s_z, const float *lp_src, const float *lp_ext,
                            float lambda_src, float lambda_ext, float rho, int N, int blank,
                            int8_t *zq_out, float *lp_rnnt, float *fused, double *row_margin)
{
    int8_t *zq = zq_out ? zq_out : (int8_t *)malloc((size_t)N * out->cols);
    joint_z_core(enc_proj, frame_row, pred_proj, N, out->cols, inv_s_z, out->bits, zq, NULL, row_margin);
    oq_joint_out(out, zq, lp_src, lp_ext, lambda_src, lambda_ext, rho, N, blank, lp_rnnt, fused);
    if (!zq_out) free(zq);
}

void oq_joint_fuse(const float *enc_proj, const int32_t *frame_row, const float *pred_proj,
                   const oq_linear_t *out, float inv_s_z, const float *lp_src, const float *lp_ext,
                   float lambda_src, float lambda_ext, float rho, int N, int blank,
                   int8_t *zq_out, float *lp_rnnt, float *fused)
{
    joint_fuse_core(enc_proj, frame_row, pred_proj, out, inv_s_z, lp_src, lp_ext, lambda_src, lambda_ext, rho, N, blank,
                    zq_out, lp_rnnt, fused, NULL);
}

/* ------------------------------------------------------------------ */
/* Beam selection and the time-synchronous search                       */
/* ------------------------------------------------------------------ */

/* Per utterance: candidates (w,k) with value score[w] + fused[w,k] (fp32 add:
 * this sum decides a ranking, taken in the GPU path's precision); keep the W
 * best by (value descending, flat index w*V+k ascending); -inf is never kept.
 * force_blank != 0 restricts the candidates to k == blank.  Unfilled ranks get
 * parent = token = -1, score = -inf.
 * Pinned by: numpy lexsort restatement, tie case, -inf case. */
static void beam_step_core(const float *score, const float *fused, int B, int W, int V, int blank,
                           int force_blank, int32_t *parent_out, int32_t *token_out, float *score_out,
                           double *utt_gap /* [B] or NULL: lowered to the smallest difference between
                                              consecutive values among the picks and the best candidate
                                              left out (what a perturbation of the values must exceed to
                                              change the picks or their order) */)
{
    for (int b = 0; b < B; ++b) {
        int nc = W * V;
        float *val = (float *)malloc(sizeof(float) * (size_t)nc);
        uint8_t *taken = (uint8_t *)calloc((size_t)nc, 1);
        for (int w = 0; w < W; ++w)
            for (int k = 0; k < V; ++k) {
                float v = score[b * W + w] + fused[((int64_t)b * W + w) * V + k];
                if (force_blank && k != blank) v = -INFINITY;
                val[w * V + k] = v;
            }
        for (int r = 0; r < W; ++r) {
            int best = -1;
            for (int c = 0; c < nc; ++c) {
                if (taken[c] || !(val[c] > -INFINITY)) continue;
                if (best < 0 || val[c] > val[best]) best = c; /* first index wins a tie */
            }
            if (best < 0) {
                parent_out[b * W + r] = -1; token_out[b * W + r] = -1; score_out[b * W + r] = -INFINITY;
            } else {
                taken[best] = 1;
                parent_out[b * W + r] = best / V; token_out[b * W + r] = best % V; score_out[b * W + r] = val[best];
            }
        }
        if (utt_gap) {
            float prev = INFINITY;
            for (int r = 0; r <= W; ++r) {
                float v = -INFINITY;
                if (r < W) {
                    v = score_out[b * W + r];
                } else {   /* the best candidate that was not picked */
                    for (int c = 0; c < nc; ++c)
                        if (!taken[c] && val[c] > v) v = val[c];
                }
                if (!(v > -INFINITY)) break;
                if (r > 0 && (double)prev - (double)v < utt_gap[b]) utt_gap[b] = (double)prev - (double)v;
                prev = v;
            }
        }
        free(val); free(taken);
    }
}

void oq_beam_step(const float *score, const float *fused, int B, int W, int V, int blank,
                  int force_blank, int32_t *parent_out, int32_t *token_out, float *score_out)
{
    beam_step_core(score, fused, B, W, V, blank, force_blank, parent_out, token_out, score_out, NULL);
}

/* oq_beam_step that also lowers utt_gap[b] (caller-initialised) as described at beam_step_core. */
void oq_beam_step_gap(const float *score, const float *fused, int B, int W, int V, int blank,
                      int force_blank, int32_t *parent_out, int32_t *token_out, float *score_out, double *utt_gap)
{
    beam_step_core(score, fused, B, W, V, blank, force_blank, parent_out, token_out, score_out, utt_gap);
}

/* A language model or the prediction network: embedding lookup, the symmetric
 * quantizer on the embedding (FIX boundary, Sec. 3.2), L stacked quantized
 * LSTM steps, one quantized linear layer.  The LM applies log-softmax to the
 * linear output, the prediction network does not.
 * The external LM of Sec. 2 has a bottleneck layer between its LSTM stack and
 * its output layer (has_mid): a second quantized linear layer whose fp32 output
 * is quantized (linear layers quantize their inputs, Sec. 3.2) and feeds `out`.
 * The paper names no activation for it; none is applied. */
typedef struct {
    const float *embed;   /* [V, E] fp32 */
    int32_t E, L;
    float inv_s_e;        /* 7/alpha of the embedding quantizer */
    oq_lstm_t layer[OQ_MAX_LAYERS];
    oq_linear_t out;
    int32_t log_softmax;  /* 1: LM, 0: prediction network */
    int32_t has_mid;
    oq_linear_t mid;      /* [M, H_top]; then out is [rows, M] and out.s_a the step of the codes of mid's output */
    float inv_s_mid;      /* 7/alpha of the quantizer on mid's output */
} oq_net_t;

typedef struct {
    oq_net_t pred, lm_src, lm_ext;
    oq_linear_t joint_out;
    float inv_s_z;
    float lambda_src, lambda_ext, rho;
    int32_t V, blank, use_src, use_ext;
} oq_model_t;

typedef struct {
    int8_t *h[OQ_MAX_LAYERS];
    float *c[OQ_MAX_LAYERS];
    float *y; /* cached output: p [J] or log-probs [V] */
} net_state;

static void ns_alloc(const oq_net_t *net, net_state *s)
{
    for (int l = 0; l < net->L; ++l) {
        s->h[l] = (int8_t *)calloc((size_t)net->layer[l].H, 1);
        s->c[l] = (float *)calloc((size_t)net->layer[l].H, sizeof(float));
    }
    s->y = (float *)calloc((size_t)net->out.rows, sizeof(float));
}
static void ns_free(const oq_net_t *net, net_state *s)
{
    for (int l = 0; l < net->L; ++l) { free(s->h[l]); free(s->c[l]); }
    free(s->y);
}
static void ns_copy(const oq_net_t *net, net_state *d, const net_state *s)
{
    for (int l = 0; l < net->L; ++l) {
        memcpy(d->h[l], s->h[l], (size_t)net->layer[l].H);
        memcpy(d->c[l], s->c[l], (size_t)net->layer[l].H * sizeof(float));
    }
    memcpy(d->y, s->y, (size_t)net->out.rows * sizeof(float));
}

/* Feed one symbol: dst = advance(src, token).  dst and src must differ. */
/* margin (optional): lowered to the smallest oq_tie_distance of the quantizers whose input is computed here
 * (hidden states, the bottleneck's output; the embedding's quantizer sees a stored fp32 value and decides the
 * same way in any implementation). */
static void net_advance(const oq_net_t *net, const net_state *src, int token, net_state *dst, double *margin)
{
    int maxw = net->E;
    for (int l = 0; l < net->L; ++l) if (net->layer[l].H > maxw) maxw = net->layer[l].H;
    int8_t *xin = (int8_t *)malloc((size_t)maxw);
    oq_quantize_sym4(net->embed + (int64_t)token * net->E, net->E, net->inv_s_e, xin);
    for (int l = 0; l < net->L; ++l) {
        double rm = INFINITY;
        lstm_step_core(&net->layer[l], xin, NULL, src->h[l], src->c[l], NULL, 1,
                       dst->h[l], dst->c[l], NULL, NULL, NULL, NULL, margin ? &rm : NULL);
        if (margin && rm < *margin) *margin = rm;
        memcpy(xin, dst->h[l], (size_t)net->layer[l].H);
    }
    if (net->has_mid) {
        float *ym = (float *)malloc((size_t)net->mid.rows * sizeof(float));
        int8_t *qm = (int8_t *)malloc((size_t)net->mid.rows);
        oq_linear(&net->mid, xin, 1, ym, NULL);
        oq_quantize_sym(ym, net->mid.rows, net->inv_s_mid, net->out.bits, qm); /* the output layer's own input quantizer */
        if (margin)
            for (int r = 0; r < net->mid.rows; ++r) {
                const double d = oq_tie_distance(ym[r], net->inv_s_mid, net->out.bits);
                if (d < *margin) *margin = d;
            }
        oq_linear(&net->out, qm, 1, dst->y, NULL);
        free(ym); free(qm);
    } else {
        oq_linear(&net->out, xin, 1, dst->y, NULL);
    }
    if (net->log_softmax) oq_log_softmax(dst->y, 1, net->out.rows, dst->y);
    free(xin);
}

/* Exposed for tests: run `n_tok` symbols through a net from the zero state and
 * return the cached output after each one ([n_tok, out.rows]). */
void oq_net_run(const oq_net_t *net, const int32_t *tokens, int n_tok, float *y_all)
{
    net_state a, b;
    ns_alloc(net, &a); ns_alloc(net, &b);
    for (int i = 0; i < n_tok; ++i) {
        net_advance(net, &a, tokens[i], &b, NULL);
        memcpy(y_all + (int64_t)i * net->out.rows, b.y, (size_t)net->out.rows * sizeof(float));
        net_state t = a; a = b; b = t;
    }
    ns_free(net, &a); ns_free(net, &b);
}

typedef struct {
    int32_t *tok; int len, cap;
    float score;
    net_state pred, src, ext;
} hyp_t;

static void hyp_alloc(const oq_model_t *M, hyp_t *h)
{
    h->tok = NULL; h->len = 0; h->cap = 0; h->score = -INFINITY;
    ns_alloc(&M->pred, &h->pred);
    if (M->use_src) ns_alloc(&M->lm_src, &h->src);
    if (M->use_ext) ns_alloc(&M->lm_ext, &h->ext);
}
static void hyp_free(const oq_model_t *M, hyp_t *h)
{
    free(h->tok);
    ns_free(&M->pred, &h->pred);
    if (M->use_src) ns_free(&M->lm_src, &h->src);
    if (M->use_ext) ns_free(&M->lm_ext, &h->ext);
}
static void hyp_copy(const oq_model_t *M, hyp_t *d, const hyp_t *s)
{
    if (d->cap < s->len + 1) { d->cap = s->len + 16; d->tok = (int32_t *)realloc(d->tok, sizeof(int32_t) * (size_t)d->cap); }
    if (s->len) memcpy(d->tok, s->tok, sizeof(int32_t) * (size_t)s->len);
    d->len = s->len; d->score = s->score;
    ns_copy(&M->pred, &d->pred, &s->pred);
    if (M->use_src) ns_copy(&M->lm_src, &d->src, &s->src);
    if (M->use_ext) ns_copy(&M->lm_ext, &d->ext, &s->ext);
}
/* d = s extended by `token` (all three networks advance from s's state). */
static void hyp_extend(const oq_model_t *M, hyp_t *d, const hyp_t *s, int token, float score, double *margin)
{
    if (d->cap < s->len + 1) { d->cap = s->len + 16; d->tok = (int32_t *)realloc(d->tok, sizeof(int32_t) * (size_t)d->cap); }
    if (s->len) memcpy(d->tok, s->tok, sizeof(int32_t) * (size_t)s->len);
    d->tok[s->len] = token; d->len = s->len + 1; d->score = score;
    net_advance(&M->pred, &s->pred, token, &d->pred, margin);
    if (M->use_src) net_advance(&M->lm_src, &s->src, token, &d->src, margin);
    if (M->use_ext) net_advance(&M->lm_ext, &s->ext, token, &d->ext, margin);
}

/* Time-synchronous beam search with at most max_sym labels per frame, one
 * utterance at a time (Sec. 2 describes a beam of up to 16 hypotheses kept per
 * iteration of the decoding loop; the frame-synchronous variant with an
 * emission cap is the measured configuration's).
 *
 *   beam: up to W hypotheses.  Start: the empty sequence, score 0, networks
 *   advanced once on symbol 0 from the zero state.
 *   for each frame t:  A <- beam, Nx <- empty
 *     for round v = 0..max_sym:
 *       F[w,:] = joint_fuse(e[t], hypothesis w of A)           (Eq. 1)
 *       pick the W best (w,k) by oq_beam_step (blank only when v == max_sym)
 *       picked blank   -> copy of hypothesis w with the new score joins Nx
 *       picked label k -> hypothesis w extended by k joins the next A
 *       stop the frame when the next A is empty
 *     beam <- the W best of Nx by (score descending, insertion order)
 *   No recombination of equal label sequences.
 *
 * enc_proj [T,B,J] fp32.  Outputs per utterance, best first: tokens
 * [B,W,max_len] (padded with -1), lengths [B,W] (-1 for an unused rank),
 * scores [B,W].
 * Pinned by: W=1 vs an independent greedy loop, exhaustive enumeration on a
 * tiny case, permutation of utterances, monotone scores. */
static void decode_core(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int max_sym,
                        int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                        double *qmargin, double *smargin)
{
    const int V = M->V, J = M->joint_out.cols;
    const int want = qmargin != NULL && smargin != NULL;
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        int nx_cap = W * (max_sym + 1);
        double qm = INFINITY, sm = INFINITY;   /* bookkeeping only, see oq_decode_margins */
        double *rowm = (double *)malloc(sizeof(double) * (size_t)W);
        hyp_t *beam = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)W);
        hyp_t *A = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)W);
        hyp_t *A2 = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)W);
        hyp_t *Nx = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)nx_cap);
        for (int w = 0; w < W; ++w) { hyp_alloc(M, &beam[w]); hyp_alloc(M, &A[w]); hyp_alloc(M, &A2[w]); }
        for (int i = 0; i < nx_cap; ++i) hyp_alloc(M, &Nx[i]);
        float *S = (float *)malloc(sizeof(float) * (size_t)W);
        float *F = (float *)malloc(sizeof(float) * (size_t)W * V);
        float *P = (float *)malloc(sizeof(float) * (size_t)W * J);
        float *Ls = (float *)malloc(sizeof(float) * (size_t)W * V);
        float *Le = (float *)malloc(sizeof(float) * (size_t)W * V);
        int32_t *frow = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
        int32_t *par = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
        int32_t *tk = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
        float *ns = (float *)malloc(sizeof(float) * (size_t)W);

        /* start hypothesis: zero state advanced on symbol 0 */
        {
            hyp_t zero; hyp_alloc(M, &zero);
            hyp_extend(M, &beam[0], &zero, 0, 0.0f, want ? &qm : NULL);
            beam[0].len = 0; /* the start symbol is not part of the label sequence */
            hyp_free(M, &zero);
        }
        int n_beam = 1;

        for (int t = 0; t < T; ++t) {
            int nA = n_beam, nNx = 0;
            for (int w = 0; w < nA; ++w) hyp_copy(M, &A[w], &beam[w]);
            for (int v = 0; v <= max_sym && nA > 0; ++v) {
                for (int w = 0; w < W; ++w) {
                    frow[w] = t * B + b;
                    S[w] = w < nA ? A[w].score : -INFINITY;
                    const hyp_t *h = &A[w < nA ? w : 0];
                    memcpy(P + (int64_t)w * J, h->pred.y, sizeof(float) * (size_t)J);
                    if (M->use_src) memcpy(Ls + (int64_t)w * V, h->src.y, sizeof(float) * (size_t)V);
                    if (M->use_ext) memcpy(Le + (int64_t)w * V, h->ext.y, sizeof(float) * (size_t)V);
                }
                joint_fuse_core(enc_proj, frow, P, &M->joint_out, M->inv_s_z,
                                M->use_src ? Ls : NULL, M->use_ext ? Le : NULL,
                                M->lambda_src, M->lambda_ext, M->rho, W, M->blank, NULL, NULL, F, want ? rowm : NULL);
                if (want)
                    for (int w = 0; w < nA; ++w) if (rowm[w] < qm) qm = rowm[w];
                beam_step_core(S, F, 1, W, V, M->blank, v == max_sym, par, tk, ns, want ? &sm : NULL);
                int nA2 = 0;
                for (int r = 0; r < W; ++r) {
                    if (par[r] < 0) break;
                    if (tk[r] == M->blank) {
                        hyp_copy(M, &Nx[nNx], &A[par[r]]);
                        Nx[nNx].score = ns[r];
                        ++nNx;
                    } else {
                        hyp_extend(M, &A2[nA2], &A[par[r]], tk[r], ns[r], want ? &qm : NULL);
                        ++nA2;
                    }
                }
                hyp_t *tmp = A; A = A2; A2 = tmp;
                nA = nA2;
            }
            /* beam <- W best of Nx, ties by insertion order */
            uint8_t *used = (uint8_t *)calloc((size_t)nx_cap, 1);
            n_beam = 0;
            for (int r = 0; r < W; ++r) {
                int best = -1;
                for (int i = 0; i < nNx; ++i) {
                    if (used[i]) continue;
                    if (best < 0 || Nx[i].score > Nx[best].score) best = i;
                }
                if (best < 0) break;
                used[best] = 1;
                hyp_copy(M, &beam[n_beam++], &Nx[best]);
            }
            if (want) {   /* consecutive differences among the new beam and the best candidate left out */
                float left = -INFINITY;
                for (int i = 0; i < nNx; ++i) if (!used[i] && Nx[i].score > left) left = Nx[i].score;
                for (int r = 0; r < n_beam; ++r) {
                    const float nextv = r + 1 < n_beam ? beam[r + 1].score : left;
                    if (nextv > -INFINITY && (double)beam[r].score - (double)nextv < sm) sm = (double)beam[r].score - (double)nextv;
                }
            }
            free(used);
        }
        if (want) { qmargin[b] = qm; smargin[b] = sm; }
        free(rowm);
        for (int w = 0; w < W; ++w) {
            int32_t *dst = tokens_out + ((int64_t)b * W + w) * max_len;
            for (int i = 0; i < max_len; ++i) dst[i] = -1;
            if (w < n_beam) {
                int len = beam[w].len < max_len ? beam[w].len : max_len;
                memcpy(dst, beam[w].tok, sizeof(int32_t) * (size_t)len);
                len_out[b * W + w] = beam[w].len;
                score_out[b * W + w] = beam[w].score;
            } else {
                len_out[b * W + w] = -1;
                score_out[b * W + w] = -INFINITY;
            }
        }
        for (int w = 0; w < W; ++w) { hyp_free(M, &beam[w]); hyp_free(M, &A[w]); hyp_free(M, &A2[w]); }
        for (int i = 0; i < nx_cap; ++i) hyp_free(M, &Nx[i]);
        free(beam); free(A); free(A2); free(Nx);
        free(S); free(F); free(P); free(Ls); free(Le); free(frow); free(par); free(tk); free(ns);
    }
}

void oq_decode(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int max_sym,
               int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out)
{
    decode_core(M, enc_proj, T, B, W, max_sym, max_len, tokens_out, len_out, score_out, NULL, NULL);
}

/* oq_decode plus, per utterance, how far its result is from depending on the last
 * bits of the arithmetic (bookkeeping for free-running comparisons with an fp32
 * implementation; the search itself is unchanged):
 *   qmargin[b]: the smallest oq_tie_distance over every quantizer decision on a
 *     computed value (hidden states, z, bottleneck output) of a live hypothesis;
 *   smargin[b]: the smallest difference between consecutive values in any selection
 *     (among the picks of a round and the best candidate left out; among the new
 *     beam of a frame and the best entry left out).  0 for an exact tie.
 * A result is robust to perturbations below both.  Pinned by: a hand-built near-tie
 * lowers the margin to the planted distance; margins do not change the outputs. */
void oq_decode_margins(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int max_sym,
                       int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                       double *qmargin, double *smargin)
{
    decode_core(M, enc_proj, T, B, W, max_sym, max_len, tokens_out, len_out, score_out, qmargin, smargin);
}

/* Alignment-length synchronous search with recombination (Sec. 2: the paper
 * decodes with the alignment-length synchronous search of its reference on
 * that algorithm, beam width 1 to 16; the paper itself prints no pseudo-code,
 * so this follows the published algorithm as understood).  All hypotheses of
 * the beam have consumed the same number i of alignment steps (labels + blanks):
 * a hypothesis with u labels stands at frame t = i - u.
 *
 *   beam: W slots, slot 0 = the empty sequence (score 0), the others dead.
 *   finals: the W best finished hypotheses so far.
 *   for i = 0 .. T + u_max - 1:
 *     F[w,:] = joint_fuse(e[t_w], hypothesis w)                       (Eq. 1)
 *     candidates (w,k) with value score_w + F[w,k]; a label is not a candidate
 *       when hypothesis w already holds u_max labels;
 *     a blank at the last frame (t_w == T-1) finishes hypothesis w: it joins the
 *       finals with that value and is not a candidate;
 *     picks: the W best candidates by oq_beam_step's order; pick r becomes slot r
 *       (blank: the same hypothesis one frame later; label: extended, all networks
 *       advanced);
 *     recombination: picks with equal label sequences are one hypothesis: the
 *       best-ranked of them keeps its slot with score log(sum exp(scores)), the
 *       others die (their slots stay empty for the next iteration);
 *     finals <- the W best of finals + new finals by (score descending, insertion
 *       order; new finals are inserted in slot order).
 *
 * With a beam wide enough that nothing is pruned, the final score of a label
 * sequence is the log of its total probability over all alignments plus its
 * label-wise fusion terms: that is what pins this function (RNN-T forward
 * recursion in numpy).  Also pinned by: permutation of utterances, u_max = 0
 * (all-blank path only).
 * Parity unpinned: two choices of this function are readings that neither the
 * paper (which prints no algorithm) nor any pin fixes, because the forward-
 * recursion pin runs without pruning: (1) the W best candidates are picked
 * first and equal label sequences are merged afterwards, so a merge frees slots
 * that stay empty (merging before picking would fill them with further
 * candidates); (2) the finished list is cut to its W best at every insertion.
 * Outputs as oq_decode; ranks beyond the number of finals are empty. */
typedef struct { int32_t *tok; int len; float score; } fin_t;

/* Reuse of cached hypotheses (Sec. 4.1 names it as what makes the decoding time fall sub-linearly at small
 * beams): the state of the prediction network and of the LMs after a label sequence depends on that sequence
 * alone, so a hypothesis that reaches a sequence some other hypothesis has already reached can take over its
 * network states instead of advancing the networks again.  The result of the search is the same bit for bit;
 * only the number of network advances changes, which is what the counters report.
 *   cache_mode 0: none (every label pick that keeps its slot advances the networks);
 *   cache_mode 1: the current beam is the cache (a sequence that a live hypothesis of the beam holds);
 *   cache_mode 2: every sequence ever extended in this utterance stays cached. */
typedef struct { int32_t *tok; int len; hyp_t h; } cache_ent;

static int same_seq(const int32_t *a, int la, const int32_t *b, int lb, int extra_b)
{   /* is a == b followed by extra_b (extra_b < 0: b alone)? */
    const int lbb = lb + (extra_b >= 0);
    if (la != lbb) return 0;
    for (int p = 0; p < la; ++p)
        if (a[p] != (p < lb ? b[p] : extra_b)) return 0;
    return 1;
}

static void decode_alsd_core(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int u_max,
                             int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                             double *qmargin, double *smargin, int cache_mode, int64_t *requested, int64_t *performed)
{
    const int V = M->V, J = M->joint_out.cols;
    const int want = qmargin != NULL && smargin != NULL;
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        double qm = INFINITY, sm = INFINITY;   /* bookkeeping only, see oq_decode_margins */
        double *rowm = (double *)malloc(sizeof(double) * (size_t)W);
        hyp_t *cur = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)W);
        hyp_t *nxt = (hyp_t *)malloc(sizeof(hyp_t) * (size_t)W);
        for (int w = 0; w < W; ++w) { hyp_alloc(M, &cur[w]); hyp_alloc(M, &nxt[w]); }
        fin_t *fin = (fin_t *)calloc((size_t)W + 1, sizeof(fin_t));
        cache_ent *cache = NULL;
        int n_cache = 0, cap_cache = 0;
        int64_t n_req = 0, n_done = 0;
        int nfin = 0;
        float *S = (float *)malloc(sizeof(float) * (size_t)W);
        float *F = (float *)malloc(sizeof(float) * (size_t)W * V);
        float *P = (float *)malloc(sizeof(float) * (size_t)W * J);
        float *Ls = (float *)malloc(sizeof(float) * (size_t)W * V);
        float *Le = (float *)malloc(sizeof(float) * (size_t)W * V);
        int32_t *frow = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
        int32_t *par = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
        int32_t *tk = (int32_t *)malloc(sizeof(int32_t) * (size_t)W);
        float *ns = (float *)malloc(sizeof(float) * (size_t)W);
        int *lead = (int *)malloc(sizeof(int) * (size_t)W);
        {
            hyp_t zero; hyp_alloc(M, &zero);
            hyp_extend(M, &cur[0], &zero, 0, 0.0f, want ? &qm : NULL);
            cur[0].len = 0;
            hyp_free(M, &zero);
        }
        for (int i = 0; i < T + u_max; ++i) {
            int alive = 0;
            for (int w = 0; w < W; ++w) {
                const int live = cur[w].score > -INFINITY;
                alive += live;
                const hyp_t *h = &cur[live ? w : 0];
                int t = live ? i - cur[w].len : 0;
                if (t < 0) t = 0;
                if (t > T - 1) t = T - 1;
                frow[w] = t * B + b;
                S[w] = live ? cur[w].score : -INFINITY;
                memcpy(P + (int64_t)w * J, h->pred.y, sizeof(float) * (size_t)J);
                if (M->use_src) memcpy(Ls + (int64_t)w * V, h->src.y, sizeof(float) * (size_t)V);
                if (M->use_ext) memcpy(Le + (int64_t)w * V, h->ext.y, sizeof(float) * (size_t)V);
            }
            if (!alive) break;
            joint_fuse_core(enc_proj, frow, P, &M->joint_out, M->inv_s_z,
                            M->use_src ? Ls : NULL, M->use_ext ? Le : NULL,
                            M->lambda_src, M->lambda_ext, M->rho, W, M->blank, NULL, NULL, F, want ? rowm : NULL);
            if (want)
                for (int w = 0; w < W; ++w) if (cur[w].score > -INFINITY && rowm[w] < qm) qm = rowm[w];
            /* finished hypotheses and excluded labels leave the candidate set */
            for (int w = 0; w < W; ++w) {
                if (!(cur[w].score > -INFINITY)) continue;
                const int t = i - cur[w].len;
                if (t == T - 1) {
                    const float v = S[w] + F[(int64_t)w * V + M->blank];
                    F[(int64_t)w * V + M->blank] = -INFINITY;
                    if (want)   /* how close the newcomer is to any final it is ranked against */
                        for (int q = 0; q < nfin; ++q) {
                            const double d = fabs((double)fin[q].score - (double)v);
                            if (d < sm) sm = d;
                        }
                    /* insert after every final that is at least as good (insertion order on ties) */
                    int pos = nfin;
                    while (pos > 0 && fin[pos - 1].score < v) --pos;
                    if (pos < W) {
                        if (nfin == W) { free(fin[W - 1].tok); nfin = W - 1; }
                        for (int q = nfin; q > pos; --q) fin[q] = fin[q - 1];
                        fin[pos].len = cur[w].len; fin[pos].score = v;
                        fin[pos].tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(cur[w].len + 1));
                        if (cur[w].len) memcpy(fin[pos].tok, cur[w].tok, sizeof(int32_t) * (size_t)cur[w].len);
                        ++nfin;
                    }
                }
                if (cur[w].len >= u_max)
                    for (int k = 0; k < V; ++k)
                        if (k != M->blank) F[(int64_t)w * V + k] = -INFINITY;
            }
            beam_step_core(S, F, 1, W, V, M->blank, 0, par, tk, ns, want ? &sm : NULL);
            /* recombination on the label sequences the picks stand for */
            for (int r = 0; r < W; ++r) {
                lead[r] = -1;
                if (par[r] < 0) continue;
                lead[r] = r;
                const hyp_t *hr = &cur[par[r]];
                const int lr = hr->len + (tk[r] != M->blank);
                for (int q = 0; q < r; ++q) {
                    if (par[q] < 0 || lead[q] != q) continue;
                    const hyp_t *hq = &cur[par[q]];
                    const int lq = hq->len + (tk[q] != M->blank);
                    if (lq != lr) continue;
                    int same = 1;
                    for (int p = 0; p < lr && same; ++p) {
                        const int a = p < hr->len ? hr->tok[p] : tk[r];
                        const int c = p < hq->len ? hq->tok[p] : tk[q];
                        same = a == c;
                    }
                    if (same) { lead[r] = q; break; }
                }
            }
            for (int r = 0; r < W; ++r) {
                nxt[r].score = -INFINITY;
                nxt[r].len = 0;
                if (par[r] < 0 || lead[r] != r) continue;
                double m = -INFINITY, sum = 0.0;
                for (int q = r; q < W; ++q)
                    if (par[q] >= 0 && lead[q] == r && (double)ns[q] > m) m = (double)ns[q];
                for (int q = r; q < W; ++q)
                    if (par[q] >= 0 && lead[q] == r) sum += exp((double)ns[q] - m);
                const float sc = (float)(m + log(sum));
                if (tk[r] == M->blank) { hyp_copy(M, &nxt[r], &cur[par[r]]); nxt[r].score = sc; }
                else {
                    const hyp_t *pr = &cur[par[r]];
                    const hyp_t *hit = NULL;
                    ++n_req;
                    if (cache_mode == 1) {
                        for (int j = 0; j < W && !hit; ++j)
                            if (cur[j].score > -INFINITY && same_seq(cur[j].tok, cur[j].len, pr->tok, pr->len, tk[r])) hit = &cur[j];
                    } else if (cache_mode == 2) {
                        for (int j = 0; j < n_cache && !hit; ++j)
                            if (same_seq(cache[j].tok, cache[j].len, pr->tok, pr->len, tk[r])) hit = &cache[j].h;
                    }
                    if (hit) {   /* the networks' states after this sequence exist already: take them over */
                        const hyp_t *src = hit;
                        hyp_copy(M, &nxt[r], src);
                        if (nxt[r].cap < pr->len + 1) { nxt[r].cap = pr->len + 16; nxt[r].tok = (int32_t *)realloc(nxt[r].tok, sizeof(int32_t) * (size_t)nxt[r].cap); }
                        if (pr->len) memcpy(nxt[r].tok, pr->tok, sizeof(int32_t) * (size_t)pr->len);
                        nxt[r].tok[pr->len] = tk[r];
                        nxt[r].len = pr->len + 1;
                        nxt[r].score = sc;
                    } else {
                        ++n_done;
                        hyp_extend(M, &nxt[r], pr, tk[r], sc, want ? &qm : NULL);
                        if (cache_mode == 2) {
                            if (n_cache == cap_cache) { cap_cache = cap_cache ? 2 * cap_cache : 64; cache = (cache_ent *)realloc(cache, sizeof(cache_ent) * (size_t)cap_cache); }
                            cache_ent *ce = &cache[n_cache++];
                            ce->len = nxt[r].len;
                            ce->tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(ce->len + 1));
                            memcpy(ce->tok, nxt[r].tok, sizeof(int32_t) * (size_t)ce->len);
                            hyp_alloc(M, &ce->h);
                            hyp_copy(M, &ce->h, &nxt[r]);
                        }
                    }
                }
            }
            hyp_t *tmp = cur; cur = nxt; nxt = tmp;
        }
        for (int w = 0; w < W; ++w) {
            int32_t *dst = tokens_out + ((int64_t)b * W + w) * max_len;
            for (int q = 0; q < max_len; ++q) dst[q] = -1;
            if (w < nfin) {
                const int len = fin[w].len < max_len ? fin[w].len : max_len;
                if (len) memcpy(dst, fin[w].tok, sizeof(int32_t) * (size_t)len);
                len_out[b * W + w] = fin[w].len;
                score_out[b * W + w] = fin[w].score;
            } else {
                len_out[b * W + w] = -1;
                score_out[b * W + w] = -INFINITY;
            }
        }
        if (want) { qmargin[b] = qm; smargin[b] = sm; }
        free(rowm);
        if (requested) requested[b] = n_req;
        if (performed) performed[b] = n_done;
        for (int j = 0; j < n_cache; ++j) { free(cache[j].tok); hyp_free(M, &cache[j].h); }
        free(cache);
        for (int q = 0; q < nfin; ++q) free(fin[q].tok);
        for (int w = 0; w < W; ++w) { hyp_free(M, &cur[w]); hyp_free(M, &nxt[w]); }
        free(cur); free(nxt); free(fin);
        free(S); free(F); free(P); free(Ls); free(Le); free(frow); free(par); free(tk); free(ns); free(lead);
    }
}

void oq_decode_alsd(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int u_max,
                    int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out)
{
    decode_alsd_core(M, enc_proj, T, B, W, u_max, max_len, tokens_out, len_out, score_out, NULL, NULL, 0, NULL, NULL);
}

/* oq_decode_alsd with the margins of oq_decode_margins; smargin also covers the
 * ranking of every newly finished hypothesis against the finished list. */
void oq_decode_alsd_margins(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int u_max,
                            int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                            double *qmargin, double *smargin)
{
    decode_alsd_core(M, enc_proj, T, B, W, u_max, max_len, tokens_out, len_out, score_out, qmargin, smargin, 0, NULL, NULL);
}

/* oq_decode_alsd with reuse of cached hypotheses (see cache_ent above).  requested[b]: label picks of
 * utterance b that kept their slot, i.e. network advances without a cache; performed[b]: advances actually
 * made.  Pinned by: identical outputs in all three modes; with nothing pruned and V - 1 labels, mode 2
 * performs exactly one advance per distinct label sequence of length 1 .. u_max. */
void oq_decode_alsd_cached(const oq_model_t *M, const float *enc_proj, int T, int B, int W, int u_max,
                           int max_len, int32_t *tokens_out, int32_t *len_out, float *score_out,
                           int cache_mode, int64_t *requested, int64_t *performed)
{
    decode_alsd_core(M, enc_proj, T, B, W, u_max, max_len, tokens_out, len_out, score_out, NULL, NULL, cache_mode,
                     requested, performed);
}

/* Score of one fixed alignment, for the exhaustive-search pin: `actions` is a
 * sequence of symbols (blank advances the frame, a label extends the
 * hypothesis) consumed from frame 0; returns the sum of fused scores along it
 * (fp32 accumulation, as the search does).  The caller guarantees exactly T
 * blanks. */
float oq_score_alignment(const oq_model_t *M, const float *enc_proj, int B, int b,
                         const int32_t *actions, int n_act)
{
    const int V = M->V, J = M->joint_out.cols;
    hyp_t cur, nxt, zero;
    hyp_alloc(M, &cur); hyp_alloc(M, &nxt); hyp_alloc(M, &zero);
    hyp_extend(M, &cur, &zero, 0, 0.0f, NULL);
    cur.len = 0;
    float *F = (float *)malloc(sizeof(float) * (size_t)V);
    (void)J;
    int t = 0;
    float S = 0.0f;
    for (int a = 0; a < n_act; ++a) {
        int32_t frow = t * B + b;
        oq_joint_fuse(enc_proj, &frow, cur.pred.y, &M->joint_out, M->inv_s_z,
                      M->use_src ? cur.src.y : NULL, M->use_ext ? cur.ext.y : NULL,
                      M->lambda_src, M->lambda_ext, M->rho, 1, M->blank, NULL, NULL, F);
        S = S + F[actions[a]];
        if (actions[a] == M->blank) {
            ++t;
        } else {
            hyp_extend(M, &nxt, &cur, actions[a], S, NULL);
            hyp_t tmp = cur; cur = nxt; nxt = tmp;
        }
    }
    free(F);
    hyp_free(M, &cur); hyp_free(M, &nxt); hyp_free(M, &zero);
    return S;
}

int oq_struct_sizes(int which)
{
    switch (which) {
    case 0: return (int)sizeof(oq_lstm_t);
    case 1: return (int)sizeof(oq_linear_t);
    case 2: return (int)sizeof(oq_net_t);
    case 3: return (int)sizeof(oq_model_t);
    default: return -1;
    }
}
