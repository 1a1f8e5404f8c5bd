// Weight quantization + nibble packing, unpacking, and the activation quantizer.
// Sec. 3.1 (MAX range picker per row, symmetric linear quantization) and
// Sec. 3.2 (weights are quantized once, activations at every step).
#include "qrnnt_common.h"

extern "C" const char *qrnnt_status_str(qrnnt_status s)
{
    switch (s) {
    case QRNNT_OK: return "ok";
    case QRNNT_ERR_NULL: return "required pointer is NULL";
    case QRNNT_ERR_SHAPE: return "bad shape";
    case QRNNT_ERR_ALIGN: return "misaligned pointer";
    case QRNNT_ERR_RANGE: return "argument out of range";
    case QRNNT_ERR_WORKSPACE: return "workspace too small";
    case QRNNT_ERR_LAYOUT: return "wrong weight layout";
    case QRNNT_ERR_UNSUPPORTED: return "unsupported size";
    case QRNNT_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" uint32_t qrnnt_abi_version(void) { return 3u; }

static size_t pack_bytes(int32_t rows, int32_t cols, int32_t layout, int bits)
{
    if (rows <= 0 || cols <= 0) return 0;
    const size_t per = bits == 8 ? 2 : 1;   // an 8-bit matrix takes two blocks where a 4-bit one takes one
    if (layout == QRNNT_LAYOUT_ROWMAJOR) return (size_t)rows * (size_t)(qr_round_up(cols, 64) / 2) * per;
    if (layout == QRNNT_LAYOUT_TILED || layout == QRNNT_LAYOUT_TILED_GATES) {
        if (layout == QRNNT_LAYOUT_TILED_GATES && rows % 4 != 0) return 0;
        // TILED_GATES works in groups of 16 cells = 64 rows
        const int rp = layout == QRNNT_LAYOUT_TILED_GATES ? qr_round_up(rows, 64) : qr_round_up(rows, 16);
        return (size_t)(rp / 16) * (size_t)(qr_round_up(cols, QRNNT_KCHUNK) / QRNNT_KCHUNK) * QRNNT_BLOCK_BYTES * per;
    }
    return 0;
}

extern "C" size_t qrnnt_pack_int4_bytes(int32_t rows, int32_t cols, int32_t layout) { return pack_bytes(rows, cols, layout, 4); }
extern "C" size_t qrnnt_pack_int8_bytes(int32_t rows, int32_t cols, int32_t layout) { return pack_bytes(rows, cols, layout, 8); }

// Per-row alpha = max|w|; scale = alpha/7, inv = 7/alpha (fp32 divisions); an
// all-zero row gets scale 1 (its codes are zero anyway).
__global__ __launch_bounds__(256) void row_scale_kernel(const float *__restrict__ w, int rows, int cols, float qmax,
                                                         float *__restrict__ scale)
{
    __shared__ float red[4];
    const int r = blockIdx.x;
    const float *wr = w + (size_t)r * cols;
    float m = 0.0f;
    for (int k = threadIdx.x; k < cols; k += blockDim.x) m = fmaxf(m, fabsf(wr[k]));
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        scale[r] = (a == 0.0f) ? 1.0f : a / qmax;
    }
}

// One thread per 32-bit word of the packed output.
// TILED: word index = ((rt*nkc + kc)*64 + lane)*4 + d.
template <bool FP32>
__global__ __launch_bounds__(256) void pack_tiled_kernel(const void *__restrict__ src, const float *__restrict__ inv_alpha7,
                                                          int rows, int cols, int nkc, int gates, size_t n_words,
                                                          uint32_t *__restrict__ out)
{
    size_t widx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (widx >= n_words) return;
    const int d = (int)(widx & 3);
    const int lane = (int)((widx >> 2) & 63);
    const size_t blk = widx >> 8;
    const int kc = (int)(blk % nkc);
    const int rt = (int)(blk / nkc);
    const int tr = rt * 16 + (lane & 15);
    uint32_t word = 0;
    const int H = rows >> 2;
    const int cell = qr_gates_cell(rt, (lane & 15) >> 2);
    if (gates ? cell < H : tr < rows) {
        const int r = gates ? (tr & 3) * H + cell : tr;
        float inv = 0.0f;
        if (FP32) inv = inv_alpha7[r];
        const int kbase = kc * QRNNT_KCHUNK + (lane >> 4) * 16 + d * 4;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int k = kbase + b + half * 64;
                int q = 0;
                if (k < cols) {
                    if (FP32) {
                        q = qr_quant4(((const float *)src)[(size_t)r * cols + k], inv);
                    } else {
                        int v = ((const int8_t *)src)[(size_t)r * cols + k];
                        q = v < -8 ? -8 : (v > 7 ? 7 : v);
                    }
                }
                word |= (uint32_t)(q & 0xF) << (8 * b + 4 * half);
            }
        }
    }
    out[widx] = word;
}

// The 8-bit form: two blocks per (row tile, 128-column chunk), the second 64 columns after the first;
// word index = (((rt*nkc + kc)*2 + half)*64 + lane)*4 + d, four int8 codes per word.
template <bool FP32>
__global__ __launch_bounds__(256) void pack_tiled8_kernel(const void *__restrict__ src, const float *__restrict__ inv_alpha,
                                                           int rows, int cols, int nkc, int gates, size_t n_words,
                                                           uint32_t *__restrict__ out)
{
    size_t widx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (widx >= n_words) return;
    const int d = (int)(widx & 3);
    const int lane = (int)((widx >> 2) & 63);
    const int half = (int)((widx >> 8) & 1);
    const size_t blk = widx >> 9;
    const int kc = (int)(blk % nkc);
    const int rt = (int)(blk / nkc);
    const int tr = rt * 16 + (lane & 15);
    uint32_t word = 0;
    const int H = rows >> 2;
    const int cell = qr_gates_cell(rt, (lane & 15) >> 2);
    if (gates ? cell < H : tr < rows) {
        const int r = gates ? (tr & 3) * H + cell : tr;
        const float inv = FP32 ? inv_alpha[r] : 0.0f;
        const int kbase = kc * QRNNT_KCHUNK + half * 64 + (lane >> 4) * 16 + d * 4;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = kbase + b;
            int q = 0;
            if (k < cols)
                q = FP32 ? qr_quant(((const float *)src)[(size_t)r * cols + k], inv, 8) : ((const int8_t *)src)[(size_t)r * cols + k];
            word |= (uint32_t)(q & 0xFF) << (8 * b);
        }
    }
    out[widx] = word;
}

template <bool FP32>
__global__ __launch_bounds__(256) void pack_rowmajor8_kernel(const void *__restrict__ src, const float *__restrict__ inv_alpha,
                                                              int rows, int cols, int bpr, int8_t *__restrict__ out)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)rows * bpr) return;
    const int r = (int)(idx / bpr), k = (int)(idx % bpr);
    int q = 0;
    if (k < cols)
        q = FP32 ? qr_quant(((const float *)src)[(size_t)r * cols + k], inv_alpha[r], 8) : ((const int8_t *)src)[(size_t)r * cols + k];
    out[idx] = (int8_t)q;
}

// ROWMAJOR: one thread per output byte.
template <bool FP32>
__global__ __launch_bounds__(256) void pack_rowmajor_kernel(const void *__restrict__ src, const float *__restrict__ inv_alpha7,
                                                             int rows, int cols, int bpr, uint8_t *__restrict__ out)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)rows * bpr) return;
    const int r = (int)(idx / bpr), j = (int)(idx % bpr);
    int q[2] = {0, 0};
    for (int h = 0; h < 2; ++h) {
        const int k = 2 * j + h;
        if (k < cols) {
            if (FP32) {
                q[h] = qr_quant4(((const float *)src)[(size_t)r * cols + k], inv_alpha7[r]);
            } else {
                int v = ((const int8_t *)src)[(size_t)r * cols + k];
                q[h] = v < -8 ? -8 : (v > 7 ? 7 : v);
            }
        }
    }
    out[idx] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
}

// inv[r] = 7/alpha with alpha recovered exactly as the row maximum.
__global__ __launch_bounds__(256) void row_inv_kernel(const float *__restrict__ w, int rows, int cols, float qmax,
                                                       float *__restrict__ inv)
{
    __shared__ float red[4];
    const int r = blockIdx.x;
    const float *wr = w + (size_t)r * cols;
    float m = 0.0f;
    for (int k = threadIdx.x; k < cols; k += blockDim.x) m = fmaxf(m, fabsf(wr[k]));
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        inv[r] = (a == 0.0f) ? 0.0f : qmax / a;
    }
}

static qrnnt_status pack_any(int bits, const void *src, int32_t src_dtype, int32_t rows, int32_t cols, int32_t layout,
                             void *packed_out, float *row_scale_out, void *stream)
{
    QR_REQUIRE(src != nullptr && packed_out != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(src_dtype == QRNNT_SRC_INT8_CODES || src_dtype == QRNNT_SRC_FP32, QRNNT_ERR_RANGE);
    QR_REQUIRE(src_dtype != QRNNT_SRC_FP32 || row_scale_out != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(rows > 0 && cols > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(layout == QRNNT_LAYOUT_ROWMAJOR || layout == QRNNT_LAYOUT_TILED || layout == QRNNT_LAYOUT_TILED_GATES,
               QRNNT_ERR_LAYOUT);
    QR_REQUIRE(layout != QRNNT_LAYOUT_TILED_GATES || rows % 4 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(qr_aligned(packed_out, 16), QRNNT_ERR_ALIGN);
    QR_REQUIRE(src_dtype != QRNNT_SRC_FP32 || qr_aligned(src, 4), QRNNT_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    const bool fp32 = src_dtype == QRNNT_SRC_FP32;
    // For fp32 sources the packed blob's own tail is not available as scratch, so the
    // per-row 7/alpha lives in row_scale_out until the codes are written, then is
    // replaced by alpha/7.
    const float qmax = bits == 8 ? 127.0f : 7.0f;
    if (fp32) row_inv_kernel<<<rows, 256, 0, st>>>((const float *)src, rows, cols, qmax, row_scale_out);
    if (bits == 8 && layout == QRNNT_LAYOUT_ROWMAJOR) {
        const int bpr = qr_round_up(cols, 64);
        const size_t n = (size_t)rows * bpr;
        const unsigned grid = (unsigned)((n + 255) / 256);
        if (fp32)
            pack_rowmajor8_kernel<true><<<grid, 256, 0, st>>>(src, row_scale_out, rows, cols, bpr, (int8_t *)packed_out);
        else
            pack_rowmajor8_kernel<false><<<grid, 256, 0, st>>>(src, nullptr, rows, cols, bpr, (int8_t *)packed_out);
    } else if (bits == 8) {
        const int nkc = qr_round_up(cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
        const size_t n_words = pack_bytes(rows, cols, layout, 8) / 4;
        const unsigned grid = (unsigned)((n_words + 255) / 256);
        const int gates = layout == QRNNT_LAYOUT_TILED_GATES;
        if (fp32)
            pack_tiled8_kernel<true><<<grid, 256, 0, st>>>(src, row_scale_out, rows, cols, nkc, gates, n_words,
                                                           (uint32_t *)packed_out);
        else
            pack_tiled8_kernel<false><<<grid, 256, 0, st>>>(src, nullptr, rows, cols, nkc, gates, n_words,
                                                            (uint32_t *)packed_out);
    } else if (layout == QRNNT_LAYOUT_ROWMAJOR) {
        const int bpr = qr_round_up(cols, 64) / 2;
        const size_t n = (size_t)rows * bpr;
        const unsigned grid = (unsigned)((n + 255) / 256);
        if (fp32)
            pack_rowmajor_kernel<true><<<grid, 256, 0, st>>>(src, row_scale_out, rows, cols, bpr, (uint8_t *)packed_out);
        else
            pack_rowmajor_kernel<false><<<grid, 256, 0, st>>>(src, nullptr, rows, cols, bpr, (uint8_t *)packed_out);
    } else {
        const int nkc = qr_round_up(cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
        const size_t n_words = qrnnt_pack_int4_bytes(rows, cols, layout) / 4;
        const unsigned grid = (unsigned)((n_words + 255) / 256);
        const int gates = layout == QRNNT_LAYOUT_TILED_GATES;
        if (fp32)
            pack_tiled_kernel<true><<<grid, 256, 0, st>>>(src, row_scale_out, rows, cols, nkc, gates, n_words,
                                                          (uint32_t *)packed_out);
        else
            pack_tiled_kernel<false><<<grid, 256, 0, st>>>(src, nullptr, rows, cols, nkc, gates, n_words,
                                                           (uint32_t *)packed_out);
    }
    if (fp32) row_scale_kernel<<<rows, 256, 0, st>>>((const float *)src, rows, cols, qmax, row_scale_out);
    return qr_launch_status();
}

extern "C" qrnnt_status qrnnt_pack_int4(const void *src, int32_t src_dtype, int32_t rows, int32_t cols, int32_t layout,
                                        void *packed_out, float *row_scale_out, void *stream)
{
    return pack_any(4, src, src_dtype, rows, cols, layout, packed_out, row_scale_out, stream);
}

extern "C" qrnnt_status qrnnt_pack_int8(const void *src, int32_t src_dtype, int32_t rows, int32_t cols, int32_t layout,
                                        void *packed_out, float *row_scale_out, void *stream)
{
    return pack_any(8, src, src_dtype, rows, cols, layout, packed_out, row_scale_out, stream);
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t *__restrict__ packed, int rows, int cols, int layout,
                                                      int bits, int8_t *__restrict__ codes)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)rows * cols) return;
    const int r = (int)(idx / cols), k = (int)(idx % cols);
    int nib;
    if (bits == 8) {
        if (layout == QRNNT_LAYOUT_ROWMAJOR) {
            codes[idx] = (int8_t)packed[(size_t)r * qr_round_up(cols, 64) + k];
        } else {
            const int nkc = qr_round_up(cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
            const int H = rows >> 2;
            const int tr = (layout == QRNNT_LAYOUT_TILED_GATES) ? qr_gates_tiled_row(r % H, r / H) : r;
            const int rt = tr >> 4, kc = k / QRNNT_KCHUNK, kk = k % QRNNT_KCHUNK;
            const int half = kk >> 6, k16 = (kk & 63) >> 4, d = (kk & 15) >> 2, b = kk & 3;
            const int lane = k16 * 16 + (tr & 15);
            codes[idx] = (int8_t)packed[(((size_t)rt * nkc + kc) * 2 + half) * QRNNT_BLOCK_BYTES + lane * 16 + d * 4 + b];
        }
        return;
    }
    if (layout == QRNNT_LAYOUT_ROWMAJOR) {
        const int bpr = qr_round_up(cols, 64) / 2;
        uint8_t byte = packed[(size_t)r * bpr + k / 2];
        nib = (k & 1) ? (byte >> 4) : (byte & 0xF);
    } else {
        const int nkc = qr_round_up(cols, QRNNT_KCHUNK) / QRNNT_KCHUNK;
        const int H = rows >> 2;
        const int tr = (layout == QRNNT_LAYOUT_TILED_GATES) ? qr_gates_tiled_row(r % H, r / H) : r;
        const int rt = tr >> 4, kc = k / QRNNT_KCHUNK, kk = k % QRNNT_KCHUNK;
        const int half = kk >> 6, k16 = (kk & 63) >> 4, d = (kk & 15) >> 2, b = kk & 3;
        const int lane = k16 * 16 + (tr & 15);
        uint8_t byte = packed[((size_t)rt * nkc + kc) * QRNNT_BLOCK_BYTES + lane * 16 + d * 4 + b];
        nib = half ? (byte >> 4) : (byte & 0xF);
    }
    codes[idx] = (int8_t)(nib >= 8 ? nib - 16 : nib);
}

extern "C" qrnnt_status qrnnt_unpack_int4(const qrnnt_qmat *m, int8_t *codes_out, void *stream)
{
    QR_REQUIRE(m != nullptr && m->packed != nullptr && codes_out != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(m->rows > 0 && m->cols > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(m->layout == QRNNT_LAYOUT_ROWMAJOR || m->layout == QRNNT_LAYOUT_TILED ||
                   m->layout == QRNNT_LAYOUT_TILED_GATES,
               QRNNT_ERR_LAYOUT);
    QR_REQUIRE(m->layout != QRNNT_LAYOUT_TILED_GATES || m->rows % 4 == 0, QRNNT_ERR_SHAPE);
    const size_t n = (size_t)m->rows * m->cols;
    QR_REQUIRE(m->bits == 0 || m->bits == 4 || m->bits == 8, QRNNT_ERR_RANGE);
    unpack_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>((const uint8_t *)m->packed, m->rows,
                                                                                 m->cols, m->layout, qr_bits(m), codes_out);
    return qr_launch_status();
}

__global__ __launch_bounds__(256) void quantize_kernel(const float *__restrict__ x, int64_t n, float inv,
                                                        int8_t *__restrict__ q)
{
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 3 < n) {
        const v4f v = *(const v4f *)(x + i);
        uint32_t w = (uint32_t)(qr_quant4(v.x, inv) & 0xFF) | ((uint32_t)(qr_quant4(v.y, inv) & 0xFF) << 8) |
                     ((uint32_t)(qr_quant4(v.z, inv) & 0xFF) << 16) | ((uint32_t)(qr_quant4(v.w, inv) & 0xFF) << 24);
        *(uint32_t *)(q + i) = w;
    } else {
        for (; i < n; ++i) q[i] = (int8_t)qr_quant4(x[i], inv);
    }
}

__global__ __launch_bounds__(256) void quantize8_kernel(const float *__restrict__ x, int64_t n, float inv,
                                                         int8_t *__restrict__ q)
{
    int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i + 3 < n) {
        const v4f v = *(const v4f *)(x + i);
        uint32_t w = (uint32_t)(qr_quant(v.x, inv, 8) & 0xFF) | ((uint32_t)(qr_quant(v.y, inv, 8) & 0xFF) << 8) |
                     ((uint32_t)(qr_quant(v.z, inv, 8) & 0xFF) << 16) | ((uint32_t)(qr_quant(v.w, inv, 8) & 0xFF) << 24);
        *(uint32_t *)(q + i) = w;
    } else {
        for (; i < n; ++i) q[i] = (int8_t)qr_quant(x[i], inv, 8);
    }
}

extern "C" qrnnt_status qrnnt_quantize_act8(const float *x, int64_t n, float inv_scale, int8_t *q, void *stream)
{
    QR_REQUIRE(x != nullptr && q != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(n > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(inv_scale > 0.0f, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(x, 16) && qr_aligned(q, 4), QRNNT_ERR_ALIGN);
    const int64_t n4 = (n + 3) / 4;
    quantize8_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, (hipStream_t)stream>>>(x, n, inv_scale, q);
    return qr_launch_status();
}

extern "C" qrnnt_status qrnnt_quantize_act(const float *x, int64_t n, float inv_scale, int8_t *q, void *stream)
{
    QR_REQUIRE(x != nullptr && q != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(n > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(inv_scale > 0.0f, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(x, 16) && qr_aligned(q, 4), QRNNT_ERR_ALIGN);
    const int64_t n4 = (n + 3) / 4;
    QR_REQUIRE(n4 <= (int64_t)INT32_MAX * 256, QRNNT_ERR_SHAPE);   // one thread per 4 elements, the grid's x limit
    quantize_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, (hipStream_t)stream>>>(x, n, inv_scale, q);
    return qr_launch_status();
}

// rows x cols fp32 (contiguous) -> codes with a row pitch of ld_out bytes; one thread per 4 output bytes, the
// columns behind `cols` are written as zero.
__global__ __launch_bounds__(256) void quantize_rows_kernel(const float *__restrict__ x, int64_t rows, int cols, int ld_out,
                                                             float inv, int bits, int8_t *__restrict__ q)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int wpr = ld_out >> 2;
    if (idx >= rows * wpr) return;
    const int64_t r = idx / wpr;
    const int c0 = (int)(idx - r * wpr) * 4;
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (c0 + i < cols) w |= (uint32_t)(qr_quant(x[r * cols + c0 + i], inv, bits) & 0xFF) << (8 * i);
    *(uint32_t *)(q + r * ld_out + c0) = w;
}

extern "C" int32_t qrnnt_act_pitch(int32_t cols) { return cols > 0 ? qr_act_pitch(cols) : 0; }

extern "C" qrnnt_status qrnnt_quantize_act_rows(const float *x, int64_t rows, int32_t cols, float inv_scale, int32_t bits,
                                                int8_t *q, int32_t ld_out, void *stream)
{
    QR_REQUIRE(x != nullptr && q != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(rows > 0 && cols > 0 && ld_out >= cols && ld_out % 16 == 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(inv_scale > 0.0f && (bits == 4 || bits == 8), QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(x, 4) && qr_aligned(q, 16), QRNNT_ERR_ALIGN);
    QR_REQUIRE(rows <= (int64_t)INT32_MAX * 256 / (ld_out >> 2), QRNNT_ERR_SHAPE);   // the grid's x limit
    const int64_t n = rows * (ld_out >> 2);
    quantize_rows_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(x, rows, cols, ld_out, inv_scale, bits, q);
    return qr_launch_status();
}
