// Diagnostics: issue rates of the matrix instructions that could carry the W4A4 contraction on gfx950, measured
// in registers (no memory traffic in the loop).  Codes in [-8, 7] are exact in int8, fp8-E4M3 and fp6-E3M2 (and
// [-7, 7] in fp6-E2M3), and sums of up to 2048 products stay below 2^24, so these forms would give the same
// integers (Sec. 3.1 / 3.2: the method only fixes the integer grid, not the unit that multiplies); fp4-E2M1 lacks
// 5 and 7 and is listed for its rate only.  Which form to build on is a question of rate and of operand layout.  bench.py reports these rates next to the kernels' achieved ones.
#include "qrnnt_common.h"

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// 8 accumulator chains of the 16 x 16 forms (4 of the 32 x 32 forms) per wave.  Every chain gets two instructions
// per loop iteration (operands swapped for the second), the pattern of the contraction kernels, whose 128-column
// chunk is two K steps into one accumulator; the compiler keeps such a loop free of register moves, so the loop
// body is the matrix instructions and the branch (a body with one instruction per chain and iteration made it
// shuffle the accumulators between the instructions, which halved the measured rate of the 4-pass forms).
template <int FORM>
__global__ __launch_bounds__(256, 2) void mfma_rate_kernel(int iters, float *sink)
{
    const int lane = threadIdx.x;
    const v4i a4 = {lane, lane + 1, 3, 4}, b4 = {lane * 3, 7, 1, 2};
    const v8i a8 = {lane, lane + 1, 3, 4, 5, 6, 0, 0}, b8 = {lane * 3, 7, 1, 2, 9, 8, 0, 0};
    constexpr bool WIDE = FORM == 1 || FORM == 3;        // 32 x 32 forms: 16 accumulator registers per chain
    constexpr bool INT = FORM <= 1;
    constexpr int fmt = FORM == 4 ? 2 : FORM == 5 ? 3 : FORM == 6 ? 4 : 0;   // fp8-E4M3 0, fp6-E2M3 2, fp6-E3M2 3, fp4-E2M1 4
    v4i ci[8];
    v4f cf[8];
    v16i ci32[4];
    v16f cf32[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) { ci[i] = v4i{0, 0, 0, 0}; cf[i] = v4f{0, 0, 0, 0}; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) { ci32[i][j] = 0; cf32[i][j] = 0.0f; }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < (WIDE ? 4 : 8); ++i) {
            if (INT && !WIDE) {
                ci[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a4, b4, ci[i], 0, 0, 0);
                ci[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b4, a4, ci[i], 0, 0, 0);
            }
            if (INT && WIDE) {
                ci32[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a4, b4, ci32[i], 0, 0, 0);
                ci32[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b4, a4, ci32[i], 0, 0, 0);
            }
            if (!INT && !WIDE) {
                cf[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, cf[i], fmt, fmt, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
                cf[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b8, a8, cf[i], fmt, fmt, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
            }
            if (!INT && WIDE) {
                cf32[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, cf32[i], fmt, fmt, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
                cf32[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b8, a8, cf32[i], fmt, fmt, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += cf[i][0] + (float)ci[i][0];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += (float)ci32[i][0] + cf32[i][0];
    if (s == 123456.789f) sink[0] = s;   // keeps the chains alive; practically never stores (sink holds one float)
}

// The same instructions inside a loop shaped like the contraction kernels' 128-column chunk, without the global
// loads: one barrier, the wave's operand reads from LDS for its 64 x 64 tile (192 bytes per lane for the int8 and
// the fp6 forms: 4-bit weights + 8-bit codes, or 6 + 6 bits; 256 for fp8), the nibble unpack where the form needs
// one, and the chunk's matrix instructions (32 of 16x16x64, 16 of the others).  Every LDS index below is bounded by
// constants (lane < 64, wave coordinates < 2, tile < 4), so the kernel touches nothing but its own 32 KB.
template <int FORM>   // 0 int8 16x16x64 . 1 int8 32x32x32 . 2 fp8 16x16x128 . 4 fp6 16x16x128
__global__ __launch_bounds__(256, 3) void mfma_chunk_kernel(int iters, float *sink)
{
    __shared__ v4i lds[2048];   // 16-byte units: [0, 1024) weight side, [1024, 2048) activation side
    const int tid = threadIdx.x, lane = tid & 63, wm = (tid >> 7) & 1, wn = (tid >> 6) & 1;
    for (int i = tid; i < 2048; i += 256) lds[i] = v4i{i, i * 3, 7, 1};
    v4i acc[4][4];
    v4f accf[4][4];
    v16i acc32[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) { acc[i][j] = v4i{0, 0, 0, 0}; accf[i][j] = v4f{0, 0, 0, 0}; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc32[i >> 1][i & 1][j] = 0;
    const v2i *lds2 = (const v2i *)lds;   // 8-byte units
    for (int it = 0; it < iters; ++it) {
        __syncthreads();
        if (FORM == 0) {
            v4i b[4][2];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int h = 0; h < 2; ++h) b[nt][h] = lds[1024 + ((wn * 4 + nt) * 2 + h) * 64 + lane];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                const v4i w = lds[(wm * 4 + mt) * 64 + lane];
                const v4i lo = (w << 4) & 0xF0F0F0F0, hi = w & 0xF0F0F0F0;
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(lo, b[nt][0], acc[mt][nt], 0, 0, 0);
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(hi, b[nt][1], acc[mt][nt], 0, 0, 0);
                }
            }
        }
        if (FORM == 1) {
            v4i b[2][4], w[4];
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                for (int k = 0; k < 4; ++k) b[nt][k] = lds[1024 + ((wn * 2 + nt) * 4 + k) * 64 + lane];
#pragma unroll
            for (int r = 0; r < 4; ++r) w[r] = lds[(wm * 4 + r) * 64 + lane];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const v4i x = w[mt * 2 + (k & 1)];
                    const v4i a = k < 2 ? ((x << 4) & 0xF0F0F0F0) : (x & 0xF0F0F0F0);
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc32[mt][nt] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[nt][k], acc32[mt][nt], 0, 0, 0);
                }
        }
        if (FORM == 2 || FORM == 4) {
            constexpr int fmt = FORM == 4 ? 2 : 0;
            v8i b[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const v4i x = lds[1024 + (wn * 4 + nt) * 64 + lane];
                if (FORM == 2) {
                    const v4i y = lds[1024 + 512 + (wn * 4 + nt) * 64 + lane];
                    b[nt] = v8i{x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
                } else {
                    const v2i y = lds2[2048 + 1024 + (wn * 4 + nt) * 64 + lane];
                    b[nt] = v8i{x[0], x[1], x[2], x[3], y[0], y[1], 0, 0};
                }
            }
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                const v4i x = lds[(wm * 4 + mt) * 64 + lane];
                v8i a;
                if (FORM == 2) {
                    const v4i y = lds[512 + (wm * 4 + mt) * 64 + lane];
                    a = v8i{x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
                } else {
                    const v2i y = lds2[1024 + (wm * 4 + mt) * 64 + lane];
                    a = v8i{x[0], x[1], x[2], x[3], y[0], y[1], 0, 0};
                }
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    accf[mt][nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b[nt], accf[mt][nt], fmt, fmt, 0, 0x7F7F7F7F, 0,
                                                                                    0x7F7F7F7F);
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) s += (float)acc[i][j][0] + accf[i][j][0];
#pragma unroll
    for (int i = 0; i < 4; ++i) s += (float)acc32[i >> 1][i & 1][0];
    if (s == 123456.789f) sink[0] = s;
}

struct Form {
    const char *name;
    double macs;          // multiply-accumulates of one unit of the loop: a wave-level instruction, or a wave's chunk
    int per_iter;         // units per loop iteration and wave
    int wg_per_cu;        // workgroups launched per compute unit
    void (*launch)(int blocks, int iters, float *sink, hipStream_t st);
};

template <int FORM>
void launch_form(int blocks, int iters, float *sink, hipStream_t st)
{
    mfma_rate_kernel<FORM><<<blocks, 256, 0, st>>>(iters, sink);
}

template <int FORM>
void launch_chunk(int blocks, int iters, float *sink, hipStream_t st)
{
    mfma_chunk_kernel<FORM><<<blocks, 256, 0, st>>>(iters, sink);
}

constexpr double CHUNK_MACS = 64.0 * 64 * 128;   // a wave's 64 x 64 tile over 128 columns
const Form forms[] = {
    {"int8 16x16x64", 16.0 * 16 * 64, 16, 2, launch_form<0>},
    {"int8 32x32x32", 32.0 * 32 * 32, 8, 2, launch_form<1>},
    {"fp8-E4M3 16x16x128", 16.0 * 16 * 128, 16, 2, launch_form<2>},
    {"fp8-E4M3 32x32x64", 32.0 * 32 * 64, 8, 2, launch_form<3>},
    {"fp6-E2M3 16x16x128", 16.0 * 16 * 128, 16, 2, launch_form<4>},
    {"fp6-E3M2 16x16x128", 16.0 * 16 * 128, 16, 2, launch_form<5>},
    {"fp4-E2M1 16x16x128", 16.0 * 16 * 128, 16, 2, launch_form<6>},
    {"chunk loop with LDS operand reads: int8 16x16x64", CHUNK_MACS, 1, 3, launch_chunk<0>},
    {"chunk loop with LDS operand reads: int8 32x32x32", CHUNK_MACS, 1, 3, launch_chunk<1>},
    {"chunk loop with LDS operand reads: fp8-E4M3 16x16x128", CHUNK_MACS, 1, 3, launch_chunk<2>},
    {"chunk loop with LDS operand reads: fp6-E2M3 16x16x128", CHUNK_MACS, 1, 3, launch_chunk<4>},
};
constexpr int N_FORMS = (int)(sizeof(forms) / sizeof(forms[0]));

}  // namespace

extern "C" int32_t qrnnt_diag_mfma_forms(void) { return N_FORMS; }

extern "C" const char *qrnnt_diag_mfma_form_name(int32_t form)
{
    return (form >= 0 && form < N_FORMS) ? forms[form].name : "";
}

extern "C" qrnnt_status qrnnt_diag_mfma_rate(int32_t form, int32_t iters, float *sink, double *tops_out, void *stream)
{
    QR_REQUIRE(sink != nullptr && tops_out != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(form >= 0 && form < N_FORMS, QRNNT_ERR_RANGE);
    QR_REQUIRE(iters >= 1 && iters <= (1 << 22), QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(sink, 4), QRNNT_ERR_ALIGN);
    hipStream_t st = (hipStream_t)stream;
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, qr_current_device()) != hipSuccess || n_cu <= 0)
        return QRNNT_ERR_HIP;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return QRNNT_ERR_HIP;
    }
    const Form &f = forms[form];
    const int blocks = f.wg_per_cu * n_cu;   // 4 waves per workgroup: wg_per_cu waves on every SIMD
    f.launch(blocks, iters < 64 ? iters : 64, sink, st);   // warm-up
    (void)hipEventRecord(e0, st);
    f.launch(blocks, iters, sink, st);
    (void)hipEventRecord(e1, st);
    float ms = 0.0f;
    const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.0f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!ok) return QRNNT_ERR_HIP;
    const double instr = (double)iters * f.per_iter * blocks * 4;   // wave-level instructions
    *tops_out = 2.0 * f.macs * instr / ((double)ms * 1e-3) / 1e12;
    return qr_launch_status();
}
