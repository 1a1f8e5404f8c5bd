// Diagnostics: issue rates of the matrix instructions that could carry the W4A4 contraction on gfx950, measured
// in registers (no memory traffic in the loop).  Codes in [-8, 7] are exact in int8, fp8-E4M3 and fp6-E3M2 (and
// [-7, 7] in fp6-E2M3), and sums of up to 2048 products stay below 2^24, so these forms would give the same
// integers (Sec. 3.1 / 3.2: the method only fixes the integer grid, not the unit that multiplies); fp4-E2M1 lacks
// 5 and 7 and is listed for its rate only.  Which form to build on is a question of rate and of operand layout.  bench.py reports these rates next to the kernels' achieved ones.
#include "qrnnt_common.h"

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

// 8 accumulator chains of the 16 x 16 forms (4 of the 32 x 32 forms) per wave.  Every chain gets two instructions
// per loop iteration (operands swapped for the second), the pattern of the contraction kernels, whose 128-column
// chunk is two K steps into one accumulator; the compiler keeps such a loop free of register moves, so the loop
// body is the matrix instructions and the branch (a body with one instruction per chain and iteration made it
// shuffle the accumulators between the instructions, which halved the measured rate of the 4-pass forms).
template <int FORM>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float *sink)
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

struct Form {
    const char *name;
    double macs;          // multiply-accumulates of one wave-level instruction
    int per_iter;         // instructions per loop iteration
    void (*launch)(int blocks, int iters, float *sink, hipStream_t st);
};

template <int FORM>
void launch_form(int blocks, int iters, float *sink, hipStream_t st)
{
    mfma_rate_kernel<FORM><<<blocks, 256, 0, st>>>(iters, sink);
}

const Form forms[] = {
    {"int8 16x16x64", 16.0 * 16 * 64, 16, launch_form<0>},      {"int8 32x32x32", 32.0 * 32 * 32, 8, launch_form<1>},
    {"fp8-E4M3 16x16x128", 16.0 * 16 * 128, 16, launch_form<2>}, {"fp8-E4M3 32x32x64", 32.0 * 32 * 64, 8, launch_form<3>},
    {"fp6-E2M3 16x16x128", 16.0 * 16 * 128, 16, launch_form<4>}, {"fp6-E3M2 16x16x128", 16.0 * 16 * 128, 16, launch_form<5>},
    {"fp4-E2M1 16x16x128", 16.0 * 16 * 128, 16, launch_form<6>},
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
    const int blocks = 2 * n_cu;   // 4 waves per workgroup: two waves on every SIMD
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return QRNNT_ERR_HIP;
    }
    const Form &f = forms[form];
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
