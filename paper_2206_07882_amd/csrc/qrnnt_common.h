// Internal helpers shared by the HIP translation units of libqrnnt (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qrnnt.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

#define QRNNT_WAVE 64
#define QRNNT_KCHUNK 128        // columns covered by one 1 KiB tiled block
#define QRNNT_BLOCK_BYTES 1024  // 16 rows x 128 nibbles

__host__ __device__ static inline int qr_round_up(int a, int b) { return (a + b - 1) / b * b; }

// TILED_GATES row order.  Tiled row 16*rt + 4*grp + gate holds gate `gate` of cell
// 16*(rt/4) + 4*grp + rt%4: an MFMA output lane (grp, col) of row tile rt receives the
// four gate sums of that cell, and over the 4 row tiles of a 64-row group the lane
// owns 4 consecutive cells (16 bytes of cell state, 4 bytes of hidden codes).
__host__ __device__ static inline int qr_gates_cell(int rt, int grp) { return ((rt >> 2) << 4) + (grp << 2) + (rt & 3); }
__host__ __device__ static inline int qr_gates_tiled_row(int cell, int gate)
{
    return ((((cell >> 4) << 2) + (cell & 3)) << 4) + (((cell >> 2) & 3) << 2) + gate;
}
static inline bool qr_aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Row pitch in bytes of an activation-code matrix with `cols` columns: rows start on 16-byte boundaries, the
// columns behind `cols` are padding that may hold anything (it meets the zero padding of the packed weights).
__host__ __device__ static inline int qr_act_pitch(int cols) { return qr_round_up(cols, 16); }

// What the launchers cache about a device (compute units, occupancy of a kernel, "attribute already set") is kept
// per device, indexed by the device that is current on the calling thread.
#define QR_MAX_DEVICES 64
static inline int qr_current_device()
{
    int d = 0;
    if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= QR_MAX_DEVICES) d = 0;
    return d;
}

#define QR_REQUIRE(cond, err) \
    do {                      \
        if (!(cond)) return (err); \
    } while (0)

static inline qrnnt_status qr_launch_status() { return hipGetLastError() == hipSuccess ? QRNNT_OK : QRNNT_ERR_HIP; }

// Host-side validation of a packed-matrix descriptor used by a compute kernel.
static inline qrnnt_status qr_check_qmat(const qrnnt_qmat *m, int want_layout)
{
    QR_REQUIRE(m != nullptr && m->packed != nullptr && m->row_scale != nullptr, QRNNT_ERR_NULL);
    QR_REQUIRE(m->rows > 0 && m->cols > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(m->layout == want_layout, QRNNT_ERR_LAYOUT);
    QR_REQUIRE(m->bits == 0 || m->bits == 4 || m->bits == 8, QRNNT_ERR_RANGE);
    QR_REQUIRE(qr_aligned(m->packed, 16), QRNNT_ERR_ALIGN);
    return QRNNT_OK;
}

#ifdef __HIPCC__

// Splits one 128-bit packed fragment into two int8x16 MFMA operands.  Each
// nibble is moved to the top half of its byte, i.e. the operand holds 16*w as a
// signed int8 with no sign-extension work; accumulators therefore hold 16*acc
// and are shifted right by 4 (exact) once per tile.
__device__ __forceinline__ void qr_unpack(v4i p, v4i &lo, v4i &hi)
{
    const int m = (int)0xF0F0F0F0u;
    hi = p & m;
    lo = (p << 4) & m;
}

// D[16 x 16] += A[16 x 64] * B[64 x 16], int8 in, int32 out.  Lane l supplies
// row l%16 of A and column l%16 of B for the 16-wide K slice l/16, and receives
// D[4*(l/16) + i][l%16] in element i of the result.
__device__ __forceinline__ v4i qr_mfma(v4i a, v4i b, v4i c)
{
    return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// sigmoid and tanh on the hardware exp2 / reciprocal units (about 1 ulp each):
// relative error of sigmoid <= ~|v| * 1e-7 + 3e-7, absolute error of tanh <= ~3e-7,
// far inside the 1e-5 / 1e-6 parity bars, at a tenth of the libm instruction count.
__device__ __forceinline__ float qr_sigmoid(float v)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896f * v));
}
__device__ __forceinline__ float qr_tanh(float v)
{
    return 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-2.885390081777927f * v)) - 1.0f;
}
// sigmoid(v) given u = -log2(e) * v (the constant folded into whatever produced u)
__device__ __forceinline__ float qr_sigmoid_scaled(float u) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(u)); }

// exp and log on the hardware exp2 / log2 units (about 1 ulp each), for the log-softmax epilogues
__device__ __forceinline__ float qr_exp(float v) { return __builtin_amdgcn_exp2f(1.4426950408889634f * v); }
__device__ __forceinline__ float qr_log(float v) { return 0.6931471805599453f * __builtin_amdgcn_logf(v); }

// Symmetric 4-bit quantizer: clamp(rne(x * inv_step)), product in fp32.
__device__ __forceinline__ int qr_quant4(float x, float inv_step)
{
    float t = x * inv_step;
    float r = __builtin_rintf(t);
    r = fminf(fmaxf(r, -8.0f), 7.0f);
    return (int)r;
}

// The same quantizer at 4 or 8 bits: clamp to [-2^(bits-1), 2^(bits-1) - 1].
__device__ __forceinline__ int qr_quant(float x, float inv_step, int bits)
{
    const float hi = bits == 8 ? 127.0f : 7.0f;
    float r = __builtin_rintf(x * inv_step);
    r = fminf(fmaxf(r, -hi - 1.0f), hi);
    return (int)r;
}

// bits field of a qrnnt_qmat: 0 is read as 4.
static inline int qr_bits(const qrnnt_qmat *m) { return m->bits == 8 ? 8 : 4; }

// Wave-wide max / min of a 32-bit unsigned value on the DPP path (row scans, then
// the two cross-row broadcasts of gfx9), result broadcast through lane 63.
template <bool IS_MAX>
__device__ __forceinline__ unsigned qr_wave_reduce_u32(unsigned v)
{
    const unsigned id = IS_MAX ? 0u : 0xFFFFFFFFu;
#define QR_DPP_STEP(ctrl, rmask)                                                                       \
    {                                                                                                  \
        const unsigned o = (unsigned)__builtin_amdgcn_update_dpp((int)id, (int)v, ctrl, rmask, 0xf, false); \
        v = IS_MAX ? (v > o ? v : o) : (v < o ? v : o);                                                \
    }
    QR_DPP_STEP(0x111, 0xf)   // row_shr:1
    QR_DPP_STEP(0x112, 0xf)   // row_shr:2
    QR_DPP_STEP(0x114, 0xf)   // row_shr:4
    QR_DPP_STEP(0x118, 0xf)   // row_shr:8
    QR_DPP_STEP(0x142, 0xa)   // row_bcast:15 into rows 1 and 3
    QR_DPP_STEP(0x143, 0xc)   // row_bcast:31 into rows 2 and 3
#undef QR_DPP_STEP
    return (unsigned)__builtin_amdgcn_readlane((int)v, 63);
}

// Monotone map fp32 -> uint32 (larger float <=> larger unsigned); never returns 0 for a non-NaN input.
__device__ __forceinline__ unsigned qr_float_key(float f)
{
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float qr_key_float(unsigned k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

#endif  // __HIPCC__
