// Beam selection: per utterance the W best (parent, token) extensions (Sec. 2:
// the beam width is the number of hypotheses kept per decoding iteration).
// Selection runs on the GPU so that the decoding loop never returns to the host.
#include "kernels.h"
#include "select.h"

namespace {

// One workgroup (4 waves) per utterance.  The W*V candidate values are formed once
// (fp32 add) and kept in registers; see select.h.
template <int PER>
__device__ __forceinline__ void select_w_regs(const float *__restrict__ sc, const float *__restrict__ fu, int W, int V,
                                              int blank, int force_blank, int tid, unsigned *slots, int &my_c, float &my_v)
{
    const int C = W * V;
    float val[PER];
    const int c0 = tid * PER;
    int w = c0 / V, k = c0 - w * V;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int c = c0 + i;
        float v = -INFINITY;
        if (c < C && (!force_blank || k == blank)) v = (sc[w] + fu[c]) + 0.0f;   // + 0: -0 becomes +0, one key per value
        val[i] = v;
        if (++k == V) { k = 0; ++w; }
    }
    qr_block_select_from_regs<PER>(val, c0, W, tid, slots, my_c, my_v);
}

// Up to 64 * PER candidates held by one wave, lane l owning indices l*PER .. l*PER+PER-1: the pruned
// rank-based selection of select.h.  Returns false when more than 64 candidates survive its threshold.
template <int PER>
__device__ __forceinline__ bool select_w_pruned(const float *__restrict__ sc, const float *__restrict__ fu, int W, int V,
                                                int blank, int force_blank, int lane, unsigned *scratch, int &my_c,
                                                float &my_v)
{
    const int C = W * V;
    float val[PER];
    const int c0 = lane * PER;
    int w = c0 / V, k = c0 - w * V;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int c = c0 + i;
        float v = -INFINITY;
        if (c < C && (!force_blank || k == blank)) v = (sc[w] + fu[c]) + 0.0f;   // + 0: -0 becomes +0, one key per value
        val[i] = v;
        if (++k == V) { k = 0; ++w; }
    }
    auto index_of = [&](int s) { return c0 + s; };
    return qr_select_pruned<PER>(val, index_of, W, lane, scratch, (int *)scratch + 64, my_c, my_v);
}

// Thread r < W ends up with pick r.  Uniform control flow across the workgroup.
__device__ __forceinline__ void select_w(const float *__restrict__ sc, const float *__restrict__ fu, int W, int V,
                                         int blank, int force_blank, int tid, unsigned *slots, int &my_c, float &my_v)
{
    const int C = W * V;   // uniform
    // fast path: wave 0 alone, candidates in its registers (the other waves only meet it at the barrier)
    __shared__ unsigned pruned_scratch[128];
    __shared__ int pruned_ok;
    if (C <= 64 * 16) {
        if (tid < 64) {
            const bool ok = C <= 64 * 4 ? select_w_pruned<4>(sc, fu, W, V, blank, force_blank, tid, pruned_scratch, my_c, my_v)
                                         : select_w_pruned<16>(sc, fu, W, V, blank, force_blank, tid, pruned_scratch, my_c, my_v);
            if (tid == 0) pruned_ok = ok ? 1 : 0;
        }
        __syncthreads();
        if (pruned_ok) return;   // uniform
    }
    if (C <= 256) select_w_regs<1>(sc, fu, W, V, blank, force_blank, tid, slots, my_c, my_v);
    else if (C <= 256 * 3) select_w_regs<3>(sc, fu, W, V, blank, force_blank, tid, slots, my_c, my_v);
    else if (C <= 256 * 6) select_w_regs<6>(sc, fu, W, V, blank, force_blank, tid, slots, my_c, my_v);
    else {
        my_c = -1;
        my_v = -INFINITY;
        if (tid < 64) {   // any size: wave 0 re-forms the candidates from memory in every round
            auto value = [&](int c) -> float {
                const int w = c / V, k = c - w * V;
                return (force_blank && k != blank) ? -INFINITY : (sc[w] + fu[c]) + 0.0f;
            };
            qr_select_from_mem(value, C, W, tid, my_c, my_v);
        }
    }
}

__global__ __launch_bounds__(256) void beam_step_kernel(const float *__restrict__ score, const float *__restrict__ fused,
                                                         int W, int V, int blank, int force_blank,
                                                         int32_t *__restrict__ parent_out, int32_t *__restrict__ token_out,
                                                         float *__restrict__ score_out)
{
    __shared__ unsigned slots[16];
    const int b = blockIdx.x, tid = threadIdx.x;
    int c;
    float v;
    select_w(score + (int64_t)b * W, fused + (int64_t)b * W * V, W, V, blank, force_blank, tid, slots, c, v);
    if (tid < W) {
        parent_out[(int64_t)b * W + tid] = c >= 0 ? c / V : -1;
        token_out[(int64_t)b * W + tid] = c >= 0 ? c % V : -1;
        score_out[(int64_t)b * W + tid] = v;
    }
}

}  // namespace

void qr_launch_beam(const float *score, const float *fused, int B, int W, int V, int blank, int force_blank,
                    int32_t *parent_out, int32_t *token_out, float *score_out, hipStream_t st)
{
    beam_step_kernel<<<B, 256, 0, st>>>(score, fused, W, V, blank, force_blank, parent_out, token_out, score_out);
}

extern "C" qrnnt_status qrnnt_beam_step(const float *score, const float *fused, int32_t B, int32_t W, int32_t V,
                                        int32_t blank, int32_t force_blank, int32_t *parent_out, int32_t *token_out,
                                        float *score_out, void *stream)
{
    QR_REQUIRE(score && fused && parent_out && token_out && score_out, QRNNT_ERR_NULL);
    QR_REQUIRE(B > 0 && W > 0 && V > 0, QRNNT_ERR_SHAPE);
    QR_REQUIRE(W <= 64, QRNNT_ERR_UNSUPPORTED);
    QR_REQUIRE(blank >= 0 && blank < V, QRNNT_ERR_RANGE);
    qr_launch_beam(score, fused, B, W, V, blank, force_blank, parent_out, token_out, score_out, (hipStream_t)stream);
    return qr_launch_status();
}
