// Beam selection: per utterance the W best (parent, token) extensions (Sec. 2:
// the beam width is the number of hypotheses kept per decoding iteration).
// Selection runs on the GPU so that the decoding loop never returns to the host.
#include "kernels.h"

namespace {

// Total order: larger value first, then smaller flat index.
__device__ __forceinline__ bool better(float v, int c, float bv, int bc) { return v > bv || (v == bv && c < bc); }

// One wave per utterance; W rounds, each an arg-best over the W*V candidates
// that come strictly after the previous pick in the total order, so nothing has
// to be marked as taken.
__global__ __launch_bounds__(64) void beam_step_kernel(const float *__restrict__ score, const float *__restrict__ fused,
                                                        int W, int V, int blank, int force_blank,
                                                        int32_t *__restrict__ parent_out, int32_t *__restrict__ token_out,
                                                        float *__restrict__ score_out)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int C = W * V;
    const float *sc = score + (int64_t)b * W;
    const float *fu = fused + (int64_t)b * W * V;
    float last_v = INFINITY;
    int last_c = -1;
    for (int r = 0; r < W; ++r) {
        float bv = -INFINITY;
        int bc = 0x7fffffff;
        if (last_c != -2) {
            for (int c = lane; c < C; c += 64) {
                const int w = c / V, k = c - w * V;
                if (force_blank && k != blank) continue;
                const float v = sc[w] + fu[c];
                if (!(v > -INFINITY)) continue;
                const bool after = v < last_v || (v == last_v && c > last_c);
                if (after && better(v, c, bv, bc)) { bv = v; bc = c; }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const float ov = __shfl_xor(bv, off);
                const int oc = __shfl_xor(bc, off);
                if (better(ov, oc, bv, bc)) { bv = ov; bc = oc; }
            }
        }
        const bool found = bc != 0x7fffffff;
        if (lane == 0) {
            parent_out[(int64_t)b * W + r] = found ? bc / V : -1;
            token_out[(int64_t)b * W + r] = found ? bc % V : -1;
            score_out[(int64_t)b * W + r] = found ? bv : -INFINITY;
        }
        if (found) { last_v = bv; last_c = bc; } else { last_c = -2; }   // exhausted: remaining ranks stay empty
    }
}

}  // namespace

void qr_launch_beam(const float *score, const float *fused, int B, int W, int V, int blank, int force_blank,
                    int32_t *parent_out, int32_t *token_out, float *score_out, hipStream_t st)
{
    beam_step_kernel<<<B, 64, 0, st>>>(score, fused, W, V, blank, force_blank, parent_out, token_out, score_out);
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
