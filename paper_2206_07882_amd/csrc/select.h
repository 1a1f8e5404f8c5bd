// Wave-level "W best of C candidates" under the total order (value descending,
// index ascending), shared by the beam selection and the end-of-frame pruning.
// Each of the W rounds is an arg-best over the candidates that come strictly after
// the previous pick in that order, so nothing is marked as taken; the wave-wide
// step is two DPP reductions (max of the value key, then min of the index among
// the lanes that hold that value).  After round r lane r holds pick r (index -1,
// value -inf when the candidates ran out).  -inf candidates are never picked.
#pragma once

#include "qrnnt_common.h"

__device__ __forceinline__ bool qr_better(float v, int c, float bv, int bc) { return v > bv || (v == bv && c < bc); }

__device__ __forceinline__ bool qr_select_round(float bv, int bc, int r, int lane, float &last_v, int &last_c, int &my_c,
                                                float &my_v)
{
    const unsigned key = bc != 0x7fffffff ? qr_float_key(bv) : 0u;
    const unsigned gmax = qr_wave_reduce_u32<true>(key);
    if (gmax == 0u) return false;   // uniform: nothing left
    const unsigned gidx = qr_wave_reduce_u32<false>(key == gmax ? (unsigned)bc : 0xFFFFFFFFu);
    last_v = qr_key_float(gmax);
    last_c = (int)gidx;
    if (lane == r) { my_c = last_c; my_v = last_v; }
    return true;
}

// Candidates in registers: lane l owns indices c0 .. c0+PER-1 (val = -inf where absent).
template <int PER>
__device__ __forceinline__ void qr_select_from_regs(const float (&val)[PER], int c0, int W, int lane, int &my_c,
                                                    float &my_v)
{
    float last_v = INFINITY;
    int last_c = -1;
    my_c = -1;
    my_v = -INFINITY;
    for (int r = 0; r < W; ++r) {
        float bv = -INFINITY;
        int bc = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = c0 + i;
            const float v = val[i];
            const bool ok = v > -INFINITY && (v < last_v || (v == last_v && c > last_c));
            if (ok && qr_better(v, c, bv, bc)) { bv = v; bc = c; }
        }
        if (!qr_select_round(bv, bc, r, lane, last_v, last_c, my_c, my_v)) break;
    }
}

// Any size: value(c) re-forms candidate c in every round.
template <class Value>
__device__ __forceinline__ void qr_select_from_mem(Value &&value, int C, int W, int lane, int &my_c, float &my_v)
{
    float last_v = INFINITY;
    int last_c = -1;
    my_c = -1;
    my_v = -INFINITY;
    for (int r = 0; r < W; ++r) {
        float bv = -INFINITY;
        int bc = 0x7fffffff;
        for (int c = lane; c < C; c += 64) {
            const float v = value(c);
            const bool ok = v > -INFINITY && (v < last_v || (v == last_v && c > last_c));
            if (ok && qr_better(v, c, bv, bc)) { bv = v; bc = c; }
        }
        if (!qr_select_round(bv, bc, r, lane, last_v, last_c, my_c, my_v)) break;
    }
}

// Workgroup version (256 threads = 4 waves): thread t owns indices c0 .. c0+PER-1.
// Each round: local best, wave reduction, the four wave results meet in LDS
// (double-buffered by round parity, so one barrier per round).  After round r
// thread r holds pick r.  slots: 2*4*2 unsigned in LDS.
template <int PER>
__device__ __forceinline__ void qr_block_select_from_regs(const float (&val)[PER], int c0, int W, int tid,
                                                          unsigned *slots, int &my_c, float &my_v)
{
    const int lane = tid & 63, wave = tid >> 6;
    float last_v = INFINITY;
    int last_c = -1;
    my_c = -1;
    my_v = -INFINITY;
    for (int r = 0; r < W; ++r) {
        float bv = -INFINITY;
        int bc = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int c = c0 + i;
            const float v = val[i];
            const bool ok = v > -INFINITY && (v < last_v || (v == last_v && c > last_c));
            if (ok && qr_better(v, c, bv, bc)) { bv = v; bc = c; }
        }
        const unsigned key = bc != 0x7fffffff ? qr_float_key(bv) : 0u;
        const unsigned wmax = qr_wave_reduce_u32<true>(key);
        const unsigned widx = qr_wave_reduce_u32<false>(key == wmax ? (unsigned)bc : 0xFFFFFFFFu);
        unsigned *sl = slots + (r & 1) * 8;
        if (lane == 0) { sl[wave * 2] = wmax; sl[wave * 2 + 1] = widx; }
        __syncthreads();
        unsigned gmax = 0u, gidx = 0xFFFFFFFFu;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const unsigned k = sl[wv * 2], ix = sl[wv * 2 + 1];
            if (k > gmax || (k == gmax && ix < gidx)) { gmax = k; gidx = ix; }
        }
        if (gmax == 0u) break;   // uniform across the workgroup
        last_v = qr_key_float(gmax);
        last_c = (int)gidx;
        if (tid == r) { my_c = last_c; my_v = last_v; }
    }
}
