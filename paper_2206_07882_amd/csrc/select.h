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

// Pruned selection for one wave holding PER candidate slots per lane (slot s of a
// lane has flat index index_of(s), increasing with s; val = -inf where absent).
//   1. each lane's best key; the W-th largest of those 64 keys, found by bisection
//      over the key bits with one ballot per bit, is a lower bound T of the W-th best
//      candidate (W lanes hold a candidate >= T);
//   2. the candidates >= T are compacted into LDS (ballot prefix counts);
//   3. if at most 64 survive, lane l takes survivor l and counts the survivors that
//      precede it in the total order: that count is its rank, rank r < W is pick r.
// Cost: a few hundred instructions instead of W dependent wave reductions over all
// slots.  Returns false (nothing written) when more than 64 candidates survive, e.g.
// fewer than W lanes hold anything: the caller then runs the round-by-round selection.
// After a true return lane r < W holds pick r (index -1, value -inf if none).
// sk / sc: 64 words of LDS each, private to the calling wave.
template <int PER, class IndexOf>
__device__ __forceinline__ bool qr_select_pruned(const float (&val)[PER], IndexOf &&index_of, int W, int lane,
                                                 unsigned *sk, int *sc, int &my_c, float &my_v)
{
    unsigned key[PER];
    unsigned lmax = 0u;
#pragma unroll
    for (int s = 0; s < PER; ++s) {
        key[s] = val[s] > -INFINITY ? qr_float_key(val[s]) : 0u;
        lmax = key[s] > lmax ? key[s] : lmax;
    }
    unsigned T = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const unsigned trial = T | (1u << bit);
        if (__popcll(__ballot(lmax >= trial)) >= W) T = trial;   // uniform
    }
    T = T ? T : 1u;   // fewer than W lanes hold a candidate: every candidate survives
    int M = 0;
#pragma unroll
    for (int s = 0; s < PER; ++s) M += __popcll(__ballot(key[s] >= T));
    if (M > 64) return false;
    int base = 0;
#pragma unroll
    for (int s = 0; s < PER; ++s) {
        const bool keep = key[s] >= T;
        const unsigned long long mk = __ballot(keep);
        const int pos = base + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(mk >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mk, 0u));
        if (keep) { sk[pos] = key[s]; sc[pos] = index_of(s); }
        base += __popcll(mk);
    }
    __builtin_amdgcn_wave_barrier();
    const unsigned k = lane < M ? sk[lane] : 0u;
    const int c = lane < M ? sc[lane] : 0x7fffffff;
    int rank = 0;
    for (int j = 0; j < M; ++j) {
        const unsigned kj = (unsigned)__builtin_amdgcn_readlane((int)k, j);
        const int cj = __builtin_amdgcn_readlane(c, j);
        rank += (kj > k || (kj == k && cj < c)) ? 1 : 0;
    }
    __builtin_amdgcn_wave_barrier();
    sk[lane] = 0u;
    sc[lane] = -1;
    __builtin_amdgcn_wave_barrier();
    if (lane < M && rank < 64) { sk[rank] = k; sc[rank] = c; }
    __builtin_amdgcn_wave_barrier();
    const unsigned pk = sk[lane];
    const int pc = sc[lane];
    my_c = (lane < W) ? pc : -1;
    my_v = (lane < W && pc >= 0) ? qr_key_float(pk) : -INFINITY;
    return true;
}
