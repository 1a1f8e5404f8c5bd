// Routing of one utterance's W picks inside the decoding loop (Sec. 2: every
// decoding iteration keeps the W best extensions).  Blank picks join the frame's
// candidate list, label picks become the slots of the next round in selection
// order (prefix counts by ballot), the remaining slots die.  Runs in one wave:
// lane r < W holds pick r as (flat candidate index c = parent*V + token, or -1; score v).
#pragma once

#include "kernels.h"
#include "select.h"

// Returns the length of the utterance's candidate list after this round (uniform).
// own_node / own_len: trie node and length of hypothesis `lane` of the current round (fetched at the start of the
// kernel, so that the routing does not wait for memory); a pick reads its parent's from that lane.
// nx0: the length of the utterance's candidate list before this round (a.nx_count[b], fetched early as well).
__device__ __forceinline__ int qr_route_picks(const QrRouteArgs &a, int b, int lane, int c, float v, int own_node,
                                              int own_len, int nx0)
{
    if (lane == 0 && b == 0 && a.live_clear) *a.live_clear = 0;
    if (lane == 0 && b == 0 && a.n_rows_clear) *a.n_rows_clear = 0;
    const int W = a.W, V = a.V, N = a.B * a.W;
    const bool in = lane < W;
    const bool found = in && c >= 0;
    const int par = found ? c / V : 0, tok = found ? c - (c / V) * V : 0;
    const bool is_blank = found && tok == a.blank;
    const bool is_lab = found && tok != a.blank && !a.last_round;
    const unsigned long long bm = __ballot(is_blank), lm = __ballot(is_lab);
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int src_slot = b * W + par;
    const int par_node = __shfl(own_node, par), par_len = __shfl(own_len, par);
    if (is_blank) {
        const int e = nx0 + __popcll(bm & lt);
        a.nx_score[(size_t)b * a.R * W + e] = v;
        a.nx_info[(size_t)b * a.R * W + e] = v4i{a.src_buf * N + src_slot, par_node, par_len, 0};
    }
    const int cnt = nx0 + __popcll(bm);
    if (lane == 0) a.nx_count[b] = cnt;
    if (a.last_round) return cnt;
    const int n_lab = __popcll(lm);
    if (lane == 0 && n_lab > 0 && a.live_next) atomicAdd(a.live_next, 1);
    if (a.rows_next && n_lab > 0) {   // uniform; the order of the utterances in the list does not matter
        int base = 0;
        if (lane == 0) base = atomicAdd(a.n_rows_next, n_lab);
        base = __builtin_amdgcn_readfirstlane(base);
        if (is_lab) a.rows_next[base + (int)__popcll(lm & lt)] = v4i{b * W + (int)__popcll(lm & lt), src_slot, tok, 0};
    }
    if (is_lab) {
        const int dst = b * W + __popcll(lm & lt);
        const int id = a.node_base + dst;
        a.node_tok[id] = tok;
        a.node_prev[id] = par_node;
        a.score_dst[dst] = v;
        a.node_dst[dst] = id;
        a.len_dst[dst] = par_len + 1;
        a.parent_idx[dst] = src_slot;
        a.token[dst] = tok;
        a.active[dst] = 1;
    }
    if (in && lane >= n_lab) {
        const int dst = b * W + lane;
        a.score_dst[dst] = -INFINITY;
        a.node_dst[dst] = 0;
        a.len_dst[dst] = 0;
        a.parent_idx[dst] = dst;
        a.token[dst] = a.blank;
        a.active[dst] = 0;
    }
    return cnt;
}

// End of a frame for utterance b (one wave): the new beam is the W best of the cnt candidates by
// (score descending, insertion order); slot r of buffer fe_dst_buf takes score, trie node and length
// that its candidate carried along, beam_src[r] tells the state copy where the states are.  The candidates of the
// current round were stored by this same wave a moment ago: they are read back from L2 (agent-scope
// loads after a fence), not through the CU's vector cache.
// sk / sc: 64 words of LDS each, private to the calling wave (pruned selection of select.h).
__device__ __forceinline__ void qr_frame_end(const QrRouteArgs &a, int b, int lane, int cnt, unsigned *sk, int *sc_idx)
{
    const int W = a.W, R = a.R, N = a.B * a.W;
    const float *sc = a.nx_score + (size_t)b * R * W;
    auto score_at = [&](int i) { return __hip_atomic_load(sc + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 0.0f; };
    int c;
    float v;
    if (R * W <= 128) {
        float val[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) val[i] = (lane * 2 + i < cnt) ? score_at(lane * 2 + i) : -INFINITY;
        auto index_of = [&](int i) { return lane * 2 + i; };
        if (!qr_select_pruned<2>(val, index_of, W, lane, sk, sc_idx, c, v)) qr_select_from_regs<2>(val, lane * 2, W, lane, c, v);
    } else {
        qr_select_from_mem(score_at, cnt, W, lane, c, v);
    }
    if (lane < W) {
        const int dst = b * W + lane;
        const size_t o = (size_t)a.fe_dst_buf * N + dst;
        if (c >= 0) {
            // what the candidate carried along when it joined the list: three independent loads, no second hop
            const int *info = (const int *)(a.nx_info + (size_t)b * R * W + c);
            const int src = __hip_atomic_load(info, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int node = __hip_atomic_load(info + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int len = __hip_atomic_load(info + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            a.fe_score_all[o] = v;
            a.fe_node_all_w[o] = node;
            a.fe_len_all_w[o] = len;
            a.beam_src[dst] = src;
        } else {
            a.fe_score_all[o] = -INFINITY;
            a.fe_node_all_w[o] = 0;
            a.fe_len_all_w[o] = 0;
            a.beam_src[dst] = -1;
        }
    }
    if (lane == 0) a.nx_count[b] = 0;
}

// One iteration of the alignment-length synchronous search for utterance b (one wave; Sec. 2 names the search,
// the algorithm is the published one).  Lane r < W holds pick r (flat candidate index c = parent*V + token or -1,
// score v) and, as fin_new, the score with which hypothesis r of the current beam finishes now (-inf: it does not).
//   - pick r becomes slot r of the next beam: a blank keeps the parent's sequence and state (the network
//     advance copies inactive rows through), a label extends it;
//   - recombination: picks that stand for the same label sequence (same length and same 64-bit sequence hash)
//     are one hypothesis; the best-ranked keeps its slot with log(sum exp(scores)), the others die;
//   - the running list of the W best finished hypotheses takes the new ones in, ordered by (score descending,
//     insertion order), new ones in slot order.
// What lane w < W of the routing wave knows about hypothesis w of the current beam and rank w of the finished
// list: fetched at the start of the kernel, so that nothing in the routing waits for memory.
struct QrAlsdOwn {
    int len, node;
    unsigned long long hash;
    float score;
    float fin_score;  int fin_node, fin_len;
};

__device__ __forceinline__ QrAlsdOwn qr_alsd_load_own(const QrRouteArgs &a, const QrAlsdArgs &s, int b, int lane)
{
    const int own = b * a.W + (lane < a.W ? lane : 0);
    QrAlsdOwn o;
    o.len = a.len_src[own];  o.node = a.node_src[own];  o.hash = s.hash_src[own];  o.score = a.score_src[own];
    o.fin_score = s.fin_score[own];  o.fin_node = s.fin_node[own];  o.fin_len = s.fin_len[own];
    return o;
}

__device__ __forceinline__ void qr_alsd_route(const QrRouteArgs &a, const QrAlsdArgs &s, int b, int lane, int c, float v,
                                              float fin_new, const QrAlsdOwn &o)
{
    const int W = a.W, V = a.V;
    const bool in = lane < W;
    const bool found = in && c >= 0;
    const int par = found ? c / V : 0, tok = found ? c - (c / V) * V : a.blank;
    const bool is_lab = found && tok != a.blank;
    const int src_slot = b * W + par;
    const int own = b * W + (in ? lane : 0);
    // the parent's sequence, taken from the lane that holds it
    const int len_p = __shfl(o.len, par);
    const int node_p = __shfl(o.node, par);
    const unsigned long long hash_p = ((unsigned long long)(unsigned)__shfl((int)(unsigned)(o.hash >> 32), par) << 32) |
                                      (unsigned long long)(unsigned)__shfl((int)(unsigned)o.hash, par);
    const int own_node = o.node, own_len = o.len;
    const int new_len = len_p + (is_lab ? 1 : 0);
    const unsigned long long new_hash = is_lab ? hash_p * 0x9E3779B97F4A7C15ull + (unsigned long long)(tok + 1) : hash_p;
    const int h_lo = (int)(unsigned)new_hash, h_hi = (int)(unsigned)(new_hash >> 32);
    // length and "is a pick" in one word: a lane without a pick gets a value no other lane has
    const int lw = found ? new_len : -1 - lane;
    int leader = lane;
    float m = v;
    unsigned long long eq = 0ull;   // the picks that stand for this lane's label sequence
    for (int j = 0; j < W; ++j) {
        const bool same = __builtin_amdgcn_readlane(lw, j) == lw && __builtin_amdgcn_readlane(h_lo, j) == h_lo &&
                          __builtin_amdgcn_readlane(h_hi, j) == h_hi;
        const float vj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), j));
        if (same) {
            eq |= 1ull << j;
            leader = j < leader ? j : leader;
            m = fmaxf(m, vj);
        }
    }
    float sum = 0.0f;
    for (int j = 0; j < W; ++j) {
        const float vj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), j));
        if ((eq >> j) & 1ull) sum += qr_exp(vj - m);
    }
    const bool keep = found && leader == lane;
    const unsigned long long km = __ballot(keep);
    if (lane == 0 && km != 0ull && a.live_next) atomicAdd(a.live_next, 1);
    // Reuse of cached hypotheses (Sec. 4.1): the networks' states after a label sequence depend on the sequence
    // alone.  When a live hypothesis of the current beam already holds the sequence this label pick produces (the
    // usual case: y + k is in the beam and y proposes k again one frame later), the new slot takes over that
    // hypothesis' states as an inactive row of the advance instead of stepping the networks from y.
    int reuse_slot = -1;
    if (s.reuse) {   // uniform
        const int o_hlo = (int)(unsigned)o.hash, o_hhi = (int)(unsigned)(o.hash >> 32);
        for (int j = 0; j < W; ++j) {
            const bool live_j = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(o.score), j)) > -INFINITY;
            const bool same = live_j && __builtin_amdgcn_readlane(o.len, j) == new_len &&
                              __builtin_amdgcn_readlane(o_hlo, j) == h_lo && __builtin_amdgcn_readlane(o_hhi, j) == h_hi;
            if (same && keep && is_lab && reuse_slot < 0) reuse_slot = j;
        }
    }
    if (s.stats) {   // uniform
        const int n_req = (int)__popcll(__ballot(keep && is_lab)), n_hit = (int)__popcll(__ballot(reuse_slot >= 0));
        if (lane == 0 && n_req) atomicAdd(s.stats, n_req);
        if (lane == 0 && n_hit) atomicAdd(s.stats + 1, n_hit);
    }
    if (in) {
        const int dst = b * W + lane;
        if (keep) {
            int node = node_p;
            if (is_lab) {
                node = a.node_base + dst;
                a.node_tok[node] = tok;
                a.node_prev[node] = node_p;
            }
            a.score_dst[dst] = m + qr_log(sum);
            a.node_dst[dst] = node;
            a.len_dst[dst] = new_len;
            s.hash_dst[dst] = new_hash;
            a.parent_idx[dst] = reuse_slot >= 0 ? b * W + reuse_slot : src_slot;
            a.token[dst] = tok;
            a.active[dst] = (is_lab && reuse_slot < 0) ? 1 : 0;
        } else {
            a.score_dst[dst] = -INFINITY;
            a.node_dst[dst] = 0;
            a.len_dst[dst] = 0;
            s.hash_dst[dst] = 0ull;
            a.parent_idx[dst] = dst;
            a.token[dst] = a.blank;
            a.active[dst] = 0;
        }
    }
    // finished hypotheses
    const float fn = in ? fin_new : -INFINITY;
    if (__ballot(fn > -INFINITY) == 0ull) return;   // uniform
    const float fo = in ? o.fin_score : -INFINITY;
    const int fo_node = o.fin_node, fo_len = o.fin_len;
    int rank_o = 0, rank_n = 0;
    for (int j = 0; j < W; ++j) {
        const float oj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fo), j));
        const float nj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(fn), j));
        rank_o += ((oj > fo) || (oj == fo && j < lane)) ? 1 : 0;
        rank_o += (nj > fo) ? 1 : 0;
        rank_n += (oj >= fn) ? 1 : 0;
        rank_n += ((nj > fn) || (nj == fn && j < lane)) ? 1 : 0;
    }
    if (in && rank_o < W) {
        const int o = b * W + rank_o;
        s.fin_score[o] = fo;  s.fin_node[o] = fo_node;  s.fin_len[o] = fo_len;
    }
    if (in && rank_n < W) {
        const int o = b * W + rank_n;
        s.fin_score[o] = fn;  s.fin_node[o] = fn > -INFINITY ? own_node : 0;  s.fin_len[o] = fn > -INFINITY ? own_len : 0;
    }
}
