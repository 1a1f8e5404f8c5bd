// Routing of one utterance's W picks inside the decoding loop (Sec. 2: every
// decoding iteration keeps the W best extensions).  Blank picks join the frame's
// candidate list, label picks become the slots of the next round in selection
// order (prefix counts by ballot), the remaining slots die.  Runs in one wave:
// lane r < W holds pick r as (flat candidate index c = parent*V + token, or -1; score v).
#pragma once

#include "kernels.h"

__device__ __forceinline__ void qr_route_picks(const QrRouteArgs &a, int b, int lane, int c, float v)
{
    const int W = a.W, V = a.V, N = a.B * a.W;
    const bool in = lane < W;
    const bool found = in && c >= 0;
    const int par = found ? c / V : 0, tok = found ? c - (c / V) * V : 0;
    const bool is_blank = found && tok == a.blank;
    const bool is_lab = found && tok != a.blank && !a.last_round;
    const unsigned long long bm = __ballot(is_blank), lm = __ballot(is_lab);
    const unsigned long long lt = (1ull << lane) - 1ull;
    const int src_slot = b * W + par;
    const int nx0 = a.nx_count[b];
    if (is_blank) {
        const int e = nx0 + __popcll(bm & lt);
        a.nx_score[(size_t)b * a.R * W + e] = v;
        a.nx_src[(size_t)b * a.R * W + e] = a.src_buf * N + src_slot;
    }
    if (lane == 0) a.nx_count[b] = nx0 + __popcll(bm);
    if (a.last_round) return;
    const int n_lab = __popcll(lm);
    if (is_lab) {
        const int dst = b * W + __popcll(lm & lt);
        const int id = a.node_base + dst;
        a.node_tok[id] = tok;
        a.node_prev[id] = a.node_src[src_slot];
        a.score_dst[dst] = v;
        a.node_dst[dst] = id;
        a.len_dst[dst] = a.len_src[src_slot] + 1;
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
}
