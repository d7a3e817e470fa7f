// The walker (Sec. 3.2 "Walk Sampling"; Algorithm 1, walk step): one lane moves one walk of
// m steps.  Shared by the stand-alone walk kernel and the fused walk + RPE kernel.
#pragma once

#include "device_util.h"

namespace surel {

// The graph as a walker sees it: the CSR, and optionally the per-edge neighbour records
// rec[e] = (col_idx[e], row start of that neighbour, its degree, 0), id -1 for an entry that
// names no node or whose row is malformed.
struct WalkGraph {
    const int32_t* __restrict__ row_ptr;
    const int32_t* __restrict__ col_idx;
    const int4* __restrict__ rec;
    int32_t n_nodes;
    int64_t n_edges;
};

// Row of the seed (wave-uniform loads); a malformed row counts as degree 0.
__device__ __forceinline__ bool seed_row(const WalkGraph& g, int32_t u, int32_t* lo, int32_t* deg) {
    const int32_t a = g.row_ptr[u];
    const int32_t d = g.row_ptr[u + 1] - a;
    const bool bad = a < 0 || d < 0 || (int64_t)a + d > g.n_edges;
    *lo = a;
    *deg = bad ? 0 : d;
    return bad;
}

// C walks of seed u per lane, moved in lock step so that a lane has C independent gathers in
// flight (the walk is bound by memory latency).  Walk c is number w[c], takes part if
// active[c], writes positions 0..m into row[c][0..m] (LDS rows of the lane's own) and calls
// visit(c, node) after every step.  Inactive walks still write a row (all u) that the caller
// ignores.  Step s uses word (s-1)&3 of Philox(counter (u, w, (s-1)>>2, 0), key).
// Returns true if a malformed CSR row or a neighbour id outside the graph was met (the
// walker then stays in place for that step).
template <bool kRec, int C, typename Visit>
__device__ __forceinline__ bool walk_many(const WalkGraph& g, int32_t u, int32_t u_lo, int32_t u_deg,
                                          const int (&w)[C], const bool (&active)[C], int m,
                                          uint32_t key0, uint32_t key1, int32_t* const (&row)[C],
                                          Visit&& visit) {
    bool bad_graph = false;
    int32_t cur[C], cur_lo[C], cur_deg[C];  // cur_lo / cur_deg: row of `cur` (kRec only)
#pragma unroll
    for (int c = 0; c < C; ++c) {
        cur[c] = u;
        cur_lo[c] = u_lo;
        cur_deg[c] = u_deg;
        row[c][0] = u;
    }
    for (int s0 = 1; s0 <= m; s0 += 4) {
        uint32_t r[C][4];
#pragma unroll
        for (int c = 0; c < C; ++c)
            philox4x32_10((uint32_t)u, (uint32_t)w[c], (uint32_t)((s0 - 1) >> 2), 0u, key0, key1,
                          r[c]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = s0 + j;
            if (s <= m) {
                if (kRec) {
                    int4 nb[C];
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        const bool go = active[c] && cur_deg[c] > 0;
                        const uint32_t pick = go ? r[c][j] % (uint32_t)cur_deg[c] : 0u;
                        nb[c] = make_int4(cur[c], cur_lo[c], cur_deg[c], 0);
                        if (go) nb[c] = g.rec[(int64_t)cur_lo[c] + (int64_t)pick];
                    }
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        if (nb[c].x < 0) {
                            bad_graph = true;
                        } else {
                            cur[c] = nb[c].x;
                            cur_lo[c] = nb[c].y;
                            cur_deg[c] = nb[c].z;
                        }
                    }
                } else {
                    int32_t lo[C], hi[C];
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        lo[c] = 0;
                        hi[c] = 0;
                        if (active[c]) {
                            lo[c] = g.row_ptr[cur[c]];
                            hi[c] = g.row_ptr[cur[c] + 1];
                        }
                    }
                    int32_t nxt[C];
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        nxt[c] = cur[c];
                        if (lo[c] < 0 || hi[c] < lo[c] || (int64_t)hi[c] > g.n_edges) {
                            bad_graph = true;
                        } else if (hi[c] > lo[c]) {
                            const uint32_t deg = (uint32_t)(hi[c] - lo[c]);
                            nxt[c] = g.col_idx[(int64_t)lo[c] + (int64_t)(r[c][j] % deg)];
                        }
                    }
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        if ((uint32_t)nxt[c] >= (uint32_t)g.n_nodes) {
                            bad_graph = true;
                        } else {
                            cur[c] = nxt[c];
                        }
                    }
                }
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    row[c][s] = cur[c];
                    visit(c, cur[c]);
                }
            }
        }
    }
    return bad_graph;
}

}  // namespace surel
