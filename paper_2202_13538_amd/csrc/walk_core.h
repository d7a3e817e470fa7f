// The walker (Sec. 3.2 "Walk Sampling"; Algorithm 1, walk step): one lane moves one walk of
// m steps.  Shared by the stand-alone walk kernel and the fused walk + RPE kernel.
#pragma once

#include "device_util.h"

namespace surel {

// Per-edge neighbour records: one record per CSR entry e with the neighbour col_idx[e], the start
// of that neighbour's row and its degree, so that a step is one gather instead of two dependent
// ones.  Two layouts:
//   kRecWide    int4 (id, row start, degree, 0); id -1 for an entry that names no node or whose
//               row is malformed;
//   kRecPacked  one 64-bit word, id in the low id_bits, row start in the next lo_bits, degree in
//               the rest; id = n_nodes marks a bad entry, a degree field of all ones means "does
//               not fit, it is row_ptr[id + 1] - row start".  Half the bytes: the seed's own row
//               and the rows of its neighbours take fewer cache lines.
constexpr int kRecNone = 0, kRecWide = 1, kRecPacked = 2;

// Bits of the degree field of a packed record: what the two other fields leave, 31 at most.
__host__ __device__ constexpr int rec_degree_bits(int id_bits, int lo_bits) {
    return 64 - id_bits - lo_bits < 31 ? 64 - id_bits - lo_bits : 31;
}

// The graph as a walker sees it: the CSR, and optionally the records in one of the layouts.
struct WalkGraph {
    const int32_t* __restrict__ row_ptr;
    const int32_t* __restrict__ col_idx;
    const void* __restrict__ rec;
    int id_bits, lo_bits;  // kRecPacked only
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
template <int kRec, int C, typename Visit>
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
    // One group of four steps (one Philox call).  The first group is written out on its own:
    // there s0 is the constant 1, so the steps' row offsets and the Philox counter are known
    // at compile time (walks of up to four steps never leave it).
    auto group = [&](const int s0) __attribute__((always_inline)) {
        uint32_t r[C][4];
#pragma unroll
        for (int c = 0; c < C; ++c)
            philox4x32_10((uint32_t)u, (uint32_t)w[c], (uint32_t)((s0 - 1) >> 2), 0u, key0, key1,
                          r[c]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = s0 + j;
            if (s <= m) {
                if (kRec == kRecWide) {
                    const int4* rec = static_cast<const int4*>(g.rec);
                    int4 nb[C];
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        const bool go = active[c] && cur_deg[c] > 0;
                        const uint32_t pick = go ? r[c][j] % (uint32_t)cur_deg[c] : 0u;
                        nb[c] = make_int4(cur[c], cur_lo[c], cur_deg[c], 0);
                        if (go) nb[c] = rec[(int64_t)cur_lo[c] + (int64_t)pick];
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
                } else if (kRec == kRecPacked) {
                    const unsigned long long* rec = static_cast<const unsigned long long*>(g.rec);
                    const int deg_shift = g.id_bits + g.lo_bits;
                    const uint32_t deg_big = (1u << rec_degree_bits(g.id_bits, g.lo_bits)) - 1u;
                    unsigned long long nb[C];
                    bool go[C];
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        go[c] = active[c] && cur_deg[c] > 0;
                        const uint32_t pick = go[c] ? r[c][j] % (uint32_t)cur_deg[c] : 0u;
                        nb[c] = 0ull;
                        if (go[c]) nb[c] = rec[(int64_t)cur_lo[c] + (int64_t)pick];
                    }
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        if (!go[c]) continue;
                        const int32_t id = (int32_t)(nb[c] & ((1ull << g.id_bits) - 1ull));
                        const int32_t lo = (int32_t)((nb[c] >> g.id_bits) & ((1ull << g.lo_bits) - 1ull));
                        uint32_t deg = (uint32_t)(nb[c] >> deg_shift) & deg_big;
                        if (id >= g.n_nodes) {
                            bad_graph = true;
                        } else {
                            // a degree too large for its field: the record's row was validated
                            // when the records were made, so its end can be taken from the CSR
                            if (deg == deg_big) deg = (uint32_t)(g.row_ptr[id + 1] - lo);
                            cur[c] = id;
                            cur_lo[c] = lo;
                            cur_deg[c] = (int32_t)deg;
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
    };
    group(1);
    for (int s0 = 5; s0 <= m; s0 += 4) group(s0);
    return bad_graph;
}

}  // namespace surel
