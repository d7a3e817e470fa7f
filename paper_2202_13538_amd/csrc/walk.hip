// Walk sampling (Sec. 3.2 "Walk Sampling"; Algorithm 1, walk step).
//
// One wavefront per seed; a lane moves two walks at a time (two independent gathers in
// flight per lane), ceil(M/128) passes.  A pass keeps its 128
// walks in LDS ([walk][position]) and then streams them out as one contiguous block, so
// the global stores are full-width instead of lane-strided.  Walk rows are written with
// non-temporal stores: they are not read again by this kernel and should not push the
// graph out of the caches that serve the neighbour gathers.
//
// Neighbour records.  A step needs the chosen neighbour's id and then that neighbour's own
// row (start, degree) for the next step: two dependent gathers that each miss the L2 and
// pull a whole cache line for a few bytes, which is what bounds this kernel.  When the job
// is large next to the graph, a small kernel first expands the CSR into one 16-byte record
// per edge entry, (neighbour id, its row start, its degree), so that every step after the
// first is a single gather.  Both forms make exactly the same walks.
//
// Optionally the kernel also reports |V_u|, the number of distinct nodes of each seed's
// walks (Algorithm 1: V_u = set(W_u)), through an LDS hash set fed while the walkers move.
// The kernel waits on memory nearly all the time, so this costs little, and it saves the
// RPE builder a counting pass over the walks.
#include "device_util.h"
#include "distinct.h"
#include "kernels.h"
#include "walk_core.h"

namespace surel {

constexpr int kWalkWavesPerBlock = 4;
constexpr int kWalkChains = 2;  // walks a lane moves at a time

// rec[e] = (col_idx[e], row_ptr[col_idx[e]], degree of col_idx[e], 0); an entry that names no
// node, or whose row is malformed, gets id -1 (the walker will stay in place and flag it).
__global__ void edge_record_kernel(const int32_t* __restrict__ row_ptr,
                                   const int32_t* __restrict__ col_idx, int32_t n_nodes,
                                   int64_t n_edges, int4* __restrict__ rec) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_edges) return;
    const int32_t t = col_idx[e];
    int4 r = make_int4(-1, 0, 0, 0);
    if ((uint32_t)t < (uint32_t)n_nodes) {
        const int32_t lo = row_ptr[t];
        const int32_t hi = row_ptr[t + 1];
        if (lo >= 0 && hi >= lo && (int64_t)hi <= n_edges) r = make_int4(t, lo, hi - lo, 0);
    }
    rec[e] = r;
}

template <bool kCount, bool kRec>
__global__ __launch_bounds__(kWalkWavesPerBlock* kWave) void walk_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const int4* __restrict__ rec, int32_t n_nodes, int64_t n_edges,
    const int32_t* __restrict__ seeds, int64_t n_seeds, int32_t M, int32_t m, uint32_t key0,
    uint32_t key1, int32_t* __restrict__ walks, int32_t* __restrict__ set_sizes, int32_t slots,
    uint32_t* __restrict__ err) {
    extern __shared__ int32_t lds[];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t i = (int64_t)blockIdx.x * kWalkWavesPerBlock + wave;
    if (i >= n_seeds) return;  // whole waves leave; no block-wide barrier is used below

    const int L = m + 1;
    const int per_wave = kWalkChains * kWave * L + (kCount ? slots : 0);
    int32_t* stage = lds + wave * per_wave;
    uint32_t* table = reinterpret_cast<uint32_t*>(stage + kWalkChains * kWave * L);
    int32_t* out_seed = walks + i * (int64_t)M * L;

    const int32_t u = __builtin_amdgcn_readfirstlane(seeds[i]);
    if (u < 0 || u >= n_nodes) {
        if (lane == 0) {
            atomicOr(err, kDevBadSeed);
            if (kCount) set_sizes[i] = 0;
        }
        const int total = M * L;
        for (int t = lane; t < total; t += kWave) __builtin_nontemporal_store(-1, out_seed + t);
        return;
    }

    int n_distinct = 0;
    if (kCount) {
        distinct_clear(table, slots, lane);
        wave_sync();
        n_distinct = distinct_insert(table, slots, (uint32_t)u, lane == 0);
    }

    const WalkGraph g{row_ptr, col_idx, rec, n_nodes, n_edges};
    int32_t u_lo, u_deg;
    bool bad_graph = seed_row(g, u, &u_lo, &u_deg);
    for (int w0 = 0; w0 < M; w0 += kWalkChains * kWave) {
        int w[kWalkChains];
        bool active[kWalkChains];
        int32_t* row[kWalkChains];
#pragma unroll
        for (int c = 0; c < kWalkChains; ++c) {
            w[c] = w0 + c * kWave + lane;
            active[c] = w[c] < M;
            row[c] = stage + (c * kWave + lane) * L;
        }
        bad_graph |= walk_many<kRec, kWalkChains>(
            g, u, u_lo, u_deg, w, active, m, key0, key1, row, [&](int c, int32_t node) {
                if (kCount) n_distinct += distinct_insert(table, slots, (uint32_t)node, active[c]);
            });
        wave_sync();
        const int total = min(kWalkChains * kWave, M - w0) * L;
        int32_t* out = out_seed + (int64_t)w0 * L;
        for (int t = lane; t < total; t += kWave) __builtin_nontemporal_store(stage[t], out + t);
        wave_sync();
    }
    if (kCount && lane == 0) set_sizes[i] = n_distinct;
    raise_error(err, bad_graph, kDevBadGraph);
}

bool walks_want_records(int64_t n_edges, int64_t n_seeds, int32_t M, int32_t m) {
    // the expansion reads every edge entry once; it pays off when the steps after the first
    // outnumber the edge entries several times
    return m >= 2 && n_edges > 0 && n_seeds * (int64_t)M * (m - 1) >= 4 * n_edges;
}

template <bool kCount, bool kRec>
static hipError_t launch_walks_cfg(hipStream_t stream, const int32_t* row_ptr,
                                   const int32_t* col_idx, const int4* rec, int32_t n_nodes,
                                   int64_t n_edges, const int32_t* seeds, int64_t n_seeds,
                                   int32_t M, int32_t m, uint64_t rng_seed, int32_t* walks,
                                   int32_t* set_sizes, uint32_t* err) {
    const int64_t blocks = (n_seeds + kWalkWavesPerBlock - 1) / kWalkWavesPerBlock;
    const int slots = kCount ? distinct_slots(1 + M * m) : 0;
    const size_t lds_bytes = (size_t)kWalkWavesPerBlock * (kWalkChains * kWave * (m + 1) + slots) * 4;
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(
            reinterpret_cast<const void*>(walk_kernel<kCount, kRec>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    hipLaunchKernelGGL((walk_kernel<kCount, kRec>), dim3((unsigned)blocks),
                       dim3(kWalkWavesPerBlock * kWave), lds_bytes, stream, row_ptr, col_idx, rec,
                       n_nodes, n_edges, seeds, n_seeds, M, m,
                       (uint32_t)(rng_seed & 0xFFFFFFFFull), (uint32_t)(rng_seed >> 32), walks,
                       set_sizes, slots, err);
    return hipGetLastError();
}

hipError_t launch_edge_records(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                               int32_t n_nodes, int64_t n_edges, void* edge_records) {
    if (n_edges <= 0) return hipSuccess;
    const int threads = 256;
    hipLaunchKernelGGL(edge_record_kernel, dim3((unsigned)((n_edges + threads - 1) / threads)),
                       dim3(threads), 0, stream, row_ptr, col_idx, n_nodes, n_edges,
                       static_cast<int4*>(edge_records));
    return hipGetLastError();
}

hipError_t launch_walks(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                        int32_t n_nodes, int64_t n_edges, const int32_t* seeds, int64_t n_seeds,
                        int32_t M, int32_t m, uint64_t rng_seed, int32_t* walks,
                        int32_t* set_sizes, const void* edge_records, uint32_t* err) {
    if (n_seeds == 0) return hipSuccess;
    const int4* rec = static_cast<const int4*>(edge_records);
#define SUREL_WALK_ARGS \
    stream, row_ptr, col_idx, rec, n_nodes, n_edges, seeds, n_seeds, M, m, rng_seed, walks, set_sizes, err
    if (set_sizes != nullptr) {
        if (rec != nullptr) return launch_walks_cfg<true, true>(SUREL_WALK_ARGS);
        return launch_walks_cfg<true, false>(SUREL_WALK_ARGS);
    }
    if (rec != nullptr) return launch_walks_cfg<false, true>(SUREL_WALK_ARGS);
    return launch_walks_cfg<false, false>(SUREL_WALK_ARGS);
#undef SUREL_WALK_ARGS
}


}  // namespace surel
