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
// is large next to the graph, a small kernel first expands the CSR into one record per edge
// entry, (neighbour id, its row start, its degree), so that every step after the first is a
// single gather: one 64-bit word for large graphs, 16 bytes otherwise (walk_core.h).  All
// forms make exactly the same walks.
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

// The record of every CSR entry e (layouts in walk_core.h): the neighbour col_idx[e], the start
// of its row and its degree; an entry that names no node, or whose row is malformed, gets the
// layout's "bad entry" id (the walker will stay in place and flag it).
template <int kRec>
__global__ void edge_record_kernel(const int32_t* __restrict__ row_ptr,
                                   const int32_t* __restrict__ col_idx, int32_t n_nodes,
                                   int64_t n_edges, int id_bits, int lo_bits,
                                   void* __restrict__ rec) {
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_edges) return;
    const int32_t t = col_idx[e];
    bool ok = false;
    int32_t lo = 0, hi = 0;
    if ((uint32_t)t < (uint32_t)n_nodes) {
        lo = row_ptr[t];
        hi = row_ptr[t + 1];
        ok = lo >= 0 && hi >= lo && (int64_t)hi <= n_edges;
    }
    if (kRec == kRecWide) {
        static_cast<int4*>(rec)[e] = ok ? make_int4(t, lo, hi - lo, 0) : make_int4(-1, 0, 0, 0);
    } else {
        const uint32_t deg_big = (1u << rec_degree_bits(id_bits, lo_bits)) - 1u;
        unsigned long long r = (unsigned long long)(uint32_t)n_nodes;  // bad entry
        if (ok) {
            const uint32_t deg = min((uint32_t)(hi - lo), deg_big);
            r = (unsigned long long)(uint32_t)t | ((unsigned long long)(uint32_t)lo << id_bits) |
                ((unsigned long long)deg << (id_bits + lo_bits));
        }
        static_cast<unsigned long long*>(rec)[e] = r;
    }
}

template <bool kCount, int kRec>
__global__ __launch_bounds__(kWalkWavesPerBlock* kWave) void walk_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const void* __restrict__ rec, int id_bits, int lo_bits, int32_t n_nodes, int64_t n_edges,
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

    const WalkGraph g{row_ptr, col_idx, rec, id_bits, lo_bits, n_nodes, n_edges};
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

static int bits_for(uint64_t max_value) {  // bits that hold 0 .. max_value
    int b = 1;
    while (b < 64 && (max_value >> b) != 0) b += 1;
    return b;
}

EdgeRecords edge_record_plan(int32_t n_nodes, int64_t n_edges) {
    EdgeRecords plan;
    plan.id_bits = bits_for((uint64_t)n_nodes);   // n_nodes itself marks a bad entry
    plan.lo_bits = bits_for((uint64_t)n_edges);
    // packed records where they matter (an array well beyond the caches) and where ordinary
    // degrees fit their field; the wide layout otherwise
    const bool packed = n_edges >= (1ll << 22) && rec_degree_bits(plan.id_bits, plan.lo_bits) >= 12;
    plan.format = packed ? kRecPacked : kRecWide;
    return plan;
}

size_t edge_record_bytes(const EdgeRecords& plan, int64_t n_edges) {
    return (size_t)n_edges * (plan.format == kRecPacked ? 8 : 16);
}

template <bool kCount, int kRec>
static hipError_t launch_walks_cfg(hipStream_t stream, const int32_t* row_ptr,
                                   const int32_t* col_idx, const EdgeRecords& rec, int32_t n_nodes,
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
                       dim3(kWalkWavesPerBlock * kWave), lds_bytes, stream, row_ptr, col_idx,
                       rec.data, rec.id_bits, rec.lo_bits, n_nodes, n_edges, seeds, n_seeds, M, m,
                       (uint32_t)(rng_seed & 0xFFFFFFFFull), (uint32_t)(rng_seed >> 32), walks,
                       set_sizes, slots, err);
    return hipGetLastError();
}

hipError_t launch_edge_records(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                               int32_t n_nodes, int64_t n_edges, const EdgeRecords& rec) {
    if (n_edges <= 0) return hipSuccess;
    const int threads = 256;
    const dim3 grid((unsigned)((n_edges + threads - 1) / threads));
    void* data = const_cast<void*>(rec.data);
    if (rec.format == kRecPacked) {
        hipLaunchKernelGGL(edge_record_kernel<kRecPacked>, grid, dim3(threads), 0, stream, row_ptr,
                           col_idx, n_nodes, n_edges, rec.id_bits, rec.lo_bits, data);
    } else {
        hipLaunchKernelGGL(edge_record_kernel<kRecWide>, grid, dim3(threads), 0, stream, row_ptr,
                           col_idx, n_nodes, n_edges, rec.id_bits, rec.lo_bits, data);
    }
    return hipGetLastError();
}

template <bool kCount>
static hipError_t launch_walks_c(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                                 const EdgeRecords& rec, int32_t n_nodes, int64_t n_edges,
                                 const int32_t* seeds, int64_t n_seeds, int32_t M, int32_t m,
                                 uint64_t rng_seed, int32_t* walks, int32_t* set_sizes,
                                 uint32_t* err) {
#define SUREL_WALK_ARGS \
    stream, row_ptr, col_idx, rec, n_nodes, n_edges, seeds, n_seeds, M, m, rng_seed, walks, set_sizes, err
    if (rec.data == nullptr) return launch_walks_cfg<kCount, kRecNone>(SUREL_WALK_ARGS);
    if (rec.format == kRecPacked) return launch_walks_cfg<kCount, kRecPacked>(SUREL_WALK_ARGS);
    return launch_walks_cfg<kCount, kRecWide>(SUREL_WALK_ARGS);
}

hipError_t launch_walks(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                        int32_t n_nodes, int64_t n_edges, const int32_t* seeds, int64_t n_seeds,
                        int32_t M, int32_t m, uint64_t rng_seed, int32_t* walks,
                        int32_t* set_sizes, const EdgeRecords& rec, uint32_t* err) {
    if (n_seeds == 0) return hipSuccess;
    if (set_sizes != nullptr) return launch_walks_c<true>(SUREL_WALK_ARGS);
    return launch_walks_c<false>(SUREL_WALK_ARGS);
#undef SUREL_WALK_ARGS
}

}  // namespace surel
