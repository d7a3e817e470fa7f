// Walk sampling (Sec. 3.2 "Walk Sampling"; Algorithm 1, walk step).
//
// One wavefront per seed; a lane is one walk, ceil(M/64) passes.  A pass keeps its 64
// walks in LDS ([walk][position]) and then streams them out as one contiguous block, so
// the global stores are full-width instead of lane-strided.  Walk rows are written with
// non-temporal stores: they are not read again by this kernel and should not push the
// graph out of the caches that serve the neighbour gathers.
//
// Optionally the kernel also reports |V_u|, the number of distinct nodes of each seed's
// walks (Algorithm 1: V_u = set(W_u)), through an LDS hash set fed while the walkers move.
// The kernel waits on memory nearly all the time, so this costs little, and it saves the
// RPE builder a counting pass over the walks.
#include "device_util.h"
#include "distinct.h"
#include "kernels.h"

namespace surel {

constexpr int kWalkWavesPerBlock = 4;

template <bool kCount>
__global__ __launch_bounds__(kWalkWavesPerBlock* kWave) void walk_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx, int32_t n_nodes,
    int64_t n_edges, const int32_t* __restrict__ seeds, int64_t n_seeds, int32_t M, int32_t m,
    uint32_t key0, uint32_t key1, int32_t* __restrict__ walks, int32_t* __restrict__ set_sizes,
    int32_t slots, uint32_t* __restrict__ err) {
    extern __shared__ int32_t lds[];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t i = (int64_t)blockIdx.x * kWalkWavesPerBlock + wave;
    if (i >= n_seeds) return;  // whole waves leave; no block-wide barrier is used below

    const int L = m + 1;
    const int per_wave = kWave * L + (kCount ? slots : 0);
    int32_t* stage = lds + wave * per_wave;
    uint32_t* table = reinterpret_cast<uint32_t*>(stage + kWave * L);
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

    bool bad_graph = false;
    for (int w0 = 0; w0 < M; w0 += kWave) {
        const int w = w0 + lane;
        const bool active = w < M;
        int32_t cur = u;
        stage[lane * L] = u;
        for (int s0 = 1; s0 <= m; s0 += 4) {
            uint32_t r[4];
            philox4x32_10((uint32_t)u, (uint32_t)w, (uint32_t)((s0 - 1) >> 2), 0u, key0, key1, r);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int s = s0 + j;
                if (s <= m) {
                    if (active) {
                        const int32_t lo = row_ptr[cur];
                        const int32_t hi = row_ptr[cur + 1];
                        if (lo < 0 || hi < lo || (int64_t)hi > n_edges) {
                            bad_graph = true;
                        } else if (hi > lo) {
                            const uint32_t deg = (uint32_t)(hi - lo);
                            const int32_t nxt = col_idx[(int64_t)lo + (int64_t)(r[j] % deg)];
                            if ((uint32_t)nxt >= (uint32_t)n_nodes) {
                                bad_graph = true;
                            } else {
                                cur = nxt;
                            }
                        }
                    }
                    stage[lane * L + s] = cur;
                    if (kCount) n_distinct += distinct_insert(table, slots, (uint32_t)cur, active);
                }
            }
        }
        wave_sync();
        const int total = min(kWave, M - w0) * L;
        int32_t* out = out_seed + (int64_t)w0 * L;
        for (int t = lane; t < total; t += kWave) __builtin_nontemporal_store(stage[t], out + t);
        wave_sync();
    }
    if (kCount && lane == 0) set_sizes[i] = n_distinct;
    raise_error(err, bad_graph, kDevBadGraph);
}

hipError_t launch_walks(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                        int32_t n_nodes, int64_t n_edges, const int32_t* seeds, int64_t n_seeds,
                        int32_t M, int32_t m, uint64_t rng_seed, int32_t* walks,
                        int32_t* set_sizes, uint32_t* err) {
    if (n_seeds == 0) return hipSuccess;
    const int64_t blocks = (n_seeds + kWalkWavesPerBlock - 1) / kWalkWavesPerBlock;
    const uint32_t key0 = (uint32_t)(rng_seed & 0xFFFFFFFFull);
    const uint32_t key1 = (uint32_t)(rng_seed >> 32);
    const dim3 grid((unsigned)blocks), block(kWalkWavesPerBlock * kWave);
    if (set_sizes != nullptr) {
        const int slots = distinct_slots(1 + M * m);
        const size_t lds_bytes = (size_t)kWalkWavesPerBlock * (kWave * (m + 1) + slots) * 4;
        if (lds_bytes > 48 * 1024) {
            hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(walk_kernel<true>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                                (int)lds_bytes);
            if (rc != hipSuccess) return rc;
        }
        hipLaunchKernelGGL(walk_kernel<true>, grid, block, lds_bytes, stream, row_ptr, col_idx,
                           n_nodes, n_edges, seeds, n_seeds, M, m, key0, key1, walks, set_sizes,
                           slots, err);
    } else {
        const size_t lds_bytes = (size_t)kWalkWavesPerBlock * kWave * (m + 1) * 4;
        hipLaunchKernelGGL(walk_kernel<false>, grid, block, lds_bytes, stream, row_ptr, col_idx,
                           n_nodes, n_edges, seeds, n_seeds, M, m, key0, key1, walks, set_sizes, 0,
                           err);
    }
    return hipGetLastError();
}

}  // namespace surel
