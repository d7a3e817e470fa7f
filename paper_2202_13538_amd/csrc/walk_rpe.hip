// Walk sampling and RPE in one kernel (Sec. 3.2: the RPE is computed on the fly as the walks
// get sampled; Algorithm 1, walk and RPE steps).
//
// A wavefront handles one seed at a time: it walks the M walkers (128 at a time, two per
// lane) into an LDS copy of the seed's walk block, streams the block out, turns the same LDS
// words into sort keys, sorts them in registers and derives the seed's rows exactly like the
// stand-alone RPE builder.  The walk waits on memory almost all the time and the sort is pure
// VALU work, so the two overlap across the waves of a compute unit, and the walks are never
// read back from HBM.
//
// Where a seed's rows go is a prefix sum over all earlier seeds, which no wave knows by
// itself, and waiting for it in seed order would stall every wave behind the slowest one.
// So the kernel is persistent and splits the roles:
//   - workers (all waves but one) take seeds in increasing order: a workgroup draws groups of
//     8 consecutive seeds from one global counter and its waves take them one by one through
//     a word in LDS (one global atomic per group: atomics on one address are slow).  A worker
//     publishes a seed's row count as soon as the sort has it, without waiting for anything,
//     keeps the sorted keys in registers, and only writes the rows out after it has walked
//     and sorted its NEXT seed: by then the offset has long arrived, so nobody waits in
//     practice;
//   - the scanner (the wave that drew role 0) runs over the published counts in seed order and
//     writes, for every group of 8 seeds, the rows of all seeds before the group.  A worker
//     gets a seed's offset from its group's base and the counts of the seeds before it inside
//     the group.
// Every wait ends.  Seeds that have been handed out always form a prefix 0..n-1 of the seed
// list (groups come from one counter), and the seeds of a group that no wave has taken yet
// are larger than every seed a wave of that workgroup holds.  Counts are published without
// waiting; the scanner publishes the base of group g as soon as the counts of all seeds
// before it are there; a worker waits, before it takes its next seed, at most for the offset
// of a seed it has already published, i.e. for counts of smaller seeds.  So the smallest
// unpublished seed is always being worked on, or about to be taken by a wave that waits only
// for things that already exist.  The scanner was the first wave to draw a role, so it is
// running whenever anybody waits for it.  On top of that every wait is bounded by a spin
// limit: a wait that runs out raises kDevStall and the wave leaves.
#include "device_util.h"
#include "kernels.h"
#include "rpe_rows.h"
#include "walk_core.h"
#include "wave_sort.h"

namespace surel {

constexpr int kFusedChains = 2;        // walks a lane moves at a time
constexpr int kGroup = 8;              // consecutive seeds per draw from the global counter
constexpr int kScanGroupsPerLane = 4;  // groups a scanner lane takes per round (2048 seeds a round)
constexpr unsigned long long kChunkLocked = ~0ull;  // LDS chunk word: a wave is refilling it

// Scratch of one call, in 64-bit words: [0] seed counter, [1] role counter, then the group
// bases (int64, -1 = not yet; one per group plus the grand total), then the 16-bit counts
// (rows + 1, 0 = not yet), padded so that the scanner's window never leaves the buffer.
struct FusedScratch {
    int64_t n_groups;
    int64_t base_words;    // 64-bit words of the group bases
    int64_t status_words;  // 64-bit words of the counts
    int64_t total_words;
};
__host__ __device__ inline FusedScratch fused_scratch(int64_t n_seeds) {
    FusedScratch s;
    s.n_groups = (n_seeds + kGroup - 1) / kGroup;
    s.base_words = s.n_groups + 2;
    s.base_words += s.base_words & 1;  // keeps the counts 16-byte aligned
    const int64_t window = (int64_t)kWave * kScanGroupsPerLane;  // groups the scanner reads at once
    s.status_words = (s.n_groups + window) * kGroup * 2 / 8;
    s.total_words = 2 + s.base_words + s.status_words;
    return s;
}

__device__ __forceinline__ uint32_t load_u16_agent(const uint16_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_u16_agent(uint16_t* p, uint32_t v) {
    __hip_atomic_store(p, (uint16_t)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int64_t load_i64_agent(const int64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_i64_agent(int64_t* p, int64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Eight counts at once, read at device scope (past the caches that are not coherent between
// the chip's dies).  A count is written once, as one 16-bit store, so a wide read sees each
// of them either not yet or complete.
__device__ __forceinline__ uint4 load_counts8(const uint16_t* p) {
    uint4 v;
    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)"
                 : "=v"(v)
                 : "v"(p)
                 : "memory");
    return v;
}

__device__ __forceinline__ int64_t wave_bcast_i64(int64_t v, int src_lane) {
    const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)(uint64_t)v, src_lane, kWave);
    const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)((uint64_t)v >> 32), src_lane, kWave);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// One draw from a counter for the whole wave.
__device__ __forceinline__ int64_t wave_draw(uint64_t* counter, int lane) {
    uint64_t drawn = 0;
    if (lane == 0) drawn = atomicAdd(reinterpret_cast<unsigned long long*>(counter), 1ull);
    return wave_bcast_i64((int64_t)drawn, 0);
}

// Next seed for this wave.  `chunk` (LDS, one per workgroup) holds the workgroup's current
// group as (end << 32 | next); an empty one is refilled by whoever finds it empty, with one
// atomic on the global counter.  Seeds at or past n_seeds mean: nothing left.
__device__ __forceinline__ int64_t take_seed(unsigned long long* chunk, uint64_t* counter,
                                             int lane) {
    uint32_t got = 0;
    if (lane == 0) {
        for (;;) {
            const unsigned long long v =
                __hip_atomic_load(chunk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (v == kChunkLocked) {
                __builtin_amdgcn_s_sleep(1);
                continue;
            }
            const uint32_t next = (uint32_t)v;
            const uint32_t end = (uint32_t)(v >> 32);
            if (next < end) {
                if (atomicCAS(chunk, v, v + 1ull) == v) {
                    got = next;
                    break;
                }
            } else if (atomicCAS(chunk, v, kChunkLocked) == v) {
                const unsigned long long g = atomicAdd(
                    reinterpret_cast<unsigned long long*>(counter), (unsigned long long)kGroup);
                __hip_atomic_store(chunk, ((g + kGroup) << 32) | (g + 1ull), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                got = (uint32_t)g;
                break;
            }
        }
    }
    return (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)got);
}

// The scanner.  status[j] = rows of seed j plus one (0 = not published yet; the entries that
// pad the last group are preset to 1).  Writes base[g] = rows of all seeds before group g, for
// g = 0..n_groups, in order, as far as the published counts reach, round after round, and
// the grand total to *total_out.
__device__ __forceinline__ void scan_counts(const uint16_t* status, int64_t n_groups, int64_t* base,
                                            int64_t* total_out, uint32_t spin_limit,
                                            uint32_t* err, int lane) {
    __builtin_amdgcn_s_setprio(3);  // everybody's offsets depend on this wave
    int64_t pos = 0;  // groups [0, pos) are accounted for; base[0..pos] is written
    int64_t sum = 0;  // rows of the seeds before group pos
    if (lane == 0) store_i64_agent(base, 0);
    uint32_t idle = 0;
    while (pos < n_groups) {
        uint32_t rows[kScanGroupsPerLane];
        int local_f = kScanGroupsPerLane;  // first incomplete group among this lane's
#pragma unroll
        for (int j = kScanGroupsPerLane - 1; j >= 0; --j) {
            // groups past n_groups lie in the buffer's padding and read as not published
            const uint4 v = load_counts8(status + (pos + lane * kScanGroupsPerLane + j) * kGroup);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            bool complete = true;
            uint32_t r = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                complete = complete && (w[q] & 0xFFFFu) != 0u && (w[q] >> 16) != 0u;
                r += (w[q] & 0xFFFFu) + (w[q] >> 16);
            }
            rows[j] = r - (uint32_t)kGroup;
            if (!complete) local_f = j;
        }
        const uint64_t holes = __ballot(local_f < kScanGroupsPerLane);
        int f = kWave * kScanGroupsPerLane;  // groups usable this round: those before the first hole
        if (holes != 0ull) {
            const int fl = __builtin_ctzll(holes);
            f = fl * kScanGroupsPerLane + __shfl(local_f, fl, kWave);
        }
        if (f == 0) {
            if (++idle > spin_limit) {
                if (lane == 0) atomicOr(err, kDevStall);
                return;
            }
            __builtin_amdgcn_s_sleep(4);
            continue;
        }
        idle = 0;
        uint32_t lane_sum = 0;
#pragma unroll
        for (int j = 0; j < kScanGroupsPerLane; ++j) {
            if (lane * kScanGroupsPerLane + j >= f) rows[j] = 0u;
            lane_sum += rows[j];
        }
        const uint32_t incl = wave_incl_sum(lane_sum);
        int64_t run = sum + (int64_t)(incl - lane_sum);
#pragma unroll
        for (int j = 0; j < kScanGroupsPerLane; ++j) {
            const int e = lane * kScanGroupsPerLane + j;
            run += rows[j];
            if (e < f) store_i64_agent(base + pos + e + 1, run);
        }
        sum += (int64_t)wave_bcast_u32(incl, kWave - 1);
        pos += f;
    }
    if (lane == 0) *total_out = sum;
}

// Offset of `seed`'s rows once the scanner has reached its group and the seeds before it in
// the group have published: the group's base plus those counts.  -1 if the spin limit ran out.
__device__ __forceinline__ int64_t wait_offset(const uint16_t* status, const int64_t* base,
                                               int64_t seed, uint32_t spin_limit, int lane) {
    const int64_t g = seed / kGroup;
    const int before = (int)(seed - g * kGroup);  // seeds of the group in front of this one
    for (uint32_t spin = 0; spin <= spin_limit; ++spin) {
        uint32_t s = 1u;
        int64_t b = 0;
        if (lane < before) s = load_u16_agent(status + g * kGroup + lane);
        if (lane == kGroup) b = load_i64_agent(base + g);
        b = wave_bcast_i64(b, kGroup);
        const bool missing = __ballot(s == 0u) != 0ull;
        if (b >= 0 && !missing) {
            uint32_t rows = lane < before ? s - 1u : 0u;  // lanes 0..6 at most
            rows += (uint32_t)__shfl_xor((int)rows, 1, kWave);
            rows += (uint32_t)__shfl_xor((int)rows, 2, kWave);
            rows += (uint32_t)__shfl_xor((int)rows, 4, kWave);
            return b + (int64_t)wave_bcast_u32(rows, 0);
        }
        __builtin_amdgcn_s_sleep(8);
    }
    return -1;
}

// Before the main kernel: counters and counts to zero (the counts that pad the last group to
// "no rows"), every group base to "not yet".  (A kernel, not a memset, so that the call stays
// valid under stream capture.)
__global__ void walk_rpe_clear_kernel(uint64_t* __restrict__ lb, int64_t n_seeds) {
    const FusedScratch sc = fused_scratch(n_seeds);
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= sc.total_words) return;
    uint64_t v = 0ull;
    if (t >= 2 && t < 2 + sc.base_words) {
        v = ~0ull;  // -1
    } else if (t >= 2 + sc.base_words) {
        const int64_t first = (t - 2 - sc.base_words) * 4;  // first count of this word
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t j = first + q;
            if (j >= n_seeds && j < sc.n_groups * kGroup) v |= 1ull << (16 * q);
        }
    }
    lb[t] = v;
}

// E = sort keys per lane (64*E >= M*(m+1)).  The waves of a workgroup share the LDS
// allocation and the chunk word, nothing else.
template <int E, bool kRec>
__global__ __launch_bounds__(1024) void walk_rpe_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const int4* __restrict__ rec, int32_t n_nodes, int64_t n_edges,
    const int32_t* __restrict__ seeds, int64_t n_seeds, int32_t M, int32_t m, uint32_t key0,
    uint32_t key1, uint32_t magic_L, int32_t* __restrict__ walks, int64_t cap_rows,
    int64_t* __restrict__ rpe_off, int32_t* __restrict__ ids, uint16_t* __restrict__ cnt,
    int32_t lds_words_per_wave, uint64_t* __restrict__ lb, uint32_t spin_limit,
    uint32_t* __restrict__ err) {
    extern __shared__ uint32_t lds32[];
    __shared__ unsigned long long chunk;

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (threadIdx.x == 0) chunk = 0ull;  // empty
    __syncthreads();                     // the only workgroup-wide barrier of the kernel
    const FusedScratch scr = fused_scratch(n_seeds);
    int64_t* base = reinterpret_cast<int64_t*>(lb + 2);
    uint16_t* status = reinterpret_cast<uint16_t*>(lb + 2 + scr.base_words);
    if (wave_draw(lb + 1, lane) == 0) {
        scan_counts(status, scr.n_groups, base, rpe_off + n_seeds, spin_limit, err, lane);
        return;
    }

    const int L = m + 1;
    const int n_key = M * L;  // <= 64*E, checked by the host
    // the seed's walks [M][L] while it is walked, the rows of the seed before while they go out
    uint32_t* wave_lds = lds32 + wave * lds_words_per_wave;
    int32_t* block = reinterpret_cast<int32_t*>(wave_lds);
    const WalkGraph g{row_ptr, col_idx, rec, n_nodes, n_edges};

    // the seed whose offset and rows are not written yet: its sorted keys stay in registers
    uint32_t x[E];
    RpeRowScan sc{};
    int64_t held_seed = -1;
    bool held_rows = false;  // false: a seed without rows (bad seed, or no table wanted)
    // writes the held seed's offset and rows; false if the wait for the offset ran out
    auto flush = [&]() -> bool {
        const int64_t off = wait_offset(status, base, held_seed, spin_limit, lane);
        if (off < 0) {
            if (lane == 0) atomicOr(err, kDevStall);
            return false;
        }
        if (lane == 0) rpe_off[held_seed] = off;
        held_seed = -1;
        if (!held_rows) return true;
        if (off + sc.n_rows > cap_rows) {
            if (lane == 0) atomicOr(err, kDevCapacity);
        } else {
            rpe_write_rows<E>(x, sc, lane, L, wave_lds, wave_lds + sc.n_rows, off, ids, cnt);
        }
        wave_sync();  // the LDS words are free again
        return true;
    };

    for (;;) {
        const int64_t i = take_seed(&chunk, lb, lane);
        if (i >= n_seeds) break;
        int32_t* out_seed = walks + i * (int64_t)n_key;
        const int32_t u = __builtin_amdgcn_readfirstlane(seeds[i]);
        if (u < 0 || u >= n_nodes) {
            if (lane == 0) {
                atomicOr(err, kDevBadSeed);
                store_u16_agent(status + i, 1u);  // no rows
            }
            for (int t = lane; t < n_key; t += kWave) __builtin_nontemporal_store(-1, out_seed + t);
            if (held_seed >= 0 && !flush()) return;
            held_seed = i;
            held_rows = false;
            continue;
        }
        int32_t u_lo, u_deg;
        bool bad_graph = seed_row(g, u, &u_lo, &u_deg);
        for (int w0 = 0; w0 < M; w0 += kFusedChains * kWave) {
            int w[kFusedChains];
            bool active[kFusedChains];
            int32_t* row[kFusedChains];
#pragma unroll
            for (int c = 0; c < kFusedChains; ++c) {
                w[c] = w0 + c * kWave + lane;
                active[c] = w[c] < M;
                // lanes past the last walk share one scratch row behind the block
                row[c] = block + (active[c] ? w[c] : M) * L;
            }
            bad_graph |= walk_many<kRec, kFusedChains>(g, u, u_lo, u_deg, w, active, m, key0, key1,
                                                       row, [](int, int32_t) {});
        }
        raise_error(err, bad_graph, kDevBadGraph);
        wave_sync();
        // the block goes out as it lies in LDS; the same words become the sort keys
        uint32_t y[E];
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int idx = r * kWave + lane;
            if (idx < n_key) {
                const int32_t v = block[idx];
                __builtin_nontemporal_store(v, out_seed + idx);
                const uint32_t s = (uint32_t)idx - small_div((uint32_t)idx, magic_L) * (uint32_t)L;
                y[r] = ((uint32_t)v << 4) | s;
            } else {
                y[r] = kPadKey;
            }
        }
        wave_sync();  // the walk block in LDS is dead from here on
        wave_sort<E>(y, lane);
        const RpeRowScan sc_y = rpe_scan_rows<E>(y, lane);
        // the count goes out before anything is waited for: publishing never depends on others
        if (lane == 0) store_u16_agent(status + i, (uint32_t)sc_y.n_rows + 1u);
        // the seed before this one: its offset has had a whole walk and a sort to arrive
        if (held_seed >= 0 && !flush()) return;
#pragma unroll
        for (int r = 0; r < E; ++r) x[r] = y[r];
        sc = sc_y;
        held_seed = i;
        held_rows = ids != nullptr;
    }
    if (held_seed >= 0) (void)flush();
}

int64_t walk_rpe_lookback_words(int64_t n_seeds) {
    return fused_scratch(n_seeds > 0 ? n_seeds : 0).total_words;
}

// LDS words of a wave: the walk block plus one scratch row for the idle lanes of the last
// pass, or the rows of a seed (ids + counts) while they are written out, whichever is larger.
static int walk_rpe_lds_words(int M, int m) {
    const int L = m + 1;
    const int max_rows = 1 + M * m;  // App. D.4: at most m*M nodes besides the seed
    const int walk_words = (M + 1) * L;
    const int row_words = max_rows + (max_rows * L + 1) / 2;
    return walk_words > row_words ? walk_words : row_words;
}

#define SUREL_WR_PARAMS                                                                           \
    hipStream_t stream, int max_lds_bytes, int n_cu, const int32_t *row_ptr,                      \
        const int32_t *col_idx, const int4 *rec, int32_t n_nodes, int64_t n_edges,                \
        const int32_t *seeds, int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,           \
        int32_t *walks, int64_t cap_rows, int64_t *rpe_off, int32_t *ids, uint16_t *cnt,          \
        uint64_t *lb, uint32_t spin_limit, uint32_t *err
#define SUREL_WR_ARGS                                                                             \
    stream, max_lds_bytes, n_cu, row_ptr, col_idx, rec, n_nodes, n_edges, seeds, n_seeds, M, m,   \
        rng_seed, walks, cap_rows, rpe_off, ids, cnt, lb, spin_limit, err

template <int E, bool kRec>
static hipError_t launch_walk_rpe_er(SUREL_WR_PARAMS) {
    const int words = walk_rpe_lds_words(M, m);
    const size_t per_wave = (size_t)words * 4;
    const void* fn = reinterpret_cast<const void*>(walk_rpe_kernel<E, kRec>);
    // waves per compute unit that LDS (160 KB) and registers allow, split into as few equal
    // workgroups as possible (a workgroup has at most 16 waves)
    hipFuncAttributes attr;
    hipError_t rc = hipFuncGetAttributes(&attr, fn);
    if (rc != hipSuccess) return rc;
    const int regs = attr.numRegs > 0 ? attr.numRegs : 128;
    int cu_waves = 4 * (512 / ((regs + 7) / 8 * 8));
    const int by_lds = (int)((160 * 1024 - 1024) / per_wave);
    if (cu_waves > by_lds) cu_waves = by_lds;
    if (cu_waves > 32) cu_waves = 32;
    constexpr int kMaxW = 16;
    int groups = (cu_waves + kMaxW - 1) / kMaxW;
    int W = groups > 0 ? cu_waves / groups : 0;
    if (W < 1) {  // not even one wave next to other workgroups: what one workgroup may have
        W = (int)(((size_t)max_lds_bytes - 64) / per_wave);
        if (W > kMaxW) W = kMaxW;
    }
    if (W < 1) return hipErrorInvalidValue;
    const size_t lds_bytes = (size_t)W * per_wave;
    if (lds_bytes + 64 > (size_t)max_lds_bytes) return hipErrorInvalidValue;
    if (lds_bytes > 48 * 1024) {
        rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    // as many workgroups as the device holds at once, or fewer if the job is small: one wave
    // for the scanner and at most one per seed
    int per_cu = 0;
    rc = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, W * kWave, lds_bytes);
    if (rc != hipSuccess) return rc;
    if (per_cu < 1) return hipErrorInvalidValue;
    int64_t blocks = (n_seeds + 1 + W - 1) / W;
    if (blocks > (int64_t)per_cu * n_cu) blocks = (int64_t)per_cu * n_cu;
    if (blocks * W < 2) blocks = 2;  // the scanner and at least one worker

    const int64_t n_clear = fused_scratch(n_seeds).total_words;
    hipLaunchKernelGGL(walk_rpe_clear_kernel, dim3((unsigned)((n_clear + 255) / 256)), dim3(256), 0,
                       stream, lb, n_seeds);
    const uint32_t magic_L = 65536u / (uint32_t)(m + 1) + 1u;
    hipLaunchKernelGGL((walk_rpe_kernel<E, kRec>), dim3((unsigned)blocks), dim3(W * kWave),
                       lds_bytes, stream, row_ptr, col_idx, rec, n_nodes, n_edges, seeds, n_seeds, M,
                       m, (uint32_t)(rng_seed & 0xFFFFFFFFull), (uint32_t)(rng_seed >> 32), magic_L,
                       walks, cap_rows, rpe_off, ids, cnt, words, lb, spin_limit, err);
    return hipGetLastError();
}

template <int E>
static hipError_t launch_walk_rpe_e(SUREL_WR_PARAMS) {
    if (rec != nullptr) return launch_walk_rpe_er<E, true>(SUREL_WR_ARGS);
    return launch_walk_rpe_er<E, false>(SUREL_WR_ARGS);
}

hipError_t launch_walk_rpe(hipStream_t stream, int max_lds_bytes, int n_cu, const int32_t* row_ptr,
                           const int32_t* col_idx, int32_t n_nodes, int64_t n_edges,
                           const int32_t* seeds, int64_t n_seeds, int32_t M, int32_t m,
                           uint64_t rng_seed, int32_t* walks, int64_t cap_rows, int64_t* rpe_off,
                           int32_t* ids, uint16_t* cnt, const void* edge_records, uint64_t* lb,
                           uint32_t spin_limit, uint32_t* err) {
    const int4* rec = static_cast<const int4*>(edge_records);
    const int n_key = M * (m + 1);
#define SUREL_WR_CASE(E_) \
    if (n_key <= kWave * (E_)) return launch_walk_rpe_e<E_>(SUREL_WR_ARGS);
    SUREL_WR_CASE(1)
    SUREL_WR_CASE(2)
    SUREL_WR_CASE(4)
    SUREL_WR_CASE(8)
    SUREL_WR_CASE(16)
    SUREL_WR_CASE(32)
#undef SUREL_WR_CASE
    return hipErrorInvalidValue;
}

}  // namespace surel
