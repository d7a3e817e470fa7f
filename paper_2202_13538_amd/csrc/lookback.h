// Offsets of variable-size blocks inside ONE persistent kernel: how the fused walk + RPE kernel
// learns where a seed's rows go.
//
// Where an item's rows go is a prefix sum over all earlier items, which no wave knows by
// itself, and waiting for it in item order would stall every wave behind the slowest one.
// So the roles are split:
//   - workers take items in increasing order: a workgroup draws a run of consecutive items
//     from one global counter and its waves take them one by one through a word in LDS (one
//     global atomic per run: atomics on one address are slow).  A worker publishes an item's
//     row count as soon as it knows it, without waiting for anything;
//   - the scanner (the wave that drew role 0) runs over the published counts in item order and
//     writes, for every group of 8 items, the rows of all items before the group.  A worker
//     gets an item's offset from its group's base and the counts of the items before it inside
//     the group.  (The scanner stays this light on purpose: one 8-byte store per group.  A
//     scanner that wrote every item's offset itself, 2048 scattered 8-byte stores a round,
//     fell behind and slowed the fused walk + RPE kernel from 16.5 to 21.8 ms.)
// Every wait ends.  Items that have been handed out always form a prefix 0..n-1 of the list
// (runs come from one counter), and the items of a run that no wave has taken yet are larger
// than every item a wave of that workgroup holds.  Counts are published without waiting; the
// scanner publishes the base of group g as soon as the counts of all items before it are
// there; a worker only ever waits for the offset of an item it has already published, i.e.
// for counts of smaller items.  So the smallest unpublished item is always being worked on,
// or about to be taken by a wave that waits only for things that already exist.  The scanner
// was the first wave to draw a role, so it is running whenever anybody waits for it.  On top
// of that every wait is bounded by a spin limit: a wait that runs out raises kDevStall and
// the wave leaves (the row total, which the scanner writes last, then stays -1).
#pragma once

#include "device_util.h"

namespace surel {

constexpr int kGroup = 8;              // consecutive items per group base
constexpr int kScanGroupsPerLane = 4;  // groups a scanner lane takes per round (2048 items a round)
constexpr unsigned long long kChunkLocked = ~0ull;  // LDS chunk word: a wave is refilling it

// Scratch of one launch, in 64-bit words: [0] item counter, [1] role counter, then the group
// bases (int64, -1 = not yet; one per group plus the grand total), then the 16-bit counts
// (rows + 1, 0 = not yet), padded so that the scanner's window never leaves the buffer.
struct LookbackScratch {
    int64_t n_groups;
    int64_t base_words;    // 64-bit words of the group bases
    int64_t status_words;  // 64-bit words of the counts
    int64_t total_words;
};
__host__ __device__ inline LookbackScratch lookback_scratch(int64_t n_items) {
    LookbackScratch s;
    s.n_groups = (n_items + kGroup - 1) / kGroup;
    s.base_words = s.n_groups + 2;
    s.base_words += s.base_words & 1;  // keeps the counts 16-byte aligned
    const int64_t window = (int64_t)kWave * kScanGroupsPerLane;  // groups the scanner reads at once
    s.status_words = (s.n_groups + window) * kGroup * 2 / 8;
    s.total_words = 2 + s.base_words + s.status_words;
    return s;
}
__device__ __forceinline__ int64_t* lookback_base(uint64_t* lb) {
    return reinterpret_cast<int64_t*>(lb + 2);
}
__device__ __forceinline__ uint16_t* lookback_status(uint64_t* lb, const LookbackScratch& s) {
    return reinterpret_cast<uint16_t*>(lb + 2 + s.base_words);
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
// kScanGroupsPerLane * 8 consecutive counts, read at device scope (past the caches that are not
// coherent between the chip's dies) with all loads in flight together.  A count is written
// once, as one 16-bit store, so a wide read sees each of them either not yet or complete.
__device__ __forceinline__ void load_counts(const uint16_t* p, uint4 (&v)[kScanGroupsPerLane]) {
    static_assert(kScanGroupsPerLane == 4, "the loads below are written out for four");
    asm volatile(
        "global_load_dwordx4 %0, %4, off sc1\n\t"
        "global_load_dwordx4 %1, %4, off offset:16 sc1\n\t"
        "global_load_dwordx4 %2, %4, off offset:32 sc1\n\t"
        "global_load_dwordx4 %3, %4, off offset:48 sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
        : "v"(p)
        : "memory");
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

// Next item for this wave.  `chunk` (LDS, one per workgroup) holds the workgroup's current
// run as (end << 32 | next); an empty one is refilled by whoever finds it empty, with one
// atomic on the global counter that draws kDraw consecutive items.  Items at or past the end
// of the list mean: nothing left.
template <int kDraw>
__device__ __forceinline__ int64_t take_item(unsigned long long* chunk, uint64_t* counter,
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
                    reinterpret_cast<unsigned long long*>(counter), (unsigned long long)kDraw);
                __hip_atomic_store(chunk, ((g + kDraw) << 32) | (g + 1ull), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_WORKGROUP);
                got = (uint32_t)g;
                break;
            }
        }
    }
    return (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)got);
}

// The scanner.  status[j] = rows of item j plus one (0 = not published yet; the entries that
// pad the last group are preset to 1).  Writes base[g] = rows of all items before group g, for
// g = 0..n_groups, in order, as far as the published counts reach, round after round, and
// the grand total to *total_out (which the launch's clear kernel has preset to -1, so a scan
// that gives up leaves a total that nobody takes for a row count).
__device__ __forceinline__ void scan_counts(const uint16_t* status, int64_t n_groups, int64_t* base,
                                            int64_t* total_out, uint32_t spin_limit,
                                            uint32_t* err, int lane) {
    __builtin_amdgcn_s_setprio(3);  // everybody's offsets depend on this wave
    int64_t pos = 0;  // groups [0, pos) are accounted for; base[0..pos] is written
    int64_t sum = 0;  // rows of the items before group pos
    if (lane == 0) store_i64_agent(base, 0);
    uint32_t idle = 0;
    while (pos < n_groups) {
        // groups past n_groups lie in the buffer's padding and read as not published
        uint4 v[kScanGroupsPerLane];
        load_counts(status + (pos + lane * kScanGroupsPerLane) * kGroup, v);
        uint32_t rows[kScanGroupsPerLane];
        int local_f = kScanGroupsPerLane;  // first incomplete group among this lane's
#pragma unroll
        for (int j = kScanGroupsPerLane - 1; j >= 0; --j) {
            const uint32_t w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
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

// Offset of `item`'s rows once the scanner has reached its group and the items before it in
// the group have published: the group's base plus those counts.  -1 if the spin limit ran out.
__device__ __forceinline__ int64_t wait_offset(const uint16_t* status, const int64_t* base,
                                               int64_t item, uint32_t spin_limit, int lane) {
    const int64_t g = item / kGroup;
    const int before = (int)(item - g * kGroup);  // items of the group in front of this one
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

}  // namespace surel
