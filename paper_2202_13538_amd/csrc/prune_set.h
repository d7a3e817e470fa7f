// The hash set of distinct count vectors behind the pruning of the central RPE array (Sec. 3.3;
// Algorithm 1, last step), shared by the stand-alone pruning kernels and the fused walk + RPE
// kernel when it emits RPE-IDs: a global open-addressing table of 64-byte slots (state, rank,
// vector in one cache line) and a small per-workgroup cache of (vector -> slot) in LDS in front
// of it.  A vector is NW 32-bit words, entry 2k of the count vector in the upper half of word k,
// so that comparing words in order compares the counts in order.
#pragma once

#include "device_util.h"

namespace surel {

constexpr uint32_t kSlotEmpty = 0u, kSlotLocked = 1u, kSlotFull = 2u;
constexpr int kSlotWords = 16;    // 64-byte slots: [0] state, [1] rank, [2..3] unused, [4..11] vector
constexpr int kSlotVector = 4;    // first word of the vector inside a slot
constexpr int kMaxVecWords = 8;   // m + 1 <= 16 counts of 16 bits

template <int NW>
__device__ __forceinline__ uint32_t hash_vector(const uint32_t (&w)[NW]) {
    uint32_t h = 0x811C9DC5u;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        h = (h ^ w[k]) * 0x9E3779B1u;
        h ^= h >> 15;
    }
    return h;
}

// Finds (or inserts) vector w, first probe at slot h; returns its slot number, or -1 if a wait
// ran out or the table is full.  *n_inserted counts the vectors inserted so far (the size of T
// when collect has ended).
template <int NW>
__device__ __forceinline__ int32_t find_or_insert(const uint32_t (&w)[NW], uint32_t h,
                                                  uint32_t* __restrict__ slots, uint32_t slot_mask,
                                                  int64_t cap_T,
                                                  unsigned long long* __restrict__ n_inserted,
                                                  uint32_t spin_limit, uint32_t* __restrict__ err) {
    uint32_t spins = 0;
    for (uint32_t probe = 0; probe <= slot_mask;) {
        uint32_t* slot = slots + (size_t)h * kSlotWords;
        // a slot that reads as full is final, and its vector lies in the same cache line
        uint32_t st = slot[0];
        if (st != kSlotFull) {
            st = atomicCAS(slot, kSlotEmpty, kSlotLocked);
            if (st == kSlotEmpty) {
                // this lane owns the slot: is there still room in T?
                const unsigned long long before = atomicAdd(n_inserted, 1ull);
                if ((int64_t)before >= cap_T) atomicOr(err, kDevCapacity);
#pragma unroll
                for (int k = 0; k < NW; ++k)
                    __hip_atomic_store(slot + kSlotVector + k, w[k], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(slot, kSlotFull, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                return (int32_t)h;
            }
            if (st == kSlotLocked) {
                // somebody is writing this slot's vector: look again
                if (++spins > spin_limit) {
                    atomicOr(err, kDevStall);
                    return -1;
                }
                __builtin_amdgcn_s_sleep(1);
                continue;
            }
            // full, but the plain load may have come from a stale line: read past it
            bool same = true;
#pragma unroll
            for (int k = 0; k < NW; ++k)
                same = same && __hip_atomic_load(slot + kSlotVector + k, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT) == w[k];
            if (same) return (int32_t)h;
        } else {
            bool same = true;
#pragma unroll
            for (int k = 0; k < NW; ++k) same = same && slot[kSlotVector + k] == w[k];
            if (same) return (int32_t)h;
        }
        h = (h + 1u) & slot_mask;
        probe += 1;
    }
    return -1;
}

constexpr int kCacheEntries = 256;   // per-workgroup LDS cache of (vector -> slot), direct mapped
constexpr int kCacheWords = 12;      // [0] state, [1] slot, [2..3] unused, [4..11] vector


// Clears a workgroup's cache (every thread of the workgroup calls it, a barrier follows).
__device__ __forceinline__ void prune_cache_clear(uint32_t* cache, int tid, int n_threads) {
    for (int t = tid; t < kCacheEntries; t += n_threads) cache[t * kCacheWords] = 0u;
}

// The slot of vector w: from the workgroup's cache if it is there, else from the global table
// (inserting it if it is new), remembering it in the cache when its entry is still free.  An
// entry is written once, by the lane that wins its state word, and is valid for good after that
// (state, then vector and slot, then "valid": LDS operations of a wave take effect in order), so
// readers never see a mix of two vectors.  Returns the slot number, or -1 (see find_or_insert).
template <int NW>
__device__ __forceinline__ int32_t prune_lookup(const uint32_t (&w)[NW], uint32_t* cache,
                                                uint32_t* __restrict__ slots, uint32_t slot_mask,
                                                int64_t cap_T,
                                                unsigned long long* __restrict__ n_inserted,
                                                uint32_t spin_limit, uint32_t* __restrict__ err) {
    const uint32_t hv = hash_vector<NW>(w);
    uint32_t* entry = cache + ((hv >> 20) & (kCacheEntries - 1)) * kCacheWords;
    if (entry[0] == 2u) {
        bool same = true;
#pragma unroll
        for (int k = 0; k < NW; ++k) same = same && entry[4 + k] == w[k];
        if (same) return (int32_t)entry[1];
    }
    const int32_t found = find_or_insert<NW>(w, hv & slot_mask, slots, slot_mask, cap_T, n_inserted,
                                             spin_limit, err);
    if (found >= 0 && atomicCAS(entry, 0u, 1u) == 0u) {
#pragma unroll
        for (int k = 0; k < NW; ++k) entry[4 + k] = w[k];
        entry[1] = (uint32_t)found;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __hip_atomic_store(entry, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    return found;
}

// The same in front of a kernel that does not know the vector length at compile time: w holds
// kMaxVecWords words of which the first nw can be non-zero, a cache entry is 2 + nw words (state,
// slot, vector), so that short vectors get many entries out of a fixed LDS budget:
// kFusedCacheWords words hold fused_cache_entries(nw) entries (a power of two).
constexpr int kFusedCacheWords = 6144;  // 24 KB
__host__ __device__ constexpr int fused_cache_entries(int nw) {
    int e = 64;
    while (e * 2 * (2 + nw) <= kFusedCacheWords) e *= 2;
    return e;
}
__device__ __forceinline__ void fused_cache_clear(uint32_t* cache, int nw, int tid, int n_threads) {
    const int n = fused_cache_entries(nw);
    for (int t = tid; t < n; t += n_threads) cache[t * (2 + nw)] = 0u;
}
__device__ __forceinline__ int32_t prune_lookup_any(const uint32_t (&w)[kMaxVecWords], int nw,
                                                    uint32_t* cache, uint32_t* __restrict__ slots,
                                                    uint32_t slot_mask, int64_t cap_T,
                                                    unsigned long long* __restrict__ n_inserted,
                                                    uint32_t spin_limit,
                                                    uint32_t* __restrict__ err) {
    const uint32_t hv = hash_vector<kMaxVecWords>(w);
    uint32_t* entry = cache + ((hv >> 18) & (uint32_t)(fused_cache_entries(nw) - 1)) * (2 + nw);
    if (entry[0] == 2u) {
        bool same = true;
#pragma unroll
        for (int k = 0; k < kMaxVecWords; ++k)
            if (k < nw) same = same && entry[2 + k] == w[k];
        if (same) return (int32_t)entry[1];
    }
    const int32_t found = find_or_insert<kMaxVecWords>(w, hv & slot_mask, slots, slot_mask, cap_T,
                                                       n_inserted, spin_limit, err);
    if (found >= 0 && atomicCAS(entry, 0u, 1u) == 0u) {
#pragma unroll
        for (int k = 0; k < kMaxVecWords; ++k)
            if (k < nw) entry[2 + k] = w[k];
        entry[1] = (uint32_t)found;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __hip_atomic_store(entry, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    return found;
}

// For vectors of at most three words (m + 1 <= 6, the usual walk lengths) with the length known
// at compile time, the cache entries are packed: [0] 0 = free, 1 = being written, 2^31 | slot =
// valid; [1 .. NW] the vector; 2 words an entry for NW = 1, else 4, so that an entry is one LDS
// read.  The entry is read as a whole: should the read ever see the valid word next to vector
// words that are not yet there, the comparison fails and the lane asks the global table, which is
// slower and right; a valid entry never changes again.
template <int NW>
struct PackedCache {
    static_assert(NW >= 1 && NW <= 3, "packed cache entries hold up to three words");
    static constexpr int kEntryWords = NW == 1 ? 2 : 4;
    static constexpr int entries() {
        int e = 64;
        while (e * 2 * kEntryWords <= kFusedCacheWords) e *= 2;
        return e;
    }
};
constexpr uint32_t kPackedValid = 0x80000000u;

template <int NW>
__device__ __forceinline__ int32_t prune_lookup_packed(const uint32_t (&w)[NW], uint32_t* cache,
                                                       uint32_t* __restrict__ slots,
                                                       uint32_t slot_mask, int64_t cap_T,
                                                       unsigned long long* __restrict__ n_inserted,
                                                       uint32_t spin_limit,
                                                       uint32_t* __restrict__ err) {
    constexpr int EW = PackedCache<NW>::kEntryWords;
    const uint32_t hv = hash_vector<NW>(w);
    uint32_t* entry = cache + ((hv >> 18) & (uint32_t)(PackedCache<NW>::entries() - 1)) * EW;
    uint32_t e[4] = {0u, 0u, 0u, 0u};
    if constexpr (EW == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(entry);
        e[0] = v.x, e[1] = v.y;
    } else {
        const uint4 v = *reinterpret_cast<const uint4*>(entry);
        e[0] = v.x, e[1] = v.y, e[2] = v.z, e[3] = v.w;
    }
    if (e[0] & kPackedValid) {
        bool same = true;
#pragma unroll
        for (int k = 0; k < NW; ++k) same = same && e[1 + k] == w[k];
        if (same) return (int32_t)(e[0] & ~kPackedValid);
    }
    const int32_t found = find_or_insert<NW>(w, hv & slot_mask, slots, slot_mask, cap_T, n_inserted,
                                             spin_limit, err);
    if (found >= 0 && atomicCAS(entry, 0u, 1u) == 0u) {
#pragma unroll
        for (int k = 0; k < NW; ++k) entry[1 + k] = w[k];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __hip_atomic_store(entry, kPackedValid | (uint32_t)found, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    return found;
}

// Clears the whole cache: all-zero words are free entries in both layouts.
__device__ __forceinline__ void fused_cache_clear_all(uint32_t* cache, int tid, int n_threads) {
    for (int t = tid; t < kFusedCacheWords; t += n_threads) cache[t] = 0u;
}

}  // namespace surel
