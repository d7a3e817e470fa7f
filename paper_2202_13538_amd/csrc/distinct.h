// Number of distinct node ids among the entries a wave feeds in, through a small
// open-addressing hash set in LDS (the GPU stand-in for the per-seed dictionary of
// Sec. 3.3, used here only to learn |V_u| before the table is laid out).
#pragma once

#include "device_util.h"

namespace surel {

constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;  // no node id reaches 2^28

// Slots for a set of at most n_max ids: a power of two, at least twice n_max.
__host__ __device__ constexpr int distinct_slots(int n_max) {
    int s = 128;
    while (s < 2 * n_max) s *= 2;
    return s;
}

__device__ __forceinline__ void distinct_clear(uint32_t* table, int slots, int lane) {
    for (int t = lane; t < slots; t += kWave) table[t] = kEmptySlot;
}

// Inserts `id` for the lanes with `active` set; returns how many of them were new
// (wave-uniform).  All 64 lanes must call it together.  The table never fills up (it has
// twice as many slots as ids), so every probe sequence ends.
__device__ __forceinline__ int distinct_insert(uint32_t* table, int slots, uint32_t id,
                                               bool active) {
    const uint32_t mask = (uint32_t)slots - 1u;
    uint32_t slot = (id * 0x9E3779B1u) >> 7 & mask;
    bool is_new = false;
    bool pending = active;
    for (int probe = 0; probe < slots; ++probe) {
        if (__ballot(pending) == 0ull) break;
        if (pending) {
            const uint32_t old = atomicCAS(table + slot, kEmptySlot, id);
            if (old == kEmptySlot) {
                is_new = true;
                pending = false;
            } else if (old == id) {
                pending = false;
            } else {
                slot = (slot + 1u) & mask;
            }
        }
    }
    return __popcll(__ballot(is_new));
}

}  // namespace surel
