// From a wave's sorted walk keys to the rows of one seed's RPE block (Sec. 3.2 "Relative
// Positional Encoding"): a key is node id << 4 | walk position; id changes start rows,
// equal-key runs are the landing counts.  Shared by the stand-alone RPE builder and the fused
// walk + RPE kernel.
#pragma once

#include "device_util.h"

namespace surel {

constexpr uint32_t kPadKey = 0xFFFFFFFFu;  // sorts last; differs from every valid key in id and position

// What a lane knows about the rows of the wave's sorted keys (sort position p = lane*E + r).
struct RpeRowScan {
    uint32_t before;    // key just before this lane's first (kPadKey for lane 0)
    uint32_t after;     // key just after this lane's last (kPadKey for lane 63)
    uint32_t n_head;    // rows that start inside this lane
    uint32_t incl;      // rows that start in lanes 0..this
    int32_t n_rows;     // rows of the whole wave (wave-uniform)
    int32_t run_start;  // sort position where the key run open at this lane's start began
};

template <int E>
__device__ __forceinline__ RpeRowScan rpe_scan_rows(const uint32_t (&x)[E], int lane) {
    RpeRowScan sc;
    sc.before = (uint32_t)__shfl_up((int)x[E - 1], 1, kWave);
    sc.after = (uint32_t)__shfl_down((int)x[0], 1, kWave);
    if (lane == 0) sc.before = kPadKey;
    if (lane == kWave - 1) sc.after = kPadKey;
    sc.n_head = 0;
    int32_t last_start = -1;  // sort position of the last key-run start inside this lane
    uint32_t prev = sc.before;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const bool valid = x[r] != kPadKey;
        sc.n_head += (valid && (x[r] >> 4) != (prev >> 4)) ? 1u : 0u;
        if (valid && x[r] != prev) last_start = lane * E + r;
        prev = x[r];
    }
    sc.incl = wave_incl_sum(sc.n_head);
    sc.n_rows = (int32_t)wave_bcast_u32(sc.incl, kWave - 1);
    sc.run_start = __shfl_up(wave_incl_max(last_start), 1, kWave);
    if (lane == 0) sc.run_start = -1;
    return sc;
}

// Assembles the block's rows in LDS: ids_lds gets n_rows words, cnt_lds32 gets n_rows*L uint16
// (rounded up to whole words).  Ends with the LDS writes ordered before later reads.
template <int E>
__device__ __forceinline__ void rpe_assemble_rows(const uint32_t (&x)[E], const RpeRowScan& sc,
                                                  int lane, int L, uint32_t* ids_lds,
                                                  uint32_t* cnt_lds32) {
    uint16_t* cnt_lds = reinterpret_cast<uint16_t*>(cnt_lds32);
    const int n_cnt = sc.n_rows * L;
    for (int t = lane; t < (n_cnt + 1) / 2; t += kWave) cnt_lds32[t] = 0u;
    wave_sync();
    uint32_t prev = sc.before;
    int32_t run_start = sc.run_start;
    int32_t row = (int32_t)(sc.incl - sc.n_head) - 1;  // row of the last key before this lane
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const uint32_t key = x[r];
        const uint32_t next = (r + 1 < E) ? x[(r + 1 < E) ? r + 1 : r] : sc.after;
        const bool valid = key != kPadKey;
        const int32_t e = lane * E + r;
        if (valid && (key >> 4) != (prev >> 4)) {
            row += 1;
            ids_lds[row] = key >> 4;
        }
        if (valid && key != prev) run_start = e;
        if (valid && key != next)
            cnt_lds[row * L + (int)(key & 15u)] = (uint16_t)(e - run_start + 1);
        prev = key;
    }
    wave_sync();
}

// Streams an assembled block out to rows [off, off + n_rows) of the table: ids as dwords,
// counts (unless cnt is null: a table that carries RPE-IDs only) as dwords where the
// destination's alignment allows.
__device__ __forceinline__ void rpe_stream_rows(int n_rows, int lane, int L, const uint32_t* ids_lds,
                                                const uint32_t* cnt_lds32, int64_t off,
                                                int32_t* __restrict__ ids,
                                                uint16_t* __restrict__ cnt) {
    const uint16_t* cnt_lds = reinterpret_cast<const uint16_t*>(cnt_lds32);
    const int n_cnt = n_rows * L;
    int32_t* out_ids = ids + off;
    for (int t = lane; t < n_rows; t += kWave) out_ids[t] = (int32_t)ids_lds[t];
    if (cnt == nullptr) return;

    const int64_t d0 = off * L;  // first destination element (uint16 units)
    const int head = (int)(d0 & 1);
    uint16_t* out_cnt = cnt + d0;
    if (head && lane == 0) out_cnt[0] = cnt_lds[0];
    const int n_pair = (n_cnt - head) / 2;
    uint32_t* out32 = reinterpret_cast<uint32_t*>(out_cnt + head);
    if (head == 0) {
        for (int t = lane; t < n_pair; t += kWave) out32[t] = cnt_lds32[t];
    } else {
        for (int t = lane; t < n_pair; t += kWave) {
            const uint32_t a = cnt_lds[1 + 2 * t];
            const uint32_t b = cnt_lds[2 + 2 * t];
            out32[t] = a | (b << 16);
        }
    }
    if (((n_cnt - head) & 1) && lane == 0) out_cnt[n_cnt - 1] = cnt_lds[n_cnt - 1];
}

template <int E>
__device__ __forceinline__ void rpe_write_rows(const uint32_t (&x)[E], const RpeRowScan& sc,
                                               int lane, int L, uint32_t* ids_lds,
                                               uint32_t* cnt_lds32, int64_t off,
                                               int32_t* __restrict__ ids,
                                               uint16_t* __restrict__ cnt) {
    rpe_assemble_rows<E>(x, sc, lane, L, ids_lds, cnt_lds32);
    rpe_stream_rows(sc.n_rows, lane, L, ids_lds, cnt_lds32, off, ids, cnt);
}

}  // namespace surel
