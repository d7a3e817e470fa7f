// Node-level relative positional encoding (Sec. 3.2 "Relative Positional Encoding";
// Algorithm 1, RPE step): per seed, the ascending set of distinct visited nodes and, for
// each of them, the landing count at every walk position 0..m.
//
// One wavefront per seed.  Every walk entry becomes a 32-bit key (node id << 4 | position);
// the wave sorts its keys in registers with a bitonic network, then equal-key runs give the
// counts and id changes give the rows.  Rows are assembled in LDS and streamed out
// contiguously at the seed's offset.
#include "device_util.h"
#include "kernels.h"

namespace surel {

constexpr uint32_t kPadKey = 0xFFFFFFFFu;

// Waves per workgroup for a wave that sorts 64*E keys (bounded by the LDS a wave needs).
template <int E>
struct RpeCfg {
    static constexpr int kWaves = (E <= 8) ? 4 : (E == 16 ? 2 : 1);
};

// Sorts the 64*E keys of a wave ascending.  Sort position p = lane*E + r (lane-blocked).
// Bitonic merge sort written with ascending comparators only: a merge of two sorted runs
// starts with a mirror step (p against p ^ (k-1)) and continues with half-cleaners
// (p against p ^ j, j = k/4 .. 1).  Strides below E stay inside a lane (register to
// register); the others exchange registers between lanes.
template <int E>
__device__ __forceinline__ void wave_sort(uint32_t (&x)[E], int lane) {
    constexpr int P = kWave * E;
#pragma unroll
    for (int k = 2; k <= P; k <<= 1) {
        if (k <= E) {
#pragma unroll
            for (int r = 0; r < E; ++r) {
                const int q = r ^ (k - 1);
                if (q > r) {
                    const uint32_t a = min(x[r], x[q]);
                    const uint32_t b = max(x[r], x[q]);
                    x[r] = a;
                    x[q] = b;
                }
            }
        } else {
            const int lane_mask = k / E - 1;
            const bool lower = (lane & (k / (2 * E))) == 0;
            uint32_t y[E];
#pragma unroll
            for (int r = 0; r < E; ++r) y[r] = (uint32_t)__shfl_xor((int)x[E - 1 - r], lane_mask, kWave);
#pragma unroll
            for (int r = 0; r < E; ++r) x[r] = lower ? min(x[r], y[r]) : max(x[r], y[r]);
        }
#pragma unroll
        for (int j = k >> 2; j > 0; j >>= 1) {
            if (j < E) {
#pragma unroll
                for (int r = 0; r < E; ++r) {
                    if ((r & j) == 0) {
                        const uint32_t a = min(x[r], x[r | j]);
                        const uint32_t b = max(x[r], x[r | j]);
                        x[r] = a;
                        x[r | j] = b;
                    }
                }
            } else {
                const int lane_mask = j / E;
                const bool lower = (lane & lane_mask) == 0;
#pragma unroll
                for (int r = 0; r < E; ++r) {
                    const uint32_t y = (uint32_t)__shfl_xor((int)x[r], lane_mask, kWave);
                    x[r] = lower ? min(x[r], y) : max(x[r], y);
                }
            }
        }
    }
}

template <int E>
__global__ __launch_bounds__(RpeCfg<E>::kWaves* kWave) void rpe_kernel(
    const int32_t* __restrict__ walks, int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes,
    uint32_t magic_L, int32_t* __restrict__ counts, const int64_t* __restrict__ rpe_off,
    int64_t cap_rows, int32_t* __restrict__ ids, uint16_t* __restrict__ cnt,
    uint32_t* __restrict__ err) {
    constexpr int P = kWave * E;
    extern __shared__ uint32_t lds32[];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * RpeCfg<E>::kWaves + wave;
    if (i >= n_seeds) return;  // whole waves leave; no block-wide barrier is used below

    const int L = m + 1;
    const int n_key = M * L;  // <= P, checked by the host
    // per-wave LDS: P ids (uint32), then P*L counts (uint16)
    const int words_per_wave = P + (P * L) / 2;
    uint32_t* ids_lds = lds32 + wave * words_per_wave;
    uint16_t* cnt_lds = reinterpret_cast<uint16_t*>(ids_lds + P);
    uint32_t* cnt_lds32 = ids_lds + P;

    // load: entry idx of the seed's walk block has position idx mod L
    const int32_t* W = walks + i * (int64_t)n_key;
    uint32_t x[E];
    bool bad_walk = false;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const int idx = r * kWave + lane;
        if (idx < n_key) {
            int32_t v = W[idx];
            if ((uint32_t)v >= (uint32_t)n_nodes) {
                bad_walk = true;
                v = 0;
            }
            const uint32_t s = (uint32_t)idx - small_div((uint32_t)idx, magic_L) * (uint32_t)L;
            x[r] = ((uint32_t)v << 4) | s;
        } else {
            x[r] = kPadKey;
        }
    }
    raise_error(err, bad_walk, kDevBadWalk);

    wave_sort<E>(x, lane);

    // keys before this lane's first and after its last (pad where there is none: a pad key
    // differs from every valid key in both id and position)
    uint32_t before = (uint32_t)__shfl_up((int)x[E - 1], 1, kWave);
    uint32_t after = (uint32_t)__shfl_down((int)x[0], 1, kWave);
    if (lane == 0) before = kPadKey;
    if (lane == kWave - 1) after = kPadKey;

    // rows: one per distinct id
    uint32_t n_head = 0;
    int32_t last_start = -1;  // sort position of the last key-run start inside this lane
    {
        uint32_t prev = before;
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const bool valid = x[r] != kPadKey;
            n_head += (valid && (x[r] >> 4) != (prev >> 4)) ? 1u : 0u;
            if (valid && x[r] != prev) last_start = lane * E + r;
            prev = x[r];
        }
    }
    const uint32_t incl = wave_incl_sum(n_head);
    const int32_t n_rows = (int32_t)wave_bcast_u32(incl, kWave - 1);
    if (counts != nullptr && lane == 0) counts[i] = n_rows;
    if (ids == nullptr) return;

    const int64_t off = rpe_off[i];
    if (off + n_rows > cap_rows) {
        if (lane == 0) atomicOr(err, kDevCapacity);
        return;
    }

    // start of the key run that is open when this lane begins
    int32_t run_start = __shfl_up(wave_incl_max(last_start), 1, kWave);
    if (lane == 0) run_start = -1;

    const int n_cnt = n_rows * L;
    for (int t = lane; t < (n_cnt + 1) / 2; t += kWave) cnt_lds32[t] = 0u;
    wave_sync();

    {
        uint32_t prev = before;
        int32_t row = (int32_t)(incl - n_head) - 1;  // row of the last key before this lane
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const uint32_t key = x[r];
            const uint32_t next = (r + 1 < E) ? x[(r + 1 < E) ? r + 1 : r] : after;
            const bool valid = key != kPadKey;
            const int32_t e = lane * E + r;
            if (valid && (key >> 4) != (prev >> 4)) {
                row += 1;
                ids_lds[row] = key >> 4;
            }
            if (valid && key != prev) run_start = e;
            if (valid && key != next) cnt_lds[row * L + (int)(key & 15u)] = (uint16_t)(e - run_start + 1);
            prev = key;
        }
    }
    wave_sync();

    // stream the block out: ids as dwords, counts as dwords where the destination allows
    int32_t* out_ids = ids + off;
    for (int t = lane; t < n_rows; t += kWave) out_ids[t] = (int32_t)ids_lds[t];

    const int64_t d0 = off * L;  // first destination element (uint16 units)
    const int head = (int)(d0 & 1);
    uint16_t* out_cnt = cnt + d0;
    if (head && lane == 0) out_cnt[0] = cnt_lds[0];
    const int n_pair = (n_cnt - head) / 2;
    uint32_t* out32 = reinterpret_cast<uint32_t*>(out_cnt + head);
    for (int t = lane; t < n_pair; t += kWave) {
        const uint32_t a = cnt_lds[head + 2 * t];
        const uint32_t b = cnt_lds[head + 2 * t + 1];
        out32[t] = a | (b << 16);
    }
    if (((n_cnt - head) & 1) && lane == 0) out_cnt[n_cnt - 1] = cnt_lds[n_cnt - 1];
}

template <int E>
static hipError_t launch_rpe_e(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                               int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes,
                               int32_t* counts, const int64_t* rpe_off, int64_t cap_rows,
                               int32_t* ids, uint16_t* cnt, uint32_t* err) {
    constexpr int kWaves = RpeCfg<E>::kWaves;
    const int L = m + 1;
    const size_t lds_bytes = (size_t)kWaves * (kWave * E) * (4 + 2 * L);
    if (lds_bytes > (size_t)max_lds_bytes) return hipErrorInvalidValue;
    if (lds_bytes > 64 * 1024) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(rpe_kernel<E>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    const int64_t blocks = (n_seeds + kWaves - 1) / kWaves;
    const uint32_t magic_L = 65536u / (uint32_t)L + 1u;
    hipLaunchKernelGGL(rpe_kernel<E>, dim3((unsigned)blocks), dim3(kWaves * kWave), lds_bytes,
                       stream, walks, n_seeds, M, m, n_nodes, magic_L, counts, rpe_off, cap_rows,
                       ids, cnt, err);
    return hipGetLastError();
}

hipError_t launch_rpe(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                      int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes, int32_t* counts,
                      const int64_t* rpe_off, int64_t cap_rows, int32_t* ids, uint16_t* cnt,
                      uint32_t* err) {
    if (n_seeds == 0) return hipSuccess;
    const int n_key = M * (m + 1);
#define SUREL_RPE_CASE(E_)                                                                     \
    if (n_key <= kWave * (E_))                                                                 \
        return launch_rpe_e<E_>(stream, max_lds_bytes, walks, n_seeds, M, m, n_nodes, counts,  \
                                rpe_off, cap_rows, ids, cnt, err);
    SUREL_RPE_CASE(1)
    SUREL_RPE_CASE(2)
    SUREL_RPE_CASE(4)
    SUREL_RPE_CASE(8)
    SUREL_RPE_CASE(16)
    SUREL_RPE_CASE(32)
#undef SUREL_RPE_CASE
    return hipErrorInvalidValue;
}

}  // namespace surel
