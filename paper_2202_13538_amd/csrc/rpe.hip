// Node-level relative positional encoding (Sec. 3.2 "Relative Positional Encoding";
// Algorithm 1, RPE step): per seed, the ascending set of distinct visited nodes and, for
// each of them, the landing count at every walk position 0..m.
//
// Layout first, then rows.  |V_u| per seed either comes from the caller (the walk kernel can
// report it) or from a counting kernel here (an LDS hash set per seed); an exclusive scan
// turns the sizes into rpe_off.  The fill kernel then takes one wavefront per seed: every
// walk entry becomes a 32-bit key (node id << 4 | position); the wave sorts its keys in
// registers with a bitonic network, equal-key runs give the counts and id changes give the
// rows.  Rows are assembled in LDS and streamed out contiguously at the seed's offset.
#include "device_util.h"
#include "distinct.h"
#include "kernels.h"

namespace surel {

constexpr uint32_t kPadKey = 0xFFFFFFFFu;

// Compare-exchange with the lane `lane ^ MASK`: the lower lane of a pair keeps the smaller
// key.  `y < x` decides for a lower lane, its negation for an upper one (equal keys need
// no exchange, so either answer is right for them).
template <int MASK>
__device__ __forceinline__ uint32_t exchange(uint32_t x, uint32_t y, bool upper) {
    const bool take = (y < x) != upper;
    return take ? y : x;
}

// Sorts the 64*E keys of a wave ascending.  Sort position p = lane*E + r (lane-blocked).
// Bitonic merge sort written with ascending comparators only: a merge of two sorted runs
// starts with a mirror step (p against p ^ (k-1)) and continues with half-cleaners
// (p against p ^ j, j = k/4 .. 1).  Strides below E stay inside a lane (register to
// register); the others exchange registers between lanes.
template <int E, int K>
__device__ __forceinline__ void sort_merge_level(uint32_t (&x)[E], int lane) {
    if constexpr (K <= E) {
#pragma unroll
        for (int r = 0; r < E; ++r) {
            const int q = r ^ (K - 1);
            if (q > r) {
                const uint32_t a = min(x[r], x[q]);
                const uint32_t b = max(x[r], x[q]);
                x[r] = a;
                x[q] = b;
            }
        }
    } else {
        constexpr int kLaneMask = K / E - 1;
        const bool upper = (lane & (K / (2 * E))) != 0;
        uint32_t y[E];
#pragma unroll
        for (int r = 0; r < E; ++r) y[r] = lane_xor<kLaneMask>(x[E - 1 - r], lane);
#pragma unroll
        for (int r = 0; r < E; ++r) x[r] = exchange<kLaneMask>(x[r], y[r], upper);
    }
}

template <int E, int J>
__device__ __forceinline__ void sort_half_cleaner(uint32_t (&x)[E], int lane) {
    if constexpr (J >= 1) {
        if constexpr (J < E) {
#pragma unroll
            for (int r = 0; r < E; ++r) {
                if ((r & J) == 0) {
                    const uint32_t a = min(x[r], x[r | J]);
                    const uint32_t b = max(x[r], x[r | J]);
                    x[r] = a;
                    x[r | J] = b;
                }
            }
        } else {
            constexpr int kLaneMask = J / E;
            const bool upper = (lane & kLaneMask) != 0;
#pragma unroll
            for (int r = 0; r < E; ++r) {
                const uint32_t y = lane_xor<kLaneMask>(x[r], lane);
                x[r] = exchange<kLaneMask>(x[r], y, upper);
            }
        }
        sort_half_cleaner<E, J / 2>(x, lane);
    }
}

template <int E, int K>
__device__ __forceinline__ void sort_levels(uint32_t (&x)[E], int lane) {
    if constexpr (K <= kWave * E) {
        sort_merge_level<E, K>(x, lane);
        sort_half_cleaner<E, K / 4>(x, lane);
        sort_levels<E, K * 2>(x, lane);
    }
}

template <int E>
__device__ __forceinline__ void wave_sort(uint32_t (&x)[E], int lane) {
    sort_levels<E, 2>(x, lane);
}

constexpr int kRpeWaves = 4;  // waves (seeds) per workgroup

// |V_u| of every seed from the walks themselves (used when the caller has no sizes).
__global__ __launch_bounds__(kRpeWaves* kWave) void rpe_count_kernel(
    const int32_t* __restrict__ walks, int64_t n_seeds, int32_t n_key, int32_t n_nodes,
    int32_t slots, int32_t* __restrict__ set_sizes, uint32_t* __restrict__ err) {
    extern __shared__ uint32_t lds32[];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t i = (int64_t)blockIdx.x * kRpeWaves + wave;
    if (i >= n_seeds) return;  // whole waves leave; no block-wide barrier is used below
    uint32_t* table = lds32 + wave * slots;
    distinct_clear(table, slots, lane);
    wave_sync();
    const int32_t* W = walks + i * (int64_t)n_key;
    int n_distinct = 0;
    bool bad_walk = false;
    for (int t0 = 0; t0 < n_key; t0 += kWave) {
        const int t = t0 + lane;
        const bool active = t < n_key;
        int32_t v = active ? __builtin_nontemporal_load(W + t) : 0;
        if ((uint32_t)v >= (uint32_t)n_nodes) {
            bad_walk = true;
            v = 0;
        }
        n_distinct += distinct_insert(table, slots, (uint32_t)v, active);
    }
    raise_error(err, bad_walk, kDevBadWalk);
    if (lane == 0) set_sizes[i] = n_distinct;
}

// E = keys per lane, kWaves = waves (seeds) per workgroup, as many as the LDS a wave needs allows.
// rpe_off is complete when this kernel starts.
template <int E, int kWaves>
__global__ __launch_bounds__(kWaves* kWave) void rpe_fill_kernel(
    const int32_t* __restrict__ walks, int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes,
    uint32_t magic_L, const int64_t* __restrict__ rpe_off, int64_t cap_rows,
    int32_t* __restrict__ ids, uint16_t* __restrict__ cnt, uint32_t* __restrict__ err) {
    constexpr int P = kWave * E;
    extern __shared__ uint32_t lds32[];

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t i = (int64_t)blockIdx.x * kWaves + wave;
    if (i >= n_seeds) return;  // whole waves leave; no block-wide barrier is used below

    const int L = m + 1;
    const int n_key = M * L;  // <= P, checked by the host
    // per-wave LDS: P ids (uint32), then P*L counts (uint16)
    uint32_t* ids_lds = lds32 + wave * (P + (P * L) / 2);
    uint32_t* cnt_lds32 = ids_lds + P;
    uint16_t* cnt_lds = reinterpret_cast<uint16_t*>(cnt_lds32);

    const int64_t off = rpe_off[i];
    const int64_t given_rows = rpe_off[i + 1] - off;

    // load: entry idx of the seed's walk block has position idx mod L
    const int32_t* W = walks + i * (int64_t)n_key;
    uint32_t x[E];
    bool bad_walk = false;
#pragma unroll
    for (int r = 0; r < E; ++r) {
        const int idx = r * kWave + lane;
        if (idx < n_key) {
            int32_t v = __builtin_nontemporal_load(W + idx);
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

    // the layout was made from set sizes; a size that does not match the walks (sizes passed
    // in for other walks) must not make blocks overlap
    if ((int64_t)n_rows != given_rows) {
        if (lane == 0) atomicOr(err, kDevBadSizes);
        return;
    }
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
            if (valid && key != next)
                cnt_lds[row * L + (int)(key & 15u)] = (uint16_t)(e - run_start + 1);
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

hipError_t launch_rpe_count(hipStream_t stream, const int32_t* walks, int64_t n_seeds, int32_t M,
                            int32_t m, int32_t n_nodes, int32_t* set_sizes, uint32_t* err) {
    if (n_seeds == 0) return hipSuccess;
    const int n_key = M * (m + 1);
    const int slots = distinct_slots(n_key);
    const size_t lds_bytes = (size_t)kRpeWaves * slots * 4;
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(rpe_count_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    const int64_t blocks = (n_seeds + kRpeWaves - 1) / kRpeWaves;
    hipLaunchKernelGGL(rpe_count_kernel, dim3((unsigned)blocks), dim3(kRpeWaves * kWave), lds_bytes,
                       stream, walks, n_seeds, n_key, n_nodes, slots, set_sizes, err);
    return hipGetLastError();
}

template <int E, int W>
static hipError_t launch_rpe_fill_ew(hipStream_t stream, const int32_t* walks, int64_t n_seeds,
                                     int32_t M, int32_t m, int32_t n_nodes, const int64_t* rpe_off,
                                     int64_t cap_rows, int32_t* ids, uint16_t* cnt, uint32_t* err) {
    const int L = m + 1;
    const size_t lds_bytes = (size_t)W * (kWave * E) * (4 + 2 * L);
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(rpe_fill_kernel<E, W>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    const int64_t blocks = (n_seeds + W - 1) / W;
    const uint32_t magic_L = 65536u / (uint32_t)L + 1u;
    hipLaunchKernelGGL((rpe_fill_kernel<E, W>), dim3((unsigned)blocks), dim3(W * kWave), lds_bytes,
                       stream, walks, n_seeds, M, m, n_nodes, magic_L, rpe_off, cap_rows, ids, cnt,
                       err);
    return hipGetLastError();
}

template <int E>
static hipError_t launch_rpe_fill_e(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                                    int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes,
                                    const int64_t* rpe_off, int64_t cap_rows, int32_t* ids,
                                    uint16_t* cnt, uint32_t* err) {
    const size_t per_wave = (size_t)(kWave * E) * (4 + 2 * (m + 1));
#define SUREL_RPE_W(W_)                                                                        \
    if (per_wave * (W_) <= (size_t)max_lds_bytes)                                              \
        return launch_rpe_fill_ew<E, W_>(stream, walks, n_seeds, M, m, n_nodes, rpe_off, cap_rows, \
                                         ids, cnt, err);
    SUREL_RPE_W(4)
    SUREL_RPE_W(2)
    SUREL_RPE_W(1)
#undef SUREL_RPE_W
    return hipErrorInvalidValue;
}

hipError_t launch_rpe_fill(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                           int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes,
                           const int64_t* rpe_off, int64_t cap_rows, int32_t* ids, uint16_t* cnt,
                           uint32_t* err) {
    if (n_seeds == 0) return hipSuccess;
    const int n_key = M * (m + 1);
#define SUREL_RPE_CASE(E_)                                                                       \
    if (n_key <= kWave * (E_))                                                                   \
        return launch_rpe_fill_e<E_>(stream, max_lds_bytes, walks, n_seeds, M, m, n_nodes, rpe_off, \
                                     cap_rows, ids, cnt, err);
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
