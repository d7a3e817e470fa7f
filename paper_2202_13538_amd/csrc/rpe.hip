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
#include "rpe_rows.h"
#include "wave_sort.h"
#include "kernels.h"

namespace surel {

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
        bool active = t < n_key;
        const int32_t v = active ? __builtin_nontemporal_load(W + t) : 0;
        if ((uint32_t)v >= (uint32_t)n_nodes) {  // not a node: flagged and left out
            bad_walk = true;
            active = false;
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
            const int32_t v = __builtin_nontemporal_load(W + idx);
            const uint32_t s = (uint32_t)idx - small_div((uint32_t)idx, magic_L) * (uint32_t)L;
            x[r] = ((uint32_t)v << 4) | s;
            if ((uint32_t)v >= (uint32_t)n_nodes) {  // not a node: flagged and left out
                bad_walk = true;
                x[r] = kPadKey;
            }
        } else {
            x[r] = kPadKey;
        }
    }
    raise_error(err, bad_walk, kDevBadWalk);

    wave_sort<E>(x, lane);

    const RpeRowScan sc = rpe_scan_rows<E>(x, lane);

    // the layout was made from set sizes; a size that does not match the walks (sizes passed
    // in for other walks) must not make blocks overlap
    if ((int64_t)sc.n_rows != given_rows) {
        if (lane == 0) atomicOr(err, kDevBadSizes);
        return;
    }
    if (off + sc.n_rows > cap_rows) {
        if (lane == 0) atomicOr(err, kDevCapacity);
        return;
    }
    rpe_write_rows<E>(x, sc, lane, L, ids_lds, cnt_lds32, off, ids, cnt);
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
