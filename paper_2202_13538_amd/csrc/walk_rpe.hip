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
// Where a seed's rows go is a prefix sum over all earlier seeds.  The kernel is persistent and
// uses the worker / scanner scheme of lookback.h: workers take seeds in increasing order, a
// worker publishes a seed's row count as soon as the sort has it, keeps the sorted keys in
// registers, and only writes the rows out after it has walked and sorted its NEXT seed: by then
// the scanner wave has long published the offset, so nobody waits in practice.  Why every wait
// ends, and how waits are bounded, is argued in lookback.h.
#include "device_util.h"
#include "kernels.h"
#include "lookback.h"
#include "prune_set.h"
#include "rpe_rows.h"
#include "walk_core.h"
#include "wave_sort.h"

namespace surel {

constexpr int kFusedChains = 2;  // walks a lane moves at a time

// The hash set of distinct count vectors that a kernel with kCodes feeds (prune_set.h).
struct CodeSet {
    int32_t* code;                      // int32 per table row: the row's slot number
    uint32_t* slots;
    uint32_t slot_mask;
    int64_t cap_T;
    unsigned long long* n_inserted;
};

// E = sort keys per lane (64*E >= M*(m+1)).  The waves of a workgroup share the LDS
// allocation and the chunk word (with kCodes also a cache of the hash set), nothing else.
// kCodes: every finished row's count vector is looked up in the hash set while the row still
// lies in LDS (Algorithm 1's last step, pruning, done on the fly as well), and its slot number
// goes to cs.code; cnt may then be null.
// The codes of a seed's rows while they lie in LDS (cnt_lds32: the rows' 16-bit counts, densely
// packed): a lane per row reads its vector as the aligned words that cover it, shifts it into
// place, turns it into the set's word form (entry 2k in the upper half of word k, absent entries
// zero) and looks it up.  LT = m + 1 at compile time for 2 .. 6 (packed cache entries), 0 = any.
template <int LT>
__device__ __forceinline__ void row_codes(int n_rows, int lane, int L, const uint32_t* cnt_lds32,
                                          int64_t off, uint32_t* set_cache, const CodeSet& cs,
                                          uint32_t spin_limit, uint32_t* __restrict__ err) {
    const int n_words = (n_rows * L + 1) / 2;  // words the rows occupy in LDS
    for (int t = lane; t < n_rows; t += kWave) {
        const int first = t * L;
        const uint32_t shift = (uint32_t)(first & 1) * 2u;
        if constexpr (LT > 0) {
            constexpr int NW = (LT + 1) / 2;
            uint32_t raw[NW + 1];
#pragma unroll
            for (int k = 0; k <= NW; ++k)
                raw[k] = 2 * k <= LT ? cnt_lds32[min((first >> 1) + k, n_words - 1)] : 0u;
            uint32_t w[NW];
#pragma unroll
            for (int k = 0; k < NW; ++k) {
                // entries 2k (low half) and 2k+1 (high half) as they lie in memory
                uint32_t pair = __builtin_amdgcn_alignbyte(raw[k + 1], raw[k], shift);
                if (2 * k + 1 >= LT) pair &= 0xFFFFu;  // the high half is the next row's
                w[k] = (pair << 16) | (pair >> 16);
            }
            cs.code[off + t] = prune_lookup_packed<NW>(w, set_cache, cs.slots, cs.slot_mask,
                                                       cs.cap_T, cs.n_inserted, spin_limit, err);
        } else {
            uint32_t raw[kMaxVecWords + 1];
#pragma unroll
            for (int k = 0; k <= kMaxVecWords; ++k)
                raw[k] = 2 * k <= L ? cnt_lds32[min((first >> 1) + k, n_words - 1)] : 0u;
            uint32_t w[kMaxVecWords];
#pragma unroll
            for (int k = 0; k < kMaxVecWords; ++k) {
                uint32_t pair = __builtin_amdgcn_alignbyte(raw[k + 1], raw[k], shift);
                if (2 * k + 1 >= L) pair &= 0xFFFFu;
                if (2 * k >= L) pair = 0u;
                w[k] = (pair << 16) | (pair >> 16);
            }
            cs.code[off + t] = prune_lookup_any(w, (L + 1) / 2, set_cache, cs.slots, cs.slot_mask,
                                                cs.cap_T, cs.n_inserted, spin_limit, err);
        }
    }
}

template <int E, int kRec, bool kCodes>
__global__ __launch_bounds__(1024) void walk_rpe_kernel(
    const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
    const void* __restrict__ rec, int id_bits, int lo_bits, int32_t n_nodes, int64_t n_edges,
    const int32_t* __restrict__ seeds, int64_t n_seeds, int32_t M, int32_t m, uint32_t key0,
    uint32_t key1, uint32_t magic_L, int32_t* __restrict__ walks, int64_t cap_rows,
    int64_t* __restrict__ rpe_off, int32_t* __restrict__ ids, uint16_t* __restrict__ cnt,
    int32_t lds_words_per_wave, uint64_t* __restrict__ lb, uint32_t spin_limit,
    uint32_t* __restrict__ err, CodeSet cs) {
    extern __shared__ uint32_t lds32[];
    __shared__ unsigned long long chunk;
    __shared__ __align__(16) uint32_t set_cache[kCodes ? kFusedCacheWords : 1];

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (threadIdx.x == 0) chunk = 0ull;  // empty
    if constexpr (kCodes) fused_cache_clear_all(set_cache, (int)threadIdx.x, (int)blockDim.x);
    __syncthreads();                     // the only workgroup-wide barrier of the kernel
    const LookbackScratch scr = lookback_scratch(n_seeds);
    int64_t* base = lookback_base(lb);
    uint16_t* status = lookback_status(lb, scr);
    if (wave_draw(lb + 1, lane) == 0) {
        scan_counts(status, scr.n_groups, base, rpe_off + n_seeds, spin_limit, err, lane);
        return;
    }

    const int L = m + 1;
    const int n_key = M * L;  // <= 64*E, checked by the host
    // the seed's walks [M][L] while it is walked, the rows of the seed before while they go out
    uint32_t* wave_lds = lds32 + wave * lds_words_per_wave;
    int32_t* block = reinterpret_cast<int32_t*>(wave_lds);
    const WalkGraph g{row_ptr, col_idx, rec, id_bits, lo_bits, n_nodes, n_edges};

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
            uint32_t* ids_lds = wave_lds;
            uint32_t* cnt_lds32 = wave_lds + sc.n_rows;
            rpe_assemble_rows<E>(x, sc, lane, L, ids_lds, cnt_lds32);
            if constexpr (kCodes) {
                // a lane per row: its slot in the set of distinct vectors
                switch (L) {
                    case 2: row_codes<2>(sc.n_rows, lane, L, cnt_lds32, off, set_cache, cs, spin_limit, err); break;
                    case 3: row_codes<3>(sc.n_rows, lane, L, cnt_lds32, off, set_cache, cs, spin_limit, err); break;
                    case 4: row_codes<4>(sc.n_rows, lane, L, cnt_lds32, off, set_cache, cs, spin_limit, err); break;
                    case 5: row_codes<5>(sc.n_rows, lane, L, cnt_lds32, off, set_cache, cs, spin_limit, err); break;
                    case 6: row_codes<6>(sc.n_rows, lane, L, cnt_lds32, off, set_cache, cs, spin_limit, err); break;
                    default: row_codes<0>(sc.n_rows, lane, L, cnt_lds32, off, set_cache, cs, spin_limit, err); break;
                }
            }
            rpe_stream_rows(sc.n_rows, lane, L, ids_lds, cnt_lds32, off, ids, cnt);
        }
        wave_sync();  // the LDS words are free again
        return true;
    };

    for (;;) {
        const int64_t i = take_item<kGroup>(&chunk, lb, lane);
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
        const int32_t *col_idx, const EdgeRecords &rec, int32_t n_nodes, int64_t n_edges,          \
        const int32_t *seeds, int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,           \
        int32_t *walks, int64_t cap_rows, int64_t *rpe_off, int32_t *ids, uint16_t *cnt,          \
        uint64_t *lb, uint32_t spin_limit, uint32_t *err, const CodeSet &cs
#define SUREL_WR_ARGS                                                                             \
    stream, max_lds_bytes, n_cu, row_ptr, col_idx, rec, n_nodes, n_edges, seeds, n_seeds, M, m,   \
        rng_seed, walks, cap_rows, rpe_off, ids, cnt, lb, spin_limit, err, cs

template <int E, int kRec, bool kCodes>
static hipError_t launch_walk_rpe_erc(SUREL_WR_PARAMS) {
    const int words = walk_rpe_lds_words(M, m);
    const size_t per_wave = (size_t)words * 4;
    const size_t static_lds = 1024 + (kCodes ? (size_t)kFusedCacheWords * 4 : 0);
    const void* fn = reinterpret_cast<const void*>(walk_rpe_kernel<E, kRec, kCodes>);
    // A workgroup has as many waves as LDS (160 KB) and registers allow a compute unit, 16 at
    // most, so that a compute unit holds one such workgroup (two, where 32 waves fit).
    // (Kernels with few registers could have 20 or 24 waves in two or more smaller workgroups,
    // and were measured with them on the 2.9M-node graph: M = 50, m = 4, where 20 waves fit,
    // takes 8.2 ms as one workgroup of 16, 9.1 as two of 8, 11.9 as five of 4, and 11.3 as two
    // of 10, of which the second never starts beside the first: a workgroup's waves go to the
    // four SIMDs in turn, and two of 10 ask two of the SIMDs for six waves when five fit.
    // M = 25: 6.7 ms as 16, 6.9 as two of 12.  Only at M = 12 are two of 12 ahead, 5.4 against
    // 5.6 ms.)
    hipFuncAttributes attr;
    hipError_t rc = hipFuncGetAttributes(&attr, fn);
    if (rc != hipSuccess) return rc;
    const int regs = attr.numRegs > 0 ? attr.numRegs : 128;
    constexpr int kMaxW = 16;
    int cu_waves = 4 * (512 / ((regs + 7) / 8 * 8));
    const int by_lds = (int)((160 * 1024 - static_lds) / per_wave);
    if (cu_waves > by_lds) cu_waves = by_lds;
    if (cu_waves > kMaxW) cu_waves = kMaxW;
    int W = cu_waves;
    if (W < 1) {  // what one workgroup may have (the checks below turn down what does not fit)
        W = (int)(((size_t)max_lds_bytes - static_lds) / per_wave);
        if (W > kMaxW) W = kMaxW;
    }
    if (W < 1) return hipErrorInvalidValue;
    const size_t lds_bytes = (size_t)W * per_wave;
    if (lds_bytes + static_lds > (size_t)max_lds_bytes) return hipErrorInvalidValue;
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

    rc = launch_lookback_clear(stream, lb, n_seeds, rpe_off + n_seeds);
    if (rc != hipSuccess) return rc;
    const uint32_t magic_L = 65536u / (uint32_t)(m + 1) + 1u;
    hipLaunchKernelGGL((walk_rpe_kernel<E, kRec, kCodes>), dim3((unsigned)blocks), dim3(W * kWave),
                       lds_bytes, stream, row_ptr, col_idx, rec.data, rec.id_bits, rec.lo_bits, n_nodes,
                       n_edges, seeds, n_seeds, M,
                       m, (uint32_t)(rng_seed & 0xFFFFFFFFull), (uint32_t)(rng_seed >> 32), magic_L,
                       walks, cap_rows, rpe_off, ids, cnt, words, lb, spin_limit, err, cs);
    return hipGetLastError();
}

template <int E, int kRec>
static hipError_t launch_walk_rpe_er(SUREL_WR_PARAMS) {
    if (cs.code != nullptr) return launch_walk_rpe_erc<E, kRec, true>(SUREL_WR_ARGS);
    return launch_walk_rpe_erc<E, kRec, false>(SUREL_WR_ARGS);
}

template <int E>
static hipError_t launch_walk_rpe_e(SUREL_WR_PARAMS) {
    if (rec.data == nullptr) return launch_walk_rpe_er<E, kRecNone>(SUREL_WR_ARGS);
    if (rec.format == kRecPacked) return launch_walk_rpe_er<E, kRecPacked>(SUREL_WR_ARGS);
    return launch_walk_rpe_er<E, kRecWide>(SUREL_WR_ARGS);
}

hipError_t launch_walk_rpe(hipStream_t stream, int max_lds_bytes, int n_cu, const int32_t* row_ptr,
                           const int32_t* col_idx, int32_t n_nodes, int64_t n_edges,
                           const int32_t* seeds, int64_t n_seeds, int32_t M, int32_t m,
                           uint64_t rng_seed, int32_t* walks, int64_t cap_rows, int64_t* rpe_off,
                           int32_t* ids, uint16_t* cnt, const EdgeRecords& rec, uint64_t* lb,
                           uint32_t spin_limit, uint32_t* err, int32_t* code, uint32_t* slots,
                           int64_t cap_T, unsigned long long* counters) {
    const CodeSet cs{code, slots, code ? prune_slot_mask(cap_T) : 0u, cap_T, counters};
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
