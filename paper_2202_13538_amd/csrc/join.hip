// Query-based subgraph joining in its set-union form (Sec. 3.4): for a query tuple
// (b_1..b_K) the ascending union of the K node sets, and per union node the K count
// vectors in tuple order, zeros where the node is absent from a set.
//
// Two launches of one kernel: the first only counts every query's union rows, an exclusive
// scan turns the counts into join_off, the second writes the rows.  One wavefront per query.
// The K sorted id lists are staged in LDS.  A node's row
// in the union is owned by the first list that contains it, and its position is a sum of
// ranks:
//   position(x) = #{a in list 0 : a < x} + sum over j >= 1 of #{b in list j : b < x, b not in
//                 an earlier list},
// each term being a lower bound in LDS plus a lookup in a per-list prefix count of "new"
// elements.  This needs no serial merge loop and extends from pairs to triples unchanged.
// Count vectors are then moved 64 union rows at a time: a lane copies
// one (row, list) vector from the table into an LDS tile, and the tile is streamed out as
// whole dwords.
#include "device_util.h"
#include "kernels.h"

namespace surel {

constexpr uint16_t kNoSrc = 0xFFFFu;
constexpr int kJoinChunkRows = 64;  // union rows staged in LDS per output tile

// First index t in [0, n) with list[t] >= x (n if none).  n is wave-uniform.
__device__ __forceinline__ int lower_bound_lds(const uint32_t* list, int n, uint32_t x) {
    int lo = 0;
    int len = n;
    while (len > 0) {
        const int half = len >> 1;
        if (list[lo + half] < x) {
            lo += half + 1;
            len -= half + 1;
        } else {
            len = half;
        }
    }
    return lo;
}

// LDS words one wave needs for tuples of K blocks of at most max_set rows with L counts.
__host__ __device__ constexpr int join_lds_words(int K, int max_set, int L) {
    // ids: K*max_set uint32; new-prefix: (K-1)*(max_set+1) uint16; src: K*(K*max_set) uint16;
    // output tile: kJoinChunkRows*K*L uint16
    return K * max_set + ((K - 1) * (max_set + 1) + 1) / 2 + (K * K * max_set + 1) / 2 +
           (kJoinChunkRows * K * L + 1) / 2;
}

// WPB = waves per workgroup: as many as the LDS a wave needs allows.  kFill = false: write
// counts[q] only; kFill = true: join_off is complete, write the rows.
template <int K, int WPB, bool kFill>
__global__ __launch_bounds__(WPB* kWave) void join_kernel(
    const int64_t* __restrict__ rpe_off, const int32_t* __restrict__ rpe_ids,
    const uint16_t* __restrict__ rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
    const int32_t* __restrict__ queries, int64_t n_queries, int32_t* __restrict__ counts,
    const int64_t* __restrict__ join_off, int64_t cap_rows, int32_t* __restrict__ out_ids,
    uint16_t* __restrict__ out_cnt, uint32_t* __restrict__ err) {
    extern __shared__ uint32_t lds32[];

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t q = (int64_t)blockIdx.x * WPB + wave;
    if (q >= n_queries) return;  // whole waves leave; no block-wide barrier is used below
    constexpr bool has_query = true;
    constexpr bool fill = kFill;

    const int L = m + 1;
    uint32_t* ids_lds = lds32 + wave * join_lds_words(K, max_set, L);          // [K][max_set]
    uint16_t* new_pre = reinterpret_cast<uint16_t*>(ids_lds + K * max_set);     // [K-1][max_set+1]
    uint32_t* src32 = ids_lds + K * max_set + ((K - 1) * (max_set + 1) + 1) / 2;
    uint16_t* src = reinterpret_cast<uint16_t*>(src32);                         // [K][K*max_set]
    uint32_t* tile32 = src32 + (K * K * max_set + 1) / 2;
    uint16_t* tile = reinterpret_cast<uint16_t*>(tile32);                       // [64][K][L]
    const int src_stride = K * max_set;

    int64_t lo[K];
    int n[K];
    int n_out = 0;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        lo[j] = 0;
        n[j] = 0;
    }

    if (has_query) {
        // the K blocks of this query (wave-uniform)
        uint32_t problem = 0;
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int32_t b = queries[q * K + j];
            if (b < 0 || (int64_t)b >= n_blocks) {
                problem |= kDevBadQuery;
            } else {
                const int64_t a = rpe_off[b];
                const int64_t len = rpe_off[b + 1] - a;
                if (a < 0 || len < 0) {
                    problem |= kDevBadTable;
                } else if (len > (int64_t)max_set) {
                    problem |= kDevSetTooLarge;
                } else {
                    lo[j] = a;
                    n[j] = (int)len;
                }
            }
        }
        if (problem != 0) {
            if (lane == 0) atomicOr(err, problem);
#pragma unroll
            for (int j = 0; j < K; ++j) n[j] = 0;  // the query yields no rows
        }

        // stage the id lists
#pragma unroll
        for (int j = 0; j < K; ++j) {
            for (int t = lane; t < n[j]; t += kWave)
                ids_lds[j * max_set + t] = (uint32_t)rpe_ids[lo[j] + t];
        }
        wave_sync();

        // per list j >= 1: exclusive prefix count of elements that no earlier list contains
        n_out = n[0];
#pragma unroll
        for (int j = 1; j < K; ++j) {
            uint16_t* pre = new_pre + (j - 1) * (max_set + 1);
            int carry = 0;
            for (int t0 = 0; t0 < n[j]; t0 += kWave) {
                const int t = t0 + lane;
                bool is_new = false;
                if (t < n[j]) {
                    const uint32_t x = ids_lds[j * max_set + t];
                    is_new = true;
#pragma unroll
                    for (int jj = 0; jj < j; ++jj) {
                        const uint32_t* other = ids_lds + jj * max_set;
                        const int p = lower_bound_lds(other, n[jj], x);
                        if (p < n[jj] && other[p] == x) is_new = false;
                    }
                }
                const uint64_t mask = __ballot(is_new);
                const int before = (int)__builtin_amdgcn_mbcnt_hi(
                    (uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
                if (t < n[j]) pre[t] = (uint16_t)(carry + before);
                carry += __popcll(mask);
            }
            if (lane == 0) pre[n[j]] = (uint16_t)carry;
            n_out += carry;
        }

        if (fill && n_out > 0) {
            wave_sync();
            // every union row is written by the first list that holds its node
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const uint16_t* pre_j = new_pre + (j > 0 ? j - 1 : 0) * (max_set + 1);  // j >= 1 only
                for (int t = lane; t < n[j]; t += kWave) {
                    const uint32_t x = ids_lds[j * max_set + t];
                    if (j > 0 && pre_j[t + 1] == pre_j[t]) continue;  // owned by an earlier list
                    int pos = 0;
                    uint16_t s_idx[K];
#pragma unroll
                    for (int jj = 0; jj < K; ++jj) {
                        if (jj == j) {
                            pos += (j == 0) ? t : (int)pre_j[t];
                            s_idx[jj] = (uint16_t)t;
                        } else {
                            const uint32_t* other = ids_lds + jj * max_set;
                            const int p = lower_bound_lds(other, n[jj], x);
                            pos += (jj == 0) ? p : (int)new_pre[(jj - 1) * (max_set + 1) + p];
                            const bool present = jj > j && p < n[jj] && other[p] == x;
                            s_idx[jj] = present ? (uint16_t)p : kNoSrc;
                        }
                    }
#pragma unroll
                    for (int jj = 0; jj < K; ++jj) src[jj * src_stride + pos] = s_idx[jj];
                }
            }
        }
    }

    if (!kFill) {
        if (lane == 0) counts[q] = n_out;
        return;
    }
    const int64_t off = join_off[q];
    if (n_out == 0) return;
    if (off + n_out > cap_rows) {
        if (lane == 0) atomicOr(err, kDevCapacity);
        return;
    }
    wave_sync();

    const int KL = K * L;
    for (int r0 = 0; r0 < n_out; r0 += kJoinChunkRows) {
        const int rows = min(kJoinChunkRows, n_out - r0);

        // ids of these union rows (any list that holds the node gives the same id)
        if (lane < rows) {
            uint32_t id = 0;
#pragma unroll
            for (int jj = K - 1; jj >= 0; --jj) {
                const uint16_t sj = src[jj * src_stride + r0 + lane];
                if ((int)sj < n[jj]) id = ids_lds[jj * max_set + sj];  // kNoSrc is >= any n
            }
            out_ids[off + r0 + lane] = (int32_t)id;
        }

        // one lane per (row, list): copy that list's count vector, or zeros, into the tile
        for (int t = lane; t < rows * K; t += kWave) {
            const int row = t / K;
            const int j = t - row * K;
            const uint16_t sj = src[j * src_stride + r0 + row];
            int64_t base = lo[0];
            int len = n[0];
#pragma unroll
            for (int jj = 1; jj < K; ++jj) {
                if (j == jj) {
                    base = lo[jj];
                    len = n[jj];
                }
            }
            uint16_t* dst = tile + t * L;
            // kNoSrc is >= any len; the bound also keeps a malformed table from reading outside
            if ((int)sj < len) {
                const uint16_t* from = rpe_cnt + (base + sj) * L;
                for (int s = 0; s < L; ++s) dst[s] = from[s];
            } else {
                for (int s = 0; s < L; ++s) dst[s] = 0;
            }
        }
        wave_sync();

        // stream the tile out as dwords where the destination allows
        const int n_el = rows * KL;
        const int64_t d0 = (off + r0) * KL;  // first destination element (uint16 units)
        const int head = (int)(d0 & 1);
        uint16_t* out = out_cnt + d0;
        if (head && lane == 0) out[0] = tile[0];
        const int n_pair = (n_el - head) / 2;
        uint32_t* out32 = reinterpret_cast<uint32_t*>(out + head);
        if (head == 0) {
            for (int t = lane; t < n_pair; t += kWave) out32[t] = tile32[t];
        } else {
            for (int t = lane; t < n_pair; t += kWave)
                out32[t] = (uint32_t)tile[1 + 2 * t] | ((uint32_t)tile[2 + 2 * t] << 16);
        }
        if (((n_el - head) & 1) && lane == 0) out[n_el - 1] = tile[n_el - 1];
        wave_sync();
    }
}

template <int K, int WPB>
static hipError_t launch_join_kw(hipStream_t stream, const int64_t* rpe_off,
                                 const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                                 int32_t m, int32_t max_set, const int32_t* queries,
                                 int64_t n_queries, int32_t* counts, const int64_t* join_off,
                                 int64_t cap_rows, int32_t* out_ids, uint16_t* out_cnt,
                                 uint32_t* err) {
    const size_t lds_bytes = (size_t)WPB * join_lds_words(K, max_set, m + 1) * 4;
    const void* fn = counts ? reinterpret_cast<const void*>(join_kernel<K, WPB, false>)
                            : reinterpret_cast<const void*>(join_kernel<K, WPB, true>);
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    const dim3 grid((unsigned)((n_queries + WPB - 1) / WPB)), block(WPB * kWave);
    if (counts) {
        hipLaunchKernelGGL((join_kernel<K, WPB, false>), grid, block, lds_bytes, stream, rpe_off,
                           rpe_ids, rpe_cnt, n_blocks, m, max_set, queries, n_queries, counts,
                           join_off, cap_rows, out_ids, out_cnt, err);
    } else {
        hipLaunchKernelGGL((join_kernel<K, WPB, true>), grid, block, lds_bytes, stream, rpe_off,
                           rpe_ids, rpe_cnt, n_blocks, m, max_set, queries, n_queries, counts,
                           join_off, cap_rows, out_ids, out_cnt, err);
    }
    return hipGetLastError();
}

// counts != nullptr: counting launch (writes counts[q]); else: writing launch.
template <int K>
static hipError_t launch_join_k(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                                const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                                int32_t m, int32_t max_set, const int32_t* queries,
                                int64_t n_queries, int32_t* counts, const int64_t* join_off,
                                int64_t cap_rows, int32_t* out_ids, uint16_t* out_cnt,
                                uint32_t* err) {
    const size_t per_wave = (size_t)join_lds_words(K, max_set, m + 1) * 4;
#define SUREL_JOIN_CASE(W_)                                                                    \
    if (per_wave * (W_) <= (size_t)max_lds_bytes)                                              \
        return launch_join_kw<K, W_>(stream, rpe_off, rpe_ids, rpe_cnt, n_blocks, m, max_set,  \
                                     queries, n_queries, counts, join_off, cap_rows, out_ids,  \
                                     out_cnt, err);
    SUREL_JOIN_CASE(4)
    SUREL_JOIN_CASE(2)
    SUREL_JOIN_CASE(1)
#undef SUREL_JOIN_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_join(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                       const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                       int32_t m, int32_t max_set, const int32_t* queries, int64_t n_queries,
                       int32_t k, int32_t* counts, const int64_t* join_off, int64_t cap_rows,
                       int32_t* out_ids, uint16_t* out_cnt, uint32_t* err) {
    if (n_queries == 0) return hipSuccess;
    if (k == 2)
        return launch_join_k<2>(stream, max_lds_bytes, rpe_off, rpe_ids, rpe_cnt, n_blocks, m,
                                max_set, queries, n_queries, counts, join_off, cap_rows, out_ids,
                                out_cnt, err);
    if (k == 3)
        return launch_join_k<3>(stream, max_lds_bytes, rpe_off, rpe_ids, rpe_cnt, n_blocks, m,
                                max_set, queries, n_queries, counts, join_off, cap_rows, out_ids,
                                out_cnt, err);
    return hipErrorInvalidValue;
}

}  // namespace surel
