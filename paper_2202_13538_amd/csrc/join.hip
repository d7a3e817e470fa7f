// Query-based subgraph joining in its set-union form (Sec. 3.4): for a query tuple
// (b_1..b_K) the ascending union of the K node sets, and per union node the K count
// vectors in tuple order, zeros where the node is absent from a set.
//
// One wavefront per query.  The K sorted id lists are staged in LDS.  A node's row in the
// union is owned by the first list that contains it, and its position is a sum of ranks:
//   position(x) = #{a in list 0 : a < x} + sum over j >= 1 of #{b in list j : b < x, b not in
//                 an earlier list},
// each term being a lower bound in LDS plus a lookup in a per-list prefix count of "new"
// elements.  This needs no serial merge loop and extends from pairs to triples unchanged.
// The count vectors are then gathered row by row through the per-row source indices.
#include "device_util.h"
#include "kernels.h"

namespace surel {

constexpr uint16_t kNoSrc = 0xFFFFu;

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

// LDS words one wave needs for tuples of K blocks of at most max_set rows.
__host__ __device__ constexpr int join_lds_words(int K, int max_set) {
    // ids: K*max_set uint32; new-prefix: (K-1)*(max_set+1) uint16; src: K*(K*max_set) uint16
    return K * max_set + ((K - 1) * (max_set + 1) + 1) / 2 + (K * K * max_set + 1) / 2;
}

// WPB = waves per workgroup: as many as the LDS a wave needs allows.
template <int K, int WPB>
__global__ __launch_bounds__(WPB* kWave) void join_kernel(
    const int64_t* __restrict__ rpe_off, const int32_t* __restrict__ rpe_ids,
    const uint16_t* __restrict__ rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
    uint32_t magic_KL, uint32_t magic_L, const int32_t* __restrict__ queries, int64_t n_queries,
    int32_t* __restrict__ counts, const int64_t* __restrict__ join_off, int64_t cap_rows,
    int32_t* __restrict__ out_ids, uint16_t* __restrict__ out_cnt, uint32_t* __restrict__ err) {
    extern __shared__ uint32_t lds32[];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * WPB + wave;
    if (q >= n_queries) return;  // whole waves leave; no block-wide barrier is used below

    const int L = m + 1;
    uint32_t* ids_lds = lds32 + wave * join_lds_words(K, max_set);          // [K][max_set]
    uint16_t* new_pre = reinterpret_cast<uint16_t*>(ids_lds + K * max_set);  // [K-1][max_set+1]
    uint16_t* src = reinterpret_cast<uint16_t*>(
        ids_lds + K * max_set + ((K - 1) * (max_set + 1) + 1) / 2);         // [K][K*max_set]
    const int src_stride = K * max_set;

    // the K blocks of this query (wave-uniform)
    int64_t lo[K];
    int n[K];
    uint32_t problem = 0;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int32_t b = queries[q * K + j];
        lo[j] = 0;
        n[j] = 0;
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
        if (lane == 0) {
            atomicOr(err, problem);
            if (counts != nullptr) counts[q] = 0;
        }
        return;
    }

    // stage the id lists
#pragma unroll
    for (int j = 0; j < K; ++j) {
        for (int t = lane; t < n[j]; t += kWave)
            ids_lds[j * max_set + t] = (uint32_t)rpe_ids[lo[j] + t];
    }
    wave_sync();

    // per list j >= 1: exclusive prefix count of elements that no earlier list contains
    int n_out = n[0];
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
    if (counts != nullptr && lane == 0) counts[q] = n_out;
    if (out_ids == nullptr) return;

    const int64_t off = join_off[q];
    if (off + n_out > cap_rows) {
        if (lane == 0) atomicOr(err, kDevCapacity);
        return;
    }
    if (n_out == 0) return;
    wave_sync();

    // every union row is written by the first list that holds its node
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const uint16_t* pre_j = new_pre + (j > 0 ? j - 1 : 0) * (max_set + 1);  // used for j >= 1 only
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
    wave_sync();

    // ids of the union
    for (int r = lane; r < n_out; r += kWave) {
        uint32_t id = 0;
#pragma unroll
        for (int jj = K - 1; jj >= 0; --jj) {
            const uint16_t sj = src[jj * src_stride + r];
            if ((int)sj < n[jj]) id = ids_lds[jj * max_set + sj];  // kNoSrc is >= any n
        }
        out_ids[off + r] = (int32_t)id;
    }

    // count vectors: element e of the query's output block is (row, j, s)
    const int KL = K * L;
    const int n_cnt = n_out * KL;
    auto fetch = [&](int e) -> uint32_t {
        const int row = (int)div_magic32((uint32_t)e, magic_KL);
        const int c = e - row * KL;
        const int j = (int)div_magic32((uint32_t)c, magic_L);
        const int s = c - j * L;
        const uint16_t sj = src[j * src_stride + row];
        int64_t base = lo[0];
        int len = n[0];
#pragma unroll
        for (int jj = 1; jj < K; ++jj) {
            if (j == jj) {
                base = lo[jj];
                len = n[jj];
            }
        }
        // kNoSrc is >= any len; the bound also keeps a malformed table from reading outside
        return (int)sj < len ? (uint32_t)rpe_cnt[(base + sj) * L + s] : 0u;
    };
    const int64_t d0 = off * KL;  // first destination element (uint16 units)
    const int head = (int)(d0 & 1);
    uint16_t* dst = out_cnt + d0;
    if (head && lane == 0) dst[0] = (uint16_t)fetch(0);
    const int n_pair = (n_cnt - head) / 2;
    uint32_t* dst32 = reinterpret_cast<uint32_t*>(dst + head);
    for (int t = lane; t < n_pair; t += kWave) {
        const uint32_t a = fetch(head + 2 * t);
        const uint32_t b = fetch(head + 2 * t + 1);
        dst32[t] = a | (b << 16);
    }
    if (((n_cnt - head) & 1) && n_cnt > 0 && lane == 0) dst[n_cnt - 1] = (uint16_t)fetch(n_cnt - 1);
}

template <int K, int WPB>
static hipError_t launch_join_kw(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                                const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                                int32_t m, int32_t max_set, const int32_t* queries,
                                int64_t n_queries, int32_t* counts, const int64_t* join_off,
                                int64_t cap_rows, int32_t* out_ids, uint16_t* out_cnt,
                                uint32_t* err) {
    const int L = m + 1;
    const size_t lds_bytes = (size_t)WPB * join_lds_words(K, max_set) * 4;
    if (lds_bytes > (size_t)max_lds_bytes) return hipErrorInvalidValue;
    if (lds_bytes > 64 * 1024) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(join_kernel<K, WPB>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    const int64_t blocks = (n_queries + WPB - 1) / WPB;
    const uint32_t magic_KL = (uint32_t)(0x100000000ull / (uint64_t)(K * L)) + 1u;
    const uint32_t magic_L = (uint32_t)(0x100000000ull / (uint64_t)L) + 1u;
    hipLaunchKernelGGL((join_kernel<K, WPB>), dim3((unsigned)blocks), dim3(WPB * kWave),
                       lds_bytes, stream, rpe_off, rpe_ids, rpe_cnt, n_blocks, m, max_set,
                       magic_KL, magic_L, queries, n_queries, counts, join_off, cap_rows, out_ids,
                       out_cnt, err);
    return hipGetLastError();
}

template <int K>
static hipError_t launch_join_k(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                                const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                                int32_t m, int32_t max_set, const int32_t* queries,
                                int64_t n_queries, int32_t* counts, const int64_t* join_off,
                                int64_t cap_rows, int32_t* out_ids, uint16_t* out_cnt,
                                uint32_t* err) {
    const size_t per_wave = (size_t)join_lds_words(K, max_set) * 4;
#define SUREL_JOIN_CASE(W_)                                                                     \
    if (per_wave * (W_) <= (size_t)max_lds_bytes)                                               \
        return launch_join_kw<K, W_>(stream, max_lds_bytes, rpe_off, rpe_ids, rpe_cnt, n_blocks, \
                                     m, max_set, queries, n_queries, counts, join_off, cap_rows, \
                                     out_ids, out_cnt, err);
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
