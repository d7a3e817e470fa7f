// Query-level RPE-IDs per walk position (Sec. 3.4, the form the section describes first): the
// walks W_u, u in Q, are concatenated and every node occurrence x in them gets
// RPE-ID_{Q,x} = [RPE-ID_{u,x}]_{u in Q}.  The RPE table is the (unpruned) central array of
// Sec. 3.3, so RPE-ID_{u,x} is the index of (u, x)'s row in it; -1 stands for "x is not in
// V_u" (the all-zero vector).  The paper looks x up in the hash dictionary H_u; here the
// blocks' id lists are sorted, so the lookup is a binary search in LDS.  (Per-query hash
// dictionaries in LDS were measured too and lost: their probe loops diverge, and their
// footprint leaves a compute unit too few waves.)
//
// A wavefront handles one query (the grid covers the query list; a wave loops only where the
// grid cannot be that large).  It stages the K id lists in LDS, then runs over the K walk
// blocks as flat arrays: a lane takes kQiEntries walk entries at a time and searches each in
// all K lists with a fixed number of branch-free steps, so that the K * kQiEntries searches
// of a round advance together and their LDS reads overlap; the K row indices of an entry lie
// next to each other in the output and go out as one store.  The first round of every walk
// block (the whole block, for up to 512 entries) is loaded before the id lists are staged:
// a query then costs one wait for memory, not one per block.
#include "device_util.h"
#include "kernels.h"

namespace surel {

// The K row indices of one walk entry (4-byte aligned, written with one store).
template <int K>
struct __attribute__((aligned(4))) RowIds {
    int32_t v[K];
};

// kQiEntries: walk entries a lane looks up at a time (1, 2, 4 or 8: enough for a whole walk block
// of up to 512 entries in one round).
// kCode: the rows' codes (their RPE-IDs in the pruned array of Sec. 3.3) are staged next to the
// ids and go out instead of the row indices.
template <int K, int WPB, int kQiEntries, bool kCode>
__global__ __launch_bounds__(WPB* kWave) void query_ids_kernel(
    const int32_t* __restrict__ walks, const int64_t* __restrict__ rpe_off,
    const int32_t* __restrict__ rpe_ids, const int32_t* __restrict__ code, int64_t n_blocks,
    int32_t n_key, int32_t max_set,
    int64_t table_rows, const int32_t* __restrict__ queries, int64_t n_queries,
    int32_t* __restrict__ out, uint32_t* __restrict__ err) {
    extern __shared__ uint32_t lds32[];
    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // list j at [j*(max_set+1) + 1 ...); the word in front of it (index -1 of the list) is
    // never smaller than a node id, so a search may read it
    const int list_stride = max_set + 1;
    uint32_t* ids_lds = lds32 + wave * ((kCode ? 2 : 1) * K * list_stride);
    uint32_t* code_lds = ids_lds + K * list_stride;  // same places as the ids (kCode only)
    const int64_t stride = (int64_t)gridDim.x * WPB;
    for (int64_t q = (int64_t)blockIdx.x * WPB + wave; q < n_queries; q += stride) {
        // the K blocks of this query (wave-uniform)
        int32_t blk[K];
        int64_t lo[K];
        int n[K];
        uint32_t problem = 0;
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int32_t b = queries[q * K + j];
            blk[j] = 0;
            lo[j] = 0;
            n[j] = 0;
            if (b < 0 || (int64_t)b >= n_blocks) {
                problem |= kDevBadQuery;
            } else {
                const int64_t a = rpe_off[b];
                const int64_t len = rpe_off[b + 1] - a;
                if (a < 0 || len < 0 || a + len > table_rows) {
                    problem |= kDevBadTable;
                } else if (len > (int64_t)max_set) {
                    problem |= kDevSetTooLarge;
                } else {
                    blk[j] = b;
                    lo[j] = a;
                    n[j] = (int)len;
                }
            }
        }
        int32_t* out_q = out + q * (int64_t)K * n_key * K;
        if (problem != 0) {
            // the query gets no RPE-IDs at all
            if (lane == 0) atomicOr(err, problem);
            for (int t = lane; t < K * n_key * K; t += kWave) out_q[t] = -1;
            continue;
        }
        // the first kQiEntries * 64 entries of every walk block (all of it, for the usual sizes)
        // are asked for before the id lists, so that one wait covers both
        uint32_t x_first[K][kQiEntries];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int32_t* W = walks + (int64_t)blk[j] * n_key;
#pragma unroll
            for (int e = 0; e < kQiEntries; ++e)
                x_first[j][e] = (uint32_t)__builtin_nontemporal_load(W + min(e * kWave + lane, n_key - 1));
        }
        int top[K];  // largest power of two <= n[j] (0 for an empty list): the first step
        if constexpr (!kCode) {
            // ids only: list after list (asking for all of them together was measured and is
            // 5 % slower here, though it is what makes the variant with codes fast)
#pragma unroll
            for (int j = 0; j < K; ++j)
                stage_words<8>(ids_lds + j * list_stride + 1,
                               reinterpret_cast<const uint32_t*>(rpe_ids + lo[j]), n[j], lane);
        }
        // with codes: the lists' first 512 entries (all of them, usually) are asked for together,
        // ids and codes of all K blocks, before any of them is waited for
        constexpr int kStageU = 8;
        constexpr int kLists = kCode ? 2 * K : 0;
        uint32_t staged[kLists > 0 ? kLists : 1][kStageU];
#pragma unroll
        for (int l = 0; l < kLists; ++l) {
            const int j = l % K;
            const int32_t* from = (l < K ? rpe_ids : code) + lo[j];
#pragma unroll
            for (int u = 0; u < kStageU; ++u) {
                const int t = u * kWave + lane;
                staged[l][u] = t < n[j] ? (uint32_t)from[t] : 0u;
            }
        }
#pragma unroll
        for (int l = 0; l < kLists; ++l) {
            const int j = l % K;
            uint32_t* to = (l < K ? ids_lds : code_lds) + j * list_stride + 1;
#pragma unroll
            for (int u = 0; u < kStageU; ++u) {
                const int t = u * kWave + lane;
                if (t < n[j]) to[t] = staged[l][u];
            }
            if (n[j] > kStageU * kWave)  // the rest of a long list
                stage_words<8>(to + kStageU * kWave,
                               reinterpret_cast<const uint32_t*>((l < K ? rpe_ids : code) + lo[j]) +
                                   kStageU * kWave,
                               n[j] - kStageU * kWave, lane);
        }
#pragma unroll
        for (int j = 0; j < K; ++j) {
            if (lane == 0) ids_lds[j * list_stride] = 0xFFFFFFFFu;
            top[j] = n[j] > 0 ? 1 << (31 - __builtin_clz((unsigned)n[j])) : 0;
        }
        int top_max = 0;
#pragma unroll
        for (int j = 0; j < K; ++j) top_max = max(top_max, top[j]);
        wave_sync();
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const int32_t* W = walks + (int64_t)blk[j] * n_key;
            int32_t* out_j = out_q + (int64_t)j * n_key * K;
            for (int t0 = 0; t0 < n_key; t0 += kQiEntries * kWave) {
                uint32_t x[kQiEntries];
                int pos[kQiEntries][K];  // elements of list j2 that are smaller than x
#pragma unroll
                for (int e = 0; e < kQiEntries; ++e) {
                    const int t = min(t0 + e * kWave + lane, n_key - 1);
                    x[e] = t0 == 0 ? x_first[j][e] : (uint32_t)__builtin_nontemporal_load(W + t);
#pragma unroll
                    for (int j2 = 0; j2 < K; ++j2) pos[e][j2] = 0;
                }
                for (int step = top_max; step > 0; step >>= 1) {
#pragma unroll
                    for (int e = 0; e < kQiEntries; ++e) {
#pragma unroll
                        for (int j2 = 0; j2 < K; ++j2) {
                            // a step past the end of the list reads its last element again
                            // (or the guard word of an empty list) and is not taken
                            const int cand = pos[e][j2] + step;
                            const uint32_t probe =
                                ids_lds[j2 * list_stride + min(cand, n[j2])];
                            if (cand <= n[j2] && probe < x[e]) pos[e][j2] = cand;
                        }
                    }
                }
#pragma unroll
                for (int e = 0; e < kQiEntries; ++e) {
                    const int t = t0 + e * kWave + lane;
                    int32_t row[K];
#pragma unroll
                    for (int j2 = 0; j2 < K; ++j2) {
                        const int p = pos[e][j2];
                        const uint32_t at = ids_lds[j2 * list_stride + 1 + min(p, max(n[j2] - 1, 0))];
                        const bool found = p < n[j2] && at == x[e];
                        if constexpr (kCode) {
                            const uint32_t c = code_lds[j2 * list_stride + 1 + min(p, max(n[j2] - 1, 0))];
                            row[j2] = found ? (int32_t)c : -1;
                        } else {
                            row[j2] = found ? (int32_t)(lo[j2] + p) : -1;
                        }
                    }
                    if (t < n_key) {
                        // the K indices of an entry as one 4*K-byte store
                        RowIds<K> ids;
#pragma unroll
                        for (int j2 = 0; j2 < K; ++j2) ids.v[j2] = row[j2];
                        *reinterpret_cast<RowIds<K>*>(out_j + (int64_t)t * K) = ids;
                    }
                }
            }
        }
        wave_sync();  // the next query reuses the LDS words
    }
}

template <int K, int WPB, int QE, bool kCode>
static hipError_t launch_query_ids_kwe(hipStream_t stream, const int32_t* walks,
                                      const int64_t* rpe_off, const int32_t* rpe_ids,
                                      const int32_t* code,
                                      int64_t n_blocks, int32_t M, int32_t m, int32_t max_set,
                                      int64_t table_rows, const int32_t* queries,
                                      int64_t n_queries, int32_t* out, uint32_t* err) {
    const size_t lds_bytes = (size_t)WPB * (kCode ? 2 : 1) * K * (max_set + 1) * 4;
    const void* fn = reinterpret_cast<const void*>(query_ids_kernel<K, WPB, QE, kCode>);
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    // a wave per query and the hardware hands the workgroups out (a wave loops only where the
    // grid cannot be that large)
    int64_t blocks = (n_queries + WPB - 1) / WPB;
    if (blocks > 0x7FFFFFFFll) blocks = 0x7FFFFFFFll;
    hipLaunchKernelGGL((query_ids_kernel<K, WPB, QE, kCode>), dim3((unsigned)blocks),
                       dim3(WPB * kWave), lds_bytes, stream, walks, rpe_off, rpe_ids, code, n_blocks,
                       M * (m + 1), max_set,
                       table_rows, queries, n_queries, out, err);
    return hipGetLastError();
}

template <int K, int WPB, bool kCode>
static hipError_t launch_query_ids_kw(hipStream_t stream, const int32_t* walks,
                                      const int64_t* rpe_off, const int32_t* rpe_ids,
                                      const int32_t* code, int64_t n_blocks, int32_t M, int32_t m,
                                      int32_t max_set, int64_t table_rows, const int32_t* queries,
                                      int64_t n_queries, int32_t* out, uint32_t* err) {
    const int64_t n_key = (int64_t)M * (m + 1);
#define SUREL_QI_ENTRIES(QE_)                                                                  \
    return launch_query_ids_kwe<K, WPB, QE_, kCode>(stream, walks, rpe_off, rpe_ids, code, \
                                                    n_blocks, M, m, max_set, table_rows, queries, \
                                                    n_queries, out, err)
    if (n_key <= kWave) SUREL_QI_ENTRIES(1);
    if (n_key <= 2 * kWave) SUREL_QI_ENTRIES(2);
    if (n_key <= 4 * kWave) SUREL_QI_ENTRIES(4);
    SUREL_QI_ENTRIES(8);
#undef SUREL_QI_ENTRIES
}

template <int K, bool kCode>
static hipError_t launch_query_ids_k(hipStream_t stream, int max_lds_bytes,
                                     const int32_t* walks, const int64_t* rpe_off,
                                     const int32_t* rpe_ids, const int32_t* code, int64_t n_blocks,
                                     int32_t M, int32_t m,
                                     int32_t max_set, int64_t table_rows, const int32_t* queries,
                                     int64_t n_queries, int32_t* out, uint32_t* err) {
    const size_t per_wave = (size_t)(kCode ? 2 : 1) * K * (max_set + 1) * 4;
    // waves per workgroup: the choice that lets a compute unit hold the most waves
    int best = 1, best_waves = 0;
    for (int w = 4; w >= 1; w /= 2) {
        const size_t wg = per_wave * w;
        if (wg > (size_t)max_lds_bytes) continue;
        int waves = (int)((size_t)max_lds_bytes / wg) * w;
        if (waves > 32) waves = 32;
        if (waves > best_waves) {
            best_waves = waves;
            best = w;
        }
    }
#define SUREL_QI_CASE(W_)                                                                        \
    if (best == (W_))                                                                            \
        return launch_query_ids_kw<K, W_, kCode>(stream, walks, rpe_off, rpe_ids, code,   \
                                                 n_blocks, M, m, max_set, table_rows, queries,  \
                                                 n_queries, out, err);
    SUREL_QI_CASE(4)
    SUREL_QI_CASE(2)
    SUREL_QI_CASE(1)
#undef SUREL_QI_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_query_ids(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                            const int64_t* rpe_off, const int32_t* rpe_ids, const int32_t* code,
                            int64_t n_blocks,
                            int32_t M, int32_t m, int32_t max_set, int64_t table_rows,
                            const int32_t* queries, int64_t n_queries, int32_t k, int32_t* out,
                            uint32_t* err) {
    if (n_queries == 0) return hipSuccess;
    if ((size_t)(code ? 2 : 1) * k * (max_set + 1) * 4 > (size_t)max_lds_bytes)
        return hipErrorInvalidValue;
#define SUREL_QI_ARGS \
    stream, max_lds_bytes, walks, rpe_off, rpe_ids, code, n_blocks, M, m, max_set, \
        table_rows, queries, n_queries, out, err
    if (k == 2 && !code) return launch_query_ids_k<2, false>(SUREL_QI_ARGS);
    if (k == 3 && !code) return launch_query_ids_k<3, false>(SUREL_QI_ARGS);
    if (k == 2) return launch_query_ids_k<2, true>(SUREL_QI_ARGS);
    if (k == 3) return launch_query_ids_k<3, true>(SUREL_QI_ARGS);
#undef SUREL_QI_ARGS
    return hipErrorInvalidValue;
}

}  // namespace surel
