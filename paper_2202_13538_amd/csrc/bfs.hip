// Mini-batches by breadth-first search over nodes that share queries (Sec. 3.6 "Mini-batching
// for Training"; Algorithm 2, the BFS step).  One workgroup (four wavefronts, or one for small
// batches) builds one mini-batch; a launch builds many (the iterations of Algorithm 2 draw their seed-sets independently).
//
// The search is the first-in first-out one: the node set V̄ is its own queue, a node's queries
// are taken in ascending index, a query's nodes in tuple order, and a query enters the batch
// together with all its nodes or ends the search.  The workgroup reproduces that order without
// walking the queue one node at a time: it takes the next stretch of the queue whose query
// lists hold at most a chunk of entries (1,024, fewer for small batches), numbers those
// entries ("candidates") in queue order,
// and lets every query keep the smallest candidate number that names it (atomic minimum in a
// hash table).  The candidates that kept their query are the newly reached queries, in the
// order the queue would have reached them; their nodes are numbered (query's place, position
// in the tuple) and settled the same way.  Prefix sums then give every new query and node its
// place, and the limits B1, B2 cut the stretch exactly where the queue would have stopped.
#include "device_util.h"
#include "kernels.h"

namespace surel {

namespace {

constexpr int kBfsPer = 4;        // candidates (or new queries) per thread
constexpr int kBfsMaxThreads = 256;  // a workgroup has 256 threads, or 64 for small batches
constexpr int kBfsMaxChunk = kBfsMaxThreads * kBfsPer;  // candidates settled at a time, at most
constexpr int kBfsMaxK = 3;
constexpr uint32_t kBfsEmpty = 0xFFFFFFFFu;

__device__ __forceinline__ uint32_t bfs_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// A value read that sees what atomics of other waves have left in the table.
__device__ __forceinline__ uint32_t table_load(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Open addressing over (key, value) pairs: finds or claims the slot of `key` and lowers its
// value to `val` if that is smaller.  Returns the slot, or kBfsEmpty if no slot was found
// within the table (cannot happen while the table is at most half full).
__device__ __forceinline__ uint32_t insert_min(uint32_t* tab, uint32_t mask, uint32_t key,
                                               uint32_t val) {
    uint32_t h = bfs_hash(key) & mask;
    for (uint32_t probe = 0; probe <= mask; ++probe) {
        const uint32_t seen = atomicCAS(&tab[2 * h], kBfsEmpty, key);
        if (seen == kBfsEmpty || seen == key) {
            atomicMin(&tab[2 * h + 1], val);
            return h;
        }
        h = (h + 1) & mask;
    }
    return kBfsEmpty;
}

// Exclusive prefix sum of one value per thread over the workgroup of T threads; *total = the sum.
template <int T>
__device__ __forceinline__ uint32_t bfs_block_scan(uint32_t v, uint32_t* total, uint32_t* wave_sums) {
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_sum(v);
    __syncthreads();  // wave_sums may still be read from the previous scan
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < T / kWave; ++w) {
        if (w < wave) base += wave_sums[w];
        sum += wave_sums[w];
    }
    *total = sum;
    return base + incl - v;
}

struct BfsArgs {
    const int32_t* __restrict__ queries;
    int64_t n_queries;
    int32_t k;
    int32_t n_nodes;
    const int64_t* __restrict__ inc_off;
    const int32_t* __restrict__ inc_q;
    const int32_t* __restrict__ start;   // [n_batches][n_start]
    int64_t n_batches;
    int32_t n_start;
    int32_t B1, B2;
    int32_t* __restrict__ vbar;          // [n_batches][B1]
    int32_t* __restrict__ batch;         // [n_batches][B2]
    int32_t* __restrict__ tuples;        // [n_batches][B2][k] or null
    int32_t* __restrict__ counts;        // [n_batches][2]
    uint32_t* tables;                    // per workgroup: query table, node table
    uint32_t slots_q, slots_v;           // powers of two
    uint32_t chunk;                      // candidates settled at a time: at most four per thread
    uint32_t* err;
};

template <int T>
__global__ __launch_bounds__(T) void bfs_batch_kernel(BfsArgs a) {
    constexpr int kChunk = T * kBfsPer;          // a.chunk <= kChunk
    __shared__ uint32_t wave_sums[T / kWave];
    __shared__ uint32_t pre[T + 1];              // candidates before each node of the stretch
    __shared__ uint32_t cand_q[kChunk];          // query of each candidate
    __shared__ uint32_t cand_slot[kChunk];       // its slot in the query table
    __shared__ uint32_t new_q[kChunk];           // newly reached queries, in order
    __shared__ uint32_t node_slot[kChunk * kBfsMaxK];
    __shared__ uint32_t s_take;

    const int tid = threadIdx.x;
    const int k = a.k;
    uint32_t* q_tab = a.tables + (size_t)blockIdx.x * 2u * ((size_t)a.slots_q + a.slots_v);
    uint32_t* v_tab = q_tab + 2u * (size_t)a.slots_q;
    const uint32_t q_mask = a.slots_q - 1u, v_mask = a.slots_v - 1u;
    const int64_t n_entries = a.n_queries * k;
    bool bad_id = false, bad_lists = false, table_full = false;

    for (int64_t b = blockIdx.x; b < a.n_batches; b += gridDim.x) {
        int32_t* vbar = a.vbar + b * a.B1;
        int32_t* batch = a.batch + b * a.B2;
        int32_t* tuples = a.tuples ? a.tuples + b * (int64_t)a.B2 * k : nullptr;
        const int32_t* start = a.start + b * (int64_t)a.n_start;

        // both tables empty (they lie back to back; 16 bytes a store)
        uint4* clear = reinterpret_cast<uint4*>(q_tab);
        for (uint32_t i = tid; i < (a.slots_q + a.slots_v) / 2u; i += T)
            clear[i] = make_uint4(kBfsEmpty, kBfsEmpty, kBfsEmpty, kBfsEmpty);
        __threadfence();
        __syncthreads();

        uint32_t n_v = 0, n_b = 0;
        // the seed-set: distinct start nodes in the order given, B1 at most
        for (int32_t s0 = 0; s0 < a.n_start && n_v < (uint32_t)a.B1; s0 += kChunk) {
            uint32_t slot[kBfsPer];
            int32_t node[kBfsPer];
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const int32_t i = s0 + tid * kBfsPer + r;
                slot[r] = kBfsEmpty;
                node[r] = -1;
                if (i < a.n_start) {
                    node[r] = start[i];
                    if ((uint32_t)node[r] < (uint32_t)a.n_nodes) {
                        slot[r] = insert_min(v_tab, v_mask, (uint32_t)node[r], (uint32_t)i);
                        table_full |= slot[r] == kBfsEmpty;
                    } else {
                        bad_id = true;
                    }
                }
            }
            __syncthreads();
            uint32_t own = 0;
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const int32_t i = s0 + tid * kBfsPer + r;
                const bool mine = slot[r] != kBfsEmpty && table_load(&v_tab[2 * slot[r] + 1]) == (uint32_t)i;
                own |= mine ? 1u << r : 0u;
            }
            uint32_t total;
            uint32_t at = n_v + bfs_block_scan<T>((uint32_t)__popc(own), &total, wave_sums);
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r)
                if (own & (1u << r)) {
                    if (at < (uint32_t)a.B1) vbar[at] = node[r];
                    at += 1;
                }
            n_v = min(n_v + total, (uint32_t)a.B1);
            __syncthreads();
        }

        bool done = n_v == (uint32_t)a.B1;
        uint32_t head = 0;       // next node of the queue
        uint32_t j_cur = 0;      // entries of its query list already taken
        uint32_t cand_base = 0;  // candidates numbered so far
        while (!done && head < n_v) {
            // the stretch: nodes head .. head+nf, thread t looks at node head+t
            const uint32_t nf = min((uint32_t)T, n_v - head);
            uint32_t deg = 0;
            if ((uint32_t)tid < nf) {
                const int32_t u = vbar[head + tid];
                const int64_t len = a.inc_off[u + 1] - a.inc_off[u] - (tid == 0 ? (int64_t)j_cur : 0);
                bad_lists |= len < 0;
                // a list longer than a chunk is taken in pieces; how much longer does not matter
                deg = (uint32_t)max((int64_t)0, min(len, (int64_t)a.chunk + 1));
            }
            uint32_t total;
            const uint32_t excl = bfs_block_scan<T>(deg, &total, wave_sums);
            pre[tid] = excl;
            if (tid == T - 1) pre[T] = total;
            if (tid == 0) s_take = 0;
            __syncthreads();
            // nodes taken whole: the longest prefix of the stretch with at most a.chunk entries
            if ((uint32_t)tid < nf && pre[tid + 1] <= a.chunk &&
                ((uint32_t)tid + 1 == nf || pre[tid + 2] > a.chunk))
                s_take = (uint32_t)tid + 1;
            __syncthreads();
            const uint32_t take = s_take;
            const bool partial = take == 0;  // the first node's list alone is longer than a chunk
            const uint32_t n_c = partial ? a.chunk : pre[take];
            const uint32_t n_src = partial ? 1u : take;

            // candidates: entry j of node t' of the stretch, numbered cand_base + c
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const uint32_t c = (uint32_t)tid * kBfsPer + r;
                if (c < n_c) {
                    uint32_t lo = 0, hi = n_src;  // last node with pre[node] <= c
                    while (hi - lo > 1) {
                        const uint32_t mid = (lo + hi) >> 1;
                        if (pre[mid] <= c) {
                            lo = mid;
                        } else {
                            hi = mid;
                        }
                    }
                    const int32_t u = vbar[head + lo];
                    const int64_t e = a.inc_off[u] + (lo == 0 ? (int64_t)j_cur : 0) + (c - pre[lo]);
                    uint32_t q = 0, slot = kBfsEmpty;
                    if (e >= 0 && e < n_entries) q = (uint32_t)a.inc_q[e];
                    if (e >= 0 && e < n_entries && (int64_t)q < a.n_queries) {
                        slot = insert_min(q_tab, q_mask, q, cand_base + c);
                        table_full |= slot == kBfsEmpty;
                    } else {
                        bad_lists = true;
                    }
                    cand_q[c] = q;
                    cand_slot[c] = slot;
                }
            }
            __syncthreads();
            // the candidates that kept their query, in order: the newly reached queries
            uint32_t own = 0;
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const uint32_t c = (uint32_t)tid * kBfsPer + r;
                if (c < n_c && cand_slot[c] != kBfsEmpty &&
                    table_load(&q_tab[2 * cand_slot[c] + 1]) == cand_base + c)
                    own |= 1u << r;
            }
            uint32_t n_new;
            uint32_t at = bfs_block_scan<T>((uint32_t)__popc(own), &n_new, wave_sums);
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r)
                if (own & (1u << r)) new_q[at++] = cand_q[(uint32_t)tid * kBfsPer + r];
            __syncthreads();

            // their nodes: node (i, j) is numbered n_start + (n_b + i) * k + j
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const uint32_t i = (uint32_t)tid * kBfsPer + r;
                if (i < n_new) {
                    const int64_t q = new_q[i];
                    for (int j = 0; j < k; ++j) {
                        const int32_t x = a.queries[q * k + j];
                        uint32_t slot = kBfsEmpty;
                        if ((uint32_t)x < (uint32_t)a.n_nodes) {
                            slot = insert_min(v_tab, v_mask, (uint32_t)x,
                                              (uint32_t)a.n_start + (n_b + i) * (uint32_t)k + (uint32_t)j);
                            table_full |= slot == kBfsEmpty;
                        } else {
                            bad_id = true;
                        }
                        node_slot[i * kBfsMaxK + j] = slot;
                    }
                }
            }
            __syncthreads();
            uint32_t fresh[kBfsPer];  // bit j: node j of the query is new and first named here
            uint32_t n_fresh = 0;
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const uint32_t i = (uint32_t)tid * kBfsPer + r;
                fresh[r] = 0;
                if (i < n_new) {
                    for (int j = 0; j < k; ++j) {
                        const uint32_t slot = node_slot[i * kBfsMaxK + j];
                        if (slot != kBfsEmpty &&
                            table_load(&v_tab[2 * slot + 1]) ==
                                (uint32_t)a.n_start + (n_b + i) * (uint32_t)k + (uint32_t)j)
                            fresh[r] |= 1u << j;
                    }
                    n_fresh += (uint32_t)__popc(fresh[r]);
                }
            }
            uint32_t all_fresh;
            uint32_t before = n_v + bfs_block_scan<T>(n_fresh, &all_fresh, wave_sums);
            // a query is taken if the queue would have reached it: room for its nodes, and neither
            // limit met by the queries before it
            uint32_t n_ok = 0, nodes_ok = 0;
            uint32_t first_at[kBfsPer];
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const uint32_t i = (uint32_t)tid * kBfsPer + r;
                const uint32_t mine = (uint32_t)__popc(fresh[r]);
                first_at[r] = before;
                const bool ok = i < n_new && before < (uint32_t)a.B1 && before + mine <= (uint32_t)a.B1 &&
                                n_b + i < (uint32_t)a.B2;
                if (ok) {
                    n_ok += 1;
                    nodes_ok += mine;
                } else {
                    fresh[r] = 0xFFFFFFFFu;  // not taken
                }
                before += mine;
            }
            uint32_t took, took_nodes;
            (void)bfs_block_scan<T>(n_ok, &took, wave_sums);
            (void)bfs_block_scan<T>(nodes_ok, &took_nodes, wave_sums);
#pragma unroll
            for (int r = 0; r < kBfsPer; ++r) {
                const uint32_t i = (uint32_t)tid * kBfsPer + r;
                if (fresh[r] != 0xFFFFFFFFu) {
                    const int64_t q = new_q[i];
                    batch[n_b + i] = (int32_t)q;
                    uint32_t at_v = first_at[r];
                    for (int j = 0; j < k; ++j) {
                        const int32_t x = a.queries[q * k + j];
                        if (tuples) tuples[(int64_t)(n_b + i) * k + j] = x;
                        if (fresh[r] & (1u << j)) vbar[at_v++] = x;
                    }
                }
            }
            n_b += took;
            n_v += took_nodes;
            cand_base += n_c;
            if (partial) {
                j_cur += n_c;
            } else {
                head += take;
                j_cur = 0;
            }
            done = took < n_new || n_b == (uint32_t)a.B2 || n_v == (uint32_t)a.B1;
            __syncthreads();  // vbar and the LDS lists are complete before the next stretch
        }
        if (tid == 0) {
            a.counts[2 * b] = (int32_t)n_v;
            a.counts[2 * b + 1] = (int32_t)n_b;
        }
        __syncthreads();
    }
    raise_error(a.err, bad_id, kDevBadQuery);
    raise_error(a.err, bad_lists, kDevBadTable);
    raise_error(a.err, table_full, kDevStall);
}

uint32_t pow2_at_least(uint64_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

}  // namespace

// Candidates settled at a time: every one of them may turn out to be a new query whose nodes
// are entered into the node table before the limits cut, so small batches take small bites.
static uint32_t bfs_chunk(int32_t B2) {
    const uint32_t want = pow2_at_least(4ull * (uint64_t)B2);
    return want < 64u ? 64u : (want > (uint32_t)kBfsMaxChunk ? (uint32_t)kBfsMaxChunk : want);
}
// One wavefront per search where a chunk fits its four candidates a lane: more searches in
// flight per compute unit, and their barriers cost nothing.
static int bfs_threads(int32_t B2) { return bfs_chunk(B2) <= (uint32_t)(kWave * kBfsPer) ? kWave : kBfsMaxThreads; }

// Slots of the two hash tables of one workgroup: at most half of them are ever used.
static uint32_t bfs_slots_q(int32_t B2) { return pow2_at_least(2ull * ((uint64_t)B2 + bfs_chunk(B2))); }
static uint32_t bfs_slots_v(int32_t B1, int32_t B2, int32_t n_start) {
    return pow2_at_least(2ull * ((uint64_t)B1 + (uint64_t)bfs_chunk(B2) * kBfsMaxK + (uint64_t)n_start));
}

static size_t bfs_table_bytes(int32_t n_start, int32_t B1, int32_t B2) {
    return 2u * sizeof(uint32_t) * ((size_t)bfs_slots_q(B2) + bfs_slots_v(B1, B2, n_start));
}

// Searches in flight: 16 waves a compute unit, fewer if their tables would pass 4 GiB.
static int bfs_grid(int n_cu, int64_t n_batches, size_t table_bytes, int threads) {
    int64_t resident = (int64_t)n_cu * (16 * kWave / threads);
    const int64_t by_memory = (int64_t)(((size_t)4 << 30) / table_bytes);
    if (resident > by_memory) resident = by_memory > 0 ? by_memory : 1;
    return (int)(n_batches < resident ? n_batches : resident);
}

size_t bfs_scratch_bytes(int n_cu, int64_t n_batches, int32_t n_start, int32_t B1, int32_t B2) {
    const size_t per = bfs_table_bytes(n_start, B1, B2);
    return (size_t)bfs_grid(n_cu, n_batches, per, bfs_threads(B2)) * per;
}

hipError_t launch_bfs_batches(hipStream_t stream, int n_cu, const int32_t* queries,
                              int64_t n_queries, int32_t k, int32_t n_nodes, const int64_t* inc_off,
                              const int32_t* inc_q, const int32_t* start, int64_t n_batches,
                              int32_t n_start, int32_t B1, int32_t B2, int32_t* vbar, int32_t* batch,
                              int32_t* tuples, int32_t* counts, void* scratch, uint32_t* err) {
    if (n_batches == 0) return hipSuccess;
    BfsArgs a;
    a.queries = queries;
    a.n_queries = n_queries;
    a.k = k;
    a.n_nodes = n_nodes;
    a.inc_off = inc_off;
    a.inc_q = inc_q;
    a.start = start;
    a.n_batches = n_batches;
    a.n_start = n_start;
    a.B1 = B1;
    a.B2 = B2;
    a.vbar = vbar;
    a.batch = batch;
    a.tuples = tuples;
    a.counts = counts;
    a.tables = static_cast<uint32_t*>(scratch);
    a.slots_q = bfs_slots_q(B2);
    a.slots_v = bfs_slots_v(B1, B2, n_start);
    a.chunk = bfs_chunk(B2);
    a.err = err;
    const int threads = bfs_threads(B2);
    const int grid = bfs_grid(n_cu, n_batches, bfs_table_bytes(n_start, B1, B2), threads);
    if (threads == kWave) {
        bfs_batch_kernel<kWave><<<dim3((unsigned)grid), dim3(kWave), 0, stream>>>(a);
    } else {
        bfs_batch_kernel<kBfsMaxThreads><<<dim3((unsigned)grid), dim3(kBfsMaxThreads), 0, stream>>>(a);
    }
    return hipGetLastError();
}

}  // namespace surel
