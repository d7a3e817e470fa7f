// Pruning the central RPE array (Sec. 3.3; Algorithm 1, last step): many table rows carry the
// same count vector, so the distinct vectors are stored once, in an array T, and every row
// keeps the index of its vector in T (its RPE-ID after re-indexing).  The paper leaves T in
// insertion order; here T is sorted (count vectors compared entry by entry), which makes the
// result unique and testable bit for bit.
//
// Four steps, all on the device:
//   collect  every row looks its vector up in a global open-addressing hash set and inserts
//            it if it is new; the row's slot number goes to code[row].  A slot is 64 bytes
//            (state, rank, vector), aligned, so one cache line holds all of it.  Almost every
//            lookup finds its vector already there (a few vectors make up nearly all rows)
//            and is served by the caches with plain loads; only a slot that does not look
//            full yet is touched with atomics.
//   gather   the full slots are listed (their number is the size of T),
//   sort     the list is sorted with a bitonic network in global memory (it is small),
//   rank     slot.rank = position in the sorted list, T[position] = vector, and finally
//            code[row] = rank of the row's slot.
// Waiting.  A lane that finds a slot locked (another lane is writing its vector) polls it
// again; the writer needs nothing from the poller (inside one wavefront the writer's branch
// runs to its end before the next poll), so the poll ends; it is bounded by the spin limit
// all the same.
#include "device_util.h"
#include "kernels.h"
#include "prune_set.h"

namespace surel {

// The count vector of a row as NW words, entry 2k in the upper half of word k, so that
// comparing words in order compares the counts in order.  L = m + 1 entries.
template <int NW>
__device__ __forceinline__ void load_vector(const uint16_t* __restrict__ cnt, int64_t row, int L,
                                            uint32_t (&w)[NW]) {
    const uint16_t* v = cnt + row * L;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const uint32_t hi = v[2 * k];
        const uint32_t lo = (2 * k + 1 < L) ? v[2 * k + 1] : 0u;
        w[k] = (hi << 16) | lo;
    }
}

constexpr int kPruneRows = 4;        // rows a lane works on at once
// A workgroup takes tiles of 256 * kPruneRows consecutive rows; a lane has kPruneRows of them in
// flight.  A few vectors make up nearly all rows, and all compute units asking the same few
// cache lines of the global table for them would queue up at those lines' L2 channels; so every
// workgroup keeps a small cache of (vector -> slot) in LDS.  An entry is written once, by the
// lane that wins its state word, and is valid for good after that (state, then vector and slot,
// then "valid": LDS operations of a wave take effect in order), so readers never see a mix of
// two vectors.  Vectors that find their entry taken by another go to the global table.
template <int NW>
__global__ __launch_bounds__(256) void prune_collect_kernel(
    const uint16_t* __restrict__ cnt, int64_t n_rows, int L, uint32_t* __restrict__ slots,
    uint32_t slot_mask, int64_t cap_T, unsigned long long* __restrict__ n_inserted,
    int32_t* __restrict__ code, uint32_t spin_limit, uint32_t* __restrict__ err) {
    __shared__ uint32_t cache[kCacheEntries * kCacheWords];
    prune_cache_clear(cache, (int)threadIdx.x, 256);
    __syncthreads();
    const int64_t tile_rows = 256 * kPruneRows;
    const int64_t stride = (int64_t)gridDim.x * tile_rows;
    for (int64_t tile = (int64_t)blockIdx.x * tile_rows; tile < n_rows; tile += stride) {
        uint32_t w[kPruneRows][NW];
#pragma unroll
        for (int u = 0; u < kPruneRows; ++u) {
            const int64_t row = min(tile + u * 256 + (int64_t)threadIdx.x, n_rows - 1);
            load_vector<NW>(cnt, row, L, w[u]);
        }
#pragma unroll
        for (int u = 0; u < kPruneRows; ++u) {
            const int64_t row = tile + u * 256 + (int64_t)threadIdx.x;
            if (row >= n_rows) continue;
            const int32_t found = prune_lookup<NW>(w[u], cache, slots, slot_mask, cap_T, n_inserted,
                                                   spin_limit, err);
            code[row] = found;
        }
    }
}

// Lists the full slots: list[i] = (vector words, slot number), in any order.
__global__ __launch_bounds__(256) void prune_gather_kernel(const uint32_t* __restrict__ slots,
                                                           uint32_t n_slots, int64_t list_len,
                                                           unsigned long long* __restrict__ n_listed,
                                                           uint32_t* __restrict__ list) {
    const uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= n_slots) return;
    const uint32_t* slot = slots + (size_t)s * kSlotWords;
    if (slot[0] != kSlotFull) return;
    const unsigned long long at = atomicAdd(n_listed, 1ull);
    if ((int64_t)at >= list_len) return;
    uint32_t* item = list + at * (kMaxVecWords + 1);
#pragma unroll
    for (int k = 0; k < kMaxVecWords; ++k) item[k] = slot[kSlotVector + k];
    item[kMaxVecWords] = s;
}

// Entries from `first` on become padding that sorts behind every vector.
__global__ __launch_bounds__(256) void prune_pad_kernel(uint32_t* __restrict__ list, int64_t first,
                                                        int64_t len) {
    const int64_t i = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= len) return;
#pragma unroll
    for (int k = 0; k <= kMaxVecWords; ++k) list[i * (kMaxVecWords + 1) + k] = 0xFFFFFFFFu;
}

__device__ __forceinline__ bool item_less(const uint32_t (&a)[kMaxVecWords + 1],
                                          const uint32_t (&b)[kMaxVecWords + 1]) {
#pragma unroll
    for (int k = 0; k <= kMaxVecWords; ++k) {
        if (a[k] != b[k]) return a[k] < b[k];
    }
    return false;
}

// One compare-exchange step of a bitonic sorting network over `len` (a power of two) items:
// partner distance j inside merges of size k.
__global__ __launch_bounds__(256) void prune_sort_step_kernel(uint32_t* __restrict__ list,
                                                              int64_t len, int64_t j, int64_t k) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t p = i ^ j;
    if (i >= len || p <= i) return;
    uint32_t a[kMaxVecWords + 1], b[kMaxVecWords + 1];
#pragma unroll
    for (int t = 0; t <= kMaxVecWords; ++t) {
        a[t] = list[i * (kMaxVecWords + 1) + t];
        b[t] = list[p * (kMaxVecWords + 1) + t];
    }
    const bool ascending = (i & k) == 0;
    if (item_less(b, a) == ascending) {
#pragma unroll
        for (int t = 0; t <= kMaxVecWords; ++t) {
            list[i * (kMaxVecWords + 1) + t] = b[t];
            list[p * (kMaxVecWords + 1) + t] = a[t];
        }
    }
}

// T[i] = vector of the i-th item of the sorted list; its slot learns its rank.
__global__ __launch_bounds__(256) void prune_rank_kernel(const uint32_t* __restrict__ list,
                                                         int64_t n_T, int L,
                                                         uint32_t* __restrict__ slots,
                                                         uint16_t* __restrict__ T) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_T) return;
    const uint32_t* item = list + i * (kMaxVecWords + 1);
    slots[(size_t)item[kMaxVecWords] * kSlotWords + 1] = (uint32_t)i;
    for (int e = 0; e < L; ++e) {
        const uint32_t word = item[e >> 1];
        T[i * L + e] = (uint16_t)((e & 1) ? (word & 0xFFFFu) : (word >> 16));
    }
}

// code[row]: slot number -> rank of that slot (-1, or anything that is no slot number, becomes -1).
// Four rows a lane, moved as 16-byte words where the array's alignment allows (the pass is a
// plain stream over the codes; the ranks come from a few thousand hot cache lines).
constexpr int kCodesUnroll = 4;
__global__ __launch_bounds__(256) void prune_codes_kernel(const uint32_t* __restrict__ slots,
                                                          uint32_t n_slots, int64_t n_rows,
                                                          int32_t* __restrict__ code) {
    auto rank_of = [&](int32_t c) -> int32_t {
        const uint32_t s = (uint32_t)c;
        return s < n_slots ? (int32_t)slots[(size_t)s * kSlotWords + 1] : -1;
    };
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if ((reinterpret_cast<uintptr_t>(code) & 15u) == 0) {
        // kCodesUnroll 16-byte words of a lane are in flight together, non-temporal both ways:
        // every code is read once and written once
        typedef int code4_t __attribute__((ext_vector_type(4)));
        code4_t* code4 = reinterpret_cast<code4_t*>(code);
        const int64_t n4 = n_rows / 4;
        for (int64_t i0 = tid; i0 < n4; i0 += stride * kCodesUnroll) {
            code4_t c[kCodesUnroll];
#pragma unroll
            for (int u = 0; u < kCodesUnroll; ++u) {
                const int64_t i = i0 + u * stride;
                c[u] = code4_t{-1, -1, -1, -1};
                if (i < n4) c[u] = __builtin_nontemporal_load(code4 + i);
            }
#pragma unroll
            for (int u = 0; u < kCodesUnroll; ++u) {
                const int64_t i = i0 + u * stride;
                c[u].x = rank_of(c[u].x);
                c[u].y = rank_of(c[u].y);
                c[u].z = rank_of(c[u].z);
                c[u].w = rank_of(c[u].w);
                if (i < n4) __builtin_nontemporal_store(c[u], code4 + i);
            }
        }
        for (int64_t row = n4 * 4 + tid; row < n_rows; row += stride) code[row] = rank_of(code[row]);
    } else {
        for (int64_t row = tid; row < n_rows; row += stride) code[row] = rank_of(code[row]);
    }
}

int64_t prune_slots(int64_t cap_T) {
    int64_t s = 1024;
    while (s < 4 * cap_T) s *= 2;
    return s;
}
int64_t prune_list_len(int64_t cap_T) {
    int64_t s = 1;
    while (s < cap_T) s *= 2;
    return s;
}
size_t prune_slot_bytes(int64_t cap_T) { return (size_t)prune_slots(cap_T) * kSlotWords * 4; }
size_t prune_list_bytes(int64_t cap_T) {
    return (size_t)prune_list_len(cap_T) * (kMaxVecWords + 1) * 4;
}

uint32_t prune_slot_mask(int64_t cap_T) { return (uint32_t)(prune_slots(cap_T) - 1); }

hipError_t launch_prune_clear(hipStream_t stream, int64_t cap_T, uint32_t* slots,
                              unsigned long long* counters) {
    // empty table, counters to zero (the calls that use it read a total back on the host in any
    // case, so they cannot be captured into a graph, and plain memsets do)
    hipError_t rc = hipMemsetAsync(slots, 0, (size_t)prune_slots(cap_T) * kSlotWords * 4, stream);
    if (rc != hipSuccess) return rc;
    return hipMemsetAsync(counters, 0, 2 * sizeof(unsigned long long), stream);
}

hipError_t launch_prune_collect(hipStream_t stream, int n_cu, const uint16_t* cnt, int64_t n_rows,
                                int32_t m, int64_t cap_T, uint32_t* slots,
                                unsigned long long* counters, int32_t* code, uint32_t spin_limit,
                                uint32_t* err) {
    const int64_t n_slots = prune_slots(cap_T);
    hipError_t rc = launch_prune_clear(stream, cap_T, slots, counters);
    if (rc != hipSuccess) return rc;
    if (n_rows == 0) return hipSuccess;
    const int L = m + 1;
    int64_t blocks = (n_rows + 256 * kPruneRows - 1) / (256 * kPruneRows);
    // several workgroups per slot of the device, so that the last ones to start have little left
    if (blocks > (int64_t)n_cu * 32) blocks = (int64_t)n_cu * 32;
#define SUREL_PRUNE_CASE(NW_)                                                                  \
    if ((L + 1) / 2 == (NW_)) {                                                                \
        hipLaunchKernelGGL((prune_collect_kernel<NW_>), dim3((unsigned)blocks), dim3(256), 0,  \
                           stream, cnt, n_rows, L, slots, (uint32_t)(n_slots - 1), cap_T,      \
                           counters, code, spin_limit, err);                                   \
        return hipGetLastError();                                                              \
    }
    SUREL_PRUNE_CASE(1)
    SUREL_PRUNE_CASE(2)
    SUREL_PRUNE_CASE(3)
    SUREL_PRUNE_CASE(4)
    SUREL_PRUNE_CASE(5)
    SUREL_PRUNE_CASE(6)
    SUREL_PRUNE_CASE(7)
    SUREL_PRUNE_CASE(8)
#undef SUREL_PRUNE_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_prune_finish(hipStream_t stream, int n_cu, int64_t n_rows, int32_t m,
                               int64_t cap_T, int64_t n_T, uint32_t* slots,
                               unsigned long long* counters, uint32_t* list, uint16_t* T,
                               int32_t* code) {
    if (n_T > 0) {
        const int64_t n_slots = prune_slots(cap_T);
        int64_t len = 1;
        while (len < n_T) len *= 2;  // <= prune_list_len(cap_T) because n_T <= cap_T
        hipLaunchKernelGGL(prune_gather_kernel, dim3((unsigned)((n_slots + 255) / 256)), dim3(256), 0,
                           stream, slots, (uint32_t)n_slots, len, counters + 1, list);
        if (len > n_T)
            hipLaunchKernelGGL(prune_pad_kernel, dim3((unsigned)((len - n_T + 255) / 256)),
                               dim3(256), 0, stream, list, n_T, len);
        for (int64_t k = 2; k <= len; k *= 2)
            for (int64_t j = k / 2; j >= 1; j /= 2)
                hipLaunchKernelGGL(prune_sort_step_kernel, dim3((unsigned)((len + 255) / 256)),
                                   dim3(256), 0, stream, list, len, j, k);
        hipLaunchKernelGGL(prune_rank_kernel, dim3((unsigned)((n_T + 255) / 256)), dim3(256), 0,
                           stream, list, n_T, m + 1, slots, T);
    }
    if (n_rows > 0) {
        int64_t blocks = (n_rows / 4 + 256) / 256;
        if (blocks > (int64_t)n_cu * 32) blocks = (int64_t)n_cu * 32;
        hipLaunchKernelGGL(prune_codes_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, slots,
                           (uint32_t)prune_slots(cap_T), n_rows, code);
    }
    return hipGetLastError();
}

}  // namespace surel
