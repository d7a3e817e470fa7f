// The queries of every node (Sec. 3.6 "Mini-batching for Training": two nodes are neighbours
// when a query holds both, so the search walks node -> its queries -> their nodes).  Built by a
// stable radix sort of the (node, query) pairs of the query list: inc_q holds, node by node,
// the indices of the queries that name the node, ascending; inc_off[x] .. inc_off[x+1] is
// node x's part.
#include "device_util.h"
#include "kernels.h"

namespace surel {

namespace {

constexpr int kSortItems = 16;                    // pairs per lane
constexpr int kSortTile = kWave * kSortItems;     // pairs per wavefront (one workgroup)
constexpr int kSortBins = 256;                    // 8 bits a pass

// keys[t] = node of entry t of the query list (n_nodes for an id outside the graph, so that
// such entries sort behind every node's part), vals[t] = its query t / k.
__global__ __launch_bounds__(256) void incidence_pairs_kernel(const int32_t* __restrict__ queries,
                                                             int64_t n_entries, int32_t k,
                                                             int32_t n_nodes,
                                                             uint32_t* __restrict__ keys,
                                                             uint32_t* __restrict__ vals,
                                                             uint32_t* __restrict__ err) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool bad = false;
    if (t < n_entries) {
        const int32_t x = queries[t];
        bad = (uint32_t)x >= (uint32_t)n_nodes;
        keys[t] = bad ? (uint32_t)n_nodes : (uint32_t)x;
        vals[t] = (uint32_t)(t / k);
    }
    raise_error(err, bad, kDevBadQuery);
}

// hist[d * n_tiles + tile] = pairs of the tile whose key has digit d.
__global__ __launch_bounds__(kWave) void sort_hist_kernel(const uint32_t* __restrict__ keys,
                                                         int64_t n, int shift, int64_t n_tiles,
                                                         int32_t* __restrict__ hist) {
    __shared__ uint32_t bins[kSortBins];
    const int lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    for (int d = lane; d < kSortBins; d += kWave) bins[d] = 0u;
    wave_sync();
    const int64_t base = tile * kSortTile;
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t i = base + r * kWave + lane;
        if (i < n) atomicAdd(&bins[(keys[i] >> shift) & (kSortBins - 1)], 1u);
    }
    wave_sync();
    for (int d = lane; d < kSortBins; d += kWave) hist[(int64_t)d * n_tiles + tile] = (int32_t)bins[d];
}

// Moves the tile's pairs to their places: place of a pair = first place of (its digit, this
// tile) + number of earlier pairs of the tile with the same digit.  Pairs are taken 64 at a
// time in index order, so equal keys keep their order.
__global__ __launch_bounds__(kWave) void sort_scatter_kernel(const uint32_t* __restrict__ keys,
                                                            const uint32_t* __restrict__ vals,
                                                            int64_t n, int shift, int64_t n_tiles,
                                                            const int64_t* __restrict__ first,
                                                            uint32_t* __restrict__ out_keys,
                                                            uint32_t* __restrict__ out_vals) {
    __shared__ uint32_t place[kSortBins];
    const int lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    for (int d = lane; d < kSortBins; d += kWave) place[d] = (uint32_t)first[(int64_t)d * n_tiles + tile];
    wave_sync();
    const int64_t base = tile * kSortTile;
    const uint64_t below = (1ull << lane) - 1ull;
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t i = base + r * kWave + lane;
        const bool valid = i < n;
        const uint32_t key = valid ? keys[i] : 0u;
        const uint32_t val = valid ? vals[i] : 0u;
        const uint32_t d = (key >> shift) & (kSortBins - 1);
        uint64_t same = __ballot(valid);  // lanes whose pair has this lane's digit
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const uint64_t has = __ballot((d >> b) & 1u);
            same &= ((d >> b) & 1u) ? has : ~has;
        }
        const uint32_t rank = (uint32_t)__popcll(same & below);
        const uint32_t group = (uint32_t)__popcll(same);
        const uint32_t at = valid ? place[d] + rank : 0u;
        wave_sync();  // every lane has read place[] before the group's last lane moves it on
        if (valid && rank + 1 == group) place[d] += group;
        wave_sync();
        if (valid) {
            out_keys[at] = key;
            out_vals[at] = val;
        }
    }
}

// inc_off[x] = number of sorted keys below x, for x = 0..n_nodes.
__global__ __launch_bounds__(256) void incidence_offsets_kernel(const uint32_t* __restrict__ keys,
                                                               int64_t n, int32_t n_nodes,
                                                               int64_t* __restrict__ inc_off) {
    const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (x > n_nodes) return;
    int64_t lo = 0, hi = n;  // first index whose key is >= x
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if (keys[mid] < (uint32_t)x) {
            lo = mid + 1;
        } else {
            hi = mid;
        }
    }
    inc_off[x] = lo;
}

int64_t sort_tiles(int64_t n) { return (n + kSortTile - 1) / kSortTile; }

}  // namespace

size_t incidence_scratch_bytes(int64_t n_entries) {
    const int64_t n = n_entries > 0 ? n_entries : 1;
    const int64_t cells = sort_tiles(n) * kSortBins;
    size_t bytes = 4 * (((size_t)n * sizeof(uint32_t) + 255) / 256 * 256);          // two key, two value arrays
    bytes += ((size_t)cells * sizeof(int32_t) + 255) / 256 * 256;                  // digit counts
    bytes += ((size_t)(cells + 1) * sizeof(int64_t) + 255) / 256 * 256;            // their prefix sums
    bytes += ((size_t)scan_partials_len(cells) * sizeof(int64_t) + 255) / 256 * 256;
    return bytes;
}

hipError_t launch_query_incidence(hipStream_t stream, const int32_t* queries, int64_t n_queries,
                                  int32_t k, int32_t n_nodes, int64_t* inc_off, int32_t* inc_q,
                                  void* scratch, uint32_t* err) {
    const int64_t n = n_queries * k;
    if (n == 0) {  // no entries: every part is empty
        incidence_offsets_kernel<<<dim3((unsigned)(((int64_t)n_nodes + 1 + 255) / 256)), dim3(256), 0,
                                   stream>>>(nullptr, 0, n_nodes, inc_off);
        return hipGetLastError();
    }
    const int64_t n_tiles = sort_tiles(n);
    const int64_t cells = n_tiles * kSortBins;
    const size_t arr = ((size_t)n * sizeof(uint32_t) + 255) / 256 * 256;
    char* p = static_cast<char*>(scratch);
    uint32_t* key[2] = {reinterpret_cast<uint32_t*>(p), reinterpret_cast<uint32_t*>(p + arr)};
    uint32_t* val[2] = {reinterpret_cast<uint32_t*>(p + 2 * arr), reinterpret_cast<uint32_t*>(p + 3 * arr)};
    p += 4 * arr;
    int32_t* hist = reinterpret_cast<int32_t*>(p);
    p += ((size_t)cells * sizeof(int32_t) + 255) / 256 * 256;
    int64_t* first = reinterpret_cast<int64_t*>(p);
    p += ((size_t)(cells + 1) * sizeof(int64_t) + 255) / 256 * 256;
    int64_t* partials = reinterpret_cast<int64_t*>(p);

    incidence_pairs_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(
        queries, n, k, n_nodes, key[0], val[0], err);
    int bits = 1;  // keys are 0..n_nodes
    while (bits < 32 && ((uint32_t)n_nodes >> bits) != 0u) ++bits;
    int cur = 0;
    for (int shift = 0; shift < bits; shift += 8) {
        const bool last = shift + 8 >= bits;  // the last pass puts the queries where they belong
        uint32_t* out_vals = last ? reinterpret_cast<uint32_t*>(inc_q) : val[cur ^ 1];
        sort_hist_kernel<<<dim3((unsigned)n_tiles), dim3(kWave), 0, stream>>>(key[cur], n, shift,
                                                                             n_tiles, hist);
        if (hipError_t e = launch_exclusive_scan(stream, hist, cells, first, partials); e != hipSuccess)
            return e;
        sort_scatter_kernel<<<dim3((unsigned)n_tiles), dim3(kWave), 0, stream>>>(
            key[cur], val[cur], n, shift, n_tiles, first, key[cur ^ 1], out_vals);
        cur ^= 1;
    }
    incidence_offsets_kernel<<<dim3((unsigned)(((int64_t)n_nodes + 1 + 255) / 256)), dim3(256), 0,
                               stream>>>(key[cur], n, n_nodes, inc_off);
    return hipGetLastError();
}

}  // namespace surel
