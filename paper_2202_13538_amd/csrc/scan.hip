// Exclusive prefix sums that turn per-seed / per-query row counts into the offset arrays
// rpe_off and join_off.  Reduce-then-scan in three small launches: tile sums, a scan of
// the tile sums by one workgroup, and a tile-local scan that adds the tile's base.
#include "device_util.h"
#include "kernels.h"
#include "lookback.h"

namespace surel {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

// Exclusive prefix sum of one value per thread over a 256-thread workgroup; *total gets
// the workgroup's sum.  Every thread must call it.
__device__ __forceinline__ uint32_t block_excl_sum(uint32_t v, uint32_t* total) {
    __shared__ uint32_t wave_sums[kScanThreads / kWave];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_sum(v);
    __syncthreads();  // wave_sums may still be read from a previous call
    if (lane == kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / kWave; ++w) {
        if (w < wave) base += wave_sums[w];
        sum += wave_sums[w];
    }
    *total = sum;
    return base + incl - v;
}

__global__ __launch_bounds__(kScanThreads) void tile_sum_kernel(const int32_t* __restrict__ counts,
                                                               int64_t n,
                                                               int64_t* __restrict__ partials) {
    const int64_t base = (int64_t)blockIdx.x * kScanTile;
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        const int64_t idx = base + j * kScanThreads + threadIdx.x;
        if (idx < n) v += (uint32_t)counts[idx];
    }
    uint32_t total;
    block_excl_sum(v, &total);
    if (threadIdx.x == 0) partials[blockIdx.x] = (int64_t)total;
}

// In place: partials[0..n_tiles) -> exclusive prefix sums, partials[n_tiles] = grand total.
__global__ __launch_bounds__(kScanThreads) void partial_scan_kernel(int64_t* __restrict__ partials,
                                                                    int64_t n_tiles) {
    __shared__ int64_t wave_sums[kScanThreads / kWave];
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    int64_t carry = 0;
    for (int64_t start = 0; start < n_tiles; start += kScanThreads) {
        const int64_t idx = start + threadIdx.x;
        const int64_t v = idx < n_tiles ? partials[idx] : 0;
        int64_t incl = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int64_t t = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += t;
        }
        __syncthreads();
        if (lane == kWave - 1) wave_sums[wave] = incl;
        __syncthreads();
        int64_t base = 0, sum = 0;
#pragma unroll
        for (int w = 0; w < kScanThreads / kWave; ++w) {
            if (w < wave) base += wave_sums[w];
            sum += wave_sums[w];
        }
        if (idx < n_tiles) partials[idx] = carry + base + incl - v;
        carry += sum;
    }
    if (threadIdx.x == 0) partials[n_tiles] = carry;
}

__global__ __launch_bounds__(kScanThreads) void tile_scan_kernel(const int32_t* __restrict__ counts,
                                                                int64_t n,
                                                                const int64_t* __restrict__ partials,
                                                                int64_t n_tiles,
                                                                int64_t* __restrict__ off) {
    // thread t owns the kScanItems consecutive entries starting at base + t * kScanItems
    const int64_t first = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint32_t item[kScanItems];
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        item[j] = (first + j < n) ? (uint32_t)counts[first + j] : 0u;
        v += item[j];
    }
    uint32_t total;
    uint32_t run = block_excl_sum(v, &total);
    const int64_t tile_base = partials[blockIdx.x];
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (first + j < n) off[first + j] = tile_base + (int64_t)run;
        run += item[j];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) off[n] = partials[n_tiles];
}

// Before a launch that lays its output out itself: counters and counts to zero (the counts that
// pad the last group to "no rows"), every group base to "not yet", the total to -1.  (A kernel,
// not a memset, so that the call stays valid under stream capture.)
__global__ void lookback_clear_kernel(uint64_t* __restrict__ lb, int64_t n_items,
                                      int64_t* __restrict__ total_out) {
    const LookbackScratch sc = lookback_scratch(n_items);
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) *total_out = -1;
    if (t >= sc.total_words) return;
    uint64_t v = 0ull;
    if (t >= 2 && t < 2 + sc.base_words) {
        v = ~0ull;  // -1
    } else if (t >= 2 + sc.base_words) {
        const int64_t first = (t - 2 - sc.base_words) * 4;  // first count of this word
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int64_t j = first + q;
            if (j >= n_items && j < sc.n_groups * kGroup) v |= 1ull << (16 * q);
        }
    }
    lb[t] = v;
}

int64_t lookback_words(int64_t n_items) {
    return lookback_scratch(n_items > 0 ? n_items : 0).total_words;
}

hipError_t launch_lookback_clear(hipStream_t stream, uint64_t* lb, int64_t n_items,
                                 int64_t* total_out) {
    const int64_t n_clear = lookback_scratch(n_items).total_words;
    hipLaunchKernelGGL(lookback_clear_kernel, dim3((unsigned)((n_clear + 255) / 256)), dim3(256), 0,
                       stream, lb, n_items, total_out);
    return hipGetLastError();
}

int64_t scan_partials_len(int64_t n) { return (n + kScanTile - 1) / kScanTile + 1; }

hipError_t launch_exclusive_scan(hipStream_t stream, const int32_t* counts, int64_t n,
                                 int64_t* off, int64_t* partials) {
    const int64_t n_tiles = (n + kScanTile - 1) / kScanTile;
    if (n_tiles > 0) {
        hipLaunchKernelGGL(tile_sum_kernel, dim3((unsigned)n_tiles), dim3(kScanThreads), 0,
                           stream, counts, n, partials);
    }
    hipLaunchKernelGGL(partial_scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, partials,
                       n_tiles);
    if (n_tiles > 0) {
        hipLaunchKernelGGL(tile_scan_kernel, dim3((unsigned)n_tiles), dim3(kScanThreads), 0,
                           stream, counts, n, partials, n_tiles, off);
    } else {
        // n == 0: off[0] = total = 0 is written by a one-thread launch of the same kernel
        hipLaunchKernelGGL(tile_scan_kernel, dim3(1), dim3(kScanThreads), 0, stream, counts, n,
                           partials, n_tiles, off);
    }
    return hipGetLastError();
}

}  // namespace surel
