// Memory-system micro-benchmarks of the GPU that libsurel's kernels are judged against:
// streaming read / write / copy, chains of dependent random gathers from a table of a given
// size (what a walker does: the address of the next load comes out of the previous one),
// random scatters of short rows, and one pass of binning 12-byte items by a key through LDS
// (what it would cost to regroup walkers by the part of the graph they read next).  Benchmark tooling, not part of the hot path: `bench.py
// --membench` calls it through the C ABI below and prints the table.
//
// All buffers are the caller's device memory; every call runs its kernel twice on the given
// stream and times the second run with two HIP events.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

// 32-bit integer finaliser (the widely published "lowbias32" constants): a cheap bijection
// that turns counters into well-spread table indices.
__device__ __host__ inline uint32_t mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

__global__ void init_kernel(uint32_t* t, size_t n_words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n_words; i += stride) t[i] = mix32((uint32_t)i * 2654435761u + 1u);
}

// The streaming kernels.  A workgroup takes kStreamUnroll * blockDim consecutive 16-byte items
// per turn; a lane has kStreamUnroll accesses in flight, non-temporal (the data is used once).
// This shape was the fastest of a sweep over 1 / 4 / 8 accesses in flight, plain and
// non-temporal, 256 and 1024 lanes per workgroup and 1 K to 64 K workgroups (a lane with one
// plain access per turn reaches 5.8 / 5.3 / 4.7 TB/s for read / write / copy).
typedef int v4i __attribute__((ext_vector_type(4)));
constexpr int kStreamUnroll = 8;

__global__ void read_kernel(const v4i* __restrict__ a, size_t n, uint32_t* sink) {
    size_t base = (size_t)blockIdx.x * blockDim.x * kStreamUnroll + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x * kStreamUnroll;
    int acc = 0;
    for (; base < n; base += stride) {
        v4i v[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            const size_t i = base + (size_t)u * blockDim.x;
            v[u] = v4i{0, 0, 0, 0};
            if (i < n) v[u] = __builtin_nontemporal_load(a + i);
        }
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) acc += v[u].x + v[u].y + v[u].z + v[u].w;
    }
    if (acc == 0x12345678) sink[0] = (uint32_t)acc;  // keeps the loads alive
}

__global__ void write_kernel(v4i* __restrict__ b, size_t n) {
    size_t base = (size_t)blockIdx.x * blockDim.x * kStreamUnroll + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x * kStreamUnroll;
    for (; base < n; base += stride) {
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            const size_t i = base + (size_t)u * blockDim.x;
            if (i < n) __builtin_nontemporal_store(v4i{1, 2, 3, (int)i}, b + i);
        }
    }
}

__global__ void copy_kernel(const v4i* __restrict__ a, v4i* __restrict__ b, size_t n) {
    size_t base = (size_t)blockIdx.x * blockDim.x * kStreamUnroll + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x * kStreamUnroll;
    for (; base < n; base += stride) {
        v4i v[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            const size_t i = base + (size_t)u * blockDim.x;
            if (i < n) v[u] = __builtin_nontemporal_load(a + i);
        }
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            const size_t i = base + (size_t)u * blockDim.x;
            if (i < n) __builtin_nontemporal_store(v[u], b + i);
        }
    }
}

// One byte read for every two written (close to the join's filling launch): per turn a lane
// reads kStreamUnroll / 2 items and writes kStreamUnroll.
__global__ void read1_write2_kernel(const v4i* __restrict__ a, v4i* __restrict__ b, size_t n) {
    size_t base = (size_t)blockIdx.x * blockDim.x * kStreamUnroll + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x * kStreamUnroll;
    for (; base < n; base += stride) {
        v4i v[kStreamUnroll / 2];
#pragma unroll
        for (int u = 0; u < kStreamUnroll / 2; ++u) {
            const size_t i = base + (size_t)u * blockDim.x;
            v[u] = v4i{0, 0, 0, 0};
            if (i < n) v[u] = __builtin_nontemporal_load(a + i);
        }
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            const size_t i = base + (size_t)u * blockDim.x;
            if (i < n) __builtin_nontemporal_store(v[u / 2] + v4i{u, 0, 0, 0}, b + i);
        }
    }
}

// Every lane follows `chain` dependent gathers of one T (4, 8 or 16 bytes) through a table of
// mask+1 entries.
template <typename T>
__global__ void gather_kernel(const T* __restrict__ table, uint32_t mask, int chain,
                              uint32_t* sink) {
    const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t idx = mix32(tid + 12345u) & mask;
    uint32_t acc = 0;
    for (int c = 0; c < chain; ++c) {
        const T v = table[idx];
        const uint32_t first = *reinterpret_cast<const uint32_t*>(&v);
        acc += first;
        idx = mix32(first + idx * 31u + (uint32_t)c) & mask;
    }
    if (acc == 0x12345678u) sink[0] = acc;
}

// Every lane writes `rows` rows of W 32-bit words at random row positions.
template <int W>
__global__ void scatter_kernel(uint32_t* __restrict__ dst, uint32_t row_mask, int rows) {
    const uint32_t tid = blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t idx = mix32(tid + 777u);
    for (int c = 0; c < rows; ++c) {
        uint32_t* p = dst + (size_t)(idx & row_mask) * W;
#pragma unroll
        for (int j = 0; j < W; ++j) p[j] = idx + (uint32_t)j;
        idx = mix32(idx + (uint32_t)c);
    }
}

// One pass of a bucket sort: n items of three 32-bit words (word 0 is the key) go to kBins
// bins by the key's top bits.  A workgroup stages items per bin in LDS and writes a bin's items
// out 16 at a time (192 contiguous bytes) at a position drawn from the bin's global cursor, so
// that the output is written in whole cache lines although consecutive items go to different
// bins.  bin b owns out[b * cap .. (b + 1) * cap); items beyond a bin's capacity are dropped and
// counted in cursor[kBins].
constexpr int kBins = 256;
constexpr int kBinStage = 40;       // items a bin can hold in LDS
constexpr int kBinFlush = 16;       // items written out at a time
constexpr int kBinThreads = 1024;
constexpr int kBinItemsPerThread = 2;

__global__ __launch_bounds__(kBinThreads) void bin_kernel(const uint32_t* __restrict__ items,
                                                          size_t n, int shift, uint32_t cap,
                                                          uint32_t* __restrict__ out,
                                                          uint32_t* __restrict__ cursor) {
    extern __shared__ uint32_t lds[];
    uint32_t* stage = lds;                                  // [kBins][kBinStage][3]
    uint32_t* cnt = lds + kBins * kBinStage * 3;            // [kBins]
    uint32_t* gpos = cnt + kBins;                           // [kBins]
    uint32_t* nflush = gpos + kBins;                        // [kBins]
    __shared__ int any_left;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    for (int b = tid; b < kBins; b += kBinThreads) cnt[b] = 0;
    __syncthreads();
    const size_t tile = (size_t)kBinThreads * kBinItemsPerThread;
    const size_t n_tiles = (n + tile - 1) / tile;
    for (size_t t = blockIdx.x;; t += gridDim.x) {
        const bool last = t >= n_tiles;  // every workgroup's final round only empties its stages
        uint32_t it[kBinItemsPerThread][3];
        bool have[kBinItemsPerThread];
#pragma unroll
        for (int u = 0; u < kBinItemsPerThread; ++u) {
            const size_t i = t * tile + (size_t)u * kBinThreads + tid;
            have[u] = !last && i < n;
            if (have[u]) {
                it[u][0] = items[i * 3];
                it[u][1] = items[i * 3 + 1];
                it[u][2] = items[i * 3 + 2];
            }
        }
        for (;;) {
            // place what fits; what does not waits for the flush below
#pragma unroll
            for (int u = 0; u < kBinItemsPerThread; ++u) {
                if (!have[u]) continue;
                const uint32_t b = it[u][0] >> shift;
                const uint32_t pos = atomicAdd(&cnt[b], 1u);
                if (pos < (uint32_t)kBinStage) {
                    uint32_t* s = stage + ((size_t)b * kBinStage + pos) * 3;
                    s[0] = it[u][0];
                    s[1] = it[u][1];
                    s[2] = it[u][2];
                    have[u] = false;
                }
            }
            if (tid == 0) any_left = 0;
            __syncthreads();
            // every bin: how many whole groups go out, and where
            for (int b = tid; b < kBins; b += kBinThreads) {
                const uint32_t c = min(cnt[b], (uint32_t)kBinStage);
                const uint32_t nf = last ? c : c / kBinFlush * kBinFlush;
                nflush[b] = nf;
                cnt[b] = c;  // arrivals beyond the stage were not stored
                if (nf > 0) gpos[b] = atomicAdd(&cursor[b], nf);
            }
            bool mine_left = false;
#pragma unroll
            for (int u = 0; u < kBinItemsPerThread; ++u) mine_left = mine_left || have[u];
            if (mine_left) any_left = 1;
            __syncthreads();
            // a wave per bin in turn: write the groups out, move the rest to the front
            for (int b = wave; b < kBins; b += kBinThreads / 64) {
                const uint32_t nf = nflush[b];
                if (nf == 0) continue;
                const uint32_t c = cnt[b];
                const uint32_t at = gpos[b];
                const uint32_t* s = stage + (size_t)b * kBinStage * 3;
                uint32_t keep = at < cap ? min(nf, cap - at) : 0u;
                if (keep < nf && lane == 0) atomicAdd(&cursor[kBins], nf - keep);
                uint32_t* dst = out + ((size_t)b * cap + at) * 3;
                for (uint32_t w = lane; w < keep * 3; w += 64) dst[w] = s[w];
                const uint32_t rest = c - nf;  // < kBinFlush <= nf: source and target do not overlap
                uint32_t moved = 0;
                if (lane < (int)(rest * 3)) moved = s[nf * 3 + lane];
                if (lane < (int)(rest * 3)) stage[(size_t)b * kBinStage * 3 + lane] = moved;
                if (lane == 0) cnt[b] = rest;
            }
            __syncthreads();
            const bool again = any_left != 0;
            __syncthreads();  // everybody has read the flag before it is reset
            if (!again) break;
        }
        if (last) break;
    }
}

template <typename Launch>
int time_second_run(hipStream_t stream, Launch&& launch, double* h_ms) {
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -3;
    launch();
    bool ok = hipEventRecord(a, stream) == hipSuccess;
    launch();
    ok = ok && hipEventRecord(b, stream) == hipSuccess;
    ok = ok && hipEventSynchronize(b) == hipSuccess && hipGetLastError() == hipSuccess;
    float ms = 0.f;
    ok = ok && hipEventElapsedTime(&ms, a, b) == hipSuccess;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    *h_ms = (double)ms;
    return ok ? 0 : -3;
}

uint32_t pow2_mask(size_t entries) {  // largest power of two <= entries, minus one
    size_t p = 1;
    while (p * 2 <= entries) p *= 2;
    return (uint32_t)(p - 1);
}

constexpr int kThreads = 256;
constexpr int kStreamBlocks = 4096;
constexpr int kStreamThreads = 1024;
constexpr long kGatherLanes = 256L * 1024 * 64;  // 16.8 M lanes

}  // namespace

extern "C" {

// Fills d_buf[0 .. bytes) with pseudo-random words (the gather tables' contents).
int surel_membench_init(void* d_buf, size_t bytes, void* hip_stream) {
    if (!d_buf || bytes < 4) return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(init_kernel, dim3(4096), dim3(kThreads), 0, s, static_cast<uint32_t*>(d_buf),
                       bytes / 4);
    return hipStreamSynchronize(s) == hipSuccess ? 0 : -3;
}

// kind 0: read `bytes` of d_buf; 1: write them; 2: copy the first half of d_buf to the second;
// 3: write the second half and read a quarter of d_buf for it (bytes / 4 read, bytes / 2 written)
// (bytes / 2 read and bytes / 2 written).  *h_ms = kernel time.
int surel_membench_stream(int kind, void* d_buf, size_t bytes, uint32_t* d_sink, void* hip_stream,
                          double* h_ms) {
    if (!d_buf || !d_sink || !h_ms || bytes < 32 || kind < 0 || kind > 3) return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    v4i* a = static_cast<v4i*>(d_buf);
    const size_t n = bytes / 16;
    const dim3 grid(kStreamBlocks), block(kStreamThreads);
    return time_second_run(s, [&] {
        if (kind == 0) hipLaunchKernelGGL(read_kernel, grid, block, 0, s, a, n, d_sink);
        if (kind == 1) hipLaunchKernelGGL(write_kernel, grid, block, 0, s, a, n);
        if (kind == 2) hipLaunchKernelGGL(copy_kernel, grid, block, 0, s, a, a + n / 2, n / 2);
        if (kind == 3) hipLaunchKernelGGL(read1_write2_kernel, grid, block, 0, s, a, a + n / 2, n / 2);
    }, h_ms);
}

// 16.8 M lanes, each a chain of `chain` dependent gathers of `width` bytes (4, 8 or 16) from the
// first table_bytes of d_buf (rounded down to a power of two).  *h_gathers = gathers of one run.
int surel_membench_gather(void* d_buf, size_t table_bytes, int width, int chain, uint32_t* d_sink,
                          void* hip_stream, double* h_ms, double* h_gathers) {
    if (!d_buf || !d_sink || !h_ms || !h_gathers || chain < 1 || table_bytes < 1024) return -1;
    if (width != 4 && width != 8 && width != 16) return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint32_t mask = pow2_mask(table_bytes / (size_t)width);
    const dim3 grid((unsigned)(kGatherLanes / kThreads)), block(kThreads);
    *h_gathers = (double)kGatherLanes * chain;
    return time_second_run(s, [&] {
        if (width == 4) hipLaunchKernelGGL(gather_kernel<uint32_t>, grid, block, 0, s, static_cast<const uint32_t*>(d_buf), mask, chain, d_sink);
        if (width == 8) hipLaunchKernelGGL(gather_kernel<uint2>, grid, block, 0, s, static_cast<const uint2*>(d_buf), mask, chain, d_sink);
        if (width == 16) hipLaunchKernelGGL(gather_kernel<uint4>, grid, block, 0, s, static_cast<const uint4*>(d_buf), mask, chain, d_sink);
    }, h_ms);
}

// 16.8 M lanes, each writes `rows` rows of `width` bytes (4, 20 or 64) at random row positions
// inside d_buf[0 .. bytes).  *h_rows = rows of one run.
int surel_membench_scatter(void* d_buf, size_t bytes, int width, int rows, void* hip_stream,
                           double* h_ms, double* h_rows) {
    if (!d_buf || !h_ms || !h_rows || rows < 1 || bytes < 4096) return -1;
    if (width != 4 && width != 20 && width != 64) return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint32_t row_mask = pow2_mask(bytes / (size_t)width);
    const dim3 grid((unsigned)(kGatherLanes / kThreads)), block(kThreads);
    uint32_t* dst = static_cast<uint32_t*>(d_buf);
    *h_rows = (double)kGatherLanes * rows;
    return time_second_run(s, [&] {
        if (width == 4) hipLaunchKernelGGL(scatter_kernel<1>, grid, block, 0, s, dst, row_mask, rows);
        if (width == 20) hipLaunchKernelGGL(scatter_kernel<5>, grid, block, 0, s, dst, row_mask, rows);
        if (width == 64) hipLaunchKernelGGL(scatter_kernel<16>, grid, block, 0, s, dst, row_mask, rows);
    }, h_ms);
}

// One binning pass over n 12-byte items (d_items, words 0 = key = 32 random bits) into 256 bins
// of d_out (cap items each, cap = n / 256 * 5 / 4) through LDS; d_cursor: 257 words.  *h_ms =
// time of the pass; *h_dropped = items that did not fit their bin (0 for uniform keys).
int surel_membench_bin(const void* d_items, size_t n, void* d_out, size_t out_bytes,
                       uint32_t* d_cursor, void* hip_stream, double* h_ms, double* h_dropped) {
    if (!d_items || !d_out || !d_cursor || !h_ms || !h_dropped || n < 1 || n > 0x7FFFFFFFull)
        return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint32_t cap = (uint32_t)(n / kBins * 5 / 4 + kBinFlush);
    if ((size_t)cap * kBins * 12 > out_bytes) return -1;
    const size_t lds_bytes = ((size_t)kBins * kBinStage * 3 + 3 * kBins) * 4;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(bin_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
        return -3;
    int n_cu = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return -3;
    const int rc = time_second_run(s, [&] {
        (void)hipMemsetAsync(d_cursor, 0, (kBins + 1) * sizeof(uint32_t), s);
        hipLaunchKernelGGL(bin_kernel, dim3((unsigned)n_cu), dim3(kBinThreads), lds_bytes, s,
                           static_cast<const uint32_t*>(d_items), n, 24, cap,
                           static_cast<uint32_t*>(d_out), d_cursor);
    }, h_ms);
    if (rc != 0) return rc;
    uint32_t dropped = 0;
    if (hipMemcpy(&dropped, d_cursor + kBins, sizeof(uint32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return -3;
    *h_dropped = (double)dropped;
    return 0;
}

}  // extern "C"
