// Memory-system micro-benchmarks of the GPU that libsurel's kernels are judged against:
// streaming read / write / copy, chains of dependent random gathers from a table of a given
// size (what a walker does: the address of the next load comes out of the previous one), and
// random scatters of short rows.  Benchmark tooling, not part of the hot path: `bench.py
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

__global__ void read_kernel(const int4* __restrict__ a, size_t n, uint32_t* sink) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    int acc = 0;
    for (; i < n; i += stride) {
        const int4 v = a[i];
        acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 0x12345678) sink[0] = (uint32_t)acc;  // keeps the loads alive
}

__global__ void write_kernel(int4* __restrict__ b, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) b[i] = make_int4(1, 2, 3, (int)i);
}

__global__ void copy_kernel(const int4* __restrict__ a, int4* __restrict__ b, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) b[i] = a[i];
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
constexpr int kStreamBlocks = 8192;
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

// kind 0: read `bytes` of d_buf; 1: write them; 2: copy the first half of d_buf to the second
// (bytes / 2 read and bytes / 2 written).  16 bytes per lane and access.  *h_ms = kernel time.
int surel_membench_stream(int kind, void* d_buf, size_t bytes, uint32_t* d_sink, void* hip_stream,
                          double* h_ms) {
    if (!d_buf || !d_sink || !h_ms || bytes < 32 || kind < 0 || kind > 2) return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int4* a = static_cast<int4*>(d_buf);
    const size_t n = bytes / 16;
    return time_second_run(s, [&] {
        if (kind == 0) hipLaunchKernelGGL(read_kernel, dim3(kStreamBlocks), dim3(kThreads), 0, s, a, n, d_sink);
        if (kind == 1) hipLaunchKernelGGL(write_kernel, dim3(kStreamBlocks), dim3(kThreads), 0, s, a, n);
        if (kind == 2) hipLaunchKernelGGL(copy_kernel, dim3(kStreamBlocks), dim3(kThreads), 0, s, a, a + n / 2, n / 2);
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

}  // extern "C"
