// The C ABI of libsurel: argument validation, workspace management and the launch sequence
// of each call.  See include/surel.h for the contract of every entry point.
#include "../../include/surel.h"

#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "kernels.h"

struct surel_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    int max_lds_bytes = 0;
    int n_cu = 0;                 // compute units of the device
    uint32_t spin_limit = 1u << 22;  // bound of every wait inside the fused walk + RPE kernel
    uint32_t* d_err = nullptr;    // sticky device error word
    int64_t* h_pinned = nullptr;  // 2 x int64 of pinned host memory for small read-backs
    void* d_ws = nullptr;         // grow-only workspace: row counts + scan partials
    size_t ws_bytes = 0;
    void* d_rec = nullptr;        // grow-only workspace: per-edge neighbour records of the walk
    size_t rec_bytes = 0;
    void* d_lb = nullptr;         // grow-only workspace: look-back words of the fused kernel
    size_t lb_bytes = 0;
    void* d_prune = nullptr;      // grow-only workspace: hash slots, sort list, counters of prune
    size_t prune_bytes = 0;
    void* d_batch = nullptr;      // grow-only workspace: sort arrays of the incidence lists, hash
    size_t batch_bytes = 0;       // tables of the mini-batch search
    void* d_scratch = nullptr;    // this device's copy of the file-scope `scratch` array below
    bool no_spans = false;        // set while a call that must not allocate runs (no new events)
    // optional per-kernel timing (surel_profile_*)
    struct Span {
        int kernel;
        hipEvent_t start, stop;
    };
    bool profiling = false;
    std::vector<Span> spans;          // recorded, not yet read
    std::vector<hipEvent_t> free_events;
    double prof_ms[SUREL_K_COUNT] = {};
    int64_t prof_launches[SUREL_K_COUNT] = {};
};

// Scratch of surel_join_queries_noalloc: a file-scope device array instead of a workspace from
// hipMalloc, so that the call allocates nothing.  It holds the queries' row counts (int32 each)
// and, behind them, the partial sums of their scan.  Every device that runs the library holds
// its own copy until the process ends.  Host code never takes the array's name for an address:
// surel_create asks hipGetSymbolAddress for the current device's copy and keeps that pointer in
// the context.
constexpr size_t kScratchCountsBytes = (size_t)SUREL_NOALLOC_MAX_QUERIES * sizeof(int32_t);
constexpr size_t kScratchBytes = kScratchCountsBytes + 8192;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int device) {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == device) || (hipSetDevice(device) == hipSuccess);
        if (prev == device) prev = -1;
    }
    ~DeviceGuard() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// The uint16 count arrays are moved as 32-bit words wherever possible.
bool misaligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; }

// Brackets the launches made during its lifetime with two events on the context's stream
// when profiling is on; does nothing otherwise.
class KernelSpan {
  public:
    KernelSpan(surel_ctx* ctx, int kernel) : ctx_(ctx) {
        if (!ctx->profiling || ctx->no_spans) return;
        span_.kernel = kernel;
        span_.start = take();
        span_.stop = take();
        if (!span_.start || !span_.stop) {
            give_back();
            return;
        }
        active_ = hipEventRecord(span_.start, ctx->stream) == hipSuccess;
        if (!active_) give_back();
    }
    ~KernelSpan() {
        if (!active_) return;
        if (hipEventRecord(span_.stop, ctx_->stream) == hipSuccess) {
            ctx_->spans.push_back(span_);
        } else {
            give_back();
        }
    }
    KernelSpan(const KernelSpan&) = delete;
    KernelSpan& operator=(const KernelSpan&) = delete;

  private:
    hipEvent_t take() {
        if (!ctx_->free_events.empty()) {
            hipEvent_t e = ctx_->free_events.back();
            ctx_->free_events.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    void give_back() {
        if (span_.start) ctx_->free_events.push_back(span_.start);
        if (span_.stop) ctx_->free_events.push_back(span_.stop);
        span_.start = span_.stop = nullptr;
    }
    surel_ctx* ctx_;
    surel_ctx::Span span_{0, nullptr, nullptr};
    bool active_ = false;
};

// Wait for the stream and fold every recorded span into the per-kernel totals.
int drain_spans(surel_ctx* ctx) {
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    for (const surel_ctx::Span& sp : ctx->spans) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, sp.start, sp.stop) == hipSuccess) {
            ctx->prof_ms[sp.kernel] += (double)ms;
            ctx->prof_launches[sp.kernel] += 1;
        }
        ctx->free_events.push_back(sp.start);
        ctx->free_events.push_back(sp.stop);
    }
    ctx->spans.clear();
    return SUREL_OK;
}

// Grows one of the context's workspaces to `need` bytes (contents are not kept).  The old
// buffer may still be in use by earlier work on the stream, so the stream is drained first.
int grow_buffer(surel_ctx* ctx, void** buf, size_t* have, size_t need) {
    if (need <= *have) return SUREL_OK;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    if (*buf) (void)hipFree(*buf);
    *buf = nullptr;
    *have = 0;
    if (hipMalloc(buf, need) != hipSuccess) {
        (void)hipGetLastError();
        return SUREL_E_HIP;
    }
    *have = need;
    return SUREL_OK;
}

// Workspace: int32 counts[n] followed by the int64 scan partials.
int ensure_workspace(surel_ctx* ctx, int64_t n, int32_t** counts, int64_t** partials) {
    const size_t counts_bytes = align_up((size_t)(n > 0 ? n : 1) * sizeof(int32_t), 256);
    const size_t part_bytes = (size_t)surel::scan_partials_len(n) * sizeof(int64_t);
    const size_t need = counts_bytes + align_up(part_bytes, 256);
    if (int rc = grow_buffer(ctx, &ctx->d_ws, &ctx->ws_bytes, need)) return rc;
    *counts = static_cast<int32_t*>(ctx->d_ws);
    *partials = reinterpret_cast<int64_t*>(static_cast<char*>(ctx->d_ws) + counts_bytes);
    return SUREL_OK;
}

// Wait for the stream and fetch off[n] (the row total) into *h_rows.
int read_total(surel_ctx* ctx, const int64_t* d_off, int64_t n, int64_t* h_rows) {
    if (hipMemcpyAsync(ctx->h_pinned, d_off + n, sizeof(int64_t), hipMemcpyDeviceToHost,
                       ctx->stream) != hipSuccess)
        return SUREL_E_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    *h_rows = ctx->h_pinned[0];
    return SUREL_OK;
}

// The walk's per-edge neighbour records, made afresh from the CSR when the job is large enough
// to want them.  *records stays null when it is not, or when the device has no room (not an
// error: the walk then reads the CSR directly).
int make_edge_records(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                      int32_t n_nodes, int64_t n_edges, int64_t n_seeds, int32_t M, int32_t m,
                      surel::EdgeRecords* records) {
    *records = surel::EdgeRecords{};
    if (!surel::walks_want_records(n_edges, n_seeds, M, m)) return SUREL_OK;
    surel::EdgeRecords plan = surel::edge_record_plan(n_nodes, n_edges);
    const size_t need = surel::edge_record_bytes(plan, n_edges);
    (void)grow_buffer(ctx, &ctx->d_rec, &ctx->rec_bytes, need);
    if (ctx->rec_bytes < need) return SUREL_OK;
    plan.data = ctx->d_rec;
    KernelSpan span(ctx, SUREL_K_EDGE_RECORDS);
    if (surel::launch_edge_records(ctx->stream, d_row_ptr, d_col_idx, n_nodes, n_edges, plan) !=
        hipSuccess)
        return SUREL_E_HIP;
    *records = plan;
    return SUREL_OK;
}

int check_walk_shape(int32_t n_nodes, int64_t n_seeds, int32_t M, int32_t m) {
    if (n_nodes < 1 || n_nodes > SUREL_MAX_NODES) return SUREL_E_RANGE;
    if (n_seeds < 0 || n_seeds > 0x7FFFFFFFll) return SUREL_E_RANGE;
    if (M < 1 || M > SUREL_MAX_WALKS) return SUREL_E_RANGE;
    if (m < 1 || m > SUREL_MAX_STEPS) return SUREL_E_RANGE;
    return SUREL_OK;
}

}  // namespace

extern "C" {

int surel_create(surel_ctx** out, int device, void* hip_stream) {
    if (!out) return SUREL_E_NULL;
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) {
        (void)hipGetLastError();
        return SUREL_E_HIP;
    }
    DeviceGuard guard(device);
    if (!guard.ok) return SUREL_E_HIP;
    surel_ctx* ctx = new (std::nothrow) surel_ctx();
    if (!ctx) return SUREL_E_HIP;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    bool ok = hipDeviceGetAttribute(&ctx->max_lds_bytes, hipDeviceAttributeMaxSharedMemoryPerBlock,
                                    device) == hipSuccess;
    ok = ok && hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount,
                                     device) == hipSuccess && ctx->n_cu > 0;
    ok = ok && hipMalloc(reinterpret_cast<void**>(&ctx->d_err), 256) == hipSuccess;
    ok = ok && hipMemsetAsync(ctx->d_err, 0, 256, ctx->stream) == hipSuccess;
    ok = ok && hipHostMalloc(reinterpret_cast<void**>(&ctx->h_pinned), 2 * sizeof(int64_t),
                             hipHostMallocDefault) == hipSuccess;
    ok = ok && hipStreamSynchronize(ctx->stream) == hipSuccess;
    // where THIS device keeps its copy of the static scratch array (the device is current here)
    ok = ok && hipGetSymbolAddress(&ctx->d_scratch, HIP_SYMBOL(scratch)) == hipSuccess &&
         ctx->d_scratch != nullptr;
    if (!ok) {
        if (ctx->d_err) (void)hipFree(ctx->d_err);
        if (ctx->h_pinned) (void)hipHostFree(ctx->h_pinned);
        delete ctx;
        (void)hipGetLastError();
        return SUREL_E_HIP;
    }
    *out = ctx;
    return SUREL_OK;
}

void surel_destroy(surel_ctx* ctx) {
    if (!ctx) return;
    DeviceGuard guard(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (const surel_ctx::Span& sp : ctx->spans) {
        (void)hipEventDestroy(sp.start);
        (void)hipEventDestroy(sp.stop);
    }
    for (hipEvent_t e : ctx->free_events) (void)hipEventDestroy(e);
    if (ctx->d_ws) (void)hipFree(ctx->d_ws);
    if (ctx->d_rec) (void)hipFree(ctx->d_rec);
    if (ctx->d_lb) (void)hipFree(ctx->d_lb);
    if (ctx->d_prune) (void)hipFree(ctx->d_prune);
    if (ctx->d_batch) (void)hipFree(ctx->d_batch);
    if (ctx->d_err) (void)hipFree(ctx->d_err);
    if (ctx->h_pinned) (void)hipHostFree(ctx->h_pinned);
    delete ctx;
}

const char* surel_strerror(int status) {
    switch (status) {
        case SUREL_OK: return "ok";
        case SUREL_E_NULL: return "a required pointer is NULL";
        case SUREL_E_RANGE: return "a size or parameter is outside the documented limits";
        case SUREL_E_HIP: return "a HIP runtime call failed";
        case SUREL_E_CAPACITY: return "the output needs more rows than cap_rows";
        case SUREL_E_CTX: return "the context pointer is NULL";
        case SUREL_E_DEVICE: return "the device error word is non-zero";
        default: return "unknown status";
    }
}

int64_t surel_rpe_rows_bound(int64_t n_seeds, int32_t M, int32_t m) {
    if (n_seeds <= 0 || M <= 0 || m <= 0) return 0;
    return n_seeds * (1 + (int64_t)M * m);
}

int surel_sample_walks(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                       int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds,
                       int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,
                       int32_t* d_walks, int32_t* d_set_sizes) {
    if (int rc = check_walk_shape(n_nodes, n_seeds, M, m)) return rc;
    if (n_edges < 0 || n_edges > 0x7FFFFFFFll) return SUREL_E_RANGE;
    if (d_set_sizes && (int64_t)M * (m + 1) > SUREL_MAX_WALK_ENTRIES) return SUREL_E_RANGE;
    if (!d_row_ptr || (n_edges > 0 && !d_col_idx)) return SUREL_E_NULL;
    if (n_seeds > 0 && (!d_seeds || !d_walks)) return SUREL_E_NULL;
    if (!ctx) return SUREL_E_CTX;
    if (n_seeds == 0) return SUREL_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    surel::EdgeRecords records;
    if (int rc = make_edge_records(ctx, d_row_ptr, d_col_idx, n_nodes, n_edges, n_seeds, M, m,
                                   &records))
        return rc;
    KernelSpan span(ctx, SUREL_K_WALK);
    hipError_t rc = surel::launch_walks(ctx->stream, d_row_ptr, d_col_idx, n_nodes, n_edges,
                                        d_seeds, n_seeds, M, m, rng_seed, d_walks, d_set_sizes,
                                        records, ctx->d_err);
    return rc == hipSuccess ? SUREL_OK : SUREL_E_HIP;
}

// Argument checks shared by the three forms of the RPE builder.
static int check_rpe_args(int32_t n_nodes, int64_t n_seeds, int32_t M, int32_t m,
                          const int32_t* d_walks) {
    if (int rc = check_walk_shape(n_nodes, n_seeds, M, m)) return rc;
    if ((int64_t)M * (m + 1) > SUREL_MAX_WALK_ENTRIES) return SUREL_E_RANGE;
    if (n_seeds > 0 && !d_walks) return SUREL_E_NULL;
    return SUREL_OK;
}

// Waits for the stream and reports the row total that a scan or a scanner wave left at off[n]
// (-1: the kernel gave up on a bounded wait before it got there).
static int report_total(surel_ctx* ctx, const int64_t* d_off, int64_t n, bool has_outputs,
                        int64_t cap_rows, int64_t* h_rows) {
    if (int rc = read_total(ctx, d_off, n, h_rows)) return rc;
    if (*h_rows < 0) return SUREL_E_DEVICE;
    if (has_outputs && *h_rows > cap_rows) return SUREL_E_CAPACITY;
    return SUREL_OK;
}

// Phase A of the RPE builder: per-seed set sizes (the caller's, or counted here) -> rpe_off.
static int rpe_layout(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M, int32_t m,
                      int32_t n_nodes, const int32_t* d_set_sizes, int64_t* d_rpe_off) {
    int32_t* counts = nullptr;
    int64_t* partials = nullptr;
    if (int rc = ensure_workspace(ctx, n_seeds, &counts, &partials)) return rc;
    const int32_t* sizes = d_set_sizes;
    if (!sizes) {
        KernelSpan span(ctx, SUREL_K_RPE_COUNT);
        if (surel::launch_rpe_count(ctx->stream, d_walks, n_seeds, M, m, n_nodes, counts,
                                    ctx->d_err) != hipSuccess)
            return SUREL_E_HIP;
        sizes = counts;
    }
    KernelSpan span(ctx, SUREL_K_SCAN);
    if (surel::launch_exclusive_scan(ctx->stream, sizes, n_seeds, d_rpe_off, partials) != hipSuccess)
        return SUREL_E_HIP;
    return SUREL_OK;
}

// Phase B: the rows, at the offsets given.
static int rpe_rows(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M, int32_t m,
                    int32_t n_nodes, const int64_t* d_rpe_off, int64_t cap_rows,
                    int32_t* d_rpe_ids, uint16_t* d_rpe_cnt) {
    KernelSpan span(ctx, SUREL_K_RPE_FILL);
    hipError_t hrc = surel::launch_rpe_fill(ctx->stream, ctx->max_lds_bytes, d_walks, n_seeds, M, m,
                                            n_nodes, d_rpe_off, cap_rows, d_rpe_ids, d_rpe_cnt,
                                            ctx->d_err);
    if (hrc == hipErrorInvalidValue) return SUREL_E_RANGE;
    return hrc == hipSuccess ? SUREL_OK : SUREL_E_HIP;
}

int surel_build_rpe_count(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M,
                          int32_t m, int32_t n_nodes, const int32_t* d_set_sizes,
                          int64_t* d_rpe_off, int64_t* h_rows) {
    if (int rc = check_rpe_args(n_nodes, n_seeds, M, m, d_walks)) return rc;
    if (!d_rpe_off) return SUREL_E_NULL;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (int rc = rpe_layout(ctx, d_walks, n_seeds, M, m, n_nodes, d_set_sizes, d_rpe_off)) return rc;
    if (h_rows) return report_total(ctx, d_rpe_off, n_seeds, false, 0, h_rows);
    return SUREL_OK;
}

int surel_build_rpe_fill(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M,
                         int32_t m, int32_t n_nodes, const int64_t* d_rpe_off, int64_t cap_rows,
                         int32_t* d_rpe_ids, uint16_t* d_rpe_cnt) {
    if (int rc = check_rpe_args(n_nodes, n_seeds, M, m, d_walks)) return rc;
    if (cap_rows < 0) return SUREL_E_RANGE;
    if (!d_rpe_off) return SUREL_E_NULL;
    if (n_seeds > 0 && cap_rows > 0 && (!d_rpe_ids || !d_rpe_cnt)) return SUREL_E_NULL;
    if (misaligned4(d_rpe_cnt)) return SUREL_E_RANGE;
    if (!ctx) return SUREL_E_CTX;
    if (n_seeds == 0) return SUREL_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    return rpe_rows(ctx, d_walks, n_seeds, M, m, n_nodes, d_rpe_off, cap_rows, d_rpe_ids, d_rpe_cnt);
}

int surel_build_rpe(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M,
                    int32_t m, int32_t n_nodes, const int32_t* d_set_sizes, int64_t cap_rows,
                    int64_t* d_rpe_off,
                    int32_t* d_rpe_ids, uint16_t* d_rpe_cnt, int64_t* h_rows) {
    if (int rc = check_rpe_args(n_nodes, n_seeds, M, m, d_walks)) return rc;
    if (cap_rows < 0) return SUREL_E_RANGE;
    if (!d_rpe_off) return SUREL_E_NULL;
    if ((d_rpe_ids == nullptr) != (d_rpe_cnt == nullptr)) return SUREL_E_NULL;
    if (misaligned4(d_rpe_cnt)) return SUREL_E_RANGE;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (int rc = rpe_layout(ctx, d_walks, n_seeds, M, m, n_nodes, d_set_sizes, d_rpe_off)) return rc;
    if (d_rpe_ids && n_seeds > 0) {
        if (int rc = rpe_rows(ctx, d_walks, n_seeds, M, m, n_nodes, d_rpe_off, cap_rows, d_rpe_ids,
                              d_rpe_cnt))
            return rc;
    }
    if (h_rows) return report_total(ctx, d_rpe_off, n_seeds, d_rpe_ids != nullptr, cap_rows, h_rows);
    return SUREL_OK;
}

// Argument checks shared by the two fused walk + RPE calls.
static int check_fused_args(const int32_t* d_row_ptr, const int32_t* d_col_idx, int32_t n_nodes,
                            int64_t n_edges, const int32_t* d_seeds, int64_t n_seeds, int32_t M,
                            int32_t m, const int32_t* d_walks, int64_t cap_rows,
                            const int64_t* d_rpe_off) {
    if (int rc = check_walk_shape(n_nodes, n_seeds, M, m)) return rc;
    if (n_edges < 0 || n_edges > 0x7FFFFFFFll) return SUREL_E_RANGE;
    if ((int64_t)M * (m + 1) > SUREL_MAX_WALK_ENTRIES) return SUREL_E_RANGE;
    if (cap_rows < 0) return SUREL_E_RANGE;
    if (!d_row_ptr || (n_edges > 0 && !d_col_idx) || !d_rpe_off) return SUREL_E_NULL;
    if (n_seeds > 0 && (!d_seeds || !d_walks)) return SUREL_E_NULL;
    return SUREL_OK;
}

// The fused kernel (n_seeds >= 1): edge records if the job wants them, look-back scratch, launch.
// code / slots / counters: the hash set of distinct count vectors, or null.
static int fused_launch(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                        int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds, int64_t n_seeds,
                        int32_t M, int32_t m, uint64_t rng_seed, int32_t* d_walks, int64_t cap_rows,
                        int64_t* d_rpe_off, int32_t* d_rpe_ids, uint16_t* d_rpe_cnt, int32_t* d_code,
                        uint32_t* slots, int64_t cap_T, unsigned long long* counters) {
    surel::EdgeRecords records;
    if (int rc = make_edge_records(ctx, d_row_ptr, d_col_idx, n_nodes, n_edges, n_seeds, M, m,
                                   &records))
        return rc;
    const size_t lb_need = (size_t)surel::lookback_words(n_seeds) * sizeof(uint64_t);
    if (int rc = grow_buffer(ctx, &ctx->d_lb, &ctx->lb_bytes, lb_need)) return rc;
    KernelSpan span(ctx, SUREL_K_WALK_RPE);
    hipError_t hrc = surel::launch_walk_rpe(
        ctx->stream, ctx->max_lds_bytes, ctx->n_cu, d_row_ptr, d_col_idx, n_nodes, n_edges, d_seeds,
        n_seeds, M, m, rng_seed, d_walks, cap_rows, d_rpe_off, d_rpe_ids, d_rpe_cnt, records,
        static_cast<uint64_t*>(ctx->d_lb), ctx->spin_limit, ctx->d_err, d_code, slots, cap_T,
        counters);
    if (hrc == hipErrorInvalidValue) return SUREL_E_RANGE;
    return hrc == hipSuccess ? SUREL_OK : SUREL_E_HIP;
}

// rpe_off[0] = 0 of an empty seed list, by the scan's own kernels (valid under stream capture).
static int empty_table(surel_ctx* ctx, int64_t* d_rpe_off) {
    int32_t* counts = nullptr;
    int64_t* partials = nullptr;
    if (int rc = ensure_workspace(ctx, 0, &counts, &partials)) return rc;
    if (surel::launch_exclusive_scan(ctx->stream, counts, 0, d_rpe_off, partials) != hipSuccess)
        return SUREL_E_HIP;
    return SUREL_OK;
}

int surel_sample_walks_rpe(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                           int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds,
                           int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,
                           int32_t* d_walks, int64_t cap_rows, int64_t* d_rpe_off,
                           int32_t* d_rpe_ids, uint16_t* d_rpe_cnt, int64_t* h_rows) {
    if (int rc = check_fused_args(d_row_ptr, d_col_idx, n_nodes, n_edges, d_seeds, n_seeds, M, m,
                                  d_walks, cap_rows, d_rpe_off))
        return rc;
    if ((d_rpe_ids == nullptr) != (d_rpe_cnt == nullptr)) return SUREL_E_NULL;
    if (misaligned4(d_rpe_cnt)) return SUREL_E_RANGE;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (n_seeds == 0) {
        if (int rc = empty_table(ctx, d_rpe_off)) return rc;
    } else if (int rc = fused_launch(ctx, d_row_ptr, d_col_idx, n_nodes, n_edges, d_seeds, n_seeds,
                                     M, m, rng_seed, d_walks, cap_rows, d_rpe_off, d_rpe_ids,
                                     d_rpe_cnt, nullptr, nullptr, 0, nullptr)) {
        return rc;
    }
    if (h_rows) return report_total(ctx, d_rpe_off, n_seeds, d_rpe_ids != nullptr, cap_rows, h_rows);
    return SUREL_OK;
}

// The scratch of the pruning calls inside the context's workspace.
struct PruneScratch {
    uint32_t* slots;
    uint32_t* list;
    unsigned long long* counters;
};
static int prune_scratch(surel_ctx* ctx, int64_t cap_T, PruneScratch* out) {
    const size_t slot_bytes = surel::prune_slot_bytes(cap_T);
    const size_t list_bytes = align_up(surel::prune_list_bytes(cap_T), 256);
    if (int rc = grow_buffer(ctx, &ctx->d_prune, &ctx->prune_bytes, slot_bytes + list_bytes + 256))
        return rc;
    char* ws = static_cast<char*>(ctx->d_prune);
    out->slots = reinterpret_cast<uint32_t*>(ws);
    out->list = reinterpret_cast<uint32_t*>(ws + slot_bytes);
    out->counters = reinterpret_cast<unsigned long long*>(ws + slot_bytes + list_bytes);
    return SUREL_OK;
}

int surel_sample_walks_rpe_ids(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                               int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds,
                               int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,
                               int32_t* d_walks, int64_t cap_rows, int64_t* d_rpe_off,
                               int32_t* d_rpe_ids, uint16_t* d_rpe_cnt, int32_t* d_code,
                               int64_t cap_T, uint16_t* d_T, int64_t* h_rows, int64_t* h_n_T) {
    if (int rc = check_fused_args(d_row_ptr, d_col_idx, n_nodes, n_edges, d_seeds, n_seeds, M, m,
                                  d_walks, cap_rows, d_rpe_off))
        return rc;
    if (cap_T < 1 || cap_T > SUREL_MAX_DISTINCT) return SUREL_E_RANGE;
    if (!d_T || !h_rows || !h_n_T) return SUREL_E_NULL;
    if (cap_rows > 0 && (!d_rpe_ids || !d_code)) return SUREL_E_NULL;
    if (misaligned4(d_rpe_cnt)) return SUREL_E_RANGE;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    *h_n_T = 0;
    if (n_seeds == 0) {
        if (int rc = empty_table(ctx, d_rpe_off)) return rc;
        return report_total(ctx, d_rpe_off, 0, true, cap_rows, h_rows);
    }
    PruneScratch ps;
    if (int rc = prune_scratch(ctx, cap_T, &ps)) return rc;
    if (surel::launch_prune_clear(ctx->stream, cap_T, ps.slots, ps.counters) != hipSuccess)
        return SUREL_E_HIP;
    if (int rc = fused_launch(ctx, d_row_ptr, d_col_idx, n_nodes, n_edges, d_seeds, n_seeds, M, m,
                              rng_seed, d_walks, cap_rows, d_rpe_off, d_rpe_ids, d_rpe_cnt, d_code,
                              ps.slots, cap_T, ps.counters))
        return rc;
    // the two totals in one read-back: table rows, distinct vectors
    if (hipMemcpyAsync(ctx->h_pinned + 1, ps.counters, sizeof(int64_t), hipMemcpyDeviceToHost,
                       ctx->stream) != hipSuccess)
        return SUREL_E_HIP;
    if (int rc = report_total(ctx, d_rpe_off, n_seeds, true, cap_rows, h_rows)) {
        *h_n_T = ctx->h_pinned[1];
        return rc;  // rows that did not fit have no codes: nothing to finish
    }
    const int64_t n_T = ctx->h_pinned[1];
    *h_n_T = n_T;
    if (n_T > cap_T) return SUREL_E_CAPACITY;
    KernelSpan span(ctx, SUREL_K_PRUNE);
    if (surel::launch_prune_finish(ctx->stream, ctx->n_cu, *h_rows, m, cap_T, n_T, ps.slots,
                                   ps.counters, ps.list, d_T, d_code) != hipSuccess)
        return SUREL_E_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    return SUREL_OK;
}

// The join over vectors of m+1 16-bit entries per table row; absent16 fills the vector of a
// list that has no row for a node (0 for counts; 0xFFFF for 32-bit codes seen as two halves).
static int check_join_args(int32_t m, int32_t max_set, int64_t n_blocks, int64_t n_queries,
                           int32_t k, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                           const int32_t* d_queries, const int64_t* d_join_off) {
    if (m < 1 || m > SUREL_MAX_STEPS) return SUREL_E_RANGE;
    if (k < 2 || k > SUREL_MAX_TUPLE) return SUREL_E_RANGE;
    if (max_set < 1 || max_set > SUREL_MAX_SET) return SUREL_E_RANGE;
    if (n_blocks < 0 || n_queries < 0 || n_queries > 0x7FFFFFFFll) return SUREL_E_RANGE;
    if (!d_join_off) return SUREL_E_NULL;
    if (n_queries > 0 && (!d_queries || !d_rpe_off || !d_rpe_ids)) return SUREL_E_NULL;
    return SUREL_OK;
}

// Device scratch of a join call: the queries' row counts and the partials of their scan.
struct JoinScratch {
    int32_t* counts = nullptr;
    int64_t* partials = nullptr;
};

// Phase A: union sizes -> join_off.
static int join_layout(surel_ctx* ctx, const JoinScratch& ws, const int64_t* d_rpe_off,
                       const int32_t* d_rpe_ids, int64_t n_blocks, int32_t max_set,
                       const int32_t* d_queries, int64_t n_queries, int32_t k,
                       int64_t* d_join_off) {
    hipError_t hrc;
    {
        KernelSpan span(ctx, SUREL_K_JOIN_COUNT);
        hrc = surel::launch_join_count(ctx->stream, ctx->max_lds_bytes, d_rpe_off,
                                       d_rpe_ids, n_blocks, max_set, d_queries, n_queries, k,
                                       ws.counts, ctx->d_err);
    }
    if (hrc == hipErrorInvalidValue) return SUREL_E_RANGE;
    if (hrc != hipSuccess) return SUREL_E_HIP;
    KernelSpan span(ctx, SUREL_K_SCAN);
    if (surel::launch_exclusive_scan(ctx->stream, ws.counts, n_queries, d_join_off, ws.partials) !=
        hipSuccess)
        return SUREL_E_HIP;
    return SUREL_OK;
}

// Phase B: the rows, at the offsets given.
static int join_rows(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                     const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
                     const int32_t* d_queries, int64_t n_queries, int32_t k,
                     const int64_t* d_join_off, int64_t cap_rows, int32_t* d_join_ids,
                     uint16_t* d_join_cnt, uint16_t absent16) {
    KernelSpan span(ctx, SUREL_K_JOIN_FILL);
    hipError_t hrc = surel::launch_join_fill(ctx->stream, ctx->max_lds_bytes, d_rpe_off,
                                             d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set, d_queries,
                                             n_queries, k, d_join_off, cap_rows, d_join_ids,
                                             d_join_cnt, absent16, ctx->d_err);
    if (hrc == hipErrorInvalidValue) return SUREL_E_RANGE;
    return hrc == hipSuccess ? SUREL_OK : SUREL_E_HIP;
}

// The whole join with the scratch given: layout, then (unless the outputs are NULL) the rows.
static int join_vectors(surel_ctx* ctx, const JoinScratch& ws, const int64_t* d_rpe_off,
                        const int32_t* d_rpe_ids, const uint16_t* d_rpe_cnt, int64_t n_blocks,
                        int32_t m, int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                        int32_t k, int64_t cap_rows, int64_t* d_join_off, int32_t* d_join_ids,
                        uint16_t* d_join_cnt, uint16_t absent16, int64_t* h_rows) {
    if (int rc = join_layout(ctx, ws, d_rpe_off, d_rpe_ids, n_blocks, max_set, d_queries, n_queries,
                             k, d_join_off))
        return rc;
    if (d_join_ids && n_queries > 0) {
        if (int rc = join_rows(ctx, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set, d_queries,
                               n_queries, k, d_join_off, cap_rows, d_join_ids, d_join_cnt, absent16))
            return rc;
    }
    if (h_rows)
        return report_total(ctx, d_join_off, n_queries, d_join_ids != nullptr, cap_rows, h_rows);
    return SUREL_OK;
}

// Argument checks of the calls that do the whole join.
static int check_whole_join(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                            const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
                            const int32_t* d_queries, int64_t n_queries, int32_t k, int64_t cap_rows,
                            const int64_t* d_join_off, const int32_t* d_join_ids,
                            const uint16_t* d_join_cnt) {
    if (int rc = check_join_args(m, max_set, n_blocks, n_queries, k, d_rpe_off, d_rpe_ids,
                                 d_queries, d_join_off))
        return rc;
    if (cap_rows < 0) return SUREL_E_RANGE;
    if ((d_join_ids == nullptr) != (d_join_cnt == nullptr)) return SUREL_E_NULL;
    if (n_queries > 0 && d_join_ids && !d_rpe_cnt) return SUREL_E_NULL;
    if (misaligned4(d_rpe_cnt) || misaligned4(d_join_cnt)) return SUREL_E_RANGE;
    if (!ctx) return SUREL_E_CTX;
    return SUREL_OK;
}

static int join_checked(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                        const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
                        const int32_t* d_queries, int64_t n_queries, int32_t k, int64_t cap_rows,
                        int64_t* d_join_off, int32_t* d_join_ids, uint16_t* d_join_cnt,
                        uint16_t absent16, int64_t* h_rows) {
    if (int rc = check_whole_join(ctx, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set,
                                  d_queries, n_queries, k, cap_rows, d_join_off, d_join_ids,
                                  d_join_cnt))
        return rc;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    JoinScratch ws;
    if (int rc = ensure_workspace(ctx, n_queries, &ws.counts, &ws.partials)) return rc;
    return join_vectors(ctx, ws, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set, d_queries,
                        n_queries, k, cap_rows, d_join_off, d_join_ids, d_join_cnt, absent16, h_rows);
}

int surel_join_count(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                     int64_t n_blocks, int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                     int32_t k, int64_t* d_join_off, int64_t* h_rows) {
    if (int rc = check_join_args(1, max_set, n_blocks, n_queries, k, d_rpe_off, d_rpe_ids,
                                 d_queries, d_join_off))
        return rc;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    JoinScratch ws;
    if (int rc = ensure_workspace(ctx, n_queries, &ws.counts, &ws.partials)) return rc;
    if (int rc = join_layout(ctx, ws, d_rpe_off, d_rpe_ids, n_blocks, max_set, d_queries, n_queries,
                             k, d_join_off))
        return rc;
    if (h_rows) return report_total(ctx, d_join_off, n_queries, false, 0, h_rows);
    return SUREL_OK;
}

int surel_join_fill(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                    const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
                    const int32_t* d_queries, int64_t n_queries, int32_t k,
                    const int64_t* d_join_off, int64_t cap_rows, int32_t* d_join_ids,
                    uint16_t* d_join_cnt) {
    if (int rc = check_join_args(m, max_set, n_blocks, n_queries, k, d_rpe_off, d_rpe_ids,
                                 d_queries, d_join_off))
        return rc;
    if (cap_rows < 0) return SUREL_E_RANGE;
    if (n_queries > 0 && cap_rows > 0 && (!d_join_ids || !d_join_cnt || !d_rpe_cnt))
        return SUREL_E_NULL;
    if (misaligned4(d_rpe_cnt) || misaligned4(d_join_cnt)) return SUREL_E_RANGE;
    if (!ctx) return SUREL_E_CTX;
    if (n_queries == 0) return SUREL_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    return join_rows(ctx, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set, d_queries,
                     n_queries, k, d_join_off, cap_rows, d_join_ids, d_join_cnt, 0);
}

int surel_join_queries(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                       const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m,
                       int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                       int32_t k, int64_t cap_rows, int64_t* d_join_off,
                       int32_t* d_join_ids, uint16_t* d_join_cnt, int64_t* h_rows) {
    return join_checked(ctx, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set, d_queries,
                        n_queries, k, cap_rows, d_join_off, d_join_ids, d_join_cnt, 0, h_rows);
}

int surel_join_queries_noalloc(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                               const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m,
                               int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                               int32_t k, int64_t cap_rows, int64_t* d_join_off,
                               int32_t* d_join_ids, uint16_t* d_join_cnt, int64_t* h_rows) {
    if (int rc = check_whole_join(ctx, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set,
                                  d_queries, n_queries, k, cap_rows, d_join_off, d_join_ids,
                                  d_join_cnt))
        return rc;
    if (n_queries > SUREL_NOALLOC_MAX_QUERIES) return SUREL_E_RANGE;
    static_assert(kScratchBytes >= kScratchCountsBytes +
                      (SUREL_NOALLOC_MAX_QUERIES / 2048 + 2) * sizeof(int64_t),
                  "the scan's partials must fit behind the counts");
    if ((size_t)surel::scan_partials_len(n_queries) * sizeof(int64_t) >
        kScratchBytes - kScratchCountsBytes)
        return SUREL_E_RANGE;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    // the device's static array through the pointer that surel_create looked up, never through
    // the array's name; every word the kernels read from it they have written in this call
    JoinScratch ws;
    ws.counts = static_cast<int32_t*>(ctx->d_scratch);
    ws.partials = reinterpret_cast<int64_t*>(static_cast<char*>(ctx->d_scratch) + kScratchCountsBytes);
    ctx->no_spans = true;  // timing a launch would create events
    const int rc = join_vectors(ctx, ws, d_rpe_off, d_rpe_ids, d_rpe_cnt, n_blocks, m, max_set,
                                d_queries, n_queries, k, cap_rows, d_join_off, d_join_ids,
                                d_join_cnt, 0, h_rows);
    ctx->no_spans = false;
    return rc;
}

int surel_join_query_ids(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                         const int32_t* d_code, int64_t n_blocks, int32_t max_set,
                         const int32_t* d_queries, int64_t n_queries, int32_t k, int64_t cap_rows,
                         int64_t* d_join_off, int32_t* d_join_ids, int32_t* d_join_codes,
                         int64_t* h_rows) {
    // a 32-bit code is a vector of two 16-bit entries; absent = 0xFFFF 0xFFFF = -1
    return join_checked(ctx, d_rpe_off, d_rpe_ids, reinterpret_cast<const uint16_t*>(d_code),
                        n_blocks, 1, max_set, d_queries, n_queries, k, cap_rows, d_join_off,
                        d_join_ids, reinterpret_cast<uint16_t*>(d_join_codes), 0xFFFFu, h_rows);
}

int surel_query_rpe_ids(surel_ctx* ctx, const int32_t* d_walks, const int64_t* d_rpe_off,
                        const int32_t* d_rpe_ids, const int32_t* d_code, int64_t n_blocks,
                        int64_t table_rows, int32_t M, int32_t m, int32_t max_set,
                        const int32_t* d_queries, int64_t n_queries, int32_t k, int32_t* d_out) {
    if (M < 1 || M > SUREL_MAX_WALKS || m < 1 || m > SUREL_MAX_STEPS) return SUREL_E_RANGE;
    if ((int64_t)M * (m + 1) >= (int64_t)0x7FFFFFFF / 9) return SUREL_E_RANGE;
    if (k < 2 || k > SUREL_MAX_TUPLE) return SUREL_E_RANGE;
    if (max_set < 1 || max_set > SUREL_MAX_SET) return SUREL_E_RANGE;
    if (n_blocks < 0 || n_queries < 0 || n_queries > 0x7FFFFFFFll) return SUREL_E_RANGE;
    if (table_rows < 0 || table_rows > 0x7FFFFFFFll) return SUREL_E_RANGE;
    if (n_queries > 0 && (!d_walks || !d_rpe_off || !d_rpe_ids || !d_queries || !d_out))
        return SUREL_E_NULL;
    if (!ctx) return SUREL_E_CTX;
    if (n_queries == 0) return SUREL_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    KernelSpan span(ctx, SUREL_K_QUERY_IDS);
    hipError_t hrc = surel::launch_query_ids(ctx->stream, ctx->max_lds_bytes, d_walks,
                                             d_rpe_off, d_rpe_ids, d_code, n_blocks, M, m, max_set,
                                             table_rows, d_queries, n_queries, k, d_out,
                                             ctx->d_err);
    if (hrc == hipErrorInvalidValue) return SUREL_E_RANGE;
    return hrc == hipSuccess ? SUREL_OK : SUREL_E_HIP;
}

int surel_prune_rpe(surel_ctx* ctx, const uint16_t* d_rpe_cnt, int64_t n_rows, int32_t m,
                    int64_t cap_T, uint16_t* d_T, int32_t* d_code, int64_t* h_n_T) {
    if (m < 1 || m > SUREL_MAX_STEPS || n_rows < 0) return SUREL_E_RANGE;
    if (cap_T < 1 || cap_T > SUREL_MAX_DISTINCT) return SUREL_E_RANGE;
    if (!d_T || !h_n_T || (n_rows > 0 && (!d_rpe_cnt || !d_code))) return SUREL_E_NULL;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    PruneScratch ps;
    if (int rc = prune_scratch(ctx, cap_T, &ps)) return rc;
    uint32_t* slots = ps.slots;
    uint32_t* list = ps.list;
    unsigned long long* counters = ps.counters;
    KernelSpan span(ctx, SUREL_K_PRUNE);
    if (surel::launch_prune_collect(ctx->stream, ctx->n_cu, d_rpe_cnt, n_rows, m, cap_T, slots,
                                    counters, d_code, ctx->spin_limit, ctx->d_err) != hipSuccess)
        return SUREL_E_HIP;
    if (hipMemcpyAsync(ctx->h_pinned, counters, sizeof(int64_t), hipMemcpyDeviceToHost,
                       ctx->stream) != hipSuccess)
        return SUREL_E_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    const int64_t n_T = ctx->h_pinned[0];
    *h_n_T = n_T;
    if (n_T > cap_T) return SUREL_E_CAPACITY;
    if (surel::launch_prune_finish(ctx->stream, ctx->n_cu, n_rows, m, cap_T, n_T, slots, counters,
                                   list, d_T, d_code) != hipSuccess)
        return SUREL_E_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    return SUREL_OK;
}

int surel_query_incidence(surel_ctx* ctx, const int32_t* d_queries, int64_t n_queries, int32_t k,
                          int32_t n_nodes, int64_t* d_inc_off, int32_t* d_inc_q) {
    if (n_nodes < 1 || n_nodes > SUREL_MAX_NODES || n_queries < 0) return SUREL_E_RANGE;
    if (k < 1 || k > SUREL_MAX_TUPLE || n_queries > (int64_t)0x7FFFFFFF / k) return SUREL_E_RANGE;
    if (!d_inc_off || (n_queries > 0 && (!d_queries || !d_inc_q))) return SUREL_E_NULL;
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (int rc = grow_buffer(ctx, &ctx->d_batch, &ctx->batch_bytes,
                             surel::incidence_scratch_bytes(n_queries * k)))
        return rc;
    KernelSpan span(ctx, SUREL_K_BATCH);
    if (surel::launch_query_incidence(ctx->stream, d_queries, n_queries, k, n_nodes, d_inc_off,
                                      d_inc_q, ctx->d_batch, ctx->d_err) != hipSuccess)
        return SUREL_E_HIP;
    return SUREL_OK;
}

int surel_bfs_batches(surel_ctx* ctx, const int32_t* d_queries, int64_t n_queries, int32_t k,
                      int32_t n_nodes, const int64_t* d_inc_off, const int32_t* d_inc_q,
                      const int32_t* d_start, int64_t n_batches, int32_t n_start, int32_t B1,
                      int32_t B2, int32_t* d_vbar, int32_t* d_batch, int32_t* d_tuples,
                      int32_t* d_counts) {
    if (n_nodes < 1 || n_nodes > SUREL_MAX_NODES || n_queries < 0 || n_batches < 0) return SUREL_E_RANGE;
    if (k < 1 || k > SUREL_MAX_TUPLE || n_queries > (int64_t)0x7FFFFFFF / k) return SUREL_E_RANGE;
    if (n_start < 1 || n_start > SUREL_MAX_BATCH || B1 < 1 || B1 > SUREL_MAX_BATCH || B2 < 1 ||
        B2 > SUREL_MAX_BATCH)
        return SUREL_E_RANGE;
    if (n_batches > 0 && (!d_inc_off || !d_start || !d_vbar || !d_batch || !d_counts)) return SUREL_E_NULL;
    if (n_batches > 0 && n_queries > 0 && (!d_queries || !d_inc_q)) return SUREL_E_NULL;
    if (!ctx) return SUREL_E_CTX;
    if (n_batches == 0) return SUREL_OK;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (int rc = grow_buffer(ctx, &ctx->d_batch, &ctx->batch_bytes,
                             surel::bfs_scratch_bytes(ctx->n_cu, n_batches, n_start, B1, B2)))
        return rc;
    KernelSpan span(ctx, SUREL_K_BATCH);
    if (surel::launch_bfs_batches(ctx->stream, ctx->n_cu, d_queries, n_queries, k, n_nodes, d_inc_off,
                                  d_inc_q, d_start, n_batches, n_start, B1, B2, d_vbar, d_batch,
                                  d_tuples, d_counts, ctx->d_batch, ctx->d_err) != hipSuccess)
        return SUREL_E_HIP;
    return SUREL_OK;
}

int surel_set_spin_limit(surel_ctx* ctx, uint32_t spins) {
    if (!ctx) return SUREL_E_CTX;
    ctx->spin_limit = spins;
    return SUREL_OK;
}

int surel_profile_enable(surel_ctx* ctx, int on) {
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (int rc = drain_spans(ctx)) return rc;
    if (on) {
        for (int i = 0; i < SUREL_K_COUNT; ++i) {
            ctx->prof_ms[i] = 0.0;
            ctx->prof_launches[i] = 0;
        }
    }
    ctx->profiling = on != 0;
    return SUREL_OK;
}

int surel_profile_read(surel_ctx* ctx, int kernel, double* h_total_ms, int64_t* h_launches) {
    if (!ctx) return SUREL_E_CTX;
    if (kernel < 0 || kernel >= SUREL_K_COUNT) return SUREL_E_RANGE;
    if (!h_total_ms || !h_launches) return SUREL_E_NULL;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    if (int rc = drain_spans(ctx)) return rc;
    *h_total_ms = ctx->prof_ms[kernel];
    *h_launches = ctx->prof_launches[kernel];
    return SUREL_OK;
}

int surel_check(surel_ctx* ctx, uint32_t* h_flags) {
    if (!ctx) return SUREL_E_CTX;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return SUREL_E_HIP;
    uint32_t* h_word = reinterpret_cast<uint32_t*>(ctx->h_pinned + 1);
    if (hipMemcpyAsync(h_word, ctx->d_err, sizeof(uint32_t), hipMemcpyDeviceToHost,
                       ctx->stream) != hipSuccess)
        return SUREL_E_HIP;
    if (hipMemsetAsync(ctx->d_err, 0, sizeof(uint32_t), ctx->stream) != hipSuccess)
        return SUREL_E_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return SUREL_E_HIP;
    if (h_flags) *h_flags = *h_word;
    return *h_word == 0 ? SUREL_OK : SUREL_E_DEVICE;
}

}  // extern "C"
