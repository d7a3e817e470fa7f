// Host-side launch wrappers of the HIP kernels (internal to libsurel).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace surel {

// walk.hip.  The per-edge neighbour records that launch_edge_records makes of a CSR (layouts in
// walk_core.h; worth making when walks_want_records says so): edge_record_plan picks the layout
// for a graph, the caller provides edge_record_bytes(plan, n_edges) bytes in plan.data.
struct EdgeRecords {
    const void* data = nullptr;  // null: no records, the walk reads the CSR
    int format = 0;
    int id_bits = 0, lo_bits = 0;  // field widths of the packed layout
};
bool walks_want_records(int64_t n_edges, int64_t n_seeds, int32_t M, int32_t m);
EdgeRecords edge_record_plan(int32_t n_nodes, int64_t n_edges);
size_t edge_record_bytes(const EdgeRecords& plan, int64_t n_edges);
hipError_t launch_edge_records(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                               int32_t n_nodes, int64_t n_edges, const EdgeRecords& rec);

// set_sizes (optional): int32[n_seeds], receives the number of distinct nodes of every seed's
// walks; needs 1 + M*m <= 2048.
hipError_t launch_walks(hipStream_t stream, const int32_t* row_ptr, const int32_t* col_idx,
                        int32_t n_nodes, int64_t n_edges, const int32_t* seeds, int64_t n_seeds,
                        int32_t M, int32_t m, uint64_t rng_seed, int32_t* walks,
                        int32_t* set_sizes, const EdgeRecords& rec, uint32_t* err);

// walk_rpe.hip.  Walks and the RPE table in one persistent kernel: writes walks,
// rpe_off[0..n_seeds] and (unless ids is null) the rows.  lb: device scratch of
// lookback_words(n_seeds) 64-bit words (cleared by the launch itself).  n_cu: compute
// units of the device.  spin_limit bounds every wait inside the kernel (kDevStall when one runs
// out; rpe_off[n_seeds] is then -1).  Needs M*(m+1) <= 2048 and n_seeds >= 1.
// hipErrorInvalidValue = the shape does not fit the device's LDS.
// With `code` (int32 per table row) the kernel also looks every finished row's count vector up
// in the hash set of prune.hip (slots of prune_slot_bytes(cap_T) bytes, emptied by
// launch_prune_clear; counters as for launch_prune_collect) and writes the row's slot number to
// code[row]; launch_prune_finish then turns slot numbers into indices of the sorted array T.
// cnt may then be null (rows carry RPE-IDs only).
hipError_t launch_walk_rpe(hipStream_t stream, int max_lds_bytes, int n_cu, const int32_t* row_ptr,
                           const int32_t* col_idx, int32_t n_nodes, int64_t n_edges,
                           const int32_t* seeds, int64_t n_seeds, int32_t M, int32_t m,
                           uint64_t rng_seed, int32_t* walks, int64_t cap_rows, int64_t* rpe_off,
                           int32_t* ids, uint16_t* cnt, const EdgeRecords& rec, uint64_t* lb,
                           uint32_t spin_limit, uint32_t* err, int32_t* code = nullptr,
                           uint32_t* slots = nullptr, int64_t cap_T = 0,
                           unsigned long long* counters = nullptr);

// rpe.hip.  launch_rpe_count: set_sizes[i] = distinct nodes in walks[i].  launch_rpe_fill:
// writes the rows of every seed at rpe_off[i] (seeds whose block would pass cap_rows, or whose
// row count differs from rpe_off[i+1]-rpe_off[i], are skipped and flagged).
// hipErrorInvalidValue = the shape does not fit the device's LDS.
hipError_t launch_rpe_count(hipStream_t stream, const int32_t* walks, int64_t n_seeds, int32_t M,
                            int32_t m, int32_t n_nodes, int32_t* set_sizes, uint32_t* err);
hipError_t launch_rpe_fill(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                           int64_t n_seeds, int32_t M, int32_t m, int32_t n_nodes,
                           const int64_t* rpe_off, int64_t cap_rows, int32_t* ids, uint16_t* cnt,
                           uint32_t* err);

// join.hip.  launch_join_count: counts[q] = union rows of query q.  launch_join_fill: writes the
// rows of every query at join_off[q] (a query whose union does not have join_off[q+1]-join_off[q]
// rows, or whose rows would pass cap_rows, is skipped and flagged).  absent16: what the entries
// of a vector hold where a list has no row for the node (0 for counts).
// hipErrorInvalidValue = the shape does not fit the device's LDS.
hipError_t launch_join_count(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                             const int32_t* rpe_ids, int64_t n_blocks, int32_t max_set,
                             const int32_t* queries, int64_t n_queries, int32_t k, int32_t* counts,
                             uint32_t* err);
hipError_t launch_join_fill(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                            const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                            int32_t m, int32_t max_set, const int32_t* queries, int64_t n_queries,
                            int32_t k, const int64_t* join_off, int64_t cap_rows, int32_t* out_ids,
                            uint16_t* out_cnt, uint16_t absent16, uint32_t* err);

// query_ids.hip.  out int32[n_queries][k][M][m+1][k]: for every entry of the walk blocks of a
// query's k table blocks, the table rows that hold its node in each of the k blocks (-1 where
// a block does not hold it).  walks[b] must be the walk block of table block b.  code
// (optional): int32[table_rows]; if given, code[row] goes out instead of row.
hipError_t launch_query_ids(hipStream_t stream, int max_lds_bytes, const int32_t* walks,
                            const int64_t* rpe_off, const int32_t* rpe_ids, const int32_t* code,
                            int64_t n_blocks,
                            int32_t M, int32_t m, int32_t max_set, int64_t table_rows,
                            const int32_t* queries, int64_t n_queries, int32_t k, int32_t* out,
                            uint32_t* err);

// prune.hip.  Distinct count vectors of the table, sorted, and every row's index among them.
// slots: prune_slot_bytes(cap_T) bytes, list: prune_list_bytes(cap_T) bytes, counters: two
// 64-bit words (all device scratch).  launch_prune_collect fills the hash set and leaves
// counters[0] = number of distinct vectors; the host reads it and, if it fits cap_T, calls
// launch_prune_finish with it.
size_t prune_slot_bytes(int64_t cap_T);
size_t prune_list_bytes(int64_t cap_T);
uint32_t prune_slot_mask(int64_t cap_T);
// empties the hash set and its counters (memsets: not for stream capture)
hipError_t launch_prune_clear(hipStream_t stream, int64_t cap_T, uint32_t* slots,
                              unsigned long long* counters);
hipError_t launch_prune_collect(hipStream_t stream, int n_cu, const uint16_t* cnt, int64_t n_rows,
                                int32_t m, int64_t cap_T, uint32_t* slots,
                                unsigned long long* counters, int32_t* code, uint32_t spin_limit,
                                uint32_t* err);
hipError_t launch_prune_finish(hipStream_t stream, int n_cu, int64_t n_rows, int32_t m,
                               int64_t cap_T, int64_t n_T, uint32_t* slots,
                               unsigned long long* counters, uint32_t* list, uint16_t* T,
                               int32_t* code);

// incidence.hip.  The queries of every node: inc_q[inc_off[x] .. inc_off[x+1]) = indices of the
// queries that name node x, ascending (a query that names x twice is listed twice).  Entries
// outside [0, n_nodes) are flagged and left out.  scratch: incidence_scratch_bytes(n_queries*k).
size_t incidence_scratch_bytes(int64_t n_entries);
hipError_t launch_query_incidence(hipStream_t stream, const int32_t* queries, int64_t n_queries,
                                  int32_t k, int32_t n_nodes, int64_t* inc_off, int32_t* inc_q,
                                  void* scratch, uint32_t* err);

// bfs.hip.  n_batches mini-batches, each by breadth-first search from its own n_start start
// nodes over nodes that share queries, until B1 nodes or B2 queries.  vbar int32[n_batches][B1],
// batch int32[n_batches][B2], tuples int32[n_batches][B2][k] (optional), counts
// int32[n_batches][2] = (nodes, queries) of every batch.  scratch: bfs_scratch_bytes(...).
size_t bfs_scratch_bytes(int n_cu, int64_t n_batches, int32_t n_start, int32_t B1, int32_t B2);
hipError_t launch_bfs_batches(hipStream_t stream, int n_cu, const int32_t* queries,
                              int64_t n_queries, int32_t k, int32_t n_nodes, const int64_t* inc_off,
                              const int32_t* inc_q, const int32_t* start, int64_t n_batches,
                              int32_t n_start, int32_t B1, int32_t B2, int32_t* vbar, int32_t* batch,
                              int32_t* tuples, int32_t* counts, void* scratch, uint32_t* err);

// scan.hip.  Scratch of the kernels that lay their output out themselves (lookback.h): its
// size in 64-bit words for n_items seeds or queries, and the small kernel that resets it before
// such a launch (counters and counts to zero, group bases to "not yet") and presets *total_out,
// where the scanner will leave the row total, to -1.
int64_t lookback_words(int64_t n_items);
hipError_t launch_lookback_clear(hipStream_t stream, uint64_t* lb, int64_t n_items,
                                 int64_t* total_out);

// scan.hip.  off[0..n] = exclusive prefix sums of counts[0..n-1] (off[n] = total).
// partials: device scratch of scan_partials_len(n) int64.
int64_t scan_partials_len(int64_t n);
hipError_t launch_exclusive_scan(hipStream_t stream, const int32_t* counts, int64_t n,
                                 int64_t* off, int64_t* partials);

}  // namespace surel
