/*
 * libsurel: the walk -> RPE -> join hot path of SUREL on one AMD MI355X (gfx950).
 *
 * Three operations, named after the paper's statement of the problem:
 *   surel_sample_walks   M random walks of m steps from every seed node
 *                        (Sec. 3.2 "Walk Sampling"; Algorithm 1, walk step);
 *   surel_build_rpe      per seed u, the set V_u of distinct visited nodes and, for each
 *                        x in V_u, the landing counts X_{u,x}[0..m]
 *                        (Sec. 3.2 "Relative Positional Encoding"; Algorithm 1, RPE step);
 *   surel_join_queries   per query tuple Q, the union of the V_u, u in Q, and for each
 *                        node x of it the query-level RPE X_{Q,x} = [X_{u,x}]_{u in Q},
 *                        zeros where x is not in V_u (Sec. 3.4, set-union form).
 * Beside them: surel_sample_walks_rpe (the first two in one kernel; surel_sample_walks_rpe_ids:
 * with the pruning of Sec. 3.3 as well, so that table rows carry RPE-IDs), surel_query_rpe_ids
 * (Sec. 3.4's per-walk-position form of the join: RPE-IDs instead of RPE values),
 * surel_prune_rpe (Sec. 3.3: the distinct count vectors stored once, rows re-indexed),
 * surel_join_query_ids (the union join over those RPE-IDs), and
 * surel_query_incidence + surel_bfs_batches (Sec. 3.6 "Mini-batching for Training";
 * Algorithm 2: mini-batches of queries that share nodes, by breadth-first search).
 *
 * Conventions
 *   - Plain C ABI.  Pointers named d_* are DEVICE memory owned by the caller, on the
 *     device the context was created for; pointers named h_* are HOST memory.  The library
 *     never frees or keeps a caller pointer beyond the call's work on the stream.
 *   - All work is enqueued on the context's stream.  A call returns without waiting unless
 *     a non-NULL h_rows is passed (then it waits for its own work and reports the row
 *     total).  Calls on one context must not overlap from several host threads.
 *   - The context owns grow-only device workspaces (per-seed / per-query row counts, scan
 *     partials, the walk's per-edge neighbour records, the fused kernel's look-back words,
 *     the hash tables and sort arrays of pruning and mini-batching)
 *     and a device error word; nothing else is allocated.
 *   - Stream capture: a call that is given no h_* pointer only enqueues kernels (no memset,
 *     no copy, no wait), so once an eager call of the same shape has grown the workspaces it
 *     can be captured into a HIP graph and replayed.  surel_prune_rpe, surel_check and the
 *     profile calls wait for the stream and cannot be captured.
 *   - Return value: SUREL_OK (0) or a negative SUREL_E_* code.  Arguments are validated on
 *     the host before anything is enqueued, so a call that returns SUREL_E_NULL or
 *     SUREL_E_RANGE has launched nothing.  Problems only visible on the device (a seed or
 *     query index out of range, a malformed CSR row, a node set larger than max_set, an
 *     output that does not fit cap_rows) never fault: the offending item is skipped or
 *     clamped, a bit is set in the sticky error word, and surel_check reports it.
 *   - No function throws, prints, or touches errno.
 *
 *   - The uint16 count arrays (d_rpe_cnt, d_join_cnt) must start on a 4-byte boundary
 *     (SUREL_E_RANGE otherwise): they are moved as 32-bit words wherever possible.  The join
 *     READS d_rpe_cnt (and d_code) as the aligned 32-bit words that cover a vector, so the word
 *     that holds the table's last count is read whole: when rows * (m+1) is odd that is 2 bytes
 *     past the last count (never past that word).  Any buffer whose size is a multiple of 4
 *     bytes, which includes every allocation of hipMalloc or torch, satisfies this; the extra
 *     half word is discarded.
 *   - Sizing.  The variable-size outputs (RPE table, join) come in three forms each: a
 *     counting call (surel_build_rpe_count, surel_join_count: offsets and total only), a filling
 *     call that trusts the caller's offsets and launches nothing else (surel_build_rpe_fill,
 *     surel_join_fill), and a call that does both into buffers of cap_rows rows
 *     (surel_build_rpe, surel_join_queries; with NULL outputs they are counting calls too).
 *
 * Layouts (row-major, densely packed, no padding)
 *   CSR      d_row_ptr int32[n_nodes+1], d_col_idx int32[n_edges]; entries of a row are the
 *            neighbours of that node.  The walk treats every entry of a row as equally
 *            likely, so a simple graph gives the uniform walk over distinct neighbours.
 *   walks    int32[n_seeds][M][m+1]; walks[i][w][0] = seeds[i].
 *   RPE      d_rpe_off int64[n_seeds+1] (d_rpe_off[0] = 0); rows d_rpe_off[i] ..
 *            d_rpe_off[i+1]-1 belong to seed i; d_rpe_ids int32[rows] ascending inside a
 *            seed's block; d_rpe_cnt uint16[rows][m+1].
 *   queries  int32[n_queries][k]; an entry selects a seed's block of the RPE table (it is
 *            the node id when seeds = 0..n_nodes-1).
 *   join     d_join_off int64[n_queries+1]; d_join_ids int32[rows] ascending inside a
 *            query's block; d_join_cnt uint16[rows][k][m+1], halves in tuple order.
 */
#ifndef SUREL_H
#define SUREL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define SUREL_OK            0
#define SUREL_E_NULL       (-1)  /* a required pointer is NULL                              */
#define SUREL_E_RANGE      (-2)  /* a size or parameter is outside the documented limits    */
#define SUREL_E_HIP        (-3)  /* a HIP runtime call failed                               */
#define SUREL_E_CAPACITY   (-4)  /* the output needs more rows than cap_rows (see h_rows)   */
#define SUREL_E_CTX        (-5)  /* the context pointer is NULL                             */
#define SUREL_E_DEVICE     (-6)  /* the device error word is non-zero (surel_check)         */

/* bits of the device error word */
#define SUREL_DEV_BAD_SEED      0x01u  /* a seed is not in [0, n_nodes)                     */
#define SUREL_DEV_BAD_GRAPH     0x02u  /* a visited CSR row is malformed or names a bad node */
#define SUREL_DEV_BAD_WALK      0x04u  /* a walk entry is not in [0, n_nodes)               */
#define SUREL_DEV_BAD_QUERY     0x08u  /* a query entry is not in [0, n_blocks)             */
#define SUREL_DEV_SET_TOO_LARGE 0x10u  /* a block of the RPE table has more than max_set rows */
#define SUREL_DEV_CAPACITY      0x20u  /* rows beyond cap_rows were not written             */
#define SUREL_DEV_BAD_TABLE     0x40u  /* d_rpe_off is not non-decreasing at a queried block */
#define SUREL_DEV_BAD_SIZES     0x80u  /* a seed's d_set_sizes entry (or the offsets given to a
                                          filling call) do not match its number of rows; that
                                          seed's / query's rows are not written              */
#define SUREL_DEV_STALL         0x100u /* a bounded wait inside surel_sample_walks_rpe ran out
                                          (see surel_set_spin_limit), or a bounded probe of a
                                          hash table of surel_bfs_batches; outputs are
                                          incomplete                                         */

/* limits */
#define SUREL_MAX_NODES   268435455   /* 2^28 - 1: node id and step share one 32-bit sort key */
#define SUREL_MAX_STEPS   15          /* m                                                   */
#define SUREL_MAX_WALKS   65535       /* M: counts are uint16                                */
#define SUREL_MAX_WALK_ENTRIES 2048   /* build_rpe: M*(m+1) keys are sorted in one wavefront */
#define SUREL_MAX_SET     2048        /* join: rows per block of the RPE table               */
#define SUREL_MAX_TUPLE   3           /* join: k                                             */
#define SUREL_MAX_DISTINCT 16777216   /* prune: cap_T (2^24 distinct count vectors)          */
#define SUREL_MAX_BATCH   1048576     /* mini-batching: B1, B2 and the seed-set size (2^20)   */
#define SUREL_NOALLOC_MAX_QUERIES 1048576  /* surel_join_queries_noalloc: n_queries (2^20)    */

/* kernel groups for surel_profile_read */
#define SUREL_K_WALK        0   /* walk kernel                                        */
#define SUREL_K_RPE_COUNT   1   /* RPE builder: set-size kernel (when sizes not given) */
#define SUREL_K_RPE_FILL    2   /* RPE builder: sort-and-write kernel                 */
#define SUREL_K_JOIN_COUNT  3   /* join: counting launch                              */
#define SUREL_K_JOIN_FILL   4   /* join: writing launch                               */
#define SUREL_K_SCAN        5   /* the offset scans (three small launches each)       */
#define SUREL_K_WALK_RPE    6   /* fused walk + RPE kernel (surel_sample_walks_rpe)   */
#define SUREL_K_EDGE_RECORDS 7  /* expansion of the CSR into per-edge neighbour records
                                   (both walk calls, large jobs only)                 */
#define SUREL_K_QUERY_IDS   8   /* surel_query_rpe_ids                                */
#define SUREL_K_PRUNE       9   /* surel_prune_rpe (all its launches)                 */
#define SUREL_K_BATCH       10  /* surel_query_incidence and surel_bfs_batches        */
#define SUREL_K_COUNT       11

typedef struct surel_ctx surel_ctx;

/* Create a context for `device` whose work runs on `hip_stream` (a hipStream_t passed as
 * void*; NULL = the device's default stream).  The stream is borrowed, not owned.
 * Errors: SUREL_E_NULL (out), SUREL_E_HIP (no such device, allocation failure). */
int surel_create(surel_ctx** out, int device, void* hip_stream);

/* Wait for the context's stream, then free the workspace and the context.  NULL is ignored. */
void surel_destroy(surel_ctx* ctx);

/* A static, human-readable string for a status code. */
const char* surel_strerror(int status);

/* Largest possible row total of surel_build_rpe for walks made by surel_sample_walks:
 * n_seeds * (1 + M*m) (App. D.4: at most m*M distinct nodes besides the seed).  Hand-made
 * walks whose position 0 differs inside one seed can exceed it (up to M*(m+1) per seed);
 * cap_rows handling covers that.  Non-positive arguments give 0. */
int64_t surel_rpe_rows_bound(int64_t n_seeds, int32_t M, int32_t m);

/* Sec. 3.2 "Walk Sampling" / Algorithm 1: for every seed i and walk w < M, walk m steps from
 * u = d_seeds[i].  Step s (1..m) from node c with degree deg = row_ptr[c+1]-row_ptr[c] goes
 * to col_idx[row_ptr[c] + r mod deg], where r is word (s-1)&3 of Philox-4x32-10 with counter
 * (u, w, (s-1)>>2, 0) and key (rng_seed & 0xffffffff, rng_seed >> 32); a node of degree 0
 * keeps the walker in place.  The result depends on (rng_seed, u, w, s) only.
 *   d_row_ptr, d_col_idx  CSR (device, read-only); n_edges = number of col_idx entries.
 *   d_seeds               int32[n_seeds] (device, read-only).
 *   d_walks               int32[n_seeds][M][m+1] (device, written).
 *   d_set_sizes           int32[n_seeds] (device, written) or NULL: |V_u| of every seed, the
 *                         number of distinct nodes in its walks (Algorithm 1: V_u = set(W_u)).
 *                         Passing it on to surel_build_rpe saves that call a pass over the
 *                         walks.  Needs M*(m+1) <= SUREL_MAX_WALK_ENTRIES.
 * Limits: 1 <= n_nodes <= SUREL_MAX_NODES, 0 <= n_edges < 2^31, n_seeds >= 0,
 * 1 <= M <= SUREL_MAX_WALKS, 1 <= m <= SUREL_MAX_STEPS.  n_seeds = 0 is a no-op.
 * Device-detected: BAD_SEED (that seed's walks are filled with -1, its set size is 0),
 * BAD_GRAPH (the walker stays in place for that step). */
int surel_sample_walks(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                       int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds,
                       int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,
                       int32_t* d_walks, int32_t* d_set_sizes);

/* Sec. 3.2 "Relative Positional Encoding" / Algorithm 1: for every seed i, V_i = distinct
 * node ids in walks[i] (ascending) and cnt[x][s] = #{w : walks[i][w][s] == x}.
 *   d_walks      int32[n_seeds][M][m+1] (device, read-only), entries in [0, n_nodes).
 *   d_set_sizes  int32[n_seeds] (device, read-only) or NULL: |V_i| as surel_sample_walks
 *                reports it for these walks.  NULL makes the call count them itself.
 *   cap_rows     rows that d_rpe_ids / d_rpe_cnt can hold.
 *   d_rpe_off    int64[n_seeds+1] (device, written; always complete, even on overflow).
 *   d_rpe_ids    int32[cap_rows], d_rpe_cnt uint16[cap_rows][m+1] (device, written).  Both
 *                may be NULL together: then only d_rpe_off and the total are produced
 *                (use it to size the outputs exactly; surel_rpe_rows_bound avoids it).
 *   h_rows       host int64, may be NULL.  If given, the call waits and stores the row total
 *                (the number needed, also when it exceeds cap_rows).
 * Limits: as for surel_sample_walks, and M*(m+1) <= SUREL_MAX_WALK_ENTRIES.
 * Returns SUREL_E_CAPACITY if h_rows is given and the total exceeds cap_rows; rows at or
 * beyond cap_rows are never written (blocks that do not fit entirely are skipped).
 * Device-detected: BAD_WALK (an entry outside [0, n_nodes) is left out of the counts, so the
 * block of a seed that surel_sample_walks rejected, all -1, yields no rows), CAPACITY,
 * BAD_SIZES. */
int surel_build_rpe(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M,
                    int32_t m, int32_t n_nodes, const int32_t* d_set_sizes, int64_t cap_rows,
                    int64_t* d_rpe_off, int32_t* d_rpe_ids, uint16_t* d_rpe_cnt,
                    int64_t* h_rows);

/* The two phases of surel_build_rpe as calls of their own (Algorithm 1's RPE step has a
 * data-dependent output size: V_u = set(W_u)).
 * surel_build_rpe_count: the layout only.  Writes d_rpe_off[0 .. n_seeds] and, if h_rows is
 * given, waits and stores the row total.  d_set_sizes as above (NULL: counted here).
 * surel_build_rpe_fill: the rows only.  d_rpe_off (device, READ-only) must hold the offsets of
 * these walks, from surel_build_rpe_count or kept from an earlier call; nothing is counted or
 * scanned again, one kernel is launched and nothing is waited for.  A seed whose walks do not
 * have d_rpe_off[i+1] - d_rpe_off[i] distinct nodes is skipped and flagged (BAD_SIZES), as is
 * a block that would pass cap_rows (CAPACITY).
 * Arguments, limits and the other device-detected problems as for surel_build_rpe. */
int surel_build_rpe_count(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M,
                          int32_t m, int32_t n_nodes, const int32_t* d_set_sizes,
                          int64_t* d_rpe_off, int64_t* h_rows);
int surel_build_rpe_fill(surel_ctx* ctx, const int32_t* d_walks, int64_t n_seeds, int32_t M,
                         int32_t m, int32_t n_nodes, const int64_t* d_rpe_off, int64_t cap_rows,
                         int32_t* d_rpe_ids, uint16_t* d_rpe_cnt);

/* Sec. 3.2: "the RPE is computed on the fly as walks get sampled" (Algorithm 1, walk and RPE
 * steps in one pass).  Exactly the results of surel_sample_walks followed by surel_build_rpe
 * on its walks, from one kernel that never reads the walks back: d_walks as in
 * surel_sample_walks; cap_rows, d_rpe_off, d_rpe_ids, d_rpe_cnt, h_rows as in surel_build_rpe
 * (ids / cnt may be NULL together: offsets and total only; the walks are written either way).
 * Limits: those of both calls (M*(m+1) <= SUREL_MAX_WALK_ENTRIES).  n_seeds = 0 writes
 * d_rpe_off[0] = 0.
 * Device-detected: BAD_SEED (that seed's walks are filled with -1 and it gets no rows),
 * BAD_GRAPH (the walker stays in place for that step), CAPACITY, STALL (the offsets are then
 * incomplete; a call that was given h_rows returns SUREL_E_DEVICE instead of a total). */
int surel_sample_walks_rpe(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                           int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds,
                           int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,
                           int32_t* d_walks, int64_t cap_rows, int64_t* d_rpe_off,
                           int32_t* d_rpe_ids, uint16_t* d_rpe_cnt, int64_t* h_rows);

/* Algorithm 1 from end to end in one call: walks, RPE and the pruning of the central array
 * (Sec. 3.2 "computed on the fly as walks get sampled"; Sec. 3.3 "the table carries RPE-IDs";
 * Algorithm 1's last step).  The fused kernel of surel_sample_walks_rpe also looks every
 * finished row's count vector up in the set of distinct vectors while the row is still on
 * chip, so the table never has to be read back to prune it.  Results: exactly those of
 * surel_sample_walks_rpe followed by surel_prune_rpe on its d_rpe_cnt.
 *   d_walks, cap_rows, d_rpe_off, d_rpe_ids   as in surel_sample_walks_rpe (ids required unless
 *                cap_rows is 0).
 *   d_rpe_cnt    uint16[cap_rows][m+1] (device, written), or NULL: the table then carries
 *                RPE-IDs only (4 bytes a row instead of 2(m+1)), the count vectors live in d_T.
 *   d_code       int32[cap_rows] (device, written): d_T[d_code[r]] is row r's count vector.
 *   cap_T, d_T   as in surel_prune_rpe: uint16[cap_T][m+1], the distinct vectors, sorted.
 *   h_rows, h_n_T   host int64, both required: table rows and distinct vectors.  The call always
 *                waits for its own work.
 * Returns SUREL_E_CAPACITY when the table needs more than cap_rows rows or has more than cap_T
 * distinct vectors (*h_rows / *h_n_T say how many; d_T and d_code are then undefined),
 * SUREL_E_DEVICE when a bounded wait ran out.  Limits and device-detected problems: those of
 * surel_sample_walks_rpe and surel_prune_rpe. */
int surel_sample_walks_rpe_ids(surel_ctx* ctx, const int32_t* d_row_ptr, const int32_t* d_col_idx,
                               int32_t n_nodes, int64_t n_edges, const int32_t* d_seeds,
                               int64_t n_seeds, int32_t M, int32_t m, uint64_t rng_seed,
                               int32_t* d_walks, int64_t cap_rows, int64_t* d_rpe_off,
                               int32_t* d_rpe_ids, uint16_t* d_rpe_cnt, int32_t* d_code,
                               int64_t cap_T, uint16_t* d_T, int64_t* h_rows, int64_t* h_n_T);

/* Sec. 3.4, set-union form: for every query q with tuple (b_1..b_k) of table blocks, the
 * ascending union of the blocks' id lists and, per union node x and j < k, block b_j's count
 * vector for x, or m+1 zeros when x is not in block b_j.
 *   d_rpe_off / d_rpe_ids / d_rpe_cnt   an RPE table of n_blocks blocks (device, read-only).
 *   max_set      an upper bound on the rows of any queried block (1 + M*m always is one).
 *   d_queries    int32[n_queries][k] (device, read-only), entries in [0, n_blocks).
 *   cap_rows, d_join_off, d_join_ids, d_join_cnt, h_rows   as in surel_build_rpe, with
 *                d_join_cnt uint16[cap_rows][k][m+1]; ids / cnt may be NULL together.
 * Limits: 1 <= m <= SUREL_MAX_STEPS, 2 <= k <= SUREL_MAX_TUPLE, 1 <= max_set <=
 * SUREL_MAX_SET, n_blocks >= 0, n_queries >= 0.
 * Device-detected: BAD_QUERY, BAD_TABLE and SET_TOO_LARGE (that query yields zero rows),
 * CAPACITY (as above). */
int surel_join_queries(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                       const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m,
                       int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                       int32_t k, int64_t cap_rows, int64_t* d_join_off,
                       int32_t* d_join_ids, uint16_t* d_join_cnt, int64_t* h_rows);

/* The two phases of the join as calls of their own (Sec. 3.4: the size of a query's union is
 * data-dependent).
 * surel_join_count: the layout only, from the id lists alone.  Writes d_join_off[0 .. n_queries]
 * and, if h_rows is given, waits and stores the row total.
 * surel_join_fill: the rows only.  d_join_off (device, READ-only) must hold the offsets of these
 * queries over this table, from surel_join_count or kept from an earlier call; nothing is
 * counted or scanned again, one kernel is launched and nothing is waited for.  A query whose
 * union does not have d_join_off[q+1] - d_join_off[q] rows is skipped and flagged (BAD_SIZES),
 * as are rows that would pass cap_rows (CAPACITY).
 * Arguments, limits and the other device-detected problems as for surel_join_queries. */
int surel_join_count(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                     int64_t n_blocks, int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                     int32_t k, int64_t* d_join_off, int64_t* h_rows);
int surel_join_fill(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                    const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
                    const int32_t* d_queries, int64_t n_queries, int32_t k,
                    const int64_t* d_join_off, int64_t cap_rows, int32_t* d_join_ids,
                    uint16_t* d_join_cnt);

/* surel_join_queries for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * byte for byte, but the call never allocates or frees anything (no hipMalloc, no hipFree, no
 * event creation: its launches are not timed by surel_profile_enable): its device scratch (one
 * int32 per query and the partial sums of their scan) is a static array inside the library, 4 MiB
 * + 8 KiB that every device the library runs on holds until the process ends, instead of the
 * context's grow-only workspace.  Hence n_queries <= SUREL_NOALLOC_MAX_QUERIES (SUREL_E_RANGE
 * beyond).  All calls on one device share that array, whichever context they use: calls that
 * overlap on one device (two streams, two host threads) race on it and give wrong rows; calls
 * one after the other on the same stream are safe, and nothing in the array needs clearing
 * between them (every word a call reads it has written itself). */
int surel_join_queries_noalloc(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                               const uint16_t* d_rpe_cnt, int64_t n_blocks, int32_t m,
                               int32_t max_set, const int32_t* d_queries, int64_t n_queries,
                               int32_t k, int64_t cap_rows, int64_t* d_join_off,
                               int32_t* d_join_ids, uint16_t* d_join_cnt, int64_t* h_rows);

/* surel_join_queries with RPE-IDs instead of RPE values (Sec. 3.3: "the table carries RPE-IDs";
 * Sec. 3.4's closing remarks on shipping IDs instead of values): the same union rows, and for
 * every row and tuple member the code of the member's table row for that node, i.e. its index
 * in the pruned array T of surel_prune_rpe, or -1 where the member's set does not hold the
 * node (the all-zero vector).  12 bytes a row for pairs instead of 24 at m = 4.
 *   d_code       int32[table rows] (device, read-only): the codes surel_prune_rpe wrote.
 *   d_join_codes int32[cap_rows][k] (device, written; may be NULL together with d_join_ids).
 *   everything else as in surel_join_queries (whose row layout and d_join_off this call
 *   reproduces exactly).  Device-detected: as surel_join_queries. */
int surel_join_query_ids(surel_ctx* ctx, const int64_t* d_rpe_off, const int32_t* d_rpe_ids,
                         const int32_t* d_code, int64_t n_blocks, int32_t max_set,
                         const int32_t* d_queries, int64_t n_queries, int32_t k, int64_t cap_rows,
                         int64_t* d_join_off, int32_t* d_join_ids, int32_t* d_join_codes,
                         int64_t* h_rows);

/* Sec. 3.4, the per-walk-position form: the walks of a query's blocks are concatenated, and
 * every node occurrence x in them gets its query-level RPE-ID, the tuple of the RPE table's row
 * indices of x in each of the query's k blocks (the table is the unpruned central array of
 * Sec. 3.3; -1 = the block does not hold x, i.e. the all-zero vector).
 *   d_walks      int32[n_blocks][M][m+1] (device, read-only): d_walks[b] is the walk block whose
 *                RPE rows are table block b (true for the outputs of surel_sample_walks /
 *                surel_build_rpe / surel_sample_walks_rpe over one seed list).
 *   d_rpe_off, d_rpe_ids   the RPE table (device, read-only); table_rows = its number of rows
 *                (d_rpe_off[n_blocks]), at most 2^31 - 1 so that a row index fits int32.
 *   d_code       NULL, or int32[table_rows] (device, read-only), the rows' codes from
 *                surel_prune_rpe: the outputs are then d_code[row] instead of row, i.e. the
 *                RPE-IDs of Sec. 3.3 after pruning, indices into the pruned array T (what the
 *                paper ships to the GPU, where X = T[RPE-ID] is one indexing step).
 *   max_set, d_queries, n_queries, k   as in surel_join_queries.
 *   d_out        int32[n_queries][k][M][m+1][k] (device, written):
 *                d_out[q][j][w][s][j2] = row (or code of the row) of node
 *                d_walks[queries[q][j]][w][s] in block queries[q][j2], or -1.
 * Limits: 1 <= M <= SUREL_MAX_WALKS, 1 <= m <= SUREL_MAX_STEPS, M*(m+1) < 2^31 / 9,
 * 2 <= k <= SUREL_MAX_TUPLE, 1 <= max_set <= SUREL_MAX_SET, 0 <= table_rows < 2^31.
 * Device-detected: BAD_QUERY, BAD_TABLE, SET_TOO_LARGE (that query's entries are all -1). */
int surel_query_rpe_ids(surel_ctx* ctx, const int32_t* d_walks, const int64_t* d_rpe_off,
                        const int32_t* d_rpe_ids, const int32_t* d_code, int64_t n_blocks,
                        int64_t table_rows, int32_t M, int32_t m, int32_t max_set,
                        const int32_t* d_queries, int64_t n_queries, int32_t k, int32_t* d_out);

/* Sec. 3.3, last paragraph / Algorithm 1, last step ("prune T"): the count vectors of the RPE
 * table repeat a lot, so they are stored once.  d_T receives the distinct vectors, sorted
 * (vectors compared entry by entry; the paper leaves the order open, sorted makes it unique),
 * and d_code[r] the index in d_T of row r's vector: d_T[d_code[r]] == d_rpe_cnt[r].  A row of
 * surel_query_rpe_ids' output, sent through d_code, is the paper's re-indexed RPE-ID.
 *   d_rpe_cnt    uint16[n_rows][m+1] (device, read-only).
 *   cap_T        vectors that d_T can hold, 1 .. SUREL_MAX_DISTINCT.
 *   d_T          uint16[cap_T][m+1], d_code int32[n_rows] (device, written).
 *   h_n_T        host int64, required: the number of distinct vectors.  The call always waits
 *                for its own work (the sort is sized by that number).
 * The context's workspace grows by 292 bytes per unit of cap_T (rounded up to a power of two).
 * Returns SUREL_E_CAPACITY when there are more than cap_T distinct vectors (*h_n_T says how
 * many; d_T and d_code are then undefined).  Limits: 1 <= m <= SUREL_MAX_STEPS, n_rows >= 0.
 * Device-detected: STALL. */
int surel_prune_rpe(surel_ctx* ctx, const uint16_t* d_rpe_cnt, int64_t n_rows, int32_t m,
                    int64_t cap_T, uint16_t* d_T, int32_t* d_code, int64_t* h_n_T);

/* The queries of every node, the adjacency that the mini-batch search of Sec. 3.6 runs on
 * ("a neighbor of node u is a node that shares at least one query with it"): for every node x,
 * the indices of the queries that name x, ascending.  Built once per query list.
 *   d_queries    int32[n_queries][k] NODE ids (device, read-only), 1 <= k <= SUREL_MAX_TUPLE,
 *                n_queries * k < 2^31.
 *   d_inc_off    int64[n_nodes + 1] (device, written): node x's part of d_inc_q is
 *                [d_inc_off[x], d_inc_off[x+1]).
 *   d_inc_q      int32[n_queries * k] (device, written); a query that names x twice is listed
 *                twice in x's part.
 * Asynchronous.  Device-detected: BAD_QUERY (an id outside [0, n_nodes); that entry is left out
 * of every part, d_inc_off[n_nodes] is the number of entries kept). */
int surel_query_incidence(surel_ctx* ctx, const int32_t* d_queries, int64_t n_queries, int32_t k,
                          int32_t n_nodes, int64_t* d_inc_off, int32_t* d_inc_q);

/* Mini-batches for training (Sec. 3.6 "Mini-batching for Training"; Algorithm 2, the steps
 * that choose a seed-set and expand it by breadth-first search): n_batches independent
 * searches in one launch.  Search b starts from the nodes d_start[b][0..n_start) (the random
 * seed-set is the caller's draw; repeated nodes count once) and collects the node set V̄ and
 * the reached queries until V̄ has B1 nodes or the batch has B2 queries.  Where the paper leaves
 * the order open: the queue is first-in first-out, a node's queries are taken in ascending
 * index, a query's nodes in tuple order; a query enters the batch together with all of its
 * nodes, and the search ends at the first query whose new nodes no longer fit into B1.
 *   d_queries, n_queries, k, n_nodes   the query list, as for surel_query_incidence.
 *   d_inc_off, d_inc_q   what surel_query_incidence wrote for this query list (read-only).
 *   d_start      int32[n_batches][n_start] (device, read-only).
 *   d_vbar       int32[n_batches][B1] (device, written): V̄ of every batch in the order reached
 *                (start nodes first); entries past the batch's node count are not written.
 *   d_batch      int32[n_batches][B2] (device, written): the indices of the reached queries in
 *                the order reached; entries past the batch's query count are not written.
 *   d_tuples     int32[n_batches][B2][k] or NULL (device, written): the same queries as node
 *                tuples, ready to be a query list of the join calls when node x's RPE block is
 *                block x.
 *   d_counts     int32[n_batches][2] (device, written): (nodes in V̄, queries in the batch).
 * Limits: 1 <= n_start, B1, B2 <= SUREL_MAX_BATCH.  The context's workspace grows by 16 bytes
 * times (B1 + B2 + n_start + 4 c), c = 4 B2 rounded up to a power of two within [64, 1024],
 * both tables rounded up to powers of two, for each search in flight (4 per compute unit, 16
 * where B2 <= 64; fewer where that would pass 4 GiB).  Asynchronous.
 * Device-detected: BAD_QUERY (a start node or query entry outside [0, n_nodes): skipped),
 * BAD_TABLE (d_inc_off / d_inc_q are not lists of this query list: those entries are skipped). */
int surel_bfs_batches(surel_ctx* ctx, const int32_t* d_queries, int64_t n_queries, int32_t k,
                      int32_t n_nodes, const int64_t* d_inc_off, const int32_t* d_inc_q,
                      const int32_t* d_start, int64_t n_batches, int32_t n_start, int32_t B1,
                      int32_t B2, int32_t* d_vbar, int32_t* d_batch, int32_t* d_tuples,
                      int32_t* d_counts);

/* Every wait inside the fused kernel of surel_sample_walks_rpe (a wave waiting for an offset,
 * the offset scan waiting for a row count) and inside surel_prune_rpe (a lane waiting for
 * another to finish writing a hash slot) gives up after `spins` polls, raises
 * SUREL_DEV_STALL and lets the kernel end.  The default (2^22 polls, seconds) is never reached
 * by a healthy run; tests set 0 to see the bounded exit.  Errors: SUREL_E_CTX. */
int surel_set_spin_limit(surel_ctx* ctx, uint32_t spins);

/* Per-kernel timing for benchmarks.  While enabled, every kernel group the context launches
 * is bracketed by two HIP events on the context's stream (a few microseconds of host work
 * per launch).  surel_profile_enable(ctx, 1) clears the totals and starts collecting,
 * (ctx, 0) stops; both wait for the stream.  surel_profile_read waits for the stream and
 * returns, for one SUREL_K_* group, the summed device time in milliseconds and the number of
 * bracketed launches since collecting started.
 * Errors: SUREL_E_CTX, SUREL_E_RANGE (kernel), SUREL_E_NULL (h_total_ms, h_launches),
 * SUREL_E_HIP. */
int surel_profile_enable(surel_ctx* ctx, int on);
int surel_profile_read(surel_ctx* ctx, int kernel, double* h_total_ms, int64_t* h_launches);

/* Wait for the context's stream and read the device error word.  *h_flags (may be NULL)
 * receives the SUREL_DEV_* bits; the word is then cleared.  Returns SUREL_OK if it was
 * zero, SUREL_E_DEVICE otherwise, SUREL_E_HIP if the stream reported a failure. */
int surel_check(surel_ctx* ctx, uint32_t* h_flags);

#ifdef __cplusplus
}
#endif
#endif /* SUREL_H */
