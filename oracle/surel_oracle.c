/*
 * CPU oracle for the walk -> RPE -> join path of SUREL.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, single-threaded C that states what the path computes, so that a
 * reader can check it against the paper by eye.  It shares no code, header,
 * table or helper with the HIP library, and only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  The product never does.
 *
 * What each function follows:
 *   oracle_philox4x32_10   Salmon, Moraes, Dror, Shaw, "Parallel random numbers:
 *                          as easy as 1, 2, 3" (SC'11), Philox-4x32 with 10 rounds.
 *                          The paper names no generator; this build fixes this one.
 *   oracle_sample_walks    Sec. 3.2 "Walk Sampling" and Algorithm 1, step "run M
 *                          times m-step random walks" on the CSR arrays
 *                          (idxptr, indices) of Sec. 3.2.
 *   oracle_build_rpe       Sec. 3.2 "Relative Positional Encoding": V_u is the set
 *                          of distinct nodes in W_u, and X_{u,x}[i] is the landing
 *                          count of x at position i over the walks of W_u.
 *   oracle_join_queries    Sec. 3.4: X_{Q,x} is the concatenation over u in Q of
 *                          X_{u,x}, all zeros where x is not in V_u; taken over the
 *                          union of the V_u (the set-union form the section's
 *                          closing remarks describe).
 *   oracle_query_rpe_ids   Sec. 3.4, the form the section describes first: the walks
 *                          W_u, u in Q, are concatenated, and every node occurrence x
 *                          in them gets RPE-ID_{Q,x} = [RPE-ID_{u,x}]_{u in Q}, found
 *                          through H_u(x).  Here the table of oracle_build_rpe is the
 *                          (unpruned) central array T of Sec. 3.3, so RPE-ID_{u,x} is
 *                          the index of (u, x)'s row in it, and -1 stands for "x is
 *                          not in V_u" (the all-zero vector).
 *   oracle_prune_rpe       Sec. 3.3, last paragraph, and the last step of Algorithm 1: the
 *                          central array T keeps every distinct RPE vector once, and
 *                          every (u, x) keeps the index of its vector in T.  The paper
 *                          leaves the order of T open; here T is sorted (vectors compared
 *                          entry by entry), the canonical choice.
 *   oracle_bfs_batch       Sec. 3.6 "Mini-batching for Training" and the BFS step of
 *                          Algorithm 2: from a seed-set of nodes, breadth-first search
 *                          in which two nodes are neighbours when a query holds both;
 *                          reached queries are collected until the node set has B1
 *                          members or the batch B2.  The paper fixes neither the order
 *                          of the search nor what happens at the limit; here the queue
 *                          is first-in first-out, a node's queries are taken in
 *                          ascending index, a query's nodes in tuple order, and a query
 *                          enters the batch only together with all its nodes (the search
 *                          ends at the first query whose new nodes no longer fit).
 *
 * Readings where the paper is silent:
 *   - a walk is stored with its start: m+1 positions, position 0 is the seed
 *     (the RPE has m+1 slots and Sec. 3.5 writes a walk as (w_0..w_m));
 *   - a step moves to a uniformly chosen entry of the current node's CSR row:
 *     entry index = r mod degree for a 32-bit random word r; a node of degree 0
 *     keeps the walker where it is;
 *   - the random word of (start node u, walk w, step s>=1) is word (s-1)&3 of
 *     Philox4x32-10 with counter (u, w, (s-1)>>2, 0) and key (low 32 bits of
 *     rng_seed, high 32 bits of rng_seed);
 *   - counts are raw unsigned 16-bit integers (the worked example of Sec. 3.3/3.4
 *     shows integer vectors such as [2,0,0]);
 *   - V_u and the union are listed in ascending node id (the paper's hash
 *     dictionary has no order; ascending is the canonical one);
 *   - a query is an ordered tuple; its entries select rows of the RPE table
 *     (the i-th seed's block), and the halves of X_{Q,x} follow tuple order.
 *
 * Return values: >= 0 on success (row totals for the two variable-size calls),
 * -1 for a bad argument, -2 if the output capacity is too small (nothing beyond
 * the capacity is written), -3 out of memory.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox-4x32-10                                                            */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 32-bit random word that decides step s (1-based) of walk w started at node u. */
static uint32_t step_word(uint32_t u, uint32_t w, int s, uint64_t rng_seed)
{
    uint32_t ctr[4] = { u, w, (uint32_t)((s - 1) >> 2), 0u };
    uint32_t key[2] = { (uint32_t)(rng_seed & 0xFFFFFFFFu), (uint32_t)(rng_seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return out[(s - 1) & 3];
}

/* ------------------------------------------------------------------------- */
/* Walks: walks[i][w][0..m], i over seeds, w over the M walks of that seed.   */
/* ------------------------------------------------------------------------- */
int oracle_sample_walks(const int32_t *row_ptr, const int32_t *col_idx, int32_t n_nodes,
                        const int32_t *seeds, int64_t n_seeds, int32_t M, int32_t m,
                        uint64_t rng_seed, int32_t *walks)
{
    if (!row_ptr || (!col_idx && row_ptr[n_nodes] > 0) || n_nodes < 1 || n_seeds < 0 ||
        M < 1 || m < 1 || (n_seeds > 0 && (!seeds || !walks)))
        return -1;
    const int64_t L = (int64_t)m + 1;
    for (int64_t i = 0; i < n_seeds; ++i) {
        const int32_t u = seeds[i];
        if (u < 0 || u >= n_nodes)
            return -1;
        for (int32_t w = 0; w < M; ++w) {
            int32_t *walk = walks + (i * M + w) * L;
            int32_t cur = u;
            walk[0] = u;
            for (int s = 1; s <= m; ++s) {
                const uint32_t deg = (uint32_t)(row_ptr[cur + 1] - row_ptr[cur]);
                if (deg != 0u) {
                    const uint32_t r = step_word((uint32_t)u, (uint32_t)w, s, rng_seed);
                    cur = col_idx[(int64_t)row_ptr[cur] + (int64_t)(r % deg)];
                }
                walk[s] = cur;
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Node-level RPE table.                                                     */
/*   rpe_off[i]..rpe_off[i+1] are the rows of seed i; rpe_ids ascending in    */
/*   each block; rpe_cnt[row][s] = number of walks of seed i standing on      */
/*   rpe_ids[row] at position s.  ids / cnt may be NULL to only count rows.   */
/* ------------------------------------------------------------------------- */
static int cmp_i32(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int64_t oracle_build_rpe(const int32_t *walks, int64_t n_seeds, int32_t M, int32_t m,
                         int64_t cap_rows, int64_t *rpe_off, int32_t *rpe_ids,
                         uint16_t *rpe_cnt)
{
    if (n_seeds < 0 || M < 1 || M > 65535 || m < 1 || !rpe_off || (n_seeds > 0 && !walks))
        return -1;
    const int64_t L = (int64_t)m + 1;
    const int64_t per_seed = (int64_t)M * L;
    int32_t *set = (int32_t *)malloc((size_t)per_seed * sizeof(int32_t));
    uint16_t *cnt = (uint16_t *)malloc((size_t)per_seed * (size_t)L * sizeof(uint16_t));
    if (!set || !cnt) { free(set); free(cnt); return -3; }

    const int fill = rpe_ids != NULL && rpe_cnt != NULL;
    int64_t total = 0;
    int overflow = 0;
    rpe_off[0] = 0;
    for (int64_t i = 0; i < n_seeds; ++i) {
        const int32_t *W = walks + i * per_seed;
        /* V_u = set(W_u), ascending */
        memcpy(set, W, (size_t)per_seed * sizeof(int32_t));
        qsort(set, (size_t)per_seed, sizeof(int32_t), cmp_i32);
        int64_t n_set = 0;
        for (int64_t j = 0; j < per_seed; ++j)
            if (j == 0 || set[j] != set[j - 1])
                set[n_set++] = set[j];
        /* X_{u,x}[s] = #{ w : W_u[w][s] == x } */
        memset(cnt, 0, (size_t)n_set * (size_t)L * sizeof(uint16_t));
        for (int32_t w = 0; w < M; ++w) {
            for (int64_t s = 0; s < L; ++s) {
                const int32_t x = W[w * L + s];
                const int32_t *hit = (const int32_t *)bsearch(&x, set, (size_t)n_set,
                                                              sizeof(int32_t), cmp_i32);
                cnt[(hit - set) * L + s] += 1;
            }
        }
        if (fill) {
            if (total + n_set <= cap_rows) {
                memcpy(rpe_ids + total, set, (size_t)n_set * sizeof(int32_t));
                memcpy(rpe_cnt + total * L, cnt, (size_t)n_set * (size_t)L * sizeof(uint16_t));
            } else {
                overflow = 1;
            }
        }
        total += n_set;
        rpe_off[i + 1] = total;
    }
    free(set);
    free(cnt);
    return overflow ? -2 : total;
}

/* ------------------------------------------------------------------------- */
/* Query-level RPE by set union.                                             */
/*   queries[q][j], j < k, are row-block indices of the RPE table.            */
/*   join_ids: ascending union of the k id lists;                             */
/*   join_cnt[row][j][s] = X_{u_j,x}[s], zeros where x is not in V_{u_j}.      */
/* ------------------------------------------------------------------------- */
int64_t oracle_join_queries(const int64_t *rpe_off, const int32_t *rpe_ids,
                            const uint16_t *rpe_cnt, int64_t n_blocks, int32_t m,
                            const int32_t *queries, int64_t n_queries, int32_t k,
                            int64_t cap_rows, int64_t *join_off, int32_t *join_ids,
                            uint16_t *join_cnt)
{
    if (!rpe_off || n_blocks < 0 || m < 1 || n_queries < 0 || k < 1 || k > 8 || !join_off ||
        (n_queries > 0 && !queries))
        return -1;
    const int64_t L = (int64_t)m + 1;
    const int fill = join_ids != NULL && join_cnt != NULL;
    int64_t total = 0;
    int overflow = 0;
    join_off[0] = 0;
    for (int64_t q = 0; q < n_queries; ++q) {
        int64_t head[8], end[8];
        for (int j = 0; j < k; ++j) {
            const int32_t b = queries[q * k + j];
            if (b < 0 || b >= n_blocks)
                return -1;
            head[j] = rpe_off[b];
            end[j] = rpe_off[b + 1];
        }
        for (;;) {
            /* smallest id among the heads of the k lists */
            int have = 0;
            int32_t x = 0;
            for (int j = 0; j < k; ++j)
                if (head[j] < end[j] && (!have || rpe_ids[head[j]] < x)) {
                    x = rpe_ids[head[j]];
                    have = 1;
                }
            if (!have)
                break;
            const int writable = fill && total < cap_rows;
            if (fill && !writable)
                overflow = 1;
            if (writable)
                join_ids[total] = x;
            for (int j = 0; j < k; ++j) {
                const int present = head[j] < end[j] && rpe_ids[head[j]] == x;
                if (writable) {
                    uint16_t *dst = join_cnt + (total * k + j) * L;
                    if (present)
                        memcpy(dst, rpe_cnt + head[j] * L, (size_t)L * sizeof(uint16_t));
                    else
                        memset(dst, 0, (size_t)L * sizeof(uint16_t));
                }
                if (present)
                    head[j] += 1;
            }
            total += 1;
        }
        join_off[q + 1] = total;
    }
    return overflow ? -2 : total;
}

/* ------------------------------------------------------------------------- */
/* Query-level RPE-IDs per walk position.                                    */
/*   walks[b] is the walk block of table block b (the same seed).             */
/*   out[q][j][w][s][j2] = row of the table that holds (block queries[q][j2], */
/*   node walks[queries[q][j]][w][s]), or -1 if that block has no such node.  */
/* ------------------------------------------------------------------------- */
int oracle_query_rpe_ids(const int32_t *walks, const int64_t *rpe_off, const int32_t *rpe_ids,
                         int64_t n_blocks, int32_t M, int32_t m, const int32_t *queries,
                         int64_t n_queries, int32_t k, int64_t *out)
{
    if (n_blocks < 0 || M < 1 || m < 1 || n_queries < 0 || k < 1 || k > 8 || !rpe_off ||
        (n_queries > 0 && (!queries || !walks || !out)))
        return -1;
    const int64_t L = (int64_t)m + 1;
    for (int64_t q = 0; q < n_queries; ++q) {
        for (int j = 0; j < k; ++j)
            if (queries[q * k + j] < 0 || queries[q * k + j] >= n_blocks)
                return -1;
        for (int j = 0; j < k; ++j) {
            const int32_t *W = walks + (int64_t)queries[q * k + j] * M * L;
            for (int64_t t = 0; t < (int64_t)M * L; ++t) {
                const int32_t x = W[t];
                for (int j2 = 0; j2 < k; ++j2) {
                    const int32_t b = queries[q * k + j2];
                    const int32_t *set = rpe_ids + rpe_off[b];
                    const int64_t n_set = rpe_off[b + 1] - rpe_off[b];
                    const int32_t *hit =
                        n_set > 0 ? (const int32_t *)bsearch(&x, set, (size_t)n_set,
                                                             sizeof(int32_t), cmp_i32)
                                  : NULL;
                    out[(((q * k + j) * M * L) + t) * k + j2] =
                        hit ? rpe_off[b] + (int64_t)(hit - set) : -1;
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Pruning: distinct count vectors, sorted, and each row's index among them.  */
/* ------------------------------------------------------------------------- */
static int64_t g_vec_len; /* entries per vector, for the comparator (single-threaded code) */

static int cmp_vec(const void *a, const void *b)
{
    const uint16_t *x = (const uint16_t *)a, *y = (const uint16_t *)b;
    for (int64_t s = 0; s < g_vec_len; ++s)
        if (x[s] != y[s])
            return x[s] < y[s] ? -1 : 1;
    return 0;
}

/* T: uint16[cap_T][m+1], code: int32[n_rows]; both may be NULL (count only).
 * Returns the number of distinct vectors, or -2 if it exceeds cap_T (nothing is written then). */
int64_t oracle_prune_rpe(const uint16_t *rpe_cnt, int64_t n_rows, int32_t m, int64_t cap_T,
                         uint16_t *T, int32_t *code)
{
    if (n_rows < 0 || m < 1 || (n_rows > 0 && !rpe_cnt))
        return -1;
    const int64_t L = (int64_t)m + 1;
    const size_t vec_bytes = (size_t)L * sizeof(uint16_t);
    if (n_rows == 0)
        return 0;
    uint16_t *sorted = (uint16_t *)malloc((size_t)n_rows * vec_bytes);
    if (!sorted)
        return -1;
    memcpy(sorted, rpe_cnt, (size_t)n_rows * vec_bytes);
    g_vec_len = L;
    qsort(sorted, (size_t)n_rows, vec_bytes, cmp_vec);
    int64_t n_T = 0;
    for (int64_t r = 0; r < n_rows; ++r)
        if (r == 0 || cmp_vec(sorted + r * L, sorted + (r - 1) * L) != 0) {
            memmove(sorted + n_T * L, sorted + r * L, vec_bytes);
            n_T += 1;
        }
    if (T && code) {
        if (n_T > cap_T) {
            free(sorted);
            return -2;
        }
        memcpy(T, sorted, (size_t)n_T * vec_bytes);
        for (int64_t r = 0; r < n_rows; ++r) {
            const uint16_t *hit = (const uint16_t *)bsearch(rpe_cnt + r * L, sorted, (size_t)n_T,
                                                            vec_bytes, cmp_vec);
            code[r] = (int32_t)((hit - sorted) / L);
        }
    }
    free(sorted);
    return n_T;
}

/* ------------------------------------------------------------------------- */
/* Mini-batching: breadth-first search over nodes that share queries.         */
/* ------------------------------------------------------------------------- */

/* queries: int32[n_queries][k] node ids; start: the seed-set, in the order drawn (repeats are
 * dropped).  vbar: int32[B1] receives the node set in the order reached, batch: int32[B2] the
 * reached queries in the order reached; counts[0] = |vbar|, counts[1] = |batch|.
 * Returns 0, or -1 for a bad argument (also a node id outside [0, n_nodes)). */
int oracle_bfs_batch(const int32_t *queries, int64_t n_queries, int32_t k, int32_t n_nodes,
                     const int32_t *start, int64_t n_start, int64_t B1, int64_t B2,
                     int32_t *vbar, int32_t *batch, int64_t counts[2])
{
    if (n_queries < 0 || k < 1 || n_nodes < 1 || n_start < 0 || B1 < 1 || B2 < 1 || !vbar ||
        !batch || !counts || (n_queries > 0 && !queries) || (n_start > 0 && !start))
        return -1;
    for (int64_t t = 0; t < n_queries * k; ++t)
        if (queries[t] < 0 || queries[t] >= n_nodes)
            return -1;
    for (int64_t i = 0; i < n_start; ++i)
        if (start[i] < 0 || start[i] >= n_nodes)
            return -1;

    /* the queries of every node, ascending: first[x] .. first[x+1] in held[] */
    int64_t *first = (int64_t *)calloc((size_t)n_nodes + 1, sizeof(int64_t));
    int64_t *fill = (int64_t *)calloc((size_t)n_nodes + 1, sizeof(int64_t));
    int32_t *held = (int32_t *)malloc((size_t)(n_queries * k + 1) * sizeof(int32_t));
    char *in_vbar = (char *)calloc((size_t)n_nodes, 1);
    char *in_batch = (char *)calloc((size_t)n_queries + 1, 1);
    if (!first || !fill || !held || !in_vbar || !in_batch) {
        free(first); free(fill); free(held); free(in_vbar); free(in_batch);
        return -3;
    }
    for (int64_t t = 0; t < n_queries * k; ++t)
        first[queries[t] + 1] += 1;
    for (int32_t x = 0; x < n_nodes; ++x)
        first[x + 1] += first[x];
    for (int64_t q = 0; q < n_queries; ++q)
        for (int32_t j = 0; j < k; ++j) {
            const int32_t x = queries[q * k + j];
            held[first[x] + fill[x]++] = (int32_t)q;
        }

    int64_t n_v = 0, n_b = 0;
    for (int64_t i = 0; i < n_start && n_v < B1; ++i)
        if (!in_vbar[start[i]]) {
            in_vbar[start[i]] = 1;
            vbar[n_v++] = start[i];
        }
    int done = (n_v == B1);
    /* vbar doubles as the queue: nodes leave it in the order they entered */
    for (int64_t head = 0; head < n_v && !done; ++head) {
        const int32_t u = vbar[head];
        for (int64_t e = first[u]; e < first[u + 1] && !done; ++e) {
            const int32_t q = held[e];
            if (in_batch[q])
                continue;
            int64_t n_new = 0;
            for (int32_t j = 0; j < k; ++j) {
                const int32_t x = queries[(int64_t)q * k + j];
                int seen = in_vbar[x];
                for (int32_t i = 0; i < j; ++i)
                    seen |= (queries[(int64_t)q * k + i] == x);
                n_new += !seen;
            }
            if (n_v + n_new > B1) {
                done = 1;
                break;
            }
            in_batch[q] = 1;
            batch[n_b++] = q;
            for (int32_t j = 0; j < k; ++j) {
                const int32_t x = queries[(int64_t)q * k + j];
                if (!in_vbar[x]) {
                    in_vbar[x] = 1;
                    vbar[n_v++] = x;
                }
            }
            if (n_b == B2 || n_v == B1)
                done = 1;
        }
    }
    counts[0] = n_v;
    counts[1] = n_b;
    free(first); free(fill); free(held); free(in_vbar); free(in_batch);
    return 0;
}
