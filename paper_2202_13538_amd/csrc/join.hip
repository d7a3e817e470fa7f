// Query-based subgraph joining in its set-union form (Sec. 3.4): for a query tuple
// (b_1..b_K) the ascending union of the K node sets, and per union node the K count
// vectors in tuple order, zeros where the node is absent from a set.
//
// Two launches.  Counting: every query's union rows (an exclusive scan then turns the counts
// into join_off).  Filling: join_off is given (by that scan, or kept by the caller from an
// earlier call), the rows are written.  A wavefront handles one query at a time;
// the K sorted id lists are staged in LDS.  (Doing both in one launch, with the offsets from a scanner wave
// inside the kernel as the fused walk + RPE kernel has them, was built and measured: a wave has
// to wait for its query's offset between uniting and writing, which took 10.0 ms against
// 0.83 + 5.6 ms for the two launches on the 2.9M-node workload; holding one query back to hide
// that wait doubles the LDS a wave needs, and the filling launch with that footprint alone
// takes 8.9 ms.)
//
// Which union row a node lands in, and which table rows feed it ("sources"):
//   - pairs: a merge path.  Lane l owns merged positions [l*VT, (l+1)*VT): a binary search on
//     its diagonal finds where it starts in both lists, then it merges VT steps serially,
//     list 0 first on ties, so an equal pair is one row with two sources.  What the merge
//     leaves behind is two bits per union row ("list 0 has this node", "list 1 has it"), kept
//     as two bit masks in LDS: both lists are ascending like the union, so the table row of
//     list j that feeds union row r is the number of rows before r whose bit j is set, a
//     population count away for the lane that handles row r.
//   - triples: ranks.  A row is owned by the first list that holds its node; its position is
//     #{a in list 0 : a < x} + sum over j >= 1 of #{b in list j : b < x, b in no earlier list},
//     each term a lower bound in LDS plus a lookup in a prefix count of "new" elements; the
//     owner sets the row's bit in the mask of every list that holds the node.
// Count vectors.  For the usual walk lengths (m + 1 = 2 .. 6 entries per vector) a lane takes
// one union row: it gathers the row's K vectors from the table (zeros where the node is
// absent), packs them into the row's K*L/2 words in registers, and the row goes out either
// straight from the registers (vectors of whole words) or through a small LDS tile that is
// streamed out 16 bytes per lane (pairs of vectors with an odd number of entries, whose rows
// straddle words).  Other
// shapes take a generic path: a lane moves one (row, list) vector into an LDS tile laid out
// like the output.  The kernel keeps its LDS footprint small on purpose: the vectors are read
// in place, and it is the number of waves in flight that hides the latency.
#include "device_util.h"
#include "kernels.h"

namespace surel {

constexpr uint16_t kNoSrc = 0xFFFFu;
constexpr uint32_t kNoId = 0xFFFFFFFFu;  // no node id reaches 2^28
constexpr int kJoinChunkRows = 64;       // union rows staged in LDS per output tile
// Rounds of 64 union rows whose gathers a wave has in flight together.  More rounds shorten a
// wave's chain of memory round trips but cost registers, i.e. waves per compute unit: of 2 to
// 10 rounds, six made the fastest filling launch on the 2.9M-node workload (5.30 ms with two,
// 5.09 with six, 5.55 with eight); for the triples of the 1M-node workload four (1.80 ms with
// three, 1.77 with four, 1.96 with six, 2.26 with eight).
constexpr int kGatherRoundsPairs = 6;
constexpr int kGatherRoundsTuples = 4;

// First index t in [0, n) with list[t] >= x (n if none).  n is wave-uniform.
__device__ __forceinline__ int lower_bound_lds(const uint32_t* list, int n, uint32_t x) {
    int lo = 0;
    int len = n;
    while (len > 0) {
        const int half = len >> 1;
        if (list[lo + half] < x) {
            lo += half + 1;
            len -= half + 1;
        } else {
            len = half;
        }
    }
    return lo;
}

// Per-wave LDS layout, in 32-bit words.
struct JoinLds {
    int ids;      // [K][max_set] uint32
    int new_pre;  // [K-1][max_set+1] uint16 (triples only)
    int mask;     // [K][mask_words] uint32: bit r of mask j = list j feeds union row r (fill only)
    int mask_words;
    int src;      // [K][K*max_set] uint16: table row of list j that feeds union row r, or kNoSrc
    int tile;     // fill only
    int total;
};

// Rows whose K*L counts fill whole 32-bit words are put together in registers and written
// straight to the output, one lane per row; other shapes go through the LDS tile.
__host__ __device__ constexpr bool join_rows_direct(int K, int LT) {
    return LT > 0 && (K * LT) % 2 == 0;
}

// The LDS tile is needed by the generic path ([kJoinChunkRows][K][L] uint16) and by pairs whose
// count vectors have an odd number of entries (their rows are put together in the tile before
// they go out: 64 rows of LT words, plus up to 3 words in front so that the tile is aligned
// like the output it goes to).
__host__ __device__ constexpr bool join_uses_tile(int K, int LT) {
    return !join_rows_direct(K, LT) || (K == 2 && LT % 2 == 1);
}

// The sources of the union rows are kept as bit masks; the generic path expands them to indices.
__host__ __device__ constexpr bool join_uses_src(int K, int LT) { return !join_rows_direct(K, LT); }

__host__ __device__ constexpr JoinLds join_lds_layout(int K, int max_set, int L, bool fill,
                                                      int LT) {
    JoinLds o{};
    o.ids = 0;
    o.new_pre = o.ids + K * max_set;
    o.mask = o.new_pre + (K > 2 ? ((K - 1) * (max_set + 1) + 1) / 2 : 0);
    // one bit per union row, in whole 64-bit words, and two words of slack: a lane's bits are
    // put in as three 32-bit words at a time
    o.mask_words = fill ? 2 * ((K * max_set + 63) / 64) + 2 : 0;
    if (o.mask_words > 0) o.mask += o.mask & 1;  // the masks are read as 64-bit words
    o.src = o.mask + K * o.mask_words;
    const int src_end = o.src + (fill && join_uses_src(K, LT) ? (K * K * max_set + 1) / 2 : 0);
    // Only the tile of the pairs is moved 16 bytes at a time; nothing else is padded: the
    // words a wave needs decide how many waves a compute unit holds.
    const bool quads = fill && join_uses_tile(K, LT) && join_rows_direct(K, LT);
    o.tile = quads ? (src_end + 3) & ~3 : src_end;
    int tile_words = 0;
    if (fill && join_uses_tile(K, LT))
        tile_words = quads ? kWave * LT + 4 : (kJoinChunkRows * K * L + 1) / 2;
    o.total = o.tile + tile_words;
    if (quads) o.total = (o.total + 3) & ~3;  // every wave's part starts 16-byte aligned
    return o;
}

// Pairs: union size by merge path and, with kFlags, the two bit masks of the union rows (bit r
// of amask: list A holds the node of row r; bmask likewise).  The masks must be zero on entry.
template <bool kFlags>
__device__ __forceinline__ int union_pair_merge_path(const uint32_t* A, int nA, const uint32_t* B,
                                                     int nB, uint32_t* amask, uint32_t* bmask,
                                                     int lane) {
    const int T = nA + nB;
    const int VT = (T + kWave - 1) / kWave;  // at most 64: a set has at most 2048 nodes
    const int d0 = min(lane * VT, T);
    const int d1 = min(d0 + VT, T);
    // split of the first d0 merged elements: a0 from A (ties go to A first), d0 - a0 from B
    int lo = max(0, d0 - nB);
    int hi = min(d0, nA);
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (A[mid] <= B[d0 - 1 - mid]) {
            lo = mid + 1;
        } else {
            hi = mid;
        }
    }
    int a = lo, b = d0 - lo;

    // The lane's VT merge steps.  Every step that takes an A element emits a row; a step that
    // takes a B element emits one unless it equals the last A element taken (the same node:
    // ids are distinct inside a list), which may have been taken by the lane before this one.
    // Only the list that moved is read again.
    int n_emit = 0;
    uint64_t fa = 0, fb = 0;  // bit i: this lane's i-th row has a source in A / in B
    uint32_t last_a = a > 0 ? A[a - 1] : kNoId;
    uint32_t va = a < nA ? A[a] : kNoId;
    uint32_t vb = b < nB ? B[b] : kNoId;
    for (int d = d0; d < d1; ++d) {
        const bool take_a = (b >= nB) || (a < nA && va <= vb);
        if (take_a) {
            if (kFlags) {
                fa |= 1ull << n_emit;
                if (b < nB && vb == va) fb |= 1ull << n_emit;
            }
            n_emit += 1;
            last_a = va;
            a += 1;
        } else {
            if (vb != last_a) {
                if (kFlags) fb |= 1ull << n_emit;
                n_emit += 1;
            }
            b += 1;
        }
        const uint32_t* list = take_a ? A : B;
        const int at = take_a ? a : b;
        const bool more = at < (take_a ? nA : nB);
        const uint32_t next = more ? list[at] : kNoId;
        va = take_a ? next : va;
        vb = take_a ? vb : next;
    }
    const int incl = (int)wave_incl_sum((uint32_t)n_emit);
    const int n_out = (int)wave_bcast_u32((uint32_t)incl, kWave - 1);
    if (kFlags) {
        // the lane's rows start at row0: its bits go in there, as up to three 32-bit words
        const int row0 = incl - n_emit;
        const int w = row0 >> 5;
        const int sh = row0 & 31;
        const uint64_t fl[2] = {fa, fb};
        uint32_t* const mask[2] = {amask, bmask};
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint64_t low = fl[j] << sh;
            const uint32_t w0 = (uint32_t)low;
            const uint32_t w1 = (uint32_t)(low >> 32);
            const uint32_t w2 = sh ? (uint32_t)(fl[j] >> (64 - sh)) : 0u;
            if (w0) atomicOr(mask[j] + w, w0);
            if (w1) atomicOr(mask[j] + w + 1, w1);
            if (w2) atomicOr(mask[j] + w + 2, w2);
        }
    }
    return n_out;
}

// The sources of the 64 union rows r0 .. r0+63, from the masks: lane l learns for row r0 + l
// whether list j feeds it and from which of the list's rows.  before[j] = rows of list j that
// feed union rows below r0; it is moved on to r0 + 64.  A source index is checked against the
// list's length, which only a malformed (unsorted) table can exceed.
template <int K>
__device__ __forceinline__ void row_sources(const uint32_t* mask, int mask_words, int r0,
                                            const int (&n)[K], int (&before)[K], int lane,
                                            bool (&present)[K], int (&index)[K]) {
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const uint64_t bits = *reinterpret_cast<const uint64_t*>(mask + j * mask_words + (r0 >> 5));
        const int rank = (int)__builtin_amdgcn_mbcnt_hi(
            (uint32_t)(bits >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bits, 0u));
        index[j] = before[j] + rank;
        present[j] = ((bits >> lane) & 1ull) != 0ull && index[j] < n[j];
        before[j] += __popcll(bits);
    }
}

// Any K: union size and (when kFill) the masks of the union rows, by ranks.  The masks must be
// zero on entry.
template <int K, bool kFill>
__device__ __forceinline__ int union_ranked(const uint32_t* ids_lds, const int (&n)[K], int max_set,
                                            uint16_t* new_pre, uint32_t* mask, int mask_words,
                                            int lane) {
    // per list j >= 1: exclusive prefix count of elements that no earlier list contains
    int n_out = n[0];
#pragma unroll
    for (int j = 1; j < K; ++j) {
        uint16_t* pre = new_pre + (j - 1) * (max_set + 1);
        int carry = 0;
        for (int t0 = 0; t0 < n[j]; t0 += kWave) {
            const int t = t0 + lane;
            bool is_new = false;
            if (t < n[j]) {
                const uint32_t x = ids_lds[j * max_set + t];
                is_new = true;
#pragma unroll
                for (int jj = 0; jj < j; ++jj) {
                    const uint32_t* other = ids_lds + jj * max_set;
                    const int p = lower_bound_lds(other, n[jj], x);
                    if (p < n[jj] && other[p] == x) is_new = false;
                }
            }
            const uint64_t mask = __ballot(is_new);
            const int before = (int)__builtin_amdgcn_mbcnt_hi(
                (uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (t < n[j]) pre[t] = (uint16_t)(carry + before);
            carry += __popcll(mask);
        }
        if (lane == 0) pre[n[j]] = (uint16_t)carry;
        n_out += carry;
    }
    if (!kFill || n_out == 0) return n_out;
    wave_sync();
    // every union row is marked by the first list that holds its node
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const uint16_t* pre_j = new_pre + (j > 0 ? j - 1 : 0) * (max_set + 1);  // j >= 1 only
        for (int t = lane; t < n[j]; t += kWave) {
            const uint32_t x = ids_lds[j * max_set + t];
            if (j > 0 && pre_j[t + 1] == pre_j[t]) continue;  // owned by an earlier list
            int pos = 0;
            bool present[K];
#pragma unroll
            for (int jj = 0; jj < K; ++jj) {
                if (jj == j) {
                    pos += (j == 0) ? t : (int)pre_j[t];
                    present[jj] = true;
                } else {
                    const uint32_t* other = ids_lds + jj * max_set;
                    const int p = lower_bound_lds(other, n[jj], x);
                    pos += (jj == 0) ? p : (int)new_pre[(jj - 1) * (max_set + 1) + p];
                    present[jj] = jj > j && p < n[jj] && other[p] == x;
                }
            }
            // pos < K * max_set whatever the lists hold: every term is at most a list's length
#pragma unroll
            for (int jj = 0; jj < K; ++jj)
                if (present[jj]) atomicOr(mask + jj * mask_words + (pos >> 5), 1u << (pos & 31));
        }
    }
    return n_out;
}

// One count vector of LT (compile time) or L (LT == 0) entries from the table into LDS.  With
// LT known the loads are issued together, before the first of them is waited for.
template <int LT>
__device__ __forceinline__ void copy_vector(uint16_t* dst, const uint16_t* from, int L) {
    if constexpr (LT > 0) {
        uint16_t v[LT];
#pragma unroll
        for (int s = 0; s < LT; ++s) v[s] = from[s];
#pragma unroll
        for (int s = 0; s < LT; ++s) dst[s] = v[s];
    } else {
        for (int s = 0; s < L; ++s) dst[s] = from[s];
    }
}
template <int LT>
__device__ __forceinline__ void fill_vector(uint16_t* dst, int L, uint16_t value) {
    if constexpr (LT > 0) {
#pragma unroll
        for (int s = 0; s < LT; ++s) dst[s] = value;
    } else {
        for (int s = 0; s < L; ++s) dst[s] = value;
    }
}

// The blocks of one query and where its union rows come from, as join_prepare leaves them.
template <int K>
struct JoinQuery {
    int64_t lo[K];  // first table row of block j
    int n[K];       // rows of block j
};

// First half of a query: looks its K blocks up, stages their id lists in LDS and unites them.
// Returns the number of union rows, or -1 if the query is unusable (its problem is flagged and it
// yields no rows).  With kSrc the sources of every union row are left in LDS for join_write.
// K = tuple size, LT = m+1 at compile time for the usual walk lengths (2 .. 6), 0 = any.
template <int K, bool kSrc, int LT>
__device__ __forceinline__ int join_prepare(
    uint32_t* base, int lane, int64_t q, const int64_t* __restrict__ rpe_off,
    const int32_t* __restrict__ rpe_ids, int64_t n_blocks, int32_t m, int32_t max_set,
    const int32_t* __restrict__ queries, JoinQuery<K>& jq, uint32_t* __restrict__ err) {
    const int L = LT > 0 ? LT : m + 1;
    const JoinLds lay = join_lds_layout(K, max_set, L, kSrc, LT);
    uint32_t* ids_lds = base + lay.ids;
    uint16_t* new_pre = reinterpret_cast<uint16_t*>(base + lay.new_pre);
    uint32_t* mask = base + lay.mask;
    uint16_t* src = reinterpret_cast<uint16_t*>(base + lay.src);
    const int src_stride = K * max_set;

    // the K blocks of this query (wave-uniform)
    uint32_t problem = 0;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int32_t b = queries[q * K + j];
        jq.lo[j] = 0;
        jq.n[j] = 0;
        if (b < 0 || (int64_t)b >= n_blocks) {
            problem |= kDevBadQuery;
        } else {
            const int64_t a = rpe_off[b];
            const int64_t len = rpe_off[b + 1] - a;
            if (a < 0 || len < 0) {
                problem |= kDevBadTable;
            } else if (len > (int64_t)max_set) {
                problem |= kDevSetTooLarge;
            } else {
                jq.lo[j] = a;
                jq.n[j] = (int)len;
            }
        }
    }
    if (problem != 0) {
        if (lane == 0) atomicOr(err, problem);
        return -1;
    }

    // stage the id lists
#pragma unroll
    for (int j = 0; j < K; ++j)
        stage_words<8>(ids_lds + j * max_set, reinterpret_cast<const uint32_t*>(rpe_ids + jq.lo[j]),
                       jq.n[j], lane);
    wave_sync();

    if (kSrc) {
        for (int t = lane; t < K * lay.mask_words; t += kWave) mask[t] = 0u;
        wave_sync();
    }
    int n_out;
    if constexpr (K == 2) {
        n_out = union_pair_merge_path<kSrc>(ids_lds, jq.n[0], ids_lds + max_set, jq.n[1], mask,
                                            mask + lay.mask_words, lane);
    } else {
        n_out = union_ranked<K, kSrc>(ids_lds, jq.n, max_set, new_pre, mask, lay.mask_words, lane);
    }
    if constexpr (kSrc && join_uses_src(K, LT)) {
        // the generic path wants an index per (list, row)
        wave_sync();
        int before[K];
#pragma unroll
        for (int j = 0; j < K; ++j) before[j] = 0;
        for (int r0 = 0; r0 < n_out; r0 += kWave) {
            bool present[K];
            int index[K];
            row_sources<K>(mask, lay.mask_words, r0, jq.n, before, lane, present, index);
            if (r0 + lane < n_out) {
#pragma unroll
                for (int j = 0; j < K; ++j)
                    src[j * src_stride + r0 + lane] = present[j] ? (uint16_t)index[j] : kNoSrc;
            }
        }
    }
    return n_out;
}

// Second half: writes the n_out > 0 union rows of the query that join_prepare<K, true, LT> left
// in LDS to rows [off, off + n_out) of the output.
template <int K, int LT>
__device__ __forceinline__ void join_write(
    uint32_t* base, int lane, const JoinQuery<K>& jq, int n_out, int64_t off,
    const uint16_t* __restrict__ rpe_cnt, int32_t m, int32_t max_set,
    int32_t* __restrict__ out_ids, uint16_t* __restrict__ out_cnt, uint16_t absent16) {
    const int L = LT > 0 ? LT : m + 1;
    const JoinLds lay = join_lds_layout(K, max_set, L, true, LT);
    uint32_t* ids_lds = base + lay.ids;
    const uint32_t* mask = base + lay.mask;
    uint16_t* src = reinterpret_cast<uint16_t*>(base + lay.src);
    uint32_t* tile32 = base + lay.tile;
    uint16_t* tile = reinterpret_cast<uint16_t*>(tile32);
    const int src_stride = K * max_set;
    const int (&n)[K] = jq.n;
    const int64_t (&lo)[K] = jq.lo;
    wave_sync();

    if constexpr (join_rows_direct(K, LT)) {
        // one lane per union row: the K count vectors (or zeros) are packed into the row's
        // K*L/2 words in registers and stored at the row's place
        constexpr int kWords = K * LT / 2;
        constexpr int kHalf = LT / 2;       // whole words of a vector
        constexpr int kCover = LT / 2 + 1;  // aligned words that cover a vector wherever it starts
        uint32_t* out_words = reinterpret_cast<uint32_t*>(out_cnt) + off * kWords;
        // kRounds rounds of 64 rows are gathered together (all their loads are in
        // flight before the first is waited for: a wave's time is a chain of memory round
        // trips), then the rounds go out one after the other
        constexpr int kRounds = K == 2 ? kGatherRoundsPairs : kGatherRoundsTuples;
        const uint32_t absent32 = (uint32_t)absent16 * 0x10001u;
        // Where list j's vectors are: the aligned word at or before the first of them (uniform),
        // and whether that one starts in the word's upper half.  A lane then gets by with
        // 32-bit arithmetic: its vector starts odd[j] + (row in the list) * LT counts in.  A
        // list without rows has no vectors to point at: the table's first row stands in (the
        // table has rows, or there would be no union rows to write).
        const uint32_t* vec_words[K];
        uint32_t odd[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const uint16_t* first = rpe_cnt + (n[j] > 0 ? lo[j] : 0) * LT;
            odd[j] = (uint32_t)((reinterpret_cast<uintptr_t>(first) >> 1) & 1u);
            vec_words[j] = reinterpret_cast<const uint32_t*>(first - odd[j]);
        }
        int before[K];
#pragma unroll
        for (int j = 0; j < K; ++j) before[j] = 0;
        for (int r0 = 0; r0 < n_out; r0 += kRounds * kWave) {
            uint32_t raw[kRounds][K][kCover + 1];
            uint32_t shift[kRounds][K];
            bool present[kRounds][K];
            uint32_t id[kRounds];
#pragma unroll
            for (int g = 0; g < kRounds; ++g) {
                if (r0 + g * kWave >= n_out) break;  // wave-uniform: no round past the last row
                int index[K];
                row_sources<K>(mask, lay.mask_words, r0 + g * kWave, n, before, lane, present[g],
                               index);
                // the node's id, from the first list that has it (a lane past the last row
                // reads the first id and stores nothing)
                int id_at = 0;
#pragma unroll
                for (int j = K - 1; j >= 0; --j)
                    if (present[g][j]) id_at = j * max_set + index[j];
                id[g] = ids_lds[id_at];
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    // unconditional loads, from the list's first row where it has no row for
                    // the node: a branch would make every load wait for the one before it.  A
                    // vector is read as the aligned words that cover it (misaligned wide loads
                    // are taken apart lane by lane by the L1) and shifted into place
                    // afterwards; the last word may reach one count past the vector, never
                    // past the word that holds the table's last count.
                    const uint32_t first = odd[j] + (uint32_t)(present[g][j] ? index[j] : 0) * LT;
                    shift[g][j] = (first & 1u) * 2u;
                    const uint32_t* aligned = vec_words[j] + (first >> 1);
#pragma unroll
                    for (int t = 0; t < kCover; ++t)
                        raw[g][j][t] = (LT % 2 == 0 && t == kCover - 1) ? 0u : aligned[t];
                    raw[g][j][kCover] = 0u;
                }
            }
#pragma unroll
            for (int g = 0; g < kRounds; ++g) {
                if (r0 + g * kWave >= n_out) break;
                // word t of vector j holds its counts 2t and 2t+1; a vector of an odd number of
                // counts ends in the low half of its last word
                uint32_t w[kWords];
#pragma unroll
                for (int j = 0; j < K; ++j) {
                    uint32_t vec[kCover];
#pragma unroll
                    for (int t = 0; t < kCover; ++t) {
                        vec[t] = __builtin_amdgcn_alignbyte(raw[g][j][t + 1], raw[g][j][t],
                                                            shift[g][j]);
                        if (!present[g][j]) vec[t] = absent32;
                    }
                    const int start = j * LT;  // first count of the vector inside the row
                    if (start % 2 == 0) {
#pragma unroll
                        for (int t = 0; t < kHalf; ++t) w[start / 2 + t] = vec[t];
                        if (LT % 2 == 1) w[start / 2 + kHalf] = vec[kHalf] & 0xFFFFu;
                    } else {
                        w[(start - 1) / 2] |= vec[0] << 16;
#pragma unroll
                        for (int t = 0; t < kHalf; ++t)
                            w[(start + 1) / 2 + t] =
                                __builtin_amdgcn_alignbyte(vec[t + 1], vec[t], 2u);
                    }
                }
                const int r = r0 + g * kWave + lane;
                const bool live = r < n_out;
                if (live) out_ids[off + r] = (int32_t)id[g];
                if constexpr (LT % 2 == 0) {
                    // count vectors of whole words: a lane's row is stored from its registers
                    // (the rows of neighbouring lanes adjoin, so a wave's stores are contiguous)
                    if (live) {
                        uint32_t* row_words = out_words + (int64_t)r * kWords;
#pragma unroll
                        for (int d = 0; d < kWords; ++d) row_words[d] = w[d];
                    }
                } else {
                    // an odd number of 16-bit counts per list: the rows are put together in an
                    // LDS tile and go out 16 bytes per lane.  The tile starts `head` words in,
                    // so that 16-byte pieces of the tile are 16-byte pieces of the output.
                    uint32_t* dst = out_words + (int64_t)(r0 + g * kWave) * kWords;
                    const int head = (int)((reinterpret_cast<uintptr_t>(dst) >> 2) & 3u);
#pragma unroll
                    for (int d = 0; d < kWords; ++d) tile32[head + lane * kWords + d] = w[d];
                    wave_sync();
                    const int n_words = min(kWave, n_out - (r0 + g * kWave)) * kWords;
                    const int lead = min((4 - head) & 3, n_words);  // words before the first piece
                    const int n_quads = (n_words - lead) >> 2;
                    const int tail = lead + 4 * n_quads;           // words after the last piece
                    if (lane < lead) dst[lane] = tile32[head + lane];
                    const uint4* tile_quads = reinterpret_cast<const uint4*>(tile32 + head + lead);
                    uint4* dst_quads = reinterpret_cast<uint4*>(dst + lead);
                    for (int t = lane; t < n_quads; t += kWave) dst_quads[t] = tile_quads[t];
                    if (lane < n_words - tail) dst[tail + lane] = tile32[head + tail + lane];
                    wave_sync();
                }
            }
        }
        return;
    }

    const int KL = K * L;
    for (int r0 = 0; r0 < n_out; r0 += kJoinChunkRows) {
        const int rows = min(kJoinChunkRows, n_out - r0);

        // ids of these union rows (any list that holds the node gives the same id)
        if (lane < rows) {
            uint32_t id = 0;
#pragma unroll
            for (int jj = K - 1; jj >= 0; --jj) {
                const uint16_t sj = src[jj * src_stride + r0 + lane];
                if ((int)sj < n[jj]) id = ids_lds[jj * max_set + sj];  // kNoSrc is >= any n
            }
            out_ids[off + r0 + lane] = (int32_t)id;
        }

        // one lane per (row, list): that list's count vector, or zeros, into the tile
        for (int t = lane; t < rows * K; t += kWave) {
            const int row = t / K;
            const int j = t - row * K;
            const uint16_t sj = src[j * src_stride + r0 + row];
            int len = n[0];
            int64_t first = lo[0];
#pragma unroll
            for (int jj = 1; jj < K; ++jj) {
                if (j == jj) {
                    len = n[jj];
                    first = lo[jj];
                }
            }
            uint16_t* dst = tile + t * L;
            // kNoSrc is >= any len; the bound also covers a malformed (unsorted) table
            if ((int)sj < len) {
                copy_vector<LT>(dst, rpe_cnt + (first + sj) * L, L);
            } else {
                fill_vector<LT>(dst, L, absent16);
            }
        }
        wave_sync();

        // stream the tile out as dwords where the destination allows
        const int n_el = rows * KL;
        const int64_t d0 = (off + r0) * KL;  // first destination element (uint16 units)
        const int head = (int)(d0 & 1);
        uint16_t* out = out_cnt + d0;
        if (head && lane == 0) out[0] = tile[0];
        const int n_pair = (n_el - head) / 2;
        uint32_t* out32 = reinterpret_cast<uint32_t*>(out + head);
        if (head == 0) {
            for (int t = lane; t < n_pair; t += kWave) out32[t] = tile32[t];
        } else {
            for (int t = lane; t < n_pair; t += kWave)
                out32[t] = (uint32_t)tile[1 + 2 * t] | ((uint32_t)tile[2 + 2 * t] << 16);
        }
        if (((n_el - head) & 1) && lane == 0) out[n_el - 1] = tile[n_el - 1];
        wave_sync();
    }
}

// Filling.  One wavefront per workgroup and one query per wavefront; the grid covers the query
// list.  The hardware hands workgroups out as others retire, which keeps every compute unit
// full whatever the queries' sizes are and however many waves it really holds.  (A grid of
// exactly as many waves as the occupancy query promises, each looping over a strided share of
// the queries, was slower: where the device held fewer workgroups than promised, the surplus
// ran as a tail after the others, +25 % on one workload; and with four waves to a workgroup a
// slot stays taken until the slowest of the four is done.)
// join_off is complete (the caller's, or the scan of a counting launch).  A query whose union
// does not have the join_off[q+1] - join_off[q] rows that the offsets give it is flagged and
// writes nothing.
template <int K, int LT>
__global__ __launch_bounds__(kWave) void join_fill_kernel(
    const int64_t* __restrict__ rpe_off, const int32_t* __restrict__ rpe_ids,
    const uint16_t* __restrict__ rpe_cnt, int64_t n_blocks, int32_t m, int32_t max_set,
    const int32_t* __restrict__ queries, int64_t n_queries,
    const int64_t* __restrict__ join_off, int64_t cap_rows, int32_t* __restrict__ out_ids,
    uint16_t* __restrict__ out_cnt, uint16_t absent16, uint32_t* __restrict__ err) {
    extern __shared__ __align__(16) uint32_t base[];
    const int lane = lane_id();
    // (written as a loop over the wave's one query: the compiler's code for this form makes the
    // launch 2 % faster on the 2.9M-node workload than the same statements in a row)
    constexpr int kPerWave = 1;
    const int64_t q_first = (int64_t)blockIdx.x * kPerWave;
#pragma unroll 1
    for (int64_t q = q_first; q < min(q_first + kPerWave, n_queries); ++q) {
        JoinQuery<K> jq;
        // the same in every lane; said so, the loops over the rows are scalar loops
        const int n_out = __builtin_amdgcn_readfirstlane(join_prepare<K, true, LT>(
            base, lane, q, rpe_off, rpe_ids, n_blocks, m, max_set, queries, jq, err));
        const int64_t off = join_off[q];
        const int rows = n_out > 0 ? n_out : 0;  // an unusable query yields no rows
        if (join_off[q + 1] - off != (int64_t)rows) {
            if (lane == 0) atomicOr(err, kDevBadSizes);
        } else if (rows > 0 && off + rows > cap_rows) {
            if (lane == 0) atomicOr(err, kDevCapacity);
        } else if (rows > 0) {
            join_write<K, LT>(base, lane, jq, rows, off, rpe_cnt, m, max_set, out_ids, out_cnt,
                              absent16);
        }
        wave_sync();
    }
}

// Counting.  A wavefront takes join_count_queries(K) consecutive queries.  Their
// blocks are looked up by one lane each (block numbers, then the blocks' offsets: two round
// trips to memory for all of them), and while the id lists of one query are united in LDS the
// lists of the next one are already on their way into registers: a query's time is then the
// longer of its merge and one round trip, where looking up, staging and uniting one query
// after the other took three round trips and the merge.
// (Measured on the 2.9M-node workload, pairs: 0.77 ms one query after the other, four to a
// wave; 0.71 / 0.66 / 0.64 / 0.64 ms this way with 2 / 4 / 8 / 16 to a wave.  Triples of the
// 1M-node workload: 0.42, and 0.41 / 0.41 / 0.42 / 0.47.)
__host__ __device__ constexpr int join_count_queries(int K) { return K == 2 ? 8 : 4; }
constexpr int kCountStage = 8;  // words of a list a lane holds for the next query (512 ids)

template <int K>
__global__ __launch_bounds__(kWave) void join_count_kernel(
    const int64_t* __restrict__ rpe_off, const int32_t* __restrict__ rpe_ids, int64_t n_blocks,
    int32_t max_set, const int32_t* __restrict__ queries, int64_t n_queries,
    int32_t* __restrict__ counts, uint32_t* __restrict__ err) {
    extern __shared__ __align__(16) uint32_t base[];
    const JoinLds lay = join_lds_layout(K, max_set, 2, false, 0);
    uint32_t* ids_lds = base + lay.ids;
    uint16_t* new_pre = reinterpret_cast<uint16_t*>(base + lay.new_pre);
    const int lane = lane_id();
    constexpr int kCountQueries = join_count_queries(K);
    const int64_t q_first = (int64_t)blockIdx.x * kCountQueries;

    // lane l < kCountQueries looks up the blocks of query q_first + l
    int64_t my_lo[K];
    int my_n[K];
    uint32_t my_problem = 0;
#pragma unroll
    for (int j = 0; j < K; ++j) {
        my_lo[j] = 0;
        my_n[j] = 0;
    }
    if (lane < kCountQueries && q_first + lane < n_queries) {
        int32_t b[K];
#pragma unroll
        for (int j = 0; j < K; ++j) b[j] = queries[(q_first + lane) * K + j];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            if (b[j] < 0 || (int64_t)b[j] >= n_blocks) {
                my_problem |= kDevBadQuery;
            } else {
                const int64_t a = rpe_off[b[j]];
                const int64_t len = rpe_off[b[j] + 1] - a;
                if (a < 0 || len < 0) {
                    my_problem |= kDevBadTable;
                } else if (len > (int64_t)max_set) {
                    my_problem |= kDevSetTooLarge;
                } else {
                    my_lo[j] = a;
                    my_n[j] = (int)len;
                }
            }
        }
        if (my_problem != 0) {  // the query is flagged and yields no rows
            atomicOr(err, my_problem);
#pragma unroll
            for (int j = 0; j < K; ++j) my_n[j] = 0;
        }
    }
    // query i's blocks, the same in every lane
    auto blocks_of = [&](int i, int64_t (&lo)[K], int (&n)[K]) {
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const uint32_t lo_l = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(uint64_t)my_lo[j], i);
            const uint32_t lo_h = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)my_lo[j] >> 32), i);
            lo[j] = (int64_t)(((uint64_t)lo_h << 32) | lo_l);
            n[j] = __builtin_amdgcn_readlane(my_n[j], i);
        }
    };
    uint32_t staged[K][kCountStage];
    auto fetch = [&](const int64_t (&lo)[K], const int (&n)[K]) {
#pragma unroll
        for (int j = 0; j < K; ++j) {
#pragma unroll
            for (int u = 0; u < kCountStage; ++u) {
                const int t = u * kWave + lane;
                staged[j][u] = t < n[j] ? (uint32_t)rpe_ids[lo[j] + t] : 0u;
            }
        }
    };
    int64_t lo[K];
    int n[K];
    blocks_of(0, lo, n);
    fetch(lo, n);
#pragma unroll
    for (int i = 0; i < kCountQueries; ++i) {
        const int64_t q = q_first + i;
        if (q >= n_queries) break;
        // the lists of query i: from the registers, and what is longer than they hold from memory
#pragma unroll
        for (int j = 0; j < K; ++j) {
#pragma unroll
            for (int u = 0; u < kCountStage; ++u) {
                const int t = u * kWave + lane;
                if (t < n[j]) ids_lds[j * max_set + t] = staged[j][u];
            }
            if (n[j] > kCountStage * kWave)
                stage_words<8>(ids_lds + j * max_set + kCountStage * kWave,
                               reinterpret_cast<const uint32_t*>(rpe_ids + lo[j]) + kCountStage * kWave,
                               n[j] - kCountStage * kWave, lane);
        }
        wave_sync();
        int n_now[K];
#pragma unroll
        for (int j = 0; j < K; ++j) n_now[j] = n[j];
        if (i + 1 < kCountQueries && q + 1 < n_queries) {
            blocks_of(i + 1, lo, n);
            fetch(lo, n);  // in flight while query i is united
        }
        int n_out;
        if constexpr (K == 2) {
            n_out = union_pair_merge_path<false>(ids_lds, n_now[0], ids_lds + max_set, n_now[1],
                                                 nullptr, nullptr, lane);
        } else {
            n_out = union_ranked<K, false>(ids_lds, n_now, max_set, new_pre, nullptr, 0, lane);
        }
        if (lane == 0) counts[q] = n_out;
        wave_sync();  // the next query reuses the LDS words
    }
}

// What a launch is asked to do.
struct JoinJob {
    hipStream_t stream;
    int max_lds_bytes;
    const int64_t* rpe_off;
    const int32_t* rpe_ids;
    const uint16_t* rpe_cnt;
    int64_t n_blocks;
    int32_t m;
    int32_t max_set;
    const int32_t* queries;
    int64_t n_queries;
    int32_t* counts;          // counting launch: written
    const int64_t* join_off;  // filling launch: read
    int64_t cap_rows;
    int32_t* out_ids;
    uint16_t* out_cnt;
    uint16_t absent16;
    uint32_t* err;
};

template <int K, int LT>
static hipError_t launch_join_fill_cfg(const JoinJob& j) {
    const size_t lds_bytes = (size_t)join_lds_layout(K, j.max_set, j.m + 1, true, LT).total * 4;
    if (lds_bytes > (size_t)j.max_lds_bytes) return hipErrorInvalidValue;
    const void* fn = reinterpret_cast<const void*>(join_fill_kernel<K, LT>);
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    if (j.n_queries > 0x7FFFFFFFll) return hipErrorInvalidValue;
    hipLaunchKernelGGL((join_fill_kernel<K, LT>), dim3((unsigned)j.n_queries), dim3(kWave),
                       lds_bytes, j.stream, j.rpe_off, j.rpe_ids, j.rpe_cnt, j.n_blocks, j.m,
                       j.max_set, j.queries, j.n_queries, j.join_off, j.cap_rows, j.out_ids,
                       j.out_cnt, j.absent16, j.err);
    return hipGetLastError();
}

// m + 1 at compile time for the usual walk lengths
template <int K>
static hipError_t launch_join_fill_k(const JoinJob& j) {
    switch (j.m + 1) {
        case 2: return launch_join_fill_cfg<K, 2>(j);
        case 3: return launch_join_fill_cfg<K, 3>(j);
        case 4: return launch_join_fill_cfg<K, 4>(j);
        case 5: return launch_join_fill_cfg<K, 5>(j);
        case 6: return launch_join_fill_cfg<K, 6>(j);
        default: return launch_join_fill_cfg<K, 0>(j);
    }
}

template <int K>
static hipError_t launch_join_count_k(const JoinJob& j) {
    constexpr int kCountQueries = join_count_queries(K);
    const size_t lds_bytes = (size_t)join_lds_layout(K, j.max_set, 2, false, 0).total * 4;
    if (lds_bytes > (size_t)j.max_lds_bytes) return hipErrorInvalidValue;
    const void* fn = reinterpret_cast<const void*>(join_count_kernel<K>);
    if (lds_bytes > 48 * 1024) {
        hipError_t rc = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)lds_bytes);
        if (rc != hipSuccess) return rc;
    }
    const int64_t blocks = (j.n_queries + kCountQueries - 1) / kCountQueries;
    hipLaunchKernelGGL((join_count_kernel<K>), dim3((unsigned)blocks), dim3(kWave), lds_bytes,
                       j.stream, j.rpe_off, j.rpe_ids, j.n_blocks, j.max_set, j.queries,
                       j.n_queries, j.counts, j.err);
    return hipGetLastError();
}

hipError_t launch_join_count(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                             const int32_t* rpe_ids, int64_t n_blocks, int32_t max_set,
                             const int32_t* queries, int64_t n_queries, int32_t k, int32_t* counts,
                             uint32_t* err) {
    JoinJob j{};
    j.stream = stream, j.max_lds_bytes = max_lds_bytes;
    j.rpe_off = rpe_off, j.rpe_ids = rpe_ids, j.n_blocks = n_blocks, j.m = 1, j.max_set = max_set;
    j.queries = queries, j.n_queries = n_queries, j.counts = counts, j.err = err;
    if (n_queries == 0) return hipSuccess;
    if (k == 2) return launch_join_count_k<2>(j);
    if (k == 3) return launch_join_count_k<3>(j);
    return hipErrorInvalidValue;
}

hipError_t launch_join_fill(hipStream_t stream, int max_lds_bytes, const int64_t* rpe_off,
                            const int32_t* rpe_ids, const uint16_t* rpe_cnt, int64_t n_blocks,
                            int32_t m, int32_t max_set, const int32_t* queries, int64_t n_queries,
                            int32_t k, const int64_t* join_off, int64_t cap_rows, int32_t* out_ids,
                            uint16_t* out_cnt, uint16_t absent16, uint32_t* err) {
    JoinJob j{};
    j.stream = stream, j.max_lds_bytes = max_lds_bytes;
    j.rpe_off = rpe_off, j.rpe_ids = rpe_ids, j.rpe_cnt = rpe_cnt, j.n_blocks = n_blocks, j.m = m;
    j.max_set = max_set, j.queries = queries, j.n_queries = n_queries, j.join_off = join_off;
    j.cap_rows = cap_rows, j.out_ids = out_ids, j.out_cnt = out_cnt, j.absent16 = absent16;
    j.err = err;
    if (n_queries == 0) return hipSuccess;
    if (k == 2) return launch_join_fill_k<2>(j);
    if (k == 3) return launch_join_fill_k<3>(j);
    return hipErrorInvalidValue;
}

}  // namespace surel
