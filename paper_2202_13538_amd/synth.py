"""Seeded synthetic inputs: graphs in CSR form and query tuples.

This module only makes *inputs*.  It holds none of the method's arithmetic (no
random-walk step, no counting, no merging) and is the one module that both the
HIP path and the CPU oracle's tests may import.  Everything is NumPy on the
host and a pure function of the integer seeds given.

The workloads stand in, in shape only, for the graphs the paper evaluates on
(Table 1 / Table 6: node and edge counts, average degree; Fig. 7: long-tailed
degree distributions) with the (M, m) settings of Table 8 and App. D.3.  No
item of those datasets is reproduced here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "rmat_edges", "chung_lu_edges", "edges_to_csr",
    "make_graph", "uniform_tuples", "edge_nonedge_pairs", "make_queries",
    "csr_from_edge_list",
]


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration: graph recipe, walk parameters, query recipe."""
    name: str
    graph: str            # "rmat" | "chung_lu"
    n_nodes: int
    n_edges: int          # distinct undirected edges, no self-loops
    gamma: float          # Chung-Lu degree exponent (unused for rmat)
    M: int                # walks per seed
    m: int                # steps per walk
    n_queries: int
    k: int                # nodes per query (2 = pair, 3 = triple)
    query_kind: str       # "uniform" | "edge_nonedge"
    graph_seed: int = 1
    query_seed: int = 2
    rng_seed: int = 0


WORKLOADS = {
    "rmat4k": Workload("rmat4k", "rmat", 4096, 32768, 0.0, 50, 4, 1024, 2, "uniform"),
    "cl235k": Workload("cl235k", "chung_lu", 235_000, 1_300_000, 2.1, 200, 4, 65536, 2,
                       "edge_nonedge"),
    "rmat512k": Workload("rmat512k", "rmat", 1 << 19, 21_000_000, 0.0, 200, 3, 262144, 2,
                         "uniform"),
    "cl2900k": Workload("cl2900k", "chung_lu", 2_900_000, 30_000_000, 2.3, 100, 4,
                        1_048_576, 2, "edge_nonedge"),
    "cl1m_triples": Workload("cl1m_triples", "chung_lu", 1_000_000, 10_000_000, 2.2, 100, 3,
                             262144, 3, "uniform"),
}


# --------------------------------------------------------------------------- #
# edge samplers
# --------------------------------------------------------------------------- #
def _canon_keys(u: np.ndarray, v: np.ndarray, n: int) -> np.ndarray:
    """Drop self-loops, order each pair as (min, max) and pack into one int64 ``min*n+max``."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    keys = np.minimum(u, v)
    keys *= n
    keys += np.maximum(u, v)
    return keys[u != v]


def _top_up(draw, n: int, target: int, rng: np.random.Generator) -> np.ndarray:
    """Call ``draw(count)`` until exactly ``target`` distinct undirected edges exist.

    Returns the sorted int64 keys ``min*n + max``.
    """
    max_possible = n * (n - 1) // 2
    if target > max_possible:
        raise ValueError(f"{target} distinct edges do not fit in a {n}-node simple graph")
    keys = np.empty(0, dtype=np.int64)
    rounds = 0
    while keys.size < target:
        need = target - keys.size
        u, v = draw(int(need * 1.15) + 1024)
        keys = np.union1d(keys, _canon_keys(u, v, n))
        rounds += 1
        if rounds > 200:
            raise RuntimeError("edge sampler does not converge to the target count")
    if keys.size > target:
        drop = rng.choice(keys.size, size=keys.size - target, replace=False)
        mask = np.ones(keys.size, dtype=bool)
        mask[drop] = False
        keys = keys[mask]
    return keys


def rmat_edges(scale: int, n_edges: int, seed: int,
               abcd=(0.57, 0.19, 0.19, 0.05)) -> np.ndarray:
    """R-MAT: every edge picks one quadrant per address bit with probabilities a,b,c,d."""
    n = 1 << scale
    rng = np.random.default_rng(seed)
    a, b, c, _ = abcd

    def draw(count: int):
        u = np.zeros(count, dtype=np.int64)
        v = np.zeros(count, dtype=np.int64)
        for _bit in range(scale):
            r = rng.random(count, dtype=np.float32)
            row = r >= (a + b)                       # quadrants c, d: lower half
            col = ((r >= a) & (r < a + b)) | (r >= a + b + c)   # quadrants b, d: right half
            u = (u << 1) | row
            v = (v << 1) | col
        return u, v

    return _top_up(draw, n, n_edges, rng)


def _chung_lu_cdf(n: int, n_edges: int, gamma: float) -> np.ndarray:
    """Cumulative endpoint distribution for weights (i+i0)^(-1/(gamma-1)).

    ``i0`` is set by bisection so that the expected largest degree is about
    sqrt(2 * n_edges), which keeps the expected multi-edge count small.
    """
    alpha = 1.0 / (gamma - 1.0)
    idx = np.arange(n, dtype=np.float64)
    cap = np.sqrt(2.0 * n_edges)

    def max_deg(i0: float) -> float:
        w = (idx + i0) ** (-alpha)
        return 2.0 * n_edges * w[0] / w.sum()

    lo, hi = 1e-3, float(n)
    if max_deg(lo) <= cap:
        i0 = lo
    else:
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            if max_deg(mid) > cap:
                lo = mid
            else:
                hi = mid
        i0 = hi
    w = (idx + i0) ** (-alpha)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    return cdf


def chung_lu_edges(n: int, n_edges: int, gamma: float, seed: int) -> np.ndarray:
    """Chung-Lu: both endpoints of every edge drawn independently in proportion to a weight."""
    rng = np.random.default_rng(seed)
    cdf = _chung_lu_cdf(n, n_edges, gamma)

    def endpoints(count: int) -> np.ndarray:
        # Sorted uniforms make the cdf lookups sequential; the random pairing below
        # restores independence between the two endpoints of an edge.
        r = rng.random(count)
        r.sort()
        x = np.searchsorted(cdf, r, side="right")
        np.minimum(x, n - 1, out=x)
        return x

    def draw(count: int):
        u = endpoints(count)
        v = endpoints(count)
        return u, v[rng.permutation(count)]

    return _top_up(draw, n, n_edges, rng)


# --------------------------------------------------------------------------- #
# CSR assembly
# --------------------------------------------------------------------------- #
def edges_to_csr(keys: np.ndarray, n: int, perm: np.ndarray | None = None):
    """Symmetrise distinct undirected edges into an int32 CSR with ascending rows.

    ``keys`` are ``min*n + max``.  ``perm`` (optional) relabels node ``i`` as
    ``perm[i]`` first.  Returns ``(row_ptr int32[n+1], col_idx int32[2*len(keys)])``.
    """
    if 2 * keys.size >= 2 ** 31 or n >= 2 ** 31:
        raise ValueError("CSR does not fit int32 offsets")
    lo = keys // n
    hi = keys - lo * n
    if perm is not None:
        lo = perm[lo]
        hi = perm[hi]
    e = keys.size
    packed = np.empty(2 * e, dtype=np.int64)      # (src << 32) | dst, both directions
    packed[:e] = lo
    packed[e:] = hi
    packed <<= 32
    packed[:e] |= hi
    packed[e:] |= lo
    packed.sort()
    col_idx = (packed & 0xFFFFFFFF).astype(np.int32)
    packed >>= 32
    deg = np.bincount(packed, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=row_ptr[1:])
    return row_ptr.astype(np.int32), col_idx


def csr_from_edge_list(n: int, edges) -> tuple[np.ndarray, np.ndarray]:
    """CSR of a small hand-written undirected simple graph given as ``[(u, v), ...]``."""
    e = np.asarray(list(edges), dtype=np.int64).reshape(-1, 2)
    if e.size == 0:
        return np.zeros(n + 1, dtype=np.int32), np.zeros(0, dtype=np.int32)
    keys = np.unique(_canon_keys(e[:, 0], e[:, 1], n))
    return edges_to_csr(keys, n)


def make_graph(wl: Workload, permute: bool = True):
    """Build the CSR of a workload.  Node ids are randomly relabelled unless told otherwise."""
    if wl.graph == "rmat":
        scale = int(wl.n_nodes).bit_length() - 1
        if (1 << scale) != wl.n_nodes:
            raise ValueError("R-MAT needs a power-of-two node count")
        keys = rmat_edges(scale, wl.n_edges, wl.graph_seed)
    elif wl.graph == "chung_lu":
        keys = chung_lu_edges(wl.n_nodes, wl.n_edges, wl.gamma, wl.graph_seed)
    else:
        raise ValueError(wl.graph)
    perm = None
    if permute:
        perm = np.random.default_rng(wl.graph_seed + 7919).permutation(wl.n_nodes)
    return edges_to_csr(keys, wl.n_nodes, perm)


# --------------------------------------------------------------------------- #
# queries
# --------------------------------------------------------------------------- #
def uniform_tuples(n: int, count: int, k: int, seed: int) -> np.ndarray:
    """``count`` tuples of ``k`` pairwise distinct uniformly random node ids, int32[count][k]."""
    if n < k:
        raise ValueError("not enough nodes for distinct tuples")
    rng = np.random.default_rng(seed)
    out = rng.integers(0, n, size=(count, k), dtype=np.int64)
    while True:
        srt = np.sort(out, axis=1)
        bad = (srt[:, 1:] == srt[:, :-1]).any(axis=1)
        nb = int(bad.sum())
        if nb == 0:
            break
        out[bad] = rng.integers(0, n, size=(nb, k), dtype=np.int64)
    return out.astype(np.int32)


def _adjacent(row_ptr: np.ndarray, col_idx: np.ndarray, u: np.ndarray, v: np.ndarray):
    """Vectorised edge test: lower-bound bisection of ``v`` inside row ``u`` (rows ascend)."""
    lo = row_ptr[u].astype(np.int64)
    end = row_ptr[u + 1].astype(np.int64)
    hi = end.copy()
    while True:
        active = lo < hi
        if not active.any():
            break
        mid = (lo + hi) >> 1
        probe = col_idx[np.minimum(mid, col_idx.size - 1)]
        go_right = active & (probe < v)
        lo = np.where(go_right, mid + 1, lo)
        hi = np.where(active & ~go_right, mid, hi)
    found = lo < end
    return found & (col_idx[np.minimum(lo, col_idx.size - 1)] == v)


def edge_nonedge_pairs(row_ptr: np.ndarray, col_idx: np.ndarray, count: int,
                       seed: int) -> np.ndarray:
    """Half the pairs are existing edges (a uniformly chosen CSR entry), half are uniform
    distinct non-adjacent pairs; the two halves are shuffled together."""
    n = row_ptr.size - 1
    rng = np.random.default_rng(seed)
    n_pos = count // 2
    n_neg = count - n_pos
    e = rng.integers(0, col_idx.size, size=n_pos)
    pos_u = np.searchsorted(row_ptr, e, side="right") - 1
    pos_v = col_idx[e].astype(np.int64)
    neg = np.empty((0, 2), dtype=np.int64)
    while neg.shape[0] < n_neg:
        need = n_neg - neg.shape[0]
        cand = rng.integers(0, n, size=(need + need // 8 + 16, 2), dtype=np.int64)
        ok = cand[:, 0] != cand[:, 1]
        cand = cand[ok]
        ok = ~_adjacent(row_ptr, col_idx, cand[:, 0], cand[:, 1])
        neg = np.concatenate([neg, cand[ok]])[:n_neg]
    pairs = np.concatenate([np.stack([pos_u, pos_v], axis=1), neg])
    pairs = pairs[rng.permutation(pairs.shape[0])]
    return pairs.astype(np.int32)


def make_queries(wl: Workload, row_ptr: np.ndarray, col_idx: np.ndarray) -> np.ndarray:
    """Query tuples of a workload, int32[n_queries][k], entries are node ids."""
    if wl.query_kind == "uniform":
        return uniform_tuples(wl.n_nodes, wl.n_queries, wl.k, wl.query_seed)
    if wl.query_kind == "edge_nonedge":
        if wl.k != 2:
            raise ValueError("edge / non-edge queries are pairs")
        return edge_nonedge_pairs(row_ptr, col_idx, wl.n_queries, wl.query_seed)
    raise ValueError(wl.query_kind)
