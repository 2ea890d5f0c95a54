"""Seeded synthetic inputs shaped like the paper's workloads (Section V: a 169,343-node citation graph
with 1,166,243 edges and 128 features; a 2,449,029-node co-purchase graph with 61,859,140 edges and 100
features; random and low-cut equal-sized partitions, Appendix "Partitioning Details").

This module only *draws inputs*: graphs, node-to-partition maps, features, weights and upstream gradients.
It holds none of the method's arithmetic (no masks, no compression, no layer math, no halo indexing), so
both the CPU oracle's tests and the HIP path may be fed from it.

Everything is a pure function of its integer seed (numpy Philox streams), independent of thread count.
"""
from __future__ import annotations

import dataclasses
import math
import os

import numpy as np
import scipy.sparse as sp

# Seeds of the benchmark configurations.
SEED_GRAPH = 17611
SEED_PART = 17612
SEED_FEAT = 17613
SEED_WEIGHT = 17614
SEED_GRAD = 17615
MASK_KEY = 0x240617611


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


@dataclasses.dataclass
class Graph:
    """Global shift operator S as CSR (sorted columns), fp32 values, int64 rowptr, int32 colidx."""
    n: int
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    n_undirected: int          # undirected edges without self-loops
    self_loops: bool

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])


# --------------------------------------------------------------------------------------------------
# undirected edge lists
# --------------------------------------------------------------------------------------------------

def sbm_edges(block_sizes, p_in: float, p_out: float, seed: int) -> tuple[int, np.ndarray, np.ndarray]:
    """Stochastic block model: each unordered pair is an edge with prob. p_in (same block) or p_out."""
    n = int(sum(block_sizes))
    block = np.repeat(np.arange(len(block_sizes)), block_sizes)
    rng = _rng(seed)
    us, vs = [], []
    for i in range(n - 1):  # row-at-a-time keeps memory O(n); n is a few thousand here
        same = block[i + 1:] == block[i]
        p = np.where(same, p_in, p_out)
        hit = np.nonzero(rng.random(n - 1 - i) < p)[0]
        us.append(np.full(hit.shape, i, dtype=np.int64))
        vs.append(hit.astype(np.int64) + i + 1)
    return n, np.concatenate(us), np.concatenate(vs)          # u < v, sorted by (u, v)


def chung_lu_edges(n: int, n_edges: int, exponent: float, seed: int) -> tuple[np.ndarray, np.ndarray]:
    """Chung-Lu style power-law graph with exactly `n_edges` distinct undirected edges, no loops.

    Expected-degree weights w_i ~ (i+1)^(-1/(exponent-1)), scaled to sum 2*n_edges and capped at
    sqrt(2*n_edges) (so that w_u*w_v/sum(w) <= 1). Endpoints are drawn independently in proportion to w,
    loops and repeats are dropped, and the surplus is thinned uniformly to the exact edge count. Node
    ids are shuffled so that id order carries no degree information. Returned pairs have u < v and are
    sorted by (u, v).
    """
    rng = _rng(seed)
    alpha = 1.0 / (exponent - 1.0)
    w = (np.arange(n, dtype=np.float64) + 1.0) ** (-alpha)
    cap = math.sqrt(2.0 * n_edges)
    for _ in range(8):
        w *= (2.0 * n_edges) / w.sum()
        np.minimum(w, cap, out=w)
    prob = w / w.sum()
    relabel = rng.permutation(n).astype(np.int64)

    def endpoints(m: int) -> np.ndarray:
        # m independent draws in proportion to w, returned in ascending order: draw how often each node
        # is hit (one multinomial) instead of searching a cumulative table m times
        return np.repeat(np.arange(n, dtype=np.int64), rng.multinomial(m, prob))

    have = np.empty(0, dtype=np.int64)
    want = n_edges
    over = 1.12
    while have.shape[0] < want:
        m = int((want - have.shape[0]) * over) + 1024
        u = relabel[endpoints(m)]
        v = relabel[endpoints(m)[rng.permutation(m)]]     # random pairing of the two endpoint multisets
        keep = u != v
        u, v = u[keep], v[keep]
        key = np.minimum(u, v) * n + np.maximum(u, v)
        del u, v
        have = np.unique(key) if have.shape[0] == 0 else np.union1d(have, key)
        over *= 1.5
    if have.shape[0] > want:
        drop = rng.choice(have.shape[0], size=have.shape[0] - want, replace=False)
        mask = np.ones(have.shape[0], dtype=bool)
        mask[drop] = False
        have = have[mask]
    return have // n, have % n


# --------------------------------------------------------------------------------------------------
# shift operators
# --------------------------------------------------------------------------------------------------

def _symmetric_csr(n: int, u: np.ndarray, v: np.ndarray, self_loops: bool):
    """Pattern of A (+ I) as (rowptr int64, colidx int32) with ascending columns, from distinct
    undirected pairs u < v sorted by (u, v)."""
    m = u.shape[0]
    assert (u < v).all()
    up_cnt = np.bincount(u, minlength=n).astype(np.int64)          # entries (u -> v): columns above the row
    up_ptr = np.concatenate(([0], np.cumsum(up_cnt)))
    # entries (v -> u): transpose of the upper triangle by a counting sort (columns ascend within a row)
    lower = sp.csr_matrix((np.ones(m, dtype=np.int8), v.astype(np.int32), up_ptr), shape=(n, n)).tocsc()
    lo_ptr = lower.indptr.astype(np.int64)
    lo_cnt = np.diff(lo_ptr)
    self_cnt = 1 if self_loops else 0
    rowptr = np.concatenate(([0], np.cumsum(lo_cnt + self_cnt + up_cnt)))
    colidx = np.empty(int(rowptr[-1]), dtype=np.int32)
    dest = np.repeat(rowptr[:-1] - lo_ptr[:-1], lo_cnt) + np.arange(m, dtype=np.int64)
    colidx[dest] = lower.indices
    dest = np.repeat(rowptr[:-1] + lo_cnt + self_cnt - up_ptr[:-1], up_cnt) + np.arange(m, dtype=np.int64)
    colidx[dest] = v
    if self_loops:
        colidx[rowptr[:-1] + lo_cnt] = np.arange(n, dtype=np.int32)
    return rowptr, colidx


def gcn_operator(n: int, u: np.ndarray, v: np.ndarray) -> Graph:
    """S = D~^{-1/2} (A + I) D~^{-1/2}, degrees of the whole graph (self-loop included)."""
    rowptr, colidx = _symmetric_csr(n, u, v, self_loops=True)
    deg = np.diff(rowptr)
    dinv = 1.0 / np.sqrt(deg.astype(np.float64))
    vals = (np.repeat(dinv, deg) * dinv[colidx]).astype(np.float32)
    return Graph(n, rowptr, colidx, vals, int(u.shape[0]), True)


def sage_mean_operator(n: int, u: np.ndarray, v: np.ndarray) -> Graph:
    """S = D^{-1} A (mean over neighbours, no self-loop; isolated nodes have an empty row)."""
    rowptr, colidx = _symmetric_csr(n, u, v, self_loops=False)
    deg = np.diff(rowptr)
    with np.errstate(divide="ignore"):
        vals = np.repeat(1.0 / deg.astype(np.float64), deg).astype(np.float32)
    return Graph(n, rowptr, colidx, vals, int(u.shape[0]), False)


# --------------------------------------------------------------------------------------------------
# node -> partition maps (equal-sized parts, sizes differ by at most one)
# --------------------------------------------------------------------------------------------------

def _equal_chunks(order: np.ndarray, n_parts: int) -> np.ndarray:
    n = order.shape[0]
    part = np.empty(n, dtype=np.int32)
    bounds = (np.arange(n_parts + 1, dtype=np.int64) * n) // n_parts
    for q in range(n_parts):
        part[order[bounds[q]:bounds[q + 1]]] = q
    return part


def random_partition(n: int, n_parts: int, seed: int) -> np.ndarray:
    return _equal_chunks(_rng(seed).permutation(n), n_parts)


def block_partition(block_sizes) -> np.ndarray:
    return np.repeat(np.arange(len(block_sizes), dtype=np.int32), block_sizes)


def bfs_contiguous_partition(g: Graph, n_parts: int) -> np.ndarray:
    """Breadth-first visiting order (restarted at the lowest unvisited id), cut into equal chunks:
    a cheap low-cut stand-in for a min-cut partitioner."""
    n = g.n
    seen = np.zeros(n, dtype=bool)
    order = np.empty(n, dtype=np.int64)
    filled = 0
    next_root = 0
    while filled < n:
        while seen[next_root]:
            next_root += 1
        frontier = np.array([next_root], dtype=np.int64)
        seen[next_root] = True
        while frontier.shape[0]:
            order[filled:filled + frontier.shape[0]] = frontier
            filled += frontier.shape[0]
            starts = g.rowptr[frontier]
            lens = g.rowptr[frontier + 1] - starts
            total = int(lens.sum())
            if total == 0:
                break
            offs = np.repeat(starts - np.concatenate(([0], np.cumsum(lens)[:-1])), lens) + np.arange(total)
            nb = g.colidx[offs].astype(np.int64)
            nb = nb[~seen[nb]]
            # first occurrence order, deterministic
            _, first = np.unique(nb, return_index=True)
            frontier = nb[np.sort(first)]
            seen[frontier] = True
    return _equal_chunks(order, n_parts)


# --------------------------------------------------------------------------------------------------
# dense inputs
# --------------------------------------------------------------------------------------------------

_NORMAL_CHUNK_ROWS = 1 << 16


def _normal_rows(n: int, width: int, seed: int, salt: int) -> np.ndarray:
    """[n, width] i.i.d. N(0, 1) in fp32. Rows are drawn in fixed chunks, chunk c from the Philox stream keyed
    (seed, salt + c), so the values do not depend on how many threads fill the chunks."""
    out = np.empty((n, width), dtype=np.float32)
    starts = range(0, n, _NORMAL_CHUNK_ROWS)

    def fill(c_r0):
        c, r0 = c_r0
        r1 = min(n, r0 + _NORMAL_CHUNK_ROWS)
        _rng(seed, salt + c).standard_normal(out=out[r0:r1], dtype=np.float32)

    jobs = list(enumerate(starts))
    if len(jobs) <= 1:
        for j in jobs:
            fill(j)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            list(pool.map(fill, jobs))
    return out


def features(n: int, width: int, seed: int) -> np.ndarray:
    return _normal_rows(n, width, seed, 0)


def glorot(fan_in: int, fan_out: int, seed: int, stream: int = 0) -> np.ndarray:
    lim = math.sqrt(6.0 / (fan_in + fan_out))
    return ((_rng(seed, stream).random((fan_in, fan_out), dtype=np.float32) * 2.0 - 1.0) * lim).astype(np.float32)


def upstream_grad(n: int, width: int, seed: int) -> np.ndarray:
    out = _normal_rows(n, width, seed, 1 << 20)
    out /= np.float32(n)
    return out


# --------------------------------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------------------------------

@dataclasses.dataclass
class Workload:
    name: str
    graph: Graph
    part: np.ndarray
    n_parts: int
    conv: str                  # "gcn" | "sage"
    widths: tuple              # F_0 .. F_L
    ratios: tuple              # (num, den) pairs the configuration is run at
    dtype: str = "f32"


def _arxiv_like_edges():
    return chung_lu_edges(169_343, 1_166_243, 2.5, SEED_GRAPH)


def _products_like_edges():
    return chung_lu_edges(2_449_029, 61_859_140, 2.3, SEED_GRAPH)


def linear_schedule_config3(t: int) -> tuple[int, int]:
    """Ratio of the 16 -> 1 linear schedule over 100 steps as an exact rational (num, den)."""
    return 1584 - 15 * t, 99


@dataclasses.dataclass
class LabelledGraph:
    """A node-classification task on a synthetic graph: class labels, features that carry a weak class signal
    under unit noise (so that averaging over neighbours, i.e. communication, helps), and a train / test split."""
    graph: Graph
    part: np.ndarray
    n_parts: int
    conv: str
    widths: tuple
    features: np.ndarray       # [n, F_0] fp32
    labels: np.ndarray         # [n] int32 class ids
    train: np.ndarray          # [n] bool: node is used for training (the rest is held out)


def labelled_sbm(n_blocks: int = 4, block_size: int = 500, p_in: float = 0.02, p_out: float = 0.002, width: int = 16,
                 hidden: int = 32, signal: float = 0.35, n_parts: int = 4, conv: str = "sage",
                 seed: int = SEED_GRAPH + 100) -> LabelledGraph:
    """Stochastic block model whose blocks are the classes. Node features = signal * (a fixed random sign vector of
    the node's class) + N(0, 1) noise; nodes are dealt to `n_parts` equal random partitions (so most neighbours of
    a node live on other partitions); every second node (by a random permutation) is a training node."""
    sizes = (block_size,) * n_blocks
    n, u, v = sbm_edges(sizes, p_in, p_out, seed)
    g = sage_mean_operator(n, u, v) if conv == "sage" else gcn_operator(n, u, v)
    labels = np.repeat(np.arange(n_blocks, dtype=np.int32), block_size)
    rng = _rng(seed, 1)
    means = rng.integers(0, 2, size=(n_blocks, width)).astype(np.float32) * 2.0 - 1.0
    feats = (signal * means[labels] + _normal_rows(n, width, seed, 2)).astype(np.float32)
    train = np.zeros(n, dtype=bool)
    train[rng.permutation(n)[: n // 2]] = True
    return LabelledGraph(g, random_partition(n, n_parts, seed + 1), n_parts, conv, (width, hidden, n_blocks), feats,
                         labels, train)


def make_workload(name: str) -> Workload:
    if name == "tiny":
        sizes = (1000, 1000)
        n, u, v = sbm_edges(sizes, 0.01, 0.0005, SEED_GRAPH)
        g = gcn_operator(n, u, v)
        return Workload(name, g, block_partition(sizes), 2, "gcn", (16, 32, 8), ((4, 1),))
    if name == "medium":
        u, v = _arxiv_like_edges()
        g = gcn_operator(169_343, u, v)
        return Workload(name, g, random_partition(g.n, 4, SEED_PART), 4, "gcn", (128, 256, 256, 40),
                        ((1, 1), (2, 1), (4, 1), (8, 1), (16, 1)))
    if name == "medium_bfs16":
        u, v = _arxiv_like_edges()
        g = gcn_operator(169_343, u, v)
        return Workload(name, g, bfs_contiguous_partition(g, 16), 16, "gcn", (128, 256, 256, 40),
                        tuple(linear_schedule_config3(t) for t in range(100)))
    if name == "large_sage":
        u, v = _products_like_edges()
        g = sage_mean_operator(2_449_029, u, v)
        return Workload(name, g, random_partition(g.n, 8, SEED_PART), 8, "sage", (100, 256, 256, 47), ((8, 1),))
    if name == "large_gcn_bf16":
        u, v = _products_like_edges()
        g = gcn_operator(2_449_029, u, v)
        return Workload(name, g, random_partition(g.n, 32, SEED_PART), 32, "gcn", (100, 512, 512, 47),
                        ((1, 1), (4, 1), (32, 1)), dtype="bf16")
    # Evidence workloads (not configurations of the benchmark): the large graph's size, widths and ratio with a
    # different structure, to tell what the aggregation kernels' rates owe to the input's locality.
    if name == "large_sage_bfs8":        # the same graph, 8 contiguous chunks of a breadth-first order
        u, v = _products_like_edges()
        g = sage_mean_operator(2_449_029, u, v)
        return Workload(name, g, bfs_contiguous_partition(g, 8), 8, "sage", (100, 256, 256, 47), ((8, 1),))
    if name == "large_sage_banded8":     # every node linked to its 25 successors: 50 neighbours, all nearby; 8 id blocks
        n, band = 2_449_029, 25
        u = np.repeat(np.arange(n, dtype=np.int64), band)
        v = u + np.tile(np.arange(1, band + 1, dtype=np.int64), n)
        keep = v < n
        g = sage_mean_operator(n, u[keep], v[keep])
        return Workload(name, g, _equal_chunks(np.arange(n, dtype=np.int64), 8), 8, "sage", (100, 256, 256, 47), ((8, 1),))
    # The bf16 configuration's graph, widths and storage cut into 4 instead of 32 random parts: a quarter of the entries
    # local and a dozen entries per halo row, to show where the order of eq. (2)'s two products matters.
    if name == "large_gcn_bf16_p4":
        u, v = _products_like_edges()
        g = gcn_operator(2_449_029, u, v)
        return Workload(name, g, random_partition(g.n, 4, SEED_PART), 4, "gcn", (100, 512, 512, 47), ((4, 1),), dtype="bf16")
    raise ValueError(f"unknown workload {name!r}")


def small_random_graph(n: int, avg_deg: float, conv: str, seed: int) -> Graph:
    """Erdos-Renyi-like helper for unit tests (a few hundred nodes)."""
    rng = _rng(seed)
    m = int(n * avg_deg / 2)
    u = rng.integers(0, n, size=m * 2)
    v = rng.integers(0, n, size=m * 2)
    keep = u != v
    lo = np.minimum(u[keep], v[keep]).astype(np.int64)
    hi = np.maximum(u[keep], v[keep]).astype(np.int64)
    key = np.unique(lo * n + hi)[:m]
    u, v = key // n, key % n
    return gcn_operator(n, u, v) if conv == "gcn" else sage_mean_operator(n, u, v)
