"""Seeded synthetic inputs: graphs (as raw CSR patterns) and dense tensors.

This module produces *inputs only*.  It holds none of the method's arithmetic
(no self-loop insertion, no normalisation, no transpose, no layer maths): both
the fp64 oracle and the HIP path receive the arrays made here and do every
step of the method themselves.  It depends on NumPy alone, so it can be
imported without the HIP library and without the oracle.

The graphs stand in for the citation / social graphs of the paper's
evaluation (Table "Graph datasets used in this work"): an Erdos-Renyi G(n, M)
graph at Cora scale and R-MAT graphs with the skewed degree distribution
(hubs) that the paper's discussion of the CSR format singles out as the hard
case for GPUs (App. D.1).

Conventions
-----------
* A pattern is returned as ``(rowptr[int32, n+1], col[int32, q])`` with the
  column indices of every row strictly ascending, no duplicate entries and
  **no diagonal** (self-loops are a step of the method, not of the input).
* Row i of the pattern lists the nodes j that node i aggregates from.  For the
  undirected graphs the pattern is symmetric; for the directed GAT graph a
  sampled arc u -> v becomes the entry (row v, column u).
* All randomness comes from ``numpy.random.Generator(PCG64)`` streams spawned
  from one root seed in the fixed order given by ``STREAMS``.
"""
from __future__ import annotations

import dataclasses
import numpy as np

STREAMS = ("graph", "X", "W", "dY", "a_src", "a_dst", "labels", "relabel", "W2", "b")


def streams(seed: int) -> dict:
    """One independent generator per named stream, spawned in a fixed order."""
    kids = np.random.SeedSequence(seed).spawn(len(STREAMS))
    return {name: np.random.Generator(np.random.PCG64(k)) for name, k in zip(STREAMS, kids)}


def substream(seed: int, name: str, index: int) -> np.random.Generator:
    """Generator number ``index`` below the named stream (same tree as ``streams``)."""
    ss = np.random.SeedSequence(seed, spawn_key=(STREAMS.index(name), index))
    return np.random.Generator(np.random.PCG64(ss))


# --------------------------------------------------------------------------
# graphs
# --------------------------------------------------------------------------
def coo_to_csr(n: int, row: np.ndarray, col: np.ndarray):
    """Sort (row, col) pairs, drop duplicates and diagonal entries -> CSR pattern."""
    row = np.asarray(row, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    keep = row != col
    key = row[keep] * np.int64(n) + col[keep]
    del row, col, keep
    key = np.unique(key)                       # sorted, deduplicated
    r = (key // n).astype(np.int32)
    c = (key % n).astype(np.int32)
    del key
    counts = np.bincount(r, minlength=n)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2**31
    return rowptr.astype(np.int32), c


def erdos_renyi_gnm(n: int, m_pairs: int, rng: np.random.Generator):
    """G(n, M): exactly ``m_pairs`` distinct unordered pairs {i, j}, i != j, symmetrised."""
    total = n * (n - 1) // 2
    assert 0 <= m_pairs <= total
    chosen = np.empty(0, dtype=np.int64)
    while chosen.size < m_pairs:               # rejection on duplicates, order-preserving
        need = m_pairs - chosen.size
        draw = rng.integers(0, total, size=need + need // 8 + 16, dtype=np.int64)
        chosen = np.concatenate([chosen, draw])
        _, first = np.unique(chosen, return_index=True)
        chosen = chosen[np.sort(first)][:m_pairs]
    # unrank pair index p -> (i, j) with i > j : p = i(i-1)/2 + j
    i = np.floor((1.0 + np.sqrt(1.0 + 8.0 * chosen.astype(np.float64))) / 2.0).astype(np.int64)
    i = np.where(i * (i - 1) // 2 > chosen, i - 1, i)
    i = np.where((i + 1) * i // 2 <= chosen, i + 1, i)
    j = chosen - i * (i - 1) // 2
    assert np.all((0 <= j) & (j < i) & (i < n))
    return coo_to_csr(n, np.concatenate([i, j]), np.concatenate([j, i]))


def rmat_arcs(scale: int, n_samples: int, rng: np.random.Generator,
              a=0.57, b=0.19, c=0.19, d=0.05, chunk=1 << 24):
    """Sample ``n_samples`` arcs (u, v) of an R-MAT graph on 2**scale nodes."""
    assert abs(a + b + c + d - 1.0) < 1e-12
    u = np.zeros(n_samples, dtype=np.int32)
    v = np.zeros(n_samples, dtype=np.int32)
    for lo in range(0, n_samples, chunk):
        hi = min(n_samples, lo + chunk)
        uu = np.zeros(hi - lo, dtype=np.int32)
        vv = np.zeros(hi - lo, dtype=np.int32)
        for _ in range(scale):
            r = rng.random(hi - lo, dtype=np.float32)
            ubit = r >= np.float32(a + b)                       # quadrants c, d
            vbit = ((r >= np.float32(a)) & ~ubit) | (r >= np.float32(a + b + c))
            uu = (uu << 1) | ubit
            vv = (vv << 1) | vbit
        u[lo:hi] = uu
        v[lo:hi] = vv
    return u, v


def rmat_graph(scale: int, avg_degree: int, directed: bool, rng_graph, rng_relabel):
    """R-MAT pattern with ``avg_degree`` directed entries per node before dedup.

    Undirected: n*avg_degree/2 samples, each stored in both directions.
    Directed:   n*avg_degree samples, arc u -> v stored as entry (v, u).
    A seeded random relabelling spreads the hubs over the id range.
    """
    n = 1 << scale
    n_samples = n * avg_degree if directed else n * avg_degree // 2
    u, v = rmat_arcs(scale, n_samples, rng_graph)
    relabel = rng_relabel.permutation(n).astype(np.int32)
    u = relabel[u]
    v = relabel[v]
    if directed:
        return coo_to_csr(n, v, u)
    return coo_to_csr(n, np.concatenate([u, v]), np.concatenate([v, u]))


def random_directed_graph(n: int, q: int, rng: np.random.Generator, allow_diagonal=False):
    """Small uniformly random directed pattern for unit tests (about q entries)."""
    r = rng.integers(0, n, size=q)
    c = rng.integers(0, n, size=q)
    if allow_diagonal:
        key = np.unique(r.astype(np.int64) * n + c)
        rr = (key // n).astype(np.int32)
        counts = np.bincount(rr, minlength=n)
        rowptr = np.zeros(n + 1, dtype=np.int32)
        rowptr[1:] = np.cumsum(counts)
        return rowptr, (key % n).astype(np.int32)
    return coo_to_csr(n, r, c)


# --------------------------------------------------------------------------
# dense tensors
# --------------------------------------------------------------------------
def normal(rng, *shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def glorot_uniform(rng, shape, fan_in: int, fan_out: int) -> np.ndarray:
    lim = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-lim, lim, size=shape).astype(np.float32)


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    name: str
    kind: str                  # "gcn" | "gcn2" | "gat"
    n: int
    rowptr: np.ndarray         # raw pattern, no diagonal
    col: np.ndarray
    tensors: dict              # name -> float32 / int32 arrays
    dims: dict                 # f_in, f_out (list for sweeps), heads, ...


def _graph(kind, seed, **kw):
    s = streams(seed)
    if kind == "er":
        return erdos_renyi_gnm(kw["n"], kw["pairs"], s["graph"]), s
    return rmat_graph(kw["scale"], kw["avg_degree"], kw.get("directed", False),
                      s["graph"], s["relabel"]), s


def gcn_single(name, graph_kind, f_in, f_outs, seed=0, **gkw) -> Workload:
    (rowptr, col), s = _graph(graph_kind, seed, **gkw)
    n = rowptr.size - 1
    k_max = max(f_outs)
    t = {"X": normal(s["X"], n, f_in)}
    # one W / dY draw per F_out, each from its own child stream so that the
    # arrays for one F_out do not depend on which others are requested
    for k in f_outs:
        t[f"W{k}"] = glorot_uniform(substream(seed, "W", k), (f_in, k), f_in, k)
        t[f"dY{k}"] = normal(substream(seed, "dY", k), n, k)
        t[f"b{k}"] = normal(substream(seed, "b", k), k)
    return Workload(name, "gcn", n, rowptr, col, t, {"f_in": f_in, "f_outs": list(f_outs), "k_max": k_max})


def config1(seed=0):
    return gcn_single("cfg1-er2048", "er", 512, [16], seed, n=2048, pairs=8192)


def config2(seed=0, scale=17, avg_degree=14, f_in=128, f_outs=(16, 128, 512)):
    return gcn_single(f"cfg2-rmat{scale}", "rmat", f_in, f_outs, seed, scale=scale, avg_degree=avg_degree)


def config5(seed=0, scale=22, avg_degree=32, f_in=64, f_outs=(64, 256)):
    return gcn_single(f"cfg5-rmat{scale}", "rmat", f_in, f_outs, seed, scale=scale, avg_degree=avg_degree)


def config3(seed=0, scale=20, avg_degree=50, dims=(100, 256, 47)) -> Workload:
    (rowptr, col), s = _graph("rmat", seed, scale=scale, avg_degree=avg_degree)
    n = rowptr.size - 1
    f0, f1, f2 = dims
    t = {
        "X": normal(s["X"], n, f0),
        "W1": glorot_uniform(s["W"], (f0, f1), f0, f1),
        "W2": glorot_uniform(s["W2"], (f1, f2), f1, f2),
        "labels": s["labels"].integers(0, f2, size=n, dtype=np.int32),
    }
    return Workload(f"cfg3-rmat{scale}", "gcn2", n, rowptr, col, t, {"dims": list(dims)})


def config4(seed=0, scale=17, avg_degree=14, f_in=256, heads=8, f_out=8) -> Workload:
    (rowptr, col), s = _graph("rmat", seed, scale=scale, avg_degree=avg_degree, directed=True)
    n = rowptr.size - 1
    hk = heads * f_out
    t = {
        "X": normal(s["X"], n, f_in),
        "W": glorot_uniform(s["W"], (f_in, hk), f_in, hk),
        "a_src": glorot_uniform(s["a_src"], (heads, f_out), heads, f_out),
        "a_dst": glorot_uniform(s["a_dst"], (heads, f_out), heads, f_out),
        "b": normal(s["b"], hk),
        "dY": normal(s["dY"], n, hk),
    }
    return Workload(f"cfg4-rmat{scale}", "gat", n, rowptr, col, t,
                    {"f_in": f_in, "heads": heads, "f_out": f_out, "slope": 0.2})
