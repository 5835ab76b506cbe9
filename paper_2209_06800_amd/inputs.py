"""Seeded synthetic inputs: graphs, node-range bounds, features and weights.

This module holds no part of the method's arithmetic (no partitioning, no
aggregation, no normalisation, no GEMM).  It only draws graphs and tensors that
have the shapes, degree distributions and value distributions of the paper's
workloads (Table 1 / section 7 "Benchmarks & Datasets"), so that the CPU oracle
and the HIP path can be fed the very same arrays.  It imports neither of them.

Graph convention used by everything downstream: a *canonical CSR* -- undirected
(both directions stored), no self-loops, no duplicate edges, column ids sorted
ascending inside each row; ``row_ptr`` is int64[N+1], ``col`` is int32[nnz].

The real datasets (reddit, ogbn-products) are not available; ``config(4)`` and
``config(5)`` are seeded stand-ins with the same node count, edge count and
feature width as the corresponding rows of the paper's Table 1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 220906800


# --------------------------------------------------------------------------- #
# graph canonicalisation
# --------------------------------------------------------------------------- #
def canonical_csr(n: int, src: np.ndarray, dst: np.ndarray):
    """Symmetrise, drop self-loops and duplicates, sort -> (row_ptr i64, col i32)."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    key = np.concatenate([src * n + dst, dst * n + src])
    del src, dst
    key.sort(kind="stable")
    if key.size:
        uniq = np.empty(key.size, dtype=bool)
        uniq[0] = True
        np.not_equal(key[1:], key[:-1], out=uniq[1:])
        key = key[uniq]
    rows = key // n
    col = (key - rows * n).astype(np.int32)
    counts = np.bincount(rows, minlength=n).astype(np.int64)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    return row_ptr, col


def csr_from_adjacency_lists(adj: List[List[int]]):
    """Tiny helper for hand-written graphs in tests (rows kept as given)."""
    row_ptr = np.zeros(len(adj) + 1, dtype=np.int64)
    for i, a in enumerate(adj):
        row_ptr[i + 1] = row_ptr[i] + len(a)
    col = np.array([u for a in adj for u in a], dtype=np.int32)
    return row_ptr, col


# --------------------------------------------------------------------------- #
# graph generators
# --------------------------------------------------------------------------- #
def erdos_renyi_gnm(n: int, m: int, rng: np.random.Generator):
    """G(n, m): m distinct undirected pairs (no self-loops) -> canonical CSR."""
    have = np.empty(0, dtype=np.int64)
    while have.size < m:
        need = m - have.size
        a = rng.integers(0, n, size=need + need // 8 + 16, dtype=np.int64)
        b = rng.integers(0, n, size=a.size, dtype=np.int64)
        ok = a != b
        lo = np.minimum(a[ok], b[ok])
        hi = np.maximum(a[ok], b[ok])
        have = np.unique(np.concatenate([have, lo * n + hi]))
    if have.size > m:
        # drop a seeded random subset so exactly m pairs remain
        have = have[np.sort(rng.permutation(have.size)[:m])]
    return canonical_csr(n, have // n, have % n)


def rmat_pairs(scale: int, n_draws: int, a: float, b: float, c: float, d: float,
               rng: np.random.Generator, n_limit: Optional[int] = None,
               chunk: int = 1 << 23):
    """Plain R-MAT endpoint pairs (no noise, no vertex relabelling).

    Each of the ``scale`` bit levels picks one of the four quadrants with
    probabilities (a, b, c, d).  With ``n_limit`` pairs that have an endpoint
    >= n_limit are rejected and redrawn until ``n_draws`` pairs exist.
    """
    assert abs(a + b + c + d - 1.0) < 1e-9
    srcs, dsts, have = [], [], 0
    while have < n_draws:
        k = min(chunk, int((n_draws - have) * (1.3 if n_limit is not None else 1.0)) + 1024)
        s = np.zeros(k, dtype=np.int64)
        t = np.zeros(k, dtype=np.int64)
        for _ in range(scale):
            r = rng.random(k, dtype=np.float32)
            sbit = r >= np.float32(a + b)            # quadrants c, d -> source bit 1
            tbit = ((r >= np.float32(a)) & (r < np.float32(a + b))) | \
                   (r >= np.float32(a + b + c))      # quadrants b, d -> target bit 1
            s = (s << 1) | sbit
            t = (t << 1) | tbit
        if n_limit is not None:
            ok = (s < n_limit) & (t < n_limit)
            s, t = s[ok], t[ok]
        take = min(s.size, n_draws - have)
        srcs.append(s[:take])
        dsts.append(t[:take])
        have += take
    return np.concatenate(srcs), np.concatenate(dsts)


def rmat_graph(scale, n_draws, a, b, c, d, rng, n_nodes=None):
    n = (1 << scale) if n_nodes is None else n_nodes
    s, t = rmat_pairs(scale, n_draws, a, b, c, d, rng,
                      n_limit=None if n_nodes is None else n_nodes)
    return canonical_csr(n, s, t)


def chung_lu_pareto(n: int, alpha: float, d_min: float, d_max: float,
                    rng: np.random.Generator, chunk: int = 1 << 24):
    """Chung-Lu graph on truncated-Pareto expected degrees, node ids in random order.

    The density of w_v falls as w^-alpha (a Zipf-like degree law with exponent alpha), i.e.
    the tail P(w > t) falls as t^-(alpha-1); truncated to [d_min, d_max], inverse-CDF sampling.
    m = sum(w)/2 endpoint pairs are drawn with probability proportional to w.
    """
    u = rng.random(n)
    a = alpha - 1.0
    lo, hi = d_min ** (-a), d_max ** (-a)
    w = (lo - u * (lo - hi)) ** (-1.0 / a)
    m = int(w.sum() / 2)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    srcs, dsts, have = [], [], 0
    while have < m:
        k = min(chunk, m - have)
        s = np.searchsorted(cdf, rng.random(k), side="right")
        t = np.searchsorted(cdf, rng.random(k), side="right")
        srcs.append(np.minimum(s, n - 1).astype(np.int32))
        dsts.append(np.minimum(t, n - 1).astype(np.int32))
        have += k
    return canonical_csr(n, np.concatenate(srcs), np.concatenate(dsts))


# --------------------------------------------------------------------------- #
# tensors
# --------------------------------------------------------------------------- #
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(shape, rng: np.random.Generator, std: float = 1.0, chunk_rows: int = 1 << 18):
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(-1, 1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        flat[r0:r1] = rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def uniform_f32(shape, rng: np.random.Generator, lo=-1.0, hi=1.0):
    return (rng.random(shape, dtype=np.float32) * np.float32(hi - lo) + np.float32(lo))


def equal_node_bounds(n: int, parts: int) -> np.ndarray:
    """Contiguous equal-node split: bounds[p] = floor(n*p/parts)."""
    return np.array([(n * p) // parts for p in range(parts + 1)], dtype=np.int64)


# --------------------------------------------------------------------------- #
# the five configurations (and scaled-down versions with the same structure)
# --------------------------------------------------------------------------- #
@dataclass
class Layer:
    mode: str                      # "gcn" | "gin"
    eps: float
    weights: List[np.ndarray]      # each [d_in, d_out]; fp32, or uint16 bf16 bits
    acts: List[str]                # per linear: "relu" | "none"
    dims: List[int]                # [d_in, d_hidden..., d_out]


@dataclass
class Workload:
    name: str
    cfg: int
    n: int
    row_ptr: np.ndarray
    col: np.ndarray
    parts: int
    part_id: int
    bounds: np.ndarray
    dtype: str                     # "f32" | "bf16" (storage type of features and weights)
    x: np.ndarray                  # [n, dim] fp32, or uint16 bf16 bits
    layers: List[Layer]
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def dim(self) -> int:
        return int(self.x.shape[1])

    @property
    def lb(self) -> int:
        return int(self.bounds[self.part_id])

    @property
    def ub(self) -> int:
        return int(self.bounds[self.part_id + 1])


def _weights(d_in, d_out, rng, dtype):
    w = normal_f32((d_in, d_out), rng, std=0.1)
    return to_bf16_bits(w) if dtype == "bf16" else w


def config(cfg: int, shrink: int = 0) -> Workload:
    """Build configuration ``cfg`` (1..5).  ``shrink`` = k divides the node count by
    2**k while keeping generator parameters, average degree, partition count, feature
    width and layer shapes, for parity tests the oracle finishes in seconds."""
    rng = np.random.default_rng(np.random.PCG64(BASE_SEED + cfg + 1000 * shrink))
    if cfg == 1:
        n = 4096 >> shrink
        row_ptr, col = erdos_renyi_gnm(n, n * 8, rng)
        x = uniform_f32((n, 16), rng)
        layers = [Layer("gcn", 0.0, [_weights(16, 16, rng, "f32")], ["relu"], [16, 16])]
        return Workload("cfg1_er4096_gcn16", 1, n, row_ptr, col, 1, 0,
                        equal_node_bounds(n, 1), "f32", x, layers)
    if cfg == 2:
        scale = 20 - shrink
        n = 1 << scale
        row_ptr, col = rmat_graph(scale, n * 16, 0.57, 0.19, 0.19, 0.05, rng)
        x = normal_f32((n, 64), rng)
        layers = [Layer("gcn", 0.0, [_weights(64, 64, rng, "f32")], ["relu"], [64, 64])]
        return Workload("cfg2_rmat20_gcn64_p4", 2, n, row_ptr, col, 4, 0,
                        equal_node_bounds(n, 4), "f32", x, layers)
    if cfg == 3:
        scale = 22 - shrink
        n = 1 << scale
        row_ptr, col = rmat_graph(scale, n * 8, 0.57, 0.19, 0.19, 0.05, rng)
        x = to_bf16_bits(normal_f32((n, 128), rng))
        layers = [Layer("gin", 0.0,
                        [_weights(128, 128, rng, "bf16"), _weights(128, 128, rng, "bf16")],
                        ["relu", "none"], [128, 128, 128])]
        return Workload("cfg3_rmat22_gin128_bf16_p8", 3, n, row_ptr, col, 8, 0,
                        equal_node_bounds(n, 8), "bf16", x, layers)
    if cfg == 4:
        n = 232965 >> shrink
        # expected degrees keep the paper-scale floor; the cap follows the node count
        row_ptr, col = chung_lu_pareto(n, 2.1, 115.5, float(min(20000, n // 8)), rng)
        x = normal_f32((n, 602), rng)
        layers = [Layer("gcn", 0.0, [_weights(602, 256, rng, "f32")], ["relu"], [602, 256])]
        return Workload("cfg4_powerlaw233k_gcn602", 4, n, row_ptr, col, 1, 0,
                        equal_node_bounds(n, 1), "f32", x, layers)
    if cfg == 5:
        scale = 22 - shrink
        n = 2449029 >> shrink
        row_ptr, col = rmat_graph(scale, 61859140 >> shrink, 0.45, 0.22, 0.22, 0.11, rng,
                                  n_nodes=n)
        x = normal_f32((n, 100), rng)
        layers = [Layer("gcn", 0.0, [_weights(100, 256, rng, "f32")], ["relu"], [100, 256]),
                  Layer("gcn", 0.0, [_weights(256, 47, rng, "f32")], ["none"], [256, 47])]
        return Workload("cfg5_rmat2.4M_gcn2layer_p8", 5, n, row_ptr, col, 8, 0,
                        equal_node_bounds(n, 8), "f32", x, layers,
                        notes={"layer2_halo_seed": BASE_SEED + 50 + 1000 * shrink})
    raise ValueError(f"unknown config {cfg}")


def layer2_halo_table(seed: int, num_halo: int, dim: int) -> np.ndarray:
    """Synthetic stand-in for other partitions' layer-1 output: ReLU(N(0,1))."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    t = normal_f32((num_halo, dim), rng)
    np.maximum(t, 0.0, out=t)
    return t


def graph_stats(row_ptr: np.ndarray) -> Dict[str, float]:
    deg = np.diff(row_ptr)
    return {"n": int(deg.size), "nnz": int(row_ptr[-1]), "avg_deg": float(deg.mean()) if deg.size else 0.0,
            "max_deg": int(deg.max()) if deg.size else 0, "isolated": int((deg == 0).sum())}
