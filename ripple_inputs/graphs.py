"""Seeded directed Chung-Lu power-law graphs, feature matrices and the five
workload configurations.

Degree law: rank r in [0, N) carries weight proportional to
(r + i0)^(-1/(gamma-1)); the discrete probability of rank r is the integral of
that density over [r, r+1), so ranks are drawn exactly by inverting the
continuous CDF and taking the floor. Out-ranks and in-ranks are mapped to
vertex ids through two independent seeded permutations. i0 is found by
bisection so that the heaviest rank expects a given share of all edges (hubs
exist but do not saturate).
"""
from __future__ import annotations

import dataclasses
import numpy as np

OP_EDGE_ADD, OP_EDGE_DEL, OP_VERTEX_ADD, OP_VERTEX_DEL, OP_FEAT_UPDATE, OP_EDGE_REWEIGHT = 0, 1, 2, 3, 4, 5


class PowerLaw:
    """Sampler for one side (out or in) of the Chung-Lu degree law."""

    def __init__(self, n: int, gamma: float, top_share: float, perm_seed: int):
        self.n = int(n)
        self.a = 1.0 / (gamma - 1.0)
        self.e = 1.0 - self.a                      # exponent of the antiderivative
        self.i0 = self._solve_i0(top_share)
        self.lo = self.i0 ** self.e
        self.hi = (self.n + self.i0) ** self.e
        self.perm = np.random.default_rng(perm_seed).permutation(self.n).astype(np.int64)

    def _p0(self, i0: float) -> float:
        lo, hi = i0 ** self.e, (self.n + i0) ** self.e
        return ((1.0 + i0) ** self.e - lo) / (hi - lo)

    def _solve_i0(self, top_share: float) -> float:
        lo, hi = 1e-9, float(self.n)              # p0 decreases as i0 grows
        if self._p0(lo) <= top_share:
            return lo
        for _ in range(200):
            mid = np.sqrt(lo * hi)
            if self._p0(mid) > top_share:
                lo = mid
            else:
                hi = mid
        return float(np.sqrt(lo * hi))

    def _ranks(self, u: np.ndarray) -> np.ndarray:
        x = (u * (self.hi - self.lo) + self.lo) ** (1.0 / self.e) - self.i0
        r = np.floor(x).astype(np.int64)
        np.maximum(r, 0, out=r)
        np.minimum(r, self.n - 1, out=r)
        return r

    def draw(self, rng: np.random.Generator, size: int) -> np.ndarray:
        return self.perm[self._ranks(rng.random(size))]

    def same_shape(self, other: "PowerLaw") -> bool:
        return (self.n, self.e, self.i0, self.lo, self.hi) == (other.n, other.e, other.i0, other.lo, other.hi)


def draw_pair(rng: np.random.Generator, first: PowerLaw, second: PowerLaw, size: int):
    """The values of first.draw(rng, size) followed by second.draw(rng, size). Two laws of one shape
    (they differ in their permutation only) share one pass over 2*size uniforms, which saves most of
    the per-call overhead when size is small."""
    if not first.same_shape(second):
        return first.draw(rng, size), second.draw(rng, size)
    r = first._ranks(rng.random(2 * size))
    return first.perm[r[:size]], second.perm[r[size:]]


def degree_laws(n: int, gamma: float, top_share: float, seed: int):
    """The out- and in-degree samplers of the graph with this seed."""
    return PowerLaw(n, gamma, top_share, seed * 7 + 1), PowerLaw(n, gamma, top_share, seed * 7 + 2)


def chung_lu_graph(n: int, e: int, gamma: float, top_share: float, seed: int):
    """Exactly `e` distinct directed edges without self-loops.

    Returns (src, dst, out_law, in_law): uint32 arrays sorted by (src, dst)
    and the two samplers (the update stream draws new edges from the same law).
    """
    out_law, in_law = degree_laws(n, gamma, top_share, seed)
    rng = np.random.default_rng(seed)
    keys = np.empty(0, dtype=np.int64)
    while keys.size < e:
        need = e - keys.size
        m = int(need * 1.15) + 1024
        s = out_law.draw(rng, m)
        d = in_law.draw(rng, m)
        ok = s != d
        k = s[ok] * n + d[ok]
        k = np.unique(k)                           # sorted, distinct inside the draw
        if keys.size:
            k = k[~np.isin(k, keys, assume_unique=True)]
        if k.size > need:                          # unbiased trim of the surplus
            k = rng.permutation(k)[:need]
        keys = np.union1d(keys, k)
    src = (keys // n).astype(np.uint32)
    dst = (keys % n).astype(np.uint32)
    return src, dst, out_law, in_law


def features(n: int, d: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).standard_normal((n, d), dtype=np.float32)


def edge_weights(e: int, seed: int) -> np.ndarray:
    """Per-edge weights for the weighted-sum workload: uniform in [0.25, 1.75), float32."""
    return np.random.default_rng(seed).uniform(0.25, 1.75, e).astype(np.float32)


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    n: int
    e: int
    gamma: float
    top_share: float            # expected share of all edges at the heaviest rank
    d0: int
    model: str                  # 'gcn_sum' | 'sage_mean' | 'gin_sum'
    widths: tuple               # d_0 .. d_L
    store: str                  # 'f32' | 'bf16'
    batch_sizes: tuple
    mix: dict                   # fractions of logical updates per kind
    vertex_slack: int           # ids reserved for vertex additions
    graph_seed: int = 12347
    feat_seed: int = 12348
    weight_seed: int = 12349
    stream_seed: int = 12350
    weighted: bool = False      # per-edge weights (weighted-sum workloads), seed = graph_seed + 100

    @property
    def vertex_capacity(self) -> int:
        return self.n + self.vertex_slack

    @property
    def edge_capacity(self) -> int:
        return int(self.e * 1.05) + 9 * self.vertex_slack + 65536


_MIX3 = {"edge_add": 0.5, "edge_del": 0.3, "feat": 0.2, "vadd": 0.0, "vdel": 0.0}


def _mix_with_vertex_ops(vadd: float, vdel: float) -> dict:
    rest = 1.0 - vadd - vdel
    return {"edge_add": 0.5 * rest, "edge_del": 0.3 * rest, "feat": 0.2 * rest,
            "vadd": vadd, "vdel": vdel}


CONFIGS = [
    Config("tiny_gcn_sum", 2_000, 20_000, 2.1, 0.015, 32, "gcn_sum",
           (32, 64, 16), "f32", (100,), _MIX3, 4096, stream_seed=12350),
    Config("sparse_sage_mean", 169_343, 1_166_243, 2.1, 0.01, 128, "sage_mean",
           (128, 256, 256, 40), "f32", (1, 10, 100, 1000), _MIX3, 4096, stream_seed=12351),
    Config("sparse_gin_sum", 169_343, 1_166_243, 2.1, 0.01, 128, "gin_sum",
           (128, 256, 256, 40), "f32", (1000,), _mix_with_vertex_ops(0.05, 0.05),
           1 << 17, stream_seed=12352),
    Config("dense_sage_mean", 2_449_029, 123_718_280, 2.3, 0.0002, 100, "sage_mean",
           (100, 256, 256, 47), "f32", (100, 1000, 10000), _MIX3, 4096, stream_seed=12353),
    Config("dense_gcn_sum_bf16", 2_449_029, 123_718_280, 2.3, 0.0002, 100, "gcn_sum",
           (100, 256, 256, 47), "bf16", (10000,), _mix_with_vertex_ops(0.01, 0.01),
           1 << 17, stream_seed=12354),
    # beyond the five of the scope table: the paper's GC-W workload (GraphConv with weighted sum) on the
    # sparse and dense graphs
    Config("sparse_gcn_wsum", 169_343, 1_166_243, 2.1, 0.01, 128, "gcn_wsum",
           (128, 256, 256, 40), "f32", (1000,), _MIX3, 4096, stream_seed=12355, weighted=True),
    Config("dense_gcn_wsum", 2_449_029, 123_718_280, 2.3, 0.0002, 100, "gcn_wsum",
           (100, 256, 256, 47), "f32", (10000,), _MIX3, 4096, stream_seed=12356, weighted=True),
    # the paper's GC-X workload (GraphConv with max aggregation)
    Config("sparse_gcn_max", 169_343, 1_166_243, 2.1, 0.01, 128, "gcn_max",
           (128, 256, 256, 40), "f32", (1000,), _MIX3, 4096, stream_seed=12357),
    Config("dense_gcn_max", 2_449_029, 123_718_280, 2.3, 0.0002, 100, "gcn_max",
           (100, 256, 256, 47), "f32", (10000,), _MIX3, 4096, stream_seed=12358),
    # deeper models (the paper's 4-layer runs, Sec. 6.3.2) and a graph of Reddit's shape (Table 2: 233 K
    # vertices, 114.6 M edges, 602 features, 41 classes; average in-degree 492)
    Config("sparse_sage_mean_4layer", 169_343, 1_166_243, 2.1, 0.01, 128, "sage_mean",
           (128, 256, 256, 256, 40), "f32", (1000,), _MIX3, 4096, stream_seed=12359),
    Config("dense_sage_mean_4layer", 2_449_029, 123_718_280, 2.3, 0.0002, 100, "sage_mean",
           (100, 256, 256, 256, 47), "f32", (1000,), _MIX3, 4096, stream_seed=12360),
    Config("reddit_sage_mean", 232_965, 114_615_892, 2.3, 0.0002, 602, "sage_mean",
           (602, 256, 256, 41), "f32", (100, 1000), _MIX3, 4096, stream_seed=12361),
    # the paper's GA-A workload (graph attention)
    Config("sparse_gat", 169_343, 1_166_243, 2.1, 0.01, 128, "gat",
           (128, 256, 256, 40), "f32", (1000,), _MIX3, 4096, stream_seed=12362),
    Config("dense_gat", 2_449_029, 123_718_280, 2.3, 0.0002, 100, "gat",
           (100, 256, 256, 47), "f32", (10000,), _MIX3, 4096, stream_seed=12363),
]


def get_config(name_or_index) -> Config:
    if isinstance(name_or_index, int):
        return CONFIGS[name_or_index]
    for c in CONFIGS:
        if c.name == name_or_index:
            return c
    raise KeyError(name_or_index)
