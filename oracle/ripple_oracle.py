"""CPU oracle for incremental GNN inference on an evolving graph (fp64).

TEST INFRASTRUCTURE ONLY. This file is the slow, plain statement of what the
GPU library must compute. Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does, and this file
imports nothing from the product.

What it computes. The paper states that its incremental propagation yields,
at every hop, exactly what layer-wise recomputation on the updated graph
yields, up to floating-point rounding (Sec. 3.3.3, the cancelling-terms
example for h^2_D; Sec. 5, last paragraph). The oracle is therefore that
definition written out: after a batch has been applied to the graph, every
embedding of every layer is recomputed from the features with Eq. (1)-(2)
(Sec. 2.1) in float64. Independently it derives, by set operations only, which
vertices the batch can affect at each hop (Sec. 3.2's per-update-type
description; Sec. 2.2's worked example).

Readings taken where the paper leaves a choice:
  * sum / mean / weighted sum as in Table 1 (weighted sum: x_v = sum over in-neighbours u of
    alpha_uv h_u, alpha_uv a per-edge weight fixed when the edge is created; Sec. 3.3.3, "Other
    linear aggregators"); mean of an empty neighbourhood is the zero vector;
  * max / min as in Table 1, element by element over the in-neighbours' rows; an empty
    neighbourhood gives the zero vector. The paper's hybrid treatment of these aggregators
    (Sec. 3.4.2: leave unchanged / update incrementally / recompute) reaches the recomputed
    values exactly, so the oracle is again the definition; which vertices a pruned propagation
    visits is not unique, so for these layers the topological sets are an upper bound and the
    rows whose value really changes a lower bound of what an implementation may report;
  * graph attention (Sec. 3.4.1, Eq. 3): the printed score z_uv = a . (W h_u || W h_v) without a
    non-linearity would make the sink's part cancel in the softmax, against the section's own
    statement that the coefficient depends on both endpoints; the cited GAT definition is taken:
    z_uv = LeakyReLU_0.2(a_src . W h_u + a_dst . W h_v), one head, h_v = act(sum_u alpha_uv W h_u + b),
    act(b) for a vertex without in-neighbours. The hybrid scheme (recompute vertices already in the
    tree, numerator / denominator deltas for the others) reaches these values, so the oracle is
    the definition;
  * GraphConv: h = act(x W + b), no self term (Sec. 3.3.3 example);
    GraphSAGE: h = act(h_self W_self + x W_neigh + b) (Eq. 2's UPDATE takes both);
    GIN: h = act(MLP((1+eps) h_self + x)) (Sec. 6.3.1: GI-S adds the vertex's
    own embedding to its in-neighbours');
  * operations of a batch are applied in array order; invalid ones (dead or
    out-of-range endpoint, duplicate edge, missing edge, adding a live vertex,
    deleting or updating a dead one, a new weight for a missing edge or on a graph
    without weights) are rejected and skipped;
  * besides the paper's five update types there is a sixth, the replacement of an edge's weight
    alpha_uv on weighted graphs (the paper keeps weights fixed; with Table 1's weighted sum a new
    weight changes the sink's aggregate like any other change of the message alpha_uv h_u);
  * a deleted vertex loses all incident edges (Sec. 3.2) and its rows are zero;
  * affected sets are topological: a vertex is affected whether or not its
    value ends up different (Sec. 3.3.1: every vertex of the tree is updated).

Parity pins (tests/test_oracle_*.py): brute-force per-vertex neighbourhood
recursion on small graphs, the closed form (A^T)^L H W1..WL for the linear
case, the all-ones mean fixed point, isolated vertices, the paper's worked
edge-addition example for the affected sets, planted-mistake checks; for max / min the
brute force, the values printed with the paper's three max cases, max(h) = -min(-h),
min <= mean <= max, and the one-in-neighbour graph where every aggregator agrees; for attention
the brute force, zero or sink-side-only attention vectors (= the mean of the projected rows)
and the one-in-neighbour graph (= the projected row).
The numeric values of the paper's own runs are unpinned: it prints none.
"""
from __future__ import annotations

import dataclasses
import numpy as np
import scipy.sparse as sp

EDGE_ADD, EDGE_DEL, VERTEX_ADD, VERTEX_DEL, FEAT_UPDATE, EDGE_REWEIGHT = 0, 1, 2, 3, 4, 5


# --------------------------------------------------------------------------
# graph state
# --------------------------------------------------------------------------
class GraphState:
    """Simple directed graph with vertex features, float64.

    Edges live in a sorted base array of keys u*cap+v (and a second copy keyed
    v*cap+u for in-neighbour lookups), minus a set of deleted base keys, plus
    the edges added later; this keeps per-batch mutation cheap on graphs with
    10^8 edges.
    """

    def __init__(self, n_vertices: int, vertex_capacity: int, src, dst, feats, weights=None):
        self.cap = int(vertex_capacity)
        self.alive = np.zeros(self.cap, dtype=bool)
        self.alive[:n_vertices] = True
        s = np.asarray(src, dtype=np.int64)
        d = np.asarray(dst, dtype=np.int64)
        keys = s * self.cap + d
        order = np.argsort(keys, kind="stable")
        self.base = keys[order]
        if self.base.size and (np.diff(self.base) == 0).any():
            raise ValueError("initial edge list contains duplicates")
        self.weighted = weights is not None
        # per-edge weight alpha_uv (weighted sum): aligned with `base`; later edges in w_late
        self.base_w = (np.asarray(weights, dtype=np.float64)[order] if self.weighted
                       else np.ones(self.base.size))
        self.w_late = {}                            # key u*cap+v -> weight of an edge created after the start
        self.base_t = np.sort(d * self.cap + s)
        self.removed = set()                        # base keys (u*cap+v) no longer present
        self.added_out = {}                         # u -> set of v, edges not in base
        self.added_in = {}                          # v -> set of u
        self.n_added = 0
        f = np.asarray(feats, dtype=np.float64)
        self.h0 = np.zeros((self.cap, f.shape[1]), dtype=np.float64)
        self.h0[:n_vertices] = f

    # -- edges ---------------------------------------------------------------
    def _in_base(self, key: int) -> bool:
        i = int(np.searchsorted(self.base, key))
        return i < self.base.size and int(self.base[i]) == key

    def has_edge(self, u: int, v: int) -> bool:
        if v in self.added_out.get(u, ()):
            return True
        key = u * self.cap + v
        return key not in self.removed and self._in_base(key)

    def _insert(self, u: int, v: int, w: float = 1.0):
        key = u * self.cap + v
        self.w_late[key] = w                        # also overrides the weight a re-created base edge had
        if key in self.removed:
            self.removed.discard(key)
        else:
            self.added_out.setdefault(u, set()).add(v)
            self.added_in.setdefault(v, set()).add(u)
            self.n_added += 1

    def _erase(self, u: int, v: int):
        self.w_late.pop(u * self.cap + v, None)
        if v in self.added_out.get(u, ()):
            self.added_out[u].discard(v)
            self.added_in[v].discard(u)
            self.n_added -= 1
        else:
            self.removed.add(u * self.cap + v)

    def edges(self):
        """(src, dst) int64 arrays of the current edge set."""
        keep = np.ones(self.base.size, dtype=bool)
        if self.removed:
            gone = np.fromiter(self.removed, dtype=np.int64, count=len(self.removed))
            keep[np.searchsorted(self.base, gone)] = False
        extra = np.array([u * self.cap + v for u, vs in self.added_out.items() for v in vs],
                         dtype=np.int64)
        keys = np.concatenate([self.base[keep], extra])
        return keys // self.cap, keys % self.cap

    def edge_weights(self):
        """Weights alpha_uv in the order of edges()."""
        keep = np.ones(self.base.size, dtype=bool)
        if self.removed:
            gone = np.fromiter(self.removed, dtype=np.int64, count=len(self.removed))
            keep[np.searchsorted(self.base, gone)] = False
        w = self.base_w.copy()
        for key, val in self.w_late.items():        # a base edge deleted and created again
            i = int(np.searchsorted(self.base, key))
            if i < self.base.size and int(self.base[i]) == key:
                w[i] = val
        extra = np.array([self.w_late[u * self.cap + v] for u, vs in self.added_out.items() for v in vs],
                         dtype=np.float64)
        return np.concatenate([w[keep], extra])

    def n_edges(self) -> int:
        return self.base.size - len(self.removed) + self.n_added

    def out_neighbours(self, u: int) -> list:
        lo, hi = np.searchsorted(self.base, [u * self.cap, (u + 1) * self.cap])
        res = [int(k) % self.cap for k in self.base[lo:hi].tolist() if k not in self.removed]
        return res + sorted(self.added_out.get(u, ()))

    def in_neighbours(self, v: int) -> list:
        lo, hi = np.searchsorted(self.base_t, [v * self.cap, (v + 1) * self.cap])
        res = []
        for k in self.base_t[lo:hi].tolist():
            u = k % self.cap
            if u * self.cap + v not in self.removed:
                res.append(u)
        return res + sorted(self.added_in.get(v, ()))

    # -- one batch -------------------------------------------------------------
    def apply_batch(self, ops, payload) -> "BatchRecord":
        """Apply operations in array order (Sec. 3.3, Apply step).

        Returns which operations were accepted and the root sets the
        affected-set derivation needs.
        """
        ops = np.asarray(ops, dtype=np.int64).reshape(-1, 4)
        if payload is None:
            payload = np.zeros((0, self.h0.shape[1]))
        payload = np.asarray(payload, dtype=np.float64).reshape(-1, self.h0.shape[1])
        rec = BatchRecord(accepted=np.zeros(len(ops), dtype=bool))
        for i, (kind, u, v, row) in enumerate(ops.tolist()):
            if kind in (EDGE_ADD, EDGE_DEL):
                if not (0 <= u < self.cap and 0 <= v < self.cap):
                    continue
                if not (self.alive[u] and self.alive[v]):
                    continue
                present = self.has_edge(u, v)
                if kind == EDGE_ADD and not present:
                    # weighted graphs: the operation's fourth word holds the float32 bits of alpha_uv
                    w = float(np.array([row], dtype=np.uint32).view(np.float32)[0]) if self.weighted else 1.0
                    self._insert(u, v, w)
                elif kind == EDGE_DEL and present:
                    self._erase(u, v)
                else:
                    continue
                rec.sinks.add(v)
            elif kind == EDGE_REWEIGHT:
                # the weight alpha_uv of an existing edge of a weighted graph is replaced (Sec. 3.3.3, "Other linear
                # aggregators": the message along u -> v is alpha_uv times the embedding, so a new alpha changes
                # what v aggregates exactly as a changed embedding of u would); v is touched at every hop like the
                # sink of an added or deleted edge
                if not (0 <= u < self.cap and 0 <= v < self.cap) or not (self.alive[u] and self.alive[v]):
                    continue
                if not self.weighted or not self.has_edge(u, v):
                    continue
                self.w_late[u * self.cap + v] = float(np.array([row], dtype=np.uint32).view(np.float32)[0])
                rec.sinks.add(v)
            elif kind == VERTEX_ADD:
                if not (0 <= u < self.cap) or self.alive[u] or not (0 <= row < len(payload)):
                    continue
                self.alive[u] = True
                self.h0[u] = payload[row]
                rec.added.add(u)
            elif kind == VERTEX_DEL:
                if not (0 <= u < self.cap) or not self.alive[u]:
                    continue
                for y in self.out_neighbours(u):    # Sec. 3.2: all incident edges go first
                    self._erase(u, y)
                    rec.sinks.add(y)
                for x in self.in_neighbours(u):
                    self._erase(x, u)
                self.alive[u] = False
                self.h0[u] = 0.0
                rec.removed.add(u)
                rec.added.discard(u)
                rec.feat.discard(u)
            elif kind == FEAT_UPDATE:
                if not (0 <= u < self.cap) or not self.alive[u] or not (0 <= row < len(payload)):
                    continue
                self.h0[u] = payload[row]
                rec.feat.add(u)
            else:
                continue
            rec.accepted[i] = True
        return rec


@dataclasses.dataclass
class BatchRecord:
    accepted: np.ndarray
    sinks: set = dataclasses.field(default_factory=set)     # sinks of changed edges
    added: set = dataclasses.field(default_factory=set)     # vertices created
    removed: set = dataclasses.field(default_factory=set)   # vertices deleted
    feat: set = dataclasses.field(default_factory=set)      # feature replaced


# --------------------------------------------------------------------------
# layer math, Eq. (1)-(2)
# --------------------------------------------------------------------------
def _act(name: str, z: np.ndarray) -> np.ndarray:
    if name == "relu":
        return np.maximum(z, 0.0)
    if name == "none":
        return z
    raise ValueError(name)


class InAdjacency:
    """ones: sparse matrix with a 1 at (v, u) for every edge u -> v (row v lists v's in-neighbours);
    alpha: the same pattern holding the edge weights alpha_uv (weighted graphs, else None)."""

    def __init__(self, state: GraphState):
        src, dst = state.edges()
        shape = (state.cap, state.cap)
        self.ones = sp.csr_matrix((np.ones(src.size), (dst, src)), shape=shape)
        self.alpha = sp.csr_matrix((state.edge_weights(), (dst, src)), shape=shape) if state.weighted else None


def in_adjacency(state: GraphState) -> InAdjacency:
    return InAdjacency(state)


def aggregate(a_in: InAdjacency, h_prev: np.ndarray, agg: str, rows=None) -> np.ndarray:
    """Eq. (1): x_v = AGG over in-neighbours u of v of h_prev[u] (Table 1), for all v or for `rows`."""
    if agg == "wsum":                                            # sum of alpha_uv h_u
        if a_in.alpha is None:
            raise ValueError("weighted sum on a graph without edge weights")
        a = a_in.alpha if rows is None else a_in.alpha[rows]
        return a @ h_prev
    a = a_in.ones if rows is None else a_in.ones[rows]
    if agg in ("max", "min"):                                    # element-wise extreme (Table 1; Sec. 3.4.2)
        return _extreme(a, h_prev, np.maximum if agg == "max" else np.minimum)
    x = a @ h_prev                                               # sum over in-neighbours
    if agg == "mean":
        deg = np.asarray(a.getnnz(axis=1), dtype=np.float64)     # in-degree
        x = x / np.maximum(deg, 1.0)[:, None]                    # empty neighbourhood: 0
    elif agg != "sum":
        raise ValueError(agg)
    return x


SLAB_ELEMENTS = 1 << 26          # numbers gathered at a time by the max / min aggregation


def _extreme(a, h_prev: np.ndarray, op) -> np.ndarray:
    """Row v of the result: op reduced element by element over the rows h_prev[u] of v's
    in-neighbours u (the column indices of row v of `a`); a vertex without in-neighbours gets 0.
    Rows are taken in slabs so that the gathered neighbour rows stay bounded in memory."""
    a = a.tocsr()
    indptr, indices = a.indptr, a.indices
    out = np.zeros((a.shape[0], h_prev.shape[1]))
    rows = np.flatnonzero(np.diff(indptr) > 0)                   # rows with at least one in-neighbour
    budget = max(1, SLAB_ELEMENTS // max(1, h_prev.shape[1]))    # gathered neighbour rows per slab
    i = 0
    while i < rows.size:
        lo = indptr[rows[i]]
        j = int(np.searchsorted(indptr[rows + 1], lo + budget, side="right"))
        j = max(j, i + 1)
        take = rows[i:j]
        hi = indptr[take[-1] + 1]
        gathered = h_prev[indices[lo:hi]]
        # consecutive non-empty rows are adjacent in `indices`, so each segment ends where the next starts
        out[take] = op.reduceat(gathered, indptr[take] - lo, axis=0)
        i = j
    return out


def layer_rows(state: GraphState, layer: dict, h_prev: np.ndarray, a_in: InAdjacency, rows=None) -> np.ndarray:
    """Eq. (2): h_v = act(UPDATE(h_prev[v], x_v)) for all vertices or for `rows`; dead rows are 0."""
    d_in = layer["d_in"]
    if layer["agg"] == "attn":
        return _attention_rows(state, layer, h_prev, a_in, rows)
    x = aggregate(a_in, h_prev, layer["agg"], rows)
    own = h_prev if rows is None else h_prev[rows]
    w0 = np.asarray(layer["W0"], dtype=np.float64)
    b0 = np.asarray(layer["b0"], dtype=np.float64)
    if layer["self"] == "none":
        z = x @ w0 + b0
    elif layer["self"] == "concat":
        z = own @ w0[:d_in] + x @ w0[d_in:] + b0
    elif layer["self"] == "add":
        z = ((1.0 + layer["eps"]) * own + x) @ w0 + b0
    else:
        raise ValueError(layer["self"])
    if layer["d_hidden"]:
        z = _act(layer["act_inner"], z)
        z = z @ np.asarray(layer["W1"], dtype=np.float64) + np.asarray(layer["b1"], dtype=np.float64)
    h = _act(layer["act_out"], z)
    alive = state.alive if rows is None else state.alive[rows]
    h[~alive] = 0.0
    return h


LEAKY_SLOPE = 0.2


def _attention_rows(state: GraphState, layer: dict, h_prev: np.ndarray, a_in: InAdjacency, rows=None) -> np.ndarray:
    """Graph attention layer, Eq. (3) (Sec. 3.4.1), single head: with p_u = h_prev[u] W,
    z_uv = LeakyReLU(a_src . p_u + a_dst . p_v), alpha_uv = exp(z_uv) / sum over v's in-neighbours
    u' of exp(z_u'v), h_v = act(sum_u alpha_uv p_u + b); a vertex without in-neighbours gets act(b).
    layer["att"] holds a_src followed by a_dst (d_out numbers each)."""
    w0 = np.asarray(layer["W0"], dtype=np.float64)
    b0 = np.asarray(layer["b0"], dtype=np.float64)
    att = np.asarray(layer["att"], dtype=np.float64)
    d_out = layer["d_out"]
    p = h_prev @ w0
    s_src, s_dst = p @ att[:d_out], p @ att[d_out:]
    a = (a_in.ones if rows is None else a_in.ones[rows]).tocsr()
    sinks = np.arange(a.shape[0]) if rows is None else np.asarray(rows)
    counts = np.diff(a.indptr)
    z = s_src[a.indices] + np.repeat(s_dst[sinks], counts)      # one entry per in-edge u -> v, grouped by v
    z = np.where(z > 0, z, LEAKY_SLOPE * z)
    e = sp.csr_matrix((np.exp(z), a.indices, a.indptr), shape=a.shape)
    num = e @ p
    den = np.asarray(e.sum(axis=1)).ravel()
    x = np.divide(num, den[:, None], out=np.zeros_like(num), where=den[:, None] > 0)
    h = _act(layer["act_out"], x + b0)
    alive = state.alive if rows is None else state.alive[rows]
    h[~alive] = 0.0
    return h


def layer_forward(state: GraphState, layer: dict, h_prev: np.ndarray) -> np.ndarray:
    return layer_rows(state, layer, h_prev, in_adjacency(state))


def full_recompute(state: GraphState, model) -> list:
    """All embeddings of all layers on the current graph: [H^0, H^1, ..., H^L]."""
    hs = [state.h0.copy()]
    hs[0][~state.alive] = 0.0
    a_in = in_adjacency(state)
    for layer in model:
        hs.append(layer_rows(state, layer, hs[-1], a_in))
    return hs


def recompute_rows(state: GraphState, model, targets) -> list:
    """Final-layer rows of `targets`, computed from the features through their in-neighbourhood
    only (the vertex's computational graph, Sec. 1.1, evaluated layer by layer): the rows needed
    at layer l-1 are the in-neighbours of the rows needed at layer l, plus those rows themselves
    when the layer reads the vertex's own embedding. Returns, per layer l = 0..L, a pair
    (sorted row ids, their embeddings); used where recomputing everything is too slow."""
    a_in = in_adjacency(state)
    L = len(model)
    need = [None] * (L + 1)
    need[L] = np.unique(np.asarray(targets, dtype=np.int64))
    for l in range(L, 0, -1):
        nbrs = np.unique(a_in.ones[need[l]].indices)
        own = model[l - 1]["self"] != "none" or model[l - 1]["agg"] == "attn"     # attention scores read the sink's own row
        need[l - 1] = np.union1d(nbrs, need[l]) if own else nbrs
    h = np.zeros_like(state.h0)
    h[need[0]] = state.h0[need[0]]
    h[~state.alive] = 0.0
    out = [(need[0], h[need[0]].copy())]
    for l in range(1, L + 1):
        rows = need[l]
        vals = layer_rows(state, model[l - 1], h, a_in, rows)
        h = np.zeros((state.cap, model[l - 1]["d_out"]))
        h[rows] = vals
        out.append((rows, vals))
    return out


# --------------------------------------------------------------------------
# affected sets (Sec. 2.2 example, Sec. 3.2, Sec. 3.3)
# --------------------------------------------------------------------------
def affected_sets(state_after: GraphState, rec: BatchRecord, model) -> list:
    """Sorted vertex ids whose layer-l embedding the batch can change, l = 0..L.

    Hop 0: vertices whose features were written. Hop l: sinks of every changed
    edge (an edge's sink is touched at every hop, Sec. 3.2 and the inbox example
    of Sec. 3.3.2), out-neighbours in the updated graph of hop l-1's set, that
    set itself when the layer reads the vertex's own previous embedding (a self term, or
    attention, where it sets the vertex's scores; Sec. 3.4.1: a vertex of the tree stays in it), and
    created vertices (Sec. 3.2: a new vertex updates its own embeddings);
    deleted vertices are dropped.
    """
    src, dst = state_after.edges()
    alive = state_after.alive
    cur = {w for w in (rec.feat | rec.added) if alive[w]}
    out = [np.array(sorted(cur), dtype=np.int64)]
    for layer in model:
        mask = np.zeros(state_after.cap, dtype=bool)
        if cur:
            mask[list(cur)] = True
        nxt = set(dst[mask[src]].tolist())
        nxt |= rec.sinks | rec.added
        if layer["self"] != "none" or layer["agg"] == "attn":   # attention: the vertex's own row sets its scores
            nxt |= cur
        cur = {w for w in nxt if alive[w]}
        out.append(np.array(sorted(cur), dtype=np.int64))
    return out


# --------------------------------------------------------------------------
# error metric used by every comparison against this oracle
# --------------------------------------------------------------------------
def max_rel_err(got: np.ndarray, want: np.ndarray, alive: np.ndarray) -> float:
    """max over rows of ||got-want||_inf / max(||want||_inf, tau), where tau is
    the mean of ||want||_inf over live rows. Element-wise relative error is
    undefined at ReLU zeros, so rows are normalised by their own magnitude with
    the layer's typical magnitude as floor."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    row = np.abs(want).max(axis=1) if want.shape[1] else np.zeros(len(want))
    tau = float(row[alive].mean()) if alive.any() else 1.0
    tau = tau if tau > 0 else 1.0
    diff = np.abs(got - want).max(axis=1) if want.shape[1] else np.zeros(len(want))
    return float((diff / np.maximum(row, tau)).max()) if len(want) else 0.0
