"""Seeded stream of update batches over an evolving graph.

The stream keeps its own record of which edges and vertices exist so that
every operation it emits is valid when applied in array order, and so that a
batch never touches the same edge twice nor any vertex that the same batch
adds or deletes (apart from a new vertex's own edges, which directly follow
its VERTEX_ADD). One logical update is one edge add, one edge delete, one
feature replacement, one vertex delete, or one vertex add together with its
`edges_per_new_vertex` edges.

Operation record: uint32 [kind, u, v, feat_row]; edges are (u -> v); vertex
operations use u; feat_row indexes the batch's payload for VERTEX_ADD and
FEAT_UPDATE and is 0 otherwise, except that a weighted stream puts the float32
bits of the new edge's weight (uniform in [0.25, 1.75)) there for EDGE_ADD and of
the replacement weight for EDGE_REWEIGHT (mix key "reweight", weighted streams only).
"""
from __future__ import annotations

import numpy as np

from .graphs import (OP_EDGE_ADD, OP_EDGE_DEL, OP_VERTEX_ADD, OP_VERTEX_DEL,
                     OP_FEAT_UPDATE, OP_EDGE_REWEIGHT, PowerLaw, draw_pair)


class UpdateStream:
    def __init__(self, n: int, vertex_capacity: int, src, dst, out_law: PowerLaw,
                 in_law: PowerLaw, d0: int, mix: dict, seed: int,
                 edges_per_new_vertex: int = 8, weighted: bool = False):
        self.cap = int(vertex_capacity)
        self.d0 = int(d0)
        self.mix = dict(mix)
        self.out_law, self.in_law = out_law, in_law
        self.rng = np.random.default_rng(seed)
        self.weighted = bool(weighted)
        self.wrng = np.random.default_rng(seed + 7919)       # its own stream: the operations do not depend on it
        self.epv = int(edges_per_new_vertex)
        s64, d64 = np.asarray(src, np.int64), np.asarray(dst, np.int64)
        self.base = np.sort(s64 * self.cap + d64)            # keyed src-major
        self.base_t = np.sort(d64 * self.cap + s64)          # keyed dst-major
        self.base_dead = set()
        self.extra = {}                                      # key -> slot in extra_list
        self.extra_list = []
        self.extra_out = {}                                  # src -> set(dst) among extras
        self.extra_in = {}
        self.alive = np.zeros(self.cap, dtype=bool)
        self.alive[:n] = True
        self.next_id = int(n)

    # ---- bookkeeping -----------------------------------------------------
    def n_edges(self) -> int:
        return self.base.size - len(self.base_dead) + len(self.extra_list)

    def _in_base(self, key: int) -> bool:
        i = int(np.searchsorted(self.base, key))
        return i < self.base.size and int(self.base[i]) == key

    def has_edge(self, u: int, v: int) -> bool:
        key = u * self.cap + v
        if key in self.extra:
            return True
        return key not in self.base_dead and self._in_base(key)

    def _add_edge(self, u: int, v: int):
        key = u * self.cap + v
        if key in self.base_dead:
            self.base_dead.discard(key)
            return
        self.extra[key] = len(self.extra_list)
        self.extra_list.append(key)
        self.extra_out.setdefault(u, set()).add(v)
        self.extra_in.setdefault(v, set()).add(u)

    def _del_edge(self, u: int, v: int):
        key = u * self.cap + v
        slot = self.extra.pop(key, None)
        if slot is None:
            self.base_dead.add(key)
            return
        last = self.extra_list.pop()
        if last != key:
            self.extra_list[slot] = last
            self.extra[last] = slot
        self.extra_out[u].discard(v)
        self.extra_in[v].discard(u)

    def out_neighbours(self, u: int):
        lo, hi = np.searchsorted(self.base, [u * self.cap, (u + 1) * self.cap])
        res = [int(k % self.cap) for k in self.base[lo:hi] if int(k) not in self.base_dead]
        res.extend(self.extra_out.get(u, ()))
        return res

    def in_neighbours(self, v: int):
        lo, hi = np.searchsorted(self.base_t, [v * self.cap, (v + 1) * self.cap])
        res = []
        for k in self.base_t[lo:hi]:
            s = int(k % self.cap)
            if s * self.cap + v not in self.base_dead:
                res.append(s)
        res.extend(self.extra_in.get(v, ()))
        return res

    def edge_arrays(self):
        """Current edge set as (src, dst) uint32 arrays (for cross-checks)."""
        keep = np.ones(self.base.size, dtype=bool)
        if self.base_dead:
            dead = np.fromiter(self.base_dead, dtype=np.int64, count=len(self.base_dead))
            keep[np.searchsorted(self.base, dead)] = False
        keys = np.concatenate([self.base[keep], np.asarray(self.extra_list, dtype=np.int64)])
        return (keys // self.cap).astype(np.uint32), (keys % self.cap).astype(np.uint32)

    # ---- random picks ----------------------------------------------------
    def _random_alive(self, banned) -> int:
        while True:
            w = int(self.rng.integers(self.next_id))
            if self.alive[w] and w not in banned:
                return w

    def _random_existing_edge(self, used, banned):
        nb = self.base.size
        while True:
            r = int(self.rng.integers(nb + len(self.extra_list)))
            key = int(self.base[r]) if r < nb else self.extra_list[r - nb]
            if r < nb and key in self.base_dead:
                continue
            u, v = divmod(key, self.cap)
            if key in used or u in banned or v in banned:
                continue
            return u, v

    def _random_new_edge(self, used, banned):
        while True:
            us, vs = draw_pair(self.rng, self.out_law, self.in_law, 16)
            for u, v in zip(us.tolist(), vs.tolist()):
                if u == v or not (self.alive[u] and self.alive[v]):
                    continue
                if u in banned or v in banned:
                    continue
                key = u * self.cap + v
                if key in used or self.has_edge(u, v):
                    continue
                return u, v

    # ---- one batch ---------------------------------------------------------
    def counts(self, bs: int) -> dict:
        """Updates of each kind in a batch of `bs`: the mix times bs when that
        is integral for every kind, otherwise a multinomial draw from the mix."""
        names = ("edge_add", "edge_del", "feat", "vadd", "vdel", "reweight")
        exact = [self.mix.get(k, 0.0) * bs for k in names]
        if all(abs(x - round(x)) < 1e-6 for x in exact):
            return {k: int(round(x)) for k, x in zip(names, exact)}
        p = np.asarray([self.mix.get(k, 0.0) for k in names], dtype=np.float64)
        draw = self.rng.multinomial(bs, p / p.sum())
        return {k: int(x) for k, x in zip(names, draw)}

    def next_batch(self, bs: int, kinds=None):
        """Return (ops uint32[n_ops,4], payload float32[n_rows,d0], n_updates).

        `kinds` optionally fixes the logical kind of every update (used by
        bs=1 streams, which cycle through the mix instead of rounding it).
        """
        rng = self.rng
        if kinds is None:
            c = self.counts(bs)
            kinds = (["vdel"] * c["vdel"] + ["vadd"] * c["vadd"] + ["feat"] * c["feat"] +
                     ["edge_del"] * c["edge_del"] + ["edge_add"] * c["edge_add"] + ["reweight"] * c["reweight"])
        kinds = sorted(kinds, key=lambda k: {"vdel": 0, "vadd": 1}.get(k, 2))
        banned = set()              # vertices added or deleted by this batch
        used = set()                # edge keys touched by this batch
        feat_used = set()
        groups = []                 # one list of op tuples per logical update
        rows = []
        for kind in kinds:
            if kind == "vdel":
                w = self._random_alive(banned)
                banned.add(w)
                groups.append([(OP_VERTEX_DEL, w, 0, 0)])
            elif kind == "vadd":
                if self.next_id >= self.cap:
                    raise RuntimeError("vertex capacity of the stream exhausted")
                w = self.next_id
                self.next_id += 1
                banned.add(w)
                rows.append(rng.standard_normal(self.d0, dtype=np.float32))
                g = [(OP_VERTEX_ADD, w, 0, len(rows) - 1)]
                peers = set()
                while len(peers) < self.epv:
                    p = self._random_alive(banned)
                    peers.add(p)
                for p in sorted(peers):
                    u, v = (w, p) if rng.random() < 0.5 else (p, w)
                    used.add(u * self.cap + v)
                    g.append((OP_EDGE_ADD, u, v, 0))
                groups.append(g)
            elif kind == "feat":
                while True:
                    w = self._random_alive(banned)
                    if w not in feat_used:
                        break
                feat_used.add(w)
                rows.append(rng.standard_normal(self.d0, dtype=np.float32))
                groups.append([(OP_FEAT_UPDATE, w, 0, len(rows) - 1)])
            elif kind == "edge_del":
                u, v = self._random_existing_edge(used, banned)
                used.add(u * self.cap + v)
                groups.append([(OP_EDGE_DEL, u, v, 0)])
            elif kind == "edge_add":
                u, v = self._random_new_edge(used, banned)
                used.add(u * self.cap + v)
                groups.append([(OP_EDGE_ADD, u, v, 0)])
            elif kind == "reweight":                         # weighted streams only: a new weight for an existing edge
                if not self.weighted:
                    raise ValueError("edge weights can only be replaced on a weighted stream")
                u, v = self._random_existing_edge(used, banned)
                used.add(u * self.cap + v)
                groups.append([(OP_EDGE_REWEIGHT, u, v, 0)])
            else:
                raise ValueError(kind)
        order = rng.permutation(len(groups))
        ops = [op for gi in order for op in groups[gi]]
        # commit to the tracker
        for kind, u, v, _ in ops:
            if kind == OP_EDGE_ADD:
                self._add_edge(u, v)
            elif kind == OP_EDGE_DEL:
                self._del_edge(u, v)
            elif kind == OP_VERTEX_ADD:
                self.alive[u] = True
            elif kind == OP_VERTEX_DEL:
                for y in self.out_neighbours(u):
                    self._del_edge(u, y)
                for x in self.in_neighbours(u):
                    self._del_edge(x, u)
                self.alive[u] = False
        ops_arr = np.asarray(ops, dtype=np.uint32).reshape(-1, 4)
        if self.weighted:
            adds = (ops_arr[:, 0] == OP_EDGE_ADD) | (ops_arr[:, 0] == OP_EDGE_REWEIGHT)
            w = self.wrng.uniform(0.25, 1.75, int(adds.sum())).astype(np.float32)
            ops_arr[adds, 3] = w.view(np.uint32)
        payload = (np.stack(rows).astype(np.float32) if rows
                   else np.zeros((0, self.d0), dtype=np.float32))
        return ops_arr, payload, len(groups)
