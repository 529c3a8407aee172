"""Side-by-side driver for the parity tests: the same seeded inputs go to the
GPU library (through its C ABI binding) and to the CPU oracle, and every
observable is compared."""
import numpy as np

import oracle
import paper_2601_12347_amd as rp
import ripple_inputs as ri

TOL = {"f32": 1e-4, "bf16": 2e-2}      # max relative error per layer (metric: oracle.max_rel_err)


class Pair:
    def __init__(self, n, cap, src, dst, feats, model, store="f32", edge_capacity=None, project_first=True,
                 self_cache=True, deterministic=False, weights=None, split=None, packed=None):
        self.n, self.cap, self.model, self.store = n, cap, model, store
        self.widths = [model[0]["d_in"]] + [l["d_out"] for l in model]
        self.L = len(model)
        self.ora = oracle.GraphState(n, cap, src, dst, feats, weights=weights)
        if weights is None:
            self.ctx = rp.ripple_init_graph(n, cap, src, dst, feats, store=store, edge_capacity=edge_capacity)
        else:
            self.ctx = rp.ripple_init_graph_weighted(n, cap, src, dst, weights, feats, store=store,
                                                     edge_capacity=edge_capacity)
        if not project_first:
            rp.ripple_set_option(self.ctx, rp.OPT_PROJECT_FIRST, 0)
        if not self_cache:
            rp.ripple_set_option(self.ctx, rp.OPT_SELF_CACHE, 0)
        if deterministic:
            rp.ripple_set_option(self.ctx, rp.OPT_DETERMINISTIC, 1)
        if split is not None:
            rp.ripple_set_option(self.ctx, rp.OPT_SPLIT_MFMA, int(split))
        if packed is not None:
            rp.ripple_set_option(self.ctx, rp.OPT_PACKED_MESSAGES, int(packed))
        rp.ripple_load_model(self.ctx, model)
        rp.ripple_full_infer(self.ctx)
        # first layer (1-based) that aggregates with max / min: from there on the reported sets are pruned
        mono = [l + 1 for l, lay in enumerate(model) if lay["agg"] in ("max", "min")]
        self.first_mono = mono[0] if mono else None

    def close(self):
        rp.ripple_destroy(self.ctx)
        self.ctx = None

    def gpu_layer(self, l):
        return rp.ripple_get_embeddings(self.ctx, l, self.widths[l], n_rows=self.cap)

    def check_embeddings(self, tol=None, want=None):
        tol = TOL[self.store] if tol is None else tol
        want = oracle.full_recompute(self.ora, self.model) if want is None else want
        errs = []
        for l in range(self.L + 1):
            got = self.gpu_layer(l)
            assert np.isfinite(got).all()
            err = oracle.max_rel_err(got, want[l], self.ora.alive)
            errs.append(err)
            assert err <= tol, f"layer {l}: max rel err {err:.3e} > {tol}"
            assert not got[~self.ora.alive].any(), f"layer {l}: dead rows must be zero"
        return errs, want

    def check_aggregates(self, tol=None):
        """X^l[v] must equal the sum over v's in-neighbours of the stored H^{l-1}."""
        tol = 1e-4 if tol is None else tol
        src, dst = self.ora.edges()
        for l in range(1, self.L + 1):
            if self.model[l - 1]["agg"] == "attn":
                self._check_attention_numerators(l, tol)
                continue
            h_prev = self.gpu_layer(l - 1).astype(np.float64)
            width, projected, _ = rp.ripple_get_layer_info(self.ctx, l)
            if projected:                                     # the layer caches sum_u H[u] W_neigh
                lay = self.model[l - 1]
                w = np.asarray(lay["W0"], dtype=np.float64)
                h_prev = h_prev @ (w[lay["d_in"]:] if lay["self"] == "concat" else w)
            assert width == h_prev.shape[1]
            want = np.zeros_like(h_prev)
            if self.model[l - 1]["agg"] in ("max", "min"):        # the extreme of the stored rows, exactly
                want = oracle.aggregate(oracle.in_adjacency(self.ora), h_prev, self.model[l - 1]["agg"])
                got = rp.ripple_get_aggregates(self.ctx, l, width, n_rows=self.cap)
                assert np.array_equal(got[self.ora.alive], want[self.ora.alive].astype(np.float32)), f"aggregate {l}"
                continue
            if self.model[l - 1]["agg"] == "wsum":
                np.add.at(want, dst, h_prev[src] * self.ora.edge_weights()[:, None])
            else:
                np.add.at(want, dst, h_prev[src])
            got = rp.ripple_get_aggregates(self.ctx, l, width, n_rows=self.cap)
            err = oracle.max_rel_err(got, want, self.ora.alive)
            assert err <= tol, f"aggregate {l}: {err:.3e}"

    def _check_attention_numerators(self, l, tol):
        """Attention layers cache sum_u w_uv P[u] (un-normalised, Sec. 3.4.1). The weights w_uv depend on
        scores the library keeps to itself, so the cached row is compared up to its positive scale: divided
        by the denominator implied by the stored output it must give the oracle's normalised aggregate
        computed from the stored H^{l-1}; here simply: direction and, through the embeddings check, value."""
        lay = self.model[l - 1]
        h_prev = self.gpu_layer(l - 1).astype(np.float64)
        width, _, _ = rp.ripple_get_layer_info(self.ctx, l)
        assert width == lay["d_out"]
        num = rp.ripple_get_aggregates(self.ctx, l, width, n_rows=self.cap).astype(np.float64)
        lin = dict(lay, act_out="none", b0=np.zeros_like(lay["b0"]))
        want = oracle.layer_rows(self.ora, lin, h_prev, oracle.in_adjacency(self.ora))   # sum_u alpha_uv P[u]
        # num = den * want with den > 0: rows whose aggregate is not negligible must point the same way after
        # normalising both by their largest entry. Rows whose aggregate is (nearly) zero, e.g. because all
        # in-neighbours' rows are zero after a ReLU, hold only the residue of the incremental patches; their
        # value is covered by the comparison of the embeddings.
        has = (np.bincount(self.ora.edges()[1], minlength=self.cap) > 0) & self.ora.alive
        mag_w, mag_n = np.abs(want).max(axis=1), np.abs(num).max(axis=1)
        typical = mag_w[has].mean() if has.any() else 0.0
        big = has & (mag_w > 1e-2 * typical)
        limit = 1e-4 if tol is None else tol
        if big.any():
            unit_n, unit_w = num[big] / mag_n[big, None].clip(1e-300), want[big] / mag_w[big, None]
            err = np.abs(unit_n - unit_w).max()
            assert err <= 100 * limit, f"attention numerator {l}: direction off by {err:.3e}"
        assert np.isfinite(num).all() and not num[~has].any()

    def check_graph(self):
        src, dst = self.ora.edges()
        want = np.sort(src * self.cap + dst)
        for direction in (0, 1):
            s, d, n = rp.ripple_export_edges(self.ctx, direction, want.size + 16)
            assert n == want.size, (direction, n, want.size)
            got = np.sort(s.astype(np.int64) * self.cap + d)
            assert np.array_equal(got, want), f"adjacency {direction} differs from the oracle's edge set"
        deg_in, alive = rp.ripple_get_degrees(self.ctx, 1, self.cap)
        assert np.array_equal(alive, self.ora.alive)
        assert np.array_equal(deg_in, np.bincount(dst, minlength=self.cap))
        deg_out, _ = rp.ripple_get_degrees(self.ctx, 0, self.cap)
        assert np.array_equal(deg_out, np.bincount(src, minlength=self.cap))

    def step(self, ops, payload, check=True, tol=None):
        """Apply one batch on both sides; compare acceptance, affected sets and (optionally) all rows."""
        before = [self.gpu_layer(l) for l in range(self.L + 1)] if check else None
        pruned = self.first_mono is not None
        ora_before = oracle.full_recompute(self.ora, self.model) if (pruned and check) else None
        rec = self.ora.apply_batch(ops, payload)
        res = rp.ripple_apply_updates(self.ctx, ops, payload)
        assert res.n_applied == int(rec.accepted.sum()), (res.n_applied, int(rec.accepted.sum()))
        assert res.n_rejected == int((~rec.accepted).sum())
        assert res.n_edges == self.ora.n_edges()
        assert res.n_alive == int(self.ora.alive.sum())
        sets = oracle.affected_sets(self.ora, rec, self.model)
        got_sets = []
        for l in range(self.L + 1):
            got, n = rp.ripple_get_affected(self.ctx, l, self.cap)
            got = got.astype(np.int64)
            got_sets.append(got)
            assert n == res.affected[l] == len(got)
            if pruned and l >= self.first_mono:               # any set between the two bounds is valid
                assert np.all(np.diff(got) > 0)
                assert np.isin(got, sets[l]).all(), f"layer {l}: reported vertices outside the topological set"
            else:
                assert n == len(sets[l]), (l, n, len(sets[l]))
                assert np.array_equal(got, sets[l]), f"affected set of layer {l} differs"
        self.last_topological = sets
        if check:
            errs, want = self.check_embeddings(tol)
            if pruned:                                        # every row whose value really changes is reported
                for l in range(self.first_mono, self.L + 1):
                    scale = max(1e-30, float(np.abs(want[l]).max()))
                    moved = np.flatnonzero((np.abs(want[l] - ora_before[l]).max(axis=1) > 1e-3 * scale) & self.ora.alive)
                    assert np.isin(moved, got_sets[l]).all(), f"layer {l}: a changed row is missing from the reported set"
            for l in range(self.L + 1):                       # rows outside A_l keep their bits
                after = self.gpu_layer(l)
                clean = np.ones(self.cap, dtype=bool)
                clean[got_sets[l]] = False
                clean[list(rec.removed)] = False
                assert np.array_equal(after[clean], before[l][clean]), f"layer {l}: a clean row changed"
        return res, rec, sets


def make_pair(n=300, e=1500, d0=12, kind="gcn_sum", widths=(12, 20, 8), store="f32", seed=0, slack=64,
              gamma=2.1, top_share=0.03, edge_capacity=None, project_first=True, self_cache=True, deterministic=False,
              weighted=False, split=None, packed=None):
    src, dst, out_law, in_law = ri.chung_lu_graph(n, e, gamma, top_share, seed)
    feats = ri.features(n, d0, seed + 1)
    model = ri.make_model(kind, widths, seed + 2)
    weights = ri.edge_weights(len(src), seed + 3) if weighted else None
    pair = Pair(n, n + slack, src, dst, feats, model, store=store, edge_capacity=edge_capacity,
                project_first=project_first, self_cache=self_cache, deterministic=deterministic, weights=weights,
                split=split, packed=packed)
    return pair, (src, dst, out_law, in_law)


def make_stream(pair, graph, mix, seed, weighted=False):
    src, dst, out_law, in_law = graph
    return ri.UpdateStream(pair.n, pair.cap, src, dst, out_law, in_law, pair.widths[0], mix, seed, weighted=weighted)


def config_pair(cfg, store=None):
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    feats = ri.features(cfg.n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(cfg.model, cfg.widths, cfg.weight_seed)
    weights = ri.edge_weights(len(src), cfg.graph_seed + 100) if cfg.weighted else None
    pair = Pair(cfg.n, cfg.vertex_capacity, src, dst, feats, model, store=store or cfg.store,
                edge_capacity=cfg.edge_capacity, weights=weights)
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, cfg.mix,
                             cfg.stream_seed, weighted=cfg.weighted)
    return pair, stream
