"""Parity at the benchmark configurations' real sizes, and drift over long
update sequences (the library accumulates into cached sums; the oracle
recomputes from scratch every time)."""
import os
import time

import numpy as np
import pytest

import oracle
import paper_2601_12347_amd as rp
import ripple_inputs as ri
from harness import config_pair, TOL

pytestmark = pytest.mark.gpu


def test_sparse_sage_mean_all_batch_sizes():
    cfg = ri.get_config("sparse_sage_mean")
    print("case", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        pair.check_embeddings()
        for bs in cfg.batch_sizes:
            for rep in range(2):
                print(" batch size", bs, rep, flush=True)
                ops, payload, _ = stream.next_batch(bs)
                res, _, _ = pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_sparse_gcn_weighted_sum():
    """The paper's GC-W workload on the sparse graph: all rows of all layers after every batch."""
    cfg = ri.get_config("sparse_gcn_wsum")
    print("case", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        pair.check_embeddings()
        for b, bs in enumerate([10, 1000, 1000]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_sparse_gcn_max():
    """The paper's GC-X workload on the sparse graph: all rows of all layers after every batch; the
    reported sets between the rows that changed and the topological sets."""
    cfg = ri.get_config("sparse_gcn_max")
    print("case", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        pair.check_embeddings()
        for b, bs in enumerate([10, 1000, 1000]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            res, _, sets = pair.step(ops, payload)
            print("  reported", [res.affected[l] for l in range(pair.L + 1)], "topological", [len(s) for s in sets],
                  "unchanged/incremental/recomputed", [(res.mono_unchanged[l], res.mono_incremental[l], res.mono_recomputed[l])
                                                       for l in range(1, pair.L + 1)], flush=True)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_sparse_graph_attention():
    """The paper's GA-A workload on the sparse graph: all rows of all layers after every batch."""
    cfg = ri.get_config("sparse_gat")
    print("case", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        pair.check_embeddings()
        for b, bs in enumerate([10, 1000, 1000]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_sparse_four_layers():
    """Four hops (the paper's deeper models, Sec. 6.3.2): all rows of all five layers after every batch."""
    cfg = ri.get_config("sparse_sage_mean_4layer")
    print("case", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        assert pair.L == 4
        pair.check_embeddings()
        for b, bs in enumerate([1, 100, 1000]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            res, _, sets = pair.step(ops, payload)
            print("  a_l", [len(s) for s in sets], flush=True)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_sparse_gin_sum_with_vertex_operations():
    cfg = ri.get_config("sparse_gin_sum")
    print("case", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        for b in range(3):
            print(" batch", b, flush=True)
            ops, payload, n_upd = stream.next_batch(cfg.batch_sizes[0])
            assert n_upd == 1000 and len(ops) == 1000 + 50 * 8
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_drift_over_1000_batches_tiny():
    """1,000 consecutive batches; compared with from-scratch recomputation at checkpoints."""
    cfg = ri.get_config("tiny_gcn_sum")
    print("case drift", cfg.name, flush=True)
    pair, stream = config_pair(cfg)
    try:
        worst = 0.0
        for b in range(1, 1001):
            ops, payload, _ = stream.next_batch(cfg.batch_sizes[0])
            rec = pair.ora.apply_batch(ops, payload)
            res = rp.ripple_apply_updates(pair.ctx, ops, payload)
            assert res.n_applied == int(rec.accepted.sum())
            if b in (1, 10, 100, 500, 1000):
                errs, _ = pair.check_embeddings()
                worst = max(worst, max(errs))
                print(f"  batch {b}: max rel err per layer {['%.2e' % e for e in errs]}", flush=True)
        pair.check_graph()
        pair.check_aggregates()
        assert worst <= TOL["f32"]
    finally:
        pair.close()


@pytest.mark.parametrize("kind", ["gat", "gcn_max", "gcn_wsum"])
def test_drift_of_the_other_aggregators(kind):
    """400 consecutive batches on a small graph. Attention numerators and denominators and weighted sums are
    patched with differences batch after batch (rounding could pile up); max / min aggregates are exact
    selections and must not drift at all."""
    cfg = ri.get_config("tiny_gcn_sum")
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    feats = ri.features(cfg.n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(kind, cfg.widths, cfg.weight_seed)
    weighted = kind == "gcn_wsum"
    weights = ri.edge_weights(len(src), 7) if weighted else None
    from harness import Pair
    print("case drift", kind, flush=True)
    pair = Pair(cfg.n, cfg.vertex_capacity, src, dst, feats, model, edge_capacity=cfg.edge_capacity, weights=weights)
    mix = {"edge_add": 0.39, "edge_del": 0.29, "feat": 0.3, "vadd": 0.01, "vdel": 0.01}
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, mix, 99, weighted=weighted)
    try:
        worst = 0.0
        for b in range(1, 401):
            ops, payload, _ = stream.next_batch(60)
            rec = pair.ora.apply_batch(ops, payload)
            res = rp.ripple_apply_updates(pair.ctx, ops, payload)
            assert res.n_applied == int(rec.accepted.sum())
            if b in (1, 10, 100, 400):
                errs, _ = pair.check_embeddings()
                worst = max(worst, max(errs))
                print(f"  batch {b}: max rel err per layer {['%.2e' % e for e in errs]}", flush=True)
        pair.check_graph()
        pair.check_aggregates()
        assert worst <= TOL["f32"]
    finally:
        pair.close()


def test_drift_bf16_store_sparse_graph():
    """bfloat16 embeddings with float32 cached sums: error stays bounded over many batches."""
    cfg = ri.get_config("sparse_gin_sum")            # the graph and stream (with vertex operations) of config 3
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    feats = ri.features(cfg.n, 100, cfg.feat_seed)
    model = ri.make_model("gcn_sum", (100, 256, 256, 47), cfg.weight_seed)
    from harness import Pair
    print("case drift bf16", flush=True)
    pair = Pair(cfg.n, cfg.vertex_capacity, src, dst, feats, model, store="bf16", edge_capacity=cfg.edge_capacity)
    mix = {"edge_add": 0.49, "edge_del": 0.294, "feat": 0.196, "vadd": 0.01, "vdel": 0.01}
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, 100, mix, 77)
    try:
        for b in range(1, 101):
            ops, payload, _ = stream.next_batch(1000)
            rec = pair.ora.apply_batch(ops, payload)
            res = rp.ripple_apply_updates(pair.ctx, ops, payload)
            assert res.n_applied == int(rec.accepted.sum())
            if b in (1, 10, 100):
                errs, _ = pair.check_embeddings()
                print(f"  batch {b}: max rel err per layer {['%.2e' % e for e in errs]}", flush=True)
        pair.check_graph()
        pair.check_aggregates(tol=1e-3)
    finally:
        pair.close()


@pytest.fixture(scope="module")
def dense_graph():
    cfg = ri.get_config("dense_sage_mean")
    t0 = time.time()
    g = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    print(f" dense graph generated in {time.time() - t0:.0f}s", flush=True)
    return g


def cone_check(ctx, ora, cfg, model, rec, sets, rng, pruned, t0, small=False):
    """A sample of final-layer rows (affected ones, sinks of changed edges, updated vertices) recomputed
    by the oracle through their in-neighbourhood cones and compared layer by layer."""
    L = len(model)
    # (the max / min oracle gathers every neighbour row explicitly: a smaller sample keeps it to seconds;
    # rows the library pruned are sampled too and must equal the recomputation all the same)
    k_any, k_sink, k_feat = (24, 8, 4) if pruned else ((40, 14, 6) if small else (120, 40, 20))
    targets = np.unique(np.concatenate([rng.choice(sets[L], size=k_any, replace=False),
                                        np.asarray(sorted(rec.sinks))[:k_sink],
                                        np.asarray(sorted(rec.feat))[:k_feat]]))
    cone = oracle.recompute_rows(ora, model, targets)
    print(f"  oracle cone {time.time() - t0:.0f}s rows per layer {[len(r) for r, _ in cone]}", flush=True)
    tol = TOL[cfg.store]
    worst = 0.0
    for l in range(L + 1):
        rows, want = cone[l]
        if len(rows) > 200_000:                      # compare a slice of the huge lower layers
            pick = rng.choice(len(rows), size=200_000, replace=False)
            rows, want = rows[pick], want[pick]
        got = rp.ripple_get_embeddings(ctx, l, cfg.widths[l], ids=rows.astype(np.uint32))
        norm = np.abs(want).max(axis=1)
        tau = norm.mean()
        err = (np.abs(got - want).max(axis=1) / np.maximum(norm, tau)).max()
        print(f"  layer {l}: {len(rows)} rows, max rel err {err:.2e}", flush=True)
        assert err <= tol, (l, err)
        worst = max(worst, err)
    return worst


@pytest.mark.parametrize("name", ["dense_sage_mean", "dense_gcn_sum_bf16", "dense_gcn_max"])
def test_dense_configs_sampled_rows(dense_graph, name):
    """Full-size graph, the batch size the benchmark times; the oracle recomputes a sample of
    final-layer rows through their in-neighbourhood cones (recomputing all 2.4M rows of every
    layer in fp64 takes minutes), and the affected sets are compared in full."""
    cfg = ri.get_config(name)
    src, dst, out_law, in_law = dense_graph
    feats = ri.features(cfg.n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(cfg.model, cfg.widths, cfg.weight_seed)
    print("case", name, flush=True)
    t0 = time.time()
    ctx = rp.ripple_init_graph(cfg.n, cfg.vertex_capacity, src, dst, feats, store=cfg.store,
                               edge_capacity=cfg.edge_capacity)
    try:
        rp.ripple_load_model(ctx, model)
        rp.ripple_full_infer(ctx)
        print(f"  gpu bootstrap {time.time() - t0:.0f}s", flush=True)
        stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, cfg.mix,
                                 cfg.stream_seed)
        ora = oracle.GraphState(cfg.n, cfg.vertex_capacity, src, dst, feats)
        print(f"  oracle state {time.time() - t0:.0f}s", flush=True)
        bs = max(cfg.batch_sizes)
        # two batches: the kernels a hop uses in the steady state (the scan of all in-rows that also finds the
        # hop's set, where the previous batch came near its threshold) only start with the second one
        for b in range(2):
            ops, payload, _ = stream.next_batch(bs)
            rec = ora.apply_batch(ops, payload)
            res = rp.ripple_apply_updates(ctx, ops, payload)
            assert res.n_applied == int(rec.accepted.sum()) and res.n_rejected == 0
            assert res.n_edges == ora.n_edges()
            print(f"  batch {b}: hop modes {list(res.hop_mode[1:len(model) + 1])} messages "
                  f"{list(res.messages[1:len(model) + 1])}", flush=True)
        if not cfg.model.endswith(("_max", "_min")):
            # what the benchmark times: the last hop sends along more than an eighth of all edges and is
            # handled by the discovering scan; the first hop pushes
            L_ = len(model)
            assert res.messages[L_] * 8 >= res.n_edges and res.hop_mode[L_] == 3, list(res.hop_mode)
            assert res.hop_mode[1] == 1, list(res.hop_mode)
            # ... and the hop between them (4.6 M messages, 110 M in-row entries) is scattered from the sorted
            # list of its messages
            assert res.hop_mode[2] == 4, list(res.hop_mode)
        sets = oracle.affected_sets(ora, rec, model)
        print(f"  oracle sets {time.time() - t0:.0f}s sizes {[len(s) for s in sets]}", flush=True)
        L = len(model)
        pruned = cfg.model.endswith(("_max", "_min"))
        for l in range(L + 1):
            got, n = rp.ripple_get_affected(ctx, l, cfg.vertex_capacity)
            if pruned and l >= 1:                        # a valid pruned set lies inside the topological one
                assert n == len(got) and np.all(np.diff(got.astype(np.int64)) > 0)
                assert np.isin(got.astype(np.int64), sets[l]).all(), f"affected set {l}"
                print(f"  layer {l}: reported {n} of {len(sets[l])}; unchanged/incremental/recomputed "
                      f"{res.mono_unchanged[l]}/{res.mono_incremental[l]}/{res.mono_recomputed[l]}", flush=True)
            else:
                assert n == len(sets[l]) and np.array_equal(got.astype(np.int64), sets[l]), f"affected set {l}"
        rng = np.random.default_rng(5)
        cone_check(ctx, ora, cfg, model, rec, sets, rng, pruned, t0)
    finally:
        rp.ripple_destroy(ctx)


@pytest.mark.parametrize("name,bs,det", [("dense_sage_mean_4layer", 1000, 0), ("reddit_sage_mean", 1000, 0),
                                         ("dense_gat", 10000, 0), ("dense_gcn_wsum", 10000, 0),
                                         ("dense_sage_mean", 10000, 1), ("dense_sage_mean", (10000, 1000, 10000), 0)])
def test_deep_and_reddit_shaped_configs(dense_graph, name, bs, det):
    """Four layers on the dense graph, a graph of Reddit's shape (average in-degree 492, 602
    features), attention, the weighted sum (one weight per edge) and the deterministic mode of the headline model
    (60 K runs of chunks, two side entries each) at full size; and a sequence of batch sizes (10,000, 1,000, 10,000)
    that makes the size the host sorts the second hop's messages for too small for the third batch, which then has
    to fall back to the pull on the device. Affected sets are compared in full. At this density the in-neighbourhood cone of even
    a handful of final-layer rows is most of the graph, so the rows are checked hop by hop instead:
    for a sample of A_l the oracle applies layer l (fp64) to the library's own stored H^{l-1}, which
    an earlier step of the same loop has checked the same way, down to the features."""
    cfg = ri.get_config(name)
    if cfg.n == 2_449_029:
        src, dst, out_law, in_law = dense_graph
    else:
        t0 = time.time()
        src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
        print(f" graph generated in {time.time() - t0:.0f}s", flush=True)
    feats = ri.features(cfg.n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(cfg.model, cfg.widths, cfg.weight_seed)
    print("case", name, "deterministic" if det else "", flush=True)
    t0 = time.time()
    weights = ri.edge_weights(len(src), cfg.graph_seed + 100) if cfg.weighted else None
    if weights is None:
        ctx = rp.ripple_init_graph(cfg.n, cfg.vertex_capacity, src, dst, feats, store=cfg.store,
                                   edge_capacity=cfg.edge_capacity)
    else:
        ctx = rp.ripple_init_graph_weighted(cfg.n, cfg.vertex_capacity, src, dst, weights, feats, store=cfg.store,
                                            edge_capacity=cfg.edge_capacity)
    try:
        if det:
            rp.ripple_set_option(ctx, rp.OPT_DETERMINISTIC, 1)
        rp.ripple_load_model(ctx, model)
        rp.ripple_full_infer(ctx)
        stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, cfg.mix,
                                 cfg.stream_seed, weighted=cfg.weighted)
        ora = oracle.GraphState(cfg.n, cfg.vertex_capacity, src, dst, feats, weights=weights)
        print(f"  bootstrap and oracle state {time.time() - t0:.0f}s", flush=True)
        L = len(model)
        rng = np.random.default_rng(6)
        sizes = bs if isinstance(bs, tuple) else (bs, bs)
        modes = []
        for b, nb in enumerate(sizes):
            ops, payload, _ = stream.next_batch(nb)
            rec = ora.apply_batch(ops, payload)
            res = rp.ripple_apply_updates(ctx, ops, payload)
            assert res.n_applied == int(rec.accepted.sum()) and res.n_rejected == 0
            assert res.n_edges == ora.n_edges()
            sets = oracle.affected_sets(ora, rec, model)
            for l in range(L + 1):
                got, n = rp.ripple_get_affected(ctx, l, cfg.vertex_capacity)
                assert n == len(sets[l]) and np.array_equal(got.astype(np.int64), sets[l]), f"affected set {l}"
            modes.append(list(res.hop_mode[1:L + 1]))
            print(f"  batch {b}: sets {[len(s) for s in sets]} hop modes {modes[-1]} {time.time() - t0:.0f}s", flush=True)
        if isinstance(bs, tuple):
            # the 1,000-update batch takes hop 2 from the sorted list (sized by the batch before it); the batch after it
            # has fifteen times as many messages as the host sorted room for and is pulled
            assert modes[1][1] == 4 and modes[2][1] == 2, modes
        a_in = oracle.in_adjacency(ora)
        touched = np.asarray(sorted(rec.feat), dtype=np.int64)
        got0 = rp.ripple_get_embeddings(ctx, 0, cfg.widths[0], ids=touched.astype(np.uint32))
        assert np.array_equal(got0, ora.h0[touched].astype(np.float32))
        for l in range(1, L + 1):
            rows = np.unique(np.concatenate([rng.choice(sets[l], size=min(300, len(sets[l])), replace=False),
                                             np.asarray(sorted(rec.sinks), dtype=np.int64)[:60]]))
            # the rows of H^{l-1} that layer l reads for this sample, from the library
            need = np.union1d(np.unique(a_in.ones[rows].indices), rows)
            h_prev = np.zeros((cfg.vertex_capacity, cfg.widths[l - 1]))
            h_prev[need] = rp.ripple_get_embeddings(ctx, l - 1, cfg.widths[l - 1], ids=need.astype(np.uint32))
            want = oracle.layer_rows(ora, model[l - 1], h_prev, a_in, rows)
            got = rp.ripple_get_embeddings(ctx, l, cfg.widths[l], ids=rows.astype(np.uint32))
            norm = np.abs(want).max(axis=1)
            err = (np.abs(got - want).max(axis=1) / np.maximum(norm, norm.mean())).max()
            print(f"  layer {l}: {len(rows)} rows from {len(need)} inputs, max rel err {err:.2e} {time.time() - t0:.0f}s",
                  flush=True)
            assert err <= TOL[cfg.store], (l, err)
        if det:
            # a second context fed the same operations ends up with the same bits (all rows of the last layer, a
            # sample of 200,000 rows of every other layer)
            ctx2 = rp.ripple_init_graph(cfg.n, cfg.vertex_capacity, src, dst, feats, store=cfg.store,
                                        edge_capacity=cfg.edge_capacity)
            try:
                rp.ripple_set_option(ctx2, rp.OPT_DETERMINISTIC, 1)
                rp.ripple_load_model(ctx2, model)
                rp.ripple_full_infer(ctx2)
                stream2 = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, cfg.mix,
                                          cfg.stream_seed, weighted=cfg.weighted)
                for nb in sizes:
                    ops, payload, _ = stream2.next_batch(nb)
                    rp.ripple_apply_updates(ctx2, ops, payload)
                ids = np.sort(rng.choice(cfg.n, size=200_000, replace=False)).astype(np.uint32)
                for l in range(1, L + 1):
                    pick = None if l == L else ids
                    kw = dict(n_rows=cfg.vertex_capacity) if pick is None else dict(ids=pick)
                    one = rp.ripple_get_embeddings(ctx, l, cfg.widths[l], **kw)
                    two = rp.ripple_get_embeddings(ctx2, l, cfg.widths[l], **kw)
                    assert np.array_equal(one.view(np.uint32), two.view(np.uint32)), f"layer {l}: bits differ between two contexts"
                print(f"  two contexts agree bit for bit {time.time() - t0:.0f}s", flush=True)
            finally:
                rp.ripple_destroy(ctx2)
    finally:
        rp.ripple_destroy(ctx)


def test_dense_bf16_1000_consecutive_batches(dense_graph, tmp_path):
    """The fifth configuration as stated: 1,000 consecutive batches of 10,000 updates (2% vertex additions and
    deletions) on the 2.45 M-vertex graph with bf16 storage. Counts are compared after every batch; at
    batches 1, 10, 100 and 1,000 the affected sets are compared in full and sampled rows against the
    oracle's recomputation, so drift of the cached sums would show. The batches are drawn by a second
    process (the same seeded stream) while this one applies the previous batch to the oracle and the GPU."""
    cfg = ri.get_config("dense_gcn_sum_bf16")
    src, dst, out_law, in_law = dense_graph
    feats = ri.features(cfg.n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(cfg.model, cfg.widths, cfg.weight_seed)
    print("case long run", cfg.name, flush=True)
    t0 = time.time()
    stream = None
    ctx = rp.ripple_init_graph(cfg.n, cfg.vertex_capacity, src, dst, feats, store=cfg.store, edge_capacity=cfg.edge_capacity)
    try:
        rp.ripple_load_model(ctx, model)
        rp.ripple_full_infer(ctx)
        ri.BatchProducer.save_graph(str(tmp_path), src, dst)
        stream = ri.BatchProducer(cfg.name, str(tmp_path), 10000, 1000)
        ora = oracle.GraphState(cfg.n, cfg.vertex_capacity, src, dst, feats)
        rng = np.random.default_rng(8)
        lat, compactions = [], 0
        for b in range(1, 1001):
            ops, payload, _ = stream.next_batch()
            rec = ora.apply_batch(ops, payload)
            t1 = time.perf_counter()
            res = rp.ripple_apply_updates(ctx, ops, payload)
            lat.append(time.perf_counter() - t1)
            compactions += res.n_compactions
            assert res.n_applied == int(rec.accepted.sum()) and res.n_edges == ora.n_edges()
            assert res.n_alive == int(ora.alive.sum())
            if b % 50 == 0:
                print(f"  batch {b}: {time.time() - t0:.0f}s, median {np.median(lat) * 1e3:.2f} ms per batch (host buffers), "
                      f"{compactions} compactions", flush=True)
            if b in (1, 10, 100, 1000):
                sets = oracle.affected_sets(ora, rec, model)
                for l in range(len(model) + 1):
                    got, n = rp.ripple_get_affected(ctx, l, cfg.vertex_capacity)
                    assert n == len(sets[l]) and np.array_equal(got.astype(np.int64), sets[l]), f"affected set {l}"
                print(f"  batch {b}: sets {[len(x) for x in sets]}", flush=True)
                cone_check(ctx, ora, cfg, model, rec, sets, rng, False, t0, small=b in (10, 100))
    finally:
        if stream is not None:
            stream.close()
        for f in ("src.npy", "dst.npy"):
            if os.path.exists(tmp_path / f):
                os.remove(tmp_path / f)
        rp.ripple_destroy(ctx)
