"""ripple_apply_updates against the oracle: after every batch the affected
sets are identical, every row of every layer matches full recomputation within
tolerance (the paper's exactness claim, Sec. 3.3.3 and Sec. 5), rows outside
the affected sets keep their bits, and the cached sums stay consistent."""
import numpy as np
import pytest

import oracle
import paper_2601_12347_amd as rp
import ripple_inputs as ri
from harness import make_pair, make_stream, config_pair

pytestmark = pytest.mark.gpu

MIX3 = {"edge_add": 0.5, "edge_del": 0.3, "feat": 0.2, "vadd": 0.0, "vdel": 0.0}
MIXV = {"edge_add": 0.4, "edge_del": 0.3, "feat": 0.2, "vadd": 0.05, "vdel": 0.05}


@pytest.mark.parametrize("kind,widths", [
    ("gcn_sum", (12, 20, 8)),
    ("sage_mean", (16, 40, 24, 10)),
    ("gin_sum", (16, 32, 12)),
    ("gcn_mean", (10, 35, 9)),
])
def test_edge_and_feature_updates(kind, widths):
    print("case", kind, widths, flush=True)
    pair, graph = make_pair(n=600, e=4000, d0=widths[0], kind=kind, widths=widths, seed=11)
    stream = make_stream(pair, graph, MIX3, 21)
    try:
        for b, bs in enumerate([1, 10, 50, 100, 7]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("kind,widths", [("gcn_sum", (12, 20, 8)), ("sage_mean", (16, 24, 10)),
                                         ("gin_sum", (16, 32, 12))])
def test_vertex_additions_and_deletions(kind, widths):
    print("case vertex ops", kind, flush=True)
    pair, graph = make_pair(n=500, e=3500, d0=widths[0], kind=kind, widths=widths, seed=13, slack=128)
    stream = make_stream(pair, graph, MIXV, 23)
    try:
        for b in range(5):
            print(" batch", b, flush=True)
            ops, payload, _ = stream.next_batch(40)
            pair.step(ops, payload)
            pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("kind,widths", [("sage_mean", (16, 40, 24, 10)), ("gcn_sum", (100, 256, 70)),
                                         ("gin_sum", (16, 32, 12, 6))])
def test_push_and_pull_scatter_agree_with_oracle(mode, kind, widths):
    """Every way of moving the deltas (float atomics from the sources; segmented reduction over
    the in-rows of A_l; one scan of all in-rows that also finds A_l) must give the same result."""
    print("case scatter mode", mode, kind, flush=True)
    pair, graph = make_pair(n=900, e=9000, d0=widths[0], kind=kind, widths=widths, seed=51, slack=128)
    rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, mode)
    stream = make_stream(pair, graph, MIXV, 53)
    try:
        for b, bs in enumerate([3, 40, 200]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("sorted_opt", [0, 1, 2])
@pytest.mark.parametrize("kind,widths,project_first", [("sage_mean", (16, 40, 24, 10), 1), ("gcn_sum", (100, 256, 70), 0),
                                                       ("gcn_sum", (12, 300, 520, 20), 1), ("gin_sum", (16, 32, 12, 6), 1)])
def test_sorted_messages_agree_with_oracle(sorted_opt, kind, widths, project_first):
    """Hops scattered from the list of their messages, written down by the out-edge walk and sorted by destination,
    against the same hops pulled through the in-rows (option 0) and against the oracle: every row of every layer,
    the cached aggregates and the sets after every batch. Option 2 takes the list wherever a hop is pulled (the
    scatter mode is forced to pull so that hops of a few messages get there, and the report says so); option 1
    leaves the choice to the previous batch's counts. Rows of up to 520 columns, project-first layers on and off
    (unpacked projected rows travel through the list as well), a batch with more messages than the one before."""
    print("case sorted messages", sorted_opt, kind, widths, flush=True)
    pair, graph = make_pair(n=900, e=9000, d0=widths[0], kind=kind, widths=widths, seed=61, slack=128,
                            project_first=bool(project_first), packed=False)
    rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, 2)
    rp.ripple_set_option(pair.ctx, rp.OPT_SORTED_MESSAGES, sorted_opt)
    rp.ripple_set_option(pair.ctx, rp.OPT_SPARSE_FRONTIER, 0)    # hops that list their set while marking write no message list
    stream = make_stream(pair, graph, MIXV, 63)
    L = len(widths) - 1
    try:
        for b, bs in enumerate([3, 40, 200, 30, 400]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            res, _, _ = pair.step(ops, payload)
            modes = list(res.hop_mode[1:L + 1])
            print("  hop modes", modes, "messages", list(res.messages[1:L + 1]), flush=True)
            if sorted_opt == 2:
                assert all(m == 4 for m, msgs in zip(modes[1:], list(res.messages[2:L + 1])) if msgs), modes
            if sorted_opt == 0:
                assert 4 not in modes, modes
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


STREAM_CASES = [(mode, kind, widths, weighted) for kind, widths, weighted in
                [("sage_mean", (24, 256, 256, 40), False), ("gcn_sum", (24, 256, 256, 256, 12), False),
                 ("gcn_wsum", (16, 256, 256, 30), True), ("sage_mean", (24, 256, 256, 256), False),
                 ("sage_mean", (24, 256, 256, 24), False)]
                for mode in (0, 1, 2, 3) if not (weighted and mode == 1)]


@pytest.mark.parametrize("mode,kind,widths,weighted", STREAM_CASES)
def test_streaming_row_update_at_any_size(mode, kind, widths, weighted):
    """Layers of 256 -> 256 forced onto the persistent streaming row update whatever the number of rows (it is chosen
    for large hops only otherwise): hops of a handful of rows, of less than a tile, of a few tiles with a ragged last
    one. Every row of every layer, the cached aggregates and the sets against the oracle after every batch, in
    every scatter mode, with delta rows written (a 256 -> 256 layer before another) and without (before a
    project-first layer, or last), with and without a cached self term. The same option forces the kernel that takes
    both products of a narrow project-first GraphSAGE layer in one pass (256 -> 40: packed messages, 256 -> 24:
    one-line fp32 messages) onto these small hops and onto the bootstrap."""
    print("case streaming row update", mode, kind, widths, flush=True)
    pair, graph = make_pair(n=1300, e=14000, d0=widths[0], kind=kind, widths=widths, seed=171, slack=96, weighted=weighted)
    rp.ripple_set_option(pair.ctx, rp.OPT_STREAM_TRANSFORM, 2)
    rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, mode)
    rp.ripple_full_infer(pair.ctx)                       # the bootstrap through the streaming kernel as well
    stream = make_stream(pair, graph, MIXV, 173, weighted=weighted)
    try:
        pair.check_embeddings()
        for b, bs in enumerate([1, 30, 250, 250, 5]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates()
        pair.check_graph()
    finally:
        pair.close()


PACKED_CASES = [(mode, *case) for case in [("sage_mean", (12, 96, 47), "f32", False), ("gcn_sum", (80, 33), "f32", False),
                                           ("gcn_wsum", (16, 100, 40), "f32", True), ("gcn_sum", (24, 88, 44), "bf16", False)]
                for mode in (0, 1, 2, 3) if not (case[3] and mode == 1)]      # weighted layers have no push kernel


@pytest.mark.parametrize("mode,kind,widths,store,weighted", PACKED_CASES)
def test_packed_messages(mode, kind, widths, store, weighted):
    """Project-first layers of 33 to 47 columns send one-line packed messages (21 to 24-bit block floating point,
    the rounding error of a message carried into the sender's next one): every way of moving them (push, pull,
    discovering scan) matches the oracle to the fp32 tolerance, the cached aggregates stay the sum of the
    projected rows, and a twin context with the option off reports the same sets."""
    print("case packed messages", mode, kind, widths, store, flush=True)
    kw = dict(n=700, e=6500, d0=widths[0], kind=kind, widths=widths, seed=131, slack=96, store=store, weighted=weighted)
    pair, graph = make_pair(**kw)
    plain, _ = make_pair(packed=False, **kw)
    L = len(widths) - 1
    assert rp.ripple_layer_packs_messages(pair.ctx, L) and not rp.ripple_layer_packs_messages(plain.ctx, L)
    assert rp.ripple_get_layer_info(pair.ctx, L)[:2] == (widths[-1], True)
    rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, mode)
    rp.ripple_set_option(plain.ctx, rp.OPT_SCATTER_MODE, mode)
    stream = make_stream(pair, graph, MIXV, 133, weighted=weighted)
    tol = 1e-3 if store == "bf16" else None
    try:
        pair.check_aggregates(tol=tol)
        for b, bs in enumerate([4, 50, 160, 30, 90]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            res, _, _ = pair.step(ops, payload)
            res2 = rp.ripple_apply_updates(plain.ctx, ops, payload)
            assert list(res.affected) == list(res2.affected) and list(res.messages) == list(res2.messages)
            # against the unpacked twin the rows differ by far less than the tolerance allows
            a = pair.gpu_layer(L)
            b_ = plain.gpu_layer(L)
            scale = max(1e-30, float(np.abs(b_).max()))
            assert float(np.abs(a - b_).max()) <= (2e-2 if store == "bf16" else 2e-5) * scale
        pair.check_graph()
        pair.check_aggregates(tol=tol)
    finally:
        pair.close()
        plain.close()


def test_packed_messages_do_not_drift():
    """300 batches on a small graph: every vertex sends many messages; the cached aggregates of the packed
    layer must stay the sum of the stored rows' projections (what a message loses to rounding is in the next)."""
    print("case packed drift", flush=True)
    pair, graph = make_pair(n=400, e=3600, d0=10, kind="sage_mean", widths=(10, 96, 47), seed=141, slack=800)
    assert rp.ripple_layer_packs_messages(pair.ctx, 2)
    stream = make_stream(pair, graph, MIXV, 143)
    try:
        for b in range(300):
            ops, payload, _ = stream.next_batch(40)
            pair.step(ops, payload, check=(b % 60 == 59))
        pair.check_aggregates()
        errs, _ = pair.check_embeddings()
        print(" errors after 300 batches", ["%.2e" % e for e in errs], flush=True)
    finally:
        pair.close()


@pytest.mark.parametrize("kind,widths,store", [("sage_mean", (16, 40, 24, 10), "f32"), ("gcn_sum", (100, 256, 47), "f32"),
                                               ("gcn_mean", (32, 64, 12), "bf16")])
@pytest.mark.parametrize("project_first", [True, False])
def test_project_first_layers(kind, widths, store, project_first):
    """Narrow output layers cache sum_u H[u] W_neigh and scatter d_out-wide messages; switching
    that off must give the same embeddings, and both must match the oracle."""
    print("case project-first", project_first, kind, store, flush=True)
    pair, graph = make_pair(n=800, e=7000, d0=widths[0], kind=kind, widths=widths, seed=61, slack=128, store=store,
                            project_first=project_first)
    L = len(widths) - 1
    assert rp.ripple_get_layer_info(pair.ctx, L)[:2] == ((widths[-1], True) if project_first else (widths[-2], False))
    stream = make_stream(pair, graph, MIXV, 63)
    try:
        pair.check_aggregates(tol=1e-3 if store == "bf16" else None)
        for b, bs in enumerate([5, 60, 150]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates(tol=1e-3 if store == "bf16" else None)
    finally:
        pair.close()


@pytest.mark.parametrize("store", ["f32", "bf16"])
@pytest.mark.parametrize("self_cache", [True, False])
@pytest.mark.parametrize("project_first", [True, False])
def test_cached_self_projection(store, self_cache, project_first):
    """Layers that concatenate the vertex's own embedding keep H[v] W_self per vertex and refresh it
    only on A_{l-1}; with the cache switched off the full [h | x] product runs. Both must match the
    oracle, with and without project-first on the narrow last layer."""
    print("case self cache", store, self_cache, project_first, flush=True)
    widths = (20, 48, 36, 12)
    pair, graph = make_pair(n=700, e=6000, d0=widths[0], kind="sage_mean", widths=widths, seed=71, slack=128,
                            store=store, project_first=project_first, self_cache=self_cache)
    for l in range(1, 4):
        assert rp.ripple_get_layer_info(pair.ctx, l)[2] == self_cache
    stream = make_stream(pair, graph, MIXV, 73)
    try:
        for b, bs in enumerate([4, 70, 160]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_aggregates(tol=1e-3 if store == "bf16" else None)
    finally:
        pair.close()


def test_tiny_config_batches():
    cfg = ri.get_config("tiny_gcn_sum")
    print("case tiny config", flush=True)
    pair, stream = config_pair(cfg)
    try:
        for b in range(6):
            print(" batch", b, flush=True)
            ops, payload, _ = stream.next_batch(cfg.batch_sizes[0])
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("kind", ["sage_mean", "gcn_max", "sage_max", "gat", "gin_sum"])
def test_conflicting_operations_keep_array_order(kind):
    print("case conflicts", kind, flush=True)
    pair, graph = make_pair(n=200, e=900, d0=8, kind=kind, widths=(8, 16, 6), seed=17)
    src, dst = graph[0], graph[1]
    u, v = int(src[0]), int(dst[0])
    n = pair.n
    f = np.random.default_rng(5).standard_normal((4, 8)).astype(np.float32)
    ops = np.array([
        (ri.OP_EDGE_DEL, u, v, 0), (ri.OP_EDGE_ADD, u, v, 0), (ri.OP_EDGE_DEL, u, v, 0),   # same edge thrice
        (ri.OP_EDGE_ADD, n, 3, 0),                      # n is not alive yet -> rejected
        (ri.OP_VERTEX_ADD, n, 0, 0), (ri.OP_EDGE_ADD, n, 3, 0), (ri.OP_EDGE_ADD, 4, n, 0),
        (ri.OP_FEAT_UPDATE, n, 0, 1),                   # update of the vertex just created
        (ri.OP_FEAT_UPDATE, 7, 0, 2), (ri.OP_FEAT_UPDATE, 7, 0, 3),                         # twice
        (ri.OP_VERTEX_DEL, 9, 0, 0), (ri.OP_EDGE_ADD, 9, 10, 0),                            # edge on a deleted vertex
        (ri.OP_VERTEX_DEL, n, 0, 0), (ri.OP_VERTEX_ADD, n, 0, 2),                           # delete, re-create
    ], dtype=np.uint32)
    try:
        res, rec, _ = pair.step(ops, f)
        assert res.n_sub_batches > 1
        assert rec.accepted.tolist() == [True, True, True, False, True, True, True, True, True, True,
                                         True, False, True, True]
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_rejected_operations_are_counted_not_fatal():
    print("case rejects", flush=True)
    pair, graph = make_pair(n=200, e=900, d0=8, kind="gcn_sum", widths=(8, 16, 6), seed=18)
    src, dst = graph[0], graph[1]
    ops = np.array([
        (ri.OP_EDGE_ADD, int(src[5]), int(dst[5]), 0),           # exists
        (ri.OP_EDGE_DEL, 0, 0, 0),                               # self-loop never added
        (ri.OP_VERTEX_DEL, pair.cap - 1, 0, 0),                  # dead
        (ri.OP_FEAT_UPDATE, pair.cap - 2, 0, 0),                 # dead
        (ri.OP_VERTEX_ADD, 3, 0, 0),                             # alive
        (ri.OP_EDGE_ADD, 1, pair.cap - 1, 0),                    # dead endpoint
        (ri.OP_EDGE_ADD, 2, 2, 0),                               # a self-loop is legal
    ], dtype=np.uint32)
    try:
        res, rec, _ = pair.step(ops, np.ones((1, 8), np.float32))
        assert res.n_applied == 1 and res.n_rejected == 6
        pair.check_graph()
    finally:
        pair.close()


def test_structural_roundtrip_and_noop_updates():
    print("case roundtrip", flush=True)
    pair, graph = make_pair(n=300, e=1500, d0=8, kind="gcn_sum", widths=(8, 16, 6), seed=19)
    try:
        start = [pair.gpu_layer(l) for l in range(pair.L + 1)]
        add = np.array([(ri.OP_EDGE_ADD, 5, 9, 0)], dtype=np.uint32)
        if pair.ora.has_edge(5, 9):
            add[0, 0] = ri.OP_EDGE_DEL
        back = add.copy()
        back[0, 0] = ri.OP_EDGE_DEL if add[0, 0] == ri.OP_EDGE_ADD else ri.OP_EDGE_ADD
        _, _, sets_a = pair.step(add, None)
        _, _, sets_b = pair.step(back, None)
        for a, b in zip(sets_a, sets_b):
            assert np.array_equal(a, b)
        for l in range(pair.L + 1):
            err = oracle.max_rel_err(pair.gpu_layer(l), start[l], pair.ora.alive)
            assert err <= 1e-5, (l, err)
        # feature "update" to the identical vector: zero delta, rows unchanged
        same = start[0][[4]].copy()
        res, _, _ = pair.step(np.array([(ri.OP_FEAT_UPDATE, 4, 0, 0)], dtype=np.uint32), same)
        assert res.affected[0] == 1
        # empty batch: empty sets, nothing written
        before = pair.gpu_layer(pair.L)
        res = rp.ripple_apply_updates(pair.ctx, np.zeros((0, 4), np.uint32), None)
        assert list(res.affected[: pair.L + 1]) == [0] * (pair.L + 1)
        assert rp.ripple_get_affected(pair.ctx, 1, 8)[1] == 0
        assert np.array_equal(before, pair.gpu_layer(pair.L))
    finally:
        pair.close()


def test_pool_growth_relocation_and_compaction():
    print("case compaction", flush=True)
    # almost no spare edge capacity: rows relocate, the pool fills, compaction must kick in
    pair, graph = make_pair(n=300, e=2000, d0=8, kind="gcn_sum", widths=(8, 16, 6), seed=29,
                            edge_capacity=2600)
    mix = {"edge_add": 0.6, "edge_del": 0.4, "feat": 0.0, "vadd": 0.0, "vdel": 0.0}
    stream = make_stream(pair, graph, mix, 31)
    try:
        compactions = 0
        for b in range(40):
            ops, payload, _ = stream.next_batch(60)
            res, _, _ = pair.step(ops, payload, check=(b % 10 == 9))
            compactions += res.n_compactions
        print(" compactions", compactions, flush=True)
        pair.check_graph()
        rp.ripple_compact(pair.ctx)
        pair.check_graph()
        ops, payload, _ = stream.next_batch(60)
        pair.step(ops, payload)
        # capacity really exhausted -> status, state unchanged
        grow = []
        for u in range(pair.n):
            for v in range(pair.n):
                if u != v and not pair.ora.has_edge(u, v):
                    grow.append((ri.OP_EDGE_ADD, u, v, 0))
                if len(grow) >= 1000:
                    break
            if len(grow) >= 1000:
                break
        with pytest.raises(rp.RippleError) as ei:
            rp.ripple_apply_updates(pair.ctx, np.array(grow, dtype=np.uint32), None)
        assert ei.value.status == rp.binding.RIPPLE_ECAPACITY
        pair.check_graph()
        pair.check_embeddings()
    finally:
        pair.close()


def test_capacity_error_in_a_later_piece_leaves_the_earlier_pieces_applied():
    """A batch that has to be cut (it touches one edge twice) and whose second piece exceeds the edge
    capacity: the call reports the capacity error and how many operations took effect; the state is that
    of exactly those operations, and the next batch goes through."""
    print("case capacity in second piece", flush=True)
    pair, graph = make_pair(n=200, e=1200, d0=8, kind="sage_mean", widths=(8, 16, 6), seed=61, edge_capacity=1204)
    try:
        free = [(u, v) for u in range(40) for v in range(40, 60) if not pair.ora.has_edge(u, v)]
        (a0, b0), (a1, b1) = free[0], free[1]
        first = [(ri.OP_EDGE_ADD, a0, b0, 0), (ri.OP_EDGE_ADD, a1, b1, 0), (ri.OP_FEAT_UPDATE, 7, 0, 0)]
        second = [(ri.OP_EDGE_DEL, a0, b0, 0)] + [(ri.OP_EDGE_ADD, u, v, 0) for u, v in free[2:12]]
        ops = np.array(first + second, dtype=np.uint32)
        payload = np.ones((1, 8), dtype=np.float32)
        assert rp.ripple_plan_batch(ops, pair.cap, 1) == [len(first), len(ops)]
        with pytest.raises(rp.RippleError) as ei:
            rp.ripple_apply_updates(pair.ctx, ops, payload)
        assert ei.value.status == rp.binding.RIPPLE_ECAPACITY
        res = ei.value.result
        assert res.n_ops == len(ops) and res.n_ops_done == len(first) and res.n_sub_batches == 2
        rec = pair.ora.apply_batch(ops[: res.n_ops_done], payload)
        assert res.n_applied == int(rec.accepted.sum()) == 3 and res.n_rejected == 0
        assert res.n_edges == pair.ora.n_edges() == 1202
        sets = oracle.affected_sets(pair.ora, rec, pair.model)
        for l in range(pair.L + 1):
            got, n = rp.ripple_get_affected(pair.ctx, l, pair.cap)
            assert n == res.affected[l] and np.array_equal(got.astype(np.int64), sets[l]), l
        pair.check_graph()
        pair.check_embeddings()
        pair.check_aggregates()
        # a device-resident payload must not have been adopted by the context: the next batch (host payload) works
        stream = make_stream(pair, graph, {"edge_add": 0.0, "edge_del": 0.5, "feat": 0.5, "vadd": 0.0, "vdel": 0.0}, 63)
        stream._add_edge(a0, b0)
        stream._add_edge(a1, b1)
        ops2, payload2, _ = stream.next_batch(20)
        pair.step(ops2, payload2)
    finally:
        pair.close()


def test_attention_scores_beyond_the_float_range_are_reported():
    """Raw exponentials (no maximum subtracted) overflow for scores above about 88. The oracle (fp64) stays finite;
    the library must say so instead of handing out non-finite rows as if nothing had happened: scores around 60
    still match the oracle, scores above 90 make full inference and the next batch return RIPPLE_ERANGE."""
    print("case attention range", flush=True)
    n, e, d0, widths = 300, 1800, 8, (8, 12, 6)
    src, dst, out_law, in_law = ri.chung_lu_graph(n, e, 2.1, 0.03, 151)
    feats = ri.features(n, d0, 152)
    for scale, expect_error in ((11.0, False), (40.0, True)):
        model = ri.make_model("gat", widths, 153)
        for lay in model:                                   # scores grow with the attention vectors
            lay["att"] = (np.asarray(lay["att"]) * scale).astype(np.float32)
        ora = oracle.GraphState(n, n + 16, src, dst, feats)
        want = oracle.full_recompute(ora, model)
        assert all(np.isfinite(w).all() for w in want)
        ctx = rp.ripple_init_graph(n, n + 16, src, dst, feats)
        try:
            rp.ripple_load_model(ctx, model)
            if not expect_error:
                rp.ripple_full_infer(ctx)
                got = rp.ripple_get_embeddings(ctx, 2, widths[2], n_rows=n + 16)
                assert oracle.max_rel_err(got, want[2], ora.alive) <= 1e-4
                continue
            with pytest.raises(rp.RippleError) as ei:
                rp.ripple_full_infer(ctx)
            assert ei.value.status == rp.binding.RIPPLE_ERANGE and "overflow" in str(ei.value)
            # the context stays usable, and a batch that touches such rows reports the same
            ops = np.array([(ri.OP_FEAT_UPDATE, v, 0, i) for i, v in enumerate(range(0, 40))], dtype=np.uint32)
            payload = ri.features(40, d0, 154)
            with pytest.raises(rp.RippleError) as ei:
                rp.ripple_apply_updates(ctx, ops, payload)
            assert ei.value.status == rp.binding.RIPPLE_ERANGE
            assert ei.value.result.n_applied == 40          # the batch was applied all the same
        finally:
            rp.ripple_destroy(ctx)


MIXW = {"edge_add": 0.3, "edge_del": 0.2, "feat": 0.2, "vadd": 0.03, "vdel": 0.02, "reweight": 0.25}


@pytest.mark.parametrize("mode", [0, 2, 3])
@pytest.mark.parametrize("kind,widths", [("gcn_wsum", (12, 24, 10)), ("sage_wsum", (16, 96, 40))])
def test_edge_weight_replacement(mode, kind, widths):
    """The sixth operation: a quarter of the updates replace the weight of an existing edge. The sink's cached
    weighted sums gain (alpha_new - alpha_old) times the source's pre-batch row, later messages carry the new
    weight; sets, rows and cached sums are compared with the oracle after every batch, for every way of moving
    the messages (the second model ends in a packed project-first layer)."""
    print("case edge weight replacement", mode, kind, flush=True)
    pair, graph = make_pair(n=600, e=5000, d0=widths[0], kind=kind, widths=widths, seed=161, slack=128, weighted=True)
    rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, mode)
    stream = make_stream(pair, graph, MIXW, 163, weighted=True)
    try:
        for b, bs in enumerate([8, 60, 200, 40]):
            ops, payload, _ = stream.next_batch(bs)
            n_rw = int((ops[:, 0] == ri.OP_EDGE_REWEIGHT).sum())
            print(" batch", b, bs, "weight replacements", n_rw, flush=True)
            res, rec, _ = pair.step(ops, payload)
            assert n_rw > 0 and res.n_rejected == 0
        pair.check_graph()
        pair.check_aggregates()
        # rejected: missing edge; accepted twice in one batch: cut into two pieces, the later weight stays
        es, ed = pair.ora.edges()
        u, v = int(es[0]), int(ed[0])
        miss = next((a, b) for a in range(20) for b in range(20, 40) if not pair.ora.has_edge(a, b))
        bits = lambda x: int(np.array([x], dtype=np.float32).view(np.uint32)[0])
        ops = np.array([(ri.OP_EDGE_REWEIGHT, u, v, bits(0.5)), (ri.OP_EDGE_REWEIGHT, miss[0], miss[1], bits(1.0)),
                        (ri.OP_EDGE_REWEIGHT, u, v, bits(1.5))], dtype=np.uint32)
        res, rec, _ = pair.step(ops, None)
        assert res.n_applied == 2 and res.n_rejected == 1 and res.n_sub_batches == 2
        pair.check_aggregates()
    finally:
        pair.close()


def test_layers_that_ignore_weights_on_a_weighted_graph():
    """A weighted graph under a model whose first layer aggregates with the weights and whose second takes the
    plain mean: an added or deleted edge counts once for the second layer whatever its weight, and a new weight
    means nothing to it."""
    print("case mixed weighted / unweighted layers", flush=True)
    n, e = 500, 4000
    src, dst, out_law, in_law = ri.chung_lu_graph(n, e, 2.1, 0.03, 171)
    feats = ri.features(n, 12, 172)
    w = ri.edge_weights(len(src), 173)
    first = ri.make_model("gcn_wsum", (12, 20), 174)
    first[0]["act_out"] = "relu"
    model = first + ri.make_model("sage_mean", (20, 16, 6), 175)
    from harness import Pair
    pair = Pair(n, n + 64, src, dst, feats, model, weights=w)
    stream = ri.UpdateStream(n, n + 64, src, dst, out_law, in_law, 12, MIXW, 176, weighted=True)
    try:
        for b, bs in enumerate([6, 80, 150]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()


def test_bf16_store_updates():
    print("case bf16 updates", flush=True)
    pair, graph = make_pair(n=600, e=4000, d0=16, kind="gcn_sum", widths=(16, 64, 24), store="bf16", seed=37)
    stream = make_stream(pair, graph, MIXV, 41)
    try:
        for b in range(4):
            ops, payload, _ = stream.next_batch(50)
            pair.step(ops, payload)
        pair.check_aggregates(tol=1e-3)
    finally:
        pair.close()


def test_device_resident_batch():
    torch = pytest.importorskip("torch")
    print("case device pointers", flush=True)
    pair, graph = make_pair(n=400, e=2500, d0=8, kind="sage_mean", widths=(8, 16, 6), seed=43)
    stream = make_stream(pair, graph, MIX3, 47)
    try:
        ops, payload, _ = stream.next_batch(64)
        rec = pair.ora.apply_batch(ops, payload)
        ops_t = torch.from_numpy(ops.astype(np.int64)).to(torch.int32).cuda().contiguous()
        pay_t = torch.from_numpy(payload).cuda().contiguous()
        torch.cuda.synchronize()
        res = rp.ripple_apply_updates(pair.ctx, ops_t.data_ptr(), pay_t.data_ptr(), n_ops=len(ops),
                                      n_feat_rows=len(payload))
        assert res.n_applied == int(rec.accepted.sum())
        pair.check_embeddings()
        out_t = torch.empty((pair.cap, pair.widths[-1]), dtype=torch.float32, device="cuda")
        rp.ripple_get_embeddings(pair.ctx, pair.L, pair.widths[-1], n_rows=pair.cap, out=out_t.data_ptr())
        assert np.array_equal(out_t.cpu().numpy(), pair.gpu_layer(pair.L))
    finally:
        pair.close()


def test_graph_beyond_the_single_workgroup_compaction_limit():
    """300,000 vertices need more than 8,192 bitmap words, so the frontier lists come from the
    two-pass (count, then scan and emit) compaction rather than the one-workgroup kernel."""
    print("case wide bitmap", flush=True)
    pair, graph = make_pair(n=300000, e=1200000, d0=8, kind="sage_mean", widths=(8, 16, 12), seed=91,
                            slack=1000, top_share=0.005)
    stream = make_stream(pair, graph, MIXV, 92)
    try:
        for b, bs in enumerate([1, 64, 2000, 500]):
            print(" batch", b, bs, flush=True)
            if b == 3:                                        # live-vertex list through the same two passes
                rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, 3)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload, check=(b >= 2))
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("kind,widths,store", [("sage_mean", (16, 40, 24, 10), "f32"), ("gcn_sum", (100, 256, 47), "f32"),
                                               ("gin_sum", (16, 32, 12, 6), "f32"), ("gcn_mean", (32, 64, 12), "bf16")])
def test_deterministic_mode_is_bit_reproducible(kind, widths, store):
    """With RIPPLE_OPT_DETERMINISTIC every aggregate row has one owner that adds its sources in a fixed
    order: two contexts fed the same operations must agree bit for bit after every batch (bootstrap
    included), and both must match the oracle like the default mode does. The graph has rows longer
    than a wavefront owns (1,024 entries), so the workgroup variant runs too."""
    print("case deterministic", kind, store, flush=True)
    kw = dict(n=20000, e=240000, d0=widths[0], kind=kind, widths=widths, seed=81, slack=256, store=store,
              top_share=0.04, deterministic=True)
    pair, graph = make_pair(**kw)
    twin, _ = make_pair(**kw)
    deg_in, _ = rp.ripple_get_degrees(pair.ctx, 1, pair.cap)
    assert deg_in.max() > 4096, "the workgroup variant would not be exercised"
    stream = make_stream(pair, graph, MIXV, 83)
    try:
        for l in range(pair.L + 1):
            assert np.array_equal(pair.gpu_layer(l).view(np.uint32), twin.gpu_layer(l).view(np.uint32)), "bootstrap differs"
        for b, bs in enumerate([3, 80, 400, 1500]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload, check=(b != 2))
            rp.ripple_apply_updates(twin.ctx, ops, payload)
            for l in range(pair.L + 1):
                assert np.array_equal(pair.gpu_layer(l).view(np.uint32), twin.gpu_layer(l).view(np.uint32)), \
                    f"layer {l} differs between two runs of batch {b}"
            for l in range(1, pair.L + 1):
                w = rp.ripple_get_layer_info(pair.ctx, l)[0]
                assert np.array_equal(rp.ripple_get_aggregates(pair.ctx, l, w, n_rows=pair.cap).view(np.uint32),
                                      rp.ripple_get_aggregates(twin.ctx, l, w, n_rows=twin.cap).view(np.uint32))
        pair.check_graph()
        pair.check_aggregates(tol=1e-3 if store == "bf16" else None)
    finally:
        pair.close()
        twin.close()


def _in_rows(ctx, cap, n_edges):
    """The in-rows in storage order: for every sink, its sources as the store holds them."""
    s, d, n = rp.ripple_export_edges(ctx, 1, n_edges + 16)
    assert n == n_edges
    return s[:n].astype(np.int64), d[:n].astype(np.int64)


def test_deterministic_mode_keeps_in_rows_in_a_reproducible_order():
    """The deterministic mode adds a row's sources in the order the in-row stores them, so that order has to
    be a function of the input and the batches: rows are built in the order the edges were given, and
    what a batch appends to a row ends up in ascending id order, whether it is a handful of entries (ranked by
    a wavefront), more than 64 (copied aside by a workgroup) or more than 4,096 (several LDS tiles). Deletions
    in the same rows and a second context fed the same batches are checked as well."""
    print("case deterministic row order", flush=True)
    kw = dict(n=9000, e=60000, d0=16, kind="sage_mean", widths=(16, 40, 10), seed=91, slack=64, deterministic=True)
    pair, graph = make_pair(**kw)
    twin, _ = make_pair(**kw)
    src, dst = graph[0].astype(np.int64), graph[1].astype(np.int64)
    try:
        order = np.argsort(dst, kind="stable")
        got_s, got_d = _in_rows(pair.ctx, pair.cap, len(src))
        assert np.array_equal(got_d, dst[order]) and np.array_equal(got_s, src[order]), "rows are not in input order"
        rng = np.random.default_rng(92)
        have = set(zip(src.tolist(), dst.tolist()))
        sinks = {5: 5000, 6: 300, 7: 40, 8: 2}               # sink -> edges it gains in one batch
        ops = []
        for v, k in sinks.items():
            cand = [u for u in rng.permutation(9000).tolist() if (u, v) not in have][:k]
            ops += [(ri.OP_EDGE_ADD, u, v, 0) for u in cand]
        for v in (5, 6, 7):                                   # and loses: holes are filled before the appends
            ins = src[dst == v]
            ops += [(ri.OP_EDGE_DEL, int(u), v, 0) for u in ins[: min(3, len(ins))]]
        ops = np.array(ops, dtype=np.uint32)
        ops = ops[rng.permutation(len(ops))]
        before_s, before_d = _in_rows(pair.ctx, pair.cap, len(src))
        none = np.zeros((0, 16), dtype=np.float32)
        res, rec, _ = pair.step(ops, none)
        assert res.n_rejected == 0
        rp.ripple_apply_updates(twin.ctx, ops, none)
        n_edges = pair.ora.n_edges()
        a_s, a_d = _in_rows(pair.ctx, pair.cap, n_edges)
        b_s, b_d = _in_rows(twin.ctx, twin.cap, n_edges)
        assert np.array_equal(a_s, b_s) and np.array_equal(a_d, b_d), "two runs store their in-rows differently"
        for v, k in sinks.items():
            row = a_s[a_d == v]
            tail = row[len(row) - k:]
            assert np.all(np.diff(tail) > 0), f"sink {v}: the {k} appended sources are not in ascending order"
            old = set(before_s[before_d == v].tolist())
            assert not (set(tail.tolist()) & old)
        for l in range(pair.L + 1):
            assert np.array_equal(pair.gpu_layer(l).view(np.uint32), twin.gpu_layer(l).view(np.uint32))
        stream = make_stream(pair, graph, MIXV, 93)           # the stream does not know the edges above: some ops are rejected
        ops2, payload2, _ = stream.next_batch(500)
        pair.step(ops2, payload2)
        rp.ripple_apply_updates(twin.ctx, ops2, payload2)
        for l in range(pair.L + 1):
            assert np.array_equal(pair.gpu_layer(l).view(np.uint32), twin.gpu_layer(l).view(np.uint32))
        pair.check_graph()
        pair.check_aggregates()
    finally:
        pair.close()
        twin.close()


@pytest.mark.parametrize("kind,widths,store", [("gcn_wsum", (100, 256, 47), "f32"), ("sage_wsum", (16, 40, 24, 10), "f32"),
                                               ("gcn_wsum", (32, 64, 12), "bf16")])
def test_weighted_sum_aggregation(kind, widths, store):
    """Table 1's weighted sum (m = alpha (h - h_old), Sec. 3.3.3): every edge has a weight fixed at its
    creation (initial edges: an array; later ones: in the EDGE_ADD operation). Vertex deletions remove
    weighted edges, rows are relocated and the pools rebuilt along the way; the cached aggregates must
    stay sum_u alpha_uv H[u] and the embeddings must match the oracle."""
    print("case weighted sum", kind, store, flush=True)
    pair, graph = make_pair(n=1500, e=14000, d0=widths[0], kind=kind, widths=widths, seed=131, slack=256, store=store,
                            weighted=True, top_share=0.05)
    stream = make_stream(pair, graph, MIXV, 133, weighted=True)
    tol = 1e-3 if store == "bf16" else None
    try:
        pair.check_aggregates(tol=tol)
        for b, bs in enumerate([2, 50, 300, 40, 600]):
            print(" batch", b, bs, flush=True)
            if b == 3:
                rp.ripple_compact(pair.ctx)                   # the weights move with the rebuilt in-rows
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates(tol=tol)
        pair.check_graph()
    finally:
        pair.close()


def test_weighted_layer_needs_a_weighted_graph():
    pair, _ = make_pair(n=50, e=200, d0=8, kind="gcn_sum", widths=(8, 6), seed=5)
    try:
        ctx = rp.ripple_init_graph(4, 8, np.array([0, 1], dtype=np.uint32), np.array([1, 2], dtype=np.uint32),
                                   np.zeros((4, 8), dtype=np.float32))
        with pytest.raises(rp.RippleError):
            rp.ripple_load_model(ctx, ri.make_model("gcn_wsum", (8, 6), 1))
        rp.ripple_destroy(ctx)
    finally:
        pair.close()


# ---- max / min aggregation (Sec. 3.4.2) ------------------------------------------------------------
@pytest.mark.parametrize("kind,widths,store", [("gcn_max", (100, 256, 47), "f32"), ("gcn_min", (16, 40, 24, 10), "f32"),
                                               ("sage_max", (16, 40, 24, 10), "f32"), ("sage_max", (32, 64, 12), "bf16"),
                                               ("gcn_max", (24, 300, 10), "f32"), ("gcn_max", (3, 4, 3, 2), "f32")])
def test_max_min_aggregation(kind, widths, store):
    """Monotonic aggregators: a vertex keeps its aggregate, raises it from the messages or recomputes
    it, and vertices whose aggregate does not change drop out of the propagation. The cached
    aggregates must be the exact extreme of the stored rows, the embeddings must match the oracle, the
    reported sets must lie between the rows that really changed and the topological sets."""
    print("case max/min", kind, widths, store, flush=True)
    pair, graph = make_pair(n=1500, e=14000, d0=widths[0], kind=kind, widths=widths, seed=141, slack=256, store=store,
                            top_share=0.05)
    stream = make_stream(pair, graph, MIXV, 143)
    seen = np.zeros(3, dtype=np.int64)
    pruned_any = False
    try:
        pair.check_aggregates()
        for b, bs in enumerate([2, 50, 300, 40, 600]):
            print(" batch", b, bs, flush=True)
            if b == 3:
                rp.ripple_compact(pair.ctx)
            ops, payload, _ = stream.next_batch(bs)
            res, rec, sets = pair.step(ops, payload)
            pair.check_aggregates()
            for l in range(1, pair.L + 1):
                seen += [res.mono_unchanged[l], res.mono_incremental[l], res.mono_recomputed[l]]
                pruned_any |= res.affected[l] < len(sets[l])
        pair.check_graph()
        print(" unchanged / incremental / recomputed:", seen, "pruned:", pruned_any, flush=True)
        assert seen.sum() > 0
        if widths[0] <= 4:       # wide rows nearly always lose some element's extreme; narrow ones show every case
            assert (seen > 0).all(), f"all three cases must occur: {seen}"
            assert pruned_any, "no propagation was ever pruned"
    finally:
        pair.close()


def test_max_layer_between_linear_layers():
    """sum -> max -> mean: what a hop hands on (differences for a linear consumer, the old rows for a
    max / min consumer) depends on the layer that receives it."""
    print("case mixed aggregators", flush=True)
    widths = (16, 40, 24, 10)
    src, dst, out_law, in_law = ri.chung_lu_graph(1200, 10000, 2.1, 0.04, 151)
    feats = ri.features(1200, widths[0], 152)
    model = ri.make_model("sage_mean", widths, 153)
    model[0]["agg"], model[1]["agg"], model[2]["agg"] = "sum", "max", "mean"
    from harness import Pair
    pair = Pair(1200, 1200 + 128, src, dst, feats, model)
    stream = ri.UpdateStream(1200, 1200 + 128, src, dst, out_law, in_law, widths[0], MIXV, 154)
    try:
        for b, bs in enumerate([5, 120, 500]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates()
    finally:
        pair.close()


def test_max_with_hub_rows_and_repeated_feature_updates():
    """In-rows of several thousand entries are recomputed when their extreme goes away; feature updates
    alone (no structural change) exercise the keep / raise / recompute split on unchanged in-rows."""
    print("case max hubs", flush=True)
    pair, graph = make_pair(n=20000, e=240000, d0=24, kind="gcn_max", widths=(24, 48, 12), seed=161, slack=64,
                            top_share=0.04)
    feat_only = {"edge_add": 0.0, "edge_del": 0.0, "feat": 1.0, "vadd": 0.0, "vdel": 0.0}
    stream = make_stream(pair, graph, feat_only, 163)
    mixed = make_stream(pair, graph, MIX3, 164)
    try:
        deg_in, _ = rp.ripple_get_degrees(pair.ctx, 1, pair.cap)
        assert deg_in.max() > 4096
        tot = np.zeros(3, dtype=np.int64)
        for b, bs in enumerate([200, 2000]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            res, _, _ = pair.step(ops, payload)
            for l in range(1, pair.L + 1):
                tot += [res.mono_unchanged[l], res.mono_incremental[l], res.mono_recomputed[l]]
        assert (tot > 0).all(), tot
        ops, payload, _ = mixed.next_batch(3000)
        pair.step(ops, payload)
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("kind,segments", [("gcn_max", None), ("sage_min", None), ("gcn_max", 0), ("sage_min", 3)])
def test_max_min_changed_edges_of_a_hub_are_messages(kind, segments):
    """A sink with thousands of in-neighbours is not re-read for an edge that comes or goes (Sec. 3.4.2): an
    added edge can only raise the extreme, a deleted one matters only if its source held it. Hand-made
    batches aimed at the vertex with the longest in-row: additions only, deletions of sources that hold no
    column's extreme, the deletion of one that does, then changed edges whose sources also change or vanish.
    When the hub is recomputed its row is read in segments by several workgroups: also run with that switched
    off and with room for three segments only (rows that find the queue full are read by one workgroup)."""
    print("case max/min hub sink", kind, segments, flush=True)
    pair, graph = make_pair(n=20000, e=240000, d0=24, kind=kind, widths=(24, 48, 12), seed=161, slack=64, top_share=0.04)
    if segments is not None:
        rp.ripple_set_option(pair.ctx, rp.OPT_ROW_SEGMENTS, segments)
    best = np.argmin if kind.endswith("min") else np.argmax
    rng = np.random.default_rng(167)
    try:
        deg_in, _ = rp.ripple_get_degrees(pair.ctx, 1, pair.cap)
        hub = int(np.argmax(deg_in))
        assert deg_in[hub] > 4096

        def edge_ops(code, sources):
            return np.array([(code, int(u), hub, 0) for u in sources], dtype=np.uint32)

        none = np.zeros((0, 24), dtype=np.float32)
        inn = np.array(sorted(pair.ora.in_neighbours(hub)), dtype=np.int64)
        outside = np.setdiff1d(np.flatnonzero(pair.ora.alive), np.append(inn, hub))
        print(" additions", flush=True)
        res, _, _ = pair.step(edge_ops(ri.OP_EDGE_ADD, rng.choice(outside, 5, replace=False)), none)
        assert res.mono_recomputed[1] == 0 and res.mono_unchanged[1] + res.mono_incremental[1] == 1

        inn = np.array(sorted(pair.ora.in_neighbours(hub)), dtype=np.int64)
        holders = np.unique(inn[best(pair.ora.h0[inn], axis=0)])
        others = np.setdiff1d(inn, holders)
        print(" deletions that keep every extreme", flush=True)
        res, _, _ = pair.step(edge_ops(ri.OP_EDGE_DEL, rng.choice(others, 4, replace=False)), none)
        assert res.mono_recomputed[1] == 0 and res.mono_unchanged[1] == 1 and res.affected[1] == 0
        print(" deletion of the source that holds a column", flush=True)
        res, _, _ = pair.step(edge_ops(ri.OP_EDGE_DEL, holders[:1]), none)
        assert res.mono_recomputed[1] == 1 and res.affected[1] == 1

        print(" changed edges with changed and removed sources", flush=True)
        inn = np.array(sorted(pair.ora.in_neighbours(hub)), dtype=np.int64)
        outside = np.setdiff1d(np.flatnonzero(pair.ora.alive), np.append(inn, hub))
        u_add, u_del, u_gone, u_far = int(outside[3]), int(inn[7]), int(inn[11]), int(inn[13])
        ops = np.array([(ri.OP_EDGE_ADD, u_add, hub, 0), (ri.OP_FEAT_UPDATE, u_add, 0, 0),
                        (ri.OP_EDGE_DEL, u_del, hub, 0), (ri.OP_FEAT_UPDATE, u_del, 0, 1)], dtype=np.uint32)
        pair.step(ops, rng.standard_normal((2, 24)).astype(np.float32))
        res, _, _ = pair.step(np.array([(ri.OP_VERTEX_DEL, u_gone, 0, 0)], dtype=np.uint32), none)
        assert res.mono_recomputed[1] >= 1                     # the removed source's row is gone: the hub is re-read
        # an added edge whose source jumps far beyond every other row: raised, not re-read
        big = (-50.0 if kind.endswith("min") else 50.0) * np.ones((1, 24), dtype=np.float32)
        ops = np.array([(ri.OP_EDGE_DEL, u_far, hub, 0), (ri.OP_FEAT_UPDATE, u_far, 0, 0)], dtype=np.uint32)
        pair.step(ops, big)
        pair.step(np.array([(ri.OP_EDGE_ADD, u_far, hub, 0)], dtype=np.uint32), none)
        pair.check_aggregates()
        pair.check_graph()
    finally:
        pair.close()


@pytest.mark.parametrize("segments", [None, 3])
def test_attention_changed_edges_of_a_hub_are_messages(segments):
    """Edges that come and go at a vertex with thousands of in-neighbours whose own score stays: numerator
    and denominator are patched with the edge's pre-batch weight and row (Sec. 3.4.1) instead of re-reading
    the row; sources that change, appear or vanish in the same batch included. Then the hub's own features
    change, which recomputes its row (split over several workgroups)."""
    print("case attention hub sink", segments, flush=True)
    pair, graph = make_pair(n=20000, e=240000, d0=24, kind="gat", widths=(24, 48, 12), seed=161, slack=64, top_share=0.04)
    if segments is not None:                                # room for three segments: most split rows fall back to one workgroup
        rp.ripple_set_option(pair.ctx, rp.OPT_ROW_SEGMENTS, segments)
    rng = np.random.default_rng(169)
    try:
        deg_in, _ = rp.ripple_get_degrees(pair.ctx, 1, pair.cap)
        hub = int(np.argmax(deg_in))
        assert deg_in[hub] > 4096
        none = np.zeros((0, 24), dtype=np.float32)
        for b in range(3):
            print(" batch", b, flush=True)
            inn = np.array(sorted(pair.ora.in_neighbours(hub)), dtype=np.int64)
            outside = np.setdiff1d(np.flatnonzero(pair.ora.alive), np.append(inn, hub))
            adds = rng.choice(outside, 4, replace=False)
            dels = rng.choice(inn, 4, replace=False)
            ops = [(ri.OP_EDGE_ADD, int(u), hub, 0) for u in adds] + [(ri.OP_EDGE_DEL, int(u), hub, 0) for u in dels]
            rows = none
            if b >= 1:                                          # an added and a deleted source change as well
                ops += [(ri.OP_FEAT_UPDATE, int(adds[0]), 0, 0), (ri.OP_FEAT_UPDATE, int(dels[0]), 0, 1)]
                rows = rng.standard_normal((2, 24)).astype(np.float32)
            if b == 2:                                          # and an in-neighbour is removed
                ops.append((ri.OP_VERTEX_DEL, int(np.setdiff1d(inn, dels)[5]), 0, 0))
            pair.step(np.array(ops, dtype=np.uint32), rows)
        print(" the hub itself changes", flush=True)
        pair.step(np.array([(ri.OP_FEAT_UPDATE, hub, 0, 0)], dtype=np.uint32), rng.standard_normal((1, 24)).astype(np.float32))
        pair.check_aggregates()
        pair.check_graph()
    finally:
        pair.close()


def test_max_layers_are_refused_in_deterministic_mode():
    ctx = rp.ripple_init_graph(4, 8, np.array([0, 1], dtype=np.uint32), np.array([1, 2], dtype=np.uint32),
                               np.zeros((4, 8), dtype=np.float32))
    rp.ripple_set_option(ctx, rp.OPT_DETERMINISTIC, 1)
    with pytest.raises(rp.RippleError):
        rp.ripple_load_model(ctx, ri.make_model("gcn_max", (8, 6), 1))
    rp.ripple_destroy(ctx)


# ---- graph attention (Sec. 3.4.1) -------------------------------------------------------------------
@pytest.mark.parametrize("widths,store", [((100, 256, 47), "f32"), ((16, 40, 24, 10), "f32"), ((32, 64, 12), "bf16"),
                                          ((24, 300, 10), "f32")])
def test_graph_attention_layers(widths, store):
    """Single-head attention layers, hybrid-incremental: vertices already in the previous hop's set or with
    a changed in-edge recompute numerator and denominator, the others receive differences. Sets are
    the topological ones (with A_{l-1} inside A_l), embeddings match the oracle after every batch."""
    print("case attention", widths, store, flush=True)
    pair, graph = make_pair(n=1500, e=14000, d0=widths[0], kind="gat", widths=widths, seed=171, slack=256, store=store,
                            top_share=0.05)
    stream = make_stream(pair, graph, MIXV, 173)
    tol = 2e-3 if store == "bf16" else None
    try:
        pair.check_embeddings()
        pair.check_aggregates(tol=tol)
        for b, bs in enumerate([2, 50, 300, 40, 600]):
            print(" batch", b, bs, flush=True)
            if b == 3:
                rp.ripple_compact(pair.ctx)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates(tol=tol)
        pair.check_graph()
    finally:
        pair.close()


def test_attention_between_other_layers_and_feature_only_batches():
    """mean -> attention -> max -> attention; then feature-only batches, where most receivers are not in
    the previous hop's set and take the incremental path."""
    print("case attention mixed", flush=True)
    widths = (16, 40, 24, 12, 10)
    src, dst, out_law, in_law = ri.chung_lu_graph(1200, 10000, 2.1, 0.04, 181)
    feats = ri.features(1200, widths[0], 182)
    model = ri.make_model("gat", widths, 183)
    sage = ri.make_model("sage_mean", widths, 184)
    gmax = ri.make_model("gcn_max", widths, 185)
    model[0], model[2] = sage[0], gmax[2]
    from harness import Pair
    pair = Pair(1200, 1200 + 128, src, dst, feats, model)
    stream = ri.UpdateStream(1200, 1200 + 128, src, dst, out_law, in_law, widths[0], MIXV, 186)
    feat_only = ri.UpdateStream(1200, 1200 + 128, src, dst, out_law, in_law, widths[0],
                                {"edge_add": 0.0, "edge_del": 0.0, "feat": 1.0, "vadd": 0.0, "vdel": 0.0}, 187)
    try:
        pair.check_embeddings()
        for b, bs in enumerate([5, 3]):
            print(" feature batch", b, bs, flush=True)
            ops, payload, _ = feat_only.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates()
    finally:
        pair.close()
    pair = Pair(1200, 1200 + 128, src, dst, feats, model)
    try:
        for b, bs in enumerate([5, 120, 500]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates()
    finally:
        pair.close()


def test_attention_with_hub_rows():
    print("case attention hubs", flush=True)
    pair, graph = make_pair(n=20000, e=240000, d0=24, kind="gat", widths=(24, 48, 12), seed=191, slack=64, top_share=0.04)
    stream = make_stream(pair, graph, MIX3, 193)
    try:
        deg_in, _ = rp.ripple_get_degrees(pair.ctx, 1, pair.cap)
        assert deg_in.max() > 4096
        pair.check_embeddings()
        for b, bs in enumerate([20, 2000]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("kind,widths", [("sage_mean", (100, 256, 256, 47)), ("gin_sum", (32, 64, 40, 10)), ("gat", (64, 128, 16)),
                                         ("gcn_sum", (128, 130, 70))])
def test_split_products_on_the_bf16_matrix_cores(kind, widths):
    """fp32 operands split exactly into three bf16 numbers, six partial products per product: the rows must
    match the oracle like the fp32 matrix path does, and the two paths must agree far below the tolerance."""
    print("case split products", kind, widths, flush=True)
    pair, graph = make_pair(n=3000, e=30000, d0=widths[0], kind=kind, widths=widths, seed=201, slack=128, split=True)
    twin, _ = make_pair(n=3000, e=30000, d0=widths[0], kind=kind, widths=widths, seed=201, slack=128, split=False)
    stream = make_stream(pair, graph, MIXV, 203)
    try:
        pair.check_embeddings()
        for b, bs in enumerate([4, 200, 900]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            rp.ripple_apply_updates(twin.ctx, ops, payload)
            for l in range(1, pair.L + 1):
                a, b2 = pair.gpu_layer(l).astype(np.float64), twin.gpu_layer(l).astype(np.float64)
                scale = np.abs(b2).max()
                assert np.abs(a - b2).max() <= 2e-6 * scale, (l, np.abs(a - b2).max() / scale)
                print("   layer", l, "split vs fp32 path: %.2e" % (np.abs(a - b2).max() / scale), flush=True)
        pair.check_aggregates()
    finally:
        pair.close()
        twin.close()


@pytest.mark.parametrize("kind,mode", [("gcn_sum", 1), ("gcn_sum", 2), ("sage_mean", 0), ("gin_sum", 0), ("gcn_max", 0),
                                       ("gat", 0), ("gcn_wsum", 0)])
def test_maximum_row_widths(kind, mode):
    """Rows of 1024 floats (the largest the library takes) and of 400: the 16- and 8-column-block
    instantiations of every scatter kernel, products with K up to 2048 and N above 256, hidden width 1024.
    A batch of about the size of the one before it takes the small-hop paths (lists built while marking, both
    aggregation roles of max / min and attention layers in one launch), a much larger one the general ones."""
    print("case maximum widths", kind, mode, flush=True)
    widths = (1024, 400, 1024)
    weighted = kind == "gcn_wsum"
    pair, graph = make_pair(n=700, e=6000, d0=widths[0], kind=kind, widths=widths, seed=221, slack=64, top_share=0.08,
                            weighted=weighted)
    if kind == "gin_sum":
        assert pair.model[0]["d_hidden"] == 256
    stream = make_stream(pair, graph, MIXV, 223, weighted=weighted)
    try:
        rp.ripple_set_option(pair.ctx, rp.OPT_SCATTER_MODE, mode)
        pair.check_embeddings()
        for b, bs in enumerate([3, 5, 120, 150, 400]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_aggregates()
        pair.check_graph()
    finally:
        pair.close()


def test_gin_with_the_widest_hidden_layer():
    print("case gin hidden 1024", flush=True)
    src, dst, out_law, in_law = ri.chung_lu_graph(600, 5000, 2.1, 0.05, 231)
    feats = ri.features(600, 48, 232)
    model = ri.make_model("gin_sum", (48, 64, 12), 233)
    rng = np.random.default_rng(234)
    for lay in model:                                  # widen the inner layer to the limit
        lay["d_hidden"] = 1024
        lay["W0"], lay["b0"] = ri.glorot(rng, lay["d_in"], 1024), rng.uniform(-0.1, 0.1, 1024).astype(np.float32)
        lay["W1"] = ri.glorot(rng, 1024, lay["d_out"])
    from harness import Pair
    pair = Pair(600, 664, src, dst, feats, model)
    stream = ri.UpdateStream(600, 664, src, dst, out_law, in_law, 48, MIXV, 235)
    try:
        pair.check_embeddings()
        for bs in (5, 200):
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
    finally:
        pair.close()


def test_maximum_row_widths_deterministic_mode():
    print("case maximum widths, deterministic", flush=True)
    widths = (1024, 400, 1024)
    pair, graph = make_pair(n=700, e=6000, d0=widths[0], kind="sage_mean", widths=widths, seed=241, slack=64, top_share=0.08,
                            deterministic=True)
    stream = make_stream(pair, graph, MIXV, 243)
    try:
        pair.check_embeddings()
        for bs in (3, 300):
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_aggregates()
    finally:
        pair.close()


@pytest.mark.parametrize("kind", ["gcn_max", "gcn_min", "gat", "gcn_wsum", "gcn_mean", "sage_max"])
def test_degenerate_neighbourhoods(kind):
    """A graph without any edge at the start, a vertex that gains its first and loses its last
    in-neighbour, self-loops, an identical feature rewrite, an empty batch, and a batch in which every
    operation is rejected: the cases where an aggregate is empty, a denominator is zero or nothing moves."""
    print("case degenerate", kind, flush=True)
    n, d0 = 40, 6
    weighted = kind == "gcn_wsum"
    feats = ri.features(n, d0, 251)
    model = ri.make_model(kind, (d0, 9, 5), 252)
    from harness import Pair
    none = np.zeros(0, dtype=np.uint32)
    pair = Pair(n, n + 8, none, none, feats, model, weights=np.zeros(0, dtype=np.float32) if weighted else None)

    def w(x):                                           # weight word of an EDGE_ADD on a weighted graph
        return int(np.array([x], dtype=np.float32).view(np.uint32)[0]) if weighted else 0
    try:
        pair.check_embeddings()                         # every aggregate is empty
        steps = [
            [(ri.OP_EDGE_ADD, 1, 0, w(0.5))],                                   # first in-neighbour of 0
            [(ri.OP_EDGE_ADD, 2, 0, w(1.5)), (ri.OP_EDGE_ADD, 0, 0, w(0.75)), (ri.OP_EDGE_ADD, 0, 3, w(1.0))],   # a self-loop
            [(ri.OP_FEAT_UPDATE, 1, 0, 0), (ri.OP_FEAT_UPDATE, 0, 0, 1)],
            [(ri.OP_EDGE_DEL, 1, 0, 0), (ri.OP_EDGE_DEL, 2, 0, 0)],             # only the self-loop feeds 0 now
            [(ri.OP_EDGE_DEL, 0, 0, 0)],                                        # 0 loses its last in-neighbour
            [(ri.OP_EDGE_DEL, 0, 0, 0), (ri.OP_EDGE_ADD, 0, 3, w(1.0)), (ri.OP_FEAT_UPDATE, n + 2, 0, 0),
             (ri.OP_VERTEX_DEL, n + 3, 0, 0)],                                  # all rejected
            [(ri.OP_VERTEX_ADD, n, 0, 0), (ri.OP_EDGE_ADD, n, 3, w(0.25)), (ri.OP_EDGE_ADD, 3, n, w(1.25))],
            [(ri.OP_VERTEX_DEL, 3, 0, 0)],                                      # n and 0 lose their neighbour again
        ]
        rng = np.random.default_rng(253)
        for i, ops in enumerate(steps):
            print(" step", i, flush=True)
            payload = rng.standard_normal((2, d0)).astype(np.float32)
            res, rec, _ = pair.step(np.array(ops, dtype=np.uint32), payload)
            if i == 5:
                assert res.n_applied == 0 and res.n_rejected == 4
            pair.check_aggregates()
        same = pair.gpu_layer(0)[[0]].copy()            # a feature rewrite with the identical row
        before = [pair.gpu_layer(l) for l in range(pair.L + 1)]
        pair.step(np.array([(ri.OP_FEAT_UPDATE, 0, 0, 0)], dtype=np.uint32), same)
        for l in range(pair.L + 1):
            assert np.array_equal(before[l], pair.gpu_layer(l))
        res = rp.ripple_apply_updates(pair.ctx, np.zeros((0, 4), np.uint32), None)
        assert list(res.affected[: pair.L + 1]) == [0] * (pair.L + 1)
        pair.check_graph()
    finally:
        pair.close()


@pytest.mark.parametrize("kinds,widths", [(("sage_mean", "gcn_max", "gcn_mean"), (64, 16, 12, 6)),      # project-first, then max
                                          (("gcn_sum", "gcn_min", "gat"), (10, 7, 5, 3)),             # odd widths: generic products
                                          (("gat", "gcn_sum", "gcn_max"), (9, 6, 7, 5)),
                                          (("gin_sum", "gcn_max", "sage_mean"), (12, 20, 8, 6))])
def test_mixed_layer_kinds_hand_over_the_right_rows(kinds, widths):
    """What layer l writes for the next hop (differences, or the old rows when the next layer takes max / min)
    comes from whichever kernel finishes layer l: the tiled product, the generic product for odd widths,
    the element-wise update of project-first and attention layers, or the second stage of a two-stage
    update."""
    print("case mixed kinds", kinds, widths, flush=True)
    src, dst, out_law, in_law = ri.chung_lu_graph(900, 8000, 2.1, 0.04, 261)
    feats = ri.features(900, widths[0], 262)
    model = [ri.make_model(k, widths, 263 + i)[i] for i, k in enumerate(kinds)]
    from harness import Pair
    pair = Pair(900, 900 + 64, src, dst, feats, model)
    stream = ri.UpdateStream(900, 900 + 64, src, dst, out_law, in_law, widths[0], MIXV, 266)
    try:
        if kinds[0] == "sage_mean":
            assert rp.ripple_get_layer_info(pair.ctx, 1)[1], "the first layer was meant to be handled project-first"
        pair.check_embeddings()
        for b, bs in enumerate([4, 90, 350]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
            pair.check_aggregates()
    finally:
        pair.close()


def test_weighted_graph_with_max_and_attention_layers_and_hub_rows():
    """On a weighted graph the list of changed edges carries the weight in its sign field, so max / min and
    attention layers (which ignore the weights) cannot read "added or deleted" from it: sinks with long
    in-rows recompute there. Weighted sum first, then max, then attention, hub rows of several thousand
    entries, small batches (list-while-marking hops) and a large one."""
    print("case weighted graph, max and attention layers", flush=True)
    n = 12000
    src, dst, out_law, in_law = ri.chung_lu_graph(n, 150000, 2.1, 0.05, 301)
    widths = (16, 24, 12, 6)
    feats = ri.features(n, widths[0], 302)
    model = [ri.make_model(k, widths, 303 + i)[i] for i, k in enumerate(("gcn_wsum", "gcn_max", "gat"))]
    from harness import Pair
    pair = Pair(n, n + 256, src, dst, feats, model, weights=ri.edge_weights(len(src), 306))
    stream = ri.UpdateStream(n, n + 256, src, dst, out_law, in_law, widths[0], MIXV, 307, weighted=True)
    try:
        deg_in, _ = rp.ripple_get_degrees(pair.ctx, 1, pair.cap)
        assert deg_in.max() > 2048
        for b, bs in enumerate([5, 6, 5, 1500, 8]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            pair.step(ops, payload)
        pair.check_aggregates()
        pair.check_graph()
    finally:
        pair.close()


def test_attention_scores_that_drop_by_many_orders_of_magnitude():
    """Raw exponentials (the paper's numerator / denominator messages) cancel catastrophically when a dominant
    weight collapses: e^36 taken out of a denominator leaves only rounding residue. Rows whose patched
    denominator is tiny against what was added and removed are recomputed instead; the result must still
    match the oracle."""
    print("case attention cancellation", flush=True)
    n, d = 400, 4
    src, dst, out_law, in_law = ri.chung_lu_graph(n, 4000, 2.1, 0.05, 271)
    feats = ri.features(n, d, 272)
    model = ri.make_model("gat", (d, d, 3), 273)
    model[0]["W0"] = np.eye(d, dtype=np.float32)
    model[0]["att"] = np.array([12.0, 0, 0, 0, 0, 0, 0, 0], dtype=np.float32)      # score = 12 * first feature of the source
    from harness import Pair
    pair = Pair(n, n + 16, src, dst, feats, model)
    feat_only = {"edge_add": 0.0, "edge_del": 0.0, "feat": 1.0, "vadd": 0.0, "vdel": 0.0}
    stream = ri.UpdateStream(n, n + 16, src, dst, out_law, in_law, d, feat_only, 274)
    try:
        pair.check_embeddings()
        rng = np.random.default_rng(275)
        for b in range(6):
            ops, payload, _ = stream.next_batch(30)
            # push the updated vertices' first feature to the extremes: weights between e^-7 and e^36
            payload[:, 0] = rng.choice([-3.0, 3.0], size=len(payload))
            pair.step(ops, payload)
    finally:
        pair.close()


@pytest.mark.parametrize("kind,widths,weighted", [("sage_mean", (16, 40, 24, 10), False), ("gcn_sum", (100, 256, 47), False),
                                                  ("gin_sum", (12, 20, 8), False), ("gcn_wsum", (12, 20, 8), True),
                                                  ("gat", (12, 20, 8), False), ("gcn_max", (12, 20, 8), False),
                                                  ("sage_min", (12, 20, 8, 6), False)])
def test_small_frontiers_listed_while_marking(kind, widths, weighted):
    """Hops whose sets were small in the previous batch build their list while marking (unordered, no bitmap
    scan). Small batches of steady size take that path from the second batch on; a much larger batch in
    between and the batches after it fall back and return to it. Checked like every other batch; the same
    stream with the option off must report identical sets."""
    print("case sparse frontier", kind, flush=True)
    pair, graph = make_pair(n=6000, e=50000, d0=widths[0], kind=kind, widths=widths, seed=281, slack=128, weighted=weighted)
    twin, _ = make_pair(n=6000, e=50000, d0=widths[0], kind=kind, widths=widths, seed=281, slack=128, weighted=weighted)
    rp.ripple_set_option(twin.ctx, rp.OPT_SPARSE_FRONTIER, 0)
    stream = make_stream(pair, graph, MIXV, 283, weighted=weighted)
    try:
        for b, bs in enumerate([6, 6, 8, 7, 900, 10, 12, 9, 1, 1, 2]):
            print(" batch", b, bs, flush=True)
            ops, payload, _ = stream.next_batch(bs)
            res, _, sets = pair.step(ops, payload)
            rp.ripple_apply_updates(twin.ctx, ops, payload)
            for l in range(pair.L + 1):
                assert np.array_equal(rp.ripple_get_affected(twin.ctx, l, twin.cap)[0],
                                      rp.ripple_get_affected(pair.ctx, l, pair.cap)[0])
        pair.check_aggregates()
        pair.check_graph()
    finally:
        pair.close()
        twin.close()


def test_small_frontier_hint_that_turns_out_wrong():
    """Single-update batches: after two that touch a leaf, one rewrites the features of the vertex with the
    most out-neighbours (thousands), so the list-while-marking path, chosen on the previous batch's sizes,
    has to carry a set far beyond what it was meant for; then back to a leaf."""
    print("case sparse frontier, wrong hint", flush=True)
    pair, graph = make_pair(n=20000, e=240000, d0=16, kind="sage_mean", widths=(16, 24, 8), seed=291, slack=64, top_share=0.04)
    try:
        deg_out, _ = rp.ripple_get_degrees(pair.ctx, 0, pair.cap)
        hub = int(np.argmax(deg_out))
        leaves = [int(v) for v in np.flatnonzero((deg_out > 0) & (deg_out <= 3))[:6]]
        assert deg_out[hub] > 4096
        rng = np.random.default_rng(293)
        for b, v in enumerate([leaves[0], leaves[1], hub, leaves[2], hub, hub, leaves[3]]):
            print(" batch", b, "vertex", v, "out-degree", int(deg_out[v]), flush=True)
            ops = np.array([(ri.OP_FEAT_UPDATE, v, 0, 0)], dtype=np.uint32)
            res, _, sets = pair.step(ops, rng.standard_normal((1, 16)).astype(np.float32))
            if v == hub:
                assert res.affected[1] > 4096
        pair.check_aggregates()
    finally:
        pair.close()
