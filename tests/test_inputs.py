"""The input generators: exact sizes, validity of every emitted operation (as
judged by the oracle's own, separately written graph store) and agreement of
the two edge records after many batches."""
import numpy as np

import oracle
import ripple_inputs as ri


def test_chung_lu_exact_and_skewed():
    cfg = ri.get_config("tiny_gcn_sum")
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    assert src.size == cfg.e and np.all(src != dst)
    keys = src.astype(np.int64) * cfg.n + dst
    assert np.unique(keys).size == cfg.e
    outdeg = np.bincount(src, minlength=cfg.n)
    assert outdeg.max() > 20 * outdeg.mean()             # hubs exist
    assert outdeg.max() < 0.05 * cfg.e                   # ... but do not saturate
    s2, d2, _, _ = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    assert np.array_equal(src, s2) and np.array_equal(dst, d2)   # seeded


def test_stream_is_valid_and_nonconflicting():
    cfg = ri.get_config("tiny_gcn_sum")
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, 5)
    feats = ri.features(cfg.n, 8, 6)
    mix = {"edge_add": 0.4, "edge_del": 0.3, "feat": 0.2, "vadd": 0.05, "vdel": 0.05}
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, 8, mix, 7)
    st = oracle.GraphState(cfg.n, cfg.vertex_capacity, src, dst, feats)
    for b in range(12):
        ops, payload, n_upd = stream.next_batch(100)
        assert n_upd == 100 and ops.shape[0] == 100 + 5 * 8
        edge_keys = [(int(u), int(v)) for k, u, v, _ in ops if k in (ri.OP_EDGE_ADD, ri.OP_EDGE_DEL)]
        assert len(set(edge_keys)) == len(edge_keys)
        rec = st.apply_batch(ops, payload)
        assert rec.accepted.all(), b
        assert st.n_edges() == stream.n_edges()
    a = np.sort(np.asarray(st.edges()[0]) * st.cap + np.asarray(st.edges()[1]))
    es, ed = stream.edge_arrays()
    b_ = np.sort(es.astype(np.int64) * st.cap + ed)
    assert np.array_equal(a, b_)
    assert np.array_equal(st.alive, stream.alive)


def test_weighted_stream_with_weight_replacements():
    cfg = ri.get_config("tiny_gcn_sum")
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, 5)
    feats = ri.features(cfg.n, 8, 6)
    w = ri.edge_weights(len(src), 8)
    mix = {"edge_add": 0.3, "edge_del": 0.2, "feat": 0.2, "vadd": 0.0, "vdel": 0.0, "reweight": 0.3}
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, 8, mix, 7, weighted=True)
    st = oracle.GraphState(cfg.n, cfg.vertex_capacity, src, dst, feats, weights=w)
    seen = 0
    for b in range(6):
        ops, payload, n_upd = stream.next_batch(50)
        assert n_upd == 50
        seen += int((ops[:, 0] == ri.OP_EDGE_REWEIGHT).sum())
        rec = st.apply_batch(ops, payload)
        assert rec.accepted.all(), b
    assert seen == 6 * 15
    ew = st.edge_weights()
    assert ew.min() >= 0.25 and ew.max() < 1.75 and len(ew) == st.n_edges()


def test_batch_size_one_draws_every_kind():
    cfg = ri.get_config("tiny_gcn_sum")
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, 5)
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, 4, cfg.mix, 9)
    kinds = set()
    for _ in range(60):
        ops, payload, n = stream.next_batch(1)
        assert n == 1 and len(ops) == 1
        kinds.add(int(ops[0, 0]))
    assert kinds == {ri.OP_EDGE_ADD, ri.OP_EDGE_DEL, ri.OP_FEAT_UPDATE}


def test_draw_pair_equals_two_draws():
    a = ri.PowerLaw(5000, 2.2, 0.01, 3)
    b = ri.PowerLaw(5000, 2.2, 0.01, 4)
    from ripple_inputs.graphs import draw_pair
    r1, r2 = np.random.default_rng(11), np.random.default_rng(11)
    for size in (1, 16, 33):
        for _ in range(50):
            x, y = draw_pair(r1, a, b, size)
            assert np.array_equal(x, a.draw(r2, size)) and np.array_equal(y, b.draw(r2, size))
    c = ri.PowerLaw(5000, 2.5, 0.01, 4)                        # another shape: falls back to two draws
    x, y = draw_pair(r1, a, c, 16)
    assert np.array_equal(x, a.draw(r2, 16)) and np.array_equal(y, c.draw(r2, 16))


def test_producer_process_hands_over_the_same_batches(tmp_path):
    cfg = ri.get_config("tiny_gcn_sum")
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, cfg.mix, cfg.stream_seed)
    ri.BatchProducer.save_graph(str(tmp_path), src, dst)
    with ri.BatchProducer(cfg.name, str(tmp_path), 100, 5) as prod:
        for _ in range(5):
            ops, payload, n = stream.next_batch(100)
            ops2, payload2, n2 = prod.next_batch()
            assert n == n2 and np.array_equal(ops, ops2) and np.array_equal(payload, payload2)
            assert ops2.dtype == np.uint32 and payload2.dtype == np.float32
