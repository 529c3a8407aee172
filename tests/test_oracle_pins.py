"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself (brute force, closed forms, the paper's worked example)."""
import os

import numpy as np
import pytest

import oracle
import ripple_inputs as ri
from bruteforce import embed, in_lists, in_weights

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_case(seed, n=40, e=160, d0=5, kind="gcn_sum", widths=(5, 7, 6, 4), dead=()):
    rng = np.random.default_rng(seed)
    keys = rng.choice(n * n, size=e, replace=False)
    src, dst = keys // n, keys % n
    keep = src != dst
    src, dst = src[keep], dst[keep]
    feats = rng.standard_normal((n, d0))
    model = ri.make_model(kind, widths, seed + 1)
    st = oracle.GraphState(n, n + 4, src, dst, feats)
    return st, model, src, dst, feats


@pytest.mark.parametrize("kind", ["gcn_sum", "gcn_mean", "sage_mean", "sage_sum", "gin_sum"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_layerwise_equals_vertexwise_bruteforce(kind, seed):
    st, model, src, dst, feats = small_case(seed, kind=kind)
    hs = oracle.full_recompute(st, model)
    nbrs = in_lists(st.cap, src, dst)
    f = np.zeros((st.cap, feats.shape[1]))
    f[: len(feats)] = feats
    memo = {}
    for l in range(len(model) + 1):
        for v in range(st.cap):
            want = embed(v, l, model, f, nbrs, st.alive, memo)
            np.testing.assert_allclose(hs[l][v], want, rtol=1e-12, atol=1e-12)


def test_bruteforce_after_batch_with_all_update_kinds():
    st, model, src, dst, feats = small_case(7, kind="sage_mean")
    n = len(feats)
    rng = np.random.default_rng(3)
    payload = rng.standard_normal((3, feats.shape[1]))
    s0, d0_ = int(src[0]), int(dst[0])
    ops = [(ri.OP_EDGE_DEL, s0, d0_, 0), (ri.OP_EDGE_ADD, 1, 2, 0) if not st.has_edge(1, 2)
           else (ri.OP_EDGE_ADD, 1, 3, 0),
           (ri.OP_FEAT_UPDATE, 5, 0, 0), (ri.OP_VERTEX_ADD, n, 0, 1), (ri.OP_EDGE_ADD, n, 4, 0),
           (ri.OP_EDGE_ADD, 6, n, 0), (ri.OP_VERTEX_DEL, 9, 0, 0), (ri.OP_FEAT_UPDATE, 9, 0, 2)]
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), payload)
    assert rec.accepted.tolist() == [True] * 7 + [False]      # update of a deleted vertex
    hs = oracle.full_recompute(st, model)
    es, ed = st.edges()
    nbrs = in_lists(st.cap, es, ed)
    memo = {}
    for v in range(st.cap):
        want = embed(v, len(model), model, st.h0, nbrs, st.alive, memo)
        np.testing.assert_allclose(hs[-1][v], want, rtol=1e-12, atol=1e-12)
    assert not st.alive[9] and np.all(hs[-1][9] == 0)
    assert 9 not in es and 9 not in ed


def test_linear_sum_closed_form():
    """No activation, no bias, sum: H^L = (A^T)^L H^0 W^1 ... W^L."""
    st, model, src, dst, feats = small_case(11, kind="gcn_sum")
    for lay in model:
        lay["act_out"] = "none"
        lay["b0"] = np.zeros_like(lay["b0"])
    hs = oracle.full_recompute(st, model)
    a = np.zeros((st.cap, st.cap))
    for s, d in zip(src, dst):
        a[s, d] += 1.0                                   # a[u, v] = 1 for edge u -> v
    want = st.h0.copy()
    for lay in model:
        want = a.T @ want
    for lay in model:
        want = want @ np.asarray(lay["W0"], dtype=np.float64)
    np.testing.assert_allclose(hs[-1], want, rtol=1e-11, atol=1e-11)


def test_mean_of_ones_is_ones():
    n, d = 30, 4
    rng = np.random.default_rng(5)
    ring_s = np.arange(n)
    ring_d = (np.arange(n) + 1) % n                      # every vertex has an in-edge
    extra = rng.choice(n * n, size=60, replace=False)
    es, ed = extra // n, extra % n
    keep = (es != ed) & (ed != (es + 1) % n)
    src = np.concatenate([ring_s, es[keep]])
    dst = np.concatenate([ring_d, ed[keep]])
    st = oracle.GraphState(n, n, src, dst, np.ones((n, d)))
    lay = dict(d_in=d, d_hidden=0, d_out=d, agg="mean", self="none", eps=0.0, act_inner="none",
               act_out="relu", W0=np.eye(d, dtype=np.float32), b0=np.zeros(d, np.float32),
               W1=None, b1=None)
    hs = oracle.full_recompute(st, [lay, lay, lay])
    np.testing.assert_allclose(hs[-1], np.ones((n, d)), rtol=0, atol=1e-15)


@pytest.mark.parametrize("kind", ["gcn_sum", "sage_mean", "gin_sum"])
def test_isolated_vertex(kind):
    st, model, src, dst, feats = small_case(21, kind=kind, widths=(5, 6))
    iso = st.cap - 1                                   # make one spare id live and isolated
    f = np.random.default_rng(2).standard_normal((1, 5))
    st.apply_batch(np.array([(ri.OP_VERTEX_ADD, iso, 0, 0)], dtype=np.uint32), f)
    h1 = oracle.full_recompute(st, model)[1][iso]
    lay = model[0]
    W0, b0 = lay["W0"].astype(np.float64), lay["b0"].astype(np.float64)
    if kind == "gcn_sum":
        want = b0                                        # nothing aggregated: act(b), last layer no act
    elif kind == "sage_mean":
        want = f[0] @ W0[:5] + b0
    else:
        want = np.maximum(f[0] @ W0 + b0, 0) @ lay["W1"].astype(np.float64) + lay["b1"]
    np.testing.assert_allclose(h1, want, rtol=1e-13, atol=1e-13)


# ---- planted mistakes: each plausible slip must trip the brute-force pin ----
def _bf_all(model, st, src, dst):
    nbrs = in_lists(st.cap, src, dst)
    memo = {}
    L = len(model)
    return np.stack([embed(v, L, model, st.h0, nbrs, st.alive, memo) for v in range(st.cap)])


def test_planted_mistakes_are_caught():
    st, model, src, dst, feats = small_case(31, kind="sage_mean")
    good = oracle.full_recompute(st, model)[-1]
    np.testing.assert_allclose(good, _bf_all(model, st, src, dst), rtol=1e-12, atol=1e-12)
    # (a) edge direction swapped
    st_rev = oracle.GraphState(len(feats), st.cap, dst, src, feats)
    assert np.abs(oracle.full_recompute(st_rev, model)[-1] - good).max() > 1e-3
    # (b) self and neighbour halves of the SAGE weight swapped
    sw = [dict(l, W0=np.vstack([l["W0"][l["d_in"]:], l["W0"][:l["d_in"]]])) for l in model]
    assert np.abs(oracle.full_recompute(st, sw)[-1] - good).max() > 1e-3
    # (c) mean replaced by sum
    sm = [dict(l, agg="sum") for l in model]
    assert np.abs(oracle.full_recompute(st, sm)[-1] - good).max() > 1e-3
    # (d) bias dropped
    nb = [dict(l, b0=np.zeros_like(l["b0"])) for l in model]
    assert np.abs(oracle.full_recompute(st, nb)[-1] - good).max() > 1e-3
    # (e) GIN: eps sign / self term dropped
    st2, gin, s2, d2, f2 = small_case(32, kind="gin_sum")
    for l in gin:
        l["eps"] = 0.25
    g = oracle.full_recompute(st2, gin)[-1]
    np.testing.assert_allclose(g, _bf_all(gin, st2, s2, d2), rtol=1e-12, atol=1e-12)
    assert np.abs(oracle.full_recompute(st2, [dict(l, eps=-0.25) for l in gin])[-1] - g).max() > 1e-4


# ---- affected sets -------------------------------------------------------------
def _read_golden():
    sec, cur = {}, None
    with open(os.path.join(GOLDEN, "worked_example.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("["):
                cur = line.strip("[]")
                sec[cur] = []
            else:
                sec[cur].append(line.split())
    return sec


def _example_state():
    g = _read_golden()
    names = "ABCDE"
    idx = {c: i for i, c in enumerate(names)}
    src = [idx[a] for a, b in g["edges"]]
    dst = [idx[b] for a, b in g["edges"]]
    st = oracle.GraphState(5, 5, src, dst, np.random.default_rng(0).standard_normal((5, 3)))
    return g, idx, st


def _ids(idx, toks):
    return sorted(idx[t] for t in toks)


def test_paper_worked_example_edge_addition():
    g, idx, st = _example_state()
    model3 = ri.make_model("gcn_sum", (3, 3, 3, 3), 1)
    (a, b), = g["add_edge"]
    rec = st.apply_batch(np.array([(ri.OP_EDGE_ADD, idx[a], idx[b], 0)], dtype=np.uint32),
                         np.zeros((0, 3)))
    assert rec.accepted.all()
    sets = oracle.affected_sets(st, rec, model3)
    assert sets[0].tolist() == []
    assert sets[1].tolist() == _ids(idx, g["expect_hop1"][0])
    assert sets[2].tolist() == _ids(idx, g["expect_hop2"][0])
    assert set(_ids(idx, g["expect_hop3_superset"][0])) <= set(sets[3].tolist())
    sink = idx[g["sink_every_hop"][0][0]]
    assert all(sink in s for s in sets[1:])


def test_paper_worked_example_vertex_delete_and_feature_update():
    g, idx, st = _example_state()
    model = ri.make_model("gcn_sum", (3, 3, 3), 1)
    (a, b), = g["add_edge"]
    st.apply_batch(np.array([(ri.OP_EDGE_ADD, idx[a], idx[b], 0)], dtype=np.uint32), np.zeros((0, 3)))
    c = idx[g["feature_update"][0][0]]
    rec = st.apply_batch(np.array([(ri.OP_FEAT_UPDATE, c, 0, 0)], dtype=np.uint32), np.ones((1, 3)))
    sets = oracle.affected_sets(st, rec, model)
    assert sets[0].tolist() == [c]
    assert sets[1].tolist() == _ids(idx, g["expect_feature_hop1"][0])
    c = idx[g["delete_vertex"][0][0]]
    rec = st.apply_batch(np.array([(ri.OP_VERTEX_DEL, c, 0, 0)], dtype=np.uint32), np.zeros((0, 3)))
    sets = oracle.affected_sets(st, rec, model)
    assert sets[1].tolist() == _ids(idx, g["expect_delete_hop1"][0])
    es, ed = st.edges()
    assert c not in es and c not in ed and st.n_edges() == 5


@pytest.mark.parametrize("kind", ["gcn_sum", "sage_mean", "gin_sum", "gat"])
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_affected_set_equals_rows_that_change(kind, seed):
    """With linear activations and generic real inputs, the rows of H^l that a
    batch really changes are exactly the topological affected set; with ReLU
    they are a subset of it. (Attention: a vertex of the previous hop's set stays in the
    set because its own score enters all its coefficients; whether that moves the row depends on the values.)"""
    for linear in (True, False):
        st, model, src, dst, feats = small_case(100 + seed, n=60, e=150, kind=kind)
        if linear:
            for lay in model:
                lay["act_out"] = "none"
                lay["act_inner"] = "none"
        before = oracle.full_recompute(st, model)
        cfg_rng = np.random.default_rng(seed)
        n = len(feats)
        ops, rows = [], []
        es, ed = st.edges()
        pick = cfg_rng.choice(len(es), size=3, replace=False)
        for i in pick:
            ops.append((ri.OP_EDGE_DEL, int(es[i]), int(ed[i]), 0))
        while len(ops) < 6:
            u, v = cfg_rng.integers(n, size=2)
            if u != v and not st.has_edge(int(u), int(v)):
                ops.append((ri.OP_EDGE_ADD, int(u), int(v), 0))
        for w in cfg_rng.choice(n, size=2, replace=False):
            rows.append(cfg_rng.standard_normal(feats.shape[1]))
            ops.append((ri.OP_FEAT_UPDATE, int(w), 0, len(rows) - 1))
        rec = st.apply_batch(np.array(ops, dtype=np.uint32), np.array(rows))
        after = oracle.full_recompute(st, model)
        sets = oracle.affected_sets(st, rec, model)
        for l in range(len(model) + 1):
            changed = set(np.nonzero(np.abs(after[l] - before[l]).max(axis=1) > 0)[0].tolist())
            want = set(sets[l].tolist())
            if linear and kind == "gat" and l >= 1:
                # a vertex's own score moves its coefficients only if its in-neighbours' scores do not all
                # stay on one side of the LeakyReLU (a common shift cancels in the softmax), so rows of the
                # set may stay as they are; what changes by more than rounding must be in the set, and the
                # sinks of changed edges and receivers of changed rows do change
                moved = set(np.nonzero(np.abs(after[l] - before[l]).max(axis=1) > 1e-9)[0].tolist())
                assert changed <= want and len(moved) >= len(want) // 2, (l, sorted(changed ^ want))
            elif linear:
                assert changed == want, (l, kind)
            else:
                assert changed <= set(sets[l].tolist()), (l, kind)


def _changed_rows(before, after, alive):
    """Live rows of a layer that differ at all between two full recomputations."""
    diff = np.abs(after - before).max(axis=1) > 0
    return set(np.nonzero(diff & alive)[0].tolist())


@pytest.mark.parametrize("kind", ["gcn_sum", "sage_mean", "gin_sum"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_affected_set_equals_rows_that_change_with_vertex_operations(kind, seed):
    """The same pin with created and deleted vertices in the batch (Sec. 3.2, paragraphs on vertex
    addition and vertex deletion). Linear activations, non-zero biases and generic inputs: a live row
    changes exactly when the vertex is in the set. A created vertex's rows go from zero to act(b + ...),
    so it must sit in every set, with or without edges and on layers without a self term; the
    out-neighbours of a deleted vertex lose a term at every hop; the deleted vertex itself (whose rows
    become zero) is reported in no set."""
    st, model, src, dst, feats = small_case(300 + seed, n=60, e=150, kind=kind)
    for lay in model:
        lay["act_out"] = "none"
        lay["act_inner"] = "none"
    before = oracle.full_recompute(st, model)
    rng = np.random.default_rng(seed)
    n, d0 = len(feats), feats.shape[1]
    iso, src_only, sink_only, both = n, n + 1, n + 2, n + 3          # the four spare ids
    gone = [int(w) for w in rng.choice(n, size=2, replace=False)]
    others = [w for w in range(n) if w not in gone]
    a, b, c, d = (int(w) for w in rng.choice(others, size=4, replace=False))
    payload = rng.standard_normal((4, d0))
    ops = [(ri.OP_VERTEX_ADD, iso, 0, 0),                            # isolated
           (ri.OP_VERTEX_ADD, src_only, 0, 1), (ri.OP_EDGE_ADD, src_only, a, 0),   # only an out-edge
           (ri.OP_VERTEX_ADD, sink_only, 0, 2), (ri.OP_EDGE_ADD, b, sink_only, 0),  # only an in-edge
           (ri.OP_VERTEX_ADD, both, 0, 3), (ri.OP_EDGE_ADD, both, c, 0), (ri.OP_EDGE_ADD, d, both, 0),
           (ri.OP_VERTEX_DEL, gone[0], 0, 0), (ri.OP_VERTEX_DEL, gone[1], 0, 0)]
    out_of_gone = {w for g in gone for w in st.out_neighbours(g)} - set(gone)
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), payload)
    assert rec.accepted.all()
    after = oracle.full_recompute(st, model)
    sets = oracle.affected_sets(st, rec, model)
    for l in range(len(model) + 1):
        want = set(sets[l].tolist())
        assert _changed_rows(before[l], after[l], st.alive) == want, (l, kind)
        assert {iso, src_only, sink_only, both} <= want                # created vertices: every hop
        assert not (set(gone) & want)                                  # deleted vertices: no hop
        assert np.all(after[l][gone] == 0)
        if l >= 1:
            assert out_of_gone <= want                                 # they lost an in-neighbour


def test_isolated_created_vertex_is_alone_in_every_set():
    """Sec. 3.2, vertex addition: creating a vertex triggers nothing but the update of its own
    embeddings. With no edges it is the only member of the set at every hop, also on layers
    without a self term; with only an in-edge it is likewise the only member (it is the sink of the
    added edge and has nowhere to propagate to); with an out-edge its sink joins from hop 1 on."""
    for kind in ("gcn_sum", "sage_mean"):
        st, model, src, dst, feats = small_case(77, kind=kind)
        n = len(feats)
        row = np.ones((1, feats.shape[1]))
        rec = st.apply_batch(np.array([(ri.OP_VERTEX_ADD, n, 0, 0)], dtype=np.uint32), row)
        assert [s.tolist() for s in oracle.affected_sets(st, rec, model)] == [[n]] * (len(model) + 1)
        rec = st.apply_batch(np.array([(ri.OP_VERTEX_ADD, n + 1, 0, 0), (ri.OP_EDGE_ADD, 3, n + 1, 0)],
                                      dtype=np.uint32), row)
        assert [s.tolist() for s in oracle.affected_sets(st, rec, model)] == [[n + 1]] * (len(model) + 1)
        rec = st.apply_batch(np.array([(ri.OP_VERTEX_ADD, n + 2, 0, 0), (ri.OP_EDGE_ADD, n + 2, 3, 0)],
                                      dtype=np.uint32), row)
        sets = oracle.affected_sets(st, rec, model)
        assert sets[0].tolist() == [n + 2]
        assert sets[1].tolist() == [3, n + 2]
        assert {3, n + 2} | set(st.out_neighbours(3)) <= set(sets[2].tolist())


def test_deleted_vertex_is_in_no_set_even_as_an_earlier_sink():
    """Sec. 3.2, vertex deletion: the incident edges go, then the vertex; what is left to update are its
    former out-neighbours and what lies downstream of them. The deleted id itself is in no set, also
    when an earlier operation of the same batch made it the sink of a changed edge, created it, or
    replaced its features, and also at hops beyond the first."""
    st, model, src, dst, feats = small_case(78, kind="sage_mean")
    n = len(feats)
    victim = int(dst[0])
    x = next(w for w in range(n) if w != victim and not st.has_edge(w, victim))
    outs = set(st.out_neighbours(victim)) - {victim}
    row = np.ones((2, feats.shape[1]))
    ops = [(ri.OP_EDGE_ADD, x, victim, 0),          # the victim is the sink of a changed edge
           (ri.OP_FEAT_UPDATE, victim, 0, 0),       # and has its features replaced
           (ri.OP_VERTEX_ADD, n, 0, 1),             # a vertex created and deleted in one batch
           (ri.OP_EDGE_ADD, x, n, 0),
           (ri.OP_VERTEX_DEL, victim, 0, 0),
           (ri.OP_VERTEX_DEL, n, 0, 0)]
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), row)
    assert rec.accepted.all()
    assert victim in rec.sinks and n in rec.sinks   # the premise: the root sets do name them
    sets = oracle.affected_sets(st, rec, model)
    assert sets[0].tolist() == []
    for l in range(1, len(model) + 1):
        got = set(sets[l].tolist())
        assert victim not in got and n not in got, l
        assert outs <= got, l
    # downstream of the former out-neighbours at hop 2 (the updated graph's edges)
    down = {w for o in outs for w in st.out_neighbours(o)}
    assert down <= set(sets[2].tolist())


@pytest.mark.parametrize("kind", ["gcn_sum", "sage_mean", "gin_sum"])
def test_cone_recompute_equals_bruteforce_and_full(kind):
    st, model, src, dst, feats = small_case(51, n=80, e=400, kind=kind)
    full = oracle.full_recompute(st, model)
    targets = [3, 17, 42, 79, st.cap - 1]
    cone = oracle.recompute_rows(st, model, targets)
    rows, vals = cone[-1]
    assert rows.tolist() == sorted(targets)
    nbrs = in_lists(st.cap, src, dst)
    memo = {}
    for r, val in zip(rows, vals):
        want = embed(int(r), len(model), model, st.h0, nbrs, st.alive, memo)
        np.testing.assert_allclose(val, want, rtol=1e-12, atol=1e-12)
    for l in range(len(model) + 1):
        r, v = cone[l]
        np.testing.assert_allclose(v, full[l][r], rtol=1e-12, atol=1e-12)


def test_apply_batch_validation_in_array_order():
    st, model, src, dst, feats = small_case(41)
    n = len(feats)
    u, v = int(src[0]), int(dst[0])
    ops = [(ri.OP_EDGE_ADD, u, v, 0),          # duplicate -> rejected
           (ri.OP_EDGE_DEL, u, v, 0),          # ok
           (ri.OP_EDGE_DEL, u, v, 0),          # now missing -> rejected
           (ri.OP_EDGE_ADD, u, v, 0),          # ok again
           (ri.OP_EDGE_ADD, n, 0, 0),          # n is dead -> rejected
           (ri.OP_VERTEX_ADD, n, 0, 0),        # ok
           (ri.OP_VERTEX_ADD, n, 0, 0),        # already live -> rejected
           (ri.OP_EDGE_ADD, n, 0, 0),          # ok now
           (ri.OP_VERTEX_DEL, st.cap - 1, 0, 0),   # dead -> rejected
           (ri.OP_FEAT_UPDATE, st.cap + 5, 0, 0),  # out of range -> rejected
           (7, 0, 0, 0)]                       # unknown kind -> rejected
    e0 = st.n_edges()
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), np.ones((1, feats.shape[1])))
    assert rec.accepted.tolist() == [False, True, False, True, False, True, False, True,
                                     False, False, False]
    assert st.n_edges() == e0 + 1
    assert rec.sinks == {v, 0} and rec.added == {n}


def test_max_rel_err_metric():
    want = np.array([[1.0, -2.0], [0.0, 0.0], [10.0, 0.0]])
    got = want + np.array([[0.0, 0.02], [0.04, 0.0], [0.0, 0.5]])
    alive = np.array([True, True, True])
    # row norms 2, 0, 10 -> tau = 4; errors 0.02/4, 0.04/4, 0.5/10
    assert abs(oracle.max_rel_err(got, want, alive) - 0.05) < 1e-15


# ---- weighted sum (Table 1, Sec. 3.3.3 "Other linear aggregators") -------------------------------
def weighted_case(seed, n=36, e=150, d0=5, kind="gcn_wsum", widths=(5, 7, 4)):
    rng = np.random.default_rng(seed)
    keys = rng.choice(n * n, size=e, replace=False)
    src, dst = keys // n, keys % n
    keep = src != dst
    src, dst = src[keep], dst[keep]
    w = rng.uniform(0.25, 1.75, src.size)
    feats = rng.standard_normal((n, d0))
    model = ri.make_model(kind, widths, seed + 1)
    st = oracle.GraphState(n, n + 4, src, dst, feats, weights=w)
    return st, model, src, dst, w, feats


@pytest.mark.parametrize("kind", ["gcn_wsum", "sage_wsum"])
@pytest.mark.parametrize("seed", [0, 1])
def test_weighted_sum_equals_vertexwise_bruteforce(kind, seed):
    st, model, src, dst, w, feats = weighted_case(seed, kind=kind)
    hs = oracle.full_recompute(st, model)
    nbrs, alpha = in_lists(st.cap, src, dst), in_weights(src, dst, w)
    f = np.zeros((st.cap, feats.shape[1]))
    f[: len(feats)] = feats
    memo = {}
    for v in range(st.cap):
        want = embed(v, len(model), model, f, nbrs, st.alive, memo, alpha)
        np.testing.assert_allclose(hs[-1][v], want, rtol=1e-12, atol=1e-12)


def test_weighted_sum_special_cases():
    """All weights 1: the plain sum. All weights c on a linear bias-free model: c^L times the plain sum.
    A mistake that takes alpha_vu for alpha_uv, or weights the self term, fails the brute force above;
    this one pins the scale."""
    st, model, src, dst, w, feats = weighted_case(3, kind="gcn_wsum")
    ones = oracle.GraphState(st.cap - 4, st.cap, src, dst, feats, weights=np.ones(src.size))
    plain = oracle.GraphState(st.cap - 4, st.cap, src, dst, feats)
    sum_model = [dict(l, agg="sum") for l in model]
    for a, b in zip(oracle.full_recompute(ones, model), oracle.full_recompute(plain, sum_model)):
        np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-13)
    lin = [dict(l, act_out="none", b0=np.zeros_like(l["b0"])) for l in model]
    scaled = oracle.GraphState(st.cap - 4, st.cap, src, dst, feats, weights=np.full(src.size, 0.5))
    got = oracle.full_recompute(scaled, lin)[-1]
    want = oracle.full_recompute(plain, [dict(l, agg="sum") for l in lin])[-1] * 0.5 ** len(lin)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_weighted_sum_after_a_batch():
    """Edge additions carry their weight in the operation's fourth word; an edge deleted and created
    again takes the new weight. Checked against the brute force on the resulting weighted edge set."""
    st, model, src, dst, w, feats = weighted_case(5, kind="sage_wsum")
    def bits(x):
        return int(np.array([x], dtype=np.float32).view(np.uint32)[0])
    s0, d0_ = int(src[0]), int(dst[0])
    free = next((u, v) for u in range(10) for v in range(10) if u != v and not st.has_edge(u, v))
    ops = [(ri.OP_EDGE_DEL, s0, d0_, 0), (ri.OP_EDGE_ADD, free[0], free[1], bits(1.5)),
           (ri.OP_EDGE_ADD, s0, d0_, bits(0.75)), (ri.OP_EDGE_DEL, int(src[1]), int(dst[1]), 0)]
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), None)
    assert rec.accepted.all()
    es, ed = st.edges()
    ew = st.edge_weights()
    alpha = in_weights(es, ed, ew)
    assert alpha[(s0, d0_)] == 0.75 and alpha[free] == 1.5 and (int(src[1]), int(dst[1])) not in alpha
    assert alpha[(int(src[2]), int(dst[2]))] == pytest.approx(float(w[2]))
    hs = oracle.full_recompute(st, model)
    nbrs = in_lists(st.cap, es, ed)
    memo = {}
    for v in range(st.cap):
        want = embed(v, len(model), model, st.h0, nbrs, st.alive, memo, alpha)
        np.testing.assert_allclose(hs[-1][v], want, rtol=1e-12, atol=1e-12)


def test_edge_weight_replacement():
    """The sixth operation: a new weight for an existing edge of a weighted graph. The result equals the brute
    force on the re-weighted edge set; the sink is in every affected set and, with linear activations, the
    rows that change are exactly the sets; on a missing edge, a dead endpoint or an unweighted graph the
    operation is rejected; a weight replaced twice in one batch ends up with the later value."""
    def bits(x):
        return int(np.array([x], dtype=np.float32).view(np.uint32)[0])
    st, model, src, dst, w, feats = weighted_case(9, kind="gcn_wsum", widths=(5, 7, 6, 4))
    for lay in model:
        lay["act_out"] = "none"
    before = oracle.full_recompute(st, model)
    (u0, v0), (u1, v1) = (int(src[0]), int(dst[0])), (int(src[5]), int(dst[5]))
    missing = next((u, v) for u in range(12) for v in range(12) if u != v and not st.has_edge(u, v))
    ops = [(ri.OP_EDGE_REWEIGHT, u0, v0, bits(1.25)), (ri.OP_EDGE_REWEIGHT, u1, v1, bits(0.5)),
           (ri.OP_EDGE_REWEIGHT, missing[0], missing[1], bits(1.0)),        # no such edge
           (ri.OP_EDGE_REWEIGHT, u0, st.cap - 1, bits(1.0)),                  # dead endpoint
           (ri.OP_EDGE_REWEIGHT, u1, v1, bits(0.625))]                        # again: the later value stays
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), None)
    assert rec.accepted.tolist() == [True, True, False, False, True]
    assert rec.sinks == {v0, v1} and not rec.added and not rec.feat
    es, ed = st.edges()
    alpha = in_weights(es, ed, st.edge_weights())
    assert alpha[(u0, v0)] == 1.25 and alpha[(u1, v1)] == 0.625 and len(alpha) == len(src)
    after = oracle.full_recompute(st, model)
    nbrs = in_lists(st.cap, es, ed)
    memo = {}
    for v in range(st.cap):
        want = embed(v, len(model), model, st.h0, nbrs, st.alive, memo, alpha)
        np.testing.assert_allclose(after[-1][v], want, rtol=1e-12, atol=1e-12)
    sets = oracle.affected_sets(st, rec, model)
    assert sets[0].tolist() == []
    for l in range(1, len(model) + 1):
        assert {v0, v1} <= set(sets[l].tolist())
        changed = set(np.nonzero(np.abs(after[l] - before[l]).max(axis=1) > 0)[0].tolist())
        assert changed == set(sets[l].tolist()), l
    # a graph without weights has nothing to replace
    plain, _, s2, d2, _ = small_case(9)
    rec = plain.apply_batch(np.array([(ri.OP_EDGE_REWEIGHT, int(s2[0]), int(d2[0]), bits(2.0))], dtype=np.uint32), None)
    assert rec.accepted.tolist() == [False] and not rec.sinks


# ---- max / min aggregation (Table 1, Sec. 3.4.2 "Monotonic Aggregation Functions") ----------------
@pytest.mark.parametrize("kind", ["gcn_max", "gcn_min", "sage_max"])
@pytest.mark.parametrize("seed", [0, 1])
def test_extreme_aggregation_equals_vertexwise_bruteforce(kind, seed, monkeypatch):
    st, model, src, dst, feats = small_case(seed, kind=kind)
    if seed == 1:
        monkeypatch.setattr(oracle.ripple_oracle, "SLAB_ELEMENTS", 64)    # many slabs of a few rows each
    hs = oracle.full_recompute(st, model)
    nbrs = in_lists(st.cap, src, dst)
    f = np.zeros((st.cap, feats.shape[1]))
    f[: len(feats)] = feats
    memo = {}
    for l in range(len(model) + 1):
        for v in range(st.cap):
            want = embed(v, l, model, f, nbrs, st.alive, memo)
            np.testing.assert_allclose(hs[l][v], want, rtol=1e-12, atol=1e-12)


def test_max_cases_of_the_paper():
    """The values printed with the three cases of Sec. 3.4.2 (tests/golden/max_cases.txt)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "max_cases.txt")) if l.strip() and not l.startswith("#")]
    assert [r[5] for r in rows] == ["unchanged", "incremental", "recompute"]
    for b, c_old, c_new, a_before, a_after, _ in rows:
        # vertices: 0 = A, 1 = B, 2 = C; edges B -> A and C -> A
        for c_val, want in ((c_old, a_before), (c_new, a_after)):
            feats = np.array([[0.0], [float(b)], [float(c_val)]])
            st = oracle.GraphState(3, 3, np.array([1, 2]), np.array([0, 0]), feats)
            x = oracle.aggregate(oracle.in_adjacency(st), st.h0, "max")
            assert x[0, 0] == float(want)
            assert x[1, 0] == 0.0 and x[2, 0] == 0.0            # no in-neighbours: 0


def test_extreme_aggregation_identities():
    st, model, src, dst, feats = small_case(4, kind="gcn_max")
    a_in = oracle.in_adjacency(st)
    h = np.random.default_rng(9).standard_normal((st.cap, 6))
    mx, mn = oracle.aggregate(a_in, h, "max"), oracle.aggregate(a_in, h, "min")
    mean = oracle.aggregate(a_in, h, "mean")
    np.testing.assert_array_equal(mx, -oracle.aggregate(a_in, -h, "min"))       # duality
    has = np.asarray(a_in.ones.getnnz(axis=1)) > 0
    assert (mn[has] <= mean[has] + 1e-15).all() and (mean[has] <= mx[has] + 1e-15).all()
    assert (mx[~has] == 0).all() and (mn[~has] == 0).all() and (~has).any()
    # every value of the result is one of the neighbours' values, and none of them exceeds it
    nbrs = in_lists(st.cap, src, dst)
    for v in np.flatnonzero(has)[:10]:
        block = h[nbrs[v]]
        assert (block <= mx[v]).all() and (block >= mn[v]).all()
        assert all(mx[v, k] in block[:, k] and mn[v, k] in block[:, k] for k in range(6))
    # one in-neighbour each (a cycle): max = min = sum = mean = the predecessor's row
    n = 12
    cyc = oracle.GraphState(n, n, np.arange(n), (np.arange(n) + 1) % n, h[:n])
    a_c = oracle.in_adjacency(cyc)
    want = np.roll(h[:n], 1, axis=0)
    for agg in ("max", "min", "sum", "mean"):
        np.testing.assert_array_equal(oracle.aggregate(a_c, h[:n], agg), want)


def test_max_after_a_batch_with_all_update_kinds():
    st, model, src, dst, feats = small_case(11, kind="sage_max")
    n = len(feats)
    rng = np.random.default_rng(5)
    payload = rng.standard_normal((2, feats.shape[1]))
    free = next((u, v) for u in range(10) for v in range(10) if u != v and not st.has_edge(u, v))
    ops = [(ri.OP_EDGE_DEL, int(src[0]), int(dst[0]), 0), (ri.OP_EDGE_ADD, free[0], free[1], 0),
           (ri.OP_FEAT_UPDATE, 5, 0, 0), (ri.OP_VERTEX_ADD, n, 0, 1), (ri.OP_EDGE_ADD, n, 4, 0),
           (ri.OP_EDGE_ADD, 6, n, 0), (ri.OP_VERTEX_DEL, 9, 0, 0)]
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), payload)
    assert rec.accepted.all()
    hs = oracle.full_recompute(st, model)
    es, ed = st.edges()
    nbrs = in_lists(st.cap, es, ed)
    memo = {}
    for v in range(st.cap):
        want = embed(v, len(model), model, st.h0, nbrs, st.alive, memo)
        np.testing.assert_allclose(hs[-1][v], want, rtol=1e-12, atol=1e-12)


# ---- graph attention (Sec. 3.4.1, Eq. 3) ------------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 1])
def test_attention_equals_vertexwise_bruteforce(seed):
    st, model, src, dst, feats = small_case(seed, kind="gat")
    hs = oracle.full_recompute(st, model)
    nbrs = in_lists(st.cap, src, dst)
    f = np.zeros((st.cap, feats.shape[1]))
    f[: len(feats)] = feats
    memo = {}
    for l in range(len(model) + 1):
        for v in range(st.cap):
            want = embed(v, l, model, f, nbrs, st.alive, memo)
            np.testing.assert_allclose(hs[l][v], want, rtol=1e-11, atol=1e-12)


def test_attention_special_cases():
    st, model, src, dst, feats = small_case(6, kind="gat", widths=(5, 7, 4))
    # zero attention vectors: every coefficient is 1/deg, the layer is the mean of the projected rows
    flat = [dict(l, att=np.zeros_like(l["att"])) for l in model]
    mean = [dict(l, agg="mean") for l in model]
    for a, b in zip(oracle.full_recompute(st, flat), oracle.full_recompute(st, mean)):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    # a sink-side vector only: the score is the same for all in-neighbours of a vertex, again the mean
    d1 = model[0]["d_out"]
    sink_only = [dict(model[0], att=np.concatenate([np.zeros(d1), model[0]["att"][d1:]]))]
    np.testing.assert_allclose(oracle.full_recompute(st, sink_only)[1], oracle.full_recompute(st, mean[:1])[1],
                               rtol=1e-12, atol=1e-13)
    # one in-neighbour each: the coefficient is 1 whatever the scores are
    n = 12
    h = np.random.default_rng(2).standard_normal((n, 5))
    cyc = oracle.GraphState(n, n, np.arange(n), (np.arange(n) + 1) % n, h)
    got = oracle.full_recompute(cyc, model[:1])[1]
    want = np.maximum(np.roll(h, 1, axis=0) @ np.asarray(model[0]["W0"], dtype=np.float64) + model[0]["b0"], 0.0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
    # the source-side vector matters: swapping the halves changes the result
    swapped = [dict(model[0], att=np.concatenate([model[0]["att"][d1:], model[0]["att"][:d1]]))]
    assert np.abs(oracle.full_recompute(st, swapped)[1] - oracle.full_recompute(st, model[:1])[1]).max() > 1e-3


def test_attention_after_a_batch_with_all_update_kinds():
    st, model, src, dst, feats = small_case(12, kind="gat")
    n = len(feats)
    rng = np.random.default_rng(5)
    payload = rng.standard_normal((2, feats.shape[1]))
    free = next((u, v) for u in range(10) for v in range(10) if u != v and not st.has_edge(u, v))
    ops = [(ri.OP_EDGE_DEL, int(src[0]), int(dst[0]), 0), (ri.OP_EDGE_ADD, free[0], free[1], 0),
           (ri.OP_FEAT_UPDATE, 5, 0, 0), (ri.OP_VERTEX_ADD, n, 0, 1), (ri.OP_EDGE_ADD, n, 4, 0),
           (ri.OP_EDGE_ADD, 6, n, 0), (ri.OP_VERTEX_DEL, 9, 0, 0)]
    rec = st.apply_batch(np.array(ops, dtype=np.uint32), payload)
    assert rec.accepted.all()
    hs = oracle.full_recompute(st, model)
    es, ed = st.edges()
    nbrs = in_lists(st.cap, es, ed)
    memo = {}
    for v in range(st.cap):
        want = embed(v, len(model), model, st.h0, nbrs, st.alive, memo)
        np.testing.assert_allclose(hs[-1][v], want, rtol=1e-11, atol=1e-12)
    # sampled rows through their cones give the same values as the full recomputation
    cone = oracle.recompute_rows(st, model, [0, 3, 7, n])
    np.testing.assert_allclose(cone[-1][1], hs[-1][cone[-1][0]], rtol=1e-12, atol=1e-13)


def test_attention_row_depends_on_the_vertex_own_embedding():
    """Why a vertex of hop l-1's set belongs to hop l's set under attention (Sec. 3.4.1): only its own
    features change, its in-neighbours do not, and its row still moves, because the two scores lie on
    different sides of the LeakyReLU before or after."""
    n, d = 3, 2
    feats = np.array([[0.0, 0.0], [1.0, 0.0], [-1.0, 0.0]])
    lay = dict(d_in=d, d_hidden=0, d_out=d, eps=0.0, act_inner="none", act_out="none", W1=None, b1=None, agg="attn",
               self="none", W0=np.eye(d, dtype=np.float32), b0=np.zeros(d, dtype=np.float32),
               att=np.array([1.0, 0.0, 0.0, 1.0], dtype=np.float32))      # z_uv = lrelu(p_u[0] + p_v[1])
    st = oracle.GraphState(n, n, np.array([1, 2]), np.array([0, 0]), feats)
    before = oracle.full_recompute(st, [lay])[1][0].copy()
    # scores of 1 -> 0 and 2 -> 0 are lrelu(1) and lrelu(-1): weights e^1 and e^-0.2
    w1, w2 = np.exp(1.0), np.exp(-0.2)
    np.testing.assert_allclose(before, [(w1 - w2) / (w1 + w2), 0.0], rtol=1e-12, atol=1e-15)
    rec = st.apply_batch(np.array([(ri.OP_FEAT_UPDATE, 0, 0, 0)], dtype=np.uint32), np.array([[0.0, 3.0]]))
    after = oracle.full_recompute(st, [lay])[1][0]
    w1, w2 = np.exp(4.0), np.exp(2.0)                     # both scores positive now: lrelu(4), lrelu(2)
    np.testing.assert_allclose(after, [(w1 - w2) / (w1 + w2), 0.0], rtol=1e-12, atol=1e-15)
    assert abs(after[0] - before[0]) > 0.1
    assert oracle.affected_sets(st, rec, [lay])[1].tolist() == [0]
