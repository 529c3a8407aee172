"""ripple_full_infer against the oracle's layer-wise recompute (Eq. 1-2)."""
import numpy as np
import pytest

import paper_2601_12347_amd as rp
import ripple_inputs as ri
from harness import make_pair, config_pair, Pair

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,widths", [
    ("gcn_sum", (12, 20, 8)),
    ("gcn_mean", (12, 70, 33)),          # ragged widths: not multiples of 4, tails in every tile
    ("sage_mean", (16, 40, 24, 10)),
    ("sage_sum", (13, 29, 7)),
    ("gin_sum", (16, 32, 12)),
])
def test_bootstrap_matches_oracle(kind, widths):
    print("case", kind, widths, flush=True)
    pair, _ = make_pair(n=700, e=5000, d0=widths[0], kind=kind, widths=widths, seed=3)
    try:
        pair.check_graph()
        pair.check_embeddings()
        pair.check_aggregates()
    finally:
        pair.close()


def test_bootstrap_wide_layers_span_several_tiles():
    print("case wide", flush=True)
    pair, _ = make_pair(n=1500, e=9000, d0=100, kind="sage_mean", widths=(100, 256, 300, 47), seed=5)
    try:
        pair.check_embeddings()
    finally:
        pair.close()


@pytest.mark.parametrize("kind,widths", [("gcn_sum", (16, 64, 24)), ("sage_mean", (100, 256, 300, 47)),
                                         ("gin_sum", (16, 32, 12)), ("gcn_mean", (24, 128, 40))])
def test_bootstrap_bf16_store(kind, widths):
    """bfloat16 embeddings: bf16 matrix cores (default) and the fp32 matrix path on the same
    rounded inputs must both stay within the bf16 tolerance of the fp64 oracle."""
    print("case bf16", kind, flush=True)
    pair, _ = make_pair(n=900, e=7000, d0=widths[0], kind=kind, widths=widths, store="bf16", seed=4)
    try:
        errs_mfma, want = pair.check_embeddings()
        rp.ripple_set_option(pair.ctx, rp.OPT_BF16_MFMA, 0)
        rp.ripple_full_infer(pair.ctx)
        errs_f32, _ = pair.check_embeddings(want=want)
        print("  max rel err bf16 mfma", ["%.1e" % e for e in errs_mfma], "fp32 path", ["%.1e" % e for e in errs_f32], flush=True)
    finally:
        pair.close()


@pytest.mark.parametrize("name", ["sparse_sage_mean", "sparse_gcn_wsum"])
def test_streaming_and_tiled_kernels_agree_on_the_sparse_graph(name):
    """With about 170 K rows, layers of 256 -> 256 take the persistent streaming row update, the narrow last layer
    the barrier-free kernel for both of its products and the flattened row update; with the option off the tiled
    kernels run instead. Both must be within tolerance of the oracle, and within rounding of each other (the
    streaming kernel applies the mean's 1 / deg to the finished row instead of the gathered one)."""
    cfg = ri.get_config(name)
    print("case", cfg.name, flush=True)
    pair, _ = config_pair(cfg)
    try:
        errs_on, want = pair.check_embeddings()
        on = [pair.gpu_layer(l) for l in range(1, pair.L + 1)]
        rp.ripple_set_option(pair.ctx, rp.OPT_STREAM_TRANSFORM, 0)
        rp.ripple_full_infer(pair.ctx)
        errs_off, _ = pair.check_embeddings(want=want)
        off = [pair.gpu_layer(l) for l in range(1, pair.L + 1)]
        for l, (x, y) in enumerate(zip(on, off), start=1):
            diff = float(np.abs(x - y).max() / max(np.abs(y).max(), 1e-30))
            print("  layer %d: streaming vs tiled %.2e (oracle: %.1e / %.1e)" % (l, diff, errs_on[l], errs_off[l]), flush=True)
            assert diff <= 1e-5
        pair.check_aggregates()
    finally:
        pair.close()


def test_bootstrap_tiny_config():
    print("case tiny config", flush=True)
    pair, _ = config_pair(ri.get_config("tiny_gcn_sum"))
    try:
        pair.check_graph()
        pair.check_embeddings()
        pair.check_aggregates()
    finally:
        pair.close()


def test_empty_graph_and_isolated_vertices():
    print("case empty", flush=True)
    feats = ri.features(5, 8, 1)
    model = ri.make_model("gcn_sum", (8, 8, 4), 2)
    e = np.zeros(0, dtype=np.uint32)
    pair = Pair(5, 9, e, e, feats, model)
    try:
        pair.check_graph()
        pair.check_embeddings()
    finally:
        pair.close()


def test_call_order_and_argument_errors():
    print("case errors", flush=True)
    feats = ri.features(4, 8, 1)
    model = ri.make_model("gcn_sum", (8, 4), 2)
    src = np.array([0, 1], dtype=np.uint32)
    dst = np.array([1, 2], dtype=np.uint32)
    with pytest.raises(rp.RippleError) as ei:                     # endpoint beyond the live range
        rp.ripple_init_graph(4, 8, np.array([0, 5], dtype=np.uint32), dst, feats)
    assert ei.value.status == rp.binding.RIPPLE_EINVAL
    ctx = rp.ripple_init_graph(4, 8, src, dst, feats)
    try:
        with pytest.raises(rp.RippleError) as ei:
            rp.ripple_full_infer(ctx)                             # no model yet
        assert ei.value.status == rp.binding.RIPPLE_ESTATE
        with pytest.raises(rp.RippleError) as ei:
            rp.ripple_apply_updates(ctx, np.zeros((1, 4), np.uint32), None)
        assert ei.value.status == rp.binding.RIPPLE_ESTATE
        bad = ri.make_model("gcn_sum", (7, 4), 2)                 # widths do not chain with d0 = 8
        with pytest.raises(rp.RippleError) as ei:
            rp.ripple_load_model(ctx, bad)
        assert ei.value.status == rp.binding.RIPPLE_EINVAL
        rp.ripple_load_model(ctx, model)
        rp.ripple_full_infer(ctx)
        for ops in ([(9, 0, 0, 0)], [(ri.OP_EDGE_ADD, 0, 8, 0)], [(ri.OP_FEAT_UPDATE, 1, 0, 3)]):
            with pytest.raises(rp.RippleError) as ei:             # unknown kind / id / payload row
                rp.ripple_apply_updates(ctx, np.array(ops, dtype=np.uint32), np.zeros((1, 8), np.float32))
            assert ei.value.status == rp.binding.RIPPLE_EINVAL
        with pytest.raises(rp.RippleError):
            rp.ripple_get_embeddings(ctx, 5, 4, n_rows=2)
        out = rp.ripple_get_embeddings(ctx, 1, 4, ids=np.array([3, 7], dtype=np.uint32))
        assert not out[1].any()                                   # id 7 was never created
    finally:
        rp.ripple_destroy(ctx)


def test_measured_peaks_are_plausible():
    """The chip's own rates (streaming copy, random line gathers, float atomics, matrix-core loops) that bench.py
    prints beside the nominal peaks: each must lie between a loose floor and the published figure."""
    p = rp.ripple_measure_peaks()
    print("measured peaks", {k: round(v, 1) for k, v in p.items()}, flush=True)
    assert 2000.0 < p["hbm_copy_gbps"] < 8000.0
    assert 2000.0 < p["hbm_read_gbps"] < 8000.0
    assert 10.0 < p["gather_glines"] < 62.5                  # 62.5e9 lines of 128 bytes per second would be 8 TB/s
    assert 50.0 < p["atomic_gops"] < 2000.0
    assert 60.0 < p["mfma_f32_tflops"] < 157.3 * 1.02
    assert 800.0 < p["mfma_bf16_tflops"] < 2500.0 * 1.02
    assert p["compute_units"] >= 64
