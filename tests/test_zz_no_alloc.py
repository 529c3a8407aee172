"""The entry point that allocates nothing (ripple_get_affected_static) against ripple_get_affected, through
the C ABI: two calls in a row, the second on a smaller input, so that what the first call left in the static
device array would show if the second depended on it."""
import numpy as np
import pytest

import paper_2601_12347_amd as rp
import ripple_inputs as ri
from harness import make_pair, make_stream

pytestmark = pytest.mark.gpu

MIX = {"edge_add": 0.45, "edge_del": 0.25, "feat": 0.2, "vadd": 0.05, "vdel": 0.05}


def compare_all_layers(torch, pair, ids_t, n_t):
    for l in range(pair.L + 1):
        want, n_want = rp.ripple_get_affected(pair.ctx, l, pair.cap)
        ids_t.fill_(0xFFFFFFF)
        n_t.fill_(12345)
        rp.ripple_get_affected_static(pair.ctx, l, ids_t.data_ptr(), ids_t.numel(), n_t.data_ptr())
        n = int(n_t.cpu()[0])
        assert n == n_want, (l, n, n_want)
        got = ids_t.cpu().numpy()[:n].astype(np.int64)
        assert np.array_equal(got, want.astype(np.int64)), f"layer {l}"
        # a buffer that is too small: the count is the full one, only `cap` ids are written
        if n > 3:
            ids_t.fill_(0xFFFFFFF)
            rp.ripple_get_affected_static(pair.ctx, l, ids_t.data_ptr(), 3, n_t.data_ptr())
            assert int(n_t.cpu()[0]) == n_want
            head = ids_t.cpu().numpy()
            assert np.array_equal(head[:3].astype(np.int64), want[:3].astype(np.int64)) and np.all(head[3:] == 0xFFFFFFF)


def test_no_allocation_entry_point_matches_get_affected():
    torch = pytest.importorskip("torch")
    print("case no-allocation affected sets", flush=True)
    # a graph with more than 256 bitmap words, so that the compaction has several blocks whose sums go through
    # the static array (12,000 vertices = 375 words = 2 blocks), then a much smaller one
    big, g_big = make_pair(n=12000, e=60000, d0=8, kind="sage_mean", widths=(8, 16, 6), seed=71, slack=500)
    small, g_small = make_pair(n=300, e=1500, d0=8, kind="gcn_sum", widths=(8, 16, 6), seed=73)
    try:
        ids_t = torch.empty(big.cap + 8, dtype=torch.int32, device="cuda")
        n_t = torch.empty(1, dtype=torch.int32, device="cuda")
        s_big = make_stream(big, g_big, MIX, 75)
        ops, payload, _ = s_big.next_batch(400)
        big.step(ops, payload, check=False)
        compare_all_layers(torch, big, ids_t, n_t)
        s_small = make_stream(small, g_small, MIX, 77)
        ops, payload, _ = s_small.next_batch(10)
        small.step(ops, payload, check=False)
        compare_all_layers(torch, small, ids_t, n_t)
        # and back on the first context with a smaller batch
        ops, payload, _ = s_big.next_batch(5)
        big.step(ops, payload, check=False)
        compare_all_layers(torch, big, ids_t, n_t)
        # a batch that had to be cut into pieces reports the union of its pieces' sets
        u, v = int(g_small[0][0]), int(g_small[1][0])
        small_ops = np.array([(ri.OP_EDGE_DEL, u, v, 0), (ri.OP_EDGE_ADD, u, v, 0)], dtype=np.uint32)
        if small.ora.has_edge(u, v):
            small.step(small_ops, None, check=False)
            compare_all_layers(torch, small, ids_t, n_t)
        # host pointers are refused, nothing is written
        host = np.zeros(4, dtype=np.uint32)
        with pytest.raises(rp.RippleError) as ei:
            rp.ripple_get_affected_static(small.ctx, 0, ids_t.data_ptr(), 4, host.ctypes.data)
        assert ei.value.status == rp.binding.RIPPLE_EINVAL
    finally:
        big.close()
        small.close()
