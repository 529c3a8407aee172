#!/usr/bin/env python3
"""Benchmark of the incremental-propagation hot path on one MI355X.

One step = one batch of updates through ripple_apply_updates (ingest + apply,
then per layer frontier, scatter, transform), host entry to synchronised return,
with the batch's operations and feature rows already resident in HBM. Prints ONE
JSON line: updates/s over the timed batches, p50/p99 batch latency, the roofline
figures of the dominant kernel (HIP-event time measured inside the library on its
own stream, algorithmic bytes/flops from the per-batch work counters) and the CPU
oracle's rate on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# HBM bytes per launch of the kernel classes of the default workload (dense_sage_mean, 10,000 updates per
# batch), measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and scaled by a 1 GiB copy of known size
# (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0; the file named below holds commands and raw values). bench.py cannot run
# the profiler on itself; for any other workload `traffic` is null.
TRAFFIC_SOURCE = "profiles/hbm_traffic_dense_sage_mean_bs10000_pmc.txt"
MEASURED_TRAFFIC_BYTES = {
    ("dense_sage_mean", 10000): {"scatter_l3": 10.0e9, "scatter_l2": 7.2e9, "transform_l2": 4.9e9, "transform_l3": 5.0e9},
}


def algorithmic_work(st, model, widths, store, L, layer_info, n_edges=0):
    """Per (phase, layer): algorithmic bytes and flops summed over the timed batches.

    scatter(l):   every message row (delta, or projected delta) once, the walked rows' index
                  pairs and column ids once, and each distinct destination row of the cached
                  aggregate read and written once;
    frontier(l):  index pairs + column ids of the walked out-rows, the list written; not priced
                  where the hop discovered A_l while scattering (messages * 8 >= edges, the
                  library's own rule), since no frontier kernel runs there;
    transform(l): per dirty row the gathered input row, old H read, new H and delta written;
                  flops 2*K*d_out per row (plus the hidden stage for two-stage updates). For
                  project-first layers the projection of the hop's deltas (a_{l-1} rows) is
                  part of this class and the row transform reads h_self and the projected aggregate.
                  Layers with a cached self term multiply h_self W_self on A_{l-1} only.
    """
    s_h = 2 if store == "bf16" else 4
    out = {}
    for l in range(1, L + 1):
        lay = model[l - 1]
        d_prev, d_out = widths[l - 1], widths[l]
        w_agg, projected, self_cached = layer_info[l][:3]
        # a message row: the aggregate's width in fp32, or one 128-byte line where the layer packs its messages
        row_bytes = 128 if (len(layer_info[l]) > 3 and layer_info[l][3]) else w_agg * 4
        a_prev, a_l, m_l, t_l = st.rows[l - 1], st.rows[l], st.msgs[l], st.touched[l]
        out[("scatter", l)] = dict(bytes=a_prev * row_bytes + 8 * a_prev + 4 * m_l + 2 * t_l * w_agg * 4, flops=m_l * w_agg,
                                   # what a cache-less per-message scheme moves: one message row gathered per message
                                   msg_bytes=m_l * (row_bytes + 4) + 2 * t_l * w_agg * 4,
                                   lines=m_l * ((row_bytes + 127) // 128))
        discovered = l >= 2 and n_edges and m_l * 8 >= n_edges * max(st.batches, 1)
        if not discovered:
            out[("frontier", l)] = dict(bytes=8 * a_prev + 4 * m_l + 4 * a_l, flops=0)
        self_w = lay["d_in"] if lay["self"] != "none" else 0
        next_projected = l < L and layer_info[l + 1][1]
        out_bytes = d_out * s_h * 2 + (d_out * 4 if (l < L and not next_projected) else 0) + 4
        if lay["agg"] == "attn":
            # projection of A_{l-1} (row in, d_out floats out), then per dirty row numerator, denominator, old and new row
            flops = 2 * a_prev * d_prev * d_out
            nbytes = a_prev * (d_prev * s_h + d_out * 4) + a_l * (d_out * 4 + 4 + out_bytes)
        elif self_cached:
            # self term refreshed on A_{l-1} (row in, d_out floats out); per dirty row the cached self
            # term and the aggregate (projected, or multiplied by W_neigh here) are read
            flops = 2 * a_prev * self_w * d_out + (2 * a_prev * d_prev * d_out if projected else 2 * a_l * d_prev * d_out)
            nbytes = a_prev * (self_w * s_h + d_out * 4) + a_l * (d_out * 4 + w_agg * 4 + out_bytes)
            if projected:                               # rows of A_{l-1} in, message out, running sum read and written
                nbytes += a_prev * (d_prev * s_h + row_bytes + 2 * w_agg * 4) - a_prev * self_w * s_h   # one pass serves both products
        elif projected:
            flops = 2 * a_l * self_w * d_out + 2 * a_prev * d_prev * d_out
            nbytes = a_l * (self_w * s_h + w_agg * 4 + out_bytes) + a_prev * (d_prev * s_h + row_bytes + 2 * w_agg * 4)
        else:
            k = lay["d_in"] + self_w if lay["self"] == "concat" else lay["d_in"]
            if lay["d_hidden"]:
                flops = 2 * a_l * (k * lay["d_hidden"] + lay["d_hidden"] * d_out)
            else:
                flops = 2 * a_l * k * d_out
            nbytes = a_l * (lay["d_in"] * 4 + self_w * s_h + out_bytes)
        out[("transform", l)] = dict(bytes=nbytes, flops=flops)
    return out


def cpu_model():
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_batch_seconds(cfg, n, e, top_share, bs, threads):
    """One batch applied to the oracle's graph, every embedding recomputed (fp64) and the affected sets derived,
    with the linear-algebra library held to `threads` threads (None: as many as it takes by itself)."""
    import oracle
    import ripple_inputs as ri
    from contextlib import nullcontext
    try:
        from threadpoolctl import threadpool_limits, threadpool_info
    except ImportError:
        threadpool_limits, threadpool_info = None, None
    src, dst, out_law, in_law = ri.chung_lu_graph(n, e, cfg.gamma, top_share, cfg.graph_seed)
    feats = ri.features(n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(cfg.model, cfg.widths, cfg.weight_seed)
    stream = ri.UpdateStream(n, n + cfg.vertex_slack, src, dst, out_law, in_law, cfg.d0, cfg.mix, cfg.stream_seed,
                             weighted=cfg.weighted)
    st = oracle.GraphState(n, n + cfg.vertex_slack, src, dst, feats,
                           weights=ri.edge_weights(len(src), cfg.graph_seed + 100) if cfg.weighted else None)
    ops, payload, _ = stream.next_batch(bs)
    del src, dst, stream
    limit = threadpool_limits(limits=threads) if (threads and threadpool_limits) else nullcontext()
    with limit:
        used = max([p.get("num_threads", 1) for p in threadpool_info()] + [1]) if threadpool_info else (os.cpu_count() or 1)
        t0 = time.perf_counter()
        rec = st.apply_batch(ops, payload)
        oracle.full_recompute(st, model)
        oracle.affected_sets(st, rec, model)
        dt = time.perf_counter() - t0
    return dt, int(used)


def cpu_baseline(cfg, bs, scale, full_size=False):
    """The oracle as it stands, timed on this machine's host cores: one batch applied and everything
    recomputed in fp64, once with the linear-algebra library on all the threads it takes and once on one.
    Default: a bounded sample, a 1/scale copy of the workload (same recipe, N/scale vertices, E/scale edges,
    bs/scale updates); recomputation is linear in N and E (Sec. 3.5's operation count with a_l = N), so the
    full-size time per batch is the sample's times scale. full_size: the benchmark's own graph and batch
    (minutes on the dense graph). The sparse aggregation product of the oracle runs on one thread either way."""
    if full_size:
        scale = 1
    n, e = max(cfg.n // scale, 64), max(cfg.e // scale, 256)
    top = cfg.top_share if scale == 1 else min(cfg.top_share * scale, 0.05)
    sample_bs = max(bs // scale, 1)
    dt_all, used = _oracle_batch_seconds(cfg, n, e, top, sample_bs, None)
    dt_one, _ = _oracle_batch_seconds(cfg, n, e, top, sample_bs, 1) if not full_size else (None, 1)
    est_full = dt_all * scale
    what = (f"the benchmark's own graph and batch ({n} vertices, {e} edges, {sample_bs} updates): {dt_all:.1f} s"
            if scale == 1 else
            f"a 1/{scale}-scale graph of the same recipe ({n} vertices, {e} edges, {sample_bs} updates): {dt_all:.2f} s, "
            f"scaled x{scale} to the full graph ({est_full:.1f} s per batch of {bs}); an estimate, not a timing of the "
            f"full-size inputs (--cpu-baseline-full runs those)")
    out = {"value": bs / est_full, "unit": "updates/s", "cores": used, "kind": "oracle",
           "sample": "fp64 full recompute + affected sets for one batch on " + what,
           "sample_seconds": dt_all, "scaled": scale != 1, "cpu_model": cpu_model(), "host_cores": os.cpu_count(),
           "note": "the dense products use `cores` threads; the sparse aggregation product is single-threaded"}
    if dt_one is not None:
        out["value_single_thread"] = bs / (dt_one * scale)
        out["sample_seconds_single_thread"] = dt_one
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="dense_sage_mean")
    ap.add_argument("--bs", type=int, default=0, help="updates per batch (default: the config's largest)")
    ap.add_argument("--cpu-scale", type=int, default=0, help="oracle sample is a 1/scale graph (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-full", action="store_true",
                    help="time the oracle on the benchmark's own full-size graph and batch instead of the scaled sample (minutes)")
    ap.add_argument("--no-host-inputs", action="store_true", help="skip the extra batches handed over as host buffers")
    ap.add_argument("--no-peaks", action="store_true", help="skip measuring the chip's own copy / gather / atomic / matrix-core rates")
    ap.add_argument("--scatter-mode", type=int, default=0)
    ap.add_argument("--pull-ratio", type=int, default=0)
    ap.add_argument("--deterministic", action="store_true", help="bit-reproducible aggregation (RIPPLE_OPT_DETERMINISTIC)")
    ap.add_argument("--sparse-frontier", type=int, default=-1, help="0 = always scan the bitmap for the hop's list")
    ap.add_argument("--split-mfma", type=int, default=-1,
                    help="fp32 storage: 1 = products on the bf16 matrix cores with operands split in three, 0 = fp32 matrix path")
    ap.add_argument("--bf16-mfma", type=int, default=1, help="bf16 storage only: 0 = multiply on the fp32 matrix path")
    ap.add_argument("--stream-transform", type=int, default=-1,
                    help="0 = tiled kernels for the 256 -> 256 row updates and the last layer's projections; 1 = streaming kernels on large hops (default); 2 = at any size")
    ap.add_argument("--sorted-messages", type=int, default=-1, help="RIPPLE_OPT_SORTED_MESSAGES (default 1)")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="leave the library's per-kernel HIP events off (no roofline object; lowest latency)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2601_12347_amd as rp
    import ripple_inputs as ri

    cfg = ri.get_config(args.config)
    bs = args.bs or max(cfg.batch_sizes)
    t0 = time.time()
    src, dst, out_law, in_law = ri.chung_lu_graph(cfg.n, cfg.e, cfg.gamma, cfg.top_share, cfg.graph_seed)
    feats = ri.features(cfg.n, cfg.d0, cfg.feat_seed)
    model = ri.make_model(cfg.model, cfg.widths, cfg.weight_seed)
    log(f"[bench] graph {cfg.name}: {cfg.n} vertices, {cfg.e} edges generated in {time.time() - t0:.1f}s")
    t0 = time.time()
    # room for every edge the staged batches can add (a long run of large batches on a small graph outgrows the config's)
    edge_capacity = max(cfg.edge_capacity, len(src) + (args.warmup + args.steps) * bs + 4096)
    if cfg.weighted:
        ctx = rp.ripple_init_graph_weighted(cfg.n, cfg.vertex_capacity, src, dst, ri.edge_weights(len(src), cfg.graph_seed + 100),
                                            feats, store=cfg.store, edge_capacity=edge_capacity)
    else:
        ctx = rp.ripple_init_graph(cfg.n, cfg.vertex_capacity, src, dst, feats, store=cfg.store,
                                   edge_capacity=edge_capacity)
    if args.deterministic:
        rp.ripple_set_option(ctx, rp.OPT_DETERMINISTIC, 1)
    if args.split_mfma >= 0:
        rp.ripple_set_option(ctx, rp.OPT_SPLIT_MFMA, args.split_mfma)
    rp.ripple_load_model(ctx, model)
    rp.ripple_full_infer(ctx)
    log(f"[bench] graph store built and bootstrap inference done in {time.time() - t0:.1f}s")
    t0 = time.time()
    stream = ri.UpdateStream(cfg.n, cfg.vertex_capacity, src, dst, out_law, in_law, cfg.d0, cfg.mix, cfg.stream_seed,
                             weighted=cfg.weighted)
    del src, dst
    batches = []
    for _ in range(args.warmup + args.steps):
        ops, payload, n_upd = stream.next_batch(bs)
        ops_t = torch.from_numpy(ops.view(np.int32).copy()).cuda()
        pay_t = torch.from_numpy(payload).cuda() if len(payload) else None
        batches.append((ops_t, pay_t, len(ops), len(payload), n_upd))
    # a few more batches that stay on the host: the same call with operations and feature rows as host buffers
    host_batches = [] if args.no_host_inputs else [stream.next_batch(bs) for _ in range(min(args.steps, 10))]
    torch.cuda.synchronize()
    del stream
    log(f"[bench] {len(batches)} batches of {bs} updates staged in HBM in {time.time() - t0:.1f}s")

    rp.ripple_set_option(ctx, rp.OPT_SCATTER_MODE, args.scatter_mode)
    if args.sparse_frontier >= 0:
        rp.ripple_set_option(ctx, rp.OPT_SPARSE_FRONTIER, args.sparse_frontier)
    if args.sorted_messages >= 0:
        rp.ripple_set_option(ctx, rp.OPT_SORTED_MESSAGES, args.sorted_messages)
    if args.stream_transform >= 0:
        rp.ripple_set_option(ctx, rp.OPT_STREAM_TRANSFORM, args.stream_transform)
    rp.ripple_set_option(ctx, rp.OPT_BF16_MFMA, args.bf16_mfma)
    if args.pull_ratio:
        rp.ripple_set_option(ctx, rp.OPT_PULL_RATIO, args.pull_ratio)
    if args.calibrate_copy:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")        # 1 GiB read + 1 GiB written per copy
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    def run(b):
        ops_t, pay_t, n_ops, n_rows, _ = b
        return rp.ripple_apply_updates(ctx, ops_t.data_ptr(), pay_t.data_ptr() if pay_t is not None else None,
                                       n_ops=n_ops, n_feat_rows=n_rows)

    for b in batches[:args.warmup]:
        run(b)
    rp.ripple_set_option(ctx, rp.OPT_TIMING, 0 if args.no_kernel_timing else 1)
    rp.ripple_get_stats(ctx, reset=True)
    torch.cuda.synchronize()
    lat, n_updates, applied = [], 0, 0
    mono = np.zeros((3, len(model) + 1), dtype=np.int64)      # max / min hops: unchanged, incremental, recomputed
    t_begin = time.perf_counter()
    for b in batches[args.warmup:]:
        t1 = time.perf_counter()
        res = run(b)
        lat.append(time.perf_counter() - t1)
        n_updates += b[4]
        applied += res.n_applied
        for l in range(len(model) + 1):
            mono[:, l] += (res.mono_unchanged[l], res.mono_incremental[l], res.mono_recomputed[l])
    torch.cuda.synchronize()
    total = time.perf_counter() - t_begin
    st = rp.ripple_get_stats(ctx, reset=False)
    rp.ripple_set_option(ctx, rp.OPT_TIMING, 0)
    host_lat = []
    for ops, payload, _ in host_batches:                # not part of `value`: PCIe-inclusive latency of the same call
        t1 = time.perf_counter()
        rp.ripple_apply_updates(ctx, ops, payload)
        host_lat.append(time.perf_counter() - t1)

    L = len(model)
    layer_info = {l: rp.ripple_get_layer_info(ctx, l) + (rp.ripple_layer_packs_messages(ctx, l),) for l in range(1, L + 1)}
    work = algorithmic_work(st, model, cfg.widths, cfg.store, L, layer_info, n_edges=res.n_edges)
    phase_idx = {"frontier": 2, "scatter": 3, "transform": 5}
    mfma_peak = MFMA_PEAK_TFLOPS["bf16" if (cfg.store == "bf16" and args.bf16_mfma) else "f32"]
    kernels = {}
    for (ph, l), w in work.items():
        ms = st.ms[phase_idx[ph]][l] + (st.ms[6][l] if ph == "transform" else 0.0)   # 6: projection of the deltas
        n_launch = st.launches[phase_idx[ph]][l]
        if not n_launch or ms <= 0:
            continue
        ent = {"ms_per_launch": ms / n_launch, "launches": int(n_launch),
               "GBps": w["bytes"] / (ms * 1e-3) / 1e9, "hbm_frac": w["bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        if ph == "scatter":
            ent["per_message_GBps"] = w["msg_bytes"] / (ms * 1e-3) / 1e9
            ent["per_message_hbm_frac"] = ent["per_message_GBps"] / HBM_PEAK_GBS
            ent["message_lines_per_s"] = w["lines"] / (ms * 1e-3)       # 128-byte lines gathered for messages
        if ph == "transform":
            ent["TFLOPs"] = w["flops"] / (ms * 1e-3) / 1e12
            ent["mfma_frac"] = ent["TFLOPs"] / mfma_peak
        kernels[f"{ph}_l{l}"] = ent
    other = {name: st.ms[i][0] / max(st.batches, 1) for i, name in ((0, "ingest"), (1, "struct"), (7, "total"))}
    for l in range(1, L + 1):
        other[f"compact_l{l}"] = st.ms[4][l] / max(st.batches, 1)
        if st.ms[6][l] > 0:
            other[f"project_l{l}"] = st.ms[6][l] / max(st.batches, 1)
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_launch"] * kernels[k]["launches"]) if kernels else None
    roofline = None
    if dom:
        k = kernels[dom]
        ph, l = dom.split("_l")
        l = int(l)
        w = work[(ph, l)]
        # transform is priced against the matrix-core peak only where its arithmetic intensity
        # clears the ridge (peak flops / peak bytes); otherwise it is HBM-bound
        ridge = mfma_peak * 1e12 / (HBM_PEAK_GBS * 1e9)
        if ph == "transform" and w["flops"] / max(w["bytes"], 1) >= ridge:
            roofline = {"kernel": dom, "bound": "mfma", "achieved": k["TFLOPs"], "peak": mfma_peak,
                        "unit": "TFLOP/s", "frac": k["mfma_frac"], "traffic": None}
        else:
            roofline = {"kernel": dom, "bound": "hbm", "achieved": k["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": k["hbm_frac"], "traffic": None}
    measured = MEASURED_TRAFFIC_BYTES.get((cfg.name, bs), {})
    if roofline and dom in measured and args.scatter_mode == 0 and not args.deterministic and args.split_mfma <= 0:
        roofline["traffic"] = measured[dom]                 # bytes per launch; traffic / ms_per_launch is the HBM rate
        roofline["traffic_GBps"] = measured[dom] / (kernels[dom]["ms_per_launch"] * 1e-3) / 1e9
        roofline["traffic_source"] = TRAFFIC_SOURCE + " (rocprofv3 counters of an earlier run of this command, not of this run)"
    peaks = None
    if not args.no_peaks:
        peaks = rp.ripple_measure_peaks()
        if roofline:                                        # the same achieved figure against what this chip delivers
            if roofline["bound"] == "hbm":
                roofline["achievable"] = {"peak": peaks["hbm_copy_gbps"], "unit": "GB/s", "what": "streaming copy measured on this GPU",
                                          "frac": roofline["achieved"] / peaks["hbm_copy_gbps"]}
                if dom.startswith("scatter") and "message_lines_per_s" in kernels[dom]:
                    roofline["achievable"]["gather_lines_per_s"] = peaks["gather_glines"] * 1e9
                    roofline["achievable"]["gather_frac"] = kernels[dom]["message_lines_per_s"] / (peaks["gather_glines"] * 1e9)
            else:
                key = "mfma_bf16_tflops" if mfma_peak > 1000 else "mfma_f32_tflops"
                roofline["achievable"] = {"peak": peaks[key], "unit": "TFLOP/s", "what": "register-only matrix-core loop measured on this GPU",
                                          "frac": roofline["achieved"] / peaks[key]}
    lat_ms = np.array(lat) * 1e3
    result = {
        "metric": "graph updates/sec (and p50 batch latency), 3-layer GraphSAGE-mean on a 2.45M-vertex/124M-edge graph"
        if cfg.name == "dense_sage_mean" else f"graph updates/sec, {cfg.name}",
        "value": n_updates / total, "unit": "updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": total / max(args.steps, 1) * 1e3, "p50_ms": float(np.percentile(lat_ms, 50)),
        "p99_ms": float(np.percentile(lat_ms, 99)),
        **({"p50_ms_host_inputs": float(np.percentile(np.array(host_lat) * 1e3, 50)), "host_input_batches": len(host_lat)}
           if host_lat else {}),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if cfg.store == "f32" else "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: Chung-Lu gamma={cfg.gamma}, {cfg.n} vertices, {cfg.e} edges, "
                               f"widths {'->'.join(map(str, cfg.widths))}, {bs} updates/batch "
                               + ("(50% edge add, 30% edge delete, 20% feature update)" if not cfg.mix.get("vadd") else
                                  f"({cfg.mix['vadd']:.0%} vertex add, {cfg.mix['vdel']:.0%} vertex delete, rest 50/30/20 edge add/edge delete/feature update)"),
                   "batch_size": bs, "updates_applied": int(applied),
                   **({"aggregation": "deterministic"} if args.deterministic else {})},
        "per_batch": {"a_l": [st.rows[l] / max(st.batches, 1) for l in range(L + 1)],
                      "messages_l": [st.msgs[l] / max(st.batches, 1) for l in range(L + 1)],
                      "phase_ms": other,
                      # how the last timed batch moved each hop's messages: 1 pushed, 2 pulled, 3 one scan of all in-rows
                      # that also finds the hop's set, 4 from the list of the hop's messages sorted by destination
                      "hop_mode_last_batch": [int(res.hop_mode[l]) for l in range(1, L + 1)]},
        "aggregate_width": {f"l{l}": layer_info[l][0] for l in layer_info},
        **({"max_min_split_per_batch": {f"l{l}": dict(zip(("unchanged", "incremental", "recomputed"),
                                                          (mono[:, l] / max(args.steps, 1)).tolist()))
                                        for l in range(1, len(model) + 1)}} if mono.any() else {}),
        "kernels": kernels,
        "roofline": roofline,
        **({"measured_peaks": peaks} if peaks else {}),
    }
    rp.ripple_destroy(ctx)
    del batches
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        scale = args.cpu_scale or (16 if cfg.e > 10_000_000 else 1)
        t0 = time.time()
        result["cpu_baseline"] = cpu_baseline(cfg, bs, scale, full_size=args.cpu_baseline_full)
        log(f"[bench] CPU oracle sample took {time.time() - t0:.1f}s")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
