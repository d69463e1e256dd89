#!/usr/bin/env python3
"""Benchmark of the GQSA W4S50 G=16 decode GEMV path on one MI355X.

A step is one pass of the hot path over one LLaMA-7B-like decoder layer set at batch 1:
seven GEMVs (q/k/v/o 4096x4096, gate/up 11008x4096, down 4096x11008), W4, 50 % of the groups of
every row pruned, G = 16, issued as a decoder issues them: the calls that share their input in
one launch (q/k/v, gate/up), i.e. four dependent launches per layer.  Successive steps walk a
pool of distinct layers larger than 1 GB, so every call reads its weights from HBM, as real
decoding does (each layer's weights are read once per token).  Inputs are resident in HBM before
timing starts.

Prints ONE JSON line: value = achieved GB/s of the fused layer step over the algorithmic
compressed bytes (stored groups x 14 B + row pointers + x + y), with the roofline and
cpu_baseline objects, the pure-read ceiling of the same step, and compact rows for every other
named configuration (sparsity sweep, imbalanced stress shapes, small batches, 8-bit codes).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak
N_SIMD_UNITS = 1024      # 256 compute units x 4
CLOCK_HZ = 2.4e9         # peak engine clock
MIN_POOL = 1 << 30       # distinct matrices behind every "cold" figure: four times the 256 MB memory-side cache


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=240)
    p.add_argument("--warmup", type=int, default=24)
    p.add_argument("--pool-layers", type=int, default=12, help="distinct layer sets in HBM (12 = 1.07 GB)")
    p.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    p.add_argument("--separate", action="store_true", help="seven separate launches per layer instead of 4")
    p.add_argument("--skip-cpu", action="store_true", help="skip the cpu_baseline leg (for profiling runs)")
    p.add_argument("--skip-extras", action="store_true", help="only the headline: no other configuration, no baselines")
    p.add_argument("--cpu-seconds", type=float, default=12.0)
    p.add_argument("--more", action="store_true",
                   help="also the group-size sweep (G = 8 .. 128) and a vocabulary-sized matrix (about a minute more)")
    p.add_argument("--pmc-calibrate", action="store_true",
                   help="also run 8 plain copies of 256 MiB (known HBM traffic) to calibrate profiler counters")
    return p.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported "
              "(the path would shard by output rows: every GPU all of x and a slice of y)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import gqsa_inputs as gi
    import paper_2412_17560_amd as gq

    if not torch.cuda.is_available():
        print("bench.py: no HIP device", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    workers = min(16, os.cpu_count() or 8)

    # ------------------------------------------------------------------ pool of packed layers
    t_build = time.time()
    layers = []          # layers[l] = list of (handle, shape_index)
    info0 = []
    for l in range(args.pool_layers):
        mats = []
        for i, (name, N, K) in enumerate(gi.LLAMA7B_LAYER):
            W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(2, i) + 100000 * l, workers=workers)
            h = gq.gqsa_pack(W, 16, 4, 0.5)
            gq.gqsa_upload(h)
            mats.append((h, i))
            if l == 0:
                info0.append(gq.gqsa_info(h))
            del W
        layers.append(mats)
    bytes_per_call = [inf["algorithmic_bytes"] for inf in info0]
    bytes_per_step = int(sum(bytes_per_call))
    device_bytes_per_step = int(sum(inf["device_bytes"] for inf in info0))
    pool_bytes = device_bytes_per_step * args.pool_layers
    t_build = time.time() - t_build

    xs = {K: torch.from_numpy(gi.activations(1, K, seed=gi.config_seed(2, 0))).to(dev) for K in (4096, 11008)}
    ys = [torch.empty((1, N), dtype=torch.float16, device=dev) for (_, N, _) in gi.LLAMA7B_LAYER]

    launch_groups = [(0,), (1,), (2,), (3,), (4,), (5,), (6,)] if args.separate else [(0, 1, 2), (3,), (4, 5), (6,)]

    def enqueue_step(k):
        """One decoder layer: seven GEMVs.  Calls that share their input go out as one launch
        (q/k/v and gate/up), as a decoder would issue them: 4 launches per layer."""
        mats = layers[k % args.pool_layers]
        for idxs in launch_groups:
            K = gi.LLAMA7B_LAYER[idxs[0]][2]
            if len(idxs) == 1:
                gq.gqsa_gemv(mats[idxs[0]][0], xs[K], ys[idxs[0]])
            else:
                gq.gqsa_gemv_multi([mats[i][0] for i in idxs], xs[K], [ys[i] for i in idxs])

    stream = torch.cuda.Stream()
    calls_per_step = len(gi.LLAMA7B_LAYER)
    launches_per_step = len(launch_groups)

    def timed_region(fn):
        """fn enqueues the work on `stream`; returns elapsed ms measured with events on that stream."""
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            e0.record(stream)
            fn()
            e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def median(v):
        v = sorted(v)
        return v[len(v) // 2]

    def replay_ms(enqueue, n, warm, reps):
        """ms of n enqueued steps (after `warm` untimed ones): replays of a HIP graph holding the n
        steps -- every one of the `reps` timed replays is returned -- or one eager pass (--no-graph)."""
        with torch.cuda.stream(stream):
            for k in range(warm):
                enqueue(k)
        torch.cuda.synchronize()
        if args.no_graph:
            return [timed_region(lambda: [enqueue(warm + k) for k in range(n)])]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for k in range(n):
                enqueue(warm + k)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            g.replay()                      # untimed replay
        torch.cuda.synchronize()
        return [timed_region(lambda: g.replay()) for _ in range(reps)]

    if args.pmc_calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        src.random_(0, 255)
        dst = torch.empty_like(src)
        with torch.cuda.stream(stream):
            for _ in range(8):
                gq.gqsa_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------------------------ the headline
    with torch.cuda.stream(stream):
        for k in range(args.warmup):
            enqueue_step(k)
    torch.cuda.synchronize()
    eager_ms = timed_region(lambda: [enqueue_step(args.warmup + k) for k in range(args.steps)])
    mode = "eager" if args.no_graph else "hip_graph_replay"
    replays = replay_ms(enqueue_step, args.steps, 0, 7)
    total_ms = median(replays)              # median of the timed replays of exactly `steps` steps

    ms_per_step = total_ms / args.steps
    value = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    us_per_call = ms_per_step * 1e3 / calls_per_step

    out = {
        "metric": "achieved HBM GB/s over the GQSA W4S50 GEMV calls of a fused decoder-layer step (batch 1)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "llama7b_decode_layer_set_w4s50_g16_batch1",
            "calls_per_step": calls_per_step,
            "shapes_NxK": [[N, K] for (_, N, K) in gi.LLAMA7B_LAYER],
            "bits": 4, "group_size": 16, "sparsity": 0.5, "batch": 1,
            "algorithmic_bytes_per_step": bytes_per_step,
            "pool_layers": args.pool_layers,
            "pool_device_bytes": int(pool_bytes),
            "launch_mode": mode,
            "launches_per_step": launches_per_step,
            "step": "7 GEMVs of one layer as 4 dependent launches: q/k/v fused, o, gate/up fused, down",
            "timing": f"median of {len(replays)} replays of {args.steps} steps",
        },
        "us_per_call": round(us_per_call, 3),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "ms_per_step_replays_min_max": [round(min(replays) / args.steps, 6), round(max(replays) / args.steps, 6)],
        "eager_ms_per_step": round(eager_ms / args.steps, 6),
        "pool_build_s": round(t_build, 1),
    }
    # dominant kernel: gqsa_gemv_kernel<Fmt<4, 1, 0>, KGP, 1>; a launch covers one call, or the calls of a
    # layer that share x (q/k/v, gate/up).  Average launch duration is the event-timed region
    # divided by the launches in it (so it contains the gaps between dependent kernels); bytes are
    # the algorithmic bytes of the calls a launch covers.
    launches = args.steps * launches_per_step
    avg_launch_s = total_ms * 1e-3 / launches
    achieved = (bytes_per_step / launches_per_step) / avg_launch_s / 1e9
    # HBM bytes per launch as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, calibrated on gqsa_copy;
    # hbm_traffic.json beside this file records the run): valid only for the device images it was
    # measured on, so it is reported only while the images' size is still the one recorded there.
    traffic = None
    try:
        rec = json.load(open(os.path.join(ROOT, "hbm_traffic.json")))
        if rec["device_bytes_per_step"] == device_bytes_per_step and not args.separate:
            traffic = int(rec["hbm_bytes_per_step"] / launches_per_step)
    except (OSError, KeyError, ValueError):
        pass
    out["roofline"] = {
        "bound": "hbm",
        "kernel": "gqsa_gemv_kernel<Fmt<4, 1, 0>, KGP, 1>",
        "achieved": round(achieved, 2),
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "avg_launch_us": round(avg_launch_s * 1e6, 3),
        "algorithmic_bytes_per_launch": int(bytes_per_step / launches_per_step),
        "device_bytes_addressed_per_launch": int((device_bytes_per_step + sum((K + N) * 2 for (_, N, K) in gi.LLAMA7B_LAYER))
                                                 / launches_per_step),
        "traffic": traffic,
    }

    if args.skip_extras:
        finish(args, out, gi, xs, bytes_per_step, calls_per_step, workers)
        return

    def time_calls(fn_of_k, n=200, warm=20, reps=3, spread=None):
        """us per call of n back-to-back calls replayed from a HIP graph (eager if --no-graph):
        the median of `reps` replays (with a dict to fill in: also their 10th and 90th percentile)."""
        times = sorted(t * 1e3 / n for t in replay_ms(fn_of_k, n, warm, reps))
        if spread is not None:
            spread.update({"us_p10": round(times[len(times) // 10], 3), "us_p90": round(times[(9 * len(times)) // 10], 3)})
        return times[len(times) // 2]

    def rate(b, us):
        return {"us": round(us, 3), "GBps": round(b / us / 1e3, 1), "pct_peak": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2)}

    # ------------------------------------------------------------------ pure-read ceiling of the step
    # The same step with every GEMV launch replaced by a plain streaming read of as many bytes (the
    # launch's device images), same graph shape (dependent launches on one stream), walking a
    # buffer of 2 GiB: what launch latency, first-byte latency and HBM allow for these sizes.
    big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    big.random_(0, 255)
    sink = torch.zeros(gq.gqsa_stream_read_workgroups(), dtype=torch.int32, device=dev)
    launch_bytes = [sum(info0[i]["device_bytes"] for i in idxs) // 4096 * 4096 for idxs in launch_groups]
    step_span = sum(launch_bytes)
    steps_in_buffer = big.numel() // step_span

    def enqueue_read_step(k):
        off = (k % steps_in_buffer) * step_span
        for nb in launch_bytes:
            gq.gqsa_stream_read(big[off:off + nb], sink)
            off += nb

    n_read = min(args.steps, 240)
    read_ms = median(replay_ms(enqueue_read_step, n_read, 5, 5)) / n_read
    out["read_ceiling"] = {
        "what": "the step's launches replaced by plain streaming reads of the same device bytes, same graph shape, cold",
        "bytes_per_launch": [int(b) for b in launch_bytes],
        "read_ceiling_ms_per_step": round(read_ms, 6),
        "read_ceiling_GBps": round(step_span / read_ms / 1e6, 1),
        "frac_of_read_ceiling": round(read_ms / ms_per_step, 4),
    }
    us = time_calls(lambda k: gq.gqsa_stream_read(big, sink), n=20, warm=3)
    out["stream_read_GBps"] = round(big.numel() / us / 1e3, 1)
    # the same read kernel on slices as small as one packed matrix, walking the buffer (cold):
    # what a pure read of that many bytes costs, launch included
    small = []
    for idx in (0, 4):
        nbytes = info0[idx]["device_bytes"] // 4096 * 4096
        nslices = big.numel() // nbytes
        us = time_calls(lambda k, nbytes=nbytes, nslices=nslices: gq.gqsa_stream_read(
            big[(k % nslices) * nbytes:(k % nslices + 1) * nbytes], sink))
        small.append({"bytes": int(nbytes), "us_cold": round(us, 3), "GBps_cold": round(nbytes / us / 1e3, 1)})
    out["stream_read_matrix_sized"] = small
    out["empty_launch_us"] = round(time_calls(lambda k: gq.gqsa_launch_floor(256, 9216, sink)), 3)
    # our own dense fp16 GEMV on the same shapes (pool of distinct fp16 matrices > 1 GB), beside a
    # plain streaming read of as many bytes issued the same way (one launch per matrix, cold)
    dense = []
    for idx in (0, 4, 6):
        name, N, K = gi.LLAMA7B_LAYER[idx]
        nbytes = N * K * 2
        nslices = big.numel() // nbytes
        us_read = time_calls(lambda k, nbytes=nbytes, nslices=nslices: gq.gqsa_stream_read(
            big[(k % nslices) * nbytes:(k % nslices + 1) * nbytes], sink), n=100)
        n_mats = max(2, int(MIN_POOL // nbytes) + 1)
        Ws = [torch.randn((N, K), dtype=torch.float16, device=dev) * 0.02 for _ in range(n_mats)]
        yb = torch.empty((1, N), dtype=torch.float16, device=dev)
        us = time_calls(lambda k, Ws=Ws, K=K, yb=yb: gq.gqsa_dense_f16_gemv(Ws[k % len(Ws)], xs[K], yb), n=100)
        b = nbytes + (N + K) * 2
        dense.append({"shape": f"{N}x{K}", "us_cold": round(us, 3), "GBps_cold": round(b / us / 1e3, 1),
                      "stream_read_same_bytes_us": round(us_read, 3), "frac_of_stream_read_rate": round(us_read / us, 3)})
        del Ws
    out["dense_f16_gemv"] = dense

    # ------------------------------------------------------------------ single calls of the layer's shapes
    extra_handles = []

    def copies_from(e, N, K, G, bits, n, panels=False, keep_first=None):
        hs = [] if keep_first is None else [keep_first]
        while len(hs) < n:
            hs.append(gq.gqsa_import(e["rowIndex"], e["groups"], e["values"], e["scales"], e["zeros"], N, K, G, bits))
        for h in hs:
            if panels:
                gq.gqsa_build_panels(h)
            gq.gqsa_upload(h)
        return hs

    def more_copies(h, n):
        """n further device copies of a packed matrix (so that a pool of one shape exceeds
        every cache, the 256 MB memory-side one included)."""
        inf = gq.gqsa_info(h)
        cs = copies_from(gq.gqsa_export(h), inf["N"], inf["K"], inf["G"], inf["bits"], n)
        extra_handles.extend(cs)
        return cs

    def free_extras():
        for h in extra_handles:
            gq.gqsa_free(h)
        extra_handles.clear()

    per_shape = []
    for idx in (0, 4, 6):
        name, N, K = gi.LLAMA7B_LAYER[idx]
        hs = [layers[l][idx][0] for l in range(args.pool_layers)]
        if idx == 0:   # q,k,v,o are four distinct matrices of the same shape per layer
            hs = [layers[l][j][0] for l in range(args.pool_layers) for j in range(4)]
        each = gq.gqsa_info(hs[0])["device_bytes"]
        hs = hs + more_copies(hs[0], max(0, -(-MIN_POOL // each) - len(hs)))
        spread = {}
        us = time_calls(lambda k, hs=hs, K=K, idx=idx: gq.gqsa_gemv(hs[k % len(hs)], xs[K], ys[idx]), reps=10, spread=spread)
        us_warm = time_calls(lambda k, hs=hs, K=K, idx=idx: gq.gqsa_gemv(hs[0], xs[K], ys[idx]))
        b = bytes_per_call[idx]
        per_shape.append({"shape": f"{N}x{K}", "us_cold": round(us, 3), "us_cold_p10": spread.get("us_p10"),
                          "us_cold_p90": spread.get("us_p90"),
                          "GBps_cold": round(b / us / 1e3, 1),
                          "pct_peak_cold": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2),
                          "us_cache_warm": round(us_warm, 3),
                          "distinct_matrices": len(hs),
                          "mode": "200 back-to-back single calls, median of 10 replays, " + mode})
        free_extras()
    out["per_shape"] = per_shape
    out["single_call_pct_of_hbm_peak"] = {r["shape"]: r["pct_peak_cold"] for r in per_shape}

    # the launches that cover several calls sharing x, by themselves
    fused = []
    for label, idxs in (("q/k/v 3 x 4096x4096", (0, 1, 2)), ("gate/up 2 x 11008x4096", (4, 5))):
        sets = [[layers[l][j][0] for j in idxs] for l in range(args.pool_layers)]
        each = sum(gq.gqsa_info(h)["device_bytes"] for h in sets[0])
        for _ in range(max(0, -(-MIN_POOL // each) - len(sets))):
            sets.append([more_copies(h, 1)[0] for h in sets[0]])
        us = time_calls(lambda k, sets=sets, idxs=idxs: gq.gqsa_gemv_multi(
            sets[k % len(sets)], xs[4096], [ys[j] for j in idxs]))
        b = sum(bytes_per_call[j] for j in idxs)
        fused.append({"launch": label, "us_cold": round(us, 3), "GBps_cold": round(b / us / 1e3, 1),
                      "pct_peak_cold": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2),
                      "distinct_sets": len(sets)})
        free_extras()
    out["fused_launches"] = fused

    # ------------------------------------------------------------------ every other named configuration
    def packed_pool(W, bits, sparsity, G=16, keep=None, panels=False, min_bytes=MIN_POOL):
        """Distinct device copies of one packed matrix, enough of them to defeat the caches
        (panels: each with the second image for many activation rows)."""
        h0 = gq.gqsa_pack_rows(W, keep, G, bits) if keep is not None else gq.gqsa_pack(W, G, bits, sparsity)
        inf = gq.gqsa_info(h0)
        e = gq.gqsa_export(h0)
        each = inf["device_bytes"]
        if panels:
            gq.gqsa_build_panels(h0)
            each = gq.gqsa_info(h0)["panel_bytes"]
        n = max(2, min_bytes // each + 1)
        return copies_from(e, W.shape[0], W.shape[1], G, bits, n, panels=panels, keep_first=h0)

    def vector_for(K, B=1, seed=0):
        if B == 1 and K in xs:
            return xs[K]
        return torch.from_numpy(gi.activations(B, K, seed=seed)).to(dev)

    def time_variants(shapes, variants, seed_config, n=100, read_buf=None):
        """us per call over pools of distinct packed matrices; with read_buf also a plain streaming
        read of as many bytes as a matrix's device image, issued the same way (cold slices)."""
        rows = []
        for idx, (name, N, K) in shapes:
            W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(seed_config, idx), workers=workers)
            xk = vector_for(K)
            yk = torch.empty((1, N), dtype=torch.float16, device=dev)
            for variant in variants:
                bits, sparsity = variant[:2]
                G = variant[2] if len(variant) > 2 else 16
                hs = packed_pool(W, bits, sparsity, G)
                us = time_calls(lambda k, hs=hs, xk=xk, yk=yk: gq.gqsa_gemv(hs[k % len(hs)], xk, yk), n=n)
                inf = gq.gqsa_info(hs[0])
                row = {"shape": f"{N}x{K}", "bits": bits, "S": sparsity, "G": G}
                row.update(rate(inf["algorithmic_bytes"], us))
                row["partition"] = list(gq.gqsa_partition(hs[0]))
                if read_buf is not None:
                    nbytes = inf["device_bytes"] // 4096 * 4096
                    nslices = read_buf.numel() // nbytes
                    us_read = time_calls(lambda k, nbytes=nbytes, nslices=nslices: gq.gqsa_stream_read(
                        read_buf[(k % nslices) * nbytes:(k % nslices + 1) * nbytes], sink), n=n)
                    row["stream_read_same_bytes_us"] = round(us_read, 3)
                    row["us_over_stream_read"] = round(us / us_read, 3)
                rows.append(row)
                for h in hs:
                    gq.gqsa_free(h)
            del W
        return rows

    # dense 4-bit baseline (Eq. 1-3 with nothing pruned: the same kernel at S = 0) and the 8-bit
    # variant at S = 50 %, on the layer's shapes
    shapes7 = [(i, gi.LLAMA7B_LAYER[i]) for i in (0, 4, 6)]
    out["dense_w4_gemv"] = time_variants(shapes7, [(4, 0.0)], 2)
    shapes5 = [(i, s5) for i, s5 in enumerate(gi.SMALL_BATCH_SHAPES)]
    out["w8s50_gemv"] = time_variants(shapes7, [(8, 0.5)], 2, read_buf=big) + time_variants(shapes5[1:], [(8, 0.5)], 5, read_buf=big)
    del big

    # LLaMA-3-8B-like shapes over the sparsity sweep (the axes of the paper's kernel benchmark,
    # Sec. 4.4 / Fig. 6, which states that the GEMV gets faster as the sparsity rises)
    sweep = time_variants(list(enumerate(gi.LLAMA3_8B_SHAPES)), [(4, sp) for sp in gi.SPARSITY_SWEEP], 3)
    out["llama3_8b_sparsity_sweep"] = sweep
    mono = {}
    for row in sweep:
        mono.setdefault(row["shape"], []).append(row["us"])
    out["monotone_in_sparsity"] = {shape: all(b <= a for a, b in zip(t, t[1:])) for shape, t in mono.items()}

    # imbalanced sparsity stress: kept fraction per row ~ Beta(0.5, 0.5), 2 % of the rows empty,
    # 2 % full (rows of very different lengths, long carry chains)
    rows = []
    for idx, (name, N, K) in enumerate(gi.IMBALANCED_SHAPES):
        seed = gi.config_seed(4, idx)
        W = gi.dense_weight_chunked(N, K, seed=seed, workers=workers)
        keep = gi.imbalanced_keep_counts(N, K // 16, seed=seed)
        hs = packed_pool(W, 4, None, keep=keep)
        del W
        xk = torch.from_numpy(gi.activations(1, K, seed=seed)).to(dev)
        yk = torch.empty((1, N), dtype=torch.float16, device=dev)
        us = time_calls(lambda k, hs=hs, xk=xk, yk=yk: gq.gqsa_gemv(hs[k % len(hs)], xk, yk), n=60)
        inf = gq.gqsa_info(hs[0])
        row = {"shape": f"{N}x{K}", "nnz_groups": inf["nnz_groups"]}
        row.update(rate(inf["algorithmic_bytes"], us))
        rows.append(row)
        for h in hs:
            gq.gqsa_free(h)
    out["imbalanced_stress"] = rows

    # small batches, 4-bit and 8-bit codes, both shapes: the wavefront kernel (weights decoded once
    # for up to 8 rows per launch) and the matrix-core kernel on the second image
    # (gqsa_build_panels; gqsa_gemv takes it from 5 rows on).  GB/s over the bytes of the image
    # that the kernel reads plus x and y.
    rows = []
    for sidx, (name, N, K) in enumerate(gi.SMALL_BATCH_SHAPES):
        W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(5, sidx), workers=workers)
        for bits in (4, 8):
            hs = packed_pool(W, bits, 0.5)
            hp = packed_pool(W, bits, 0.5, panels=True)
            inf, infp = gq.gqsa_info(hs[0]), gq.gqsa_info(hp[0])
            for B in gi.BATCH_SWEEP:
                xb = torch.from_numpy(gi.activations(B, K, seed=gi.config_seed(5, sidx))).to(dev)
                yb = torch.empty((B, N), dtype=torch.float16, device=dev)
                us = time_calls(lambda k, hs=hs, xb=xb, yb=yb: gq.gqsa_gemv(hs[k % len(hs)], xb, yb), n=60)
                usp = time_calls(lambda k, hp=hp, xb=xb, yb=yb: gq.gqsa_gemv(hp[k % len(hp)], xb, yb, panels=True), n=60)
                bw = inf["algorithmic_bytes"] + (B - 1) * (K + N) * 2
                bp = infp["panel_bytes"] + B * (K + N) * 2
                flops = 2.0 * 16 * inf["nnz_groups"] * B
                mc = rate(bp, usp)
                # its rooflines: HBM over the panel image's bytes, and the matrix cores' share of the
                # launch -- one 16x16x16 product per (panel, 16-element chunk of K), 16 cycles of a
                # SIMD unit's matrix core each (what SQ_VALU_MFMA_BUSY_CYCLES counts, profiles/)
                products = ((N + 15) // 16) * (K // 16)
                mc["roofline"] = {"bound": "hbm", "achieved": mc["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                  "frac": round(mc["GBps"] / HBM_PEAK_GBPS, 4),
                                  "mfma_busy_frac": round(products * 16 / (N_SIMD_UNITS * usp * 1e-6 * CLOCK_HZ), 4)}
                rows.append({"shape": f"{N}x{K}", "bits": bits, "batch": B,
                             "wavefront_kernel": rate(bw, us), "matrix_core_kernel": mc,
                             "matrix_core_TFLOPs_dense_equivalent": round(2.0 * N * K * B / usp / 1e6, 1),
                             "TFLOPs_stored_weights": round(flops / min(us, usp) / 1e6, 2),
                             "gqsa_gemv_uses": "matrix_core_kernel" if B >= 5 else "wavefront_kernel"})
            for h in hs + hp:
                gq.gqsa_free(h)
        del W
    out["small_batch"] = rows
    out["small_batch_note"] = ("roofline of the matrix-core kernel: bound = hbm over the panel image's bytes; mfma_busy_frac = "
                               "products x 16 cycles / (1024 SIMD units x launch time x 2.4 GHz), the count that "
                               "SQ_VALU_MFMA_BUSY_CYCLES gives for the same launches in profiles/")

    # q/k/v at 8 and 16 rows: three matrices on the same activations in one launch of the
    # matrix-core kernel (a workgroup's panels come from all three and share the activations it
    # loads) against three launches
    Wb = gi.dense_weight_chunked(4096, 4096, seed=gi.config_seed(5, 0), workers=workers)
    hp = packed_pool(Wb, 4, 0.5, panels=True)
    del Wb
    qkv = []
    trios = [hp[i:i + 3] for i in range(0, len(hp) - 2, 3)]
    for B in (8, 16):
        xb = torch.from_numpy(gi.activations(B, 4096, seed=gi.config_seed(5, 0))).to(dev)
        ybs = [torch.empty((B, 4096), dtype=torch.float16, device=dev) for _ in range(3)]
        one = time_calls(lambda k, xb=xb, ybs=ybs: gq.gqsa_gemv_multi(trios[k % len(trios)], xb, ybs), n=48)

        def three(k, xb=xb, ybs=ybs):
            for h, yb in zip(trios[k % len(trios)], ybs):
                gq.gqsa_gemv(h, xb, yb, panels=True)
        qkv.append({"batch": B, "us_one_launch": round(one, 3), "us_three_launches": round(time_calls(three, n=48), 3),
                    "distinct_sets": len(trios)})
    out["small_batch_qkv_3x4096x4096_panels"] = qkv
    for h in hp:
        gq.gqsa_free(h)

    if args.more:   # group sizes on two shapes; a matrix large enough that launch and first-byte latency no longer count
        out["group_size_sweep"] = time_variants(shapes7[:2], [(4, sp, G) for G in (8, 16, 32, 64, 128) for sp in (0.0, 0.5)], 2)
        out["vocabulary_projection"] = time_variants([(7, ("lm_head", 128256, 4096))], [(4, 0.5)], 3)

    # the offline step (host): prune + quantise + build the device image, 4096x4096
    Wp = gi.dense_weight_chunked(4096, 4096, seed=gi.config_seed(2, 0), workers=workers)
    dp = np.exp(np.random.default_rng(1).standard_normal(4096)).astype(np.float32)
    t0 = time.time(); gq.gqsa_free(gq.gqsa_pack(Wp, 16, 4, 0.5)); t_mag = time.time() - t0
    t0 = time.time(); gq.gqsa_free(gq.gqsa_pack_hessian(Wp, dp, 16, 4, 0.5)); t_hes = time.time() - t0
    out["pack_host_4096x4096"] = {"magnitude_s": round(t_mag, 4), "hessian_metric_s": round(t_hes, 4),
                                  "Mweights_per_s": round(4096 * 4096 / t_mag / 1e6, 1),
                                  "threads": min(16, os.cpu_count() or 1)}
    # the same step on the GPU (gqsa_pack_device: W already in device memory; the time includes
    # the copy of the canonical arrays and the image back to the handle's host side, and the
    # allocation of the handle's device memory)
    Wd = torch.from_numpy(Wp).to(dev)
    dd = torch.from_numpy(dp).to(dev)
    gq.gqsa_free(gq.gqsa_pack_device(Wd, 16, 4, 0.5))        # (first use: module load)
    torch.cuda.synchronize()
    ts = []
    for _ in range(5):
        t0 = time.time(); hd = gq.gqsa_pack_device(Wd, 16, 4, 0.5); ts.append(time.time() - t0); gq.gqsa_free(hd)
    t0 = time.time(); gq.gqsa_free(gq.gqsa_pack_device(Wd, 16, 4, 0.5, hinv_diag=dd)); t_dh = time.time() - t0
    out["pack_device_4096x4096"] = {"magnitude_s": round(median(ts), 4), "hessian_metric_s": round(t_dh, 4),
                                    "Mweights_per_s": round(4096 * 4096 / median(ts) / 1e6, 1),
                                    "speedup_over_host": round(t_mag / median(ts), 2)}
    del Wp, Wd, dd

    finish(args, out, gi, xs, bytes_per_step, calls_per_step, workers)


def finish(args, out, gi, xs, bytes_per_step, calls_per_step, workers):
    """The CPU oracle leg and the paper's own figures, then the one JSON line."""
    if not args.skip_cpu:
        import oracle
        canon = []
        for i, (name, N, K) in enumerate(gi.LLAMA7B_LAYER):
            W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(2, i), workers=workers)
            canon.append(oracle.pack(W, 16, 4, sparsity=0.5))
            del W
        xh = {K: xs[K].cpu().numpy() for K in xs}
        threads = oracle.max_threads()
        for c in canon:                                  # one untimed pass
            oracle.gemv(c, xh[c.K], threads=threads)
        reps = 0
        t0 = time.time()
        while time.time() - t0 < args.cpu_seconds:
            for c in canon:
                oracle.gemv(c, xh[c.K], threads=threads)
            reps += 1
        dt = time.time() - t0
        t0 = time.time()
        oracle.pack(gi.dense_weight_chunked(4096, 4096, seed=gi.config_seed(2, 0), workers=workers), 16, 4, sparsity=0.5)
        t_opack = time.time() - t0
        per_shape_cpu = []
        for c in (canon[0], canon[4], canon[6]):         # one call per shape: 1 thread and all of them
            def median_ms(threads, reps):
                ts = []
                for _ in range(reps):
                    t1 = time.time()
                    oracle.gemv(c, xh[c.K], threads=threads)
                    ts.append((time.time() - t1) * 1e3)
                return round(sorted(ts)[len(ts) // 2], 3)
            per_shape_cpu.append({"shape": f"{c.N}x{c.K}", "ms_1_thread": median_ms(1, 3),
                                  f"ms_{threads}_threads": median_ms(threads, 5)})
        out["cpu_baseline"] = {
            "value": round(bytes_per_step * reps / dt / 1e9, 3),
            "unit": "GB/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{reps} passes over one layer set (7 GEMVs, same shapes and sparsity) in {dt:.1f} s; "
                      f"{dt / reps * 1e3 / calls_per_step:.2f} ms per call",
            "per_shape": per_shape_cpu,
            "pack_4096x4096_s_1_thread": round(t_opack, 3),
        }

    # What the paper itself reports (Sec. 4.4, Fig. 6, Tab. 4, App. H, I, M): other hardware, whole
    # models with trained weights -- context beside the numbers above, not a baseline for this metric.
    out["paper_reported"] = {
        "note": "other hardware and whole-model figures; no absolute GEMV kernel time is given in the paper",
        "gemv_1x4096x4096_w4s50_vs_2to4_sparse_kernel": {"speedup": 3.0, "hardware": "RTX 4080"},
        "task_centric_vs_data_centric_one_operator": {"speedup": [1.3, 1.5], "hardware": "not stated"},
        "llama7b_latency_ms_128_output_tokens": {"fp16": 1490.5, "w4a16": 642.24, "w4_2to4": 513.79,
                                                "w4a16_g16_sp0.5": 377.98, "hardware": "A800-40GB"},
        "llama7b_throughput_tokens_per_s": {"fp16": 92.69, "w4": 202.81, "w4s50": 343.43,
                                            "hardware": "A100-80GB"},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
