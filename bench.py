#!/usr/bin/env python3
"""Benchmark of the GQSA W4S50 G=16 decode GEMV path on one MI355X.

A step is one pass of the hot path over one LLaMA-7B-like decoder layer set at batch 1:
seven gqsa_gemv calls (q/k/v/o 4096x4096, gate/up 11008x4096, down 4096x11008), W4, 50 %
of the groups of every row pruned, G = 16.  Successive steps walk a pool of distinct layers
larger than 1 GB, so every call reads its weights from HBM, as real decoding does (each
layer's weights are read once per token).  Inputs are resident in HBM before timing starts.

Prints ONE JSON line: value = achieved GB/s over the algorithmic compressed bytes
(stored groups x 14 B + row pointers + x + y), with the roofline and cpu_baseline objects.
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


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=240)
    p.add_argument("--warmup", type=int, default=24)
    p.add_argument("--pool-layers", type=int, default=12, help="distinct layer sets in HBM (12 = 1.07 GB)")
    p.add_argument("--no-graph", action="store_true", help="time eager launches instead of a HIP graph replay")
    p.add_argument("--separate", action="store_true", help="seven separate launches per layer instead of 4")
    p.add_argument("--skip-cpu", action="store_true", help="skip the cpu_baseline leg (for profiling runs)")
    p.add_argument("--skip-extras", action="store_true", help="skip per-shape / dense / stream-read legs")
    p.add_argument("--cpu-seconds", type=float, default=12.0)
    p.add_argument("--sweep", action="store_true",
                   help="also time the Llama-3-8B-like shapes at S = 0, 30, 50, 70 %%, group sizes 16..128, the "
                        "imbalanced stress shapes and small batches on 14336x4096 (about three minutes more)")
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
    pool_bytes = sum(inf["device_bytes"] for inf in info0) * args.pool_layers
    t_build = time.time() - t_build

    xs = {K: torch.from_numpy(gi.activations(1, K, seed=gi.config_seed(2, 0))).to(dev) for K in (4096, 11008)}
    ys = [torch.empty((1, N), dtype=torch.float16, device=dev) for (_, N, _) in gi.LLAMA7B_LAYER]

    def enqueue_step(k):
        """One decoder layer: seven GEMVs.  Calls that share their input go out as one launch
        (q/k/v and gate/up), as a decoder would issue them: 4 launches per layer."""
        mats = layers[k % args.pool_layers]
        if args.separate:
            for h, i in mats:
                gq.gqsa_gemv(h, xs[gi.LLAMA7B_LAYER[i][2]], ys[i])
            return
        gq.gqsa_gemv_multi([mats[0][0], mats[1][0], mats[2][0]], xs[4096], ys[0:3])
        gq.gqsa_gemv(mats[3][0], xs[4096], ys[3])
        gq.gqsa_gemv_multi([mats[4][0], mats[5][0]], xs[4096], ys[4:6])
        gq.gqsa_gemv(mats[6][0], xs[11008], ys[6])

    stream = torch.cuda.Stream()
    calls_per_step = len(gi.LLAMA7B_LAYER)

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

    if args.pmc_calibrate:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        src.random_(0, 255)
        dst = torch.empty_like(src)
        with torch.cuda.stream(stream):
            for _ in range(8):
                gq.gqsa_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    with torch.cuda.stream(stream):
        for k in range(args.warmup):
            enqueue_step(k)
    torch.cuda.synchronize()

    eager_ms = timed_region(lambda: [enqueue_step(args.warmup + k) for k in range(args.steps)])
    mode = "eager"
    total_ms = eager_ms
    graph_ms = None
    if not args.no_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for k in range(args.steps):
                enqueue_step(args.warmup + k)
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            g.replay()                      # untimed replay
        torch.cuda.synchronize()
        graph_ms = timed_region(lambda: g.replay())
        total_ms = graph_ms
        mode = "hip_graph_replay"

    ms_per_step = total_ms / args.steps
    value = bytes_per_step / (ms_per_step * 1e-3) / 1e9
    us_per_call = ms_per_step * 1e3 / calls_per_step

    out = {
        "metric": "achieved HBM GB/s per GQSA W4S50 GEMV call (batch 1)",
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
            "launches_per_step": 7 if args.separate else 4,
        },
        "us_per_call": round(us_per_call, 3),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "eager_ms_per_step": round(eager_ms / args.steps, 6),
        "pool_build_s": round(t_build, 1),
    }
    # dominant kernel: gqsa_gemv_kernel<Fmt<4, 1>, KGP, 1>; a launch covers one call, or the calls of a
    # layer that share x (q/k/v, gate/up).  Average launch duration is the event-timed region
    # divided by the launches in it (so it contains the gaps between dependent kernels); bytes are
    # the algorithmic bytes of the calls a launch covers.
    launches_per_step = 7 if args.separate else 4
    launches = args.steps * launches_per_step
    avg_launch_s = total_ms * 1e-3 / launches
    achieved = (bytes_per_step / launches_per_step) / avg_launch_s / 1e9
    out["roofline"] = {
        "bound": "hbm",
        "kernel": "gqsa_gemv_kernel<Fmt<4, 1>, KGP, 1>",
        "achieved": round(achieved, 2),
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "avg_launch_us": round(avg_launch_s * 1e6, 3),
        "algorithmic_bytes_per_launch": int(bytes_per_step / launches_per_step),
        # HBM bytes per launch from rocprofv3 FETCH_SIZE + WRITE_SIZE (calibrated on gqsa_copy), mean
        # over the launches of a step; see profiles/*hbm_traffic.md for the runs (the figure for
        # seven separate launches comes from the same counters, one matrix per launch)
        "traffic": None if args.separate else 22670080,
    }

    # ------------------------------------------------------------------ extras: per shape, baselines
    if not args.skip_extras:
        def time_calls(fn_of_k, n=200, warm=20, reps=3, spread=None):
            """us per call of n back-to-back calls replayed from a HIP graph (eager if --no-graph):
            the fastest of `reps` replays, or -- with a dict to fill in -- their median."""
            with torch.cuda.stream(stream):
                for k in range(warm):
                    fn_of_k(k)
            torch.cuda.synchronize()
            if args.no_graph:
                return timed_region(lambda: [fn_of_k(warm + k) for k in range(n)]) * 1e3 / n
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=stream):
                for k in range(n):
                    fn_of_k(warm + k)
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                gr.replay()
            torch.cuda.synchronize()
            times = sorted(timed_region(lambda: gr.replay()) * 1e3 / n for _ in range(reps))
            if spread is not None:       # median, 10th and 90th percentile over the replays
                spread.update({"us_median": round(times[len(times) // 2], 3),
                               "us_p10": round(times[len(times) // 10], 3),
                               "us_p90": round(times[(9 * len(times)) // 10], 3)})
            return times[0] if spread is None else times[len(times) // 2]

        extra_handles = []

        def more_copies(h, n):
            """n further device copies of a packed matrix (so that a pool of one shape exceeds
            every cache, the 256 MB memory-side one included)."""
            e = gq.gqsa_export(h)
            inf = gq.gqsa_info(h)
            cs = []
            for _ in range(n):
                c = gq.gqsa_import(e["rowIndex"], e["groups"], e["values"], e["scales"], e["zeros"],
                                   inf["N"], inf["K"], inf["G"], inf["bits"])
                gq.gqsa_upload(c)
                cs.append(c)
            extra_handles.extend(cs)
            return cs

        min_pool = 1 << 30
        per_shape = []
        for idx in (0, 4, 6):
            name, N, K = gi.LLAMA7B_LAYER[idx]
            hs = [layers[l][idx][0] for l in range(args.pool_layers)]
            if idx == 0:   # q,k,v,o are four distinct matrices of the same shape per layer
                hs = [layers[l][j][0] for l in range(args.pool_layers) for j in range(4)]
            each = gq.gqsa_info(hs[0])["device_bytes"]
            hs = hs + more_copies(hs[0], max(0, -(-min_pool // each) - len(hs)))
            spread = {}
            us = time_calls(lambda k, hs=hs, K=K, idx=idx: gq.gqsa_gemv(hs[k % len(hs)], xs[K], ys[idx]),
                            reps=10, spread=spread)
            us_warm = time_calls(lambda k, hs=hs, K=K, idx=idx: gq.gqsa_gemv(hs[0], xs[K], ys[idx]))
            b = bytes_per_call[idx]
            per_shape.append({"shape": f"{N}x{K}", "us_cold": round(us, 3), "us_cold_p10": spread.get("us_p10"),
                              "us_cold_p90": spread.get("us_p90"),
                              "GBps_cold": round(b / us / 1e3, 1),
                              "pct_peak_cold": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2),
                              "us_cache_warm": round(us_warm, 3),
                              "distinct_matrices": len(hs),
                              "mode": "200 back-to-back calls, median of 10 replays, " + mode})
            for h in extra_handles:
                gq.gqsa_free(h)
            extra_handles.clear()
        out["per_shape"] = per_shape

        # the launches that cover several calls sharing x, by themselves
        fused = []
        for label, idxs in (("q/k/v 3 x 4096x4096", (0, 1, 2)), ("gate/up 2 x 11008x4096", (4, 5))):
            sets = [[layers[l][j][0] for j in idxs] for l in range(args.pool_layers)]
            each = sum(gq.gqsa_info(h)["device_bytes"] for h in sets[0])
            for _ in range(max(0, -(-min_pool // each) - len(sets))):
                sets.append([more_copies(h, 1)[0] for h in sets[0]])
            us = time_calls(lambda k, sets=sets, idxs=idxs: gq.gqsa_gemv_multi(
                sets[k % len(sets)], xs[4096], [ys[j] for j in idxs]))
            b = sum(bytes_per_call[j] for j in idxs)
            fused.append({"launch": label, "us_cold": round(us, 3), "GBps_cold": round(b / us / 1e3, 1),
                          "pct_peak_cold": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2),
                          "distinct_sets": len(sets)})
            for h in extra_handles:
                gq.gqsa_free(h)
            extra_handles.clear()
        out["fused_launches"] = fused

        def copies_of(W, bits, sparsity, G=16, min_bytes=1 << 30, panels=False):
            """Distinct device copies of one packed matrix, enough of them to defeat the caches
            (panels: each with the second image for many activation rows)."""
            h0 = gq.gqsa_pack(W, G, bits, sparsity)
            e = gq.gqsa_export(h0)
            n = max(2, min_bytes // gq.gqsa_info(h0)["device_bytes"] + 1)
            hs = [h0]
            for _ in range(n - 1):
                hs.append(gq.gqsa_import(e["rowIndex"], e["groups"], e["values"], e["scales"], e["zeros"],
                                         W.shape[0], W.shape[1], G, bits))
            for h in hs:
                if panels:
                    gq.gqsa_build_panels(h)
                gq.gqsa_upload(h)
            return hs

        def time_variants(shapes, variants, seed_config):
            rows = []
            for idx, (name, N, K) in shapes:
                W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(seed_config, idx), workers=workers)
                xk = xs[K] if K in xs else torch.from_numpy(gi.activations(1, K, seed=0)).to(dev)
                yk = torch.empty((1, N), dtype=torch.float16, device=dev)
                for variant in variants:
                    bits, sparsity = variant[:2]
                    G = variant[2] if len(variant) > 2 else 16
                    hs = copies_of(W, bits, sparsity, G)
                    us = time_calls(lambda k, hs=hs, xk=xk, yk=yk: gq.gqsa_gemv(hs[k % len(hs)], xk, yk), n=100)
                    b = gq.gqsa_info(hs[0])["algorithmic_bytes"]
                    rows.append({"shape": f"{N}x{K}", "bits": bits, "sparsity": sparsity, "G": G, "us_cold": round(us, 3),
                                 "GBps_cold": round(b / us / 1e3, 1),
                                 "pct_peak_cold": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2)})
                    for h in hs:
                        gq.gqsa_free(h)
                del W
            return rows

        # dense 4-bit baseline (Eq. 1-3 with nothing pruned: the same kernel at S = 0) and the
        # 8-bit variant at S = 50 %, on the layer's shapes
        shapes7 = [(i, gi.LLAMA7B_LAYER[i]) for i in (0, 4, 6)]
        out["dense_w4_gemv"] = time_variants(shapes7, [(4, 0.0)], 2)
        out["w8s50_gemv"] = time_variants(shapes7[:1], [(8, 0.5)], 2)
        if args.sweep:   # Llama-3-8B-like shapes over the sparsity sweep; group sizes on 4096x4096
            out["llama3_8b_sweep"] = time_variants(list(enumerate(gi.LLAMA3_8B_SHAPES)),
                                                   [(4, sp) for sp in gi.SPARSITY_SWEEP], 3)
            out["group_size_sweep"] = time_variants(shapes7[:1] + shapes7[1:2],
                                                    [(4, sp, G) for G in (8, 16, 32, 64, 128) for sp in (0.0, 0.5)], 2)
            # a matrix large enough that launch and first-byte latency no longer count: the output
            # projection of a LLaMA-3-8B-like model (vocabulary 128 256), 231 MB at W4S50
            out["vocabulary_projection"] = time_variants([(7, ("lm_head", 128256, 4096))], [(4, 0.5)], 3)

        if args.sweep:
            # imbalanced sparsity stress: kept fraction per row ~ Beta(0.5, 0.5), 2 % of the rows
            # empty, 2 % full (rows of very different lengths, long carry chains)
            rows = []
            for idx, (name, N, K) in enumerate(gi.IMBALANCED_SHAPES):
                seed = gi.config_seed(4, idx)
                W = gi.dense_weight_chunked(N, K, seed=seed, workers=workers)
                keep = gi.imbalanced_keep_counts(N, K // 16, seed=seed)
                h0 = gq.gqsa_pack_rows(W, keep, 16, 4)
                del W
                e = gq.gqsa_export(h0)
                n = max(2, (1 << 30) // gq.gqsa_info(h0)["device_bytes"] + 1)
                hs = [h0] + [gq.gqsa_import(e["rowIndex"], e["groups"], e["values"], e["scales"], e["zeros"], N, K, 16, 4)
                             for _ in range(n - 1)]
                for h in hs:
                    gq.gqsa_upload(h)
                xk = torch.from_numpy(gi.activations(1, K, seed=seed)).to(dev)
                yk = torch.empty((1, N), dtype=torch.float16, device=dev)
                us = time_calls(lambda k, hs=hs, xk=xk, yk=yk: gq.gqsa_gemv(hs[k % len(hs)], xk, yk), n=60)
                b = gq.gqsa_info(h0)["algorithmic_bytes"]
                rows.append({"shape": f"{N}x{K}", "nnz_groups": gq.gqsa_info(h0)["nnz_groups"], "us_cold": round(us, 3),
                             "GBps_cold": round(b / us / 1e3, 1),
                             "pct_peak_cold": round(100 * b / us / 1e3 / HBM_PEAK_GBPS, 2)})
                for h in hs:
                    gq.gqsa_free(h)
            out["imbalanced_stress"] = rows
            # small batches on the larger shape, 4-bit and 8-bit codes
            rows = []
            name, N, K = gi.SMALL_BATCH_SHAPES[1]
            W = gi.dense_weight_chunked(N, K, seed=gi.config_seed(5, 1), workers=workers)
            for bits in (4, 8):
                hs = copies_of(W, bits, 0.5)
                for B in gi.BATCH_SWEEP:
                    xb = torch.from_numpy(gi.activations(B, K, seed=gi.config_seed(5, 1))).to(dev)
                    yb = torch.empty((B, N), dtype=torch.float16, device=dev)
                    us = time_calls(lambda k, hs=hs, xb=xb, yb=yb: gq.gqsa_gemv(hs[k % len(hs)], xb, yb), n=60)
                    rows.append({"shape": f"{N}x{K}", "bits": bits, "batch": B, "us_cold": round(us, 3),
                                 "us_per_row": round(us / B, 3)})
                for h in hs:
                    gq.gqsa_free(h)
                # the same with the second image (gqsa_build_panels): 16 output rows x 16 activation
                # rows x one group-column per matrix-core product; gqsa_gemv takes it from 5 rows on
                hs = copies_of(W, bits, 0.5, panels=True)
                for B in (8, 16):
                    xb = torch.from_numpy(gi.activations(B, K, seed=gi.config_seed(5, 1))).to(dev)
                    yb = torch.empty((B, N), dtype=torch.float16, device=dev)
                    us = time_calls(lambda k, hs=hs, xb=xb, yb=yb: gq.gqsa_gemv(hs[k % len(hs)], xb, yb, panels=True), n=60)
                    for row in rows:
                        if row["bits"] == bits and row["batch"] == B:
                            row["us_cold_panels"] = round(us, 3)
                for h in hs:
                    gq.gqsa_free(h)
            del W
            out["small_batch_14336x4096"] = rows

        # the offline step (host): prune + quantise + build the device image, 4096x4096
        Wp = gi.dense_weight_chunked(4096, 4096, seed=gi.config_seed(2, 0), workers=workers)
        dp = np.exp(np.random.default_rng(1).standard_normal(4096)).astype(np.float32)
        t0 = time.time(); gq.gqsa_free(gq.gqsa_pack(Wp, 16, 4, 0.5)); t_mag = time.time() - t0
        t0 = time.time(); gq.gqsa_free(gq.gqsa_pack_hessian(Wp, dp, 16, 4, 0.5)); t_hes = time.time() - t0
        out["pack_host_4096x4096"] = {"magnitude_s": round(t_mag, 3), "hessian_metric_s": round(t_hes, 3),
                                      "Mweights_per_s": round(4096 * 4096 / t_mag / 1e6, 1),
                                      "threads": min(16, os.cpu_count() or 1)}
        del Wp

        # small batches on the 4096x4096 shape (weights decoded once for up to 8 rows per launch)
        hs = [layers[l][j][0] for l in range(args.pool_layers) for j in range(4)]
        small_batch = []
        for B in (1, 2, 4, 8, 16):
            xb = torch.from_numpy(gi.activations(B, 4096, seed=gi.config_seed(5, 0))).to(dev)
            yb = torch.empty((B, 4096), dtype=torch.float16, device=dev)
            us = time_calls(lambda k, xb=xb, yb=yb: gq.gqsa_gemv(hs[k % len(hs)], xb, yb), n=96)
            small_batch.append({"batch": B, "us_cold": round(us, 3), "us_per_row": round(us / B, 3)})
        # the same from the second image (matrix cores); gqsa_gemv takes it from 5 rows on
        Wb = gi.dense_weight_chunked(4096, 4096, seed=gi.config_seed(5, 0), workers=workers)
        hp = copies_of(Wb, 4, 0.5, panels=True)
        del Wb
        for row in small_batch:
            if row["batch"] in (8, 16):
                B = row["batch"]
                xb = torch.from_numpy(gi.activations(B, 4096, seed=gi.config_seed(5, 0))).to(dev)
                yb = torch.empty((B, 4096), dtype=torch.float16, device=dev)
                us = time_calls(lambda k, xb=xb, yb=yb: gq.gqsa_gemv(hp[k % len(hp)], xb, yb, panels=True), n=96)
                row["us_cold_panels"] = round(us, 3)
        # q/k/v at 8 and 16 rows: three matrices on the same activations in one launch of the
        # matrix-core kernel (a workgroup's panels come from all three and share the activations
        # it loads) against three launches
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
        out["small_batch_4096x4096"] = small_batch

        # achievable read ceiling: plain streaming kernel over 2 GiB
        big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        big.random_(0, 255)
        sink = torch.zeros(gq.gqsa_stream_read_workgroups(), dtype=torch.int32, device=dev)
        us = time_calls(lambda k: gq.gqsa_stream_read(big, sink), n=20, warm=3)
        out["stream_read_GBps"] = round(big.numel() / us / 1e3, 1)
        # the same read kernel on slices as small as one packed matrix, walking the 2 GiB buffer
        # (cold): what a pure read of that many bytes costs, launch included
        small = []
        for idx in (0, 4):
            nbytes = info0[idx]["device_bytes"] // 4096 * 4096
            nslices = big.numel() // nbytes
            us = time_calls(lambda k, nbytes=nbytes, nslices=nslices: gq.gqsa_stream_read(
                big[(k % nslices) * nbytes:(k % nslices + 1) * nbytes], sink))
            small.append({"bytes": int(nbytes), "us_cold": round(us, 3), "GBps_cold": round(nbytes / us / 1e3, 1)})
        out["stream_read_matrix_sized"] = small
        us = time_calls(lambda k: gq.gqsa_launch_floor(256, 9216, sink))
        out["empty_launch_us"] = round(us, 3)
        del big

        # our own dense fp16 GEMV on the same shapes (pool of distinct fp16 matrices > 1 GB)
        dense = []
        for idx in (0, 4, 6):
            name, N, K = gi.LLAMA7B_LAYER[idx]
            n_mats = max(2, int((1 << 30) // (N * K * 2)) + 1)
            Ws = [torch.randn((N, K), dtype=torch.float16, device=dev) * 0.02 for _ in range(n_mats)]
            yb = torch.empty((1, N), dtype=torch.float16, device=dev)
            us = time_calls(lambda k, Ws=Ws, K=K, yb=yb: gq.gqsa_dense_f16_gemv(Ws[k % len(Ws)], xs[K], yb))
            b = N * K * 2 + (N + K) * 2
            dense.append({"shape": f"{N}x{K}", "us_cold": round(us, 3), "GBps_cold": round(b / us / 1e3, 1)})
            del Ws
        out["dense_f16_gemv"] = dense

    # ------------------------------------------------------------------ CPU oracle baseline
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
