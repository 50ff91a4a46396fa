#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: PSH bucketize -> Bucket-Swin attention passes -> unpermute.

One "step" is one pass of the whole path over one batch of seeded synthetic points: one
f3d_psh_bucketize, one f3d_bucket_swin_attn per pass of the workload, and the unpermute, which the last
pass does in its own store (out_perm); --separate-unpermute runs it as f3d_unpermute instead. Either way the
step ends with the result in the input order of the points. Inputs are resident in HBM before the timed region. Prints ONE JSON line:
  value     = points / second over the whole step (whole job, one GPU)
  roofline  = the attention kernel (dominant): algorithmic FLOP (sum over scopes of 4*n_g^2*C) divided by
              its mean launch duration from HIP events on the launch stream, against 2.5 PFLOP/s bf16 MFMA
  cpu_baseline = the CPU oracle timed on this machine's host cores on a bounded sample of the same workload
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E

# HBM bytes per attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same command, keyed by
# workload; the figures and the commands are in profiles/k_attn_<workload>.md. A counter run cannot be made from
# inside the timed run, so the line carries the stored figure and says where it comes from (None = not profiled).
MEASURED_TRAFFIC_BYTES = {"indoor": 106.2e6, "lidar8": 1874.0e6}


def scope_sizes(offsets: np.ndarray, sbs: np.ndarray, m: int, mode: str, shift: int, stride: int) -> np.ndarray:
    """Rows of every attention scope (host-side bookkeeping for the FLOP count only)."""
    sizes = []
    for b in range(len(sbs) - 1):
        K = int(sbs[b + 1] - sbs[b])
        if K <= 0:
            continue
        rows = np.diff(offsets[sbs[b]:sbs[b + 1] + 1]).astype(np.int64)
        j = np.arange(K)
        if mode == "plain":
            g = j // m
        elif mode == "shift":
            g = (j + m - shift) // m
        else:
            g = (j // (m * stride)) * stride + j % stride
        sizes.append(np.bincount(g, weights=rows).astype(np.int64))
    return np.concatenate(sizes) if sizes else np.zeros(0, dtype=np.int64)


def cpu_baseline(w, sample_rows: int):
    """Time the oracle on the host: bucketize on every point, attention on sampled query rows per pass."""
    import oracle
    S = w.bucket_cap // w.scope_buckets
    t0 = time.perf_counter()
    ref = oracle.bucketize(w.coords, w.batch_offsets, w.voxel_size, S, "zorder_div")
    t_b = time.perf_counter() - t0
    q, k, v = w.qkv()
    rng = np.random.default_rng(1)
    rows = rng.choice(w.n, size=min(sample_rows, w.n), replace=False)
    sel = np.zeros(w.n, dtype=np.uint8)
    sel[rows] = 1
    t_rows = 0.0
    for mode in w.modes:
        t0 = time.perf_counter()
        oracle.attn(q, k, v, ref["perm"], ref["offsets"], ref["scan_bucket_start"], w.scope_buckets, mode, w.heads,
                    w.head_dim, row_sel=sel)
        t_rows += time.perf_counter() - t0
    t_u = 0.0
    est = t_b + t_rows * (w.n / len(rows)) + t_u
    return {"value": w.n / est, "unit": "points/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"bucketize on all {w.n} points ({t_b:.3f} s) + fp64 attention for {len(rows)} sampled query rows "
                      f"in each of the {len(w.modes)} passes ({t_rows:.2f} s), scaled to all rows",
            "seconds": round(t_b + t_rows, 3)}


def measured_ceilings(head_dim: int) -> dict:
    """What this GPU sustains on the attention kernel's instruction mix with no memory traffic (register-only
    loops, random operand bits), best over 1..8 waves per SIMD, as score elements (1024 per 32x32 tile) per second
    and as nanoseconds per tile and SIMD: the matrix core alone, the softmax's vector work alone, the tile loops
    written serially and software-pipelined as the kernel issues them, and the vector and matrix streams of a
    head_dim-32 tile with no data dependence between them."""
    import ctypes

    import torch  # noqa: F401  (the HIP runtime that is already loaded)
    mb = ctypes.CDLL(os.path.join(ROOT, "paper_2412_16481_amd", "libf3d_microbench.so"))
    mb.f3d_mb_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double)]
    kinds = ((0, "mfma_only"), (1, "softmax_only"), (2, "tile_loop"), (3, "pipelined_tile_d32"), (4, "pipelined_tile_d16"),
             (5, "vector_part_d32"), (6, "six_mfma_per_tile"), (7, "vector_and_six_mfma_independent"))
    best, single = {}, {}
    for kind, name in kinds:
        for wps in (1, 2, 3, 4, 5, 6, 8):
            ms, work = ctypes.c_float(0), ctypes.c_double(0)
            rc = mb.f3d_mb_run(kind, wps, ctypes.byref(ms), ctypes.byref(work))
            if rc != 0:
                raise RuntimeError(f"f3d_mb_run failed: hipError {rc}")
            rate = work.value / (ms.value * 1e-3)
            if wps == 1:
                single[name] = rate
            if name not in best or rate > best[name][0]:
                best[name] = (rate, wps)
    sm = torch.cuda.get_device_properties(0).multi_processor_count * 4   # SIMDs

    def ns_per_tile(rate):   # elements/s over the whole GPU -> ns per 1024-element tile on one SIMD
        return 1024.0 * sm / rate * 1e9

    res = {
        "mfma_only_tflops": best["mfma_only"][0] / 1e12, "mfma_only_waves_per_simd": best["mfma_only"][1],
        "softmax_only_gelem_per_s": best["softmax_only"][0] / 1e9,
        "softmax_only_as_attention_tflops": best["softmax_only"][0] * 4.0 * head_dim / 1e12,
        "tile_loop_gelem_per_s": best["tile_loop"][0] / 1e9, "tile_loop_waves_per_simd": best["tile_loop"][1],
        "tile_loop_as_attention_tflops_d16": best["tile_loop"][0] * 64.0 / 1e12,
        "pipelined_tile_d32_as_attention_tflops": best["pipelined_tile_d32"][0] * 128.0 / 1e12,
        "pipelined_tile_d16_as_attention_tflops": best["pipelined_tile_d16"][0] * 64.0 / 1e12,
        "ns_per_tile_and_simd": {name: {"best": ns_per_tile(best[name][0]), "waves_per_simd": best[name][1],
                                        "one_wave": ns_per_tile(single[name])} for _, name in kinds[1:]},
        "note": "register-only loops, random operand bits, best over 1..8 waves per SIMD; elements = score elements",
    }
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="lidar8",
                    help="tiny | indoor | lidar4 | wide | lidar8 (configurations 1-5; the default is the largest) | scope8k (scope 8192)")
    ap.add_argument("--hash", default="zorder_div")
    ap.add_argument("--cpu-rows", type=int, default=-1,
                    help="query rows the oracle computes per pass (-1 = about 20 s of host work, 0 = skip)")
    ap.add_argument("--separate-unpermute", dest="fuse_unpermute", action="store_false",
                    help="run f3d_unpermute as a kernel of its own instead of folding it into the last pass's store")
    ap.add_argument("--pool", type=int, default=0, metavar="RHO",
                    help="also time f3d_inbucket_pool (mean, tiles of 1024 rows, this reduction factor) on the attention output")
    ap.add_argument("--backward", action="store_true",
                    help="also time f3d_bucket_swin_attn_bwd (after a forward that stores the log-sum-exp) for every pass")
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"],
                    help="element type of q, k, v and the output: bf16 (the benchmark configurations) or f16 (the "
                         "Appendix's FP16 features; forward path only, not with --pool/--backward/--glue)")
    ap.add_argument("--bucketize-scale", type=int, default=0, metavar="SCANS",
                    help="also time f3d_psh_bucketize alone on SCANS uniform-cube scans of 131072 points each (its "
                         "bandwidth regime: the five configurations are too small to load the memory system)")
    ap.add_argument("--rebalance", action="store_true",
                    help="also time f3d_psh_bucketize with the rebalancing variants: canonical (input-order-independent) "
                         "serving order, seeded probe directions, both")
    ap.add_argument("--glue", action="store_true",
                    help="also time f3d_ln_linear as the block's QKV projection (LayerNorm, rows gathered into bucket-major "
                         "order) and as its output projection (residual, rows scattered back)")
    ap.add_argument("--overlap", action="store_true",
                    help="also time the steps as a two-stream pipeline: the bucketing of batch i+1 runs beside the attention of batch i")
    ap.add_argument("--ceilings", action="store_true",
                    help="also run the register-only issue-rate microbenchmark (MFMA only, softmax only, the attention "
                         "tile loop) and add its rates to the JSON line")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="also run one plain device copy of this many MiB (counter calibration for rocprofv3 --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU; --gpus above 1 is not supported (no collectives, no sharding)",
              file=sys.stderr)
        return 2

    import torch

    import paper_2412_16481_amd as f3d
    from paper_2412_16481_amd import workloads as wl

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.make_workload(args.workload)
    n, C, H, d, m = w.n, w.channels, w.heads, w.head_dim, w.scope_buckets
    coords = torch.from_numpy(w.coords).to(dev)
    bo = torch.from_numpy(w.batch_offsets).to(dev)
    gen = torch.Generator(device=dev).manual_seed(w.seed)
    if args.dtype == "f16" and (args.pool or args.backward or args.glue):
        sys.exit("bench.py: --dtype f16 covers the forward path only")
    # the seeded N(0,1) features of the workload, the same arrays the parity tests feed to both sides (bf16 bit
    # patterns; for --dtype f16 the same values rounded to binary16)
    q, k, v = (torch.from_numpy(a).to(dev).view(torch.bfloat16) for a in w.qkv())
    if args.dtype == "f16":
        q, k, v = (t.to(torch.float16) for t in (q, k, v))
    bucket_major = args.workload == "lidar8"      # that workload keeps its layers on bucket-major features

    max_scan = int(np.diff(w.batch_offsets).max())
    p = f3d.make_params(w.voxel_size, w.bucket_cap, m, args.hash, max_scan_points=max_scan)
    ws = torch.empty(f3d.workspace_bytes(n, w.n_scans, p), dtype=torch.uint8, device=dev)
    bk = f3d.psh_bucketize(coords, bo, p, ws)
    out = torch.empty_like(q)
    back = torch.empty_like(q)
    torch.cuda.synchronize()

    offsets = bk.offsets.cpu().numpy()
    sbs = bk.scan_bucket_start.cpu().numpy()
    placed = bk.placed_per_round.cpu().numpy()
    flops = {}
    for mode in dict.fromkeys(w.modes):
        sz = scope_sizes(offsets, sbs, m, mode, 2, 2)
        flops[mode] = float((4.0 * sz.astype(np.float64) ** 2 * C).sum())

    def step(events=None, detail=False):
        """One pass of the whole path. In the timed region only the group of attention launches is bracketed by
        events (an event costs a few microseconds of stream time); detail=True marks every part."""
        def mark(always=False):
            if events is not None and (detail or always):
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                events.append(e)
        mark()
        f3d.psh_bucketize(coords, bo, p, ws, bk)
        mark(True)
        for i, mode in enumerate(w.modes):
            last = i + 1 == len(w.modes)
            if not last or not args.fuse_unpermute:
                f3d.bucket_swin_attn(q, k, v, bk, H, d, mode, 2, 2, not bucket_major, 0.0, out)
            else:   # the last pass stores its rows straight at their input positions
                f3d.bucket_swin_attn(q, k, v, bk, H, d, mode, 2, 2, not bucket_major, 0.0, back, True)
            mark(last)
        if not args.fuse_unpermute:
            f3d.unpermute(out, bk.perm, back)
            mark()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy > 0:   # a copy of known size: FETCH_SIZE / WRITE_SIZE read against it give the scale factor
        src_c = torch.zeros(args.calibrate_copy << 20, dtype=torch.uint8, device=dev)
        dst_c = torch.empty_like(src_c)
        dst_c.copy_(src_c)
        torch.cuda.synchronize()
    all_events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev = []
        step(ev)
        all_events.append(ev)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # the attention kernel: launch duration from the events recorded on the launch stream inside the timed region
    # (mean and standard deviation over the steps, per launch); a step's own duration is the time between the
    # "bucketing done" events of consecutive steps
    attn_group = np.array([ev[0].elapsed_time(ev[1]) for ev in all_events]) / len(w.modes)
    attn_ms_per_launch = float(attn_group.mean())
    step_ms = np.array([all_events[i][0].elapsed_time(all_events[i + 1][0]) for i in range(len(all_events) - 1)])
    # every part by itself, from a short loop after the timed region (events around each launch)
    detail = []
    for _ in range(min(args.steps, 10)):
        ev = []
        step(ev, True)
        detail.append(ev)
    torch.cuda.synchronize()
    parts = np.array([[ev[i].elapsed_time(ev[i + 1]) for i in range(len(ev) - 1)] for ev in detail])  # ms
    t_buck = parts[:, 0].mean()
    t_attn = parts[:, 1:1 + len(w.modes)]
    t_unp = parts[:, -1].mean() if not args.fuse_unpermute else 0.0
    attn_flop_per_launch = np.mean([flops[mo] for mo in w.modes])
    tflops = attn_flop_per_launch / (attn_ms_per_launch * 1e-3) / 1e12
    buck_gbps = 20.0 * n / (t_buck * 1e-3) / 1e9

    res = {
        "metric": "points/sec for PSH bucketize+Bucket-Swin attn fwd; attn TFLOP/s (% MFMA peak)",
        "value": n / (ms_per_step * 1e-3),
        "unit": "points/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_std": float(step_ms.std(ddof=1)) if len(step_ms) > 1 else None,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "points": n, "scans": w.n_scans, "channels": C, "heads": H, "head_dim": d,
                   "bucket_cap": w.bucket_cap, "scope_buckets": m, "hash": args.hash, "passes": w.modes,
                   "features": "bucket-major" if bucket_major else "input order, gathered through perm",
                   "unpermute": "in the last pass's store" if args.fuse_unpermute else "separate kernel"},
        "roofline": {"bound": "mfma", "kernel": "k_attn", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / PEAK_BF16_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                     "traffic_source": f"profiles/k_attn_{w.name}.md (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE of this command)"
                                       if w.name in MEASURED_TRAFFIC_BYTES else None,
                     "flop_per_launch": attn_flop_per_launch, "ms_per_launch": attn_ms_per_launch,
                     "ms_per_launch_std": float(attn_group.std(ddof=1)) if len(attn_group) > 1 else None},
        "parts_ms": {"bucketize": float(t_buck), "attn_per_pass": [float(x) for x in t_attn.mean(axis=0)], "unpermute": float(t_unp),
                     "from": "events around every launch, in a short loop after the timed region"},
        "bucketize": {"bound": "hbm", "achieved": buck_gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                      "frac": buck_gbps / PEAK_HBM_GBPS, "bytes_per_point": 20,
                      "placed_share": {"direct": float(placed[0]) / n, "probes": float(placed[1:7].sum()) / n,
                                       "recycle": float(placed[7]) / n}},
    }
    if args.overlap:
        # Serving many batches: the bucketing of a batch (few, latency-bound workgroups) and the attention of the batch
        # before it (fills the GPU) do not depend on each other, so they run on two streams with two sets of bucketing
        # outputs. Every step still does all of its work inside the timed region; `value` above stays the one-batch-
        # at-a-time figure.
        s_b, s_a = torch.cuda.Stream(), torch.cuda.Stream()
        sets = [(ws, bk), (torch.empty_like(ws), None)]
        with torch.cuda.stream(s_b):
            sets[1] = (sets[1][0], f3d.psh_bucketize(coords, bo, p, sets[1][0]))
        torch.cuda.synchronize()
        ready = [torch.cuda.Event(), torch.cuda.Event()]
        free = [torch.cuda.Event(), torch.cuda.Event()]

        def piped(steps):
            for i in range(steps):
                wsi, bki = sets[i & 1]
                with torch.cuda.stream(s_b):
                    if i >= 2:
                        s_b.wait_event(free[i & 1])        # the attention of batch i-2 has read these arrays
                    f3d.psh_bucketize(coords, bo, p, wsi, bki)
                    ready[i & 1].record()
                with torch.cuda.stream(s_a):
                    s_a.wait_event(ready[i & 1])
                    for j, mode in enumerate(w.modes):
                        if j + 1 < len(w.modes):
                            f3d.bucket_swin_attn(q, k, v, bki, H, d, mode, 2, 2, not bucket_major, 0.0, out)
                        else:
                            f3d.bucket_swin_attn(q, k, v, bki, H, d, mode, 2, 2, not bucket_major, 0.0, back, True)
                    free[i & 1].record()
            torch.cuda.synchronize()

        piped(args.warmup + 2)
        t0 = time.perf_counter()
        piped(args.steps)
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        res["overlapped"] = {"ms_per_step": ms, "points_per_s": n / (ms * 1e-3), "streams": 2,
                             "note": "bucketing of batch i+1 beside the attention of batch i; all K steps inside the timed region"}
    if args.pool > 0:   # the stage's third operator, outside the headline step
        rho = args.pool
        pooled = f3d.inbucket_pool(coords, bk.perm, out, bo, 1024, rho, 0.1, args.hash, "mean")
        pws = torch.empty(max(256, f3d.pool_workspace_bytes(n, w.n_scans, 1024)), dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        n_out = int(pooled.pooled_offsets[-1])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            f3d.inbucket_pool(coords, bk.perm, out, bo, 1024, rho, 0.1, args.hash, "mean", pws, pooled)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        nbytes = n * (2 * C + 12 + 4 + 4) + n_out * (2 * C + 12)   # features, coordinates, perm, sub_of; pooled rows and positions
        gbps = nbytes / (ms * 1e-3) / 1e9
        res["pool"] = {"rho": rho, "tile": 1024, "op": "mean", "pooled_rows": n_out, "ms": ms, "points_per_s": n / (ms * 1e-3),
                       "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                    "frac": gbps / PEAK_HBM_GBPS, "bytes": nbytes}}
    if args.bucketize_scale > 0:   # the bucketing alone on a batch large enough to be limited by memory traffic
        big_c, big_bo = wl.many_scans(args.bucketize_scale, 131072, seed=w.seed)
        nb = int(big_c.shape[0])
        pb = f3d.make_params(0.05, 1024, 4, args.hash, max_scan_points=131072)
        cb, bob = torch.from_numpy(big_c).to(dev), torch.from_numpy(big_bo).to(dev)
        wsb = torch.empty(f3d.workspace_bytes(nb, args.bucketize_scale, pb), dtype=torch.uint8, device=dev)
        bkb = f3d.psh_bucketize(cb, bob, pb, wsb)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            f3d.psh_bucketize(cb, bob, pb, wsb, bkb)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        gbps = 20.0 * nb / (ms * 1e-3) / 1e9
        plb = bkb.placed_per_round.cpu().numpy()
        res["bucketize_scale"] = {"scans": args.bucketize_scale, "points": nb, "ms": ms, "points_per_s": nb / (ms * 1e-3),
                                  "roofline": {"bound": "hbm", "achieved": gbps, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                               "frac": gbps / PEAK_HBM_GBPS, "bytes_per_point": 20},
                                  "placed_share": {"direct": float(plb[0]) / nb, "probes": float(plb[1:7].sum()) / nb,
                                                   "recycle": float(plb[7]) / nb}}
        del cb, bob, wsb, bkb
    if args.rebalance:   # variants of Algorithm 2, outside the headline step
        var = {}
        for name, kw in (("index_axes", {}), ("canonical", {"order": "canonical"}), ("seeded", {"probe_mode": "seeded", "probe_seed": 1}),
                         ("canonical_seeded", {"order": "canonical", "probe_mode": "seeded", "probe_seed": 1})):
            pv = f3d.make_params(w.voxel_size, w.bucket_cap, m, args.hash, max_scan_points=max_scan, **kw)
            wsv = torch.empty(f3d.workspace_bytes(n, w.n_scans, pv), dtype=torch.uint8, device=dev)
            bkv = f3d.psh_bucketize(coords, bo, pv, wsv)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                f3d.psh_bucketize(coords, bo, pv, wsv, bkv)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            pl = bkv.placed_per_round.cpu().numpy()
            var[name] = {"ms": ms, "points_per_s": n / (ms * 1e-3), "workspace_bytes": int(wsv.numel()),
                         "placed_share": {"direct": float(pl[0]) / n, "probes": float(pl[1:7].sum()) / n, "recycle": float(pl[7]) / n}}
        res["rebalance_variants"] = var
    if args.backward:   # training: gradient of every pass, outside the headline step
        lse = torch.empty(n, H, dtype=torch.float32, device=dev)
        dout = torch.randn(n, C, device=dev, generator=gen, dtype=torch.float32).to(torch.bfloat16)
        bws = torch.empty(n * H * 4 + 512, dtype=torch.uint8, device=dev)
        per_mode = {}
        for mode in dict.fromkeys(w.modes):
            f3d.bucket_swin_attn(q, k, v, bk, H, d, mode, 2, 2, not bucket_major, 0.0, out, lse=lse)
            f3d.bucket_swin_attn_bwd(q, k, v, out, dout, lse, bk, H, d, mode, 2, 2, not bucket_major, workspace=bws)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                f3d.bucket_swin_attn_bwd(q, k, v, out, dout, lse, bk, H, d, mode, 2, 2, not bucket_major, workspace=bws)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            fl = 2.5 * flops[mode]   # five products of 2 n_g^2 d each per head, against the forward's two
            per_mode[mode] = {"ms": ms, "tflops": fl / (ms * 1e-3) / 1e12, "flop": fl}
        mean_tf = float(np.mean([x["tflops"] for x in per_mode.values()]))
        res["backward"] = {"per_mode": per_mode,
                           "roofline": {"bound": "mfma", "achieved": mean_tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                        "frac": mean_tf / PEAK_BF16_TFLOPS},
                           "note": "algorithmic FLOP = 2.5 x forward; the two kernels recompute S and dP, which is not counted"}
    if args.glue:
        feat = torch.randn(n, C, device=dev, generator=gen, dtype=torch.float32).to(torch.bfloat16)
        wqkv = (torch.randn(3 * C, C, device=dev, generator=gen, dtype=torch.float32) / C ** 0.5).to(torch.bfloat16)
        wo = (torch.randn(C, C, device=dev, generator=gen, dtype=torch.float32) / C ** 0.5).to(torch.bfloat16)
        gamma, beta = torch.ones(C, device=dev), torch.zeros(C, device=dev)
        bqkv, bo_ = torch.zeros(3 * C, device=dev), torch.zeros(C, device=dev)

        def timed(fn):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

        ms_qkv = timed(lambda: f3d.ln_linear(feat, wqkv, bqkv, gamma, beta, 1e-5, bk.perm, n_outs=3))
        ms_out = timed(lambda: f3d.ln_linear(out, wo, bo_, None, None, 0.0, None, feat, bk.perm))
        by_qkv = n * (2 * C + 4 + 3 * 2 * C)            # features and perm read, q, k, v written
        by_out = n * (2 * C + 4 + 2 * C + 2 * C)        # attention output and perm read, residual read, result written
        res["glue"] = {
            "qkv": {"ms": ms_qkv, "tflops": 2.0 * n * C * 3 * C / (ms_qkv * 1e-3) / 1e12,
                    "roofline": {"bound": "hbm", "achieved": by_qkv / (ms_qkv * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                 "frac": by_qkv / (ms_qkv * 1e-3) / 1e9 / PEAK_HBM_GBPS, "bytes": by_qkv}},
            "out_proj": {"ms": ms_out, "tflops": 2.0 * n * C * C / (ms_out * 1e-3) / 1e12,
                         "roofline": {"bound": "hbm", "achieved": by_out / (ms_out * 1e-3) / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                      "frac": by_out / (ms_out * 1e-3) / 1e9 / PEAK_HBM_GBPS, "bytes": by_out}}}
    if args.ceilings:
        res["ceilings"] = measured_ceilings(d)
    cpu_rows = args.cpu_rows
    if cpu_rows < 0:
        # The oracle's attention costs about scope * C multiply-adds (binary64, QK^T and PV) per query row and pass and
        # runs at roughly 9e9 of them per second on 16 host threads: sample as many rows as about 20 s pay for.
        cpu_rows = int(min(n, 1.8e11 / (w.bucket_cap * C * len(w.modes))))
    if cpu_rows > 0:
        res["cpu_baseline"] = cpu_baseline(w, cpu_rows)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
