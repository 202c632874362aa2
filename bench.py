#!/usr/bin/env python3
"""Benchmark of the BSFA forward on one MI355X.

A step is one bsfa_forward call (every stage of the hot path: Q load, K stream, QK^T, block
maximum, gate, and for kept blocks V fetch, online softmax, PV, then finalisation and skip
statistics) on the headline workload: one Llama-3.1-8B-shaped attention layer (B=1, 32 query
heads, 8 KV heads, d=128, causal, bf16) at N=131072 with per-head thresholds calibrated on a
separate seed for ~50 % block skip.  Inputs are synthetic and resident in HBM before timing.
The same kernel with thresholds = -inf (its dense path) is timed next to it, and the CPU oracle
is timed on a bounded sample of the same workload, which doubles as a parity check.

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W [--seqlen N] [--skip F]`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak (256 CUs x 4 SIMDs x 1024 FLOP/clk x 2.4 GHz)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seqlen", type=int, default=131072)
    ap.add_argument("--skip", type=float, default=0.5, help="target skip fraction of gateable tiles")
    ap.add_argument("--block-m", type=int, default=128)
    ap.add_argument("--sweep", default="", help="comma-separated extra skip targets, e.g. 0.25,0.75,0.9: adds a "
                                                "'sweep' list (time, measured skip, speed-up, eta per target) to the JSON line")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--cpu-items", type=int, default=0, help="oracle sample size (0 = sized for ~20 s)")
    ap.add_argument("--traffic-json", default=None, help="file with measured HBM bytes per launch (from rocprofv3 --pmc)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain elementwise copy of Q into O (known size: reads and writes "
                         "2*N*Hq*d bytes each) so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_07011_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shp = synth.llama_shape(args.seqlen, block_m=args.block_m)
    bm, bn, d = shp.block_m, shp.block_n, shp.head_dim

    # calibration sample (seed 1) -> thresholds; evaluation sample (seed 0)
    qc, kc, _ = synth.llama_layer(1, shp, device=dev)
    ws = torch.empty(binding.lib().bsfa_calibrate_workspace_bytes(binding.make_problem(qc, kc, None, None, bm, bn)),
                     dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sweep_targets = [float(x) for x in args.sweep.split(",") if x]
    taus = binding.bsfa_calibrate(qc, kc, [args.skip] + sweep_targets, block_m=bm, block_n=bn, workspace=ws)
    tau = taus[0]
    t_calib = time.perf_counter() - t0
    del qc, kc, ws
    torch.cuda.empty_cache()
    q, k, v = synth.llama_layer(0, shp, device=dev)
    out = torch.empty_like(q)
    tau_d = tau.to(dev)
    neg_d = torch.full_like(tau_d, float("-inf"))
    st = binding.alloc_stats(q, bm, bn, counts=True)

    def timed(thr, steps, warmup):
        for _ in range(warmup):
            binding.bsfa_forward(q, k, v, thr, out=out, skip_stats=st, block_m=bm, block_n=bn)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t_wall = time.perf_counter()
        ev[0].record()
        for s in range(steps):
            binding.bsfa_forward(q, k, v, thr, out=out, skip_stats=st, block_m=bm, block_n=bn)
            ev[s + 1].record()
        torch.cuda.synchronize()
        t_wall = time.perf_counter() - t_wall
        per = [ev[s].elapsed_time(ev[s + 1]) for s in range(steps)]       # ms, includes the tiny counter-reset launch
        return t_wall * 1e3 / steps, per, st.counts.cpu().numpy().copy()

    if args.copy_probe:
        torch.add(q, 0, out=out)
        torch.cuda.synchronize()
    ms_sparse, per_sparse, c_sparse = timed(tau_d, args.steps, args.warmup)
    ms_dense, per_dense, c_dense = timed(neg_d, args.steps, args.warmup)

    tile_flops = 2.0 * bm * bn * d                         # one of the two contractions on one tile
    f_dense_equiv = 4.0 * d * shp.n_q_heads * shp.batch * float(shp.seqlen) ** 2 / 2.0
    reach = float(c_sparse[..., 2].sum())
    skipped = float(c_sparse[..., 0].sum())
    gateable = float(c_sparse[..., 1].sum())
    f_exec_sparse = tile_flops * (2 * reach - skipped)
    f_exec_dense = tile_flops * 2 * reach
    kern_ms_sparse = float(np.mean(per_sparse))
    kern_ms_dense = float(np.mean(per_dense))
    tf_sparse_equiv = f_dense_equiv / (ms_sparse * 1e-3) / 1e12
    tf_dense = f_dense_equiv / (ms_dense * 1e-3) / 1e12
    exec_tf_sparse = f_exec_sparse / (kern_ms_sparse * 1e-3) / 1e12
    exec_tf_dense = f_exec_dense / (kern_ms_dense * 1e-3) / 1e12
    f_skip = skipped / reach
    speedup = ms_dense / ms_sparse
    eta = (1.0 - ms_sparse / ms_dense) / (f_skip / 2.0) if f_skip > 0 else None

    # HBM bytes per launch of the gated kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    # scaled by a known-size copy; read from the file written from those runs
    traffic = None
    tj = args.traffic_json or os.path.join(ROOT, "profiles", "bsfa_fwd_kernel_traffic.json")
    if os.path.exists(tj):
        rec = json.load(open(tj))
        if rec.get("seqlen") == shp.seqlen:
            traffic = rec.get("hbm_bytes_per_launch_gated")

    result = {
        "metric": "dense-equiv attention TFLOP/s at ~50% block skip (speedup vs own dense path beside it)",
        "value": round(tf_sparse_equiv, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_sparse, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Llama-3.1-8B attention layer prefill, B=1 Hq=32 Hkv=8 d=128 causal N=%d, tile %dx%d, "
                               "per-head tau calibrated on a separate seed for %.0f%% skip" % (shp.seqlen, bm, bn, 100 * args.skip),
                   "seqlen": shp.seqlen, "target_skip": args.skip},
        "skip_fraction_of_reachable": round(f_skip, 4), "skip_fraction_of_gateable": round(skipped / gateable, 4),
        "dense_path": {"ms_per_step": round(ms_dense, 3), "tflops": round(tf_dense, 2),
                       "mfma_frac_executed": round(exec_tf_dense / PEAK_BF16_TFLOPS, 4)},
        "speedup_vs_own_dense": round(speedup, 4), "ideal_speedup": round(2 / (2 - f_skip), 4),
        "skip_efficiency_eta": None if eta is None else round(eta, 4),
        "step_ms_min_median": [round(float(np.min(per_sparse)), 3), round(float(np.median(per_sparse)), 3)],
        "calibrate_s": round(t_calib, 3),
        "roofline": {"bound": "mfma", "kernel": "bsfa_fwd_kernel (gated, %.0f%% skip)" % (100 * f_skip),
                     "achieved": round(exec_tf_sparse, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(exec_tf_sparse / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                     "flops_per_launch": f_exec_sparse, "kernel_ms": round(kern_ms_sparse, 3)},
    }

    if sweep_targets:
        sweep = []
        for f_t, t_l in zip(sweep_targets, taus[1:]):
            ms_l, _, c_l = timed(t_l.to(dev), max(3, args.steps // 2), 1)
            f_l = float(c_l[..., 0].sum()) / float(c_l[..., 2].sum())
            sweep.append({"target_skip": f_t, "skip_fraction_of_reachable": round(f_l, 4), "ms_per_step": round(ms_l, 3),
                          "dense_equiv_tflops": round(f_dense_equiv / (ms_l * 1e-3) / 1e12, 2),
                          "speedup_vs_own_dense": round(ms_dense / ms_l, 4), "ideal_speedup": round(2 / (2 - f_l), 4),
                          "skip_efficiency_eta": round((1.0 - ms_l / ms_dense) / (f_l / 2.0), 4) if f_l > 0 else None})
        result["sweep"] = sweep

    if not args.no_cpu:
        from oracle import bsfa_oracle as orc
        from tests import parity
        orc.build()
        # bounded sample of (head, query tile) items of the same workload, ~20 s of oracle time
        items = parity.sample_items(shp, n_random=8, seed=0)
        if args.cpu_items:
            items = items[:args.cpu_items]
        else:
            # oracle cost grows with the tile index; cap the summed reachable key blocks
            budget = 1.2e6
            keep, tot = [], 0
            for it in sorted(items, key=lambda x: x[2]):
                nb = -(-((it[2] + 1) * bm) // bn)
                if tot + nb > budget and keep:
                    continue
                keep.append(it)
                tot += nb
            items = keep
        bst = binding.alloc_stats(q, bm, bn, counts=False, skip_mask=True)
        binding.bsfa_forward(q, k, v, tau_d, out=out, skip_stats=bst, block_m=bm, block_n=bn)
        torch.cuda.synchronize()
        qh, kh, vh = q.float().cpu(), k.float().cpu(), v.float().cpu()
        t0 = time.perf_counter()
        r = orc.forward_items(qh, kh, vh, tau.numpy(), bm, bn, True, items)
        t_cpu = time.perf_counter() - t0
        units = int((r.cls != orc.CLS_UNREACHABLE).sum())
        cpu_tf = 2 * tile_flops * units / t_cpu / 1e12
        rep = parity.compare(q, k, v, tau, bm, bn, True, out, bst.skip_mask, None, items=items, oracle_result=r)
        result["cpu_baseline"] = {"value": round(cpu_tf, 6), "unit": "TFLOP/s (dense-equivalent)", "cores": orc.threads(),
                                  "kind": "oracle", "seconds": round(t_cpu, 2),
                                  "sample": "%d (head, query-tile) items = %d tile x key-block units of the same inputs; "
                                            "full problem extrapolates to %.0f s" % (len(items), units, t_cpu / units * reach)}
        result["parity"] = {"items": rep.n_items, "max_abs": rep.max_abs, "mean_abs": rep.mean_abs,
                            "mask_mismatch_in_band": rep.mask_mismatch, "tiles_in_band": rep.in_band}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
