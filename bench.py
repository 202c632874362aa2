#!/usr/bin/env python3
"""Benchmark of the BSFA forward on one MI355X.

A step is one bsfa_forward call (every stage of the hot path: Q load, K stream, QK^T, block
maximum, gate, and for kept blocks V fetch, online softmax, PV, then finalisation and skip
statistics; the once-per-call rewrite of V into the forward workspace is part of the step) on
the headline workload: one Llama-3.1-8B-shaped attention layer (B=1, 32 query heads, 8 KV heads,
d=128, causal, bf16) at N=131072 with per-head thresholds calibrated on a separate seed for ~50 %
block skip.  Inputs are synthetic and resident in HBM before timing.  The same kernel with
thresholds = -inf (its dense path) is timed next to it.  The same line also carries the sparsity
sweep at 128K (25 / 75 / 90 % skip) and the 32K and 64K sizes at 50 % skip, every point with its
time, dense-equivalent TFLOP/s, executed fraction of the MFMA peak, skip efficiency and the error
against the CPU oracle on sampled (head, query tile) items.  The CPU oracle is timed on a bounded
sample of the headline workload.

Prints ONE JSON line.  `python bench.py --gpus 1 --steps K --warmup W [--seqlen N] [--skip F]`.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak (256 CUs x 4 SIMDs x 1024 FLOP/clk x 2.4 GHz)
NOMINAL_SCLK_MHZ = 2400.0      # the shader clock that peak is quoted at


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seqlen", type=int, default=131072)
    ap.add_argument("--skip", type=float, default=0.5, help="target skip fraction of gateable tiles")
    ap.add_argument("--block-m", type=int, default=128)
    ap.add_argument("--sweep", default="0.25,0.75,0.9",
                    help="comma-separated extra skip targets at --seqlen ('' for none): adds a 'sweep' list")
    ap.add_argument("--sizes", default="32768,65536",
                    help="comma-separated extra sequence lengths timed at --skip and dense ('' for none): adds a 'sizes' list")
    ap.add_argument("--noncausal", type=int, default=32768,
                    help="sequence length of the bidirectional leg (causal = 0; dense and --skip); 0 for none")
    ap.add_argument("--no-sclk", action="store_true",
                    help="do not sample the shader clock under load (it runs extra launches outside the timed region)")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the probe of the matrix rate the card sustains (back-to-back MFMAs, nothing else)")
    ap.add_argument("--no-fp8-leg", action="store_true",
                    help="skip the leg that runs the score product on fp8 copies of Q and K (dense and --skip at --seqlen)")
    ap.add_argument("--no-cpu", action="store_true", help="skip every CPU-oracle leg (baseline and per-point parity)")
    ap.add_argument("--no-workspace", action="store_true", help="run bsfa_forward without its workspace (V read in place)")
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
    bn = 64
    bm = args.block_m
    sweep_targets = [float(x) for x in args.sweep.split(",") if x]
    sizes = [int(x) for x in args.sizes.split(",") if x and int(x) != args.seqlen]
    if not args.no_cpu:
        from oracle import bsfa_oracle as orc
        from tests import parity
        orc.build()

    def measure(seqlen, targets, steps, warmup, parity_budget, causal=True, qk_fp8=False, want_sclk=False, min_ms=0.0):
        """Dense path and every skip target at one sequence length.  Returns (shape, tensors, thresholds,
        list of point records); the first record is the dense path."""
        shp = synth.llama_shape(seqlen, block_m=bm)
        d = shp.head_dim
        qc, kc, _ = synth.llama_layer(1, shp, device=dev)               # calibration sample (seed 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        taus = binding.bsfa_calibrate(qc, kc, targets, causal=causal, block_m=bm, block_n=bn, qk_fp8=qk_fp8)
        ws = None
        t_calib = time.perf_counter() - t0
        del qc, kc, ws
        torch.cuda.empty_cache()
        q, k, v = synth.llama_layer(0, shp, device=dev)                 # evaluation sample (seed 0)
        out = torch.empty_like(q)
        fws = None
        if not args.no_workspace:
            fws = torch.empty(binding.forward_workspace_bytes(q, k, bm, bn, qk_fp8=qk_fp8), dtype=torch.uint8, device=dev)
        st = binding.alloc_stats(q, bm, bn, counts=True)
        tile_flops = 2.0 * bm * bn * d                                  # one of the two contractions on one tile
        f_dense_equiv = 4.0 * d * shp.n_q_heads * shp.batch * float(seqlen) ** 2 / (2.0 if causal else 1.0)

        # short launches: enough of them that the timed region outlasts the chip's clock transients
        est_ms = f_dense_equiv / 1.1e15 * 1e3
        steps = max(steps, int(min_ms / est_ms))
        warmup = max(warmup, int(0.3 * min_ms / est_ms))

        def fwd(thr, stats):
            binding.bsfa_forward(q, k, v, thr, causal=causal, out=out, skip_stats=stats, block_m=bm, block_n=bn, workspace=fws,
                                 qk_fp8=qk_fp8)

        def timed(thr):
            for _ in range(warmup):
                fwd(thr, st)
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            t_wall = time.perf_counter()
            ev[0].record()
            for s in range(steps):
                fwd(thr, st)
                ev[s + 1].record()
            torch.cuda.synchronize()
            t_wall = time.perf_counter() - t_wall
            per = [ev[s].elapsed_time(ev[s + 1]) for s in range(steps)]   # ms on the launch stream (incl. the small side kernels)
            return t_wall * 1e3 / steps, per, st.counts.cpu().numpy().copy()

        def sclk(thr):
            """Shader clock (MHz) that the management interface reports while this launch keeps the GPU busy
            (outside the timed region); None if it cannot be read."""
            for _ in range(max(4, int(1500.0 / max(ms_dense or 100.0, 1.0)))):
                fwd(thr, st)
            time.sleep(0.4)
            mhz = None
            try:
                r = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20)
                for line in r.stdout.splitlines():
                    if "sclk" in line and "Mhz" in line:
                        mhz = int(line.split("(")[-1].split("Mhz")[0])
            except Exception:
                mhz = None
            torch.cuda.synchronize()
            return mhz

        def check(thr_host, thr_dev, budget, n_random):
            """Sampled oracle parity of the launch just timed (block budget bounds the CPU time)."""
            items = parity.sample_items(shp, n_random=n_random, seed=seqlen % 997)
            keep, tot = [], 0
            for it in sorted(items, key=lambda x: x[2]):
                nb = -(-((it[2] + 1) * bm) // bn) if causal else shp.m_kv
                if tot + nb > budget and keep:
                    continue
                keep.append(it)
                tot += nb
            bst = binding.alloc_stats(q, bm, bn, counts=False, skip_mask=True)
            fwd(thr_dev, bst)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            r = orc.forward_items(qh, kh, vh, thr_host.numpy(), bm, bn, causal, keep)
            t_cpu = time.perf_counter() - t0
            rep = parity.compare(qh, kh, vh, thr_host, bm, bn, causal, out, bst.skip_mask, None, items=keep, oracle_result=r)
            return rep, r, t_cpu, keep

        if not args.no_cpu:
            if qk_fp8:      # the oracle gets what the score product multiplies: Q and K rounded to fp8 (e4m3, nearest even)
                qh, kh = (t.to(torch.float8_e4m3fn).float().cpu() for t in (q, k))
                vh = v.float().cpu()
            else:
                qh, kh, vh = q.float().cpu(), k.float().cpu(), v.float().cpu()
        points = []
        neg = torch.full((shp.n_q_heads,), float("-inf"))
        ms_dense = None
        for target, thr in [(0.0, neg)] + list(zip(targets, taus)):
            thr_d = thr.to(dev)
            ms, per, c = timed(thr_d)
            reach, skipped, gateable = float(c[..., 2].sum()), float(c[..., 0].sum()), float(c[..., 1].sum())
            f_exec = tile_flops * (2 * reach - skipped)
            kern_ms = float(np.mean(per))
            f_skip = skipped / reach
            if ms_dense is None:
                ms_dense = ms
            rec = {"seqlen": seqlen, "causal": causal, "qk_fp8": qk_fp8, "target_skip": target, "skip_fraction_of_reachable": round(f_skip, 4),
                   "skip_fraction_of_gateable": round(skipped / gateable, 4) if gateable else 0.0,
                   "ms_per_step": round(ms, 3), "kernel_ms": round(kern_ms, 3), "steps": steps,
                   "step_ms_min_median": [round(float(np.min(per)), 3), round(float(np.median(per)), 3)],
                   "dense_equiv_tflops": round(f_dense_equiv / (ms * 1e-3) / 1e12, 2),
                   "executed_tflops": round(f_exec / (kern_ms * 1e-3) / 1e12, 2),
                   "mfma_frac_executed": round(f_exec / (kern_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                   "flops_per_launch": f_exec,
                   "speedup_vs_own_dense": round(ms_dense / ms, 4), "ideal_speedup": round(2 / (2 - f_skip), 4),
                   "skip_efficiency_eta": round((1.0 - ms / ms_dense) / (f_skip / 2.0), 4) if f_skip > 0 else None}
            if want_sclk:
                mhz = sclk(thr_d)
                rec["sclk_mhz_under_load"] = mhz
                if mhz:     # the same executed rate against the matrix peak at the clock the chip actually held
                    rec["mfma_frac_at_observed_clock"] = round(rec["mfma_frac_executed"] * NOMINAL_SCLK_MHZ / mhz, 4)
            if not args.no_cpu:
                rep, _, t_cpu, _ = check(thr, thr_d, parity_budget, 1)
                rec["parity"] = {"items": rep.n_items, "max_abs": rep.max_abs, "mean_abs": rep.mean_abs,
                                 "mask_mismatch_in_band": rep.mask_mismatch, "tiles_in_band": rep.in_band,
                                 "oracle_s": round(t_cpu, 2)}
            points.append(rec)
        ctx = dict(shp=shp, q=q, k=k, v=v, out=out, taus=taus, t_calib=t_calib, check=check if not args.no_cpu else None,
                   tile_flops=tile_flops, reach=float(points[0]["flops_per_launch"] / (2 * tile_flops)))
        return ctx, points

    # ---- headline size: dense, --skip, sweep -----------------------------------------------------
    ctx, pts = measure(args.seqlen, [args.skip] + sweep_targets, args.steps, args.warmup, 1.5e5, want_sclk=not args.no_sclk)
    if args.copy_probe:
        torch.add(ctx["q"], 0, out=ctx["out"])
        torch.cuda.synchronize()
    dense, head = pts[0], pts[1]
    shp = ctx["shp"]

    # HBM bytes per launch of the gated kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    # scaled by a known-size copy; not measured in this run but read from the file written from those runs
    traffic, traffic_source = None, None
    tj = args.traffic_json or os.path.join(ROOT, "profiles", "bsfa_fwd_kernel_traffic.json")
    if os.path.exists(tj):
        rec = json.load(open(tj))
        if rec.get("seqlen") == shp.seqlen:
            traffic = rec.get("hbm_bytes_per_launch_gated")
            traffic_source = os.path.relpath(tj, ROOT) + " (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE of an earlier run, scaled by a known-size copy)"

    result = {
        "metric": "dense-equiv attention TFLOP/s at ~50% block skip (speedup vs own dense path beside it)",
        "value": head["dense_equiv_tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Llama-3.1-8B attention layer prefill, B=1 Hq=32 Hkv=8 d=128 causal N=%d, tile %dx%d, "
                               "per-head tau calibrated on a separate seed for %.0f%% skip" % (shp.seqlen, bm, bn, 100 * args.skip),
                   "seqlen": shp.seqlen, "target_skip": args.skip, "forward_workspace": not args.no_workspace},
        "skip_fraction_of_reachable": head["skip_fraction_of_reachable"], "skip_fraction_of_gateable": head["skip_fraction_of_gateable"],
        "dense_path": {"ms_per_step": dense["ms_per_step"], "tflops": dense["dense_equiv_tflops"],
                       "mfma_frac_executed": dense["mfma_frac_executed"],
                       "sclk_mhz_under_load": dense.get("sclk_mhz_under_load"),
                       "mfma_frac_at_observed_clock": dense.get("mfma_frac_at_observed_clock")},
        "sclk_mhz_under_load": head.get("sclk_mhz_under_load"),
        "speedup_vs_own_dense": head["speedup_vs_own_dense"], "ideal_speedup": head["ideal_speedup"],
        "skip_efficiency_eta": head["skip_efficiency_eta"],
        "step_ms_min_median": head["step_ms_min_median"],
        "calibrate_s": round(ctx["t_calib"], 3),
        "roofline": {"bound": "mfma", "kernel": "bsfa_fwd_kernel (gated, %.0f%% skip)" % (100 * head["skip_fraction_of_reachable"]),
                     "achieved": head["executed_tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": head["mfma_frac_executed"], "traffic": traffic, "traffic_source": traffic_source,
                     "flops_per_launch": head["flops_per_launch"], "kernel_ms": head["kernel_ms"]},
    }
    if "parity" in dense:
        result["dense_path"]["parity"] = dense["parity"]
    if sweep_targets:
        result["sweep"] = pts[2:]

    if not args.no_cpu:
        # CPU baseline: the oracle on a bounded sample of (head, query tile) items of the headline launch
        # (~15 s of oracle time), which is also one more parity check
        n_random = 8
        rep, r, t_cpu, items = ctx["check"](ctx["taus"][0], ctx["taus"][0].to(dev), 9e5, n_random)
        units = int((r.cls != orc.CLS_UNREACHABLE).sum())
        cpu_tf = 2 * ctx["tile_flops"] * units / t_cpu / 1e12
        result["cpu_baseline"] = {"value": round(cpu_tf, 6), "unit": "TFLOP/s (dense-equivalent)", "cores": orc.threads(),
                                  "kind": "oracle", "seconds": round(t_cpu, 2),
                                  "sample": "%d (head, query-tile) items = %d tile x key-block units of the same inputs; "
                                            "full problem extrapolates to %.0f s" % (len(items), units, t_cpu / units * ctx["reach"])}
        result["parity"] = {"items": rep.n_items, "max_abs": rep.max_abs, "mean_abs": rep.mean_abs,
                            "mask_mismatch_in_band": rep.mask_mismatch, "tiles_in_band": rep.in_band}
    del ctx
    torch.cuda.empty_cache()

    # ---- the other sequence lengths: dense and --skip ------------------------------------------------
    if sizes:
        result["sizes"] = []
        for n in sizes:
            c2, p2 = measure(n, [args.skip], max(args.steps, 10), args.warmup, 1.0e5, min_ms=1500.0)
            result["sizes"].append({"seqlen": n, "dense": p2[0], "gated": p2[1], "calibrate_s": round(c2["t_calib"], 3)})
            del c2
            torch.cuda.empty_cache()
    # ---- what the matrix pipe sustains on this card, with nothing else running --------------------
    # (the published peak assumes the nominal clock; under dense matrix load the chip clocks down, by an
    # amount that depends on the operand values, so the ceiling is measured with the workload's distribution)
    if not args.no_mfma_probe:
        wgs = torch.cuda.get_device_properties(dev).multi_processor_count * 8
        g = torch.Generator(device="cpu").manual_seed(7)
        sink = torch.empty(binding.lib().bsfa_mfma_rate_probe_sink_bytes(wgs) // 4, dtype=torch.float32, device=dev)
        probe = {"workgroups": wgs, "threads_per_workgroup": 512, "instruction": "v_mfma_f32_32x32x16_bf16"}
        for name, ops in (("constant_operands_tflops", torch.full((4096,), 1.0e-3)),
                          ("normal_operands_tflops", torch.randn(4096, generator=g))):
            ops = ops.to(dev)
            binding.mfma_rate_probe(ops, wgs, 2000, sink)
            torch.cuda.synchronize()
            rates = []
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fl = binding.mfma_rate_probe(ops, wgs, 20000, sink)
                e1.record()
                torch.cuda.synchronize()
                rates.append(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
            probe[name] = round(float(np.median(rates)), 1)
        probe["note"] = ("back-to-back MFMAs only, two waves per SIMD; 'normal' fills the operand registers with N(0,1) "
                         "samples (the workload's distribution), 'constant' with one small value")
        result["sustained_mfma"] = probe
        sus = probe["normal_operands_tflops"]
        result["dense_path"]["frac_of_sustained_mfma"] = round(dense["executed_tflops"] / sus, 4)
        result["roofline"]["frac_of_sustained_mfma"] = round(result["roofline"]["achieved"] / sus, 4)
        del sink
    # ---- score product on fp8 operands (qk_fp8 = 1): dense and --skip at the headline length ------------
    if not args.no_fp8_leg and bm == 128:
        c4, p4 = measure(args.seqlen, [args.skip], args.steps, args.warmup, 1.0e5, qk_fp8=True)
        result["qk_fp8"] = {"seqlen": args.seqlen, "dense": p4[0], "gated": p4[1],
                            "note": "Q and K rounded to fp8 e4m3 for the score product only; thresholds calibrated in the same mode; "
                                    "parity is against the oracle on the rounded Q and K"}
        del c4
        torch.cuda.empty_cache()
    # ---- bidirectional attention (causal = 0): dense and --skip ------------------------------------
    if args.noncausal:
        c3, p3 = measure(args.noncausal, [args.skip], max(args.steps, 10), args.warmup, 1.0e5, causal=False, min_ms=1500.0)
        result["noncausal"] = {"seqlen": args.noncausal, "dense": p3[0], "gated": p3[1]}
        del c3
        torch.cuda.empty_cache()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
