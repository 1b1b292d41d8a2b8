#!/usr/bin/env python3
"""Benchmark of the Gradient Cache hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]

A step is one pass of the loss + representation-gradient path (dQ walk that forms
the row statistics as it goes, merge of its splits into lse / loss rows / dQ, dP
walk, partial sums + loss sum) over one synthetic batch of the headline workload:
B=4096 queries, P=8192 passages, d=768, bf16 storage, fp32 accumulate.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

value      algorithmic TFLOP/s = 6*B*P*d / step time (three GEMMs: S, G*P, G^T*Q)
           K steps are timed with nothing else on the stream (mean); a second pass of K
           steps, each between two HIP events, gives the median and the minimum; the
           kernel times come from a third pass with HIP events at the kernel boundaries
           (the event records cost about 6 % of a step).
roofline   for the dominant kernel (the dQ walk, grad_online_kernel<768>): the
           algorithmic flops of one launch (4*B*P*d: the scores and G*P, both of
           which it forms exactly once) / its mean duration from HIP events recorded
           by the library on the launch stream, against the MI355X dense bf16 MFMA
           peak.  The dP walk (2*B*P*d algorithmic, 4*B*P*d executed: it forms the
           scores again) is listed beside it; `whole_path_executed_frac` counts all
           8*B*P*d executed flops of a step.
cpu_baseline  the fp64 numpy oracle timed on the host cores on the same batch.
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_BYTES_PER_S = 8.0e12   # MI355X HBM3E, published
PROFILE_FILE = os.path.join("profiles", "loss_path_config3_rocprofv3.txt")


def counter_traffic():
    """HBM bytes per launch of the dominant kernel.  Hardware counters cannot be read from inside this process: they
    come from separate `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` runs of this same command, scaled by what
    the same counters read for a plain copy kernel of known size, and are written down (with their date) in a
    `TRAFFIC {json}` line of the committed summary under profiles/.  None if that file or line is missing."""
    try:
        for line in open(os.path.join(ROOT, PROFILE_FILE)):
            if line.startswith("TRAFFIC "):
                return json.loads(line[len("TRAFFIC "):])
    except (OSError, ValueError):
        pass
    return None


def cpu_baseline(q, p, r, flops):
    from oracle import gc_oracle as O
    from paper_2101_06983_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    q64, p64, r64 = synth.widen(q), synth.widen(p), synth.widen(r)
    reps, t_total = 0, 0.0
    while reps < 3 and t_total < 30.0:
        t0 = time.perf_counter()
        O.loss_and_rep_grad(q64, p64, r64)
        t_total += time.perf_counter() - t0
        reps += 1
    sec = t_total / reps
    return {"value": flops / sec / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": "full workload batch (B=4096,P=8192,d=768), fp64 numpy oracle, mean of %d runs, %.2f s each" % (reps, sec)}


def side_workload(args, gc, synth, dev):
    """Timing of the other configurations (parity-test cases; not the headline line)."""
    if args.workload == "config2":
        q, p, r = synth.config2()
        qd, pd, rd = q.to(dev), p.to(dev), r.to(dev)
        ws = gc.alloc_workspace(gc.gc_workspace_bytes(128, 256, 768, gc.GC_BF16), dev)
        out = {}
        step = lambda: out.update(gc.gc_loss_and_rep_grad_ex(qd, pd, rd, 1.0, 1.0, 0, ("loss", "dq", "dp"), ws, out))
        flops, what = 6.0 * 128 * 256 * 768, "loss+rep-grad, B=128 P=256 d=768 bf16"
    elif args.workload == "config4":
        z = synth.ntxent_views().to(dev)
        ws = gc.alloc_workspace(gc.load().gc_ntxent_workspace_bytes(16384, 128), dev)
        step = lambda: gc.gc_ntxent_loss_and_grad_bf16(z, 0.07, ws)
        flops, what = 6.0 * 16384 * 16384 * 128, "NT-Xent loss+grad, 2N=16384 d=128 bf16 tau=0.07"
    elif args.workload == "bidir":
        import numpy as np
        n, d = 8192, 768
        r = torch.from_numpy(np.random.default_rng(7).permutation(n).astype(np.int32))
        q, p, r = synth.dpr_batch(n, n, d, seed=8, positive_mix=0.5, pos_idx=r)
        qd, pd, rd = q.to(dev), p.to(dev), r.to(dev)
        ws = gc.alloc_workspace(gc.load().gc_bidirectional_workspace_bytes(n, d), dev)
        res = gc.gc_bidirectional_loss_and_rep_grad_bf16(qd, pd, rd, 1.0, 1.0, ws)
        step = lambda: gc.gc_bidirectional_loss_and_rep_grad_bf16(qd, pd, rd, 1.0, 1.0, ws, out=res)
        flops, what = 2 * 6.0 * n * n * d, "symmetric loss+rep-grad, n=8192 d=768 bf16 (two directions)"
    elif args.workload == "bilinear":
        q, p, r = synth.config3()
        om = synth.bilinear_omega(768).to(dev)
        qd, pd, rd = q.to(dev), p.to(dev), r.to(dev)
        res = gc.gc_bilinear_loss_and_grads_bf16(qd, pd, rd, om)
        step = lambda: gc.gc_bilinear_loss_and_grads_bf16(qd, pd, rd, om, workspace=res["workspace"], out=res)
        flops = 6.0 * 4096 * 8192 * 768 + 3 * 2.0 * 4096 * 768 * 768
        what = "bilinear distance f^T Omega g: loss, u, v, dOmega at B=4096 P=8192 d=768 bf16"
    elif args.workload == "deepdist":
        B, P, d, h = 1024, 2048, 768, 128
        q, p, r = synth.dpr_batch(B, P, d, seed=8200)
        om = {k: t.to(dev) for k, t in synth.deep_omega(d).items()}
        qd, pd, rd = q.to(dev), p.to(dev), r.to(dev)
        res = gc.gc_deepdist_loss_and_grads_bf16(qd, pd, rd, om, 1.0, 0.5)
        step = lambda: gc.gc_deepdist_loss_and_grads_bf16(qd, pd, rd, om, 1.0, 0.5, workspace=res["workspace"], out=res)
        # vector arithmetic of the two walks over the B*P*h (pair, k) terms: add, exp2, add, reciprocal, fma in each
        # (6 flop, an fma counted as 2), plus 3 fma in the anchor-owner walk and 2 in the target-owner one
        flops = float(B) * P * h * (12 + 10)
        what = "deep distance sum_k w_k tanh((A f)_k + (C g)_k): loss, u, v, dA, dC, dw at B=1024 P=2048 d=768 h=128 bf16"
        extra_roofline = {"bound": "alu", "peak": 157.3, "unit": "TFLOP/s",
                          "peak_note": "published fp32 vector rate (packed fp32); plain fp32 FMAs, which is what this build "
                                       "issues, peak at 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2 = 78.6, and exp2 / "
                                       "reciprocal (2 of the 7-8 instructions per term) run at a quarter of that rate"}
    else:
        xq, xp, r, params = synth.mlp_problem()
        xq, xp, r = xq.to(dev), xp.to(dev), r.to(dev)
        params = {k: v.to(dev) for k, v in params.items()}
        grads = gc.zero_mlp_grads(params)
        G = args.accumulate_group
        res = gc.gc_step_mlp_bf16(xq, xp, r, 32, 32, params, grads=grads, accumulate_group=G)
        step = lambda: gc.gc_step_mlp_bf16(xq, xp, r, 32, 32, params, out=res, accumulate_group=G)   # same buffers every step
        rows = 512 + 1024
        flops = rows * 2.0 * (1024 * 3072 + 3072 * 768) * 4 + 6.0 * 512 * 1024 * 768   # fwd + (re-fwd layer 1, 3 bwd GEMMs) + loss
        what = "Gradient Cache step, MLP 1024-3072-768, B=512 P=1024, chunk 32, accumulate_group %d" % G
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    rec = {"metric": "ms/step", "value": round(ms, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": False, "dtype": "bf16",
           "data": "synthetic", "config": {"workload": args.workload + ": " + what},
           "algorithmic_tflops": round(flops / (ms * 1e-3) / 1e12, 2)}
    if args.workload == "deepdist":
        extra_roofline["achieved"] = rec["algorithmic_tflops"]
        extra_roofline["frac"] = round(rec["algorithmic_tflops"] / extra_roofline["peak"], 4)
        rec["roofline"] = extra_roofline
        rec["dtype"] = "f32"   # the pair arithmetic is fp32 (bf16 storage of the inputs)
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default="config3", choices=["config3", "config2", "config4", "config5", "bidir", "bilinear", "deepdist"],
                    help="config3 (default) is the headline workload; the others print a shorter timing line")
    ap.add_argument("--accumulate-group", type=int, default=1,
                    help="config5 only: sub-batches per launch of Step 3 (1 = the sub-batch is the unit, as in the method)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain elementwise kernel 4 times that reads 1 GiB and writes 1 GiB (known HBM "
                         "traffic, larger than the 256 MB Infinity Cache; scales rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is the one-GPU hot path; --gpus must be 1 (no collectives are part of it)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)

    from paper_2101_06983_amd import binding as gc
    from paper_2101_06983_amd import synth

    dev = torch.device("cuda:0")
    if args.workload != "config3":
        return side_workload(args, gc, synth, dev)
    B, P, d = 4096, 8192, 768
    q, p, r = synth.config3()
    qd, pd, rd = q.to(dev), p.to(dev), r.to(dev)
    out = {k: torch.empty(s, dtype=t, device=dev) for k, (s, t) in
           dict(loss=((1,), torch.float32), dq=((B, d), torch.float32), dp=((P, d), torch.float32)).items()}
    ws = gc.alloc_workspace(gc.gc_workspace_bytes(B, P, d, gc.GC_BF16), dev)
    want = ("loss", "dq", "dp")

    def step():
        gc.gc_loss_and_rep_grad_ex(qd, pd, rd, 1.0, 1.0, 0, want, ws, out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    # timed region: exactly K steps, nothing else on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # per-step durations: the same K steps again, each between two HIP events on the launch stream (torch's current
    # stream, which the binding passes to the library): median and minimum beside the mean of the timed region
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in ev:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in ev)
    step_median, step_min = per_step[len(per_step) // 2], per_step[0]
    # kernel durations: the same K steps again with the library's HIP events at the kernel boundaries (on the launch
    # stream).  Five event records per step cost about 6 % of a step, so they stay out of the timed region above.
    gc.gc_profile_begin(args.steps)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    prof = gc.gc_profile_end()
    assert gc.gc_check_async_error(ws) == gc.GC_OK

    ms = (t1 - t0) * 1e3 / args.steps
    flops_alg = 6.0 * B * P * d
    value = flops_alg / (ms * 1e-3) / 1e12
    # profile marks in fused mode: ms_stats = dQ walk with online statistics, ms_merge = merge of its splits,
    # ms_grad = dP walk, ms_reduce = partial sums + loss sum
    k_alg = 4.0 * B * P * d          # dQ walk: S and G*P, each formed once
    achieved = k_alg / (prof["ms_stats"] * 1e-3) / 1e12
    dp_alg = 2.0 * B * P * d / (prof["ms_grad"] * 1e-3) / 1e12
    kernel_sum = prof["ms_stats"] + prof["ms_merge"] + prof["ms_grad"] + prof["ms_reduce"]
    alg_bytes = (B + P) * d * 2 + (B + P) * d * 4 + B * 4 + 4      # read Q, P, pos_idx; write dq, dp, loss
    tr = counter_traffic()
    traffic = (tr["hbm_read_bytes"] + tr["hbm_write_bytes"]) if tr else None
    rec = {
        "metric": "loss+rep-grad TFLOP/s & ms/step at B=4096,P=8192,d=768 bf16; % MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "ms_per_step_median": round(step_median, 4), "ms_per_step_min": round(step_min, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "config3 large-batch ICT-shaped: B=4096 queries, P=8192 passages, d=768, bf16 storage, "
                               "fp32 accumulate, pos_idx[i]=2i, iid N(0,1/d)", "B": B, "P": P, "d": d,
                   "loss": float(out["loss"].item())},
        "roofline": {"bound": "mfma", "kernel": "grad_online_kernel<768> (dQ walk with online statistics)",
                     "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic,
                     "traffic_from": ("%s (separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                      "measured %s)" % (PROFILE_FILE, tr["measured"])) if tr else None,
                     # fraction of the HBM peak the dominant kernel's counter traffic amounts to over its duration
                     "hbm_frac": round(traffic / (prof["ms_stats"] * 1e-3) / PEAK_HBM_BYTES_PER_S, 4) if tr else None,
                     # ... and the whole step's algorithmic bytes (inputs read once, outputs written once)
                     "hbm_frac_algorithmic_whole_step": round(alg_bytes / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S, 4),
                     "dp_walk": {"kernel": "grad_mfma_kernel<768, false>", "achieved": round(dp_alg, 2),
                                 "frac": round(dp_alg / PEAK_BF16_TFLOPS, 4),
                                 "executed_frac": round(2 * dp_alg / PEAK_BF16_TFLOPS, 4)},
                     "kernel_ms": {"dq_walk_online": round(prof["ms_stats"], 4), "merge_and_dq": round(prof["ms_merge"], 4),
                                   "dp_walk": round(prof["ms_grad"], 4), "partial_sums_and_loss": round(prof["ms_reduce"], 4)},
                     "kernel_ms_from": "HIP events on the launch stream over a second pass of the same %d steps "
                                       "(%.4f ms/step with the events recorded)" % (args.steps, (t3 - t2) * 1e3 / args.steps),
                     "kernel_ms_sum": round(kernel_sum, 4),
                     "whole_path_executed_frac": round(8.0 * B * P * d / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "whole_path_algorithmic_frac": round(6.0 * B * P * d / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(q, p, r, flops_alg)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
