#!/usr/bin/env python3
"""Benchmark of the CD-GraB pair-balancing hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4_resnet18]

A step is one whole epoch of the hot path on the named synthetic workload: for
each block of Bb flattened pairs the counter-based generator fills the staging
block in HBM (the stand-in for gradients arriving from the workers), then the
dot/Gram pass, the partial reduction, the sign resolver and the apply pass run,
and at the end the permutations and the running sum are written.

`value` is examples balanced per second with each block's rows already resident
in HBM when its timed region starts: the generator's time is measured with HIP
events on the same stream and reported separately (`generator_ms_per_step`,
`wall_ms_per_step`), never folded into `value`.

Prints one JSON line (metric, roofline of the dominant kernel, CPU-oracle
baseline on a bounded sample of the same workload).
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

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c4_resnet18")
    ap.add_argument("--block-pairs", type=int, default=0)
    ap.add_argument("--pass1-groups", type=int, default=0)
    ap.add_argument("--apply-mode", type=int, default=0,
                    help="0: library's choice by row length; 1: separate apply launch per block; "
                         "2: apply fused into the next block's dot/Gram launch")
    ap.add_argument("--gram-mode", type=int, default=0,
                    help="dense input: 0 library's choice; 1 every block computes its own Gram "
                         "matrix; 2 Gram matrices of many blocks ahead in one launch")
    ap.add_argument("--n", type=int, default=0, help="override rows per worker (shorter epoch)")
    ap.add_argument("--seed", type=int, default=2302)
    ap.add_argument("--cpu-sample-pairs", type=int, default=-1,
                    help="pairs of the workload the CPU oracle is timed on (-1: sized for ~15 s, 0: skip)")
    ap.add_argument("--no-input-drain", action="store_true",
                    help="do not let the input generator drain its written rows out of the last-level "
                         "cache before the balancer's timed region")
    ap.add_argument("--skip-undrained-step", action="store_true",
                    help="do not run the extra epoch that measures the balancer without the input drain")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (a kernel of known HBM traffic, to scale "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--no-profile-step", action="store_true",
                    help="skip the extra per-kernel-timed epoch behind the roofline object")
    return ap.parse_args()


def read_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from committed rocprofv3 --pmc
    summaries (profiles/pmc_traffic_<workload>.txt), or None."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    out = {}
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            _, kernel, value = line.split()
            out[kernel] = float(value)
    return out or None


def bench_next_rows(args):
    """Secondary measurements (not the headline): one training epoch of the softmax model
    (`c2_train`) or one evaluation of the parallel herding objective on config 2's gradients
    (`c2_herding`).  Same JSON skeleton; `roofline` only where a bound applies."""
    import numpy as np
    import torch

    import paper_2302_00845_amd as pkg
    import workloads

    w = workloads.CONFIGS["c2_softmax"]
    m, n, d = w.m, (args.n or w.n), w.d
    N = m * n
    dev = torch.device("cuda", 0)
    X, y, W0 = workloads.softmax_problem(args.seed, N)
    Xd, yd = torch.from_numpy(X).to(dev), torch.from_numpy(y).to(dev)
    perm = torch.from_numpy(workloads.random_perms(args.seed, m, n)).to(dev)
    h = pkg.Handle(device=0, timing=1)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    extra = {}
    if args.workload == "c2_train":
        Wd = torch.from_numpy(W0.copy()).to(dev)
        vel = torch.zeros(Wd.numel(), dtype=torch.float32, device=dev)
        Xw, yw = Xd.view(m, n, -1), yd.view(m, n)

        def step():
            e0.record()
            out = pkg.cdgrab_train_epoch_softmax(h, Xw, yw, Wd, perm_in=perm, velocity=vel, lr=0.001,
                                                 momentum=0.9)
            e1.record()
            t = h.timing()
            return e0.elapsed_time(e1), t, float(out["loss"].mean())
        for _ in range(args.warmup):
            step()
        runs = [step() for _ in range(args.steps)]
        ms = float(np.mean([r[0] for r in runs]))
        extra = {"steps_ms": float(np.mean([r[1]["generator_ms"] for r in runs])),
                 "balance_ms": float(np.mean([r[1]["balance_ms"] for r in runs])),
                 "mean_loss_by_epoch": [r[2] for r in runs],
                 "note": "steps_ms = 2 launches per optimisation step (deltas; rows + mean + SGD update)"}
        metric, roofline = "training examples/sec (softmax regression under CD-GraB, one epoch)", None
    else:
        G = pkg.cdgrab_pergrad(h, Xd, yd, torch.from_numpy(W0).to(dev)).view(m, n, d)

        def step():
            e0.record()
            b = pkg.cdgrab_herding_bound(h, G, perm)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1), float(b.cpu()[0])
        for _ in range(args.warmup):
            step()
        runs = [step() for _ in range(args.steps)]
        ms = float(np.mean([r[0] for r in runs]))
        nbytes = 2.0 * N * d * 4                      # every row is read in pass A and again in pass C
        gbs = nbytes / (ms * 1e-3) / 1e9
        roofline = {"kernel": "herding_segment_sums + herding_prefix_max", "bound": "hbm", "achieved": gbs,
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None}
        extra = {"herding_bound": runs[-1][1]}
        metric = "examples/sec through the parallel herding objective"
    line = {"metric": metric, "value": N / (ms * 1e-3), "unit": "examples/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32" if args.workload == "c2_train" else "f64",
            "data": "synthetic", "config": {"workload": args.workload, "m": m, "n": n, "d": d, "examples": N},
            "roofline": roofline, "cpu_baseline": None}
    line.update(extra)
    print(json.dumps(line))
    h.close()


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the balancer on ONE GPU (the m workers are a batch axis); "
              "--gpus %d is not supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2302_00845_amd as pkg
    import workloads
    from workloads import hbm_probe, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.workload in ("c2_train", "c2_herding"):
        return bench_next_rows(args)
    w = workloads.CONFIGS[args.workload]
    m, n, d = w.m, (args.n or w.n), w.d
    plan0 = pkg.cdgrab_plan_epoch(m, n, d, streamed=workloads.CONFIGS[args.workload].kind == "stream")
    fused = args.apply_mode == 2 or (args.apply_mode == 0 and bool(plan0["fused_apply"]))
    # dense input with short rows: Gram matrices of many blocks ahead in one launch
    ahead = workloads.CONFIGS[args.workload].kind != "stream" and plan0["blocks"] >= 2 and (
        args.gram_mode == 2 or (args.gram_mode == 0 and args.apply_mode == 0 and bool(plan0["gram_ahead"])))
    N = m * n
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    # ------------------------------------------------------------------ inputs
    perm_in = torch.from_numpy(workloads.random_perms(args.seed, m, n)).to(dev)
    gen_fn = gen_ctx = grads = rows_src = None
    pergrad_ms = None
    h = pkg.Handle(device=0, block_pairs=args.block_pairs, timing=1, pass1_groups=args.pass1_groups,
                   apply_mode=args.apply_mode, gram_mode=args.gram_mode)
    if w.kind == "stream":
        rows_src = synth.from_workload(w, args.seed, n=n)
        gen_fn, gen_ctx = rows_src.device_callback(str(dev))
        synth.set_input_drain(not args.no_input_drain, str(dev))
    elif w.kind == "softmax":
        X, y, W = workloads.softmax_problem(args.seed, N)
        Xd, yd, Wd = (torch.from_numpy(a).to(dev) for a in (X, y, W))
        G = torch.empty((N, d), dtype=torch.float32, device=dev)
    else:
        grads = torch.from_numpy(workloads.tiny_epoch(args.seed, m, n, d)).to(dev)

    def step():
        """One pass of the whole hot path; returns the event-timed split (ms)."""
        nonlocal grads, pergrad_ms
        if w.kind == "softmax":
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pkg.cdgrab_pergrad(h, Xd, yd, Wd, G)
            e1.record()
            grads = G.view(m, n, d)
        out = pkg.cdgrab_balance_epoch(h, m, n, d, grads=grads, gen=gen_fn, gen_ctx=gen_ctx,
                                       perm_in=perm_in, want_r32=True)
        t = h.timing()                                       # synchronises the stream
        if w.kind == "softmax":
            pergrad_ms = e0.elapsed_time(e1)
            t["balance_ms"] += pergrad_ms                    # the gradient kernel is part of the path
        return out, t

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    splits = []
    for _ in range(args.steps):
        out, t = step()
        splits.append(t)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall0) * 1e3 / max(args.steps, 1)

    path_ms = float(np.mean([t["balance_ms"] + t["finish_ms"] for t in splits]))
    gen_ms = float(np.mean([t["generator_ms"] for t in splits]))
    bb = splits[-1]["block_pairs"]
    blocks = splits[-1]["blocks"]
    value = N / (path_ms * 1e-3)

    # ------------------------------------------------------------------ roofline (dominant kernel)
    roofline = None
    kernels = {}
    if not args.no_profile_step:
        hp = pkg.Handle(device=0, block_pairs=args.block_pairs, timing=2, pass1_groups=args.pass1_groups,
                        apply_mode=args.apply_mode, gram_mode=args.gram_mode)
        if w.kind == "softmax":
            pkg.cdgrab_pergrad(hp, Xd, yd, Wd, G)
        pkg.cdgrab_balance_epoch(hp, m, n, d, grads=grads, gen=gen_fn, gen_ctx=gen_ctx, perm_in=perm_in)
        tp = hp.timing()
        pairs = N // 2
        avg_pairs = pairs / blocks
        if ahead:
            # per block: its share of the batched Gram launch (rows once) and the resolve + apply + dots
            # launch (rows of this block and of the previous one, running sum read and written)
            per_kernel = (("gram_batched+resolve_dots_apply", tp["pass1_ms"] + tp["pass2_ms"],
                           24.0 * avg_pairs * d + 16.0 * d),)
        elif not fused:
            # algorithmic bytes per launch: both rows of every pair in the block (fp32) plus the
            # double running sum (read in pass 1; read and written in pass 2)
            per_kernel = (("pass1_dots_gram", tp["pass1_ms"], 8.0 * avg_pairs * d + 8.0 * d),
                          ("pass2_apply", tp["pass2_ms"], 8.0 * avg_pairs * d + 16.0 * d))
        else:
            # fused launch: the rows of the previous block (apply) and of this block (dots + Gram),
            # the running sum read once and written once.  The epoch's first launch has nothing to
            # apply and its last block is applied by one stand-alone launch: together one more
            # fused launch's worth of bytes, so all streaming time is divided by the block count.
            per_kernel = (("pass1_dots_gram+apply", tp["pass1_ms"] + tp["pass2_ms"],
                           16.0 * avg_pairs * d + 16.0 * d),)
        for name, ms, nbytes in per_kernel:
            avg_ms = ms / blocks
            kernels[name] = {"avg_launch_ms": avg_ms, "algorithmic_bytes_per_launch": nbytes,
                             "achieved_GBs": nbytes / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else None}
        kernels["reduce_partials"] = {"avg_launch_ms": tp["reduce_ms"] / blocks}
        kernels["resolve_signs"] = {"avg_launch_ms": tp["resolve_ms"] / blocks}
        dom = max((k[0] for k in per_kernel), key=lambda k: kernels[k]["avg_launch_ms"])
        traffic = read_traffic(args.workload)
        roofline = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["achieved_GBs"],
                    "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": kernels[dom]["achieved_GBs"] / HBM_PEAK_GBS,
                    "traffic": (traffic or {}).get(dom),
                    "avg_launch_ms": kernels[dom]["avg_launch_ms"],
                    "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes_per_launch"]}
        hp.close()
    # practical ceiling: a plain streaming read of a buffer the size of one block's rows
    read_ceiling = hbm_probe.read_bandwidth(int(min(max(8.0 * bb * d, 1 << 28), 3 << 30)))
    if roofline is not None:
        roofline["plain_read_GBs"] = read_ceiling
        roofline["frac_of_plain_read"] = roofline["achieved"] / read_ceiling
    # whole balancer against the roofline: 8d + 12 d / Bb bytes per example with separate passes
    # (running sum read twice, written once per block), 8d + 8 d / Bb with the fused launch
    bytes_per_example = 8.0 * d + (8.0 if fused else 12.0) * d / bb
    if ahead:  # rows read three times (Grams ahead, then as this block and as the previous one)
        bytes_per_example = 12.0 * d + 8.0 * d / bb
    balancer_gbs = bytes_per_example * N / (path_ms * 1e-3) / 1e9

    # the same epoch without the generator's cache drain (its write-back then lands in pass 1)
    undrained = None
    if w.kind == "stream" and not args.no_input_drain and not args.skip_undrained_step:
        synth.set_input_drain(False, str(dev))
        _, tu = step()
        synth.set_input_drain(True, str(dev))
        u_ms = tu["balance_ms"] + tu["finish_ms"]
        undrained = {"value": N / (u_ms * 1e-3), "ms_per_step": u_ms,
                     "balancer_hbm_frac": bytes_per_example * N / (u_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "generator_ms_per_step": tu["generator_ms"]}

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu_baseline = None
    sample_pairs = args.cpu_sample_pairs
    if sample_pairs < 0:
        # about 12 s of single-threaded oracle work (measured: ~1.2 ns per element per pair)
        per_pair_s = max(d * 1.2e-9, 1e-6)
        sample_pairs = int(min(N // 2, max(bb, 12.0 / per_pair_s)))
        if N // 2 >= bb:
            sample_pairs = max(bb, (sample_pairs // bb) * bb)
    if sample_pairs > 0:
        import oracle
        r = np.zeros(d)
        gpu_eps = out["signs"].cpu().numpy().T.reshape(-1)[:sample_pairs]
        cpu_s, agree, replayed = 0.0, True, False
        chunk = max(1, min(sample_pairs, int(4e9 // (8 * d)) or 1))     # <= 4 GB of rows on the host at a time
        if w.kind != "stream":
            z = grads.cpu().numpy()
            flat = z.reshape(m, n // 2, 2, d).transpose(1, 0, 2, 3).reshape(N // 2, 2, d)
        for first in range(0, sample_pairs, chunk):
            cnt = min(chunk, sample_pairs - first)
            if w.kind == "stream":
                rows = rows_src.fill_pairs_device(first, cnt, str(dev)).cpu().numpy()
            else:
                rows = np.ascontiguousarray(flat[first:first + cnt])
            # once a sign inside the 1e-9 margin differs, the oracle follows the GPU's signs
            want = gpu_eps[first:first + cnt]
            t0 = time.perf_counter()
            eps, tt, nr, nc = oracle.stream_pairs(r, rows, eps_in=want if replayed else None)
            cpu_s += time.perf_counter() - t0
            if not replayed and not np.array_equal(eps, want):
                # redo this chunk as a replay (untimed) and judge by the margin rule
                replayed = True
                bad_idx = int(np.nonzero(eps != want)[0][0])
                r_prev = r.copy()
                # rewind: subtract what the free run added after the first difference
                diffs = rows[:, 1].astype(np.float64) - rows[:, 0].astype(np.float64)
                r = r_prev - (eps[bad_idx:, None] * diffs[bad_idx:]).sum(0)
                eps2, t2, nr2, nc2 = oracle.stream_pairs(r, rows[bad_idx:], eps_in=want[bad_idx:])
                tt, nr, nc = t2, nr2, nc2
                eps = want[bad_idx:]
                want = want[bad_idx:]
            if replayed:
                bad = (np.where(tt <= 0, 1, -1) != want) & (np.abs(tt) > 1e-9 * nr * nc)
                agree = agree and not bool(bad.any())
        cpu_baseline = {"value": 2 * sample_pairs / cpu_s, "unit": "examples/s", "cores": 1,
                        "kind": "oracle",
                        "sample": "first %d flattened pairs (%d examples) of %s, rows copied from HBM in "
                                  "chunks of %d pairs; balancing loop only" % (
                                      sample_pairs, 2 * sample_pairs, args.workload, chunk),
                        "seconds": cpu_s, "host_cores_available": os.cpu_count(),
                        "signs_agree_with_gpu_on_sample": agree}

    line = {
        "metric": "examples balanced/sec per epoch at m workers x d params",
        "value": value, "unit": "examples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": path_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": args.workload, "m": m, "n": n, "d": d, "examples": N,
                   "block_pairs": bb, "blocks": blocks, "input": w.kind,
                   "fused_apply": fused and not ahead, "gram_ahead": ahead,
                   "input_drain": bool(w.kind == "stream" and not args.no_input_drain),
                   "rows_dtype": "f32", "parallelism": "1 GPU, m workers as a batch axis"},
        "generator_ms_per_step": gen_ms, "wall_ms_per_step": wall_ms,
        "value_including_generator": N / ((path_ms + gen_ms) * 1e-3),
        "balancer_achieved_GBs": balancer_gbs, "balancer_hbm_frac": balancer_gbs / HBM_PEAK_GBS,
        "bytes_per_example": bytes_per_example,
        "without_input_drain": undrained,
        "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu_baseline,
    }
    if pergrad_ms is not None:
        line["pergrad_ms_per_step"] = pergrad_ms
    print(json.dumps(line))
    h.close()


if __name__ == "__main__":
    main()
