#!/usr/bin/env python3
"""Benchmark of the CD-GraB pair-balancing hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4_resnet18] [--others LIST]

A step is one whole epoch of the hot path on the named synthetic workload: for
each block of Bb flattened pairs the counter-based generator fills the staging
block in HBM (the stand-in for gradients arriving from the workers), then the
dot/Gram pass, the partial reduction, the sign resolver and the apply pass run,
and at the end the permutations and the running sum are written.

`value` is examples balanced per second on the headline workload.  The generator's
time is measured with HIP events on the same stream and reported separately
(`generator_ms_per_step`, `wall_ms_per_step`), never folded into `value`.  The
generator hands each block over as a producer on the same GPU would: written
immediately before the balancer starts, with nothing in between -- `value` is the
consumer-side figure.  A block larger than the last-level cache is written with
streaming (non-temporal) stores, the hint for data that is written once and read by
another kernel; a block that fits the cache with ordinary stores.  Secondary
measurements repeat the epoch with other hand-overs: `generator_with_plain_stores`
(ordinary stores always: a few hundred MB of a large block are then still on their way
from the last-level cache to HBM while the first balancer kernel runs, which slows it),
`generator_with_streaming_stores`, and `inputs_flushed_to_hbm` (the generator flushes
its rows out of the cache inside its own timing: the balancer alone, on rows resident
in HBM).

The line also carries a `workloads` array with the same measurement (fewer steps)
on the other four configurations and on the "next" rows (training epoch, herding
objective, independent balancing), `roofline` for the dominant kernel, and the CPU
oracle timed on a bounded sample of each workload.
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
METRIC = "examples balanced/sec per epoch at m workers x d params"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c4_resnet18",
                    help="headline workload: one of the five configurations, or c2_train / c2_herding / "
                         "c2_independent / syn_herding (the 'next' rows)")
    ap.add_argument("--others", default=None,
                    help="comma-separated workloads for the `workloads` array (default: the other four "
                         "configurations and the next rows when the headline is c4_resnet18, else none)")
    ap.add_argument("--other-steps", type=int, default=3)
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
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU-oracle work per workload, seconds (headline; the others get half; 0: skip)")
    ap.add_argument("--flush-steps", type=int, default=2,
                    help="extra epochs with the generator flushing its rows to HBM first (0: skip)")
    ap.add_argument("--flush-inputs", action="store_true",
                    help="run the timed steps themselves with the generator's flush (then `value` is the "
                         "inputs-resident figure; used for the profiles of the kernels alone)")
    ap.add_argument("--generator-stores", choices=("auto", "plain", "streaming"), default="auto",
                    help="how the synthetic producer writes the rows in the timed steps: ordinary stores, "
                         "non-temporal stores, or (auto) non-temporal for blocks larger than the last-level "
                         "cache and ordinary ones for blocks that fit it")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (a kernel of known HBM traffic, to scale "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--no-profile-step", action="store_true",
                    help="skip the extra per-kernel-timed epoch behind the roofline object")
    return ap.parse_args()


def read_traffic(workload: str):
    """HBM bytes per launch from committed rocprofv3 --pmc summaries
    (profiles/pmc_traffic_<workload>.txt), or None.  Not measured in this run."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    out = {}
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            _, kernel, value = line.split()
            out[kernel] = float(value)
    return out or None


# ---------------------------------------------------------------------------------------------
def cpu_oracle_sample(w, name, rows_src, grads, gpu_signs, d, m, n, bb, seconds, dev):
    """The oracle (one CPU thread, as it stands) on the first pairs of the workload, fed the
    bytes the GPU balanced; the HIP path's signs are imposed, so that the walk stays the
    reference after a decision inside the 1e-9 margin, and every decision is judged."""
    import numpy as np
    import oracle
    N = m * n
    per_pair_s = max(d * 1.1e-9, 2e-6)            # measured: about 1.1 ns per element per pair
    sample_pairs = int(min(N // 2, max(1, seconds / per_pair_s)))
    if N // 2 >= bb and sample_pairs >= bb:
        sample_pairs = (sample_pairs // bb) * bb
    r = np.zeros(d)
    eps_all = np.ascontiguousarray(gpu_signs.T).reshape(-1)[:sample_pairs]
    chunk = max(1, min(sample_pairs, int(2e9 // (8 * d)) or 1))     # <= 2 GB of rows on the host at a time
    if w.kind != "stream":
        z = grads.cpu().numpy()
        flat = z.reshape(m, n // 2, 2, d).transpose(1, 0, 2, 3).reshape(N // 2, 2, d)
    cpu_s, agree, flips = 0.0, True, 0
    for first in range(0, sample_pairs, chunk):
        cnt = min(chunk, sample_pairs - first)
        if w.kind == "stream":
            rows = rows_src.fill_pairs_device(first, cnt, str(dev)).cpu().numpy()
        else:
            rows = np.ascontiguousarray(flat[first:first + cnt])
        want = eps_all[first:first + cnt]
        t0 = time.perf_counter()
        _, tt, nr, nc = oracle.stream_pairs(r, rows, eps_in=want)
        cpu_s += time.perf_counter() - t0
        differs = np.where(tt <= 0, 1, -1) != want
        flips += int(differs.sum())
        agree = agree and not bool((differs & (np.abs(tt) > 1e-9 * nr * nc)).any())
    return {"value": 2 * sample_pairs / cpu_s, "unit": "examples/s", "cores": 1, "kind": "oracle",
            "sample": "first %d pairs (%d examples) of %s, rows copied from HBM; balancing loop only, "
                      "the HIP path's signs imposed" % (sample_pairs, 2 * sample_pairs, name),
            "seconds": cpu_s, "host_cores_available": os.cpu_count(),
            "signs_agree_with_gpu_on_sample": agree, "in_margin_flips_on_sample": flips}


def measure_config(name, args, steps, warmup, cpu_seconds):
    """One of the five configurations through cdgrab_pergrad (softmax) + cdgrab_balance_epoch."""
    import numpy as np
    import torch

    import paper_2302_00845_amd as pkg
    import workloads
    from workloads import hbm_probe, synth

    w = workloads.CONFIGS[name]
    m, n, d = w.m, (args.n or w.n), w.d
    N = m * n
    dev = torch.device("cuda", 0)
    opts = dict(device=0, block_pairs=args.block_pairs, pass1_groups=args.pass1_groups,
                apply_mode=args.apply_mode, gram_mode=args.gram_mode)

    # ------------------------------------------------------------------ inputs
    perm_in = torch.from_numpy(workloads.random_perms(args.seed, m, n)).to(dev)
    gen_fn = gen_ctx = grads = rows_src = None
    pergrad_ms = None
    h = pkg.Handle(timing=1, **opts)
    if w.kind == "stream":
        rows_src = synth.from_workload(w, args.seed, n=n)
        gen_fn, gen_ctx = rows_src.device_callback(str(dev))
        synth.set_input_drain(bool(args.flush_inputs), str(dev))
        synth.set_store_mode(args.generator_stores)
    elif w.kind == "softmax":
        X, y, W = workloads.softmax_problem(args.seed, N)
        Xd, yd, Wd = (torch.from_numpy(a).to(dev) for a in (X, y, W))
        G = torch.empty((N, d), dtype=torch.float32, device=dev)
    else:
        grads = torch.from_numpy(workloads.tiny_epoch(args.seed, m, n, d)).to(dev)

    def step(handle):
        """One pass of the whole hot path; returns its outputs and the event-timed split (ms)."""
        nonlocal grads, pergrad_ms
        if w.kind == "softmax":
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pkg.cdgrab_pergrad(handle, Xd, yd, Wd, G)
            e1.record()
            grads = G.view(m, n, d)
        out = pkg.cdgrab_balance_epoch(handle, m, n, d, grads=grads, gen=gen_fn, gen_ctx=gen_ctx,
                                       perm_in=perm_in, want_r32=True)
        t = handle.timing()                                  # synchronises the stream
        if w.kind == "softmax":
            pergrad_ms = e0.elapsed_time(e1)
            t["balance_ms"] += pergrad_ms                    # the gradient kernel is part of the path
        return out, t

    for _ in range(warmup):
        step(h)
    torch.cuda.synchronize()
    t_wall0 = time.perf_counter()
    splits = []
    for _ in range(steps):
        out, t = step(h)
        splits.append(t)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall0) * 1e3 / max(steps, 1)

    path_ms = float(np.mean([t["balance_ms"] + t["finish_ms"] for t in splits]))
    gen_ms = float(np.mean([t["generator_ms"] for t in splits]))
    bb = splits[-1]["block_pairs"]
    blocks = splits[-1]["blocks"]
    plan = pkg.cdgrab_plan_epoch(m, n, d, block_pairs=args.block_pairs, streamed=w.kind == "stream")
    fused = args.apply_mode == 2 or (args.apply_mode == 0 and bool(plan["fused_apply"]))
    ahead = args.gram_mode == 2 or (args.gram_mode == 0 and args.apply_mode == 0 and bool(plan["gram_ahead"]))
    fused = fused and not ahead
    # whole balancer against the roofline: 8d + 12 d / Bb bytes per example with separate passes
    # (each row twice; double running sum read twice, written once per block), 8d + 8 d / Bb with the
    # fused launch, 12d + 8 d / Bb with the Gram matrices ahead (rows read three times)
    bytes_per_example = (12.0 * d + 8.0 * d / bb) if ahead else (8.0 * d + (8.0 if fused else 12.0) * d / bb)
    if w.kind == "softmax":
        bytes_per_example += 4.0 * d + 4.0 * 785              # the gradient kernel writes the row, reads x
    res = {
        "workload": name, "m": m, "n": n, "d": d, "examples": N, "steps": steps, "warmup": warmup,
        "value": N / (path_ms * 1e-3), "unit": "examples/s", "ms_per_step": path_ms,
        "block_pairs": bb, "blocks": blocks, "input": w.kind, "fused_apply": fused, "gram_ahead": ahead,
        "inputs": ("handed over by the generator right before each block, not flushed; store mode %s"
                   % args.generator_stores if w.kind == "stream" and not args.flush_inputs
                   else "resident in HBM"),
        "generator_ms_per_step": gen_ms, "wall_ms_per_step": wall_ms,
        "bytes_per_example": bytes_per_example,
        "balancer_achieved_GBs": bytes_per_example * N / (path_ms * 1e-3) / 1e9,
    }
    res["balancer_hbm_frac"] = res["balancer_achieved_GBs"] / HBM_PEAK_GBS
    if pergrad_ms is not None:
        res["pergrad_ms_per_step"] = pergrad_ms
        res["pergrad_write_GBs"] = 4.0 * d * N / (pergrad_ms * 1e-3) / 1e9
    if w.kind != "stream" and d < (1 << 18):
        res["note"] = "short rows: bound by the chain of dependent launches, not by bytes (no roofline claim)"

    # ------------------------------------------------------------------ per-kernel timing (one more epoch)
    if not args.no_profile_step:
        hp = pkg.Handle(timing=2, **opts)
        _, tp = step(hp)
        avg_pairs = (N // 2) / blocks
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
        kernels = {}
        for kname, ms, nbytes in per_kernel:
            avg_ms = ms / blocks
            kernels[kname] = {"avg_launch_ms": avg_ms, "algorithmic_bytes_per_launch": nbytes,
                              "achieved_GBs": nbytes / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else None}
        kernels["reduce_partials"] = {"avg_launch_ms": tp["reduce_ms"] / blocks}
        kernels["resolve_signs"] = {"avg_launch_ms": tp["resolve_ms"] / blocks}
        dom = max((k[0] for k in per_kernel), key=lambda k: kernels[k]["avg_launch_ms"])
        traffic = read_traffic(name)
        res["roofline"] = {
            "kernel": dom, "bound": "hbm", "achieved": kernels[dom]["achieved_GBs"], "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": kernels[dom]["achieved_GBs"] / HBM_PEAK_GBS,
            "traffic": (traffic or {}).get(dom),
            "traffic_source": ("profiles/pmc_traffic_%s.txt (rocprofv3 --pmc on rows resident in HBM; "
                               "not measured in this run)" % name) if traffic else None,
            "avg_launch_ms": kernels[dom]["avg_launch_ms"],
            "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes_per_launch"]}
        res["kernels"] = kernels
        hp.close()

    # ------------------------------------------------------------------ other ways of handing rows over
    def extra_epochs(count):
        step(h)
        runs = [step(h)[1] for _ in range(count)]
        ms = float(np.mean([t["balance_ms"] + t["finish_ms"] for t in runs]))
        r = {"value": N / (ms * 1e-3), "ms_per_step": ms, "steps": count,
             "balancer_hbm_frac": bytes_per_example * N / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
             "generator_ms_per_step": float(np.mean([t["generator_ms"] for t in runs]))}
        if not args.no_profile_step:
            hq = pkg.Handle(timing=2, **opts)
            _, tq = step(hq)
            hq.close()
            r["kernels_avg_launch_ms"] = {"pass1_dots_gram": tq["pass1_ms"] / blocks,
                                          "pass2_apply": tq["pass2_ms"] / blocks}
            if not fused and not ahead and tq["pass1_ms"] > 0 and tq["pass2_ms"] > 0:
                pairs_blk = (N // 2) / blocks
                r["kernels_hbm_frac"] = {
                    "pass1_dots_gram": (8.0 * pairs_blk * d + 8.0 * d) / (tq["pass1_ms"] / blocks * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "pass2_apply": (8.0 * pairs_blk * d + 16.0 * d) / (tq["pass2_ms"] / blocks * 1e-3) / 1e9 / HBM_PEAK_GBS}
        return r

    if w.kind == "stream" and not args.flush_inputs and args.flush_steps > 0:
        # the generator flushing its rows out of the last-level cache before it hands them over
        synth.set_input_drain(True, str(dev))
        res["inputs_flushed_to_hbm"] = extra_epochs(args.flush_steps)
        synth.set_input_drain(False, str(dev))
        # the generator writing with the store flavour the timed steps did not use
        used = args.generator_stores
        if used == "auto":   # the generator streams blocks larger than 384 MB (workloads/synth_hip.hip)
            used = "streaming" if 8.0 * bb * d > (384 << 20) else "plain"
        other = "plain" if used == "streaming" else "streaming"
        synth.set_store_mode(other)
        res["generator_with_%s_stores" % other] = extra_epochs(args.flush_steps)
        synth.set_store_mode(args.generator_stores)
        res["inputs"] += " (%s stores)" % used

    if cpu_seconds > 0:
        res["cpu_baseline"] = cpu_oracle_sample(w, name, rows_src, grads, out["signs"].cpu().numpy(), d, m, n,
                                                bb, cpu_seconds, dev)
    if res.get("roofline") is not None:
        # practical ceiling: a plain streaming read of a buffer the size of one block's rows
        ceiling = hbm_probe.read_bandwidth(int(min(max(8.0 * bb * d, 1 << 28), 3 << 30)))
        res["roofline"]["plain_read_GBs"] = ceiling
        res["roofline"]["frac_of_plain_read"] = res["roofline"]["achieved"] / ceiling
    h.close()
    del h
    torch.cuda.empty_cache()
    return res


def measure_synthetic_herding(args, steps, warmup):
    """The parallel herding objective on the vectors of the paper's synthetic study (App. E):
    10^6 unit vectors in 16 dimensions (64-byte rows), 100 workers, random orders."""
    import numpy as np
    import torch

    import paper_2302_00845_amd as pkg
    import workloads

    N, d, m = 1_000_000, 16, 100
    n = N // m
    dev = torch.device("cuda", 0)
    z = torch.from_numpy(workloads.herding_vectors(args.seed, N, d).reshape(m, n, d)).to(dev)
    perm = torch.from_numpy(workloads.random_perms(args.seed, m, n)).to(dev)
    h = pkg.Handle(device=0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    times = []
    for it in range(warmup + steps):
        e0.record()
        b = pkg.cdgrab_herding_bound(h, z, perm)
        e1.record()
        torch.cuda.synchronize()
        if it >= warmup:
            times.append(e0.elapsed_time(e1))
    ms = float(np.mean(times))
    gbs = 2.0 * N * d * 4 / (ms * 1e-3) / 1e9          # every row is read twice
    res = {"workload": "syn_herding", "metric": "examples/sec through the parallel herding objective",
           "m": m, "n": n, "d": d, "examples": N, "steps": steps, "warmup": warmup, "value": N / (ms * 1e-3),
           "unit": "examples/s", "ms_per_step": ms, "dtype": "f64", "herding_bound": float(b.cpu()[0]),
           "roofline": {"kernel": "herding_segment_sums + herding_prefix_max", "bound": "hbm", "achieved": gbs,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": None},
           "note": "128 MB of traffic in all: bound by the three dependent launches, not by bytes"}
    h.close()
    return res


def measure_next_row(name, args, steps, warmup):
    """The rows built after the hot path, on config 2's problem: one training epoch of the softmax
    model (`c2_train`), one evaluation of the parallel herding objective on its gradients
    (`c2_herding`), and uncoordinated per-worker balancing with m = 64 (`c2_independent`)."""
    import numpy as np
    import torch

    import paper_2302_00845_amd as pkg
    import workloads

    if name == "syn_herding":
        return measure_synthetic_herding(args, steps, warmup)

    w = workloads.CONFIGS["c2_softmax"]
    m, n, d = w.m, (args.n or w.n), w.d
    if name == "c2_independent":
        m, n = 64, 936                                       # 59 904 of the 60 000 examples, 64 workers
    N = m * n
    dev = torch.device("cuda", 0)
    X, y, W0 = workloads.softmax_problem(args.seed, N)
    Xd, yd = torch.from_numpy(X).to(dev), torch.from_numpy(y).to(dev)
    perm = torch.from_numpy(workloads.random_perms(args.seed, m, n)).to(dev)
    h = pkg.Handle(device=0, timing=1)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    extra, roofline, dtype = {}, None, "f64"
    if name == "c2_train":
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
        for _ in range(warmup):
            step()
        runs = [step() for _ in range(steps)]
        extra = {"steps_ms": float(np.mean([r[1]["generator_ms"] for r in runs])),
                 "balance_ms": float(np.mean([r[1]["balance_ms"] for r in runs])),
                 "mean_loss_by_epoch": [r[2] for r in runs],
                 "note": "steps_ms = 2 launches per optimisation step (deltas; rows + mean + SGD update)"}
        metric, dtype = "training examples/sec (softmax regression under CD-GraB, one epoch)", "f32"
    else:
        G = pkg.cdgrab_pergrad(h, Xd, yd, torch.from_numpy(W0).to(dev)).view(m, n, d)
        if name == "c2_herding":
            def step():
                e0.record()
                b = pkg.cdgrab_herding_bound(h, G, perm)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1), float(b.cpu()[0])
            metric = "examples/sec through the parallel herding objective"
            nbytes = 2.0 * N * d * 4                  # every row is read in pass A and again in pass C
            kname = "herding_segment_sums + herding_prefix_max"
        else:
            def step():
                e0.record()
                pkg.cdgrab_balance_epoch_independent(h, G, perm)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1), None
            metric = "examples/sec through m independent pair-balancing walks (ID-GraB (PairBal))"
            nbytes, kname = None, None
        for _ in range(warmup):
            step()
        runs = [step() for _ in range(steps)]
        if nbytes is not None:
            gbs = nbytes / (float(np.mean([r[0] for r in runs])) * 1e-3) / 1e9
            roofline = {"kernel": kname, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": gbs / HBM_PEAK_GBS, "traffic": None}
            extra = {"herding_bound": runs[-1][1]}
    ms = float(np.mean([r[0] for r in runs]))
    res = {"workload": name, "metric": metric, "m": m, "n": n, "d": d, "examples": N, "steps": steps,
           "warmup": warmup, "value": N / (ms * 1e-3), "unit": "examples/s", "ms_per_step": ms, "dtype": dtype,
           "roofline": roofline}
    res.update(extra)
    h.close()
    del h
    torch.cuda.empty_cache()
    return res


NEXT_ROWS = ("c2_train", "c2_herding", "c2_independent", "syn_herding")


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the balancer on ONE GPU (the m workers are a batch axis); "
              "--gpus %d is not supported, run with --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import workloads
    from workloads import hbm_probe

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        hbm_probe.copy_bandwidth(1 << 30)

    def run(name, steps, warmup, cpu_seconds):
        if name in NEXT_ROWS:
            return measure_next_row(name, args, steps, warmup)
        return measure_config(name, args, steps, warmup, cpu_seconds)

    head = run(args.workload, args.steps, args.warmup, args.cpu_seconds)
    if args.others is None:
        others = ([c for c in workloads.CONFIGS if c != "c4_resnet18"] + list(NEXT_ROWS)
                  if args.workload == "c4_resnet18" and not args.n else [])
    else:
        others = [s for s in args.others.split(",") if s]
    array = [run(name, args.other_steps, 1, args.cpu_seconds / 2) for name in others]

    line = {
        "metric": head.get("metric", METRIC),
        "value": head["value"], "unit": "examples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head.get("dtype", "f64"), "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "m", "n", "d", "examples", "block_pairs", "blocks", "input",
                                        "fused_apply", "gram_ahead", "inputs") if k in head},
    }
    line["config"].update({"rows_dtype": "f32", "parallelism": "1 GPU, m workers as a batch axis"})
    for k in ("generator_ms_per_step", "wall_ms_per_step", "balancer_achieved_GBs", "balancer_hbm_frac",
              "bytes_per_example", "inputs_flushed_to_hbm", "generator_with_plain_stores",
              "generator_with_streaming_stores", "pergrad_ms_per_step", "pergrad_write_GBs", "note",
              "steps_ms", "balance_ms", "mean_loss_by_epoch", "herding_bound"):
        if k in head:
            line[k] = head[k]
    if "generator_ms_per_step" in head:
        line["value_including_generator"] = head["examples"] / (
            (head["ms_per_step"] + head["generator_ms_per_step"]) * 1e-3)
    line["roofline"] = head.get("roofline")
    line["kernels"] = head.get("kernels")
    line["cpu_baseline"] = head.get("cpu_baseline")
    line["workloads"] = array
    # Everything measured goes to stderr as one JSON document; stdout gets the ONE line of the
    # contract, kept short (a few KB): the headline in full, the other workloads as compact entries.
    print("bench detail: " + json.dumps(line), file=sys.stderr)
    print(json.dumps(compact_line(line)))


def _sig(x, digits=6):
    """Floats rounded to `digits` significant digits, recursively (shorter JSON)."""
    if isinstance(x, float):
        return float("%.*g" % (digits, x))
    if isinstance(x, dict):
        return {k: _sig(v, digits) for k, v in x.items()}
    if isinstance(x, (list, tuple)):
        return [_sig(v, digits) for v in x]
    return x


def compact_line(line):
    out = dict(line)
    if out.get("roofline"):
        out["roofline"] = {k: v for k, v in out["roofline"].items() if k != "traffic_source"}
        out["roofline"]["traffic_note"] = "from profiles/ (rocprofv3 --pmc), not measured in this run"
    for k in ("bytes_per_example", "balancer_achieved_GBs"):
        out.pop(k, None)
    for k in ("inputs_flushed_to_hbm", "generator_with_plain_stores", "generator_with_streaming_stores"):
        if out.get(k):
            out[k] = {a: b for a, b in out[k].items() if a in ("value", "ms_per_step", "balancer_hbm_frac",
                                                               "kernels_avg_launch_ms", "kernels_hbm_frac")}
    if out.get("kernels"):
        out["kernels"] = {k: {"avg_launch_ms": v["avg_launch_ms"]} for k, v in out["kernels"].items()}
    if out.get("cpu_baseline"):
        out["cpu_baseline"] = {k: v for k, v in out["cpu_baseline"].items() if k != "host_cores_available"}
    small = []
    for w in out.get("workloads") or []:
        e = {"workload": w["workload"], "m": w["m"], "n": w["n"], "d": w["d"], "value": w["value"],
             "ms_per_step": w["ms_per_step"]}
        if "balancer_hbm_frac" in w:
            e["balancer_hbm_frac"] = w["balancer_hbm_frac"]
        if w.get("inputs_flushed_to_hbm"):
            e["flushed_hbm_frac"] = w["inputs_flushed_to_hbm"]["balancer_hbm_frac"]
        if w.get("roofline"):
            e["kernel"] = w["roofline"]["kernel"]
            e["frac"] = w["roofline"]["frac"]
            if "avg_launch_ms" in w["roofline"]:
                e["avg_launch_ms"] = w["roofline"]["avg_launch_ms"]
        if w.get("cpu_baseline"):
            c = w["cpu_baseline"]
            e["cpu_baseline"] = {"value": c["value"], "cores": c["cores"], "seconds": c["seconds"],
                                 "signs_agree": c["signs_agree_with_gpu_on_sample"]}
        if "note" in w and "launch" in w["note"]:
            e["bound"] = "launch chain"
        small.append(e)
    out["workloads"] = small
    return _sig(out)


if __name__ == "__main__":
    main()
