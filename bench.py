#!/usr/bin/env python3
"""Throughput of the dynamic-batching hot path on one MI355X.

A step is one pass of the whole path over one global batch: per-worker forward/backward on
the ragged split b[K], weighted aggregation, SGD update (with the 16-bit weight refresh), and
the host controller that resizes b[K] from the synthetic iteration times.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps 200] [--warmup 20] [--workload 4] [--no-cpu-baseline]
                    [--no-other-workloads]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16": 2500.0, "fp32": 157.3, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, GB/s

# Bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE (scaled by a plain copy of known
# size; profiles/bench_workload4_rocprofv3.md), valid for workload 4 and only as long as the
# kernel source they were taken from is unchanged (sha1 of the file, first 12 hex digits).
# "gemm_wgrad" on workload 4 is the 256 x 128-tile aggregating kernel alone (three launches per
# step); the output layer's 128 x 128-tile launch is the class "gemm_wgrad_small_tiles".
MEASURED_TRAFFIC = {
    "gemm_wgrad": {"bytes_per_launch": 1.5754e9, "source": "paper_2305_12213_amd/csrc/gemm.hip",
                   "sha1": "31cdb370ab36"},
    # one launch per step: the four weight matrices with their 16-bit copies, and the biases
    "sgd_update": {"bytes_per_launch": 8.837e8,
                   "source": "paper_2305_12213_amd/csrc/kernels_update.hip", "sha1": "18ce68426c28"},
}


def measured_traffic(kernel, workload):
    import hashlib
    m = MEASURED_TRAFFIC.get(kernel)
    if not m or workload != 4:
        return None
    try:
        sha = hashlib.sha1(open(os.path.join(ROOT, m["source"]), "rb").read()).hexdigest()[:12]
    except OSError:
        return None
    return m["bytes_per_launch"] if sha == m["sha1"] else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the four smaller workloads")
    ap.add_argument("--aggregate", choices=["gradient", "update", "pass"], default="gradient",
                    help="where the weighted aggregation runs: inside the weight-gradient kernel "
                         "(dynb_forward_backward_aggregate, default), inside the update kernel "
                         "(dynb_model_aggregate_update), or as a pass of its own")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run one plain device copy of MIB mebibytes (a dispatch of known "
                         "traffic to scale FETCH_SIZE / WRITE_SIZE counter readings by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (K workers are simulated on it); "
                 "--gpus must be 1")

    import numpy as np
    import torch
    from paper_2305_12213_amd import binding, synth

    binding.load()
    torch.cuda.set_device(0)
    cfg = synth.config(args.workload)
    spec, seed = cfg["spec"], synth.BASE_SEED + cfg["index"]
    G, K = cfg["global_batch"], cfg["K"]
    n_batches = min(args.warmup + args.steps, 16)   # distinct global batches, cycled through

    model = binding.Model(spec)
    P, Pp = model.num_params(), model.padded_params()
    params = torch.from_numpy(synth.flatten_params(synth.init_params(spec, cfg["init"], seed), 256)).cuda()
    nbytes = model.workspace_bytes(G, K)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    model.bind(params, ws, nbytes, G, K)
    grads = torch.empty(K, Pp, device="cuda")
    out = torch.empty(Pp, device="cuda")
    velocity = torch.zeros(Pp, device="cuda") if cfg["momentum"] else None
    opt = binding.make_optimizer("momentum" if cfg["momentum"] else "sgd", lr=cfg["lr"],
                                 momentum=cfg["momentum"])
    xs, ys = [], []
    for s in range(n_batches):          # a fresh global batch per step, resident in HBM
        x, y = synth.make_batch(spec, cfg["x_dist"], G, seed, s)
        xs.append(torch.from_numpy(x).cuda()); ys.append(torch.from_numpy(y).cuda())
    torch.cuda.synchronize()

    state = {"b": list(cfg["b0"]), "step": 0, "trace": []}

    def one_step():
        s = state["step"]
        b = state["b"]
        if args.aggregate == "pass":          # three calls: gradients, aggregate, update
            binding.forward_backward(model, xs[s % n_batches], ys[s % n_batches], b, grads)
            binding.weighted_aggregate(grads, b, Pp, out)
            binding.model_update(model, out, opt, velocity)
        elif args.aggregate == "update":      # aggregate folded into the update kernel
            binding.forward_backward(model, xs[s % n_batches], ys[s % n_batches], b, grads)
            binding.model_aggregate_update(model, grads, b, opt, velocity)
        else:                                 # aggregate folded into the weight-gradient kernel
            binding.forward_backward_aggregate(model, xs[s % n_batches], ys[s % n_batches], b,
                                               grads, out)
            binding.model_update(model, out, opt, velocity)
        t = synth.iteration_times(b, cfg["speeds"])
        state["b"] = binding.controller_step(t, b, G, cfg["gains"])
        state["trace"].append(b)
        state["step"] = s + 1

    for _ in range(args.warmup):
        one_step()
    # K steps between two synchronisations (the wall-clock figure `value` is computed from), each
    # step also bracketed by HIP events on the launch stream (torch's current stream is the one
    # the binding hands to the library)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        one_step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    median_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else \
        0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    timed_splits = state["trace"][args.warmup:]

    # the same step on two fixed splits: uniform (no raggedness) and an adversarial one whose
    # sizes straddle every tile and granule boundary (workload 4 only: both sum to 4096)
    other = {}
    if cfg["index"] == 4 and not args.copy_calibration:
        fixed = {"uniform": [G // K] * K,
                 "adversarial": [1, 2, 3, 17, 31, 33, 63, 65, 127, 129, 255, 257, 511, 513, 1023, 1066]}
        for name, bs in fixed.items():
            assert sum(bs) == G and len(bs) == K
            def fixed_step(bs=bs):
                binding.forward_backward_aggregate(model, xs[0], ys[0], bs, grads, out)
                binding.model_update(model, out, opt, velocity)
                binding.controller_step(synth.iteration_times(bs, cfg["speeds"]), bs, G, cfg["gains"])
            for _ in range(args.warmup):
                fixed_step()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                fixed_step()
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t1) / args.steps
            other[name] = {"b": bs, "ms_per_step": 1e3 * dt, "samples_per_s": G / dt}

    # the weighted aggregation as a pass of its own over the gradients the last step wrote
    # (dynb_weighted_aggregate: K reads + 1 write of P_pad floats), event-timed
    agg_pass = None
    if not args.copy_calibration:
        b_last = timed_splits[-1]
        reps = max(5, args.steps)
        for _ in range(2):
            binding.weighted_aggregate(grads, b_last, Pp, out)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            binding.weighted_aggregate(grads, b_last, Pp, out)
            ev[i + 1].record()
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
        ms = ts[len(ts) // 2]
        nbytes_agg = (K + 1) * Pp * 4
        agg_pass = {"ms": ms, "bytes": nbytes_agg, "gbps": nbytes_agg / ms / 1e6,
                    "frac_of_hbm_peak": nbytes_agg / ms / 1e6 / PEAK["hbm"]}

    if args.copy_calibration:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, device="cuda"); dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    # per-kernel-class durations: the same steps again with HIP events around every launch
    binding.profile_reset()
    binding.profile_enable(True)
    state["step"] = args.warmup
    state["b"] = timed_splits[0]
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    prof = binding.profile_read()
    binding.profile_enable(False)
    kernels = {}
    for name, v in prof.items():
        if v["launches"]:
            kernels[name] = {"ms_per_step": v["ms"] / args.steps,
                             "launches_per_step": v["launches"] / args.steps,
                             "avg_launch_ms": v["ms"] / v["launches"],
                             "tflops": v["flops"] / v["ms"] / 1e9 if v["ms"] else 0.0,
                             "gbps": v["bytes"] / v["ms"] / 1e6 if v["ms"] else 0.0}
    dominant = max(kernels, key=lambda n: kernels[n]["ms_per_step"])
    bf = spec["dtype"] == "bf16"
    if dominant.startswith("gemm") and not dominant.startswith("gemm_wgrad"):
        peak = PEAK["mfma_bf16"] if bf else PEAK["fp32"]
        roofline = {"kernel": dominant, "bound": "mfma" if bf else "alu",
                    "achieved": kernels[dominant]["tflops"], "peak": peak, "unit": "TFLOP/s",
                    "frac": kernels[dominant]["tflops"] / peak, "traffic": None}
    else:
        # the per-worker weight gradient writes K*P floats, aggregation and update are pure streams
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": kernels[dominant]["gbps"],
                    "peak": PEAK["hbm"], "unit": "GB/s",
                    "frac": kernels[dominant]["gbps"] / PEAK["hbm"], "traffic": None}
    roofline["avg_launch_ms"] = kernels[dominant]["avg_launch_ms"]
    roofline["traffic"] = measured_traffic(dominant, cfg["index"])

    result = {
        "metric": "samples/s fwd+bwd+weighted-agg+update at ragged K-way b_k",
        "value": G * args.steps / elapsed, "unit": "samples/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf else "f32", "data": "synthetic",
        "config": {"workload": "configs[%d]: %s" % (cfg["index"], cfg["name"]), "global_batch": G,
                   "workers": K, "b_timed_first": timed_splits[0], "b_timed_last": timed_splits[-1],
                   "params": P},
        "ms_per_step_median_events": median_ms,
        "roofline": roofline,
        "other_splits": other,
        "kernels": kernels,
    }
    # the HBM-bound parts against the 8 TB/s peak (algorithmic bytes / event-timed duration) and
    # the matrix products against the bf16 MFMA peak
    frac = {}
    for name, peak_key, field in (("gemm_wgrad", "hbm", "gbps"), ("gemm_wgrad_small_tiles", "hbm", "gbps"),
                                  ("sgd_update", "hbm", "gbps"),
                                  ("gemm_fwd", "mfma_bf16" if bf else "fp32", "tflops"),
                                  ("gemm_dgrad", "mfma_bf16" if bf else "fp32", "tflops"),
                                  ("gemm_small_tiles", "mfma_bf16", "tflops")):
        if name in kernels:
            frac[name] = {"achieved": kernels[name][field],
                          "unit": "GB/s" if field == "gbps" else "TFLOP/s",
                          "peak": PEAK[peak_key], "frac": kernels[name][field] / PEAK[peak_key]}
    if agg_pass:
        frac["weighted_aggregate_pass"] = {"achieved": agg_pass["gbps"], "unit": "GB/s",
                                           "peak": PEAK["hbm"], "frac": agg_pass["frac_of_hbm_peak"],
                                           "ms": agg_pass["ms"]}
    result["fractions_of_peak"] = frac
    if cfg["index"] == 4 and not args.copy_calibration and not args.no_other_workloads:
        del xs, ys, grads, out
        torch.cuda.empty_cache()
        result["other_workloads"] = {"configs[%d]" % i: small_workload(i) for i in range(4)}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, timed_splits[-1])
    print(json.dumps(result))


def small_workload(ci, steps=30, warmup=5):
    """Throughput of one of the other workloads: the same step (gradients with their aggregate,
    update, controller) over the batch sizes its controller produces; event-timed median."""
    import torch
    from paper_2305_12213_amd import binding, synth
    cfg = synth.config(ci)
    spec, seed = cfg["spec"], synth.BASE_SEED + ci
    G, K = cfg["global_batch"], cfg["K"]
    model = binding.Model(spec)
    Pp = model.padded_params()
    params = torch.from_numpy(synth.flatten_params(synth.init_params(spec, cfg["init"], seed), 256)).cuda()
    nbytes = model.workspace_bytes(G, K)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    model.bind(params, ws, nbytes, G, K)
    grads = torch.empty(K, Pp, device="cuda"); out = torch.empty(Pp, device="cuda")
    velocity = torch.zeros(Pp, device="cuda") if cfg["momentum"] else None
    opt = binding.make_optimizer("momentum" if cfg["momentum"] else "sgd", lr=cfg["lr"],
                                 momentum=cfg["momentum"])
    batches = []
    for s in range(4):
        x, y = synth.make_batch(spec, cfg["x_dist"], G, seed, s)
        batches.append((torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()))
    b = list(cfg["b0"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = 0.0
    for i in range(warmup + steps):
        if i == warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev[0].record()
        x, y = batches[i % len(batches)]
        binding.forward_backward_aggregate(model, x, y, b, grads, out)
        binding.model_update(model, out, opt, velocity)
        b = binding.controller_step(synth.iteration_times(b, cfg["speeds"]), b, G, cfg["gains"])
        if i >= warmup:
            ev[i - warmup + 1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    med = ts[len(ts) // 2]
    return {"workload": cfg["name"], "global_batch": G, "workers": K, "b_last": b,
            "ms_per_step_median_events": med, "ms_per_step_wall": 1e3 * wall,
            "samples_per_s": G / wall}


def cpu_baseline(cfg, b):
    """The CPU checker, as it stands (float64 numpy; its matrix products go to the BLAS numpy is
    linked with), on the host cores this process may use: one whole step of the workload on all
    of them, and a scaled-down step (the smallest workers of the same split) on one thread."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle import network as on
    from paper_2305_12213_amd import synth

    spec, seed = cfg["spec"], synth.BASE_SEED + cfg["index"]
    G = cfg["global_batch"]
    bf = spec["dtype"] == "bf16"
    params = synth.init_params(spec, cfg["init"], seed)
    x, y = synth.make_batch(spec, cfg["x_dist"], G, seed, 0)
    cores = len(os.sched_getaffinity(0))
    # (the box exports the thread count its share of the machine allows)
    threads = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))

    def step(bs, xs, ys):
        t0 = time.perf_counter()
        _, gk = on.worker_gradients(spec, params, xs, ys, bs, emulate_bf16=bf)
        agg = on.weighted_aggregate(gk, bs)
        on.sgd_update(params, agg, cfg["lr"])
        return time.perf_counter() - t0

    with threadpool_limits(limits=threads):
        dt_all = step(list(b), x, y)
    # one thread: the smallest workers of the split, about 1/64 of the batch
    order = sorted(range(len(b)), key=lambda k: b[k])
    off = np.concatenate([[0], np.cumsum(b)])
    chosen, n = [], 0
    for k in order:
        if b[k] == 0:
            continue
        if chosen and n + b[k] > max(1, G // 64):
            break
        chosen.append(k); n += b[k]
    idx = np.concatenate([np.arange(off[k], off[k + 1]) for k in sorted(chosen)])
    with threadpool_limits(limits=1):
        dt_one = step([b[k] for k in sorted(chosen)], x[idx], y[idx])
    return {"value": G / dt_all, "unit": "samples/s", "cores": threads,
            "cores_available": cores, "kind": "oracle (numpy float64, BLAS matrix products)",
            "sample": "one whole step (per-worker fwd+bwd, aggregate, update) of the timed split, "
                      "%d samples in %.1f s on %d threads" % (G, dt_all, threads),
            "one_thread": {"value": n / dt_one, "unit": "samples/s",
                           "sample": "the same step over workers %s of the split, %d of %d "
                                     "samples, %.1f s" % (sorted(chosen), n, G, dt_one)}}


if __name__ == "__main__":
    main()
