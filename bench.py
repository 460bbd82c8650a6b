#!/usr/bin/env python3
"""Benchmark: lock-step NUTS throughput on one MI355X.

A "step" is one complete nuts_sample call on the headline workload (configuration 3: Bayesian
logistic regression 1000x25, binary64, 4096 chains, 1000 iterations, step 0.05, max depth 10) with
the target already resident on the GPU.  Prints one JSON line:
  value      leapfrog gradient evaluations per second, summed over all chains
  roofline   binary64 matrix-core roofline of the gradient (4*N*d flop per evaluation)
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload (context only)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = {8: 78.6, 4: 157.3}   # dense binary64 / binary32 matrix-core peaks of MI355X
KERNEL_NAMES = {1: "nuts_wave_kernel", 2: "nuts_tile_kernel", 3: "nuts_elem_kernel", 4: "nuts_grid_grad_kernel",
                5: "nuts_dense_kernel"}


def cpu_baseline(w, leaf_steps, sampler, target_seconds=12.0):
    """The oracle as it stands on a bounded sample of the same workload: chains 0..n-1, first iterations.
    A short pilot run sizes the sample so that it takes about `target_seconds` on this host."""
    from oracle import nuts_ref
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or (os.cpu_count() or 1)))
    t = nuts_ref.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                        prior_scale=w.prior_scale)

    def run(n_chains, n_iters):
        t0 = time.perf_counter()
        _, _, nl = nuts_ref.sample(t, n_chains, n_iters, w.step_size, w.max_tree_depth, w.seed, n_threads=cores,
                                   leaf_steps=leaf_steps, sampler=sampler)
        return int(nl.sum()), time.perf_counter() - t0

    # pilots grow until one takes half a second; its chain-iterations per second size the sample
    n_chains, n_iters = min(cores, w.n_chains), min(2, w.n_iters)
    while True:
        _, pilot_s = run(n_chains, n_iters)
        if pilot_s >= 0.5 or (n_iters >= min(w.n_iters, 300) and n_chains >= min(w.n_chains, 4096)):
            break
        if n_iters < min(w.n_iters, 300):
            n_iters = min(w.n_iters, 300, n_iters * 4)
        else:
            n_chains = min(w.n_chains, 4096, n_chains * 4)
    scale = target_seconds / max(pilot_s, 1e-3)
    if scale > 1.0:
        grow_iters = min(scale, min(w.n_iters, 300) / n_iters)
        n_iters = max(1, int(n_iters * grow_iters))
        n_chains = max(1, min(w.n_chains, 4096, int(n_chains * scale / grow_iters) // cores * cores or n_chains))
    n_grad, dt = run(n_chains, n_iters)
    return {"value": n_grad / dt, "unit": "grad-evals/s", "cores": cores, "kind": "oracle",
            "sample": f"chains 0..{n_chains - 1}, first {n_iters} iterations of the same workload, "
                      f"{n_grad} gradient evaluations in {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..5 (headline: 3); 6: the shape of the paper's own logistic-regression experiment")
    ap.add_argument("--chains", type=int, default=None)
    ap.add_argument("--iters", type=int, default=None)
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 wave kernel, 2 tile kernel")
    ap.add_argument("--leaf-steps", type=int, default=1,
                    help="leapfrog steps per tree leaf (headline: 1; Section 4.1 of the paper ran 4)")
    ap.add_argument("--sampler", type=int, default=0, help="0 multinomial (headline), 1 slice (the published form)")
    ap.add_argument("--schedule", type=int, default=0, help="0 free-running (headline), 1 synchronised at trajectory boundaries")
    ap.add_argument("--step-size", type=float, default=None, help="override the configuration's step size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="first run one plain device copy of this many MiB (a dispatch of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (chains are independent: more GPUs would each take a "
                 "range of chains, offset by first_chain, with no exchange). Use --gpus 1.")

    import torch
    import paper_1910_11141_amd.binding as nuts
    from paper_1910_11141_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = workloads.make(a.config, n_chains=a.chains, n_iters=a.iters)
    if a.step_size is not None:
        w.step_size = a.step_size
    tgt = nuts.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                      prior_scale=w.prior_scale)
    tdt = torch.float64 if w.dtype.itemsize == 8 else torch.float32
    out = (torch.empty((w.n_iters, w.n_chains, w.dim), dtype=tdt, device="cuda"),
           torch.empty((w.n_iters, w.n_chains), dtype=torch.int32, device="cuda"),
           torch.empty((w.n_iters, w.n_chains), dtype=torch.int32, device="cuda"))

    if a.copy_calibration:
        n = a.copy_calibration * (1 << 20) // 8
        src = torch.arange(n, dtype=torch.float64, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # reads and writes copy_calibration MiB each
        torch.cuda.synchronize()
        del src, dst

    def step():
        nuts.nuts_sample(tgt, w.n_chains, w.n_iters, w.step_size, w.max_tree_depth, w.seed, variant=a.variant,
                         out=out, leaf_steps=a.leaf_steps, sampler=a.sampler, schedule=a.schedule)

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    kernel_ms = []
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
        kernel_ms.append(nuts.nuts_get_stats(tgt)["kernel_ms"])   # waits on the kernel's own stop event
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stats = nuts.nuts_get_stats(tgt)
    n_grad = int(out[2].sum().item())
    assert n_grad == stats["leaf_slots_useful"]
    mean_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3

    if w.kind == workloads.LOGREG:
        flops = 4.0 * w.n_data * w.dim * n_grad
        roof = {"bound": "mfma", "achieved": flops / mean_kernel_s / 1e12, "peak": PEAK_MFMA_TFLOPS[w.dtype.itemsize],
                "unit": "TFLOP/s"}
    elif w.kind == workloads.GAUSS_DENSE:
        flops = 2.0 * w.dim * w.dim * n_grad
        roof = {"bound": "mfma", "achieved": flops / mean_kernel_s / 1e12, "peak": PEAK_MFMA_TFLOPS[w.dtype.itemsize],
                "unit": "TFLOP/s"}
    else:
        nbytes = 4.0 * w.dim * w.dtype.itemsize * n_grad
        roof = {"bound": "hbm", "achieved": nbytes / mean_kernel_s / 1e9, "peak": 8000.0, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM-side bytes per launch: measured with rocprofv3 counters (not collectable from inside this
    # process); the committed summary under profiles/ applies only to the exact workload it was taken on.
    roof["traffic"] = None
    tpath = os.path.join(ROOT, "profiles", f"nuts_tile_kernel_{w.name}_traffic.json")
    if stats["variant"] == 2 and os.path.exists(tpath):
        t = json.load(open(tpath))
        if (t["n_chains"], t["n_iters"]) == (w.n_chains, w.n_iters) and a.leaf_steps == 1 and a.step_size is None \
                and a.sampler == 0 and a.schedule == 0:
            roof["traffic"] = t["fetch_bytes_per_launch"] + t["write_bytes_per_launch"]
            roof["traffic_unit"] = "bytes/launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size)"
    roof["kernel"] = KERNEL_NAMES[stats["variant"]]
    roof["kernel_ms"] = mean_kernel_s * 1e3

    line = {
        "metric": "leapfrog grad-evals/sec (all chains)",
        "value": n_grad * a.steps / dt,
        "unit": "grad-evals/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": dt / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if w.dtype.itemsize == 8 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n_chains": w.n_chains, "n_iters": w.n_iters, "dim": w.dim,
                   "n_data": w.n_data, "step_size": w.step_size, "max_tree_depth": w.max_tree_depth,
                   "leaf_steps": a.leaf_steps, "sampler": ["multinomial", "slice"][a.sampler],
                   "schedule": ["free", "trajectory"][a.schedule], "variant": stats["variant"]},
        "chain_iters_per_s": w.n_chains * w.n_iters * a.steps / dt,
        "grad_evals_per_step": n_grad,
        "occupancy": stats["occupancy"],
        "best_kernel_grad_evals_per_s": n_grad / (min(kernel_ms) / 1e3),
        "roofline": roof,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, a.leaf_steps, a.sampler)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
