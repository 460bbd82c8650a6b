#!/usr/bin/env python3
"""Benchmark and measurement tool: lock-step NUTS on one MI355X.

Default run: a "step" is one complete nuts_sample call on the headline workload (configuration 3: Bayesian
logistic regression 1000x25, binary64, 4096 chains, 1000 iterations, step 0.05, max depth 10) with the target
already resident on the GPU.  Prints one JSON line:
  value         leapfrog gradient evaluations per second, summed over all chains
  roofline      the bound of the kernel that ran, on the method's own work (see roofline_of below)
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload (context only)
  longest_chain_over_mean   leapfrog steps of the chain that takes most / mean over chains: the launch lasts as long as
                its longest chain, the mean sets the work

Other modes (none of them is the driver's default):
  --sweep throughput    gradient evaluations per second against the number of chains (the measurement of
                        Section 4.1 / Figure 6 of the paper), one JSON line per chain count
  --sweep utilization   gradient-slot occupancy against the number of chains, free-running against synchronised
                        at trajectory boundaries (Section 4.2 / Figure 7), one JSON line per chain count
  --sweep pcvm          throughput and utilisation of the program-counter virtual machine
  --rocprof-summary DB [DB ...]        short text summary of rocprofv3 result databases (what profiles/ keeps)
  --traffic-json OUT --fetch-db A --write-db B    HBM bytes per gradient evaluation of the benchmarked kernel from
                        two counter passes (FETCH_SIZE, WRITE_SIZE) of `bench.py --copy-calibration 256 --steps 1 --warmup 0`
  --issue-ceiling-json OUT --sq-db A   what the kernel's own instruction mix allows (see issue_ceiling below)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = {8: 78.6, 4: 157.3}   # dense binary64 / binary32 matrix-core peaks of MI355X
PEAK_VECTOR_TFLOPS = {8: 78.6, 4: 157.3}  # plain vector arithmetic: 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz (x 2 packed in binary32)
PEAK_HBM_GBS = 8000.0
KERNEL_NAMES = {1: "nuts_wave_kernel", 2: "nuts_tile_kernel", 3: "nuts_elem_kernel", 4: "nuts_grid_grad_kernel",
                5: "nuts_dense_kernel", 6: "nuts_quad_kernel"}
# ticks of one SIMD per instruction, from the instruction-issue microbenchmark (profiles/mi355x_issue_ubench.txt)
TICKS_PER_MFMA_F64_16X16X4 = 64.0
TICKS_PER_VALU = 5.07


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


# ---------------------------------------------------------------------------------------------- rooflines

def profile_json(kind, kernel, workload_name):
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload_name}_{kind}.json")
    return json.load(open(path)) if os.path.exists(path) else None


def roofline_of(w, workloads, stats, n_grad, kernel_s, plain_run):
    """The roofline line of the kernel that ran, on the method's own work per gradient evaluation:
      logistic regression      4 N d flop (the two GEMMs) against the matrix peak of its dtype ("mfma");
      dense Gaussian, quad kernel   2 d^2 flop (P theta as MFMA blocks) against the binary64 matrix peak ("mfma");
      dense Gaussian           2 nnz(P) + 8 d flop (the matrix-vector product over the entries that are not zero,
                               the log-density, the leapfrog updates) against the plain vector peak ("alu"): the
                               register kernel does these on the vector ALUs, one chain per wavefront, and what
                               limits it is the latency of one chain's serial step, not a throughput;
      element-wise Gaussians   4 d sizeof(T) bytes (position and momentum in and out) against HBM ("hbm").
    `traffic` is the HBM-side bytes of one launch from the committed counter summary of the same kernel and
    chain count (bytes per gradient evaluation there x this launch's evaluations), or null; `wasted_traffic`
    the ratio of that to the algorithmic bytes.  Where the kernel moves fewer bytes than the basis charges
    (so that the basis fraction would exceed 1), `frac` is the fraction of the HBM peak it really draws."""
    item = w.dtype.itemsize
    kernel = KERNEL_NAMES[stats["variant"]]
    alg_bytes = None
    if w.kind == workloads.LOGREG:
        work = 4.0 * w.n_data * w.dim * n_grad
        roof = {"bound": "mfma", "achieved": work / kernel_s / 1e12, "peak": PEAK_MFMA_TFLOPS[item], "unit": "TFLOP/s"}
        # the chain state in and out, plus the data read once per lock-step round and shared by the chains of the call
        alg_bytes = (6.0 * w.dim * item + float(w.n_data) * w.dim * item / w.n_chains) * n_grad
    elif w.kind == workloads.GAUSS_DENSE and kernel == "nuts_quad_kernel":
        work = 2.0 * w.dim * w.dim * n_grad   # P theta for every chain, on the matrix cores
        roof = {"bound": "mfma", "achieved": work / kernel_s / 1e12, "peak": PEAK_MFMA_TFLOPS[item], "unit": "TFLOP/s"}
        alg_bytes = 6.0 * w.dim * item * n_grad
    elif w.kind == workloads.GAUSS_DENSE:
        import numpy as np
        nnz = int(np.count_nonzero(w.precision))
        work = (2.0 * nnz + 8.0 * w.dim) * n_grad
        roof = {"bound": "alu", "achieved": work / kernel_s / 1e12, "peak": PEAK_VECTOR_TFLOPS[item], "unit": "TFLOP/s",
                "flop_per_grad_eval": 2.0 * nnz + 8.0 * w.dim,
                "note": "one chain per wavefront: limited by the latency of a chain's serial step, not by arithmetic"}
        alg_bytes = 6.0 * w.dim * item * n_grad
    else:
        alg_bytes = 4.0 * w.dim * item * n_grad
        roof = {"bound": "hbm", "achieved": alg_bytes / kernel_s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = None
    t = profile_json("traffic", kernel, w.name)
    if t and "bytes_per_grad_eval" in t and t["n_chains"] == w.n_chains and plain_run:
        roof["traffic"] = t["bytes_per_grad_eval"] * n_grad
        roof["traffic_unit"] = ("bytes/launch: bytes per gradient evaluation from the committed rocprofv3 FETCH_SIZE + WRITE_SIZE "
                                "passes of this kernel and chain count (scaled by a copy of known size) x this launch's evaluations")
        roof["wasted_traffic"] = roof["traffic"] / alg_bytes
        if roof["bound"] == "hbm":
            measured = roof["traffic"] / kernel_s / 1e9
            roof["measured_traffic_gbs"] = measured
            if roof["frac"] > 1.0:
                # the kernel keeps state in registers and moves less than the basis charges: the basis no longer
                # describes it, so the fraction reported is the HBM bandwidth it really draws
                roof["basis_frac"] = roof["frac"]
                roof["achieved"] = measured
                roof["frac"] = measured / PEAK_HBM_GBS
                roof["note"] = ("moves fewer bytes than the 4 d sizeof(T) basis (state stays in registers): no longer HBM-bound; "
                                "bound by vector-instruction issue (profiles/nuts_elem_kernel_cfg5_diag_gauss_d1000_sq_counters.txt)")
    if roof["frac"] > 1.0:   # no committed traffic figure for this shape: a fraction above 1 would say nothing
        roof["basis_frac"] = roof["frac"]
        roof["frac"] = None
        roof["note"] = "moves fewer bytes than the basis charges; no traffic summary for this chain count"
    c = profile_json("issue_ceiling", kernel, w.name)
    if c and roof["bound"] == "mfma" and plain_run:
        # what the kernel's instruction mix allows if its SIMDs never idled (matrix and vector instructions of a
        # SIMD do not overlap on this chip): useful MFMA ticks / (MFMA ticks + vector-instruction ticks)
        roof["issue_ceiling_frac"] = c["ceiling_frac"]
        roof["frac_of_issue_ceiling"] = roof["frac"] / c["ceiling_frac"]
    ticks = stats.get("phase_ticks") or [0, 0, 0]
    if kernel == "nuts_tile_kernel" and sum(ticks) > 0:
        # the tile kernel times its three phases itself (shader-clock reads of wave 0 of every workgroup): the share of
        # the launch spent in the batched gradient (the two GEMMs and the logistic functions), and the matrix rate there
        share = ticks[1] / float(sum(ticks))
        roof["gradient_phase"] = {"share_of_kernel_time": share, "achieved": roof["achieved"] / share,
                                  "frac": roof["achieved"] / share / roof["peak"], "unit": roof["unit"]}
    roof["kernel"] = kernel
    roof["kernel_ms"] = kernel_s * 1e3
    return roof


# ---------------------------------------------------------------------------------------------- profile tools

def rocprof_summary(path):
    """A rocprofv3 result database (rocpd sqlite, the default output) as text: per-kernel call counts and
    durations and, if the run collected counters, per-dispatch counter values."""
    import sqlite3

    def short(name, width=72):
        name = name.replace("(anonymous namespace)::", "")
        return name if len(name) <= width else name[: width - 3] + "..."

    db = sqlite3.connect(path)
    out = [f"== {path}"]
    rows = list(db.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
    if rows:
        out.append(f"{'kernel':72s} {'calls':>6s} {'total_ms':>11s} {'avg_ms':>11s} {'%':>7s}")
        for name, calls, total, avg, pct in rows:
            out.append(f"{short(name):72s} {calls:6d} {total / 1e3:11.3f} {avg / 1e3:11.3f} {pct:7.3f}")
    # a counter comes in one row per shader engine and XCD: summed per dispatch here
    pmc = list(db.execute("select name, counter_name, sum(counter_value), max(duration) from pmc_events "
                          "group by dispatch_id, counter_name order by dispatch_id, counter_name"))
    if len(pmc) > 200:   # a run of many launches: one row per kernel and counter
        agg = {}
        for name, cname, val, dur in pmc:
            v, n = agg.get((name, cname), (0.0, 0))
            agg[(name, cname)] = (v + val, n + 1)
        out.append("")
        out.append(f"{'kernel (all its dispatches)':72s} {'counter':>28s} {'sum':>16s} {'dispatches':>10s}")
        for (name, cname), (v, n) in agg.items():
            out.append(f"{short(name):72s} {cname:>28s} {v:16.3f} {n:10d}")
    elif pmc:
        out.append("")
        out.append(f"{'dispatch (in order)':72s} {'counter':>28s} {'value':>16s} {'dur_us':>10s}")
        for name, cname, val, dur in pmc:
            out.append(f"{short(name):72s} {cname:>28s} {val:16.3f} {dur / 1e3:10.1f}")
    return "\n".join(out)


def counter_sums(path, kernel_prefix):
    """counter -> (sum over the dispatches whose kernel name contains kernel_prefix, number of such dispatches)"""
    import sqlite3
    db = sqlite3.connect(path)
    sums = {}
    for name, cname, val in db.execute("select name, counter_name, counter_value from pmc_events"):
        if kernel_prefix in name:
            s, n = sums.get(cname, (0.0, 0))
            sums[cname] = (s + val, n + 1)
    return sums


def copy_scale(path, counter, copy_kib):
    """The factor that turns a counter's reading into KiB: a plain device copy of copy_kib KiB each way is the
    largest __amd_rocclr_copyBuffer dispatch of the run."""
    import sqlite3
    db = sqlite3.connect(path)
    best = max((val for name, cname, val in db.execute("select name, counter_name, sum(counter_value) from pmc_events "
                                                       "group by dispatch_id, counter_name")
                if "copyBuffer" in name and cname == counter), default=0.0)
    if best <= 0:
        raise SystemExit(f"{path}: no copy dispatch with counter {counter} (run bench.py with --copy-calibration)")
    return copy_kib / best


def make_traffic_json(a):
    line = json.loads(open(a.bench_line).read().strip().splitlines()[-1])
    kernel = line["roofline"]["kernel"]
    family = "nuts_grid_" if kernel.startswith("nuts_grid") else kernel   # every kernel of a grid round counts
    fetch, nf = counter_sums(a.fetch_db, family).get("FETCH_SIZE", (0.0, 0))
    write, nw = counter_sums(a.write_db, family).get("WRITE_SIZE", (0.0, 0))
    if not nf or not nw:
        raise SystemExit("the databases hold no FETCH_SIZE / WRITE_SIZE dispatches of " + family)
    fs, ws = copy_scale(a.fetch_db, "FETCH_SIZE", a.copy_kib), copy_scale(a.write_db, "WRITE_SIZE", a.copy_kib)
    n_grad = line["grad_evals_per_step"]
    out = {"kernel": kernel, "workload": line["config"]["workload"], "n_chains": line["config"]["n_chains"],
           "n_iters": line["config"]["n_iters"], "grad_evals_per_launch": n_grad,
           "fetch_bytes_per_launch": fetch * fs * 1024.0, "write_bytes_per_launch": write * ws * 1024.0,
           "fetch_scale": fs, "write_scale": ws,
           "bytes_per_grad_eval": (fetch * fs + write * ws) * 1024.0 / n_grad,
           "source": "bench.py --traffic-json from two rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE), KiB per dispatch, each "
                     "scaled by what the same counter reads for a plain device copy of known size"}
    json.dump(out, open(a.traffic_json, "w"), indent=1)
    print(json.dumps(out))


def issue_ceiling(a):
    """What the headline kernel's own instruction mix allows.  On this chip a SIMD issues either a matrix or a
    vector instruction at a time, from whatever wave (profiles/mi355x_issue_ubench.txt), so with no idle cycle at
    all the useful share of its time is
        useful MFMA ticks / (MFMA instructions x 64 ticks + vector instructions x 5.07 ticks),
    useful = the multiply-adds of the two GEMMs at the true dimension (4 N d flop per gradient evaluation / 2048 flop
    per instruction), as opposed to the instructions issued, which pad d.  The counts come from one rocprofv3 pass
    (SQ_INSTS_MFMA, SQ_INSTS_VALU, SQ_BUSY_CU_CYCLES) of `bench.py --steps 1 --warmup 0`."""
    line = json.loads(open(a.bench_line).read().strip().splitlines()[-1])
    kernel = line["roofline"]["kernel"]
    sums = counter_sums(a.sq_db, kernel)
    mfma, valu, busy = sums["SQ_INSTS_MFMA"][0], sums["SQ_INSTS_VALU"][0], sums["SQ_BUSY_CU_CYCLES"][0]
    cfg = line["config"]
    useful_mfma = 4.0 * cfg["n_data"] * cfg["dim"] * line["grad_evals_per_step"] / 2048.0
    mfma_ticks, valu_ticks = mfma * TICKS_PER_MFMA_F64_16X16X4, valu * TICKS_PER_VALU
    out = {"kernel": kernel, "workload": cfg["workload"], "n_chains": cfg["n_chains"], "n_iters": cfg["n_iters"],
           "mfma_instructions": mfma, "useful_mfma_instructions": useful_mfma, "valu_instructions": valu,
           "simd_ticks_available": 4.0 * busy, "mfma_ticks": mfma_ticks, "valu_ticks": valu_ticks,
           "issue_utilisation": (mfma_ticks + valu_ticks) / (4.0 * busy),
           "ceiling_frac": useful_mfma * TICKS_PER_MFMA_F64_16X16X4 / (mfma_ticks + valu_ticks),
           "source": "bench.py --issue-ceiling-json from one rocprofv3 --pmc pass (SQ_INSTS_MFMA SQ_INSTS_VALU SQ_BUSY_CU_CYCLES) "
                     "and the tick costs of profiles/mi355x_issue_ubench.txt"}
    json.dump(out, open(a.issue_ceiling_json, "w"), indent=1)
    print(json.dumps(out))


# ---------------------------------------------------------------------------------------------- sweeps

def need_gpu(what):
    import torch
    if not torch.cuda.is_available():
        sys.exit(f"bench.py {what} needs a GPU (this build has no CPU path)")
    torch.cuda.set_device(0)


def sweep_throughput(a):
    """Section 4.1 / Figure 6: useful gradient evaluations per second (leapfrog steps the chains asked for / kernel
    time, best of --repeats) against the number of chains; default workload: the shape of the paper's own experiment."""
    need_gpu("--sweep throughput")
    import torch
    import paper_1910_11141_amd.binding as nuts
    from paper_1910_11141_amd import workloads
    cfg = a.config if a.config_given else 6
    iters = a.iters or 20
    w = workloads.make(cfg, n_iters=iters)
    tgt = nuts.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y, prior_scale=w.prior_scale)
    for n_chains in [int(x) for x in (a.chain_counts or "1,2,4,8,16,32,64,128,256,512,1024,2048,4096").split(",")]:
        best, out = None, None
        for _ in range(a.repeats + 1):   # the first run also warms up
            out = nuts.nuts_sample(tgt, n_chains, iters, w.step_size, w.max_tree_depth, w.seed, variant=a.variant,
                                   leaf_steps=a.leaf_steps, sampler=a.sampler)
            torch.cuda.synchronize()
            st = nuts.nuts_get_stats(tgt)
            best = st if best is None or st["kernel_ms"] < best["kernel_ms"] else best
        n_grad = int(out[2].sum().item())
        print(json.dumps({"workload": w.name, "n_chains": n_chains, "n_iters": iters, "leaf_steps": a.leaf_steps,
                          "sampler": a.sampler, "grad_evals": n_grad, "grad_evals_per_s": n_grad / (best["kernel_ms"] * 1e-3),
                          "ms": best["kernel_ms"], "occupancy": best["occupancy"], "variant": best["variant"]}), flush=True)


def sweep_utilization(a):
    """Section 4.2 / Figure 7: the same workload free-running (gradient steps of different iterations share a batch)
    and synchronised at trajectory boundaries; outputs must be identical; occupancy = useful / issued gradient slots."""
    need_gpu("--sweep utilization")
    import torch
    import paper_1910_11141_amd.binding as nuts
    from paper_1910_11141_amd import workloads
    cfg = a.config if a.config_given else 2
    iters = a.iters or 10   # the paper's figure batches across 10 trajectories
    w = workloads.make(cfg, n_iters=iters)
    tgt = nuts.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y, prior_scale=w.prior_scale)
    for n_chains in [int(x) for x in (a.chain_counts or "1,2,4,8,16,32,64,128,256,512,1024").split(",")]:
        point = {"workload": w.name, "n_chains": n_chains, "n_iters": iters, "leaf_steps": a.leaf_steps}
        outs = {}
        for name, schedule in (("free", nuts.NUTS_SCHEDULE_FREE), ("trajectory", nuts.NUTS_SCHEDULE_TRAJECTORY)):
            best = None
            for _ in range(a.repeats):
                out = nuts.nuts_sample(tgt, n_chains, iters, w.step_size, w.max_tree_depth, w.seed, variant=a.variant,
                                       leaf_steps=a.leaf_steps, schedule=schedule)
                torch.cuda.synchronize()
                st = nuts.nuts_get_stats(tgt)
                best = st if best is None or st["kernel_ms"] < best["kernel_ms"] else best
            outs[name] = out
            n_grad = int(out[2].sum().item())
            point[name] = {"occupancy": best["occupancy"], "grad_evals_per_s": n_grad / (best["kernel_ms"] * 1e-3),
                           "ms": best["kernel_ms"], "variant": best["variant"]}
        point["grad_evals"] = int(outs["free"][2].sum().item())
        point["identical_outputs"] = all(bool(torch.equal(x, y)) for x, y in zip(outs["free"], outs["trajectory"]))
        nl = outs["free"][2].to(torch.float64)
        point["longest_over_mean_trajectory"] = float((nl.max(dim=1).values / nl.mean(dim=1)).mean().item())
        print(json.dumps(point), flush=True)


def sweep_pcvm(a):
    """The program-counter virtual machine: scheduler steps and member-steps per second, and utilisation (members
    that executed a block / members the masked execution paid for), for the four ways of running it."""
    need_gpu("--sweep pcvm")
    import torch
    from paper_1910_11141_amd import pcvm, pcvm_programs
    prog = pcvm_programs.ALL[a.program]()
    g = torch.Generator(device="cpu").manual_seed(1910_11141)
    base = torch.randint(1, a.max_input + 1, (prog.n_inputs, a.batch), generator=g, dtype=torch.int64)
    for label, srt, queued, policy in (("fixed groups, earliest block", False, False, 0), ("queue, earliest block", False, True, 0),
                                       ("queue, block most lanes wait for", False, True, 1),
                                       ("fixed groups, inputs sorted", True, False, 0)):
        ins = base[:, torch.argsort(base[0])] if srt else base
        ins = ins.cuda().contiguous()
        best = None
        for _ in range(a.repeats):
            out, st, _ = pcvm.pcvm_run(prog, ins, 32, queued=queued, policy=policy)
            best = st if best is None or st["kernel_ms"] < best["kernel_ms"] else best
        s = best["kernel_ms"] * 1e-3
        print(json.dumps({"run": label, "program": prog.name, "batch": a.batch, "max_input": a.max_input,
                          "kernel_ms": best["kernel_ms"], "group_steps_per_s": best["steps"] / s,
                          "active_member_steps_per_s": best["active_member_steps"] / s, "utilization": best["utilization"],
                          "checksum": int(out.sum().item())}), flush=True)


# ---------------------------------------------------------------------------------------------- main

def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=None, help="benchmark configuration 1..5 (headline: 3); 6: the shape of the paper's own logistic-regression experiment")
    ap.add_argument("--chains", type=int, default=None)
    ap.add_argument("--iters", type=int, default=None)
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 wave kernel, 2 tile kernel, ...")
    ap.add_argument("--leaf-steps", type=int, default=1,
                    help="leapfrog steps per tree leaf (headline: 1; Section 4.1 of the paper ran 4)")
    ap.add_argument("--sampler", type=int, default=0, help="0 multinomial (headline), 1 slice (the published form)")
    ap.add_argument("--schedule", type=int, default=0, help="0 free-running (headline), 1 synchronised at trajectory boundaries")
    ap.add_argument("--step-size", type=float, default=None, help="override the configuration's step size")
    ap.add_argument("--dense-target", default=None, choices=[None, "random-spd"],
                    help="configuration 2 only: replace the AR(1) precision by a random dense SPD matrix of the same dimension")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="first run one plain device copy of this many MiB (a dispatch of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--sweep", choices=["throughput", "utilization", "pcvm"], default=None)
    ap.add_argument("--chain-counts", type=str, default=None, help="sweeps: comma-separated chain counts")
    ap.add_argument("--repeats", type=int, default=3, help="sweeps: timed repetitions per point (best is reported)")
    ap.add_argument("--program", default="fibonacci", help="--sweep pcvm")
    ap.add_argument("--batch", type=int, default=1 << 20, help="--sweep pcvm")
    ap.add_argument("--max-input", type=int, default=20, help="--sweep pcvm")
    ap.add_argument("--rocprof-summary", nargs="+", metavar="DB")
    ap.add_argument("--traffic-json", metavar="OUT")
    ap.add_argument("--issue-ceiling-json", metavar="OUT")
    ap.add_argument("--fetch-db"), ap.add_argument("--write-db"), ap.add_argument("--sq-db")
    ap.add_argument("--bench-line", help="file with the JSON line bench.py printed in the profiled run")
    ap.add_argument("--copy-kib", type=float, default=262144.0, help="KiB the calibration copy moved each way")
    a = ap.parse_args()
    a.config_given = a.config is not None
    if a.config is None:
        a.config = 3
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (chains are independent: more GPUs would each take a "
                 "range of chains, offset by first_chain, with no exchange). Use --gpus 1.")
    if a.rocprof_summary:
        for p in a.rocprof_summary:
            print(rocprof_summary(p))
            print()
        return
    if a.traffic_json:
        return make_traffic_json(a)
    if a.issue_ceiling_json:
        return issue_ceiling(a)
    if a.sweep:
        return {"throughput": sweep_throughput, "utilization": sweep_utilization, "pcvm": sweep_pcvm}[a.sweep](a)

    import torch
    import paper_1910_11141_amd.binding as nuts
    from paper_1910_11141_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = workloads.make(a.config, n_chains=a.chains, n_iters=a.iters)
    if a.dense_target == "random-spd":
        assert w.kind == workloads.GAUSS_DENSE, "--dense-target applies to configuration 2"
        w.precision = workloads.random_spd_precision(w.dim, 7)
        w.name = f"random_spd_gauss_d{w.dim}"
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
    per_chain = out[2].sum(dim=0, dtype=torch.int64)
    n_grad = int(per_chain.sum().item())
    assert n_grad == stats["leaf_slots_useful"]
    mean_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    plain_run = a.leaf_steps == 1 and a.step_size is None and a.sampler == 0 and a.schedule == 0 and a.variant == 0
    roof = roofline_of(w, workloads, stats, n_grad, mean_kernel_s, plain_run)

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
        # leapfrog steps of the chain that takes most / mean over chains: chains step one leapfrog per lock-step round, a
        # round costs the same however many of a workgroup's chains are still running, and every chain runs the same number
        # of iterations, so the launch lasts at least as long as its longest chain while the mean sets the work: what lies
        # above 1 is the share of the launch in which the machine drains
        "longest_chain_over_mean": float(per_chain.max().item()) / float(per_chain.double().mean().item()),
        "best_kernel_grad_evals_per_s": n_grad / (min(kernel_ms) / 1e3),
        "roofline": roof,
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, a.leaf_steps, a.sampler)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
