"""Gradient-slot utilisation against the number of chains, for both schedules (the measurement behind
Figure 7 / Section 4.2 of the paper, on this library's kernels).

    python -m paper_1910_11141_amd.utilization_sweep [--config 2] [--iters 10] [--chains 1,2,4,...]
                                                     [--leaf-steps 4] [--variant 1]

For every chain count it runs the same workload twice, once free-running (gradient steps of different
iterations share a batch) and once synchronised at trajectory boundaries, checks that the outputs are
identical, and prints one JSON line with the occupancy nuts_get_stats reports (useful gradient slots /
issued slots) and the measured gradient evaluations per second of each schedule.
"""
import argparse
import json
import sys


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--iters", type=int, default=10, help="trajectories per chain (the paper's figure batches across 10)")
    ap.add_argument("--chains", type=str, default="1,2,4,8,16,32,64,128,256,512,1024")
    ap.add_argument("--leaf-steps", type=int, default=1)
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--repeats", type=int, default=3, help="timed repetitions per point (best is reported)")
    a = ap.parse_args(argv)

    import torch
    from . import binding as nuts
    from . import workloads

    if not torch.cuda.is_available():
        sys.exit("utilization_sweep needs a GPU")
    w = workloads.make(a.config, n_iters=a.iters)
    tgt = nuts.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                      prior_scale=w.prior_scale)
    for n_chains in [int(x) for x in a.chains.split(",")]:
        point = {"workload": w.name, "n_chains": n_chains, "n_iters": a.iters, "leaf_steps": a.leaf_steps}
        outs = {}
        for name, schedule in (("free", nuts.NUTS_SCHEDULE_FREE), ("trajectory", nuts.NUTS_SCHEDULE_TRAJECTORY)):
            best = None
            for _ in range(a.repeats):
                out = nuts.nuts_sample(tgt, n_chains, a.iters, w.step_size, w.max_tree_depth, w.seed,
                                       variant=a.variant, leaf_steps=a.leaf_steps, schedule=schedule)
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


if __name__ == "__main__":
    main()
