"""Gradient evaluations per second against the number of chains (the measurement behind Figure 6 /
Section 4.1 of the paper, on this library's kernels).

    python -m paper_1910_11141_amd.throughput_sweep [--config 6] [--iters 20] [--chains 1,2,4,...]
                                                    [--leaf-steps 4] [--sampler 1] [--variant 0]

Configuration 6 has the shape of the paper's own experiment (Bayesian logistic regression, 10 000
synthetic points, 100 regressors, binary32).  For every chain count it prints one JSON line with the
useful gradient evaluations per second (leapfrog steps the chains asked for / kernel time, best of
`--repeats`), the occupancy of the gradient slots and the kernel variant that ran.
"""
import argparse
import json
import sys


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=6)
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--chains", type=str, default="1,2,4,8,16,32,64,128,256,512,1024,2048,4096")
    ap.add_argument("--leaf-steps", type=int, default=1, help="the paper's runs used 4")
    ap.add_argument("--sampler", type=int, default=0, help="0 multinomial, 1 slice (the paper's)")
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--repeats", type=int, default=3, help="timed repetitions per point (best is reported)")
    a = ap.parse_args(argv)

    import torch
    from . import binding as nuts
    from . import workloads

    if not torch.cuda.is_available():
        sys.exit("throughput_sweep needs a GPU")
    w = workloads.make(a.config, n_iters=a.iters)
    tgt = nuts.Target(w.kind, w.dim, w.dtype, precision=w.precision, scales=w.scales, X=w.X, y=w.y,
                      prior_scale=w.prior_scale)
    for n_chains in [int(x) for x in a.chains.split(",")]:
        best, out = None, None
        for _ in range(a.repeats + 1):   # the first run also warms up
            out = nuts.nuts_sample(tgt, n_chains, a.iters, w.step_size, w.max_tree_depth, w.seed, variant=a.variant,
                                   leaf_steps=a.leaf_steps, sampler=a.sampler)
            torch.cuda.synchronize()
            st = nuts.nuts_get_stats(tgt)
            best = st if best is None or st["kernel_ms"] < best["kernel_ms"] else best
        n_grad = int(out[2].sum().item())
        print(json.dumps({"workload": w.name, "n_chains": n_chains, "n_iters": a.iters, "leaf_steps": a.leaf_steps,
                          "sampler": a.sampler, "grad_evals": n_grad,
                          "grad_evals_per_s": n_grad / (best["kernel_ms"] * 1e-3), "ms": best["kernel_ms"],
                          "occupancy": best["occupancy"], "variant": best["variant"]}), flush=True)


if __name__ == "__main__":
    main()
