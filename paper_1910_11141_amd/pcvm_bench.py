"""Throughput of the program-counter virtual machine on one MI355X.

    python -m paper_1910_11141_amd.pcvm_bench [--program fibonacci] [--batch 1048576] [--max-input 20]

Prints one JSON line: scheduler steps and member-steps per second of the interpreter kernel, and the
utilisation (members that executed a block / members the masked execution paid for)."""
import argparse
import json
import sys


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--program", default="fibonacci")
    ap.add_argument("--batch", type=int, default=1 << 20)
    ap.add_argument("--max-input", type=int, default=20)
    ap.add_argument("--depth", type=int, default=32)
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--sorted", action="store_true", help="sort the inputs so that a group holds similar work")
    ap.add_argument("--queued", action="store_true", help="hand members to lanes from a queue (pcvm_run_queued)")
    ap.add_argument("--policy", type=int, default=0, help="queued runs: 0 earliest block, 1 block most lanes wait for")
    a = ap.parse_args(argv)

    import torch
    from . import pcvm, pcvm_programs

    if not torch.cuda.is_available():
        sys.exit("pcvm_bench needs a GPU")
    prog = pcvm_programs.ALL[a.program]()
    g = torch.Generator(device="cpu").manual_seed(1910_11141)
    ins = torch.randint(1, a.max_input + 1, (prog.n_inputs, a.batch), generator=g, dtype=torch.int64)
    if a.sorted:
        ins = ins[:, torch.argsort(ins[0])]
    ins = ins.cuda().contiguous()
    best = None
    for _ in range(a.repeats):
        out, st, _ = pcvm.pcvm_run(prog, ins, a.depth, queued=a.queued, policy=a.policy)
        best = st if best is None or st["kernel_ms"] < best["kernel_ms"] else best
    s = best["kernel_ms"] * 1e-3
    print(json.dumps({"program": prog.name, "batch": a.batch, "max_input": a.max_input, "sorted": a.sorted, "queued": a.queued,
                      "policy": ["earliest", "most-waiting"][a.policy],
                      "kernel_ms": best["kernel_ms"], "group_steps_per_s": best["steps"] / s,
                      "active_member_steps_per_s": best["active_member_steps"] / s,
                      "issued_member_steps_per_s": best["issued_member_steps"] / s,
                      "utilization": best["utilization"], "checksum": int(out.sum().item())}))


if __name__ == "__main__":
    main()
