"""Reference interpreter for *local static* autobatching: Algorithm 1 of the paper, step by step.

TEST INFRASTRUCTURE ONLY (see oracle/pcvm_ref.py).  The batching follows the control structure of the
program: recursion is carried by the host language (this Python function calls itself), each call works on the
locally active members of its caller, and members at different call depths can never share a block execution.
It exists as the comparison point of Sections 2 and 4.2: the same programs run under Algorithm 2 need no more,
and usually fewer, block executions.  Primitives are the oracle's own (pcvm_ref.primitive)."""
from __future__ import annotations

import numpy as np

from .pcvm_ref import primitive


class Run:
    def __init__(self, program, observer=None):
        self.program = program
        self.frames = []            # the host call stack: one dict per active call
        self.block_executions = 0
        self.active_member_steps = 0
        self.observer = observer    # called with (self) before every block execution

    def call(self, name, args, A):
        """Local-static(F, Z, x, A): run function `name` for the members of the active set A."""
        F = self.program[name]
        Z = A.size
        I = len(F["blocks"])
        pc = np.zeros(Z, dtype=np.int64)             # "Initialize length Z program counter"
        var = {v: a.copy() for v, a in zip(F["inputs"], args)}
        assigned = {v: A.copy() for v in F["inputs"]}
        returned_at = np.full(Z, -1, dtype=np.int64)  # label of the block a member returned from (for the figures)
        frame = {"function": name, "A": A, "pc": pc, "var": var, "assigned": assigned, "returned_at": returned_at,
                 "labels": [b[0] for b in F["blocks"]]}
        self.frames.append(frame)
        zeros = np.zeros(Z, dtype=np.int64)

        def write(y, values, mask):
            if y not in var:
                var[y] = zeros.copy()
                assigned[y] = np.zeros(Z, dtype=bool)
            var[y][mask] = values[mask]
            assigned[y] |= mask

        while (pc[A] < I).any():
            i = int(pc[A].min())
            local = A & (pc == i)                    # locally active set A'
            if self.observer:
                self.observer(self)
            label, ops, term = F["blocks"][i]
            self.block_executions += 1
            self.active_member_steps += int(local.sum())
            for op in ops:
                if op[0] == "prim":
                    _, y, fn, a, b, imm = op
                    o = primitive(fn, var.get(a, zeros), var.get(b, zeros), imm)
                    write(y, o, local)
                else:
                    _, y, callee, arg_names = op
                    frame["in_call"] = True
                    o = self.call(callee, [var[v] for v in arg_names], local)     # recursion in the host language
                    frame["in_call"] = False
                    write(y, o, local)
            if term[0] == "jump":
                pc[local] = term[1]
            elif term[0] == "branch":
                x = var[term[1]]
                pc[local] = np.where(x[local] != 0, term[2], term[3])
            else:
                returned_at[local] = label
                pc[local] = I
        self.frames.pop()
        return var[F["output"]]


def run(program, entry, inputs, observer=None):
    inputs = np.asarray(inputs, dtype=np.int64).reshape(len(program[entry]["inputs"]), -1)
    r = Run(program, observer)
    out = r.call(entry, [row for row in inputs], np.ones(inputs.shape[1], dtype=bool))
    return out, {"block_executions": r.block_executions, "active_member_steps": r.active_member_steps,
                 "issued_member_steps": r.block_executions * inputs.shape[1]}
