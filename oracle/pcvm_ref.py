"""Reference ("oracle") interpreter for program-counter autobatching: Algorithm 2 of the paper, step by step.

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the smoke check; the product never imports it.  It is
written for clarity with the paper's names (pc, pc_stack, x_stack, the locally active set A, masking style,
"run the earliest block"), in plain numpy over [depth, batch] arrays, and shares no code with the HIP runtime.
It decodes the same program tables (paper_1910_11141_amd/pcvm_programs.py only describes programs).

Readings of the paper (Section 3, Algorithm 2, Figures 3 and 5):
  * A stack index counts the entries of its stack (Figure 3 prints them that way); the top is entry index - 1.
  * The program-counter stack holds one entry per live frame: PushJump i j sets the current frame's entry to the
    return block j and pushes the callee's entry block i; Return pops.  A batch member whose program-counter
    stack is empty has halted (its pc^top reads I, the number of blocks).
  * Variables hold 64-bit integers with wrap-around arithmetic.  Operations are total, so that the junk a masked
    lane computes can never fault: x mod 0 = 0, shifts use the low 6 bits of the count.
  * Update y = f(x) overwrites the top entry in place (the Pop-then-Push pair that the fifth optimisation of
    Section 3.2 cancels).  A variable that is never pushed keeps index 0 and lives in row 0 (the third
    optimisation: no stack is needed for it).
  * The batch may be cut into groups of `group` members that are scheduled independently (each takes the earliest
    block among its own members); group = batch size is the algorithm exactly as printed.  Results do not depend
    on the grouping (Section 3, "Why does this work?").
"""
from __future__ import annotations

import numpy as np

PUSH, UPDATE, POP = 0, 1, 2
(CONST, COPY, ADD, SUB, MUL, ADDI, MULI, LE, LT, EQ, LEI, EQI, MOD, ANDI, SHRI) = range(15)
JUMP, BRANCH, PUSHJUMP, RETURN = 0, 1, 2, 3


class StackOverflow(RuntimeError):
    pass


class StepLimit(RuntimeError):
    pass


def primitive(fn, a, b, imm):
    """y = f(a, b, imm) element-wise on int64 arrays, wrap-around."""
    with np.errstate(over="ignore"):
        imm = np.int64(imm)
        if fn == CONST:
            return np.full_like(a, imm)
        if fn == COPY:
            return a.copy()
        if fn == ADD:
            return a + b
        if fn == SUB:
            return a - b
        if fn == MUL:
            return a * b
        if fn == ADDI:
            return a + imm
        if fn == MULI:
            return a * imm
        if fn == LE:
            return (a <= b).astype(np.int64)
        if fn == LT:
            return (a < b).astype(np.int64)
        if fn == EQ:
            return (a == b).astype(np.int64)
        if fn == LEI:
            return (a <= imm).astype(np.int64)
        if fn == EQI:
            return (a == imm).astype(np.int64)
        if fn == MOD:       # truncated remainder (sign of the dividend), 0 for a zero or -1 divisor
            safe = np.where((b == 0) | (b == -1), np.int64(1), b)
            r = np.fmod(a, safe)
            return np.where((b == 0) | (b == -1), np.int64(0), r)
        if fn == ANDI:
            return a & imm
        if fn == SHRI:      # arithmetic shift
            return a >> np.int64(int(imm) & 63)
    raise ValueError(f"unknown primitive {fn}")


class Machine:
    """State of Algorithm 2 for one group of Z batch members."""

    def __init__(self, program, inputs, depth):
        self.P = program
        self.I = len(program.blocks)
        self.D = int(depth)
        inputs = np.asarray(inputs, dtype=np.int64).reshape(program.n_inputs, -1)
        self.Z = inputs.shape[1]
        # program counter with a stack dimension of its own, and its stack indexes
        self.pc = np.zeros((self.D, self.Z), dtype=np.int64)
        self.pc_stack = np.zeros(self.Z, dtype=np.int64)
        # every variable: zeros with leading dimensions D, Z, and a stack index per member
        self.var = np.zeros((program.n_vars, self.D, self.Z), dtype=np.int64)
        self.var_stack = np.zeros((program.n_vars, self.Z), dtype=np.int64)
        everyone = np.ones(self.Z, dtype=bool)
        for v in range(program.n_inputs):       # PUSH T onto x
            self._push(v, inputs[v], everyone)
        self._push_pc(np.zeros(self.Z, dtype=np.int64), everyone)   # every member waits at block 0
        self.steps = 0
        self.active_member_steps = 0
        self.trace = []     # (block executed, number of locally active members) per step

    # ---- stacks
    def _top(self, v):
        idx = np.maximum(self.var_stack[v] - 1, 0)
        return self.var[v, idx, np.arange(self.Z)]

    def _push(self, v, values, A):
        if (self.var_stack[v][A] >= self.D).any():
            raise StackOverflow(f"stack of variable {self.P.var_names[v]} exceeds depth {self.D}")
        cols = np.nonzero(A)[0]
        self.var[v, self.var_stack[v][cols], cols] = values[cols]
        self.var_stack[v][cols] += 1

    def _update(self, v, values, A):
        cols = np.nonzero(A)[0]
        self.var[v, np.maximum(self.var_stack[v][cols] - 1, 0), cols] = values[cols]

    def _pop(self, v, A):
        if (self.var_stack[v][A] <= 0).any():
            raise RuntimeError(f"pop from the empty stack of variable {self.P.var_names[v]}")
        self.var_stack[v][A] -= 1

    def pc_top(self):
        idx = np.maximum(self.pc_stack - 1, 0)
        top = self.pc[idx, np.arange(self.Z)]
        return np.where(self.pc_stack > 0, top, self.I)

    def _push_pc(self, values, A):
        if (self.pc_stack[A] >= self.D).any():
            raise StackOverflow(f"program-counter stack exceeds depth {self.D}")
        cols = np.nonzero(A)[0]
        self.pc[self.pc_stack[cols], cols] = values[cols]
        self.pc_stack[cols] += 1

    def _set_pc_top(self, values, A):
        cols = np.nonzero(A)[0]
        self.pc[self.pc_stack[cols] - 1, cols] = values[cols]

    # ---- one pass of the while loop
    def halted(self):
        return bool((self.pc_top() >= self.I).all())

    def step(self):
        pc_top = self.pc_top()
        i = int(pc_top.min())                  # the earliest block anyone waits for
        A = pc_top == i                        # locally active set
        blk = self.P.blocks[i]
        for op in self.P.ops[blk["first_op"]: blk["first_op"] + blk["n_ops"]]:
            if op["kind"] == POP:
                self._pop(op["dst"], A)
                continue
            o = primitive(op["fn"], self._top(op["a"]), self._top(op["b"]), op["imm"])   # on all members: masking
            if op["kind"] == PUSH:
                self._push(op["dst"], o, A)
            else:
                self._update(op["dst"], o, A)
        t = blk["term"]
        full = lambda value: np.full(self.Z, value, dtype=np.int64)
        if t == JUMP:
            self._set_pc_top(full(blk["i"]), A)
        elif t == BRANCH:
            x_top = self._top(blk["x"])
            self._set_pc_top(np.where(x_top != 0, blk["i"], blk["j"]).astype(np.int64), A)
        elif t == PUSHJUMP:
            self._set_pc_top(full(blk["j"]), A)     # where this frame resumes
            self._push_pc(full(blk["i"]), A)        # the callee's entry
        elif t == RETURN:
            self.pc_stack[A] -= 1
        else:
            raise ValueError(f"unknown terminator {t}")
        self.steps += 1
        self.active_member_steps += int(A.sum())
        self.trace.append((i, int(A.sum())))

    def output(self):
        return self._top(self.P.output_var)

    # ---- views used by the pins
    def stack_of(self, name, member):
        v = self.P.var_names.index(name)
        return [int(x) for x in self.var[v, : self.var_stack[v, member], member]]

    def pc_stack_of(self, member, as_labels=True):
        entries = [int(x) for x in self.pc[: self.pc_stack[member], member]]
        return [self.P.labels[e] for e in entries] if as_labels else entries


def run(program, inputs, depth, group=None, max_steps=10_000_000):
    """Run to completion.  Returns (outputs [batch], stats dict, trace of the first group)."""
    inputs = np.asarray(inputs, dtype=np.int64).reshape(program.n_inputs, -1)
    Z = inputs.shape[1]
    group = Z if group is None else int(group)
    out = np.zeros(Z, dtype=np.int64)
    steps = active = issued = 0
    first_trace = None
    for g0 in range(0, Z, group):
        m = Machine(program, inputs[:, g0: g0 + group], depth)
        while not m.halted():
            if m.steps >= max_steps:
                raise StepLimit(f"no halt within {max_steps} steps")
            m.step()
        out[g0: g0 + group] = m.output()
        steps += m.steps
        active += m.active_member_steps
        issued += m.steps * group          # every lane of the group takes part in every step, masked or not
        if first_trace is None:
            first_trace = m.trace
    return out, {"steps": steps, "active_member_steps": active, "issued_member_steps": issued}, first_trace
