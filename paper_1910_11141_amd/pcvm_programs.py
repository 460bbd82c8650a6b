"""Program tables for the program-counter virtual machine: inputs shared by the HIP runtime and the CPU oracle.

This module only *describes* programs in the control-flow-graph language of Figure 4 of the paper
(blocks of Push / Pop operations ending in Jump, Branch, PushJump or Return) and encodes them as flat
integer tables.  It evaluates nothing: what an operation means is implemented once in the HIP runtime
and once, independently, in the oracle.

Encoding (little-endian, C layout, the same as `pcvm_op` / `pcvm_block` in include/pcvm.h):
    op    = (kind, fn, dst, a, b, pad: int32; imm: int64)                     32 bytes
    block = (first_op, n_ops, term, x, i, j, label, pad: int32)               32 bytes
Variables are numbered 0..n_vars-1 and hold 64-bit integers; variables 0..n_inputs-1 receive the inputs.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# operation kinds
PUSH, UPDATE, POP = 0, 1, 2          # UPDATE writes the top of the stack in place (a Pop followed by a Push, fused)
# primitive functions f of  y = f(a, b, imm)
CONST, COPY, ADD, SUB, MUL, ADDI, MULI, LE, LT, EQ, LEI, EQI, MOD, ANDI, SHRI = range(15)
# terminators
JUMP, BRANCH, PUSHJUMP, RETURN = 0, 1, 2, 3

OP_DTYPE = np.dtype([("kind", "<i4"), ("fn", "<i4"), ("dst", "<i4"), ("a", "<i4"), ("b", "<i4"), ("pad", "<i4"),
                     ("imm", "<i8")])
BLOCK_DTYPE = np.dtype([("first_op", "<i4"), ("n_ops", "<i4"), ("term", "<i4"), ("x", "<i4"), ("i", "<i4"),
                        ("j", "<i4"), ("label", "<i4"), ("pad", "<i4")])


@dataclass
class Program:
    name: str
    var_names: list
    n_inputs: int
    output_var: int
    ops: np.ndarray       # OP_DTYPE
    blocks: np.ndarray    # BLOCK_DTYPE
    labels: list = field(default_factory=list)   # source line of every block (documentation and figures)

    @property
    def n_vars(self):
        return len(self.var_names)


class _Builder:
    def __init__(self, name, var_names, n_inputs, output):
        self.name, self.vars, self.n_inputs = name, list(var_names), n_inputs
        self.output = self.vars.index(output)
        self.ops, self.blocks, self.names = [], [], {}

    def v(self, name):
        return self.vars.index(name)

    def block(self, name, label, ops, term):
        """ops: tuples (kind, dst, fn, a, b, imm) with variable names; term: (JUMP, i) | (BRANCH, x, i, j) |
        (PUSHJUMP, callee, return_to) | (RETURN,) with block names."""
        self.names[name] = len(self.blocks)
        self.blocks.append((name, label, ops, term))

    def build(self) -> Program:
        ops, blocks = [], []
        for name, label, bops, term in self.blocks:
            first = len(ops)
            for kind, dst, fn, a, b, imm in bops:
                ops.append((kind, fn, self.v(dst), self.v(a) if a is not None else 0,
                            self.v(b) if b is not None else 0, 0, imm))
            t = term[0]
            x = self.v(term[1]) if t == BRANCH else 0
            i = self.names[term[2 if t == BRANCH else 1]] if t != RETURN else 0
            j = self.names[term[3 if t == BRANCH else 2]] if t in (BRANCH, PUSHJUMP) else 0
            blocks.append((first, len(bops), t, x, i, j, label, 0))
        return Program(self.name, self.vars, self.n_inputs, self.output, np.array(ops, dtype=OP_DTYPE),
                       np.array(blocks, dtype=BLOCK_DTYPE), [b[1] for b in self.blocks])


def push(dst, fn, a=None, b=None, imm=0):
    return (PUSH, dst, fn, a, b, imm)


def update(dst, fn, a=None, b=None, imm=0):
    return (UPDATE, dst, fn, a, b, imm)


def pop(x):
    return (POP, x, COPY, None, None, 0)


def fibonacci() -> Program:
    """The recursive Fibonacci program of Figures 1 and 3 of the paper (fib(0) = fib(1) = 1), lowered by hand
    to the language of Figure 4.  Block labels are the source lines a block starts at (2, 4, 6, 7, 9), as in
    the figures.  `n` and `left` are the two variables that live across a recursive call and so keep stacks;
    `cond`, `right` and `ret` never do (they only ever use the top entry).  The callee pops its own `n`; the
    caller's `n` is last used for the second call's argument, so the pop of the old `n` and the push of the
    callee's cancel into one in-place update (the fifth optimisation of Section 3.2)."""
    b = _Builder("fibonacci", ["n", "left", "ret", "cond", "right"], 1, "ret")
    b.block("L2", 2, [update("cond", LEI, "n", imm=1)], (BRANCH, "cond", "L4", "L6"))
    b.block("L4", 4, [update("ret", CONST, imm=1), pop("n")], (RETURN,))
    b.block("L6", 6, [push("n", ADDI, "n", imm=-2)], (PUSHJUMP, "L2", "L7"))
    b.block("L7", 7, [push("left", COPY, "ret"), update("n", ADDI, "n", imm=-1)], (PUSHJUMP, "L2", "L9"))
    b.block("L9", 9, [update("right", COPY, "ret"), update("ret", ADD, "left", "right"), pop("left")], (RETURN,))
    return b.build()


def collatz_steps() -> Program:
    """Number of Collatz steps from n >= 1 down to 1: a data-dependent loop, no recursion."""
    b = _Builder("collatz_steps", ["n", "steps", "c", "t"], 1, "steps")
    b.block("init", 1, [update("steps", CONST, imm=0)], (JUMP, "test"))
    b.block("test", 2, [update("c", LEI, "n", imm=1)], (BRANCH, "c", "done", "body"))
    b.block("body", 3, [update("steps", ADDI, "steps", imm=1), update("c", ANDI, "n", imm=1)],
            (BRANCH, "c", "odd", "even"))
    b.block("odd", 4, [update("t", MULI, "n", imm=3), update("n", ADDI, "t", imm=1)], (JUMP, "test"))
    b.block("even", 5, [update("n", SHRI, "n", imm=1)], (JUMP, "test"))
    b.block("done", 6, [], (RETURN,))
    return b.build()


def gcd() -> Program:
    """Euclid, written as a tail-recursive call: gcd(a, b) = a if b == 0 else gcd(b, a mod b)."""
    p = _Builder("gcd", ["a", "b", "ret", "c", "t"], 2, "ret")
    p.block("entry", 1, [update("c", EQI, "b", imm=0)], (BRANCH, "c", "base", "rec"))
    p.block("base", 2, [update("ret", COPY, "a"), pop("a"), pop("b")], (RETURN,))
    p.block("rec", 3, [update("t", MOD, "a", "b"), push("a", COPY, "b"), push("b", COPY, "t")],
            (PUSHJUMP, "entry", "after"))
    p.block("after", 4, [pop("a"), pop("b")], (RETURN,))
    return p.build()


def parity() -> Program:
    """is_even(n) through the mutually recursive pair is_even / is_odd: two functions calling each other."""
    p = _Builder("parity", ["n", "ret", "c"], 1, "ret")
    p.block("even", 1, [update("c", EQI, "n", imm=0)], (BRANCH, "c", "even_base", "even_rec"))
    p.block("even_base", 2, [update("ret", CONST, imm=1), pop("n")], (RETURN,))
    p.block("even_rec", 3, [update("n", ADDI, "n", imm=-1)], (PUSHJUMP, "odd", "leave"))
    p.block("odd", 4, [update("c", EQI, "n", imm=0)], (BRANCH, "c", "odd_base", "odd_rec"))
    p.block("odd_base", 5, [update("ret", CONST, imm=0), pop("n")], (RETURN,))
    p.block("odd_rec", 6, [update("n", ADDI, "n", imm=-1)], (PUSHJUMP, "even", "leave"))
    p.block("leave", 7, [], (RETURN,))
    return p.build()


def binomial() -> Program:
    """C(n, k) = C(n-1, k-1) + C(n-1, k) with C(n, 0) = C(n, n) = 1: two arguments, a full binary call tree."""
    p = _Builder("binomial", ["n", "k", "left", "ret", "c", "d", "right"], 2, "ret")
    p.block("entry", 1, [update("c", EQI, "k", imm=0), update("d", EQ, "n", "k"), update("c", ADD, "c", "d")],
            (BRANCH, "c", "base", "first"))
    p.block("base", 2, [update("ret", CONST, imm=1), pop("n"), pop("k")], (RETURN,))
    p.block("first", 3, [push("n", ADDI, "n", imm=-1), push("k", ADDI, "k", imm=-1)], (PUSHJUMP, "entry", "second"))
    p.block("second", 4, [push("left", COPY, "ret"), update("n", ADDI, "n", imm=-1)], (PUSHJUMP, "entry", "sum"))
    p.block("sum", 5, [update("right", COPY, "ret"), update("ret", ADD, "left", "right"), pop("left")], (RETURN,))
    return p.build()


def ackermann() -> Program:
    """Ackermann's function A(m, n): a call whose argument is the result of another call."""
    p = _Builder("ackermann", ["m", "n", "ret", "c"], 2, "ret")
    p.block("entry", 1, [update("c", EQI, "m", imm=0)], (BRANCH, "c", "m0", "mpos"))
    p.block("m0", 2, [update("ret", ADDI, "n", imm=1), pop("m"), pop("n")], (RETURN,))
    p.block("mpos", 3, [update("c", EQI, "n", imm=0)], (BRANCH, "c", "n0", "npos"))
    # A(m, 0) = A(m-1, 1): the frame's own arguments are dead, so they are overwritten for the callee
    p.block("n0", 4, [update("m", ADDI, "m", imm=-1), update("n", CONST, imm=1)], (PUSHJUMP, "entry", "leave"))
    # A(m, n) = A(m-1, A(m, n-1)): inner call on pushed copies, outer call reuses this frame's m
    p.block("npos", 5, [push("n", ADDI, "n", imm=-1), push("m", COPY, "m")], (PUSHJUMP, "entry", "outer"))
    p.block("outer", 6, [update("m", ADDI, "m", imm=-1), update("n", COPY, "ret")], (PUSHJUMP, "entry", "leave"))
    p.block("leave", 7, [], (RETURN,))
    return p.build()


ALL = {"fibonacci": fibonacci, "collatz_steps": collatz_steps, "gcd": gcd, "parity": parity, "binomial": binomial,
       "ackermann": ackermann}


# ---------------------------------------------------------------------------------------------------------------
# The same Fibonacci program in the language of Figure 2 (functions whose blocks hold Primitive and Call
# operations): the input of *local static* autobatching (Algorithm 1), which only the CPU oracle implements.
# A function is (inputs, output, blocks); a block is (label, ops, terminator) with
#   ops:        ("prim", y, fn, a, b, imm) | ("call", y, function name, [argument variables])
#   terminator: ("jump", block) | ("branch", x, block_if_true, block_if_false) | ("return",)

def fibonacci_local():
    fib = {
        "inputs": ["n"], "output": "ret",
        "blocks": [
            (2, [("prim", "cond", LEI, "n", None, 1)], ("branch", "cond", 1, 2)),
            (4, [("prim", "ret", CONST, None, None, 1)], ("return",)),
            (6, [("prim", "n2", ADDI, "n", None, -2)], ("jump", 3)),
            (7, [("call", "left", "fibonacci", ["n2"]), ("prim", "n1", ADDI, "n", None, -1)], ("jump", 4)),
            (9, [("call", "right", "fibonacci", ["n1"]), ("prim", "ret", ADD, "left", "right", 0)], ("return",)),
        ],
    }
    return {"fibonacci": fib}
