"""ctypes binding of the program-counter virtual machine (include/pcvm.h): argument marshalling only."""
from __future__ import annotations

import ctypes as C

from . import binding as _b
from .pcvm_programs import Program

PCVM_OK, PCVM_E_INVALID_ARG, PCVM_E_ALLOC, PCVM_E_DEVICE = 0, -1, -2, -3
PCVM_E_STACK_OVERFLOW, PCVM_E_STACK_UNDERFLOW, PCVM_E_STEP_LIMIT = -5, -6, -7
PCVM_MAX_VARS, PCVM_MAX_DEPTH, PCVM_GROUP = 16, 4096, 64
PCVM_SCHED_EARLIEST, PCVM_SCHED_MOST_WAITING = 0, 1

EXPORTS = ("pcvm_run", "pcvm_run_queued", "pcvm_set_stream", "pcvm_last_error")


class pcvm_program(C.Structure):
    _fields_ = [("n_vars", C.c_int32), ("n_inputs", C.c_int32), ("output_var", C.c_int32), ("n_blocks", C.c_int32),
                ("n_ops", C.c_int32), ("reserved", C.c_int32), ("blocks", C.c_void_p), ("ops", C.c_void_p)]


class pcvm_stats(C.Structure):
    _fields_ = [("steps", C.c_uint64), ("active_member_steps", C.c_uint64), ("issued_member_steps", C.c_uint64),
                ("kernel_ms", C.c_double), ("n_groups", C.c_int32), ("reserved", C.c_int32)]


class PcvmError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"pcvm error {code}: {message}")
        self.code = code


_ready = False


def lib() -> C.CDLL:
    global _ready
    L = _b.lib()
    if not _ready:
        L.pcvm_run.argtypes = [C.POINTER(pcvm_program), C.c_int64, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p,
                               C.c_void_p, C.c_int64, C.POINTER(pcvm_stats)]
        L.pcvm_run.restype = C.c_int
        L.pcvm_run_queued.argtypes = [C.POINTER(pcvm_program), C.c_int64, C.c_void_p, C.c_int32, C.c_int64, C.c_int32,
                                      C.c_void_p, C.POINTER(pcvm_stats)]
        L.pcvm_run_queued.restype = C.c_int
        L.pcvm_set_stream.argtypes = [C.c_void_p]
        L.pcvm_set_stream.restype = C.c_int
        L.pcvm_last_error.argtypes = []
        L.pcvm_last_error.restype = C.c_char_p
        _ready = True
    return L


def pcvm_last_error() -> str:
    return (lib().pcvm_last_error() or b"").decode()


def describe(program: Program) -> pcvm_program:
    """The C view of a program table (keeps the numpy arrays alive through attributes of the result)."""
    p = pcvm_program(program.n_vars, program.n_inputs, program.output_var, len(program.blocks), len(program.ops), 0,
                     program.blocks.ctypes.data, program.ops.ctypes.data if len(program.ops) else None)
    p._keep = (program.blocks, program.ops)
    return p


def pcvm_run(program: Program, inputs, stack_depth: int, max_steps: int = 1 << 40, trace_capacity: int = 0,
             queued: bool = False, policy: int = PCVM_SCHED_EARLIEST):
    """inputs: CUDA int64 tensor [n_inputs, batch] (or [batch] for one input).
    Returns (outputs [batch] CUDA int64, stats dict, trace [n, 2] CUDA int32 or None).
    queued=True calls pcvm_run_queued (members handed to lanes from a queue; no trace)."""
    import torch

    dev = torch.device("cuda", torch.cuda.current_device()) if torch.cuda.is_available() else None
    if dev is None:
        batch = int(inputs.shape[-1])
        rc = lib().pcvm_run(C.byref(describe(program)), batch, None, int(stack_depth), int(max_steps), None, None, 0, None)
        raise PcvmError(rc, pcvm_last_error())
    inputs = inputs.reshape(program.n_inputs, -1)
    assert inputs.is_cuda and inputs.dtype == torch.int64 and inputs.is_contiguous()
    batch = int(inputs.shape[1])
    out = torch.empty(batch, dtype=torch.int64, device=dev)
    trace = torch.full((trace_capacity, 2), -1, dtype=torch.int32, device=dev) if trace_capacity else None
    st = pcvm_stats()
    if queued:
        assert not trace_capacity, "a queued run has no trace"
        rc = lib().pcvm_run_queued(C.byref(describe(program)), batch, C.c_void_p(inputs.data_ptr()), int(stack_depth),
                                   int(max_steps), int(policy), C.c_void_p(out.data_ptr()), C.byref(st))
    else:
        rc = lib().pcvm_run(C.byref(describe(program)), batch, C.c_void_p(inputs.data_ptr()), int(stack_depth),
                            int(max_steps), C.c_void_p(out.data_ptr()),
                            C.c_void_p(trace.data_ptr()) if trace is not None else None, int(trace_capacity),
                            C.byref(st))
    if rc != PCVM_OK:
        raise PcvmError(rc, pcvm_last_error())
    stats = {"steps": st.steps, "active_member_steps": st.active_member_steps,
             "issued_member_steps": st.issued_member_steps, "kernel_ms": st.kernel_ms, "n_groups": st.n_groups,
             "utilization": st.active_member_steps / max(1, st.issued_member_steps)}
    return out, stats, trace
