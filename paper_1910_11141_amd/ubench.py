"""Instruction-issue microbenchmark of one MI355X compute unit (csrc/ubench/issue_ubench.hip).

    python -m paper_1910_11141_amd.ubench            # prints the table that profiles/ keeps

Measures how many shader-clock ticks a SIMD needs per binary64 MFMA and per vector instruction, and
whether the two overlap (a) when they come from two waves of one SIMD and (b) inside one wave's own
instruction stream; then fills the chip with binary64 MFMAs to see which rate it sustains.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnuts_ubench.so")

MIX = {"idle": 0, "mfma_f64_16x16x4": 1, "mfma_f64_16x16x4_dependent": 2, "v_fma_f64": 3, "v_fma_f32": 4,
       "v_xor_b32": 5, "v_mul_hi_u32": 6, "ds_read_b128": 7, "mfma_f64+4*v_fma_f64 (one wave)": 8,
       "mfma_f64+4*v_fma_f32 (one wave)": 9, "mfma_f64+4*v_xor_b32 (one wave)": 10, "mfma_f64_4x4x4_4b": 11,
       "mfma_f32_32x32x2": 12, "mfma_f32+4*v_fma_f32 (one wave)": 13, "v_exp_f32": 14,
       "mfma_f64+ds_read_b128 (one wave)": 15, "mfma_f64_4x4x4_4b_dependent": 16,
       "mfma_f32_4x4x1_16b": 17, "mfma_f32_4x4x1_16b_dependent": 18}

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with __graft_entry__.build()")
        import torch  # noqa: F401  (one HIP runtime per process: torch's comes first)
        L = C.CDLL(LIB_PATH)
        L.nuts_ubench_pair.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double)]
        L.nuts_ubench_mfma_peak.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.nuts_ubench_fill.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.nuts_ubench_logistic.argtypes = [C.c_void_p, C.c_longlong, C.c_void_p, C.c_void_p]
        L.nuts_ubench_log_unit.argtypes = [C.c_void_p, C.c_longlong, C.c_void_p]
        L.nuts_ubench_circle_point.argtypes = [C.c_void_p, C.c_longlong, C.c_void_p, C.c_void_p]
        L.nuts_ubench_exp_bounded.argtypes = [C.c_void_p, C.c_longlong, C.c_void_p]
        L.nuts_ubench_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def pair(mix_a: str, mix_b: str, iters: int = 2000) -> dict:
    """Waves 0..3 run mix_a, waves 4..7 mix_b (wave w and w+4 share a SIMD).  Returns, per side, the mean
    ticks per instruction (per group for the one-wave mixes) and the mean loop duration in ticks."""
    out = (C.c_double * 48)()
    rc = lib().nuts_ubench_pair(MIX[mix_a], MIX[mix_b], iters, out)
    if rc:
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    rows = [list(out[6 * w:6 * w + 6]) for w in range(8)]
    res = {"simd": [int(r[2]) for r in rows]}
    for side, ws in (("a", range(0, 4)), ("b", range(4, 8))):
        ticks = sum(rows[w][0] for w in ws) / 4
        wall = sum(rows[w][1] for w in ws) / 4
        n = rows[ws[0]][4]
        res[side] = {"ticks": ticks, "per_instr": ticks / n if n else float("nan"),
                     "shader_mhz": ticks / wall * 100.0 if wall else float("nan")}
    return res


def mfma_peak(blocks: int = 256 * 8, iters: int = 20000, reps: int = 3):
    t, ms = C.c_double(), C.c_double()
    rc = lib().nuts_ubench_mfma_peak(blocks, iters, reps, C.byref(t), C.byref(ms))
    if rc:
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    return t.value, ms.value


def fill(mix: str, blocks: int = 256 * 4, iters: int = 20000, reps: int = 3):
    """The whole chip on one mix: (binary64 matrix TFLOP/s, ms per launch)."""
    t, ms = C.c_double(), C.c_double()
    rc = lib().nuts_ubench_fill(MIX[mix], blocks, iters, reps, C.byref(t), C.byref(ms))
    if rc:
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    return t.value, ms.value


def logistic(z):
    """log(2 cosh(z/2)) and (1/2) tanh(|z|/2) as the sampler kernels compute them (z: CUDA float64 tensor)."""
    import torch
    assert z.is_cuda and z.dtype == torch.float64 and z.is_contiguous()
    a, b = torch.empty_like(z), torch.empty_like(z)
    torch.cuda.synchronize()
    if lib().nuts_ubench_logistic(z.data_ptr(), z.numel(), a.data_ptr(), b.data_ptr()):
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    return a, b


def log_unit(x):
    """log(x) for 0 < x <= 1 as the gradient loop of the tile kernel computes it (x: CUDA float64 tensor)."""
    import torch
    assert x.is_cuda and x.dtype == torch.float64 and x.is_contiguous()
    out = torch.empty_like(x)
    torch.cuda.synchronize()
    if lib().nuts_ubench_log_unit(x.data_ptr(), x.numel(), out.data_ptr()):
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    return out


def circle_point(phi):
    """(sin(phi), cos(phi)) for 0 <= phi <= 2 pi as the tile kernel's Box-Muller draws compute them (phi: CUDA
    float64 tensor)."""
    import torch
    assert phi.is_cuda and phi.dtype == torch.float64 and phi.is_contiguous()
    sn, cs = torch.empty_like(phi), torch.empty_like(phi)
    torch.cuda.synchronize()
    if lib().nuts_ubench_circle_point(phi.data_ptr(), phi.numel(), sn.data_ptr(), cs.data_ptr()):
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    return sn, cs


def exp_bounded(x):
    """exp(x) for x <= 700 as the tile kernel turns energy errors into weights (x: CUDA float64 tensor)."""
    import torch
    assert x.is_cuda and x.dtype == torch.float64 and x.is_contiguous()
    out = torch.empty_like(x)
    torch.cuda.synchronize()
    if lib().nuts_ubench_exp_bounded(x.data_ptr(), x.numel(), out.data_ptr()):
        raise RuntimeError(lib().nuts_ubench_last_error().decode())
    return out


def report() -> str:
    lines = ["# one workgroup of 8 waves on one compute unit; waves w and w+4 share a SIMD (SIMD ids as read: "
             + str(pair("idle", "idle", 1)["simd"]) + ")",
             "# ticks = shader clock (s_memtime); per instruction, mean over the 4 waves of a side", ""]
    lines.append(f"{'alone (other side idle)':44s} {'ticks/instr':>12s} {'shader MHz':>11s}")
    alone = {}
    for name in MIX:
        if name == "idle":
            continue
        r = pair(name, "idle")
        alone[name] = r["a"]["ticks"]
        lines.append(f"{name:44s} {r['a']['per_instr']:12.2f} {r['a']['shader_mhz']:11.0f}")
    lines += ["", "two waves of one SIMD, each with its own mix: loop durations alone and side by side",
              f"{'A':28s} {'B':16s} {'A alone':>10s} {'B alone':>10s} {'A beside B':>11s} {'B beside A':>11s} {'sum':>10s} {'max':>10s}"]
    for b in ("v_fma_f64", "v_fma_f32", "v_xor_b32", "v_mul_hi_u32", "v_exp_f32", "ds_read_b128", "mfma_f64_16x16x4"):
        a = "mfma_f64_16x16x4"
        r = pair(a, b)
        lines.append(f"{a:28s} {b:16s} {alone[a]:10.0f} {alone[b]:10.0f} {r['a']['ticks']:11.0f} {r['b']['ticks']:11.0f} "
                     f"{alone[a] + alone[b]:10.0f} {max(alone[a], alone[b]):10.0f}")
    r = pair("mfma_f32_32x32x2", "v_fma_f32")
    lines.append(f"{'mfma_f32_32x32x2':28s} {'v_fma_f32':16s} {alone['mfma_f32_32x32x2']:10.0f} {alone['v_fma_f32']:10.0f} "
                 f"{r['a']['ticks']:11.0f} {r['b']['ticks']:11.0f} {alone['mfma_f32_32x32x2'] + alone['v_fma_f32']:10.0f} "
                 f"{max(alone['mfma_f32_32x32x2'], alone['v_fma_f32']):10.0f}")
    lines += ["", "whole chip, 1024 workgroups x 4 waves (4 waves per SIMD, all resident at once), one mix each:",
              f"{'mix':44s} {'matrix TFLOP/s':>15s} {'ms':>9s}   implied clock (a SIMD does 32 matrix flop per tick)"]
    for name, iters in (("mfma_f64_16x16x4", 20000), ("mfma_f64_4x4x4_4b", 60000), ("mfma_f64+4*v_fma_f64 (one wave)", 15000)):
        t, ms = fill(name, iters=iters)
        clock = f"{t * 1e12 / (1024 * 32) / 1e6:8.0f} MHz" if name == "mfma_f64_16x16x4" else ""
        lines.append(f"{name:44s} {t:15.1f} {ms:9.2f}   {clock}")
    return "\n".join(lines)


if __name__ == "__main__":
    print(report())
