"""CPU oracle for the MLP-Offload update phase (arXiv 2509.02480) - TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes front for ``mlpo_oracle.c``: the slow, plain definition of what one update step computes
(Algorithm 1's per-subgroup body - upcast the half-precision gradients, AdamW on the fp32 master state, downcast the
parameters - plus the gradient statistics that precede it).  Nothing in the product package may import this module;
only tests, the smoke check and the benchmark's CPU-baseline leg do.  It imports nothing from the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mlpo_oracle.c")
_LIB = os.path.join(_HERE, "libmlpo_oracle.so")

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction, no fast-math).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.run(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"], check=True)
    return _LIB


class _HParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("bias_correction", C.c_int32), ("l2_mode", C.c_int32)]


class _Consts(C.Structure):
    _fields_ = [(k, C.c_float) for k in ("beta1", "beta2", "omb1", "omb2", "eps", "step_size", "sqbc2", "decay", "l2")]


class _Subgroup(C.Structure):
    _fields_ = [("p", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p), ("g", C.c_void_p), ("p16", C.c_void_p),
                ("n", C.c_uint64)]


@dataclass
class HParams:
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01
    bias_correction: bool = True
    l2_mode: bool = False

    def _c(self) -> _HParams:
        return _HParams(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay, int(self.bias_correction),
                        int(self.l2_mode))


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_bf16_to_f32.restype = C.c_float
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        L.orc_f32_to_bf16_rne.restype = C.c_uint16
        L.orc_f32_to_bf16_rne.argtypes = [C.c_float]
        L.orc_bf16_to_f32_array.restype = None
        L.orc_bf16_to_f32_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_f32_to_bf16_rne_array.restype = None
        L.orc_f32_to_bf16_rne_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_f16_to_f32_array.restype = None
        L.orc_f16_to_f32_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_f32_to_f16_rne_array.restype = None
        L.orc_f32_to_f16_rne_array.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.orc_grad_accumulate_h.restype = None
        L.orc_grad_accumulate_h.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_int32]
        L.orc_grad_stats_h.restype = None
        L.orc_grad_stats_h.argtypes = [C.c_void_p, C.c_uint64, C.c_float, C.c_int32, C.POINTER(C.c_double),
                                       C.POINTER(C.c_uint32)]
        L.orc_adamw_f32_h.restype = None
        L.orc_adamw_f32_h.argtypes = [C.c_void_p] * 5 + [C.c_uint64, C.POINTER(_HParams), C.c_int64, C.c_float,
                                                         C.c_int32]
        L.orc_adamw_f64_h.restype = None
        L.orc_adamw_f64_h.argtypes = [C.c_void_p] * 4 + [C.c_uint64, C.POINTER(_HParams), C.c_int64, C.c_double,
                                                         C.c_int32]
        L.orc_step_h.restype = C.c_int
        L.orc_step_h.argtypes = [C.POINTER(_Subgroup), C.c_int32, C.c_void_p, C.POINTER(_HParams), C.c_int64,
                                 C.c_float, C.c_float, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_uint32),
                                 C.POINTER(C.c_float)]
        L.orc_grad_accumulate.restype = None
        L.orc_grad_accumulate.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32]
        L.orc_grad_stats.restype = None
        L.orc_grad_stats.argtypes = [C.c_void_p, C.c_uint64, C.c_float, C.POINTER(C.c_double), C.POINTER(C.c_uint32)]
        L.orc_norm_finish.restype = None
        L.orc_norm_finish.argtypes = [C.c_double, C.c_float, C.c_float] + [C.POINTER(C.c_float)] * 3
        L.orc_adamw_consts.restype = None
        L.orc_adamw_consts.argtypes = [C.POINTER(_HParams), C.c_int64, C.POINTER(_Consts)]
        L.orc_adamw_f32.restype = None
        L.orc_adamw_f32.argtypes = [C.c_void_p] * 5 + [C.c_uint64, C.POINTER(_HParams), C.c_int64, C.c_float]
        L.orc_adamw_f64.restype = None
        L.orc_adamw_f64.argtypes = [C.c_void_p] * 4 + [C.c_uint64, C.POINTER(_HParams), C.c_int64, C.c_double]
        L.orc_step.restype = C.c_int
        L.orc_step.argtypes = [C.POINTER(_Subgroup), C.c_int32, C.c_void_p, C.POINTER(_HParams), C.c_int64, C.c_float,
                               C.c_float, C.POINTER(C.c_float), C.POINTER(C.c_uint32), C.POINTER(C.c_float)]
        L.orc_threads.restype = C.c_int
        L.orc_adamw_f32_chunked.restype = None
        L.orc_adamw_f32_chunked.argtypes = L.orc_adamw_f32.argtypes
        L.orc_grad_stats_chunked.restype = None
        L.orc_grad_stats_chunked.argtypes = [C.c_void_p, C.c_uint64, C.c_float, C.c_void_p, C.POINTER(C.c_double),
                                             C.POINTER(C.c_uint32)]
        _lib = L
    return _lib


def _chk(a: np.ndarray, dtype, writable=False) -> int:
    if a.dtype != dtype or not a.flags.c_contiguous or a.ndim != 1:
        raise TypeError(f"need a contiguous 1-d {np.dtype(dtype)} array, got {a.dtype} {a.shape}")
    if writable and not a.flags.writeable:
        raise TypeError("array must be writable")
    return a.ctypes.data


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32."""
    flat = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    out = np.empty(flat.size, np.float32)
    lib().orc_bf16_to_f32_array(flat.ctypes.data, out.ctypes.data, flat.size)
    return out.reshape(np.shape(bits))


def f32_to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 bit patterns (nearest, ties to even)."""
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    out = np.empty(flat.size, np.uint16)
    lib().orc_f32_to_bf16_rne_array(flat.ctypes.data, out.ctypes.data, flat.size)
    return out.reshape(np.shape(x))


HALF = {"bf16": 0, "fp16": 1}      # the two half-precision formats: every routine takes ``half`` = one of the names


def f16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen IEEE binary16 bit patterns (uint16) to fp32."""
    flat = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    out = np.empty(flat.size, np.float32)
    lib().orc_f16_to_f32_array(flat.ctypes.data, out.ctypes.data, flat.size)
    return out.reshape(np.shape(bits))


def f32_to_f16_rne(x: np.ndarray) -> np.ndarray:
    """Round fp32 to IEEE binary16 bit patterns (nearest, ties to even)."""
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    out = np.empty(flat.size, np.uint16)
    lib().orc_f32_to_f16_rne_array(flat.ctypes.data, out.ctypes.data, flat.size)
    return out.reshape(np.shape(x))


def half_to_f32(bits: np.ndarray, half: str = "bf16") -> np.ndarray:
    return f16_to_f32(bits) if HALF[half] else bf16_to_f32(bits)


def f32_to_half_rne(x: np.ndarray, half: str = "bf16") -> np.ndarray:
    return f32_to_f16_rne(x) if HALF[half] else f32_to_bf16_rne(x)


def grad_accumulate(acc: np.ndarray, g: np.ndarray, first: bool, half: str = "bf16") -> None:
    """One micro-batch's half-precision gradients g into the accumulation buffer acc, in place (copy when
    ``first``)."""
    if acc.size != g.size:
        raise ValueError("acc and g differ in length")
    lib().orc_grad_accumulate_h(_chk(acc, np.uint16, True), _chk(g, np.uint16), acc.size, 1 if first else 0,
                                HALF[half])


def grad_stats(g: np.ndarray, inv_scale: float, sumsq: float = 0.0, found_inf: int = 0, half: str = "bf16"):
    """(sum of squares of unscaled gradients in fp64, non-finite flag), accumulated onto the values passed in."""
    s = C.c_double(sumsq)
    f = C.c_uint32(found_inf)
    lib().orc_grad_stats_h(_chk(g, np.uint16), g.size, inv_scale, HALF[half], C.byref(s), C.byref(f))
    return s.value, f.value


def norm_finish(sumsq: float, inv_scale: float, max_norm: float):
    """(norm, clip_coef, gmul) as fp32 values."""
    n, c, g = C.c_float(), C.c_float(), C.c_float()
    lib().orc_norm_finish(sumsq, inv_scale, max_norm, C.byref(n), C.byref(c), C.byref(g))
    return np.float32(n.value), np.float32(c.value), np.float32(g.value)


def adamw_consts(hp: HParams, step: int) -> dict:
    c = _Consts()
    h = hp._c()
    lib().orc_adamw_consts(C.byref(h), step, C.byref(c))
    return {k: np.float32(getattr(c, k)) for k, _ in _Consts._fields_}


def adamw_f32(p, m, v, g, p16, hp: HParams, step: int, gmul: float = 1.0, chunked: bool = False,
              half: str = "bf16") -> None:
    """One applied AdamW step in place on fp32 p, m, v from half-precision g; writes the half-precision p16.
    step is 1-based.  The chunked (multi-threaded, timing only) form exists for bf16."""
    n = p.size
    assert m.size == n and v.size == n and g.size == n and p16.size == n
    h = hp._c()
    args = (_chk(p, np.float32, True), _chk(m, np.float32, True), _chk(v, np.float32, True), _chk(g, np.uint16),
            _chk(p16, np.uint16, True), n, C.byref(h), step, float(np.float32(gmul)))
    if chunked:
        assert half == "bf16"
        lib().orc_adamw_f32_chunked(*args)
    else:
        lib().orc_adamw_f32_h(*args, HALF[half])


def adamw_f64(p, m, v, g, hp: HParams, step: int, gmul: float = 1.0, half: str = "bf16") -> None:
    """The same step with all state and arithmetic in fp64 (brute-force form used for pinning)."""
    n = p.size
    assert m.size == n and v.size == n and g.size == n
    h = hp._c()
    lib().orc_adamw_f64_h(_chk(p, np.float64, True), _chk(m, np.float64, True), _chk(v, np.float64, True),
                          _chk(g, np.uint16), n, C.byref(h), step, float(gmul), HALF[half])


def grad_stats_chunked(g: np.ndarray, inv_scale: float):
    n_chunks = (g.size + (1 << 20) - 1) >> 20
    partial = np.zeros(max(n_chunks, 1), np.float64)
    s = C.c_double(0.0)
    f = C.c_uint32(0)
    lib().orc_grad_stats_chunked(_chk(g, np.uint16), g.size, inv_scale, partial.ctypes.data, C.byref(s), C.byref(f))
    return s.value, f.value


def threads() -> int:
    return lib().orc_threads()


def step(subgroups, hp: HParams, steps_applied: int, inv_scale: float = 1.0, max_norm: float = 0.0, order=None,
         half: str = "bf16"):
    """One whole update step over ``subgroups`` (a list of dicts with numpy arrays p, m, v, g, p16).

    Returns (applied, norm, found_inf, gmul).  ``steps_applied`` counts the steps applied before this one."""
    n_sg = len(subgroups)
    arr = (_Subgroup * max(n_sg, 1))()
    for k, s in enumerate(subgroups):
        n = s["p"].size
        assert all(s[key].size == n for key in ("m", "v", "g", "p16"))
        arr[k] = _Subgroup(_chk(s["p"], np.float32, True), _chk(s["m"], np.float32, True),
                           _chk(s["v"], np.float32, True), _chk(s["g"], np.uint16), _chk(s["p16"], np.uint16, True), n)
    ordp = None
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.int32)
        assert sorted(order.tolist()) == list(range(n_sg))
        ordp = order.ctypes.data
    h = hp._c()
    nrm, gm, fl = C.c_float(), C.c_float(), C.c_uint32()
    applied = lib().orc_step_h(arr, n_sg, ordp, C.byref(h), steps_applied, inv_scale, max_norm, HALF[half],
                               C.byref(nrm), C.byref(fl), C.byref(gm))
    return bool(applied), np.float32(nrm.value), int(fl.value), np.float32(gm.value)
