"""ctypes binding of the C oracle (oracle/pg_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Takes the plain-data chain description of pg_workloads and numpy buffers (float32 for f32,
uint16 bit patterns for bf16).  Imports nothing from the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pg_oracle.c")
_HDR = os.path.join(_HERE, "pg_oracle.h")
_SO = os.path.join(_HERE, "libpg_oracle.so")
# The mutation test points this at a deliberately broken build to show that the pins notice.
_SO_OVERRIDE = os.environ.get("PG_ORACLE_SO_OVERRIDE")

_DT = {"f32": 0, "bf16": 1}
_OP = {"add": 0, "mul": 1, "gelu": 2, "rmsnorm": 3, "gemv": 4, "scale_bias_relu": 5}
_KIND = {"ext": 1, "int": 2, "weight": 3}
_NP = {"f32": np.float32, "bf16": np.uint16}


class _Kernel(C.Structure):
    _fields_ = [("op", C.c_int32), ("dtype", C.c_int32), ("out_index", C.c_int32),
                ("in_kind", C.c_int32 * 3), ("in_index", C.c_int32 * 3),
                ("n", C.c_int64), ("m", C.c_int64), ("rows", C.c_int64), ("cols", C.c_int64),
                ("inner", C.c_int64), ("channels", C.c_int64), ("eps", C.c_double)]


_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: no fused multiply-adds the source does not ask for."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)):
        return _SO
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


def lib():
    global _lib
    if _lib is None:
        if _SO_OVERRIDE:
            L = C.CDLL(_SO_OVERRIDE)
        else:
            build(force=False)
            L = C.CDLL(_SO)
        L.orc_bf16_from_f64.restype = C.c_uint16
        L.orc_bf16_from_f64.argtypes = [C.c_double]
        L.orc_bf16_to_f64.restype = C.c_double
        L.orc_bf16_to_f64.argtypes = [C.c_uint16]
        L.orc_f32_from_f64.restype = C.c_float
        L.orc_f32_from_f64.argtypes = [C.c_double]
        L.orc_gelu_f64.restype = C.c_double
        L.orc_gelu_f64.argtypes = [C.c_double]
        vp, i64 = C.c_void_p, C.c_int64
        L.orc_op_add.argtypes = [C.c_int, vp, vp, vp, i64, i64]
        L.orc_op_mul.argtypes = [C.c_int, vp, vp, vp, i64, i64]
        L.orc_op_gelu.argtypes = [C.c_int, vp, vp, i64]
        L.orc_op_rmsnorm.argtypes = [C.c_int, vp, vp, vp, i64, i64, C.c_double]
        L.orc_op_gemv.argtypes = [C.c_int, vp, vp, vp, i64, i64, i64]
        L.orc_op_scale_bias_relu.argtypes = [C.c_int, vp, vp, vp, vp, i64, i64, i64]
        L.orc_chain_run.argtypes = [C.POINTER(_Kernel), C.c_int32, C.c_int32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
        L.orc_select.argtypes = [C.POINTER(C.c_double), C.c_int32, C.POINTER(C.c_uint8)]
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    lib()
    C.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def max_threads() -> int:
    lib()
    return int(C.CDLL("libgomp.so.1").omp_get_max_threads())


def bf16_from_f64(x: float) -> int:
    return int(lib().orc_bf16_from_f64(float(x)))


def bf16_to_f64(bits: int) -> float:
    return float(lib().orc_bf16_to_f64(int(bits)))


def gelu_f64(x: float) -> float:
    return float(lib().orc_gelu_f64(float(x)))


def _ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _chk(a: np.ndarray, dtype: str, min_numel: int, what: str) -> np.ndarray:
    if a.dtype != _NP[dtype]:
        raise TypeError(f"{what}: expected {_NP[dtype]}, got {a.dtype}")
    if a.size < min_numel:
        raise ValueError(f"{what}: {a.size} elements < {min_numel}")
    return np.ascontiguousarray(a)


def run_op(op: str, dtype: str, ins: Sequence[np.ndarray], n: int, m: int = 0, rows: int = 1, cols: int = 0,
           inner: int = 0, channels: int = 0, eps: float = 0.0) -> np.ndarray:
    """One op on numpy buffers; returns a fresh output array in the storage dtype."""
    L = lib()
    d = _DT[dtype]
    if op in ("add", "mul"):
        m = m or n
        a, b = _chk(ins[0], dtype, n, "a"), _chk(ins[1], dtype, m, "b")
        out = np.empty(n, _NP[dtype])
        rc = (L.orc_op_add if op == "add" else L.orc_op_mul)(d, _ptr(out), _ptr(a), _ptr(b), n, m)
    elif op == "gelu":
        a = _chk(ins[0], dtype, n, "a")
        out = np.empty(n, _NP[dtype])
        rc = L.orc_op_gelu(d, _ptr(out), _ptr(a), n)
    elif op == "rmsnorm":
        x, g = _chk(ins[0], dtype, rows * cols, "x"), _chk(ins[1], dtype, cols, "g")
        out = np.empty(rows * cols, _NP[dtype])
        rc = L.orc_op_rmsnorm(d, _ptr(out), _ptr(x), _ptr(g), rows, cols, eps)
    elif op == "gemv":
        W, h = _chk(ins[0], dtype, n * cols, "W"), _chk(ins[1], dtype, rows * cols, "h")
        out = np.empty(rows * n, _NP[dtype])
        rc = L.orc_op_gemv(d, _ptr(out), _ptr(W), _ptr(h), rows, n, cols)
    elif op == "scale_bias_relu":
        x = _chk(ins[0], dtype, n, "x")
        s, b = _chk(ins[1], dtype, channels, "s"), _chk(ins[2], dtype, channels, "b")
        out = np.empty(n, _NP[dtype])
        rc = L.orc_op_scale_bias_relu(d, _ptr(out), _ptr(x), _ptr(s), _ptr(b), n, channels, inner)
    else:
        raise ValueError(op)
    if rc != 0:
        raise ValueError(f"oracle op {op} rejected its arguments")
    return out


def _pack(chain) -> "C.Array":
    arr = (_Kernel * len(chain.kernels))()
    for i, k in enumerate(chain.kernels):
        kk = arr[i]
        kk.op, kk.dtype, kk.out_index = _OP[k.op], _DT[k.dtype], k.out
        for j in range(3):
            if j < len(k.ins):
                kk.in_kind[j], kk.in_index[j] = _KIND[k.ins[j].kind], k.ins[j].index
            else:
                kk.in_kind[j], kk.in_index[j] = 0, 0
        kk.n, kk.m, kk.rows, kk.cols = k.n, (k.m or k.n), k.rows, k.cols
        kk.inner, kk.channels, kk.eps = k.inner, k.channels, k.eps
    return arr


def run_chain(chain, weights: Sequence[np.ndarray], inputs: Sequence[np.ndarray],
              k_begin: int = 0, k_end: Optional[int] = None,
              ints: Optional[List[np.ndarray]] = None) -> List[np.ndarray]:
    """Run kernels [k_begin, k_end) of `chain` on one iteration's inputs; returns the internal
    buffers (all of them).  Fresh internal buffers are filled with a NaN pattern so that a read
    of something no kernel wrote shows up."""
    L = lib()
    k_end = len(chain.kernels) if k_end is None else k_end
    ws = [_chk(w, t.dtype, t.numel, f"weight {i}") for i, (w, t) in enumerate(zip(weights, chain.weights))]
    es = [_chk(e, t.dtype, t.numel, f"ext {i}") for i, (e, t) in enumerate(zip(inputs, chain.ext))]
    if len(ws) != len(chain.weights) or len(es) != len(chain.ext):
        raise ValueError("wrong number of weights or inputs")
    if ints is None:
        ints = []
        for t in chain.ints:
            if t.dtype == "bf16":
                ints.append(np.full(t.numel, 0x7FC0, np.uint16))
            else:
                ints.append(np.full(t.numel, np.nan, np.float32))
    vp = C.c_void_p
    e_arr = (vp * max(1, len(es)))(*[e.ctypes.data for e in es])
    w_arr = (vp * max(1, len(ws)))(*[w.ctypes.data for w in ws])
    i_arr = (vp * max(1, len(ints)))(*[b.ctypes.data for b in ints])
    rc = L.orc_chain_run(_pack(chain), k_begin, k_end, e_arr, w_arr, i_arr)
    if rc != 0:
        raise ValueError(f"oracle rejected kernel {-rc - 1}")
    return ints


def select(cost: np.ndarray) -> np.ndarray:
    """cost: [n_seg, 3] float64 (eager, graph-copy, graph-indirect); non-finite = unavailable."""
    cost = np.ascontiguousarray(cost, dtype=np.float64).reshape(-1, 3)
    out = np.zeros(cost.shape[0], np.uint8)
    rc = lib().orc_select(cost.ctypes.data_as(C.POINTER(C.c_double)), cost.shape[0],
                          out.ctypes.data_as(C.POINTER(C.c_uint8)))
    if rc != 0:
        raise ValueError(f"segment {-rc - 1} has no available variant")
    return out
