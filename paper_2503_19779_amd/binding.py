"""ctypes binding of libpygraph_hip.so: argument marshalling only.

PyTorch supplies device memory and streams; tensors cross the boundary as raw device pointers.
A chain description is any object with `.kernels`, `.ext`, `.ints`, `.weights` in the plain-data
form of `pg_workloads.spec` (duck-typed; nothing is imported from there).
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

EAGER, GRAPH_COPY, GRAPH_INDIRECT, SELECTED, GRAPH_UPDATE = 0, 1, 2, 3, 4
TABLE_KERNARG, TABLE_MEMCPY, TABLE_GRAPH_MEMCPY, TABLE_HOST = 0, 1, 2, 3
COPY_KERNEL, COPY_MEMCPY = 0, 1

_DT = {"f32": 0, "bf16": 1}
_OP = {"add": 0, "mul": 1, "gelu": 2, "rmsnorm": 3, "gemv": 4, "scale_bias_relu": 5}
_KIND = {"ext": 1, "int": 2, "weight": 3}
_STATUS = {1: "PG_EINVAL", 2: "PG_ESTATE", 3: "PG_EHIP", 4: "PG_ENOMEM", 5: "PG_EUNAVAIL"}


class PgError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{_STATUS.get(status, status)}: {msg}")
        self.status = status


class _Ref(C.Structure):
    _fields_ = [("kind", C.c_int32), ("index", C.c_int32)]


class _TensorDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("reserved", C.c_int32), ("numel", C.c_int64)]


class _KernelDesc(C.Structure):
    _fields_ = [("op", C.c_int32), ("dtype", C.c_int32), ("segment", C.c_int32), ("reserved", C.c_int32),
                ("out", _Ref), ("in_", _Ref * 3),
                ("n", C.c_int64), ("m", C.c_int64), ("rows", C.c_int64), ("cols", C.c_int64), ("inner", C.c_int64),
                ("eps", C.c_float), ("reserved2", C.c_int32)]


class _Stats(C.Structure):
    _fields_ = [("n_kernels", C.c_int32), ("n_segments", C.c_int32), ("n_ext", C.c_int32),
                ("n_ext_reading_kernels", C.c_int32), ("copy_bytes_per_replay", C.c_int64),
                ("table_bytes_per_replay", C.c_int64), ("workspace_bytes", C.c_int64),
                ("copy_chunks", C.c_int32), ("captured", C.c_int32)]


_lib = None


def lib():
    """Load the HIP library; build it first if it is missing or was built from other sources than the
    tree's (compared by content hash, so a copied tree with fresh file times does not rebuild).  No
    fallback exists: if it can be neither loaded nor built this raises."""
    global _lib
    if _lib is None:
        _build.build_library(force=False)
        L = C.CDLL(_build.LIB)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        KP, TP = C.POINTER(_KernelDesc), C.POINTER(_TensorDesc)
        PP = C.POINTER(vp)
        L.pg_chain_workspace_bytes.argtypes = [KP, i32, TP, i32, TP, i32, C.POINTER(C.c_size_t)]
        L.pg_chain_build.argtypes = [KP, i32, TP, i32, TP, i32, PP, TP, i32, vp, C.c_size_t, C.POINTER(vp)]
        L.pg_capture.argtypes = [vp, vp]
        for name in ("pg_eager", "pg_replay_copy", "pg_replay_indirect", "pg_replay_update", "pg_refresh_copy", "pg_refresh_indirect"):
            getattr(L, name).argtypes = [vp, PP, vp]
        L.pg_eager_range.argtypes = [vp, PP, i32, i32, vp]
        L.pg_eager_static.argtypes = [KP, i32, TP, i32, TP, i32, PP, TP, i32, PP, i32, vp, C.c_size_t, vp]
        L.pg_select.argtypes = [C.POINTER(C.c_double), i32, C.POINTER(C.c_uint8)]
        L.pg_time_kernels.argtypes = [vp, PP, i32, i32, vp, C.POINTER(C.c_float)]
        L.pg_time_refresh_copy.argtypes = [vp, PP, vp, C.POINTER(C.c_float)]
        L.pg_profile.argtypes = [vp, PP, vp, i32, i32, C.POINTER(C.c_double)]
        L.pg_profile_in_context.argtypes = [vp, PP, vp, PP, i32, vp, i32, i32, C.POINTER(C.c_double)]
        L.pg_run_selected.argtypes = [vp, C.POINTER(C.c_uint8), PP, vp]
        L.pg_time_loop.argtypes = [vp, i32, C.POINTER(C.c_uint8), PP, i32, i32, vp, C.POINTER(C.c_double)]
        L.pg_time_loop_each.argtypes = [vp, i32, C.POINTER(C.c_uint8), PP, i32, i32, vp, C.POINTER(C.c_float)]
        L.pg_chain_int_buffer.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(C.c_size_t)]
        L.pg_chain_placeholder.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(C.c_size_t)]
        L.pg_chain_pointer_table.argtypes = [vp, C.POINTER(vp), C.POINTER(C.c_size_t)]
        L.pg_chain_stats.argtypes = [vp, C.POINTER(_Stats)]
        L.pg_chain_launch_shape.argtypes = [vp, i32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.pg_set_table_refresh.argtypes = [vp, i32]
        L.pg_set_copy_refresh.argtypes = [vp, i32]
        L.pg_set_dispatch_merge.argtypes = [vp, i32]
        L.pg_chain_graph_dispatches.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
        L.pg_chain_destroy.argtypes = [vp]
        L.pg_chain_destroy.restype = None
        L.pg_last_error.restype = C.c_char_p
        L.pg_last_hip_error.restype = C.c_int
        L.pg_version.restype = C.c_char_p
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise PgError(status, lib().pg_last_error().decode())


def version() -> str:
    return lib().pg_version().decode()


def select(cost) -> np.ndarray:
    """Per-segment choice from a [n_seg, 3] cost table (eager, graph-copy, graph-indirect)."""
    cost = np.ascontiguousarray(cost, dtype=np.float64).reshape(-1, 3)
    out = np.zeros(cost.shape[0], np.uint8)
    _check(lib().pg_select(cost.ctypes.data_as(C.POINTER(C.c_double)), cost.shape[0],
                           out.ctypes.data_as(C.POINTER(C.c_uint8))))
    return out


STATIC_SCRATCH_BYTES = 4 << 20     # PG_STATIC_SCRATCH_BYTES of the header


def eager_static(spec, weights: Sequence, ext: Sequence, out_index: int, out, stream) -> None:
    """pg_eager_static: one eager pass of `spec` with its internal buffers in the library's static device
    array; the first out.numel() elements of internal buffer out_index land in the caller's tensor `out`."""
    ks, ext_d, ints_d, w_d = pack_descriptor(spec)
    wp = _ptr_array(weights, len(spec.weights))
    xp = _ptr_array(ext, len(spec.ext))
    s = stream if isinstance(stream, int) else stream.cuda_stream
    _check(lib().pg_eager_static(ks, len(spec.kernels), ext_d, len(spec.ext), ints_d, len(spec.ints),
                                 wp, w_d, len(spec.weights), xp, out_index, out.data_ptr(),
                                 out.numel() * out.element_size(), s))


def pack_descriptor(spec):
    """(kernel array, ext array, int array, weight array) in the library's C layout."""
    ks = (_KernelDesc * max(1, len(spec.kernels)))()
    for i, k in enumerate(spec.kernels):
        d = ks[i]
        d.op, d.dtype, d.segment = _OP[k.op], _DT[k.dtype], k.segment
        d.out.kind, d.out.index = _KIND["int"], k.out
        for j in range(3):
            if j < len(k.ins):
                d.in_[j].kind, d.in_[j].index = _KIND[k.ins[j].kind], k.ins[j].index
        d.n, d.m, d.rows, d.cols, d.inner, d.eps = k.n, k.m, k.rows, k.cols, k.inner, k.eps

    def tds(ts):
        arr = (_TensorDesc * max(1, len(ts)))()
        for i, t in enumerate(ts):
            arr[i].dtype, arr[i].numel = _DT[t.dtype], t.numel
        return arr
    return ks, tds(spec.ext), tds(spec.ints), tds(spec.weights)


def _torch():
    import torch
    return torch


def to_device(a: np.ndarray, device="cuda:0"):
    """numpy float32 / uint16 (bf16 bit patterns) -> device tensor of float32 / bfloat16."""
    torch = _torch()
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_numpy(t) -> np.ndarray:
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def _ptr_array(items: Sequence, n: int):
    arr = (C.c_void_p * max(1, n))()
    for i, it in enumerate(items):
        arr[i] = it if isinstance(it, int) else it.data_ptr()
    return arr


class Chain:
    """One chain on one GPU.  Owns the workspace tensor; borrows weights and external inputs."""

    def __init__(self, spec, weights: Sequence, device="cuda:0", workspace=None, _host_only_base: int = 0):
        L = lib()
        self._h = None
        self.spec = spec
        self.n_ext = len(spec.ext)
        self._desc = pack_descriptor(spec)
        ks, ext, ints, ws = self._desc
        need = C.c_size_t(0)
        _check(L.pg_chain_workspace_bytes(ks, len(spec.kernels), ext, len(spec.ext), ints, len(spec.ints), C.byref(need)))
        self.workspace_bytes = need.value
        self.weights = list(weights)      # keep them alive
        if len(self.weights) != len(spec.weights):
            raise ValueError("wrong number of weight tensors")
        if _host_only_base:
            # host-logic tests without a GPU: building a chain touches no device memory
            self.workspace, ws_ptr, ws_len = None, _host_only_base, need.value
        else:
            if workspace is None:
                workspace = _torch().empty(max(need.value, 256), dtype=_torch().uint8, device=device)
            self.workspace, ws_ptr, ws_len = workspace, workspace.data_ptr(), workspace.numel()
        self._ws_ptr = ws_ptr
        wp = _ptr_array(self.weights, len(self.weights))
        h = C.c_void_p()
        _check(L.pg_chain_build(ks, len(spec.kernels), ext, len(spec.ext), ints, len(spec.ints),
                                wp, ws, len(spec.weights), ws_ptr, ws_len, C.byref(h)))
        self._h = h

    @classmethod
    def host_only(cls, spec, base: int = 0x7000_0000_0000):
        """A chain over made-up addresses, for tests of validation, layout and accounting."""
        weights = [base - (i + 1) * (1 << 32) for i in range(len(spec.weights))]
        return cls(spec, weights, _host_only_base=base)

    def raw_layout(self, kind: str, index: Optional[int] = None):
        """(offset in the workspace, bytes) of a placeholder ('ext'), internal buffer ('int') or the table."""
        fn = {"ext": lib().pg_chain_placeholder, "int": lib().pg_chain_int_buffer, "table": lib().pg_chain_pointer_table}[kind]
        p, nb = C.c_void_p(), C.c_size_t()
        _check(fn(self._h, C.byref(p), C.byref(nb)) if kind == "table" else fn(self._h, index, C.byref(p), C.byref(nb)))
        return p.value - self._ws_ptr, nb.value

    # -- lifetime
    def close(self):
        if getattr(self, "_h", None):
            if self.workspace is not None:
                # pg_chain_destroy wants every stream the chain ran on idle: nothing may still replay its graphs
                _torch().cuda.synchronize(self.workspace.device)
            lib().pg_chain_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the calls
    def _ext(self, ext):
        if len(ext) != self.n_ext:
            raise ValueError(f"expected {self.n_ext} external tensors, got {len(ext)}")
        return _ptr_array(ext, self.n_ext)

    @staticmethod
    def _s(stream):
        return stream if isinstance(stream, int) else stream.cuda_stream

    def capture(self, stream):
        _check(lib().pg_capture(self._h, self._s(stream)))

    def eager(self, ext, stream):
        _check(lib().pg_eager(self._h, self._ext(ext), self._s(stream)))

    def eager_range(self, ext, k_begin: int, k_end: int, stream):
        _check(lib().pg_eager_range(self._h, self._ext(ext), k_begin, k_end, self._s(stream)))

    def replay_copy(self, ext, stream):
        _check(lib().pg_replay_copy(self._h, self._ext(ext), self._s(stream)))

    def replay_indirect(self, ext, stream):
        _check(lib().pg_replay_indirect(self._h, self._ext(ext), self._s(stream)))

    def replay_update(self, ext, stream):
        _check(lib().pg_replay_update(self._h, self._ext(ext), self._s(stream)))

    def refresh_copy(self, ext, stream):
        _check(lib().pg_refresh_copy(self._h, self._ext(ext), self._s(stream)))

    def refresh_indirect(self, ext, stream):
        _check(lib().pg_refresh_indirect(self._h, self._ext(ext), self._s(stream)))

    def run_selected(self, mode, ext, stream):
        mode = np.ascontiguousarray(mode, dtype=np.uint8)
        if mode.size != self.stats()["n_segments"]:
            raise ValueError("one mode per segment expected")
        _check(lib().pg_run_selected(self._h, mode.ctypes.data_as(C.POINTER(C.c_uint8)), self._ext(ext), self._s(stream)))

    def profile(self, ext, stream, iters: int = 20, inner: int = 5) -> np.ndarray:
        n_seg = self.stats()["n_segments"]
        cost = np.zeros((n_seg, 3), np.float64)
        _check(lib().pg_profile(self._h, self._ext(ext), self._s(stream), iters, inner,
                                cost.ctypes.data_as(C.POINTER(C.c_double))))
        return cost

    def profile_in_context(self, ext, background: "Chain", background_ext, background_mode: int, stream,
                           iters: int = 9, inner: int = 3) -> np.ndarray:
        """The cost table measured between iterations of another chain (marginal cost of each segment and mode)."""
        n_seg = self.stats()["n_segments"]
        cost = np.zeros((n_seg, 3), np.float64)
        _check(lib().pg_profile_in_context(self._h, self._ext(ext), background._h, background._ext(background_ext),
                                           background_mode, self._s(stream), iters, inner,
                                           cost.ctypes.data_as(C.POINTER(C.c_double))))
        return cost

    def time_loop(self, mode: int, ext_sets: Sequence[Sequence], iters: int, stream, modes=None) -> float:
        """Mean microseconds per iteration over `iters` back-to-back iterations of one mode."""
        n_sets = len(ext_sets)
        flat = (C.c_void_p * max(1, n_sets * self.n_ext))()
        for s, ext in enumerate(ext_sets):
            if len(ext) != self.n_ext:
                raise ValueError("wrong number of external tensors in a set")
            for i, it in enumerate(ext):
                flat[s * self.n_ext + i] = it if isinstance(it, int) else it.data_ptr()
        mp = None
        if modes is not None:
            modes = np.ascontiguousarray(modes, dtype=np.uint8)
            mp = modes.ctypes.data_as(C.POINTER(C.c_uint8))
        us = C.c_double(0)
        _check(lib().pg_time_loop(self._h, mode, mp, flat, n_sets, iters, self._s(stream), C.byref(us)))
        return us.value

    def time_loop_each(self, mode: int, ext_sets: Sequence[Sequence], iters: int, stream, modes=None) -> np.ndarray:
        """Completion-to-completion microseconds of each of `iters` back-to-back iterations of one mode."""
        n_sets = len(ext_sets)
        flat = (C.c_void_p * max(1, n_sets * self.n_ext))()
        for s, ext in enumerate(ext_sets):
            if len(ext) != self.n_ext:
                raise ValueError("wrong number of external tensors in a set")
            for i, it in enumerate(ext):
                flat[s * self.n_ext + i] = it if isinstance(it, int) else it.data_ptr()
        mp = None
        if modes is not None:
            modes = np.ascontiguousarray(modes, dtype=np.uint8)
            mp = modes.ctypes.data_as(C.POINTER(C.c_uint8))
        out = np.zeros(iters, np.float32)
        _check(lib().pg_time_loop_each(self._h, mode, mp, flat, n_sets, iters, self._s(stream), out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def time_kernels(self, ext, stream, k_begin: int = 0, k_end: Optional[int] = None) -> np.ndarray:
        """GPU execution time (microseconds) of each kernel in [k_begin, k_end), launched eagerly."""
        k_end = len(self.spec.kernels) if k_end is None else k_end
        out = np.zeros(max(0, k_end - k_begin), np.float32)
        _check(lib().pg_time_kernels(self._h, self._ext(ext), k_begin, k_end, self._s(stream),
                                     out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def time_refresh_copy(self, ext, stream) -> float:
        us = C.c_float(0)
        _check(lib().pg_time_refresh_copy(self._h, self._ext(ext), self._s(stream), C.byref(us)))
        return us.value

    def set_table_refresh(self, how: int):
        _check(lib().pg_set_table_refresh(self._h, how))

    def set_copy_refresh(self, how: int):
        _check(lib().pg_set_copy_refresh(self._h, how))

    def set_dispatch_merge(self, on: bool):
        """Takes effect at the next capture()."""
        _check(lib().pg_set_dispatch_merge(self._h, 1 if on else 0))

    def graph_dispatches(self):
        """(kernel nodes per replay with dispatch merging, without it)."""
        a, b = C.c_int32(), C.c_int32()
        _check(lib().pg_chain_graph_dispatches(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    # -- views into the workspace
    def _view(self, fn, index, dtype: Optional[str]):
        torch = _torch()
        p, nb = C.c_void_p(), C.c_size_t()
        if index is None:
            _check(fn(self._h, C.byref(p), C.byref(nb)))
        else:
            _check(fn(self._h, index, C.byref(p), C.byref(nb)))
        off = p.value - self.workspace.data_ptr()
        raw = self.workspace[off:off + nb.value]
        if dtype is None:
            return raw
        return raw.view(torch.float32 if dtype == "f32" else torch.bfloat16)

    def int_buffer(self, i: int):
        return self._view(lib().pg_chain_int_buffer, i, self.spec.ints[i].dtype)

    def placeholder(self, i: int):
        return self._view(lib().pg_chain_placeholder, i, self.spec.ext[i].dtype)

    def pointer_table(self):
        torch = _torch()
        return self._view(lib().pg_chain_pointer_table, None, None).view(torch.int64)

    def stats(self) -> dict:
        s = _Stats()
        _check(lib().pg_chain_stats(self._h, C.byref(s)))
        return {f: getattr(s, f) for f, _ in _Stats._fields_}

    def launch_shape(self, kernel: int):
        """(workgroups, threads per workgroup) of one kernel of the chain."""
        g, b = C.c_uint32(), C.c_uint32()
        _check(lib().pg_chain_launch_shape(self._h, kernel, C.byref(g), C.byref(b)))
        return g.value, b.value

    def output(self, i: int) -> np.ndarray:
        """Internal buffer i as numpy (float32, or uint16 bf16 bit patterns); synchronises."""
        return to_numpy(self.int_buffer(i))
