"""Helpers for the GPU parity tests: move seeded inputs to the device, run a chain in every mode
through the C ABI, compare with the CPU oracle."""
from __future__ import annotations

import sys

import numpy as np
import torch

import oracle
import paper_2503_19779_amd as pg
from paper_2503_19779_amd.binding import to_device, to_numpy
from pg_workloads import make_weights, make_inputs, bf16_bits_to_f32

MODES = {"eager": pg.EAGER, "copy": pg.GRAPH_COPY, "indirect": pg.GRAPH_INDIRECT}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def as_f64(a: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


def tol_f32(o: np.ndarray, rtol: float = 1e-5) -> np.ndarray:
    """fp32 chains: |g - o| <= rtol * max(|o|, 1) (the data are O(1) by construction)."""
    return rtol * np.maximum(np.abs(o), 1.0)


def tol_bf16(o: np.ndarray, rtol: float = 2e-2) -> np.ndarray:
    """bf16 chains: |g - o| <= rtol * max(|o|, rms(o))."""
    rms = float(np.sqrt(np.mean(o * o))) if o.size else 0.0
    return rtol * np.maximum(np.abs(o), max(rms, 1e-30))


def assert_close(g: np.ndarray, o: np.ndarray, dtype: str, what: str = "", rtol=None):
    gf, of = as_f64(g), as_f64(o)
    assert gf.shape == of.shape, (what, gf.shape, of.shape)
    assert np.all(np.isfinite(of)), what + ": oracle output not finite"
    tol = tol_f32(of, rtol or 1e-5) if dtype == "f32" else tol_bf16(of, rtol or 2e-2)
    err = np.abs(gf - of)
    bad = ~(err <= tol)
    if bad.any():
        i = int(np.argmax(np.where(bad, err / tol, 0)))
        raise AssertionError(f"{what}: {int(bad.sum())} of {gf.size} elements outside tolerance; worst at {i}: "
                             f"gpu {gf[i]!r} oracle {of[i]!r} tol {tol[i]!r}")
    return float((err / tol).max()) if gf.size else 0.0


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.dtype == b.dtype and a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


class Harness:
    """A chain on cuda:0 with its weights resident, a stream, and graphs captured."""

    def __init__(self, spec, weights_np=None, capture=True, device="cuda:0"):
        self.spec = spec
        self.device = device
        self.w_np = make_weights(spec) if weights_np is None else weights_np
        self.w_dev = [to_device(w, device) for w in self.w_np]
        self.chain = pg.Chain(spec, self.w_dev, device)
        self.stream = torch.cuda.Stream(device=device)
        self._keep = []
        if capture:
            self.chain.capture(self.stream)

    def inputs(self, t: int):
        """Iteration t's inputs, as numpy and as freshly allocated device tensors."""
        x_np = make_inputs(self.spec, t)
        x_dev = [to_device(x, self.device) for x in x_np]
        self._keep.append(x_dev)
        if len(self._keep) > 4:
            self._keep.pop(0)
        return x_np, x_dev

    def run(self, mode: str, ext, modes=None):
        c = self.chain
        if mode == "eager":
            c.eager(ext, self.stream)
        elif mode == "copy":
            c.replay_copy(ext, self.stream)
        elif mode == "indirect":
            c.replay_indirect(ext, self.stream)
        elif mode == "selected":
            c.run_selected(modes, ext, self.stream)
        else:
            raise ValueError(mode)
        self.stream.synchronize()
        return [c.output(o) for o in self.spec.outputs]

    def scrub(self):
        """Overwrite every internal buffer and placeholder with NaN patterns, so that a mode cannot
        pass by finding the previous mode's results still in place."""
        c = self.chain
        for i, t in enumerate(self.spec.ints):
            c.int_buffer(i).fill_(float("nan"))
        for i, t in enumerate(self.spec.ext):
            c.placeholder(i).fill_(float("nan"))
        torch.cuda.synchronize()

    def oracle(self, x_np, k_end=None):
        ints = oracle.run_chain(self.spec, self.w_np, x_np, 0, k_end)
        return [ints[o][: ] for o in self.spec.outputs]

    def close(self):
        self.chain.close()


def check_all_modes(h: Harness, t: int, dtype: str, what: str, rtol=None, out_numel=None):
    """Run iteration t in the three modes from scrubbed buffers; modes must agree bit for bit and
    match the oracle.  Returns the worst error / tolerance ratio."""
    x_np, x_dev = h.inputs(t)
    want = h.oracle(x_np)
    got = {}
    for mode in ("eager", "copy", "indirect"):
        h.scrub()
        got[mode] = h.run(mode, x_dev)
    worst = 0.0
    for oi in range(len(h.spec.outputs)):
        n = out_numel[oi] if out_numel else want[oi].size
        e, c, i = (got[m][oi][:n] for m in ("eager", "copy", "indirect"))
        assert same_bits(e, c), f"{what}: eager and graph-copy differ (output {oi}, iteration {t})"
        assert same_bits(e, i), f"{what}: eager and graph-indirect differ (output {oi}, iteration {t})"
        worst = max(worst, assert_close(e, want[oi][:n], dtype, f"{what} output {oi} iteration {t}", rtol))
    return worst


def stepwise_check(h, x_np, x_dev, rows=None, rtol=None, kernels=None, stats=None):
    """Run the chain one kernel at a time; compare each kernel's output, element by element, with the
    oracle's single-op routine applied to the inputs that GPU kernel actually read.  `x_dev` may hold
    tensors or raw device addresses.  `rows`: for chains whose buffers are all [B, H] row-major with
    row-independent ops, check only these rows (keeps the oracle affordable).  `kernels`: compare only
    these kernel indices (all are run).  `rtol` None = the stated tolerance of the kernel's dtype.
    `stats`, if a dict, receives `flip_kernels` / `flip_elements`: kernels / elements whose bits differ
    from the oracle's (a chain with none is bit-identical to the oracle's own run, by induction).
    Returns the worst error / tolerance ratio."""
    spec, c = h.spec, h.chain
    worst, flip_k, flip_e = 0.0, 0, 0
    for k, kk in enumerate(spec.kernels):
        compare = kernels is None or k in kernels
        ins = []
        if compare:
            for r in kk.ins:
                if r.kind == "ext":
                    ins.append(x_np[r.index])
                elif r.kind == "weight":
                    ins.append(h.w_np[r.index])
                else:
                    ins.append(c.output(r.index))
        c.eager_range(x_dev, k, k + 1, h.stream)
        h.stream.synchronize()
        if not compare:
            continue
        got = c.output(kk.out)
        if rows is not None:
            B = spec.meta["batch"]
            Hh = spec.meta["hidden"]
            sel = lambda a: a.reshape(B, Hh)[rows].reshape(-1)
            if kk.op == "rmsnorm":
                want = oracle.run_op("rmsnorm", kk.dtype, [sel(ins[0]), ins[1]], kk.n, rows=len(rows), cols=kk.cols, eps=kk.eps)
            elif kk.op == "gemv":
                want = oracle.run_op("gemv", kk.dtype, [ins[0], sel(ins[1])], kk.n, rows=len(rows), cols=kk.cols)
            elif kk.op == "gelu":
                want = oracle.run_op("gelu", kk.dtype, [sel(ins[0])], len(rows) * Hh)
            else:
                want = oracle.run_op(kk.op, kk.dtype, [sel(ins[0]), sel(ins[1])], len(rows) * Hh)
            got = sel(got[:B * Hh])
        else:
            want = oracle.run_op(kk.op, kk.dtype, ins, kk.n, kk.m, kk.rows, kk.cols, kk.inner, kk.channels, kk.eps)
            got = got[:want.size]
        worst = max(worst, assert_close(got, want, kk.dtype, f"kernel {k} ({kk.op})", rtol))
        nd = int(np.count_nonzero(as_f64(got) != as_f64(want)))      # +0 and -0 count as equal
        flip_k += nd > 0
        flip_e += nd
    if stats is not None:
        stats["flip_kernels"], stats["flip_elements"] = flip_k, flip_e
    return worst
