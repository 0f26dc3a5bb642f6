"""The five benchmark chains, as plain data.

The paper measures on TorchBench / HuggingFace / TIMM models, which are not available here;
these synthetic chains stand in for them and keep the structure the paper describes: hundreds
of short dependent kernels per iteration (Sec. 2.1), a handful to a few hundred external
parameters per graph whose sizes span KB to tens of MB (Sec. 5, table of bytes copied before
and after indirection), and a large-tensor case where launch cost is irrelevant and copying
is what hurts (Sec. 5, the HPC-style workloads that regress under graphs).
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from .spec import ChainSpec, KernelSpec, TensorSpec, Ref, EXT, INT, WEIGHT

BASE_SEED = 20250319


def _e(i): return Ref(EXT, i)
def _i(i): return Ref(INT, i)
def _w(i): return Ref(WEIGHT, i)


# --------------------------------------------------------------------------------------------
# config 1: 64 fp32 elementwise kernels on 4096-element tensors, 4 external inputs
# --------------------------------------------------------------------------------------------
def elementwise_chain(n_kernels: int = 64, numel: int = 4096, dtype: str = "f32",
                      seed: int = BASE_SEED + 1) -> ChainSpec:
    """State x (internal).  Kernel k: k%3==0 add, 1 mul, 2 GELU; with t = k//3 the add reads
    external a[(2t)%4], the mul reads a[(2t+1)%4]; kernel 0 is x <- a[3] + a[0], so no state
    survives from the previous iteration."""
    ks: List[KernelSpec] = []
    for k in range(n_kernels):
        t = k // 3
        if k == 0:
            ks.append(KernelSpec("add", dtype, 0, (_e(3), _e(0)), numel, m=numel))
        elif k % 3 == 0:
            ks.append(KernelSpec("add", dtype, 0, (_i(0), _e((2 * t) % 4)), numel, m=numel))
        elif k % 3 == 1:
            ks.append(KernelSpec("mul", dtype, 0, (_i(0), _e((2 * t + 1) % 4)), numel, m=numel))
        else:
            ks.append(KernelSpec("gelu", dtype, 0, (_i(0),), numel))
    ext = [TensorSpec(dtype, numel) for _ in range(4)]
    return ChainSpec(f"elementwise{n_kernels}_{dtype}_{numel}", ks, ext, [TensorSpec(dtype, numel)], [],
                     [0], seed)


# --------------------------------------------------------------------------------------------
# config 2 / 5: decode-step chain
# --------------------------------------------------------------------------------------------
def decode_chain(batch: int = 1, layers: int = 24, blocks_per_layer: int = 5, hidden: int = 2048,
                 n_ext: int = 32, seed: int = BASE_SEED + 2, eps: float = 1e-6) -> ChainSpec:
    """layers*blocks_per_layer sub-blocks of RMSNorm -> GEMV -> GELU -> residual add on a bf16
    residual stream x[batch, hidden]; external e_0 is the initial stream, e_j (j >= 1) is added
    to the stream by one extra kernel before sub-block floor(S*j/n_ext).  With the defaults:
    480 + 31 = 511 kernels, 33 of which read an external operand."""
    S = layers * blocks_per_layer
    H, B = hidden, batch
    X, T1, T2 = 0, 1, 2
    inject_at = {}
    for j in range(1, n_ext):
        inject_at.setdefault((S * j) // n_ext, []).append(j)
    ks: List[KernelSpec] = []
    for s in range(S):
        for j in inject_at.get(s, []):
            if s == 0:
                raise ValueError("an inject before sub-block 0 would read an unwritten stream")
            ks.append(KernelSpec("add", "bf16", X, (_i(X), _e(j)), B * H, m=B * H))
        x_ref = _e(0) if s == 0 else _i(X)
        ks.append(KernelSpec("rmsnorm", "bf16", T1, (x_ref, _w(S + s)), H, rows=B, cols=H, eps=eps))
        ks.append(KernelSpec("gemv", "bf16", T2, (_w(s), _i(T1)), H, rows=B, cols=H))
        ks.append(KernelSpec("gelu", "bf16", T2, (_i(T2),), B * H))
        ks.append(KernelSpec("add", "bf16", X, (x_ref, _i(T2)), B * H, m=B * H))
    ext = [TensorSpec("bf16", B * H) for _ in range(n_ext)]
    ints = [TensorSpec("bf16", B * H) for _ in range(3)]
    weights = ([TensorSpec("bf16", H * H, ("normal", 0.0, 0.02)) for _ in range(S)] +
               [TensorSpec("bf16", H, ("normal", 1.0, 0.02)) for _ in range(S)])
    return ChainSpec(f"decode_b{B}_L{layers}x{blocks_per_layer}_h{H}", ks, ext, ints, weights, [X], seed,
                     meta={"batch": B, "hidden": H, "sub_blocks": S})


def decode_buckets(buckets: Tuple[int, ...] = (1, 2, 4, 8, 16, 32, 64, 128), seed: int = BASE_SEED + 5,
                   **kw) -> List[ChainSpec]:
    """One chain per batch-size bucket; all share one seed, hence one set of weights."""
    return [decode_chain(batch=b, seed=seed, **kw) for b in buckets]


def bucket_sequence(n_buckets: int = 8, length: int = 1000, seed: int = BASE_SEED + 5) -> np.ndarray:
    """i.i.d. uniform bucket index per iteration."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5EED))
    return rng.integers(0, n_buckets, size=length)


# --------------------------------------------------------------------------------------------
# config 3: parameter-refresh stress
# --------------------------------------------------------------------------------------------
def refresh_stress_chain(n_tensors: int = 256, log2_min: float = 10.0, log2_max: float = 24.0,
                         seed: int = BASE_SEED + 3, carry: int = 512) -> ChainSpec:
    """n_tensors bf16 externals with byte sizes 2^U, U ~ Uniform[log2_min, log2_max], rounded
    down to a multiple of 1 KB.  Kernel k reads all of external k and a `carry`-element vector
    c = the head of the previous kernel's output (a constant weight for k = 0):
    k%3==0: in_k + c[i mod carry]; 1: in_k * c[i mod carry]; 2: GELU(in_k).  Outputs alternate
    between two internal buffers of the largest size."""
    rng = np.random.Generator(np.random.PCG64(seed))
    u = rng.uniform(log2_min, log2_max, size=n_tensors)
    nbytes = (np.floor(2.0 ** u).astype(np.int64) // 1024) * 1024
    nbytes = np.maximum(nbytes, 1024)
    numel = (nbytes // 2).tolist()
    max_el = int(2 ** log2_max) // 2
    ks: List[KernelSpec] = []
    for k in range(n_tensors):
        c = _w(0) if k == 0 else _i((k - 1) % 2)
        if k % 3 == 0:
            ks.append(KernelSpec("add", "bf16", k % 2, (_e(k), c), numel[k], m=carry))
        elif k % 3 == 1:
            ks.append(KernelSpec("mul", "bf16", k % 2, (_e(k), c), numel[k], m=carry))
        else:
            ks.append(KernelSpec("gelu", "bf16", k % 2, (_e(k),), numel[k]))
    ext = [TensorSpec("bf16", n) for n in numel]
    ints = [TensorSpec("bf16", max_el), TensorSpec("bf16", max_el)]
    return ChainSpec(f"refresh_stress_{n_tensors}", ks, ext, ints, [TensorSpec("bf16", carry)],
                     [(n_tensors - 1) % 2], seed, meta={"out_numel": numel[-1]})


# --------------------------------------------------------------------------------------------
# config 4: large tensors, launch cost hidden
# --------------------------------------------------------------------------------------------
def large_tensor_chain(n_kernels: int = 40, shape: Tuple[int, int, int, int] = (32, 64, 112, 112),
                       n_segments: int = 4, seed: int = BASE_SEED + 4) -> ChainSpec:
    """n_kernels of fp32 per-channel scale + bias + ReLU on an NCHW tensor; s = 1 + 0.1 N(0,1),
    b = 0.1 N(0,1) per kernel; only kernel 0 reads the (single) external input; outputs
    ping-pong between two internal buffers; kernels are split evenly into segments."""
    N, C, Hh, Ww = shape
    numel = N * C * Hh * Ww
    per_seg = (n_kernels + n_segments - 1) // n_segments
    ks: List[KernelSpec] = []
    for k in range(n_kernels):
        src = _e(0) if k == 0 else _i((k - 1) % 2)
        ks.append(KernelSpec("scale_bias_relu", "f32", k % 2, (src, _w(2 * k), _w(2 * k + 1)), numel,
                             segment=k // per_seg, inner=Hh * Ww, channels=C))
    weights = []
    for _ in range(n_kernels):
        weights.append(TensorSpec("f32", C, ("normal", 1.0, 0.1)))
        weights.append(TensorSpec("f32", C, ("normal", 0.0, 0.1)))
    ints = [TensorSpec("f32", numel), TensorSpec("f32", numel)]
    return ChainSpec(f"sbr{n_kernels}_{N}x{C}x{Hh}x{Ww}", ks, [TensorSpec("f32", numel)], ints, weights,
                     [(n_kernels - 1) % 2], seed)


# --------------------------------------------------------------------------------------------
# a tiny chain that uses every op once or more; for brute-force checks
# --------------------------------------------------------------------------------------------
def tiny_mixed_chain(dtype: str = "bf16", seed: int = 7, segments: bool = False) -> ChainSpec:
    """8-element tensors, 10 kernels, all six ops, two externals, in-place and broadcast forms."""
    sg = (lambda k: k // 4) if segments else (lambda k: 0)
    ks = [
        KernelSpec("add", dtype, 0, (_e(0), _e(1)), 8, m=8),                                   # x0 = e0 + e1
        KernelSpec("rmsnorm", dtype, 1, (_i(0), _w(0)), 4, rows=2, cols=4, eps=1e-3),           # t = rms(x0 as [2,4])
        KernelSpec("gemv", dtype, 2, (_w(1), _i(1)), 4, rows=2, cols=4),                        # y[2,4] = W[4,4] t
        KernelSpec("gelu", dtype, 2, (_i(2),), 8),                                             # y = gelu(y)
        KernelSpec("mul", dtype, 0, (_i(0), _i(2)), 8, m=8),                                   # x0 = x0 * y
        KernelSpec("scale_bias_relu", dtype, 1, (_i(0), _w(2), _w(3)), 8, inner=4, channels=2),  # t = relu(x0*s+b)
        KernelSpec("add", dtype, 1, (_i(1), _w(4)), 8, m=4),                                   # t = t + c[i%4]
        KernelSpec("mul", dtype, 2, (_e(1), _i(1)), 8, m=2),                                   # y = e1 * t[i%2]
        KernelSpec("gelu", dtype, 0, (_e(0),), 8),                                             # x0 = gelu(e0)
        KernelSpec("add", dtype, 0, (_i(0), _i(2)), 8, m=8),                                   # x0 = x0 + y
    ]
    ks = [KernelSpec(k.op, k.dtype, k.out, k.ins, k.n, sg(i), k.m, k.rows, k.cols, k.inner, k.channels, k.eps)
          for i, k in enumerate(ks)]
    ext = [TensorSpec(dtype, 8), TensorSpec(dtype, 8)]
    ints = [TensorSpec(dtype, 8) for _ in range(3)]
    weights = [TensorSpec(dtype, 4, ("normal", 1.0, 0.1)), TensorSpec(dtype, 16, ("normal", 0.0, 0.5)),
               TensorSpec(dtype, 2, ("normal", 1.0, 0.5)), TensorSpec(dtype, 2, ("normal", 0.0, 0.5)),
               TensorSpec(dtype, 4)]
    return ChainSpec(f"tiny_mixed_{dtype}", ks, ext, ints, weights, [0, 1, 2], seed)
