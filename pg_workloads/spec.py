"""Plain-data description of a kernel chain (a linear kernel-launch DAG).

Terms (paper, Sec. 4 "Graph-Capture Layer"): an *external* operand comes from outside the
graph and changes every iteration; an *internal* buffer is produced by an earlier kernel of the
same chain; a *weight* is caller-owned and keeps its address for the chain's life.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

EXT, INT, WEIGHT = "ext", "int", "weight"

OPS = ("add", "mul", "gelu", "rmsnorm", "gemv", "scale_bias_relu")
DTYPES = ("f32", "bf16")
DTYPE_BYTES = {"f32": 4, "bf16": 2}


@dataclass(frozen=True)
class Ref:
    kind: str          # EXT | INT | WEIGHT
    index: int


@dataclass(frozen=True)
class TensorSpec:
    dtype: str
    numel: int
    # how the generator draws it: ("normal", mean, std)
    dist: Tuple = ("normal", 0.0, 1.0)

    @property
    def nbytes(self) -> int:
        return self.numel * DTYPE_BYTES[self.dtype]


@dataclass(frozen=True)
class KernelSpec:
    op: str
    dtype: str
    out: int                      # index of the internal buffer written
    ins: Tuple[Ref, ...]          # add/mul: (a, b); gelu: (a,); rmsnorm: (x, g); gemv: (W, h); sbr: (x, s, b)
    n: int                        # output elements (per row for rmsnorm / gemv)
    segment: int = 0
    m: int = 0                    # add/mul: broadcast period of b (b[i mod m]); 0 -> n
    rows: int = 1                 # rmsnorm / gemv batch rows
    cols: int = 0                 # gemv: input width K; rmsnorm: hidden
    inner: int = 0                # scale_bias_relu: H*W
    channels: int = 0             # scale_bias_relu: C
    eps: float = 0.0              # rmsnorm


@dataclass
class ChainSpec:
    name: str
    kernels: List[KernelSpec]
    ext: List[TensorSpec]
    ints: List[TensorSpec]
    weights: List[TensorSpec]
    outputs: List[int]            # internal buffers that hold the iteration's result
    seed: int = 0
    note: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def n_segments(self) -> int:
        return (max(k.segment for k in self.kernels) + 1) if self.kernels else 0

    def ext_bytes(self) -> int:
        return sum(t.nbytes for t in self.ext)

    def n_ext_reading_kernels(self) -> int:
        return sum(1 for k in self.kernels if any(r.kind == EXT for r in k.ins))

    def truncated(self, n_kernels: int, outputs: Optional[List[int]] = None) -> "ChainSpec":
        """The same chain cut after its first n_kernels kernels."""
        ks = self.kernels[:n_kernels]
        return ChainSpec(self.name + f"[:{n_kernels}]", ks, self.ext, self.ints, self.weights,
                         outputs if outputs is not None else [ks[-1].out], self.seed, self.note,
                         dict(self.meta))
