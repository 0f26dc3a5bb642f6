"""Pure-Python evaluation of tiny chains, written independently of the C oracle: loops,
math.erfc, math.fsum, and rounding done with integer arithmetic on exact rationals.  Used only
to pin the oracle on 8-element inputs; far too slow for anything else."""
from __future__ import annotations

import math
import struct
from fractions import Fraction
from typing import List, Sequence


# ---- storage formats ---------------------------------------------------------------------
def bf16_bits_to_float(b: int) -> float:
    return struct.unpack("<f", struct.pack("<I", (b & 0xFFFF) << 16))[0]


def round_to_bf16_bits(x: float) -> int:
    """Nearest bf16 (ties to even) of a finite Python float, via exact rational arithmetic."""
    if x != x:
        return 0x7FC0
    sign = 0x8000 if math.copysign(1.0, x) < 0 else 0
    if math.isinf(x):
        return sign | 0x7F80
    if x == 0.0:
        return sign
    q = Fraction(abs(x))
    # exponent e with 2^e <= q < 2^(e+1)
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fraction(2) ** e > q:
        e -= 1
    e = max(e, -126)
    scaled = q / Fraction(2) ** (e - 7)          # in units of the spacing; < 256 for normals
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    # n in [0, 256]; n == 256 carries into the next binade, the bit layout handles it:
    if e == -126 and n < 128:
        bits = n                                  # subnormal: exponent field 0
    else:
        bits = ((e + 127) << 7) + (n - 128)       # n-128 may equal 128 -> carries into the exponent
    if bits >= 0x7F80:
        bits = 0x7F80
    return sign | bits


def round_to_f32(x: float) -> float:
    try:
        return struct.unpack("<f", struct.pack("<f", x))[0]
    except OverflowError:
        return math.copysign(math.inf, x)


class Fmt:
    def __init__(self, dtype: str):
        self.dtype = dtype

    def load(self, buf: Sequence, i: int) -> float:
        return bf16_bits_to_float(int(buf[i])) if self.dtype == "bf16" else float(buf[i])

    def store(self, v: float):
        return round_to_bf16_bits(v) if self.dtype == "bf16" else round_to_f32(v)


# ---- ops -----------------------------------------------------------------------------------
def gelu(a: float) -> float:
    return 0.5 * a * math.erfc(-a / math.sqrt(2.0))


def run_chain(chain, weights: Sequence[Sequence], inputs: Sequence[Sequence]) -> List[list]:
    ints: List[list] = [[None] * t.numel for t in chain.ints]

    def buf(ref):
        return {"ext": inputs, "weight": weights, "int": ints}[ref.kind][ref.index]

    for k in chain.kernels:
        f = Fmt(k.dtype)
        src = [buf(r) for r in k.ins]
        out: list = [None] * (k.n if k.op not in ("rmsnorm", "gemv") else k.rows * k.n)
        if k.op in ("add", "mul"):
            m = k.m or k.n
            for i in range(k.n):
                a, b = f.load(src[0], i), f.load(src[1], i % m)
                out[i] = f.store(a + b if k.op == "add" else a * b)
        elif k.op == "gelu":
            for i in range(k.n):
                out[i] = f.store(gelu(f.load(src[0], i)))
        elif k.op == "rmsnorm":
            H = k.cols
            for r in range(k.rows):
                xs = [f.load(src[0], r * H + i) for i in range(H)]
                ms = math.fsum(v * v for v in xs) / H
                scale = 1.0 / math.sqrt(ms + k.eps)
                for i in range(H):
                    out[r * H + i] = f.store(xs[i] * scale * f.load(src[1], i))
        elif k.op == "gemv":
            K, N = k.cols, k.n
            for r in range(k.rows):
                for j in range(N):
                    acc = math.fsum(f.load(src[0], j * K + i) * f.load(src[1], r * K + i) for i in range(K))
                    out[r * N + j] = f.store(acc)
        elif k.op == "scale_bias_relu":
            for i in range(k.n):
                c = (i // k.inner) % k.channels
                v = f.load(src[0], i) * f.load(src[1], c) + f.load(src[2], c)
                out[i] = f.store(v if v > 0.0 else 0.0)
        else:
            raise ValueError(k.op)
        dst = ints[k.out]
        for i, v in enumerate(out):
            dst[i] = v
    return ints


def select(cost: Sequence[Sequence[float]]) -> List[int]:
    """Exhaustive argmin: the available variant no other available variant beats; first on ties."""
    res = []
    for row in cost:
        avail = [m for m in range(3) if math.isfinite(row[m])]
        if not avail:
            raise ValueError("no variant")
        winners = [m for m in avail if all(row[m] <= row[o] for o in avail)]
        res.append(min(winners))
    return res
