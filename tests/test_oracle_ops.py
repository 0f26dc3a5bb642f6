"""Pins for the oracle's per-kernel arithmetic: closed forms, textbook values, exact-integer
cases and CPU library routines in fp64.  Each block names the mistake it would catch."""
import math

import numpy as np
import pytest
import torch

import oracle
from conftest import read_golden
from pg_workloads import f32_to_bf16_bits, bf16_bits_to_f32


def f32(a):
    return np.asarray(a, dtype=np.float32)


def bf(a):
    return f32_to_bf16_bits(f32(a))


def unbf(b):
    return bf16_bits_to_f32(b).astype(np.float64)


# ---------------------------------------------------------------- GELU
def test_gelu_textbook_values():
    # x * Phi(x) with Phi from a printed table: catches a wrong constant (sqrt 2), erf/erfc mix-up, sign of the argument
    for x, phi in read_golden("normal_cdf_table.txt"):
        x, phi = float(x), float(phi)
        assert oracle.gelu_f64(x) == pytest.approx(x * phi, abs=2e-10 * max(1.0, x))
        assert oracle.gelu_f64(-x) == pytest.approx(-x * (1 - phi), abs=2e-10 * max(1.0, x))


def test_gelu_closed_forms():
    assert oracle.gelu_f64(0.0) == 0.0
    for x in (0.3, 1.0, 2.5, 7.0):
        assert oracle.gelu_f64(x) - oracle.gelu_f64(-x) == pytest.approx(x, rel=1e-14)   # Phi(x)+Phi(-x)=1
    # large |x|: identity on the right, (signed) zero on the left, after rounding to storage
    for dtype, conv, back in (("f32", f32, lambda a: a.astype(np.float64)), ("bf16", bf, unbf)):
        xs = conv([10.0, 12.5, 40.0, 1000.0])
        assert np.array_equal(oracle.run_op("gelu", dtype, [xs], 4), xs)
        neg = oracle.run_op("gelu", dtype, [conv([-40.0, -100.0, -1e4])], 3)
        assert np.all(back(neg) == 0.0)
    # minimum of x*Phi(x): derivative Phi(x) + x*phi(x) = 0 near x = -0.7518, value about -0.1700
    grid = np.linspace(-3, 0, 30001)
    vals = np.array([oracle.gelu_f64(float(v)) for v in grid])
    i = int(np.argmin(vals))
    assert grid[i] == pytest.approx(-0.75179, abs=2e-4)
    assert vals[i] == pytest.approx(-0.16997, abs=2e-5)
    x = grid[i]
    assert 0.5 * math.erfc(-x / math.sqrt(2)) + x * math.exp(-x * x / 2) / math.sqrt(2 * math.pi) == pytest.approx(0, abs=1e-4)
    # the left tail keeps relative accuracy (a 1 - erf formulation would lose it)
    assert oracle.gelu_f64(-8.0) == pytest.approx(-8.0 * 6.220960574271e-16, rel=1e-10)


def test_gelu_against_torch_fp64():
    rng = np.random.Generator(np.random.PCG64(5))
    x = rng.standard_normal(4096) * 3
    want = torch.nn.functional.gelu(torch.from_numpy(x), approximate="none").numpy()
    got = np.array([oracle.gelu_f64(float(v)) for v in x])
    # torch evaluates 1 + erf, which loses relative (not absolute) accuracy in the left tail
    assert np.allclose(got, want, rtol=1e-12, atol=1e-15)
    # storage rounding: f32 in, f32 out
    xf = x.astype(np.float32)
    out = oracle.run_op("gelu", "f32", [xf], xf.size)
    want32 = torch.nn.functional.gelu(torch.from_numpy(xf).double()).float().numpy()
    ok = xf > -5          # further left torch's own fp64 value is off by more than an f32 ulp
    assert np.array_equal(out[ok], want32[ok]) and ok.sum() > 3800
    assert np.allclose(out, want32, rtol=1e-5, atol=1e-15)


# ---------------------------------------------------------------- ADD / MUL
@pytest.mark.parametrize("op", ["add", "mul"])
def test_add_mul_f32_are_single_ieee_operations(op):
    # evaluate-in-fp64-then-round equals the fp32 operation for + and x (53 >= 2*24+2): any extra
    # rounding, wrong operand or wrong broadcast index shows as a bit difference
    rng = np.random.Generator(np.random.PCG64(6))
    a = (rng.standard_normal(1000) * 10.0 ** rng.integers(-6, 6, 1000)).astype(np.float32)
    b = (rng.standard_normal(1000) * 10.0 ** rng.integers(-6, 6, 1000)).astype(np.float32)
    want = a + b if op == "add" else a * b
    assert np.array_equal(oracle.run_op(op, "f32", [a, b], 1000), want)
    # broadcast: b[i mod m]
    m = 8
    want = a + np.tile(b[:m], 125) if op == "add" else a * np.tile(b[:m], 125)
    assert np.array_equal(oracle.run_op(op, "f32", [a, b[:m]], 1000, m=m), want)
    # m not dividing n: the period still runs from index 0
    want = a[:10] + b[np.arange(10) % 3] if op == "add" else a[:10] * b[np.arange(10) % 3]
    assert np.array_equal(oracle.run_op(op, "f32", [a[:10], b[:3]], 10, m=3), want)


@pytest.mark.parametrize("op", ["add", "mul"])
def test_add_mul_bf16_round_once(op):
    rng = np.random.Generator(np.random.PCG64(7))
    a, b = bf(rng.standard_normal(512)), bf(rng.standard_normal(512))
    exact = unbf(a) + unbf(b) if op == "add" else unbf(a) * unbf(b)        # exact in fp64
    got = oracle.run_op(op, "bf16", [a, b], 512)
    want = np.array([oracle.bf16_from_f64(float(v)) for v in exact], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert np.all(np.abs(unbf(got) - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-40)
    assert not np.array_equal(oracle.run_op(op, "bf16", [a, b], 512), a)    # not a no-op


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_closed_forms():
    H, eps = 64, 1e-6
    ones = f32(np.ones(H))
    for c in (0.5, -3.0, 7.25):
        out = oracle.run_op("rmsnorm", "f32", [f32(np.full(H, c)), ones], H, rows=1, cols=H, eps=eps)
        assert np.array_equal(out, f32(np.full(H, c / math.sqrt(c * c + eps))))
    out = oracle.run_op("rmsnorm", "f32", [f32(np.zeros(H)), ones], H, rows=1, cols=H, eps=eps)
    assert np.all(out == 0)
    # one-hot a*e_k: a / sqrt(a^2/H + eps) at k (catches sum-vs-mean and a misplaced eps)
    a, k = 3.0, 17
    x = np.zeros(H); x[k] = a
    out = oracle.run_op("rmsnorm", "f32", [f32(x), ones], H, rows=1, cols=H, eps=eps)
    assert out[k] == np.float32(a / math.sqrt(a * a / H + eps)) and np.count_nonzero(out) == 1
    # a large eps must sit inside the root, added to the mean: x=1 everywhere, eps=3 -> 1/2
    out = oracle.run_op("rmsnorm", "f32", [ones, ones], H, rows=1, cols=H, eps=3.0)
    assert np.array_equal(out, f32(np.full(H, 0.5)))


def test_rmsnorm_invariants_and_gain_and_rows():
    rng = np.random.Generator(np.random.PCG64(8))
    R, H, eps = 3, 128, 1e-5
    x = rng.standard_normal(R * H).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    ones = f32(np.ones(H))
    o1 = oracle.run_op("rmsnorm", "f32", [x, ones], H, rows=R, cols=H, eps=eps).astype(np.float64).reshape(R, H)
    ms = (x.astype(np.float64).reshape(R, H) ** 2).mean(axis=1)
    assert np.allclose((o1 ** 2).mean(axis=1), ms / (ms + eps), rtol=1e-6)         # mean(o^2) = ms/(ms+eps)
    on = oracle.run_op("rmsnorm", "f32", [f32(-4 * x), ones], H, rows=R, cols=H, eps=0.0)
    op = oracle.run_op("rmsnorm", "f32", [x, ones], H, rows=R, cols=H, eps=0.0)
    assert np.allclose(on, -op, rtol=1e-6)                                         # RMSNorm(ax) = sign(a) RMSNorm(x)
    og = oracle.run_op("rmsnorm", "f32", [x, g], H, rows=R, cols=H, eps=eps).reshape(R, H)
    assert np.allclose(og, o1 * g[None, :], rtol=1e-6)                             # gain indexed by column, shared by rows
    # rows are independent: row 1 alone gives the same bits
    alone = oracle.run_op("rmsnorm", "f32", [x[H:2 * H], g], H, rows=1, cols=H, eps=eps)
    assert np.array_equal(alone, og[1])


def test_rmsnorm_against_torch_fp64():
    rng = np.random.Generator(np.random.PCG64(9))
    R, H, eps = 4, 256, 1e-6
    xb, gb = bf(rng.standard_normal(R * H) * 5), bf(1 + 0.02 * rng.standard_normal(H))
    xt, gt = torch.from_numpy(unbf(xb)).reshape(R, H), torch.from_numpy(unbf(gb))
    want = torch.nn.functional.rms_norm(xt, (H,), weight=gt, eps=eps).numpy().reshape(-1)
    got = oracle.run_op("rmsnorm", "bf16", [xb, gb], H, rows=R, cols=H, eps=eps)
    want_bits = np.array([oracle.bf16_from_f64(float(v)) for v in want], dtype=np.uint16)
    # the two fp64 evaluations differ by rounding order (1e-16); a bf16 flip needs a value within that of a midpoint
    assert np.count_nonzero(got != want_bits) == 0
    assert np.allclose(unbf(got), want, rtol=2.0 ** -8)


# ---------------------------------------------------------------- GEMV
def test_gemv_structured_matrices():
    rng = np.random.Generator(np.random.PCG64(10))
    N, K, R = 6, 8, 2
    h = rng.standard_normal(R * K).astype(np.float32)
    eye = np.eye(K, dtype=np.float32)
    assert np.array_equal(oracle.run_op("gemv", "f32", [eye.reshape(-1), h], K, rows=R, cols=K), h)
    ones = np.ones((N, K), np.float32)
    out = oracle.run_op("gemv", "f32", [ones.reshape(-1), h], N, rows=R, cols=K).reshape(R, N)
    sums = h.astype(np.float64).reshape(R, K).sum(axis=1)
    assert np.allclose(out, np.repeat(sums[:, None], N, axis=1), rtol=1e-6)
    # W = e_j e_i^T picks h[r, i] into y[r, j]: catches a transposed W and swapped row/col strides
    j, i = 4, 1
    W = np.zeros((N, K), np.float32); W[j, i] = 1
    out = oracle.run_op("gemv", "f32", [W.reshape(-1), h], N, rows=R, cols=K).reshape(R, N)
    want = np.zeros((R, N), np.float32); want[:, j] = h.reshape(R, K)[:, i]
    assert np.array_equal(out, want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gemv_integer_values_are_exact(dtype):
    # small integers: every partial sum is exact in any precision, so the result is the integer
    # matrix product exactly, for any summation order
    rng = np.random.Generator(np.random.PCG64(12))
    N, K, R = 16, 32, 3
    W = rng.integers(-2, 3, (N, K)); h = rng.integers(-4, 5, (R, K))
    want = (h @ W.T).astype(np.float64)      # |.| <= 256: exact in bf16's 8 bits only if <= 256
    conv = f32 if dtype == "f32" else bf
    got = oracle.run_op("gemv", dtype, [conv(W.reshape(-1)), conv(h.reshape(-1))], N, rows=R, cols=K)
    gotf = got.astype(np.float64) if dtype == "f32" else unbf(got)
    if dtype == "bf16":
        want_bits = np.array([oracle.bf16_from_f64(float(v)) for v in want.reshape(-1)], dtype=np.uint16)
        assert np.array_equal(got, want_bits)
        small = np.abs(want.reshape(-1)) <= 256
        assert np.array_equal(gotf[small], want.reshape(-1)[small])
    else:
        assert np.array_equal(gotf, want.reshape(-1))


def test_bf16_results_are_rounded_once_from_fp64():
    # Sums that need more than fp32's 24 bits and sit next to a bf16 midpoint: rounding the fp64
    # sum to fp32 first lands exactly on the midpoint and the tie then goes the other way.
    # 1 + 2^-8 + 2^-30 is above the midpoint of 0x3F80/0x3F81; 1 + 2^-7 + 2^-8 - 2^-30 is below the
    # midpoint of 0x3F81/0x3F82.  Expected bit patterns written out by hand.
    one = np.ones(3, np.float32)
    up = np.array([1.0, 2.0 ** -8, 2.0 ** -30], np.float32)
    down = np.array([1.0 + 2.0 ** -7, 2.0 ** -8, -(2.0 ** -30)], np.float32)
    assert unbf(bf(up)).tolist() == up.tolist() and unbf(bf(down)).tolist() == down.tolist()   # inputs are bf16 values
    W = np.concatenate([bf(up), bf(down)])
    got = oracle.run_op("gemv", "bf16", [W, bf(one)], 2, rows=1, cols=3)
    assert got.tolist() == [0x3F81, 0x3F81]


def test_gemv_against_torch_fp64():
    rng = np.random.Generator(np.random.PCG64(13))
    N, K, R = 48, 96, 5
    Wb, hb = bf(rng.standard_normal(N * K) * 0.02), bf(rng.standard_normal(R * K))
    want = (torch.from_numpy(unbf(hb)).reshape(R, K) @ torch.from_numpy(unbf(Wb)).reshape(N, K).T).numpy().reshape(-1)
    got = oracle.run_op("gemv", "bf16", [Wb, hb], N, rows=R, cols=K)
    assert np.allclose(unbf(got), want, rtol=2.0 ** -8, atol=1e-30)
    want_bits = np.array([oracle.bf16_from_f64(float(v)) for v in want], dtype=np.uint16)
    assert np.count_nonzero(got != want_bits) <= 1          # summation order may flip a value at a midpoint


# ---------------------------------------------------------------- scale + bias + ReLU
def test_scale_bias_relu_exact_and_layout():
    rng = np.random.Generator(np.random.PCG64(14))
    N, Cc, inner = 2, 3, 5
    x = rng.integers(-8, 9, N * Cc * inner).astype(np.float32)
    s = f32([0.5, -2.0, 4.0]); b = f32([1.0, -3.0, 0.0])
    want = np.maximum(0, x.reshape(N, Cc, inner) * s[None, :, None] + b[None, :, None]).reshape(-1)
    got = oracle.run_op("scale_bias_relu", "f32", [x, s, b], x.size, channels=Cc, inner=inner)
    assert np.array_equal(got, want)                        # powers of two and integers: exact
    assert np.any(got == 0) and np.any(got > 0)
    with pytest.raises(ValueError):
        oracle.run_op("scale_bias_relu", "f32", [x[:29], s, b], 29, channels=Cc, inner=inner)


def test_scale_bias_relu_against_torch_fp64():
    rng = np.random.Generator(np.random.PCG64(15))
    N, Cc, inner = 2, 4, 49
    x = rng.standard_normal(N * Cc * inner).astype(np.float32)
    s = (1 + 0.1 * rng.standard_normal(Cc)).astype(np.float32); b = (0.1 * rng.standard_normal(Cc)).astype(np.float32)
    xt = torch.from_numpy(x).double().reshape(N, Cc, inner)
    want = torch.relu(xt * torch.from_numpy(s).double()[None, :, None] + torch.from_numpy(b).double()[None, :, None])
    got = oracle.run_op("scale_bias_relu", "f32", [x, s, b], x.size, channels=Cc, inner=inner)
    assert np.array_equal(got, want.float().numpy().reshape(-1))   # product exact in fp64; one rounding of the sum


def test_bad_arguments_are_rejected():
    a = f32(np.ones(4))
    with pytest.raises(TypeError):
        oracle.run_op("add", "bf16", [a, a], 4)
    with pytest.raises(ValueError):
        oracle.run_op("add", "f32", [a, a[:2]], 4, m=3)
    assert oracle.lib().orc_op_add(7, a.ctypes.data, a.ctypes.data, a.ctypes.data, 4, 4) == -1
