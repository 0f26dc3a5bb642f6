"""GPU parity, one kernel at a time: every op through the C ABI in all three modes against the
CPU oracle, at sizes that span several tiles and a ragged tail, with aligned and misaligned
operands; and the batched copy kernel against a byte compare."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_19779_amd as pg
from gpu_util import Harness, assert_close, same_bits, say, as_f64
from paper_2503_19779_amd.binding import to_device, to_numpy
from pg_workloads import ChainSpec, KernelSpec, TensorSpec, Ref, EXT, INT, WEIGHT, f32_to_bf16_bits

pytestmark = pytest.mark.gpu

NP = {"f32": np.float32, "bf16": np.uint16}
EB = {"f32": 4, "bf16": 2}


def draw(rng, n, dtype, scale=1.0, mean=0.0):
    x = (rng.standard_normal(n) * scale + mean).astype(np.float32)
    return f32_to_bf16_bits(x) if dtype == "bf16" else x


def run_single(spec, ext_np, w_np, offsets=None, what=""):
    """One-kernel chain: all modes agree bit for bit; returns the output (numpy)."""
    h = Harness(spec, weights_np=w_np)
    offsets = offsets or [0] * len(ext_np)
    holders, ptrs = [], []
    for x, off in zip(ext_np, offsets):
        # place the tensor `off` bytes into a larger allocation to control its alignment
        raw = torch.empty(x.nbytes + 64, dtype=torch.uint8, device="cuda:0")
        raw[off:off + x.nbytes].copy_(torch.from_numpy(x.view(np.uint8)))
        holders.append(raw)
        ptrs.append(raw.data_ptr() + off)
    outs = {}
    for mode in ("eager", "copy", "indirect"):
        h.scrub()
        outs[mode] = h.run(mode, ptrs)[0]
    assert same_bits(outs["eager"], outs["copy"]), what + ": eager vs graph-copy"
    assert same_bits(outs["eager"], outs["indirect"]), what + ": eager vs graph-indirect"
    h.close()
    return outs["eager"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("op", ["add", "mul", "gelu"])
@pytest.mark.parametrize("n,m,offs", [(1, 0, (0, 0)), (7, 0, (0, 0)), (4096, 0, (0, 0)), (4099, 0, (0, 0)),
                                       (300001, 0, (0, 0)), (9000, 8, (0, 0)), (9001, 24, (0, 0)), (5000, 7, (0, 0)),
                                       (4099, 0, (4, 0)), (4100, 0, (0, 8)), (70000, 512, (0, 0)),
                                       (2500003, 0, (0, 0)), (2500003, 4096, (4, 0))])      # beyond 4 MB: four vectors per lane
def test_elementwise(op, dtype, n, m, offs):
    rng = np.random.Generator(np.random.PCG64(100 + n))
    say(f"elementwise {op} {dtype} n={n} m={m} offs={offs}")
    a = draw(rng, n, dtype, 2.0)
    nb = m or n
    b = draw(rng, nb, dtype)
    if op == "gelu":
        k = KernelSpec("gelu", dtype, 0, (Ref(EXT, 0),), n)
        ext, xs, of = [TensorSpec(dtype, n)], [a], [offs[0]]
    else:
        k = KernelSpec(op, dtype, 0, (Ref(EXT, 0), Ref(EXT, 1)), n, m=m)
        ext, xs, of = [TensorSpec(dtype, n), TensorSpec(dtype, nb)], [a, b], list(offs)
    spec = ChainSpec("one", [k], ext, [TensorSpec(dtype, n)], [], [0])
    got = run_single(spec, xs, [], of, f"{op} {dtype} n={n}")
    want = oracle.run_chain(spec, [], xs)[0]
    if op != "gelu" and dtype == "f32":
        assert same_bits(got, want)            # + and x are single IEEE operations
    if op != "gelu" and dtype == "bf16":
        assert same_bits(got, want)            # exact in fp32, then one rounding: must agree exactly
    assert_close(got, want, dtype, f"{op} {dtype} n={n}")


def test_bf16_rounding_edges_on_the_gpu():
    """The store's fp32 -> bf16 conversion: ties to even, subnormal results, overflow to infinity,
    signed zeros -- bit for bit as the oracle rounds."""
    a = np.array([0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x0080, 0x0001, 0x0003, 0x7F7F, 0xFF7F, 0x0000, 0x8000, 0x0040,
                  0x4000, 0x3F81, 0x0100, 0x00FF], np.uint16)
    b = np.array([0x3B80, 0x3C00, 0x3B81, 0x3C40, 0x3F00, 0x3F00, 0x3F00, 0x7F7F, 0xFF7F, 0x8000, 0x8000, 0x3E80,
                  0x3F81, 0x3F81, 0x3F40, 0x3F00], np.uint16)
    n = a.size
    for op in ("add", "mul"):
        k = KernelSpec(op, "bf16", 0, (Ref(EXT, 0), Ref(EXT, 1)), n, m=n)
        spec = ChainSpec("e", [k], [TensorSpec("bf16", n)] * 2, [TensorSpec("bf16", n)], [], [0])
        got = run_single(spec, [a, b], [], None, "edges " + op)
        want = oracle.run_chain(spec, [], [a, b])[0]
        assert same_bits(got, want), (op, [hex(x) for x in got], [hex(x) for x in want])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gelu_special_values(dtype):
    vals = np.array([0.0, -0.0, 10.0, 12.5, 40.0, 1000.0, -40.0, -100.0, -1e4, 1.0, -1.0, -0.75, 5.0, -5.0, -8.0, 3e-20], np.float32)
    a = f32_to_bf16_bits(vals) if dtype == "bf16" else vals
    n = a.size
    spec = ChainSpec("g", [KernelSpec("gelu", dtype, 0, (Ref(EXT, 0),), n)], [TensorSpec(dtype, n)], [TensorSpec(dtype, n)], [], [0])
    got = as_f64(run_single(spec, [a], []))
    x = as_f64(a)
    assert got[0] == 0 and got[1] == 0
    assert np.array_equal(got[2:6], x[2:6])                 # identity for large x
    assert np.all(got[6:9] == 0)                            # zero for very negative x
    want = as_f64(oracle.run_chain(spec, [], [a])[0])
    rel = 2e-6 if dtype == "f32" else 2.0 ** -8
    assert np.all(np.abs(got - want) <= rel * np.abs(want) + 1e-37)   # pure relative, the left tail included


def test_gelu_bf16_every_input():
    """All 65536 bf16 bit patterns through the GELU kernel (the 16-byte form) and, as a tensor of 16384
    elements less, through whichever form a small tensor takes: for every finite input the stored bf16 is
    the one the fp64 definition rounds to (the kernel's fp32 evaluation stays inside the distance that
    separates each exact value from its nearest rounding boundary); a NaN stays a NaN."""
    a = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for lo, hi in ((0, 65536), (0, 4096), (4096, 4096 + 1000)):
        part = a[lo:hi].copy()
        n = part.size
        say(f"gelu bf16 bit patterns {lo:#x}..{hi:#x}")
        spec = ChainSpec("g", [KernelSpec("gelu", "bf16", 0, (Ref(EXT, 0),), n)], [TensorSpec("bf16", n)], [TensorSpec("bf16", n)], [], [0])
        got = run_single(spec, [part], [])
        want = oracle.run_chain(spec, [], [part])[0]
        nan_in = (part & 0x7fff) > 0x7f80
        nan_want = (want & 0x7fff) > 0x7f80          # NaN inputs and -inf (-inf * 0)
        assert np.all(nan_want[nan_in])
        assert np.array_equal((got & 0x7fff) > 0x7f80, nan_want)
        differ = np.nonzero((got != want) & ~nan_want)[0]
        assert differ.size == 0, [(hex(part[i]), hex(got[i]), hex(want[i])) for i in differ[:10]]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,cols,off", [(1, 8, 0), (3, 100, 0), (1, 2048, 0), (5, 2048, 0), (2, 8200, 0), (2, 9000, 0),
                                            (1, 2048, 4), (3, 37, 0)])
def test_rmsnorm(dtype, rows, cols, off):
    if dtype == "bf16" and off % 2:
        pytest.skip("offset not element aligned")
    say(f"rmsnorm {dtype} rows={rows} cols={cols} off={off}")
    rng = np.random.Generator(np.random.PCG64(200 + cols))
    x = draw(rng, rows * cols, dtype, 3.0)
    g = draw(rng, cols, dtype, 0.02, 1.0)
    k = KernelSpec("rmsnorm", dtype, 0, (Ref(EXT, 0), Ref(WEIGHT, 0)), cols, rows=rows, cols=cols, eps=1e-6)
    spec = ChainSpec("r", [k], [TensorSpec(dtype, rows * cols)], [TensorSpec(dtype, rows * cols)], [TensorSpec(dtype, cols)], [0])
    got = run_single(spec, [x], [g], [off], "rmsnorm")
    want = oracle.run_chain(spec, [g], [x])[0]
    assert_close(got, want, dtype, "rmsnorm", rtol=(1e-5 if dtype == "f32" else 2.0 ** -7))
    # closed form: constant vector, unit gain
    c = np.full(rows * cols, 3.0, np.float32)
    ones = np.ones(cols, np.float32)
    if dtype == "bf16":
        c, ones = f32_to_bf16_bits(c), f32_to_bf16_bits(ones)
    got = as_f64(run_single(spec, [c], [ones], [0], "rmsnorm const"))
    assert np.allclose(got, 3.0 / np.sqrt(9.0 + 1e-6), rtol=(1e-6 if dtype == "f32" else 2.0 ** -8))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,n,cols", [(1, 5, 24), (1, 2048, 2048), (5, 33, 520), (3, 7, 13), (9, 64, 4096), (1, 130, 2056),
                                         (17, 16, 64), (2, 100, 2048), (130, 40, 2048), (128, 256, 2048), (33, 50, 8), (16, 31, 6152),
                                         # matrix-core form: several row groups, several K passes, ragged last tile and column block
                                         (40, 48, 4096), (100, 33, 2048), (64, 2048, 2048), (20, 16, 2056), (72, 24, 8200), (8, 64, 2048),
                                         # the 16-column form with two tiles of rows per workgroup and an idle last row group; the first 32-column shape
                                         (72, 100, 2048), (80, 2048, 2048), (81, 70, 2048),
                                         # one tile of rows: 8 columns per workgroup, with and without the upper half of the tile
                                         (16, 2048, 2048), (12, 100, 1024), (9, 20, 2048), (6, 16, 2040), (7, 27, 8), (3, 64, 2048), (4, 100, 512),
                                         (4, 15, 2048), (3, 40, 4096),
                                         # one row of exactly one chunk (h shared through LDS): ragged last workgroup, odd n
                                         (1, 1027, 2048), (1, 1030, 1024), (1, 4096, 2048), (2, 2048, 2048), (2, 1029, 2048), (2, 1030, 1024),
                                         (3, 1024, 2048), (4, 2048, 2048), (4, 1100, 1024), (3, 1031, 1024)])
def test_gemv(dtype, rows, n, cols):
    say(f"gemv {dtype} rows={rows} n={n} cols={cols}")
    rng = np.random.Generator(np.random.PCG64(300 + cols + n))
    W = draw(rng, n * cols, dtype, 0.02)
    hh = draw(rng, rows * cols, dtype)
    k = KernelSpec("gemv", dtype, 0, (Ref(WEIGHT, 0), Ref(EXT, 0)), n, rows=rows, cols=cols)
    spec = ChainSpec("g", [k], [TensorSpec(dtype, rows * cols)], [TensorSpec(dtype, rows * n)], [TensorSpec(dtype, n * cols)], [0])
    got = run_single(spec, [hh], [W], None, "gemv")
    want = oracle.run_chain(spec, [W], [hh])[0]
    assert_close(got, want, dtype, "gemv", rtol=(1e-5 if dtype == "f32" else 2.0 ** -7))
    # integer-valued operands: every partial sum is exact in fp32, so the bits must match any summation order
    Wi = rng.integers(-2, 3, n * cols).astype(np.float32)
    hi = rng.integers(-4, 5, rows * cols).astype(np.float32)
    if dtype == "bf16":
        Wi, hi = f32_to_bf16_bits(Wi), f32_to_bf16_bits(hi)
    got = run_single(spec, [hi], [Wi], None, "gemv int")
    assert same_bits(got, oracle.run_chain(spec, [Wi], [hi])[0])


@pytest.mark.parametrize("rows,n,cols", [(1, 64, 520), (2, 40, 520), (5, 33, 520), (40, 48, 520), (20, 16, 2056), (72, 24, 8200), (9, 20, 2048)])
def test_gemv_propagates_non_finite_activations_like_the_oracle(rows, n, cols):
    """An Inf and a NaN among the first columns of h: every form of the kernel (vector, and the matrix-core
    forms whose last K chunk is partly beyond cols) yields +-Inf / NaN exactly where the oracle does, and
    finite values elsewhere."""
    say(f"gemv non-finite rows={rows} n={n} cols={cols}")
    rng = np.random.Generator(np.random.PCG64(360 + cols + rows))
    W = draw(rng, n * cols, "bf16", 0.02)
    hh = draw(rng, rows * cols, "bf16").reshape(rows, cols)
    hh[0, 3] = 0x7F80                    # +Inf in row 0
    if rows > 1:
        hh[rows - 1, 5] = 0x7FC0         # NaN in the last row
    hh = hh.reshape(-1)
    k = KernelSpec("gemv", "bf16", 0, (Ref(WEIGHT, 0), Ref(EXT, 0)), n, rows=rows, cols=cols)
    spec = ChainSpec("g", [k], [TensorSpec("bf16", rows * cols)], [TensorSpec("bf16", rows * n)], [TensorSpec("bf16", n * cols)], [0])
    got = as_f64(run_single(spec, [hh], [W], None, "gemv non-finite"))
    want = as_f64(oracle.run_chain(spec, [W], [hh])[0])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(np.isposinf(got), np.isposinf(want)) and np.array_equal(np.isneginf(got), np.isneginf(want))
    assert np.isinf(want[:n]).all() and (rows == 1 or np.isnan(want[-n:]).all())
    fin = np.isfinite(want)
    if fin.any():
        assert_close(got[fin].astype(np.float32), want[fin].astype(np.float32), "f32", "finite rows", rtol=2.0 ** -7)


@pytest.mark.parametrize("dtype,rows,n,cols,off", [("bf16", 1, 2048, 2048, 2), ("bf16", 1, 1100, 2048, 6), ("f32", 1, 1024, 1024, 4),
                                                   ("bf16", 8, 64, 2048, 2), ("bf16", 40, 48, 2048, 10), ("bf16", 2, 1024, 2048, 2), ("bf16", 4, 1024, 2048, 14)])
def test_gemv_with_a_misaligned_activation(dtype, rows, n, cols, off):
    # h sits `off` bytes past a 16-byte boundary: every form fetches it by element loads, same lanes, same order
    say(f"gemv misaligned {dtype} rows={rows} n={n} cols={cols} off={off}")
    rng = np.random.Generator(np.random.PCG64(350 + n + off))
    W = draw(rng, n * cols, dtype, 0.02)
    hh = draw(rng, rows * cols, dtype)
    k = KernelSpec("gemv", dtype, 0, (Ref(WEIGHT, 0), Ref(EXT, 0)), n, rows=rows, cols=cols)
    spec = ChainSpec("g", [k], [TensorSpec(dtype, rows * cols)], [TensorSpec(dtype, rows * n)], [TensorSpec(dtype, n * cols)], [0])
    got = run_single(spec, [hh], [W], [off], "gemv misaligned")
    assert same_bits(got, run_single(spec, [hh], [W], [0], "gemv aligned"))
    assert_close(got, oracle.run_chain(spec, [W], [hh])[0], dtype, "gemv", rtol=(1e-5 if dtype == "f32" else 2.0 ** -7))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,C,inner,off", [(2, 3, 5, 0), (2, 8, 900, 0), (3, 4, 49, 0), (1, 64, 12544, 0), (2, 8, 900, 8)])
def test_scale_bias_relu(dtype, N, C, inner, off):
    say(f"sbr {dtype} {N}x{C}x{inner} off={off}")
    rng = np.random.Generator(np.random.PCG64(400 + inner))
    n = N * C * inner
    x = draw(rng, n, dtype)
    s = draw(rng, C, dtype, 0.1, 1.0)
    b = draw(rng, C, dtype, 0.1)
    k = KernelSpec("scale_bias_relu", dtype, 0, (Ref(EXT, 0), Ref(WEIGHT, 0), Ref(WEIGHT, 1)), n, inner=inner, channels=C)
    spec = ChainSpec("s", [k], [TensorSpec(dtype, n)], [TensorSpec(dtype, n)], [TensorSpec(dtype, C), TensorSpec(dtype, C)], [0])
    got = run_single(spec, [x], [s, b], [off], "sbr")
    want = oracle.run_chain(spec, [s, b], [x])[0]
    # fused multiply-add, one rounding: equals the oracle except at double-rounding ties
    assert np.count_nonzero(got != want) <= max(1, n // 100000)
    assert_close(got, want, dtype, "sbr")


def test_scale_bias_relu_with_external_scale_and_bias():
    # every operand external: exercises the three-slot indirect variant
    rng = np.random.Generator(np.random.PCG64(17))
    N, C, inner = 2, 4, 36
    n = N * C * inner
    x, s, b = draw(rng, n, "f32"), draw(rng, C, "f32", 0.1, 1.0), draw(rng, C, "f32", 0.1)
    k = KernelSpec("scale_bias_relu", "f32", 0, (Ref(EXT, 0), Ref(EXT, 1), Ref(EXT, 2)), n, inner=inner, channels=C)
    spec = ChainSpec("s", [k], [TensorSpec("f32", n), TensorSpec("f32", C), TensorSpec("f32", C)], [TensorSpec("f32", n)], [], [0])
    got = run_single(spec, [x, s, b], [], None, "sbr ext")
    assert_close(got, oracle.run_chain(spec, [], [x, s, b])[0], "f32", "sbr ext")


# ------------------------------------------------------------------ the batched copy kernel
def test_copy_kernel_sizes_and_misalignments():
    """Placeholder == source, byte for byte, for sizes around every boundary of the kernel (vector
    width, chunk size) and every element-aligned source misalignment."""
    sizes = [2, 4, 14, 16, 18, 30, 1022, 1024, 1026, 8190, 8192, 8194, 16384 + 6, 65534, 65536, 65538, 16 * 2 ** 20, 16 * 2 ** 20 + 2]
    ext = [TensorSpec("bf16", s // 2) for s in sizes]
    # one kernel that reads the first external so that the chain is valid; the copy list covers all of them
    ks = [KernelSpec("gelu", "bf16", 0, (Ref(EXT, 0),), 1)]
    spec = ChainSpec("copy", ks, ext, [TensorSpec("bf16", 1)], [], [0])
    h = Harness(spec)
    rng = np.random.Generator(np.random.PCG64(9))
    for mis in (0, 2, 4, 6, 8, 10, 12, 14):
        say(f"copy kernel misalignment {mis}")
        holders, ptrs, srcs = [], [], []
        for s in sizes:
            data = rng.integers(0, 256, s, dtype=np.uint8)
            raw = torch.empty(s + 64, dtype=torch.uint8, device="cuda:0")
            raw[mis:mis + s].copy_(torch.from_numpy(data))
            holders.append(raw); ptrs.append(raw.data_ptr() + mis); srcs.append(data)
        h.scrub()
        guard = [h.chain.workspace.clone()]
        h.chain.refresh_copy(ptrs, h.stream)
        h.stream.synchronize()
        for i, data in enumerate(srcs):
            got = h.chain.placeholder(i).view(torch.uint8).cpu().numpy()
            assert got.size == data.size and np.array_equal(got, data), f"tensor {i} size {sizes[i]} misalignment {mis}"
        # nothing outside the placeholders was written
        after = h.chain.workspace.cpu().numpy()
        before = guard[0].cpu().numpy()
        mask = np.ones(after.size, bool)
        for i in range(len(sizes)):
            off, nb = h.chain.raw_layout("ext", i)
            mask[off:off + nb] = False
        assert np.array_equal(after[mask], before[mask])
    st = h.chain.stats()
    assert st["copy_bytes_per_replay"] == sum(sizes)
    h.close()


def test_copy_kernel_many_tensors_in_groups():
    """More tensors than one launch's argument block carries (two launches)."""
    n_t = 600
    ext = [TensorSpec("f32", 3 + (i % 7)) for i in range(n_t)]
    ks = [KernelSpec("gelu", "f32", 0, (Ref(EXT, n_t - 1),), 3)]
    spec = ChainSpec("copy", ks, ext, [TensorSpec("f32", 4)], [], [0])
    h = Harness(spec)
    x_np, x_dev = h.inputs(0)
    h.scrub()
    h.chain.refresh_copy(x_dev, h.stream)
    h.chain.refresh_indirect(x_dev, h.stream)
    h.stream.synchronize()
    for i in range(n_t):
        assert np.array_equal(to_numpy(h.chain.placeholder(i)), x_np[i]), i
    table = h.chain.pointer_table().cpu().numpy()
    assert table.tolist() == [t.data_ptr() for t in x_dev]
    h.close()
