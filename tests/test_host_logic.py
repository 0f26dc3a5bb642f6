"""Host-side logic of the HIP library, without a GPU: the library loads and exports what the
header declares, descriptor validation, workspace layout, byte accounting and selection."""
import ctypes as C
import dataclasses
import itertools
import math
import os
import re
import threading

import numpy as np
import pytest

import bruteforce
import oracle
import paper_2503_19779_amd as pg
from paper_2503_19779_amd import binding
from conftest import ROOT, read_golden
from pg_workloads import (ChainSpec, KernelSpec, TensorSpec, Ref, EXT, INT, WEIGHT, elementwise_chain, decode_chain,
                          refresh_stress_chain, large_tensor_chain, tiny_mixed_chain)


def test_library_exports_every_declared_symbol():
    names = set()
    for h in ("pygraph_hip.h", "pygraph_hip_bench.h"):
        hdr = open(os.path.join(ROOT, "include", h)).read()
        hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
        names |= set(re.findall(r"\b(pg_[a-z_]+)\s*\(", hdr))
    assert {"pg_time_loop", "pg_eager_static", "pg_set_dispatch_merge", "pg_profile_in_context"} <= names
    assert {"pg_chain_build", "pg_capture", "pg_replay_copy", "pg_replay_indirect", "pg_select", "pg_eager"} <= names
    L = pg.lib()
    for n in sorted(names):
        assert hasattr(L, n), n
    assert "gfx950" in pg.version()


def test_struct_layouts_match_the_header():
    # sizes the C compiler gives the header's structs, checked by compiling a probe against the header
    import subprocess, tempfile
    src = '#include "pygraph_hip.h"\n#include <stdio.h>\nint main(){printf("%zu %zu %zu %zu\\n", sizeof(pg_kernel_desc), sizeof(pg_tensor_desc), sizeof(pg_stats), sizeof(pg_ref));return 0;}\n'
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "p.c"), "w").write(src)
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), "-o", os.path.join(d, "p"), os.path.join(d, "p.c")], check=True)
        out = subprocess.run([os.path.join(d, "p")], capture_output=True, text=True, check=True).stdout.split()
    assert [int(v) for v in out] == [C.sizeof(binding._KernelDesc), C.sizeof(binding._TensorDesc),
                                     C.sizeof(binding._Stats), C.sizeof(binding._Ref)]


# ------------------------------------------------------------------ selection
def test_select_matches_oracle_and_brute_force():
    vals = [1.0, 2.0, 2.0, math.nan, math.inf]
    rows = [r for r in itertools.product(vals, repeat=3) if any(math.isfinite(v) for v in r)]
    for r in rows:
        assert pg.select([r]).tolist() == bruteforce.select([r]) == oracle.select(np.array([r])).tolist()
    rng = np.random.Generator(np.random.PCG64(4))
    for _ in range(100):
        t = rng.uniform(0.5, 50, (int(rng.integers(1, 9)), 3))
        t[rng.uniform(size=t.shape) < 0.2] = math.nan
        t[:, 0] = np.where(np.isnan(t).all(axis=1), 1.0, t[:, 0])
        assert np.array_equal(pg.select(t), oracle.select(t))
        assert np.array_equal(pg.select(t * 3.0), pg.select(t))


def test_select_paper_examples_and_errors():
    for name, no_graph, graph, want in read_golden("select_examples.txt"):
        assert int(pg.select([[float(no_graph), float(graph), math.nan]])[0]) == int(want), name
    assert pg.select([[2.0, 2.0, 2.0]])[0] == pg.EAGER
    assert pg.select([[math.inf, 2.0, 2.0]])[0] == pg.GRAPH_COPY
    with pytest.raises(pg.PgError) as e:
        pg.select([[math.nan, math.nan, math.inf]])
    assert e.value.status == 1
    with pytest.raises(pg.PgError):
        pg.select([[1.0, -2.0, 3.0]])
    with pytest.raises(pg.PgError):
        pg.select(np.zeros((0, 3)))


def test_select_is_deterministic_across_calls_and_threads():
    rng = np.random.Generator(np.random.PCG64(5))
    t = rng.uniform(1, 10, (64, 3))
    want = pg.select(t)
    bad = []

    def work():
        for _ in range(250):
            if not np.array_equal(pg.select(t), want):
                bad.append(1)
    th = [threading.Thread(target=work) for _ in range(4)]
    [x.start() for x in th]
    [x.join() for x in th]
    assert not bad


# ------------------------------------------------------------------ build: accounting and layout
@pytest.mark.parametrize("make", [elementwise_chain, decode_chain, refresh_stress_chain, large_tensor_chain,
                                  lambda: tiny_mixed_chain("bf16", segments=True)])
def test_bytes_accounting_and_layout(make):
    spec = make()
    ch = pg.Chain.host_only(spec)
    st = ch.stats()
    assert st["n_kernels"] == len(spec.kernels) and st["n_ext"] == len(spec.ext)
    assert st["n_segments"] == spec.n_segments and st["captured"] == 0
    assert st["copy_bytes_per_replay"] == spec.ext_bytes()            # payload of a copy refresh
    assert st["table_bytes_per_replay"] == 8 * len(spec.ext)          # 8 bytes per indirected parameter
    assert st["n_ext_reading_kernels"] == spec.n_ext_reading_kernels()
    assert st["copy_chunks"] == sum(-(-t.nbytes // 8192) for t in spec.ext)
    spans = [ch.raw_layout("ext", i) for i in range(len(spec.ext))] + [ch.raw_layout("int", i) for i in range(len(spec.ints))]
    spans.append(ch.raw_layout("table"))
    for (off, nb), t in zip(spans, list(spec.ext) + list(spec.ints)):
        assert nb == t.nbytes
    spans.sort()
    for (o0, n0), (o1, _) in zip(spans, spans[1:]):
        assert o0 % 256 == 0 and o0 + n0 <= o1
    assert spans[-1][0] + spans[-1][1] <= st["workspace_bytes"] == ch.workspace_bytes
    ch.close()


def test_indirection_moves_eight_bytes_per_parameter_like_the_papers_table():
    # the paper's per-application residuals are all 8 B x (number of indirected parameters)
    for app, after in read_golden("pi_residual_bytes.txt"):
        after = int(after)
        assert after % 8 == 0 and after <= 336
        n = after // 8
        ks = [KernelSpec("add", "f32", 0, (Ref(EXT, 0), Ref(EXT, n - 1)), 16, m=16)]
        ks += [KernelSpec("add", "f32", 0, (Ref(INT, 0), Ref(EXT, j)), 16, m=16) for j in range(n)]
        spec = ChainSpec(app, ks, [TensorSpec("f32", 16)] * n, [TensorSpec("f32", 16)], [], [0])
        ch = pg.Chain.host_only(spec)
        assert ch.stats()["table_bytes_per_replay"] == after, app
        ch.close()


# ------------------------------------------------------------------ build: validation
def _base():
    return tiny_mixed_chain("f32")


def _mutate(spec, k_index, **changes):
    ks = list(spec.kernels)
    ks[k_index] = dataclasses.replace(ks[k_index], **changes)
    return dataclasses.replace(spec, kernels=ks)


BAD = {
    "read before any write": lambda s: _mutate(s, 0, ins=(Ref(INT, 1), Ref(EXT, 1))),
    "ext index out of range": lambda s: _mutate(s, 0, ins=(Ref(EXT, 0), Ref(EXT, 9))),
    "weight index out of range": lambda s: _mutate(s, 1, ins=(Ref(INT, 0), Ref(WEIGHT, 77))),
    "output index out of range": lambda s: _mutate(s, 0, out=5),
    "n larger than the buffers": lambda s: _mutate(s, 0, n=9),
    "broadcast period larger than b": lambda s: _mutate(s, 6, m=5),
    "gemv output aliases its input": lambda s: _mutate(s, 2, out=1),
    "rmsnorm in place": lambda s: _mutate(s, 1, out=0),
    "second operand aliases output": lambda s: _mutate(s, 4, ins=(Ref(INT, 2), Ref(INT, 0))),
    "rmsnorm n != cols": lambda s: _mutate(s, 1, n=3),
    "zero rows": lambda s: _mutate(s, 2, rows=0),
    "sbr n not a multiple of channels*inner": lambda s: _mutate(s, 5, inner=3),
    "sbr channels*inner far beyond n": lambda s: _mutate(s, 5, inner=0xffffffff),
    "segment goes backwards": lambda s: _mutate(s, 2, segment=1),
    "segment gap": lambda s: _mutate(s, len(s.kernels) - 1, segment=2),
    "dtype mismatch": lambda s: _mutate(s, 3, dtype="bf16"),
    "too many operands": lambda s: _mutate(s, 3, ins=(Ref(INT, 2), Ref(INT, 1))),
    "negative eps": lambda s: _mutate(s, 1, eps=-1.0),
    "reads beyond what was written": lambda s: dataclasses.replace(
        s, ints=[TensorSpec("f32", 16)] + list(s.ints[1:]),
        kernels=list(s.kernels) + [KernelSpec("add", "f32", 1, (Ref(EXT, 0), Ref(INT, 0)), 8, m=16)]),
}


@pytest.mark.parametrize("name", sorted(BAD))
def test_malformed_descriptors_are_rejected(name):
    spec = BAD[name](_base())
    with pytest.raises(pg.PgError) as e:
        pg.Chain.host_only(spec)
    assert e.value.status == 1, name
    assert "kernel" in str(e.value) or "segment" in str(e.value)


@pytest.mark.timeout(30)
def test_size_query_of_a_descriptor_that_validation_rejects_returns():
    """The workspace-size query lays the chain out, planner of merged dispatches included, before the full
    validation of pg_chain_build has run: a kernel whose output is also its broadcast operand (or its RMSNorm
    gain) must come back as an error or a size, at once -- the planner refuses such a kernel as the first of a
    run and must still move on."""
    H = 2048
    for bad in (KernelSpec("rmsnorm", "bf16", 0, (Ref(EXT, 0), Ref(INT, 0)), H, rows=1, cols=H, eps=1e-6),
                KernelSpec("add", "bf16", 0, (Ref(EXT, 0), Ref(INT, 0)), H, m=8),
                KernelSpec("mul", "f32", 0, (Ref(EXT, 0), Ref(INT, 0)), H, m=1)):
        dt = bad.dtype
        first = KernelSpec("add", dt, 0, (Ref(EXT, 0), Ref(EXT, 0)), H, m=H)
        spec = ChainSpec("bad", [first, bad, first], [TensorSpec(dt, H)], [TensorSpec(dt, H)], [], [0])
        with pytest.raises(pg.PgError) as e:
            pg.Chain.host_only(spec)
        assert e.value.status == 1 and "kernel 1" in str(e.value)


def test_wellformed_variants_are_accepted():
    s = _base()
    pg.Chain.host_only(s).close()
    pg.Chain.host_only(tiny_mixed_chain("bf16", segments=True)).close()
    # a broadcast period that does not divide n is legal
    pg.Chain.host_only(_mutate(s, 6, m=3)).close()


def test_build_argument_errors():
    spec = _base()
    L = pg.lib()
    ks, ext, ints, ws = binding.pack_descriptor(spec)
    need = C.c_size_t()
    assert L.pg_chain_workspace_bytes(ks, len(spec.kernels), ext, len(spec.ext), ints, len(spec.ints), C.byref(need)) == 0
    wp = (C.c_void_p * len(spec.weights))(*[0x1000 * (i + 1) for i in range(len(spec.weights))])
    h = C.c_void_p()

    def build(ws_ptr=0x100000, ws_len=None, wptrs=wp, nk=len(spec.kernels)):
        return L.pg_chain_build(ks, nk, ext, len(spec.ext), ints, len(spec.ints), wptrs, ws, len(spec.weights),
                                ws_ptr, need.value if ws_len is None else ws_len, C.byref(h))
    assert build() == 0 and h.value
    L.pg_chain_destroy(h)
    assert build(ws_len=need.value - 1) == 4 and h.value is None                      # PG_ENOMEM
    assert "needs" in L.pg_last_error().decode()
    assert build(ws_ptr=0x100010) == 1                                                # misaligned workspace
    assert build(ws_ptr=0) == 1
    assert build(nk=0) == 1
    bad_w = (C.c_void_p * len(spec.weights))(*[0x1000 * (i + 1) + (8 if i == 1 else 0) for i in range(len(spec.weights))])
    assert build(wptrs=bad_w) == 1
    assert L.pg_chain_build(ks, len(spec.kernels), ext, len(spec.ext), ints, len(spec.ints), wp, ws, len(spec.weights),
                            0x100000, need.value, None) == 1
    L.pg_chain_destroy(None)                                                          # a no-op
    # the size query rejects what would overflow its own layout arithmetic
    huge = dataclasses.replace(spec, ints=[TensorSpec("f32", 1 << 41)] + list(spec.ints[1:]))
    ks2, ext2, ints2, _ = binding.pack_descriptor(huge)
    assert L.pg_chain_workspace_bytes(ks2, len(huge.kernels), ext2, len(huge.ext), ints2, len(huge.ints), C.byref(need)) == 1


def test_calls_out_of_order_or_with_bad_pointers():
    spec = _base()
    ch = pg.Chain.host_only(spec)
    fake_stream = 0x1234
    ext = [0x2000, 0x3000]
    with pytest.raises(pg.PgError) as e:
        ch.replay_copy(ext, fake_stream)
    assert e.value.status == 2                                                        # PG_ESTATE: not captured
    for call in (ch.replay_indirect, ch.replay_update, ch.refresh_copy, ch.refresh_indirect):
        with pytest.raises(pg.PgError) as e:
            call(ext, fake_stream)
        assert e.value.status == 2
    with pytest.raises(pg.PgError) as e:
        ch.run_selected([0], ext, fake_stream)
    assert e.value.status == 2
    with pytest.raises(pg.PgError) as e:
        ch.eager(ext, 0)                                                              # NULL stream
    assert e.value.status == 1
    with pytest.raises(pg.PgError) as e:
        ch.eager([0x2000, 0], fake_stream)                                            # null tensor
    assert e.value.status == 1
    with pytest.raises(pg.PgError) as e:
        ch.eager([0x2000, 0x3002], fake_stream)                                       # f32 at a 2-byte offset
    assert e.value.status == 1
    with pytest.raises(pg.PgError):
        ch.capture(0)
    with pytest.raises(pg.PgError):
        ch.set_table_refresh(7)
    for how in (pg.TABLE_KERNARG, pg.TABLE_MEMCPY, pg.TABLE_GRAPH_MEMCPY, pg.TABLE_HOST, pg.TABLE_KERNARG):
        ch.set_table_refresh(how)
    with pytest.raises(pg.PgError):
        ch.set_copy_refresh(-1)
    ch.set_copy_refresh(pg.COPY_MEMCPY)
    ch.set_copy_refresh(pg.COPY_KERNEL)
    ch.close()


# ------------------------------------------------------------------ launch shapes (host only)
def _gemv_chain(dtype, rows, n, cols):
    k = KernelSpec("gemv", dtype, 0, (Ref(WEIGHT, 0), Ref(EXT, 0)), n, rows=rows, cols=cols)
    return ChainSpec("g", [k], [TensorSpec(dtype, rows * cols)], [TensorSpec(dtype, rows * n)], [TensorSpec(dtype, n * cols)], [0])


@pytest.mark.parametrize("rows,want", [(1, 256), (2, 256), (4, 256), (8, 256), (16, 256), (32, 256), (64, 512), (80, 512), (81, 256), (128, 256), (48, 384)])
def test_decode_gemv_fills_the_chip_at_every_bucket(rows, want):
    """The 2048 x 2048 bf16 GEMV is laid out over at least one workgroup per CU (256) at every batch
    size: weight streaming needs every CU pulling (the shape is fixed on the host, so no GPU is needed
    to check it)."""
    ch = pg.Chain.host_only(_gemv_chain("bf16", rows, 2048, 2048))
    assert ch.launch_shape(0) == (want, 256)
    ch.close()


def test_launch_shapes_of_other_kernels_and_bad_index():
    ch = pg.Chain.host_only(decode_chain())
    shapes = {k.op: ch.launch_shape(i) for i, k in enumerate(ch.spec.kernels)}
    assert shapes["rmsnorm"] == (1, 256) and shapes["add"] == (1, 256) and shapes["gelu"] == (4, 256) and shapes["gemv"] == (256, 256)
    with pytest.raises(pg.PgError):
        ch.launch_shape(len(ch.spec.kernels))
    with pytest.raises(pg.PgError):
        ch.launch_shape(-1)
    ch.close()
    # small and ragged GEMVs: one wave per weight row, or 8 columns per workgroup on the matrix cores
    for (rows, n, cols), want in (((1, 5, 24), 2), ((1, 130, 2056), 33), ((5, 33, 520), 5), ((9, 64, 4096), 4), ((100, 33, 2048), 8), ((40, 48, 4096), 9)):
        c2 = pg.Chain.host_only(_gemv_chain("bf16", rows, n, cols))
        assert c2.launch_shape(0) == (want, 256), (rows, n, cols, c2.launch_shape(0))
        c2.close()
