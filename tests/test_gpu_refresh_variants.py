"""GPU parity of the alternative parameter-refresh mechanisms through the C ABI: the per-tensor
device-to-device memcpy form of the copy refresh (the baseline of Sec. 2.2), the host-side
rewrite of kernel-node arguments (the graph API's own alternative to Sec. 3's indirection), and
scalars passed as one-element tensors (Sec. 2.2: scalars become graph constants unless they
are tensors).  Each must give the eager path's bits and match the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2503_19779_amd as pg
from gpu_util import Harness, assert_close, check_all_modes, same_bits, say
from paper_2503_19779_amd.binding import to_device, to_numpy
from pg_workloads import (ChainSpec, KernelSpec, TensorSpec, Ref, EXT, INT, WEIGHT, tiny_mixed_chain,
                          elementwise_chain, decode_chain, refresh_stress_chain, large_tensor_chain)

pytestmark = pytest.mark.gpu


def run_update(h, x):
    h.chain.replay_update(x, h.stream)
    h.stream.synchronize()
    return [h.chain.output(o) for o in h.spec.outputs]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("segments", [False, True])
def test_update_mode_tiny(dtype, segments):
    h = Harness(tiny_mixed_chain(dtype, seed=5, segments=segments))
    for t in range(5):                       # both executable instances, each more than once
        x_np, x = h.inputs(t)
        ref = h.run("eager", x)
        want = h.oracle(x_np)
        h.scrub()
        got = run_update(h, x)
        for oi in range(len(ref)):
            assert same_bits(got[oi], ref[oi]), (t, oi)
            assert_close(got[oi], want[oi], dtype, f"update tiny {dtype} output {oi} iteration {t}")
    h.close()


def test_update_mode_decode_reduced_unsynchronised():
    """Replays issued back to back with different inputs at different addresses, the output
    snapshotted on the stream after each: a rewrite of the arguments for replay t+1 must not reach
    replay t while it runs."""
    spec = decode_chain(batch=3, layers=4, blocks_per_layer=3, hidden=520, n_ext=6)
    h = Harness(spec)
    sets = [h.inputs(t) for t in range(4)]
    h._keep = [s[1] for s in sets]
    ref = []
    for x_np, x in sets:
        ref.append(h.run("eager", x)[0])
        assert_close(ref[-1], h.oracle(x_np)[0], "bf16", "decode reduced eager")
    h.scrub()
    run_update(h, sets[0][1])                # builds the graphs
    snaps = []
    out = h.chain.int_buffer(spec.outputs[0])
    with torch.cuda.stream(h.stream):
        for it in range(12):
            h.chain.replay_update(sets[it % 4][1], h.stream)
            snaps.append(out.clone())
    h.stream.synchronize()
    for it, s in enumerate(snaps):
        assert same_bits(to_numpy(s), ref[it % 4]), f"replay {it}"
    h.close()


def test_update_mode_config1_and_recapture():
    h = Harness(elementwise_chain())
    for t in range(3):
        x_np, x = h.inputs(t)
        ref = h.run("eager", x)[0]
        h.scrub()
        got = run_update(h, x)[0]
        assert same_bits(got, ref)
        assert_close(got, h.oracle(x_np)[0], "f32", f"config 1 update iteration {t}")
    h.chain.capture(h.stream)                # drops the update graphs; the next call rebuilds them
    x_np, x = h.inputs(7)
    ref = h.run("eager", x)[0]
    h.scrub()
    assert same_bits(run_update(h, x)[0], ref)
    # interleaved with the other modes
    for mode in ("copy", "indirect"):
        h.scrub()
        assert same_bits(h.run(mode, x)[0], ref)
        h.scrub()
        assert same_bits(run_update(h, x)[0], ref)
    us = h.chain.time_loop(pg.GRAPH_UPDATE, [x], 5, h.stream)
    assert us > 0
    h.close()


def test_update_mode_needs_capture():
    h = Harness(tiny_mixed_chain("f32"), capture=False)
    _, x = h.inputs(0)
    with pytest.raises(pg.PgError) as e:
        h.chain.replay_update(x, h.stream)
    assert e.value.status == 2
    h.close()


@pytest.mark.parametrize("segments", [False, True])
def test_copy_refresh_by_memcpy_tiny(segments):
    h = Harness(tiny_mixed_chain("bf16", seed=9, segments=segments))
    h.chain.set_copy_refresh(pg.COPY_MEMCPY)
    for t in range(3):
        check_all_modes(h, t, "bf16", "tiny, per-tensor memcpy")
    if segments:
        x_np, x = h.inputs(4)
        ref = h.run("eager", x)
        h.scrub()
        got = h.run("selected", x, modes=[1, 0, 1])
        for a, b in zip(got, ref):
            assert same_bits(a, b)
    h.close()


def test_copy_refresh_by_memcpy_stress_reduced():
    """Config 3 at reduced size through one memcpy per tensor: every placeholder equals its source
    byte for byte (odd sizes and unaligned sources included), and the chain's output is unchanged."""
    spec = refresh_stress_chain(n_tensors=24, log2_max=20.0)
    h = Harness(spec)
    x_np, x = h.inputs(0)
    n_out = spec.meta["out_numel"]             # the rest of the output buffer is never written
    ref = h.run("copy", x)[0][:n_out]
    h.chain.set_copy_refresh(pg.COPY_MEMCPY)
    h.scrub()
    h.chain.refresh_copy(x, h.stream)
    h.stream.synchronize()
    for i, src in enumerate(x_np):
        assert same_bits(to_numpy(h.chain.placeholder(i)), src), i
    h.scrub()
    assert same_bits(h.run("copy", x)[0][:n_out], ref)
    h.chain.set_copy_refresh(pg.COPY_KERNEL)
    h.scrub()
    assert same_bits(h.run("copy", x)[0][:n_out], ref)
    with pytest.raises(pg.PgError):
        h.chain.set_copy_refresh(2)
    h.close()


def scalar_chain(dtype):
    """y = gelu(x * s + b) with s and b one-element external tensors (period-1 broadcast), then
    y = y * s again from another segment; 1000 elements."""
    n = 1000
    e, i = (lambda k: Ref(EXT, k)), (lambda k: Ref(INT, k))
    ks = [KernelSpec("mul", dtype, 0, (e(0), e(1)), n, 0, m=1),
          KernelSpec("add", dtype, 0, (i(0), e(2)), n, 0, m=1),
          KernelSpec("gelu", dtype, 0, (i(0),), n, 1),
          KernelSpec("mul", dtype, 0, (i(0), e(1)), n, 1, m=1)]
    ext = [TensorSpec(dtype, n), TensorSpec(dtype, 1), TensorSpec(dtype, 1)]
    return ChainSpec(f"scalar_as_tensor_{dtype}", ks, ext, [TensorSpec(dtype, n)], [], [0], 31)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scalars_as_one_element_tensors(dtype):
    """A scalar that changes every iteration reaches a replayed graph only as a tensor: here the
    scale and the bias are one-element externals at fresh addresses each iteration."""
    h = Harness(scalar_chain(dtype))
    outs = []
    for t in range(4):
        check_all_modes(h, t, dtype, f"scalar as tensor {dtype}")
        x_np, x = h.inputs(t)
        ref = h.run("eager", x)[0]
        h.scrub()
        assert same_bits(run_update(h, x)[0], ref)
        outs.append(ref)
    assert not same_bits(outs[0], outs[1])   # the scalars did change the result
    h.close()


def test_chain_without_external_inputs_in_every_path():
    """A chain that reads only weights: nothing to refresh, every replay path still runs it."""
    n = 3000
    ks = [KernelSpec("mul", "f32", 0, (Ref(WEIGHT, 0), Ref(WEIGHT, 1)), n, 0, m=n),
          KernelSpec("gelu", "f32", 0, (Ref(INT, 0),), n, 0),
          KernelSpec("add", "f32", 0, (Ref(INT, 0), Ref(WEIGHT, 1)), n, 1, m=n)]
    spec = ChainSpec("no_ext", ks, [], [TensorSpec("f32", n)], [TensorSpec("f32", n), TensorSpec("f32", n)], [0], 5)
    h = Harness(spec)
    want = h.oracle([])[0]
    ref = h.run("eager", [])[0]
    assert_close(ref, want, "f32", "no external inputs")
    for how in (pg.TABLE_KERNARG, pg.TABLE_MEMCPY, pg.TABLE_GRAPH_MEMCPY, pg.TABLE_HOST):
        h.chain.set_table_refresh(how)
        for mode in ("copy", "indirect"):
            h.scrub()
            assert same_bits(h.run(mode, [])[0], ref), (how, mode)
    h.chain.set_copy_refresh(pg.COPY_MEMCPY)
    h.scrub()
    assert same_bits(h.run("copy", [])[0], ref)
    h.scrub()
    assert same_bits(run_update(h, [])[0], ref)
    cost = h.chain.profile([], h.stream, iters=3, inner=2)
    assert np.all(np.isnan(cost[:, 2])) and np.all(cost[:, :2] > 0)      # no indirect variant anywhere
    assert pg.select(cost).max() <= 1
    st = h.chain.stats()
    assert st["copy_bytes_per_replay"] == 0 and st["table_bytes_per_replay"] == 0
    h.close()
