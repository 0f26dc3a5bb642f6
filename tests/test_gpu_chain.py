"""GPU parity of whole chains through the C ABI: the three replay modes agree bit for bit and match
the CPU oracle; replays use fresh inputs at fresh addresses (stale-parameter and poison checks);
selection and mixed-mode execution; the benchmark chains at reduced and at full size."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2503_19779_amd as pg
from gpu_util import Harness, assert_close, check_all_modes, same_bits, say, as_f64, tol_bf16
from paper_2503_19779_amd.binding import to_device, to_numpy
from pg_workloads import (tiny_mixed_chain, elementwise_chain, decode_chain, refresh_stress_chain,
                          large_tensor_chain, make_inputs)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("segments", [False, True])
def test_tiny_mixed_chain(dtype, segments):
    h = Harness(tiny_mixed_chain(dtype, seed=3, segments=segments))
    for t in range(3):
        check_all_modes(h, t, dtype, f"tiny {dtype}", rtol=(1e-5 if dtype == "f32" else 2e-2))
    h.close()


def test_config1_elementwise_chain_100_iterations():
    """64 fp32 kernels on 4096 elements, inputs refreshed from the seed every iteration."""
    h = Harness(elementwise_chain())
    worst = 0.0
    for t in range(100):
        if t < 5 or t % 25 == 0:
            worst = max(worst, check_all_modes(h, t, "f32", "config 1"))
        else:   # every iteration: modes agree bit for bit (rotating through the modes' order) and match the oracle
            x_np, x_dev = h.inputs(t)
            outs = [h.run(m, x_dev)[0] for m in (("copy", "indirect", "eager") if t % 2 else ("indirect", "eager", "copy"))]
            assert same_bits(outs[0], outs[1]) and same_bits(outs[0], outs[2]), t
            worst = max(worst, assert_close(outs[0], h.oracle(x_np)[0], "f32", f"config 1 iteration {t}"))
    say(f"config 1: worst error / tolerance over 100 iterations = {worst:.3f}")
    h.close()


def test_fresh_addresses_and_poison():
    """A replay must read this iteration's tensors, not the capture-time ones nor the previous
    iteration's (paper, Sec. 2.2: stale parameters are silent corruption)."""
    h = Harness(elementwise_chain(n_kernels=12, numel=4096), capture=False)
    x0_np, x0 = h.inputs(0)
    h.chain.eager(x0, h.stream)            # touch the chain before capture, with inputs that will be poisoned
    h.chain.capture(h.stream)
    for x in x0:
        x.fill_(float("nan"))              # poison whatever the capture may have remembered
    x1_np, x1 = h.inputs(1)
    x2_np, x2 = h.inputs(2)
    assert {t.data_ptr() for t in x1}.isdisjoint({t.data_ptr() for t in x2})
    want1, want2 = h.oracle(x1_np)[0], h.oracle(x2_np)[0]
    for mode in ("copy", "indirect", "eager"):
        h.scrub()
        g1 = h.run(mode, x1)[0]
        assert_close(g1, want1, "f32", f"{mode} iteration 1")
        snapshot = [x.clone() for x in x1]
        for x in x1:
            x.fill_(float("nan"))          # iteration 1's tensors die; iteration 2 must not look at them
        g2 = h.run(mode, x2)[0]
        assert_close(g2, want2, "f32", f"{mode} iteration 2")
        assert not same_bits(g1, g2)
        for x, s in zip(x1, snapshot):
            x.copy_(s)
    # the pointer table holds exactly this call's addresses: 8 bytes per external input
    h.chain.refresh_indirect(x2, h.stream)
    h.stream.synchronize()
    assert h.chain.pointer_table().cpu().numpy().tolist() == [t.data_ptr() for t in x2]
    # copy mode leaves every placeholder equal to its source
    h.chain.refresh_copy(x1, h.stream)
    h.stream.synchronize()
    for i, x in enumerate(x1_np):
        assert same_bits(to_numpy(h.chain.placeholder(i)), x)
    h.close()


def test_idempotence_and_interleaving():
    h = Harness(tiny_mixed_chain("bf16", seed=5, segments=True))
    x_np, x = h.inputs(0)
    y_np, y = h.inputs(1)
    ref_x = h.run("eager", x)
    ref_y = h.run("eager", y)
    n_seg = h.spec.n_segments
    seq = ["copy", "indirect", "eager", "copy", "copy", "indirect", "indirect", "eager"]
    for i, mode in enumerate(seq):
        ext, ref = (x, ref_x) if i % 3 else (y, ref_y)
        got = h.run(mode, ext)
        assert all(same_bits(a, b) for a, b in zip(got, ref)), (i, mode)
    # every per-segment mixture of modes gives the same bits
    import itertools
    for modes in itertools.product(range(3), repeat=n_seg):
        h.scrub()
        got = h.run("selected", x, modes=list(modes))
        assert all(same_bits(a, b) for a, b in zip(got, ref_x)), modes
    h.close()


@pytest.mark.parametrize("how", [pg.TABLE_KERNARG, pg.TABLE_MEMCPY, pg.TABLE_GRAPH_MEMCPY, pg.TABLE_HOST])
def test_table_refresh_mechanisms(how):
    """Every way of getting the pointers to the kernels (writer kernel, memcpy from a pinned ring, a
    copy node inside the graph, a host-resident table); enough replays to wrap the staging ring and to
    reuse both instances of the alternating mechanisms many times."""
    h = Harness(elementwise_chain(n_kernels=9, numel=1024))
    h.chain.set_table_refresh(how)
    sets = [h.inputs(t) for t in range(3)]
    h._keep = [s[1] for s in sets]
    want = [h.oracle(s[0])[0] for s in sets]
    for it in range(200):
        i = it % 3
        h.chain.replay_indirect(sets[i][1], h.stream)
        if it % 37 == 0 or it > 190:
            h.stream.synchronize()
            assert_close(h.chain.output(0), want[i], "f32", f"replay {it}")
    # back-to-back replays without host synchronisation, checked at the end
    for it in range(150):
        h.chain.replay_indirect(sets[it % 3][1], h.stream)
    h.stream.synchronize()
    assert_close(h.chain.output(0), want[149 % 3], "f32", "after 150 unsynchronised replays")
    h.close()


def test_profile_select_run_selected():
    """Slow-path profiling fills a cost table; selection is a pure function of it; running the
    selection gives the eager bits."""
    spec = large_tensor_chain(n_kernels=8, shape=(2, 8, 30, 30), n_segments=4)
    h = Harness(spec)
    x_np, x = h.inputs(0)
    cost = h.chain.profile(x, h.stream, iters=5, inner=2)
    assert cost.shape == (4, 3)
    assert np.all(np.isfinite(cost[:, :2])) and np.all(cost[:, :2] > 0)
    assert np.isfinite(cost[0, 2]) and np.all(np.isnan(cost[1:, 2]))      # only segment 0 reads an external
    sel = pg.select(cost)
    assert np.array_equal(sel, oracle.select(cost))
    ref = h.run("eager", x)[0]
    h.scrub()
    got = h.run("selected", x, modes=sel)[0]
    assert same_bits(got, ref)
    assert_close(got, h.oracle(x_np)[0], "f32", "selected")
    with pytest.raises(pg.PgError) as e:                                  # indirect does not exist for segment 1
        h.chain.run_selected([0, 2, 0, 0], x, h.stream)
    assert e.value.status == 5
    h.stream.synchronize()
    h.close()


def test_decode_chain_reduced():
    """The decode chain's wiring at reduced depth and width (still several tiles per kernel), B = 3."""
    spec = decode_chain(batch=3, layers=2, blocks_per_layer=3, hidden=520, n_ext=4)
    h = Harness(spec)
    for t in range(3):
        r = check_all_modes(h, t, "bf16", "decode reduced")
        say(f"decode reduced iteration {t}: worst error / tolerance {r:.3f}")
    h.close()


def test_refresh_stress_reduced():
    """Config 3 at reduced size: sizes log-uniform 1 KB .. 1 MB, 24 tensors.  Every placeholder equals
    its source byte for byte; outputs of kernels cut anywhere in the chain match the oracle."""
    spec = refresh_stress_chain(n_tensors=24, log2_max=20.0)
    h = Harness(spec)
    x_np, x = h.inputs(0)
    n_out = spec.meta["out_numel"]
    check_all_modes(h, 1, "bf16", "refresh stress reduced", out_numel=[n_out])
    h.scrub()
    h.chain.refresh_copy(x, h.stream)
    h.stream.synchronize()
    for i, src in enumerate(x_np):
        assert same_bits(to_numpy(h.chain.placeholder(i)), src), i
    for k in (1, 5, 12, 23):
        h.scrub()
        h.chain.eager_range(x, 0, k + 1, h.stream)
        h.stream.synchronize()
        kk = spec.kernels[k]
        want = oracle.run_chain(spec, h.w_np, x_np, 0, k + 1)[kk.out][:kk.n]
        assert_close(h.chain.output(kk.out)[:kk.n], want, "bf16", f"kernel {k}")
    h.close()


def test_selected_is_as_fast_as_the_best_single_mode():
    """Sec. 4.3: the selected mixture is at least as good as the best of its candidates.  A timing
    check, so with a wide margin: config 1 (launch-bound: a graph should win) and a large-tensor chain
    (graphs cannot win; copying the input must lose)."""
    for spec, w in ((elementwise_chain(), None), (large_tensor_chain(n_kernels=12, shape=(8, 64, 56, 56), n_segments=3), None)):
        h = Harness(spec)
        sets = [h.inputs(t)[1] for t in range(3)]
        h._keep = sets
        cost = h.chain.profile(sets[0], h.stream, iters=9, inner=3)
        sel = pg.select(cost)
        us = {}
        for name, mode, modes in (("eager", pg.EAGER, None), ("copy", pg.GRAPH_COPY, None), ("indirect", pg.GRAPH_INDIRECT, None),
                                  ("selected", pg.SELECTED, sel)):
            h.chain.time_loop(mode, sets, 10, h.stream, modes)
            us[name] = min(h.chain.time_loop(mode, sets, 50, h.stream, modes) for _ in range(3))
        say(f"{spec.name}: {us} selected {sel.tolist()}")
        assert us["selected"] <= 1.25 * min(us["eager"], us["copy"], us["indirect"]), us
        h.close()


@pytest.mark.parametrize("how", [pg.TABLE_GRAPH_MEMCPY, pg.TABLE_HOST])
def test_alternating_table_mechanisms_in_mixed_modes(how):
    """Segments in different modes within one call, inputs at fresh addresses every iteration, under
    the two table mechanisms that alternate instances; then back to the default mechanism."""
    spec = tiny_mixed_chain("bf16", seed=11, segments=True)
    h = Harness(spec)
    h.chain.set_table_refresh(how)
    for t in range(6):
        x_np, x = h.inputs(t)
        ref = h.run("eager", x)
        want = h.oracle(x_np)
        for modes in ([2, 2, 2], [1, 0, 2], [2, 1, 0], [0, 2, 1]):
            h.scrub()
            got = h.run("selected", x, modes=modes)
            for a, b in zip(got, ref):
                assert same_bits(a, b), (t, modes)
        h.scrub()
        got = h.run("indirect", x)
        for a, b, w in zip(got, ref, want):
            assert same_bits(a, b)
            assert_close(a, w, "bf16", f"table mechanism {how} iteration {t}")
    cost = h.chain.profile(h.inputs(7)[1], h.stream, iters=3, inner=2)
    assert np.all(np.isfinite(cost)) and np.all(cost > 0)
    h.chain.set_table_refresh(pg.TABLE_KERNARG)
    x_np, x = h.inputs(9)
    ref = h.run("eager", x)
    h.scrub()
    for a, b in zip(h.run("indirect", x), ref):
        assert same_bits(a, b)
    h.chain.capture(h.stream)            # a re-capture drops the alternating graphs; they are rebuilt on demand
    h.chain.set_table_refresh(how)
    h.scrub()
    for a, b in zip(h.run("indirect", x), ref):
        assert same_bits(a, b)
    h.close()


def test_event_timed_loop_agrees_with_the_host_timed_one():
    """Per-iteration times from events on the stream: positive, as many as asked for, and their mean
    close to the host-clock mean of the same loop."""
    h = Harness(elementwise_chain())
    sets = [h.inputs(t)[1] for t in range(3)]
    h._keep = sets
    for mode in (pg.EAGER, pg.GRAPH_COPY, pg.GRAPH_INDIRECT):
        h.chain.time_loop(mode, sets, 10, h.stream)
        mean = h.chain.time_loop(mode, sets, 50, h.stream)
        each = h.chain.time_loop_each(mode, sets, 50, h.stream)
        assert each.shape == (50,) and np.all(each > 0)
        assert 0.5 * mean < float(np.median(each)) < 2.0 * mean, (mode, mean, float(np.median(each)))
    x_np, x = h.inputs(5)
    assert_close(h.run("indirect", x)[0], h.oracle(x_np)[0], "f32", "after the timed loops")
    h.close()
