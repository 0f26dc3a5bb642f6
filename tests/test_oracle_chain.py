"""Pins for the oracle's chain rule and selection rule: a pure-Python brute force on 8-element
chains (bit-for-bit), structural properties of the chain rule, the paper's worked selection
examples, and exhaustive small cost tables."""
import itertools
import math

import numpy as np
import pytest

import bruteforce
import oracle
from conftest import read_golden
from pg_workloads import (tiny_mixed_chain, elementwise_chain, decode_chain, refresh_stress_chain,
                          large_tensor_chain, make_weights, make_inputs, bf16_bits_to_f32)


def as_f64(a):
    return bf16_bits_to_f32(a).astype(np.float64) if a.dtype == np.uint16 else a.astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_tiny_chain_equals_brute_force_bit_for_bit(dtype, seed):
    chain = tiny_mixed_chain(dtype, seed=seed)
    w = make_weights(chain)
    for t in range(3):
        x = make_inputs(chain, t)
        got = oracle.run_chain(chain, w, x)
        want = bruteforce.run_chain(chain, [a.tolist() for a in w], [a.tolist() for a in x])
        for gi, wi in zip(got, want):
            wi = np.array(wi, dtype=gi.dtype)
            assert np.array_equal(gi.view(np.uint32 if dtype == "f32" else np.uint16),
                                  wi.view(np.uint32 if dtype == "f32" else np.uint16))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_config_chains_equal_brute_force(dtype):
    # the benchmark chains' own wiring, shrunk to 8 elements (config 1) and hidden 8 (config 2)
    c1 = elementwise_chain(n_kernels=12, numel=8, dtype=dtype, seed=5)
    c2 = decode_chain(batch=2, layers=2, blocks_per_layer=2, hidden=8, n_ext=3, seed=6)
    for chain in (c1, c2):
        w, x = make_weights(chain), make_inputs(chain, 0)
        got = oracle.run_chain(chain, w, x)
        want = bruteforce.run_chain(chain, [a.tolist() for a in w], [a.tolist() for a in x])
        for o in chain.outputs:
            assert np.array_equal(got[o], np.array(want[o], dtype=got[o].dtype))


def test_chain_is_a_fold_of_single_ops():
    # running the chain == applying the single-op routine kernel by kernel on the same buffers
    chain = tiny_mixed_chain("bf16", seed=4)
    w, x = make_weights(chain), make_inputs(chain, 0)
    ints = [np.zeros(t.numel, np.uint16) for t in chain.ints]
    src = {"ext": x, "weight": w, "int": ints}
    for k in chain.kernels:
        ins = [src[r.kind][r.index] for r in k.ins]
        ints[k.out][:] = oracle.run_op(k.op, k.dtype, ins, k.n, k.m, k.rows, k.cols, k.inner, k.channels, k.eps)
    got = oracle.run_chain(chain, w, x)
    for a, b in zip(got, ints):
        assert np.array_equal(a, b)


def test_truncation_and_resumption():
    chain = tiny_mixed_chain("f32", seed=9)
    w, x = make_weights(chain), make_inputs(chain, 1)
    full = oracle.run_chain(chain, w, x)
    part = oracle.run_chain(chain, w, x, 0, 6)
    rest = oracle.run_chain(chain, w, x, 6, None, ints=[p.copy() for p in part])
    for a, b in zip(full, rest):
        assert np.array_equal(a, b, equal_nan=True)
    assert not np.array_equal(part[0], full[0])
    # a resumed run executes kernels [k_begin, k_end) and nothing before them: kernel 5 reads
    # whatever the caller left in buffer 0, here a constant no earlier kernel would produce
    ints = [p.copy() for p in oracle.run_chain(chain, w, x, 0, 5)]
    ints[0][:] = 3.0
    got = oracle.run_chain(chain, w, x, 5, 6, ints=ints)
    assert np.array_equal(got[0], np.full(8, 3.0, np.float32))
    assert np.array_equal(got[1], oracle.run_op("scale_bias_relu", "f32", [got[0], w[2], w[3]], 8, inner=4, channels=2))


def test_a_kernel_the_oracle_rejects_stops_the_chain_and_is_named():
    import dataclasses
    chain = tiny_mixed_chain("f32", seed=9)
    w, x = make_weights(chain), make_inputs(chain, 0)
    ks = list(chain.kernels)
    ks[5] = dataclasses.replace(ks[5], inner=3)          # 8 elements are not a whole number of [2, 3] planes
    bad = dataclasses.replace(chain, kernels=ks)
    with pytest.raises(ValueError, match="kernel 5"):
        oracle.run_chain(bad, w, x)


def test_no_state_survives_an_iteration():
    # outputs depend on this iteration's inputs only: garbage left in the internal buffers by a
    # previous iteration must not change them (every buffer is written before it is read)
    for chain in (tiny_mixed_chain("bf16", seed=2), elementwise_chain(12, 64, "f32"),
                  decode_chain(batch=2, layers=1, blocks_per_layer=3, hidden=16, n_ext=3)):
        w = make_weights(chain)
        x0, x1 = make_inputs(chain, 0), make_inputs(chain, 1)
        clean = oracle.run_chain(chain, w, x1)
        dirty = oracle.run_chain(chain, w, x0)
        again = oracle.run_chain(chain, w, x1, ints=dirty)
        for o in chain.outputs:
            assert np.array_equal(clean[o], again[o])
        assert any(not np.array_equal(clean[o], oracle.run_chain(chain, w, x0)[o]) for o in chain.outputs)


def test_config_chain_shapes():
    c1 = elementwise_chain()
    assert len(c1.kernels) == 64 and [k.op for k in c1.kernels].count("add") == 22
    assert c1.n_ext_reading_kernels() == 43 and len(c1.kernels[0].ins) == 2
    c2 = decode_chain()
    assert len(c2.kernels) == 511 and c2.n_ext_reading_kernels() == 33
    assert [k.op for k in c2.kernels].count("gemv") == 120
    assert sum(w.nbytes for w in c2.weights[:120]) == 120 * 8388608
    c3 = refresh_stress_chain()
    assert len(c3.kernels) == 256 and all(t.nbytes % 1024 == 0 and 1024 <= t.nbytes <= 2 ** 24 for t in c3.ext)
    assert 300e6 < c3.ext_bytes() < 600e6
    c4 = large_tensor_chain()
    assert len(c4.kernels) == 40 and c4.n_segments == 4 and c4.ext[0].nbytes == 102760448
    assert c4.n_ext_reading_kernels() == 1


def test_decode_chain_stays_in_range_and_gelu_matters():
    # the reading of the decode chain (gains 1 + N(0, 0.02^2), weights N(0, 0.02^2)) keeps the
    # residual stream finite and O(10): a sanity check of the workload recipe through the oracle
    chain = decode_chain(batch=1, layers=2, blocks_per_layer=5, hidden=256, n_ext=4)
    w, x = make_weights(chain), make_inputs(chain, 0)
    out = as_f64(oracle.run_chain(chain, w, x)[0])
    assert np.all(np.isfinite(out)) and 0.5 < out.std() < 50


# ------------------------------------------------------------------ selection
def test_select_paper_examples():
    for name, no_graph, graph, want in read_golden("select_examples.txt"):
        cost = np.array([[float(no_graph), float(graph), math.nan]])
        assert int(oracle.select(cost)[0]) == (0 if int(want) == 0 else 1), name
        # with indirection available and cheaper still, it is taken
        cost[0, 2] = min(float(no_graph), float(graph)) * 0.9
        assert int(oracle.select(cost)[0]) == 2


def test_select_equals_exhaustive_argmin_on_small_tables():
    vals = [1.0, 2.0, 2.0, math.nan, math.inf]
    rows = [r for r in itertools.product(vals, repeat=3) if any(math.isfinite(v) for v in r)]
    for r in rows:
        assert oracle.select(np.array([r])).tolist() == bruteforce.select([r])
    rng = np.random.Generator(np.random.PCG64(1))
    for _ in range(200):
        idx = rng.integers(0, len(rows), 3)
        table = [rows[i] for i in idx]
        assert oracle.select(np.array(table)).tolist() == bruteforce.select(table)   # per segment, independent


def test_select_properties():
    rng = np.random.Generator(np.random.PCG64(2))
    cost = rng.uniform(1, 100, (16, 3))
    cost[3, 2] = math.nan; cost[5, 0] = math.inf
    sel = oracle.select(cost)
    assert np.array_equal(sel, np.nanargmin(np.where(np.isfinite(cost), cost, np.nan), axis=1))
    assert np.array_equal(oracle.select(cost * 7.5), sel)                 # scale invariance
    low = cost.copy(); low[np.arange(16), sel] *= 0.5
    assert np.array_equal(oracle.select(low), sel)                        # a cheaper winner still wins
    assert oracle.select(np.array([[2.0, 2.0, 2.0]]))[0] == 0             # ties: the simpler variant
    assert oracle.select(np.array([[3.0, 2.0, 2.0]]))[0] == 1
    with pytest.raises(ValueError):
        oracle.select(np.array([[1.0, 2.0, 3.0], [math.nan, math.inf, math.nan]]))
    for _ in range(50):
        assert np.array_equal(oracle.select(cost), sel)                   # deterministic


def test_result_does_not_depend_on_the_thread_count():
    """The oracle is parallel only across independent outputs, each summed in a fixed order: one
    thread and all threads give the same bits (so the timed oracle is the checked oracle)."""
    spec = decode_chain(batch=3, layers=2, blocks_per_layer=2, hidden=264, n_ext=3)
    w, x = make_weights(spec), make_inputs(spec, 0)
    n_max = oracle.max_threads()
    try:
        oracle.set_threads(1)
        one = oracle.run_chain(spec, w, x)
        oracle.set_threads(max(2, n_max))
        many = oracle.run_chain(spec, w, x)
    finally:
        oracle.set_threads(n_max)
    for a, b in zip(one, many):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
