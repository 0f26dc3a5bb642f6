"""Dispatch merging at capture: a graph that plays runs of small kernels with one dispatch (operands
handed on in registers) leaves the same bits behind as eager launches and as the graph with one node
per kernel -- at every batch size that merges, with external and broadcast operands inside a run, with
more live buffers than register slots, and on chains where a run must be cut because a kernel re-reads
a buffer in another pattern than element for element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_19779_amd as pg
from gpu_util import Harness, assert_close, same_bits, say, stepwise_check
from pg_workloads import (ChainSpec, KernelSpec, TensorSpec, Ref, EXT, INT, WEIGHT, decode_chain, elementwise_chain,
                          make_inputs)

pytestmark = pytest.mark.gpu


def _all_modes(h, x_dev):
    outs = {}
    for mode in ("eager", "copy", "indirect"):
        h.scrub()
        outs[mode] = h.run(mode, x_dev)
    return outs


@pytest.mark.parametrize("batch", [1, 2, 3, 4])
def test_merged_graphs_equal_eager_and_unmerged_graphs(batch):
    spec = decode_chain(batch=batch, layers=3, blocks_per_layer=4, hidden=2048, n_ext=6)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    # the first RMSNorm; then per sub-block the GEMV and one dispatch for GELU, add, (input add,) next RMSNorm
    assert unmerged == len(spec.kernels) and merged == 1 + 2 * 12, (merged, unmerged)
    h.chain.capture(h.stream)
    x_np, x_dev = h.inputs(0)
    want = h.oracle(x_np)[0]
    on = _all_modes(h, x_dev)
    assert same_bits(on["eager"][0], on["copy"][0]) and same_bits(on["eager"][0], on["indirect"][0])
    assert_close(on["eager"][0], want, "bf16", f"decode chain batch {batch}")
    for t in range(1, 8):
        x_np, x_dev = h.inputs(t)
        ref = h.run("eager", x_dev)[0]
        h.scrub()
        assert same_bits(h.run("indirect" if t % 2 else "copy", x_dev)[0], ref), t
    h.chain.set_dispatch_merge(False)
    h.chain.capture(h.stream)
    off = _all_modes(h, x_dev)
    assert same_bits(off["copy"][0], ref) and same_bits(off["indirect"][0], ref)
    h.close()


def _mixed_run_chain(dtype, n):
    """One run-friendly chain with every hazard the planner has to respect: external operands inside a
    run, a broadcast operand from a weight, more live buffers than register slots, a kernel that re-reads
    a buffer of the run with a broadcast period (the run must be cut before it), a write to a buffer that
    the run has read with a broadcast period (cut as well), in-place and out-of-place forms."""
    cols = 2048 if dtype == "bf16" else 1024
    rows = n // cols
    ks = [KernelSpec("add", dtype, 0, (Ref(EXT, 0), Ref(EXT, 1)), n, m=n),            # x0 = e0 + e1
          KernelSpec("mul", dtype, 1, (Ref(INT, 0), Ref(WEIGHT, 0)), n, m=24),        # x1 = x0 * w0[i % 24]
          KernelSpec("add", dtype, 2, (Ref(INT, 1), Ref(INT, 0)), n, m=n),            # x2 = x1 + x0
          KernelSpec("add", dtype, 3, (Ref(INT, 2), Ref(EXT, 2)), n, m=n),            # x3 = x2 + e2      (4th live buffer)
          KernelSpec("mul", dtype, 0, (Ref(INT, 0), Ref(INT, 3)), n, m=n),            # x0 = x0 * x3      (x0 may have left its slot)
          KernelSpec("rmsnorm", dtype, 1, (Ref(INT, 0), Ref(WEIGHT, 1)), cols, rows=rows, cols=cols, eps=1e-5),
          KernelSpec("add", dtype, 2, (Ref(INT, 2), Ref(INT, 1)), n, m=8),            # x2 += x1[i % 8]: x1 was produced in the run
          KernelSpec("mul", dtype, 3, (Ref(INT, 2), Ref(INT, 3)), n, m=16),           # x3 = x2 * x3[i % 16]: in-place on a broadcast operand is not allowed -> different buffers
          KernelSpec("add", dtype, 1, (Ref(INT, 1), Ref(EXT, 0)), n, m=n)]            # x1 += e0
    # kernel 7 as written would overlap out with operand 1; use a fifth buffer for its output
    ks[7] = KernelSpec("mul", dtype, 4, (Ref(INT, 2), Ref(INT, 3)), n, m=16)
    ks.append(KernelSpec("add", dtype, 3, (Ref(INT, 4), Ref(INT, 1)), n, m=n))          # x3 = x4 + x1: writes what kernel 7 read with a period
    if dtype == "bf16":
        ks.insert(3, KernelSpec("gelu", dtype, 2, (Ref(INT, 2),), n))
    ext = [TensorSpec(dtype, n) for _ in range(3)]
    ints = [TensorSpec(dtype, n) for _ in range(5)]
    weights = [TensorSpec(dtype, 24, ("normal", 1.0, 0.3)), TensorSpec(dtype, cols, ("normal", 1.0, 0.1))]
    return ChainSpec(f"mixed_run_{dtype}_{n}", ks, ext, ints, weights, [0, 1, 2, 3, 4], 5150)


@pytest.mark.parametrize("dtype,rows", [("bf16", 1), ("bf16", 3), ("bf16", 4), ("f32", 1), ("f32", 4)])
def test_runs_with_external_broadcast_and_evicted_operands(dtype, rows):
    n = rows * (2048 if dtype == "bf16" else 1024)
    spec = _mixed_run_chain(dtype, n)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    say(f"{spec.name}: {unmerged} kernels in {merged} dispatches")
    assert merged < unmerged and merged >= 3
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        want = h.oracle(x_np)
        outs = _all_modes(h, x_dev)
        for o in range(len(spec.outputs)):
            assert same_bits(outs["eager"][o], outs["copy"][o]) and same_bits(outs["eager"][o], outs["indirect"][o]), (t, o)
        h.scrub()
        stepwise_check(h, x_np, x_dev)            # every kernel against the oracle on the inputs it read
    h.chain.set_dispatch_merge(False)
    h.chain.capture(h.stream)
    off = _all_modes(h, x_dev)
    for o in range(len(spec.outputs)):
        assert same_bits(off["copy"][o], outs["eager"][o]) and same_bits(off["indirect"][o], outs["eager"][o])
    h.close()


def test_runs_of_elementwise_kernels():
    """Config 1: add and mul on 4096 fp32 elements merge pairwise into single-workgroup dispatches, the
    fp32 GELU between them stays a kernel of its own; bf16 chains of small kernels merge four at a time."""
    spec = elementwise_chain()
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    assert unmerged == 64 and merged == 43, merged
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        want = h.oracle(x_np)[0]
        outs = _all_modes(h, x_dev)
        assert same_bits(outs["eager"][0], outs["copy"][0]) and same_bits(outs["eager"][0], outs["indirect"][0])
        assert_close(outs["eager"][0], want, "f32", "config 1")
    h.close()
    spec = elementwise_chain(n_kernels=40, numel=5000, dtype="bf16")
    h = Harness(spec, capture=False)
    assert h.chain.graph_dispatches() == (10, 40)
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        want = h.oracle(x_np)[0]
        outs = _all_modes(h, x_dev)
        assert same_bits(outs["eager"][0], outs["copy"][0]) and same_bits(outs["eager"][0], outs["indirect"][0])
        assert_close(outs["eager"][0], want, "bf16", "bf16 elementwise chain", rtol=0.25)   # 40 kernels deep: the step checks are elsewhere
    h.close()
