"""Dispatch merging at capture: a graph that plays runs of small kernels with one dispatch (operands
handed on in registers) leaves the same bits behind as eager launches and as the graph with one node
per kernel -- at every batch size that merges, with external and broadcast operands inside a run, with
more live buffers than register slots, and on chains where a run must be cut because a kernel re-reads
a buffer in another pattern than element for element."""
import dataclasses

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


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 8, 13, 16, 17, 24, 32, 48, 63, 64, 72, 80, 81, 100, 128])
def test_merged_graphs_equal_eager_and_unmerged_graphs(batch):
    spec = decode_chain(batch=batch, layers=3, blocks_per_layer=4, hidden=2048, n_ext=6)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    # per sub-block one dispatch: the GEMV with the RMSNorm as its prologue and GELU, add (and input add) as its
    # epilogue.  Sub-blocks 1..11 overwrite the stream they normalise and write its other copy; eleven is odd,
    # so the last of them is split into RMSNorm + GEMV dispatch and leaves the stream in its first copy.
    # From five rows on the GEMV runs on the matrix cores: GELU, add (and input add) still ride in its dispatch; the
    # RMSNorm is a prologue up to 32 rows (one tile of rows per workgroup, one workgroup per CU) and stands alone above.
    assert unmerged == len(spec.kernels) and merged == (12 + 1 if batch <= 32 else 2 * 12), (merged, unmerged)
    h.chain.capture(h.stream)
    x_np, x_dev = h.inputs(0)
    want = h.oracle(x_np)[0]
    on = _all_modes(h, x_dev)
    assert same_bits(on["eager"][0], on["copy"][0]) and same_bits(on["eager"][0], on["indirect"][0])
    if batch <= 4:
        assert_close(on["eager"][0], want, "bf16", f"decode chain batch {batch}")
    else:       # the matrix-core forms: every kernel against the oracle on the inputs it read, first and last row
        h.scrub()
        stepwise_check(h, x_np, x_dev, rows=[0, batch - 1])
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


@pytest.mark.parametrize("batch,cuts", [(1, (5,)), (2, (4, 9)), (4, (1, 2, 3)), (7, (2, 5)), (16, (3,)), (29, (4,))])
def test_prologue_runs_leave_every_segment_in_the_first_copy(batch, cuts):
    """The decode chain cut into segments after the given sub-blocks: a segment with an odd number of
    renaming runs splits its last one, so that any mixture of modes per segment (eager reads and writes the
    first copy only) sees the stream where it expects it; the step-by-step check pins every kernel."""
    spec = decode_chain(batch=batch, layers=2, blocks_per_layer=5, hidden=2048, n_ext=4)
    ks, seg, sub = [], 0, -1
    for k in spec.kernels:
        if k.op == "rmsnorm":
            sub += 1
            if sub in cuts:
                seg += 1
        ks.append(dataclasses.replace(k, segment=seg))
    spec = ChainSpec(spec.name + "_cut", ks, spec.ext, spec.ints, spec.weights, spec.outputs, spec.seed, meta=dict(spec.meta))
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    say(f"{spec.name}: {unmerged} kernels in {merged} dispatches")
    assert merged < 2 * 10
    h.chain.capture(h.stream)
    n_seg = len(cuts) + 1
    for t in range(4):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        assert same_bits(outs["eager"][0], outs["copy"][0]) and same_bits(outs["eager"][0], outs["indirect"][0]), t
        for pattern in range(3 ** n_seg if n_seg <= 3 else 0, 0, -7):      # a spread of per-segment mode mixtures
            modes = [(pattern // 3 ** i) % 3 for i in range(n_seg)]
            modes[0] = modes[0] or 1
            # a segment without external operands has no indirect mode
            modes = [m if (m != 2 or _seg_has_ext(spec, i)) else 1 for i, m in enumerate(modes)]
            h.scrub()
            assert same_bits(h.run("selected", x_dev, modes)[0], outs["eager"][0]), (t, modes)
        h.scrub()
        stepwise_check(h, x_np, x_dev)
    h.close()


def _seg_has_ext(spec, seg):
    return any(r.kind == EXT for k in spec.kernels if k.segment == seg for r in k.ins)


@pytest.mark.parametrize("rows", [1, 3, 5, 8, 11, 16, 17, 25, 32, 33])
def test_prologue_hazards(rows):
    """RMSNorm -> GEMV pairs whose neighbours make the prologue form harder: (a) the GEMV itself overwrites
    the normalised stream; (b) the stream's buffer is larger than what the run rewrites (no renaming: the run
    must not take the prologue form and overwrite x, or else keep the rest of the buffer visible); (c) a
    kernel of the epilogue reads the normalised rows back (stored by one workgroup only: must be cut);
    (d) the gain comes from an internal buffer; (e) x and the gain are external."""
    H = 2048
    N = rows * H
    X, T1, T2, BIG, G = 0, 1, 2, 3, 4
    ks = [KernelSpec("add", "bf16", X, (Ref(EXT, 0), Ref(EXT, 0)), N, m=N),                                   # x = 2 e0
          KernelSpec("add", "bf16", BIG, (Ref(EXT, 2), Ref(EXT, 2)), 2 * N, m=2 * N),                         # big = 2 e2   (2N elements)
          KernelSpec("mul", "bf16", G, (Ref(WEIGHT, 1), Ref(WEIGHT, 1)), H, m=H),                             # g = w1^2
          # (e) external x and gain, epilogue writes x's internal namesake
          KernelSpec("rmsnorm", "bf16", T1, (Ref(EXT, 0), Ref(EXT, 1)), H, rows=rows, cols=H, eps=1e-6),
          KernelSpec("gemv", "bf16", T2, (Ref(WEIGHT, 0), Ref(INT, T1)), H, rows=rows, cols=H),
          KernelSpec("add", "bf16", X, (Ref(INT, X), Ref(INT, T2)), N, m=N),
          # (a) the GEMV writes x
          KernelSpec("rmsnorm", "bf16", T1, (Ref(INT, X), Ref(WEIGHT, 1)), H, rows=rows, cols=H, eps=1e-6),
          KernelSpec("gemv", "bf16", X, (Ref(WEIGHT, 0), Ref(INT, T1)), H, rows=rows, cols=H),
          KernelSpec("gelu", "bf16", X, (Ref(INT, X),), N),
          # (d) gain from an internal buffer, (c) the epilogue's second kernel reads T1 back
          KernelSpec("rmsnorm", "bf16", T1, (Ref(INT, X), Ref(INT, G)), H, rows=rows, cols=H, eps=1e-6),
          KernelSpec("gemv", "bf16", T2, (Ref(WEIGHT, 0), Ref(INT, T1)), H, rows=rows, cols=H),
          KernelSpec("add", "bf16", X, (Ref(INT, X), Ref(INT, T2)), N, m=N),
          KernelSpec("add", "bf16", T2, (Ref(INT, T2), Ref(INT, T1)), N, m=N),
          # (b) normalise the head of the big buffer, then overwrite that head
          KernelSpec("rmsnorm", "bf16", T1, (Ref(INT, BIG), Ref(WEIGHT, 1)), H, rows=rows, cols=H, eps=1e-6),
          KernelSpec("gemv", "bf16", T2, (Ref(WEIGHT, 0), Ref(INT, T1)), H, rows=rows, cols=H),
          KernelSpec("add", "bf16", BIG, (Ref(INT, BIG), Ref(INT, T2)), N, m=N),
          KernelSpec("add", "bf16", BIG, (Ref(INT, BIG), Ref(EXT, 2)), 2 * N, m=2 * N),                       # reads the tail the run left alone
          ]
    spec = ChainSpec(f"prologue_hazards_{rows}", ks,
                     [TensorSpec("bf16", N), TensorSpec("bf16", H, ("normal", 1.0, 0.1)), TensorSpec("bf16", 2 * N)],
                     [TensorSpec("bf16", N), TensorSpec("bf16", N), TensorSpec("bf16", N), TensorSpec("bf16", 2 * N), TensorSpec("bf16", H)],
                     [TensorSpec("bf16", H * H, ("normal", 0.0, 0.02)), TensorSpec("bf16", H, ("normal", 1.0, 0.1))],
                     [X, T1, T2, BIG], 6010)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    say(f"{spec.name}: {unmerged} kernels in {merged} dispatches")
    assert merged < unmerged
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        for o in range(len(spec.outputs)):
            assert same_bits(outs["eager"][o], outs["copy"][o]) and same_bits(outs["eager"][o], outs["indirect"][o]), (t, o)
        h.scrub()
        stepwise_check(h, x_np, x_dev)
    h.close()


@pytest.mark.parametrize("rows,n", [(1, 1027), (3, 1100), (4, 2040), (6, 1030), (8, 40), (12, 72), (16, 1029), (17, 33), (20, 1030), (32, 48),
                                    (32, 1100), (33, 1030)])
def test_prologue_with_other_output_widths(rows, n):
    """RMSNorm -> GEMV -> GELU -> add where the GEMV's output has n columns, not the 2048 of the stream (a ragged
    last column block in every form, fewer column blocks than CUs, a single one): the prologue rides in front
    (up to 32 rows), the normalised rows are stored once, and a later kernel reads them back."""
    H = 2048
    N = rows * n
    ks = [KernelSpec("add", "bf16", 0, (Ref(EXT, 0), Ref(EXT, 0)), rows * H, m=rows * H),                       # x = 2 e0
          KernelSpec("rmsnorm", "bf16", 1, (Ref(INT, 0), Ref(WEIGHT, 1)), H, rows=rows, cols=H, eps=1e-6),      # t = norm(x)
          KernelSpec("gemv", "bf16", 2, (Ref(WEIGHT, 0), Ref(INT, 1)), n, rows=rows, cols=H),                   # y = t W^T
          KernelSpec("gelu", "bf16", 2, (Ref(INT, 2),), N),
          KernelSpec("add", "bf16", 2, (Ref(INT, 2), Ref(EXT, 1)), N, m=N),
          KernelSpec("mul", "bf16", 0, (Ref(INT, 0), Ref(INT, 1)), rows * H, m=rows * H),                       # x = x * t: reads the stored rows
          KernelSpec("rmsnorm", "bf16", 1, (Ref(EXT, 0), Ref(WEIGHT, 1)), H, rows=rows, cols=H, eps=1e-6),      # external x this time
          KernelSpec("gemv", "bf16", 3, (Ref(WEIGHT, 0), Ref(INT, 1)), n, rows=rows, cols=H),
          KernelSpec("add", "bf16", 3, (Ref(INT, 3), Ref(INT, 2)), N, m=N),
          ]
    spec = ChainSpec(f"prologue_width_{rows}x{n}", ks,
                     [TensorSpec("bf16", rows * H), TensorSpec("bf16", N)],
                     [TensorSpec("bf16", rows * H), TensorSpec("bf16", rows * H), TensorSpec("bf16", N), TensorSpec("bf16", N)],
                     [TensorSpec("bf16", n * H, ("normal", 0.0, 0.02)), TensorSpec("bf16", H, ("normal", 1.0, 0.1))],
                     [0, 1, 2, 3], 6020)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    say(f"{spec.name}: {unmerged} kernels in {merged} dispatches")
    # up to 32 rows [add] [RMSNorm, GEMV, GELU, add] [mul] [RMSNorm, GEMV, add]; above, each RMSNorm joins the elementwise kernel in front of it
    assert merged == 4, (merged, unmerged)
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        for o in range(len(spec.outputs)):
            assert same_bits(outs["eager"][o], outs["copy"][o]) and same_bits(outs["eager"][o], outs["indirect"][o]), (t, o)
        h.scrub()
        stepwise_check(h, x_np, x_dev)
    h.close()


@pytest.mark.parametrize("rows", [1, 3, 6, 12, 20, 70, 100])
@pytest.mark.parametrize("order", [0, 1])
def test_decoder_tail_with_a_broadcast_operand_and_either_operand_order(rows, order):
    """GEMV -> GELU -> add -> add, the tail of a decoder block, which the GEMV's dispatch recognises and plays
    straight through: here the second add takes a bias with a period of one row, and the adds name their
    operand from memory first (order 0) or second (order 1)."""
    H = 2048
    N = rows * H
    X, Y, Z = 1, 0, 2
    S = X if order == 0 else Z        # in place only over the first operand: with y named first the sum goes to a third buffer
    ks = [KernelSpec("add", "bf16", X, (Ref(EXT, 1), Ref(EXT, 1)), N, m=N),                          # x = 2 e1
          KernelSpec("gemv", "bf16", Y, (Ref(WEIGHT, 0), Ref(EXT, 0)), H, rows=rows, cols=H),        # y
          KernelSpec("gelu", "bf16", Y, (Ref(INT, Y),), N),                                          # y = gelu(y)
          KernelSpec("add", "bf16", S, (Ref(INT, X), Ref(INT, Y)) if order == 0 else (Ref(INT, Y), Ref(INT, X)), N, m=N),   # s = x + y / y + x
          KernelSpec("add", "bf16", S, (Ref(INT, S), Ref(WEIGHT, 1)), N, m=H),                       # s += bias[col]: a period of one row
          KernelSpec("gemv", "bf16", Y, (Ref(WEIGHT, 0), Ref(INT, S)), H, rows=rows, cols=H),        # a second block: reads s
          KernelSpec("gelu", "bf16", Y, (Ref(INT, Y),), N),
          KernelSpec("add", "bf16", Z if order == 0 else X, (Ref(EXT, 1), Ref(INT, Y)) if order == 0 else (Ref(INT, Y), Ref(EXT, 1)), N, m=N)]   # two kernels only
    spec = ChainSpec(f"decoder_tail_{rows}_{order}", ks,
                     [TensorSpec("bf16", N), TensorSpec("bf16", N)],
                     [TensorSpec("bf16", N), TensorSpec("bf16", N), TensorSpec("bf16", N)],
                     [TensorSpec("bf16", H * H, ("normal", 0.0, 0.02)), TensorSpec("bf16", H, ("normal", 0.0, 0.5))],
                     [0, 1, 2], 6030)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    say(f"{spec.name}: {unmerged} kernels in {merged} dispatches")
    assert merged == 3, (merged, unmerged)      # [add] [GEMV, GELU, add, add] [GEMV, GELU, add]
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        for o in range(len(spec.outputs)):
            assert same_bits(outs["eager"][o], outs["copy"][o]) and same_bits(outs["eager"][o], outs["indirect"][o]), (t, o)
        h.scrub()
        stepwise_check(h, x_np, x_dev)
    h.close()


@pytest.mark.parametrize("rows,n", [(1, 1027), (2, 2048), (3, 1030), (4, 1100),
                                    (5, 1027), (8, 2048), (13, 1030), (16, 40), (17, 1100), (40, 1029), (63, 48), (64, 1030), (70, 1030), (80, 2048), (81, 40), (100, 2048), (130, 70)])
def test_gemv_with_elementwise_epilogue(rows, n):
    """A GEMV (ragged last workgroup for odd n) followed by GELU in place, an add with an external operand,
    a mul with a broadcast weight and further kernels: the first three ride in the GEMV's dispatch, the rest
    form a run of their own.  A second GEMV is followed by a kernel that overwrites the buffer the GEMV reads
    h from: that one must not ride along."""
    H = 2048
    N = rows * n
    ks = [KernelSpec("gemv", "bf16", 0, (Ref(WEIGHT, 0), Ref(EXT, 0)), n, rows=rows, cols=H),      # y
          KernelSpec("gelu", "bf16", 0, (Ref(INT, 0),), N),                                          # y = gelu(y)
          KernelSpec("add", "bf16", 1, (Ref(EXT, 1), Ref(INT, 0)), N, m=N),                          # x = e1 + y
          KernelSpec("mul", "bf16", 1, (Ref(INT, 1), Ref(WEIGHT, 1)), N, m=5),                       # x *= w1[i % 5]
          KernelSpec("add", "bf16", 2, (Ref(INT, 1), Ref(INT, 0)), N, m=N),                          # z = x + y      (fourth: its own dispatch)
          KernelSpec("gemv", "bf16", 3, (Ref(WEIGHT, 0), Ref(INT, 4)), n, rows=rows, cols=H),        # needs int 4 = h2, written below first
          ]
    # h2 must exist before the second GEMV: produce it first from the external h
    ks.insert(5, KernelSpec("add", "bf16", 4, (Ref(EXT, 0), Ref(EXT, 0)), rows * H, m=rows * H))     # h2 = 2 * e0
    ks.append(KernelSpec("mul", "bf16", 3, (Ref(INT, 3), Ref(INT, 2)), N, m=N))                      # epilogue of the second GEMV
    ks.append(KernelSpec("add", "bf16", 4, (Ref(EXT, 0), Ref(EXT, 0)), rows * H, m=rows * H))        # rewrites h2: other element count, separate anyway
    spec = ChainSpec(f"gemv_epilogue_{rows}x{n}", ks,
                     [TensorSpec("bf16", rows * H), TensorSpec("bf16", N)],
                     [TensorSpec("bf16", N), TensorSpec("bf16", N), TensorSpec("bf16", N), TensorSpec("bf16", N), TensorSpec("bf16", rows * H)],
                     [TensorSpec("bf16", n * H, ("normal", 0.0, 0.02)), TensorSpec("bf16", 5, ("normal", 1.0, 0.3))], [0, 1, 2, 3, 4], 6006)
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    say(f"{spec.name}: {unmerged} kernels in {merged} dispatches")
    # [gemv gelu add mul] [add] [add] [gemv mul] [add]; the two adds in the middle merge too when they have the same
    # element count (a whole number of vectors); below 1024 columns of output the one-to-four-row GEMV has no epilogue form
    assert unmerged == 9 and merged == (4 if n == H else 5), merged
    h.chain.capture(h.stream)
    for t in range(4):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        for o in range(5):
            assert same_bits(outs["eager"][o], outs["copy"][o]) and same_bits(outs["eager"][o], outs["indirect"][o]), (t, o)
        h.scrub()
        stepwise_check(h, x_np, x_dev)
    h.close()


def test_epilogue_never_overwrites_what_the_gemv_is_reading():
    """A kernel after the GEMV that writes the buffer h comes from has the right shape to ride along only
    when n == cols; it must still get a dispatch of its own (other workgroups are still reading h)."""
    H = 2048
    ks = [KernelSpec("add", "bf16", 0, (Ref(EXT, 0), Ref(EXT, 0)), H, m=H),                  # h = 2 e0
          KernelSpec("gemv", "bf16", 1, (Ref(WEIGHT, 0), Ref(INT, 0)), H, rows=1, cols=H),   # y = W h
          KernelSpec("add", "bf16", 0, (Ref(INT, 1), Ref(EXT, 0)), H, m=H),                  # h = y + e0   <- writes h
          KernelSpec("gelu", "bf16", 1, (Ref(INT, 1),), H)]
    spec = ChainSpec("epilogue_hazard", ks, [TensorSpec("bf16", H)], [TensorSpec("bf16", H), TensorSpec("bf16", H)],
                     [TensorSpec("bf16", H * H, ("normal", 0.0, 0.02))], [0, 1], 6007)
    h = Harness(spec, capture=False)
    assert h.chain.graph_dispatches() == (3, 4)      # [add] [gemv] [add gelu]
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        for o in range(2):
            assert same_bits(outs["eager"][o], outs["copy"][o]) and same_bits(outs["eager"][o], outs["indirect"][o]), (t, o)
        h.scrub()
        stepwise_check(h, x_np, x_dev)
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


@pytest.mark.parametrize("n_kernels,numel,nodes", [(9, 7, 3), (13, 16384, 4), (30, 16385, 30), (30, 20000, 20), (12, 1 << 20, 8)])
def test_runs_of_small_and_large_fp32_kernels(n_kernels, numel, nodes):
    """fp32 runs on small tensors (up to 16384 elements) work one element per lane and take the GELU along, four
    kernels per dispatch; larger ones work in 16-byte vectors (a whole number of them) and leave the GELU, which is
    evaluated in fp64, a dispatch of its own."""
    spec = elementwise_chain(n_kernels=n_kernels, numel=numel)
    h = Harness(spec, capture=False)
    assert h.chain.graph_dispatches() == (nodes, n_kernels)
    h.chain.capture(h.stream)
    for t in range(3):
        x_np, x_dev = h.inputs(t)
        outs = _all_modes(h, x_dev)
        assert same_bits(outs["eager"][0], outs["copy"][0]) and same_bits(outs["eager"][0], outs["indirect"][0])
        h.scrub()
        stepwise_check(h, x_np, x_dev)
    h.close()


def test_runs_of_elementwise_kernels():
    """Config 1: add, mul and GELU on 4096 fp32 elements merge four at a time into dispatches of one element per
    lane; bf16 chains of small kernels merge four at a time in 16-byte vectors."""
    spec = elementwise_chain()
    h = Harness(spec, capture=False)
    merged, unmerged = h.chain.graph_dispatches()
    assert unmerged == 64 and merged == 16, merged
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
