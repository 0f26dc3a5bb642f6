"""pg_eager_static (one eager pass with the internal buffers in the library's static device array)
against pg_eager on a caller-provided workspace and against the CPU oracle: two calls in a row, the
second on a smaller chain, then the first chain again; a chain that does not fit is refused before
anything is launched."""
import numpy as np
import pytest
import torch

import oracle
import paper_2503_19779_amd as pg
from gpu_util import Harness, assert_close, same_bits, say
from paper_2503_19779_amd.binding import to_device, to_numpy
from pg_workloads import decode_chain, elementwise_chain, make_inputs, make_weights

pytestmark = pytest.mark.gpu


def _one(spec, t, stream):
    """(static result, workspace-eager result, oracle result) for iteration t of `spec`."""
    h = Harness(spec, capture=False)
    x_np, x_dev = h.inputs(t)
    o = spec.outputs[0]
    numel = spec.ints[o].numel
    out = torch.full((numel,), float("nan"), dtype=torch.bfloat16 if spec.ints[o].dtype == "bf16" else torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    pg.eager_static(spec, h.w_dev, x_dev, o, out, stream)
    stream.synchronize()
    got = to_numpy(out)
    h.scrub()
    ref = h.run("eager", x_dev)[0]
    want = h.oracle(x_np)[0]
    h.close()
    return got, ref, want


def test_static_scratch_matches_workspace_eager_on_two_calls_in_a_row():
    stream = torch.cuda.Stream()
    big = decode_chain(batch=4, layers=2, blocks_per_layer=3, hidden=1024, n_ext=4)      # 27 kernels, 3 x 8 KB internal
    small = decode_chain(batch=1, layers=1, blocks_per_layer=2, hidden=256, n_ext=2, seed=77)   # 9 kernels, 3 x 512 B
    f32 = elementwise_chain(n_kernels=12, numel=1000)
    for name, spec, t in (("first", big, 0), ("second, smaller", small, 1), ("first again", big, 2), ("fp32", f32, 0)):
        say(f"pg_eager_static: {name}: {spec.name}, {len(spec.kernels)} kernels")
        got, ref, want = _one(spec, t, stream)
        assert same_bits(got, ref), name
        dt = spec.kernels[0].dtype
        assert_close(got, want, dt, f"pg_eager_static, {name}")


def test_static_scratch_rejects_what_does_not_fit():
    stream = torch.cuda.Stream()
    too_big = elementwise_chain(n_kernels=3, numel=pg.STATIC_SCRATCH_BYTES // 4 + 64)     # one fp32 buffer just over the array
    h = Harness(too_big, capture=False)
    x_np, x_dev = h.inputs(0)
    out = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    with pytest.raises(pg.PgError) as e:
        pg.eager_static(too_big, h.w_dev, x_dev, 0, out, stream)
    assert e.value.status == 4 and "static scratch" in str(e.value)
    fits = elementwise_chain(n_kernels=3, numel=pg.STATIC_SCRATCH_BYTES // 4)           # exactly the array
    h2 = Harness(fits, capture=False)
    x2_np, x2_dev = h2.inputs(0)
    out2 = torch.empty(fits.ints[0].numel, dtype=torch.float32, device="cuda:0")
    pg.eager_static(fits, h2.w_dev, x2_dev, 0, out2, stream)
    stream.synchronize()
    assert same_bits(to_numpy(out2), h2.run("eager", x2_dev)[0])
    with pytest.raises(pg.PgError):
        pg.eager_static(fits, h2.w_dev, x2_dev, 3, out2, stream)      # no such internal buffer
    with pytest.raises(pg.PgError):
        pg.eager_static(fits, h2.w_dev, x2_dev, 0, torch.empty(fits.ints[0].numel + 1, dtype=torch.float32, device="cuda:0"), stream)
    h.close()
    h2.close()
