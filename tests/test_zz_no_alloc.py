"""dash_eval_layer_noalloc (the entry point for callers that cannot allocate: its scratch buffer is a fixed device
array inside the library) against dash_eval_layer, through the C ABI: two calls in a row, the second with a smaller
input, every output byte equal; sizes past the array's capacity are refused."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import both, upload_bundle

pytestmark = pytest.mark.gpu


def _case(ctx, orc, kind, n, repeat, layer_id, elem_base, seed):
    """garble one activation layer over n values, then evaluate it through both entry points"""
    from paper_2302_06361_amd import Labels, Layer, RELU, SCALE
    from paper_2302_06361_amd.binding import NOALLOC_SCRATCH_BYTES
    k = ctx.k
    P = int(np.prod(ctx.primes))
    X = np.random.default_rng(seed).integers(0, P, n)
    zero = [orc.input_labels(1000 * seed, n, i) for i in range(k)]
    act = [orc.encode(i, X, zero[i]) for i in range(k)]
    lay = Layer(RELU if kind == "relu" else SCALE, layer_id, n, elem_base=elem_base, repeat=repeat)
    oe, tb, sb = ctx.layer_sizes(lay)
    assert 0 < sb <= NOALLOC_SCRATCH_BYTES
    tz, ta = upload_bundle(ctx, zero), upload_bundle(ctx, act)
    oz = Labels(ctx, n, zero=True)
    tables = torch.zeros(tb, dtype=torch.uint8, device=ctx.device)
    scratch = torch.zeros(sb + 256, dtype=torch.uint8, device=ctx.device)
    ctx.garble_layer(lay, tz, oz, tables, scratch)
    want, got = Labels(ctx, n, zero=True), Labels(ctx, n, zero=True)
    scratch.fill_(0x5A)
    ctx.eval_layer(lay, ta, tables, want, scratch)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ctx.eval_layer_noalloc(lay, ta, tables, got)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for i in range(k):
        a, b = want.to_numpy(i), got.to_numpy(i)
        assert (a == b).all(), (kind, n, "residue", i)
        assert got.pad_is_zero(i)
    # and both are what the oracle evaluates
    if kind == "relu":
        r0, rt = orc.relu_garble(layer_id, zero, elem_base)
        r = orc.relu_eval(layer_id, act, rt, elem_base)
    else:
        r0, rt = orc.scale_garble(layer_id, zero, repeat, elem_base)
        r = orc.scale_eval(layer_id, act, rt, repeat, elem_base)
    for i in range(k):
        assert (got.to_numpy(i) == r[i]).all(), (kind, n, "oracle, residue", i)


def test_noalloc_eval_equals_eval_two_calls_second_smaller():
    ctx, orc = both(8)
    _case(ctx, orc, "scale", 700, 2, 9, 12345, seed=1)      # uses most scratch wires, several tiles and a ragged tail
    _case(ctx, orc, "relu", 130, 1, 10, 7, seed=2)          # smaller: the array still holds the first call's wires
    _case(ctx, orc, "scale", 1, 1, 11, 0, seed=3)


def test_noalloc_eval_refuses_what_does_not_fit():
    from paper_2302_06361_amd import Labels, Layer, SCALE, DashError
    from paper_2302_06361_amd.binding import NOALLOC_SCRATCH_BYTES
    ctx, orc = both(8)
    n = 200000
    lay = Layer(SCALE, 3, n, repeat=1)
    oe, tb, sb = ctx.layer_sizes(lay)
    assert sb > NOALLOC_SCRATCH_BYTES
    t = Labels(ctx, 16)          # never touched: the size check comes before anything is launched
    with pytest.raises(DashError, match="size not supported"):
        ctx.eval_layer_noalloc(lay, t, torch.zeros(16, dtype=torch.uint8, device=ctx.device), t)
    torch.cuda.synchronize()
