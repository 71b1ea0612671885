"""GPU parity: linear layers on LabelTensors (dense, conv with padding / stride, sum-pool, bias)
through the C ABI against the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import both, upload_bundle, assert_bundle_equal

pytestmark = pytest.mark.gpu


def run_linear(k, batch, in_h, in_w, in_c, out_c, kh, stride, pad, wlo, whi, bias, seed, garble=True, pool=False):
    from paper_2302_06361_amd import Labels, Layer, DENSE, CONV2D, SUMPOOL
    ctx, orc = both(k)
    g = np.random.default_rng(seed)
    n_in = batch * in_h * in_w * in_c
    x = [workloads.uniform_labels(g, n_in, orc.lam(p), p) for p in orc.primes]
    tin = upload_bundle(ctx, x)
    if pool:
        ref = [orc.sumpool2(i, x[i], batch, in_h, in_w, in_c) for i in range(k)]
        lay = Layer(SUMPOOL, 1, batch, in_h=in_h, in_w=in_w, in_c=in_c)
    else:
        W = g.integers(wlo, whi + 1, (out_c, kh, kh, in_c)).astype(np.int32)
        b = g.integers(-1000, 1000, out_c).astype(np.int32) if bias else None
        ones = [orc.one0(i) if garble else orc.one(i) for i in range(k)]
        ref = [orc.conv2d(i, x[i], batch, in_h, in_w, in_c, out_c, kh, kh, stride, pad, W, b, ones[i]) for i in range(k)]
        wp = ctx.weights_prepare(W.reshape(out_c, -1))
        bd = torch.as_tensor(b).to(ctx.device) if bias else None
        dense = in_h == 1 and in_w == 1 and kh == 1
        lay = Layer(DENSE if dense else CONV2D, 1, batch, in_h=in_h, in_w=in_w, in_c=in_c, out_c=out_c, kh=kh, kw=kh,
                    stride=stride, pad=pad, weights=wp, bias=bd)
    oe, tb, sb = ctx.layer_sizes(lay)
    assert tb == 0 and oe * batch == ref[0].shape[0]
    tout = Labels(ctx, oe * batch, zero=True)
    if garble:
        ctx.garble_layer(lay, tin, tout)
    else:
        ctx.eval_layer(lay, tin, None, tout)
    torch.cuda.synchronize()
    assert_bundle_equal(tout, ref, "linear output")


@pytest.mark.parametrize("garble", [True, False])
def test_dense_small_with_bias(garble):
    run_linear(8, 3, 1, 1, 50, 7, 1, 1, 0, -8, 7, True, 1, garble)


def test_dense_mlp_shapes():
    run_linear(8, 1, 1, 1, 784, 128, 1, 1, 0, -8, 7, False, 2)
    run_linear(8, 1, 1, 1, 128, 10, 1, 1, 0, -8, 7, False, 3)


def test_dense_12_primes_wide_weights():
    run_linear(12, 5, 1, 1, 300, 33, 1, 1, 0, -64, 63, True, 4)


def test_conv_lenet_shapes():
    run_linear(8, 2, 28, 28, 1, 6, 5, 1, 2, -8, 7, False, 5)
    run_linear(8, 2, 14, 14, 6, 16, 5, 1, 0, -8, 7, True, 6)


def test_conv_stride_and_padding():
    run_linear(5, 2, 9, 9, 3, 4, 3, 2, 1, -3, 3, True, 7)
    run_linear(5, 1, 8, 8, 2, 5, 4, 2, 0, -3, 3, False, 8)
    # few outputs and a long reduction (the form with 16 lanes per output), taps outside the image, odd channel count
    run_linear(5, 1, 6, 6, 8, 3, 3, 1, 1, -3, 3, True, 12)
    run_linear(8, 2, 5, 5, 7, 2, 5, 2, 2, -8, 7, True, 13, garble=False)


def test_conv_vgg_block_shape():
    run_linear(12, 1, 8, 8, 16, 32, 3, 1, 1, -16, 15, False, 9)


def test_sumpool():
    run_linear(8, 3, 10, 10, 16, 16, 1, 1, 0, 0, 0, False, 10, pool=True)
    run_linear(12, 2, 6, 4, 5, 5, 1, 1, 0, 0, 0, False, 11, pool=True)


def test_dense_mfma_ragged_tiles_and_bias():
    """dense layers large enough for the MFMA kernel: several K stages, ragged M, K and group tails"""
    run_linear(12, 5, 1, 1, 500, 300, 1, 1, 0, -64, 63, True, 21)
    run_linear(8, 7, 1, 1, 128, 257, 1, 1, 0, -8, 7, False, 22, garble=False)
    run_linear(12, 3, 1, 1, 1030, 70, 1, 1, 0, -64, 63, True, 23, garble=False)


def test_dense_mfma_config4_sample():
    """config 4 shape on a slice: K = 4096 inputs, 96 output rows, batch 2, all 12 primes, weights in [-64, 63]"""
    run_linear(12, 2, 1, 1, 4096, 96, 1, 1, 0, -64, 63, False, 24)


def test_dense_mfma_large_accumulators_and_stage_counts():
    """K = 13000: (p - 1)^2 K passes 2^24 for p = 37, so the two-step reduction of the accumulators runs (with and
    without bias); K = 250 and 192: four and three K stages (every exit of the software pipeline)"""
    run_linear(12, 1, 1, 1, 13000, 70, 1, 1, 0, -64, 63, True, 25)
    run_linear(12, 2, 1, 1, 13000, 40, 1, 1, 0, -64, 63, False, 26, garble=False)
    run_linear(8, 3, 1, 1, 250, 130, 1, 1, 0, -8, 7, False, 27)
    run_linear(8, 3, 1, 1, 192, 130, 1, 1, 0, -8, 7, True, 28)


def test_conv_mfma_shapes():
    """convolutions that take the MFMA kernel as an implicit GEMM (channels a multiple of 4): stride, padding,
    bias, batches, a 1x1 kernel, pixel counts that leave ragged group tiles, K not a multiple of 64"""
    run_linear(12, 2, 9, 7, 8, 40, 3, 2, 1, -16, 15, True, 31)
    run_linear(8, 3, 6, 6, 4, 70, 5, 1, 2, -8, 7, False, 32)
    run_linear(8, 1, 5, 5, 64, 64, 1, 1, 0, -8, 7, True, 33, garble=False)
    run_linear(12, 1, 16, 16, 12, 48, 3, 1, 1, -16, 15, False, 34)
    run_linear(5, 2, 7, 7, 20, 33, 3, 1, 0, -3, 3, True, 35)


def test_dense_mfma_both_tile_shapes(monkeypatch):
    """the 256 x 256 and the 128 x 512 block tiles of the MFMA kernel, forced in turn"""
    for shape in ("big", "wide"):
        monkeypatch.setenv("DASH_GEMM_TILE", shape)
        run_linear(12, 5, 1, 1, 500, 300, 1, 1, 0, -64, 63, True, 41)
        run_linear(8, 40, 1, 1, 192, 100, 1, 1, 0, -8, 7, False, 42, garble=False)
        run_linear(12, 2, 9, 7, 8, 40, 3, 2, 1, -16, 15, True, 43)
