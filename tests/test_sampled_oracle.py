"""The sampled use of the oracle (tests/sampled.py: single wires of a network recomputed from the seeds, the
zero-labels-only garblers, En of the plain values) against the oracle run over the whole network, on networks
small enough for both.  CPU only."""
import numpy as np
import pytest

import workloads
from oracle import net as onet
from sampled import SampledOracle, table_slices


def conv_chain_net(seed=9):
    """strided convolution feeding a convolution directly (as in the paper's models f and F), biases, pooling"""
    b = workloads._Builder(seed, 4, 2, 7 * 7 * 2, -2, 2)
    b.net["x"] = b.g.integers(0, 4, 2 * 98).astype(np.int64)
    b.conv(7, 7, 2, 3, 3, stride=1, pad=1, bias=True); b.relu(); b.scale(2)
    b.conv(7, 7, 3, 4, 2, stride=2, pad=0, bias=True)
    b.conv(3, 3, 4, 4, 2, stride=1, pad=0, bias=True); b.relu(); b.scale(1); b.sumpool(2, 2, 4)
    b.dense(3, bias=True); b.sign()
    return b.net


@pytest.mark.parametrize("make", [lambda: workloads.vgg(seed=5, batch=2, width=(3, 4, 5), hw=8),
                                  lambda: workloads.tiny_cnn(seed=8, k=4, batch=2, repeat=2),
                                  conv_chain_net], ids=["vgg-reduced", "tiny-cnn", "conv-chain"])
def test_sampled_wires_equal_whole_network_run(make):
    net = make()
    b = 1
    ref = onet.run(net, 1, b, 0, keep=True)
    so = SampledOracle(net, b)
    g = np.random.default_rng(3)
    checked = 0
    for li, L in enumerate(net["layers"]):
        if L["kind"] not in ("relu", "scale", "sign"):
            continue
        n = so.n[li]
        count = min(5, n)
        for start in {0, n - count, int(g.integers(0, n - count + 1))}:
            r = so.activation(li, start, count)
            for i in range(so.orc.k):
                assert (r["zero_in"][i] == ref["gb"]["zero"][li][i][start:start + count]).all(), (li, "zero in", i)
                assert (r["act_in"][i] == ref["acts"][li][i][start:start + count]).all(), (li, "act in", i)
                assert (r["zero_out"][i] == ref["gb"]["zero"][li + 1][i][start:start + count]).all(), (li, "zero out", i)
                assert (r["act_out"][i] == ref["acts"][li + 1][i][start:start + count]).all(), (li, "act out", i)
            full = ref["gb"]["tables"][L["id"]]
            total = 0
            for off_full, off_run, nbytes in table_slices(so.orc, L, n, start, count):
                assert (r["tables"][off_run:off_run + nbytes] == full[off_full:off_full + nbytes]).all(), (li, off_full)
                total += nbytes
            assert total == r["tables"].size
            checked += 1
    assert checked >= 6


def test_zero_only_garbling_equals_full_garbling():
    """the garblers' zero-labels-only mode returns the zero labels of the full run; a ReLU's output zero labels
    do not depend on its input labels (they are V0 - U0, both drawn)"""
    orc = onet.make_oracle(workloads.tiny(k=5, repeat=1))
    g = workloads.rng(11)
    n = 6
    in0 = [workloads.uniform_labels(g, n, orc.lam(p), p) for p in orc.primes]
    full, _ = orc.relu_garble(3, in0, elem_base=77)
    only = orc.relu_garble(3, in0, elem_base=77, zero_only=True)
    other = orc.relu_garble(3, [np.zeros_like(a) for a in in0], elem_base=77, zero_only=True)
    for a, b_, c in zip(full, only, other):
        assert (a == b_).all() and (a == c).all()
    sfull, _ = orc.scale_garble(4, in0, 3, elem_base=5)
    sonly = orc.scale_garble(4, in0, 3, elem_base=5, zero_only=True)
    for a, b_ in zip(sfull, sonly):
        assert (a == b_).all()
