"""Whole-network pins for the oracle: the decoded output equals the plain integer evaluation of
the same quantized network, and every layer boundary keeps  active = zero + value * R_p.
"""
import numpy as np
import pytest

import workloads
from oracle import net as onet
from oracle import plain


def check_network(net, batch=None, batch_base=0, rule=0):
    batch = net["batch"] if batch is None else batch
    r = onet.run(net, batch, batch_base, rule, keep=True)
    orc = r["orc"]
    P = orc.P
    n_in = net["n_in"]
    x = net["x"][batch_base * n_in:(batch_base + batch) * n_in]
    vals = plain.run_network(net["layers"], x, P, batch)
    # (1) decoded output == plain evaluation
    assert r["valid"].all()
    assert (r["values"] == plain.to_signed(vals[-1], P)).all()
    # (2) label invariant on every layer boundary, every residue, every component
    zeros, acts = r["gb"]["zero"], r["acts"]
    assert len(zeros) == len(vals) == len(acts)
    for b in range(len(vals)):
        for i, p in enumerate(orc.primes):
            d = orc.delta(p).astype(np.int64)
            want = (zeros[b][i].astype(np.int64) + (vals[b] % p)[:, None] * d[None, :]) % p
            assert (acts[b][i] == want).all(), (b, p)
    return r, vals


@pytest.mark.parametrize("k,repeat", [(2, 1), (3, 1), (3, 2), (4, 2), (5, 1)])
def test_tiny_dense_network(k, repeat):
    check_network(workloads.tiny(seed=10 + k, k=k, repeat=repeat, wmax=1 if k == 2 else 2))


def test_tiny_network_floor_rule_labels():
    check_network(workloads.tiny(seed=3, k=3, repeat=1), rule=1)


def test_tiny_sign_activation_network():
    check_network(workloads.tiny(seed=4, k=4, sign=True))


def test_tiny_cnn_padding_pooling_flatten():
    r, vals = check_network(workloads.tiny_cnn(seed=8, k=4, repeat=1))
    # both ReLU branches occur in this network
    P = r["orc"].P
    pre = plain.to_signed(vals[1], P)
    assert (pre < 0).any() and (pre > 0).any()


def test_batch_elements_are_independent_circuits():
    """garbling batch element 1 alone gives the same labels as garbling it inside the batch"""
    net = workloads.tiny(seed=21, k=3, batch=3, repeat=1)
    full = onet.run(net, keep=False)
    one = onet.run(net, batch=1, batch_base=1)
    n_out = len(one["values"])
    assert (full["values"][n_out:2 * n_out] == one["values"]).all()
    for i in range(3):
        assert (full["act_out"][i][n_out:2 * n_out] == one["act_out"][i]).all()
        assert (full["gb"]["d"][i][n_out:2 * n_out] == one["gb"]["d"][i]).all()


@pytest.mark.parametrize("centered", [False, True])
def test_mlp_config1(centered):
    """config 1 (784 -> 128 -> ReLU -> /2^6 -> 10, 8 primes, 128-bit labels), full size"""
    net = workloads.mlp(seed=1, centered=centered)
    r, vals = check_network(net)
    P = r["orc"].P
    pre = plain.to_signed(vals[1], P)
    assert np.abs(pre).max() < P // 2          # no wrap-around in this network
    if centered:
        assert (pre > 0).sum() > 10 and (pre < 0).sum() > 10
    sizes = r["gb"]["tables"]
    assert sizes[2].size == 128 * r["orc"].relu_bytes_per_elem()
    assert sizes[3].size == 128 * 6 * r["orc"].scale_bytes_per_elem()


def test_paper_model_c_shape():
    """Model C of the paper's table of architectures (strided convolution without padding, biases, 9 primes,
    no rescaling), random weights"""
    check_network(workloads.paper_model("C", seed=6))
