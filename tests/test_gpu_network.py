"""GPU parity: whole networks (Gb, En, Ev, De) through the C ABI against the oracle: zero and active
labels on every layer boundary, every table byte, decoded values; decoded values against the plain
integer evaluation as well."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import assert_bundle_equal, assert_tables_equal
from oracle import net as onet
from oracle import plain

pytestmark = pytest.mark.gpu


def run_net(net, rule=0, batch=None, batch_base=0):
    from paper_2302_06361_amd import Context, GarbledNetwork
    batch = net["batch"] if batch is None else batch
    ref = onet.run(net, batch, batch_base, rule, keep=True)
    ctx = Context(net["primes"], net["seed"], net["digits"], rule)
    g = GarbledNetwork(ctx, net, batch, batch_base)
    n_in = net["n_in"]
    x = net["x"][batch_base * n_in:(batch_base + batch) * n_in]
    g.garble()
    g.encode(torch.as_tensor(x).to(ctx.device))
    g.evaluate()
    values, valid = g.decode()
    torch.cuda.synchronize()
    for b in range(len(g.zero)):
        assert_bundle_equal(g.zero[b], ref["gb"]["zero"][b], "zero labels, boundary %d" % b)
        assert_bundle_equal(g.act[b], ref["acts"][b], "active labels, boundary %d" % b)
    for li, L in enumerate(net["layers"]):
        if L["id"] in ref["gb"]["tables"]:
            assert_tables_equal(g.tables[li], ref["gb"]["tables"][L["id"]], "tables of layer %d" % L["id"])
    assert valid.cpu().numpy().all()
    assert (values.cpu().numpy() == ref["values"]).all()
    want = plain.to_signed(plain.run_network(net["layers"], x, ctx_P(net), batch)[-1], ctx_P(net))
    assert (values.cpu().numpy() == want).all()


def ctx_P(net):
    return int(np.prod(net["primes"]))


@pytest.mark.parametrize("k,repeat", [(2, 1), (3, 2), (4, 2), (5, 1)])
def test_tiny_dense(k, repeat):
    run_net(workloads.tiny(seed=10 + k, k=k, repeat=repeat, wmax=1 if k == 2 else 2))


def test_tiny_floor_rule():
    run_net(workloads.tiny(seed=3, k=3, repeat=1), rule=1)


def test_tiny_sign_activation():
    run_net(workloads.tiny(seed=4, k=4, sign=True))


def test_tiny_cnn():
    run_net(workloads.tiny_cnn(seed=8, k=4, repeat=1))


def test_batch_chunk_matches_full_batch_labels():
    """a layer call over a sub-range of the batch (elem_base) reproduces the same wires"""
    run_net(workloads.tiny(seed=21, k=3, batch=3, repeat=1), batch=1, batch_base=2)


@pytest.mark.parametrize("centered", [False, True])
def test_mlp_config1(centered):
    run_net(workloads.mlp(seed=1, centered=centered))


@pytest.mark.parametrize("name", ["A", "B", "C", "D"])
def test_paper_model_shapes(name):
    """the MNIST-sized models of the paper's table of architectures (strided convolutions, biases, 8- and 9-prime
    bases, no rescaling) with random weights: every label, table byte and output against the oracle"""
    run_net(workloads.paper_model(name, seed=6))


def test_layer_calls_can_be_captured_in_a_graph():
    """garble and evaluate only enqueue kernels on the caller's stream: captured in HIP graphs and replayed
    several times, with eager work and synchronisations in between, every replay reproduces the eager tables
    and outputs"""
    from paper_2302_06361_amd import Context, GarbledNetwork
    net = workloads.paper_model("C", seed=6)
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = GarbledNetwork(ctx, net)
    x = torch.as_tensor(net["x"]).to(ctx.device)
    g.garble(); g.encode(x); g.evaluate(); g.decode()
    torch.cuda.synchronize()
    ref_values = g.values.clone()
    ref_tables = [None if t is None else t.clone() for t in g.tables]
    ref_act = [t.clone() for t in g.act[-1].tensors]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on a side stream, as capture requires
        g.garble(); g.evaluate(); g.decode()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    gg, ge = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(gg):
        g.garble()
    with torch.cuda.graph(ge):
        g.evaluate(); g.decode()
    for rep in range(3):
        for t in g.tables:
            if t is not None:
                t.fill_(rep)
        g.values.zero_()
        for t in g.act[-1].tensors:
            t.fill_(0xEE)
        torch.cuda.synchronize()
        gg.replay()
        g.encode(x)                        # eager work between the replays
        torch.cuda.synchronize()
        ge.replay()
        torch.cuda.synchronize()
        for t, r in zip(g.tables, ref_tables):
            assert t is None or bool((t == r).all().item()), rep
        assert bool((g.values == ref_values).all().item()) and bool(g.valid.all().item()), rep
        for t, r in zip(g.act[-1].tensors, ref_act):
            assert bool((t == r).all().item()), rep
