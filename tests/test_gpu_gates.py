"""GPU parity: batches of projection gates (garble and eval) through the C ABI against the oracle,
bit-exact on output zero labels, ciphertext tables and evaluated labels."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import both, upload_bundle, assert_tables_equal

pytestmark = pytest.mark.gpu


def run_proj(ctx, orc, pi, qi, n, seed, layer=9, elem_base=10 ** 9, shared_phi=False):
    from paper_2302_06361_amd import Labels, Layer, PROJ
    p, q = orc.primes[pi], orc.primes[qi]
    g = np.random.default_rng(seed)
    in0 = workloads.uniform_labels(g, n, orc.lam(p), p)
    phi = workloads.proj_phi(g, 1 if shared_phi else n, p, q)
    a = g.integers(0, p, n)
    act = ((in0.astype(np.int64) + a[:, None] * orc.delta(p).astype(np.int64)[None, :]) % p).astype(np.uint8)
    # GPU
    tin0, tact = Labels(ctx, n, only=[pi]), Labels(ctx, n, only=[pi])
    tin0.from_numpy(pi, in0)
    tact.from_numpy(pi, act)
    tout0, tout = Labels(ctx, n, only=[qi], zero=True), Labels(ctx, n, only=[qi], zero=True)
    phid = torch.as_tensor(phi).to(ctx.device)
    lay = Layer(PROJ, layer, n, elem_base=elem_base, p_index=pi, q_index=qi, phi=phid, phi_stride=0 if shared_phi else p)
    oe, tb, sb = ctx.layer_sizes(lay)
    assert oe == n and tb == n * p * ctx.pitch(q) and sb == 0
    tables = torch.zeros(tb, dtype=torch.uint8, device=ctx.device)
    ctx.garble_layer(lay, tin0, tout0, tables)
    ctx.eval_layer(lay, tact, tables, tout)
    torch.cuda.synchronize()
    # oracle
    rout0, rtable = orc.proj_garble(p, q, in0, phi[0] if shared_phi else phi, layer, 0, elem_base)
    rout = orc.proj_eval(p, q, act, rtable, layer, 0, elem_base)
    assert (tout0.to_numpy(qi) == rout0).all(), "output zero labels"
    assert tout0.pad_is_zero(qi)
    assert_tables_equal(tables, rtable.reshape(-1), "tables %d->%d" % (p, q))
    assert (tout.to_numpy(qi) == rout).all(), "evaluated labels"
    assert tout.pad_is_zero(qi)
    # and the result is the label of phi(a)
    f = (phi[0][a] if shared_phi else phi[np.arange(n), a]).astype(np.int64)
    want = (rout0.astype(np.int64) + f[:, None] * orc.delta(q).astype(np.int64)[None, :]) % q
    assert (rout == want).all()


@pytest.mark.parametrize("pi,qi", [(0, 0), (0, 11), (1, 1), (11, 0), (11, 11), (5, 7), (2, 3), (7, 4), (10, 9), (3, 1)])
def test_projection_gates_pairs(pi, qi):
    ctx, orc = both(12)
    run_proj(ctx, orc, pi, qi, 777, seed=pi * 12 + qi)      # three blocks and a ragged tail


@pytest.mark.parametrize("n", [1, 63, 64, 65, 256, 257, 2500])
def test_projection_gates_sizes(n):
    ctx, orc = both(12)
    run_proj(ctx, orc, 6, 2, n, seed=n)


def test_projection_gates_floor_rule_and_shared_table():
    ctx, orc = both(12, rule=1)
    run_proj(ctx, orc, 4, 8, 300, seed=1)
    run_proj(ctx, orc, 1, 5, 300, seed=2, shared_phi=True)


def test_projection_gates_explicit_label_lengths():
    ctx, orc = both(5, lam=(100, 20, 56, 7, 128))
    for pi, qi in [(0, 1), (1, 0), (2, 3), (3, 4), (4, 2), (4, 4), (0, 0)]:
        run_proj(ctx, orc, pi, qi, 300, seed=70 + pi * 6 + qi)


def test_context_refuses_bases_whose_product_overflows():
    from paper_2302_06361_amd import Context, DashError
    primes = [2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 41, 43, 47, 53]       # product 3.3e19 > 2^62
    with pytest.raises(DashError, match="size not supported"):
        Context(primes, bytes(16), digits=(2, 3))
    with pytest.raises(DashError, match="invalid argument"):
        Context([2, 3, 5], bytes(16), digits=(2, 5, 9), lam=(128, 0, 56))


def test_projection_gates_empty_batch():
    from paper_2302_06361_amd import Labels, Layer, PROJ
    ctx, orc = both(12)
    t = Labels(ctx, 0, only=[1, 2])
    phid = torch.zeros(3, dtype=torch.uint8, device=ctx.device)
    lay = Layer(PROJ, 1, 0, p_index=1, q_index=2, phi=phid, phi_stride=3)
    assert ctx.layer_sizes(lay) == (0, 0, 0)
    ctx.garble_layer(lay, t, t, None)
    ctx.eval_layer(lay, t, None, t)
    torch.cuda.synchronize()


def test_projection_all_144_pairs_small():
    ctx, orc = both(12)
    for pi in range(12):
        for qi in range(12):
            run_proj(ctx, orc, pi, qi, 70, seed=1000 + pi * 12 + qi, elem_base=2 ** 33 + 5)


def test_both_table_layouts_of_the_gate_kernels(monkeypatch):
    """the kernels with bank-replicated AES tables (taken for large launches) and with the shared tables, forced
    in turn for launches of every size"""
    for threshold in ("1", "1000000000000"):
        monkeypatch.setenv("DASH_BANKED_MIN_LANES", threshold)
        ctx, orc = both(12)
        for pi, qi in [(0, 0), (0, 11), (11, 0), (5, 7), (3, 1), (9, 9)]:
            run_proj(ctx, orc, pi, qi, 1500, seed=50 + pi * 12 + qi)
        run_proj(ctx, orc, 6, 2, 1, seed=3)


@pytest.mark.parametrize("threshold", ["1", "1000000000000"])
def test_projection_groups_in_one_call(monkeypatch, threshold):
    """dash_garble_layers / dash_eval_layers: independent PROJ calls of different sizes, element bases and layer ids in
    ONE call (groups with the same layer id and output modulus share kernel launches, each job with its own gate count),
    an empty group among them; both table layouts of the kernels forced in turn; every group against the oracle"""
    from paper_2302_06361_amd import Labels, Layer, PROJ
    monkeypatch.setenv("DASH_BANKED_MIN_LANES", threshold)
    ctx, orc = both(12)
    g = np.random.default_rng(99)
    spec = [(0, 3, 700, 5, 10), (4, 3, 1, 5, 2 ** 33), (11, 3, 257, 5, 999), (3, 3, 0, 5, 0), (2, 0, 300, 5, 4000), (7, 0, 513, 5, 70000),
            (1, 9, 64, 6, 123), (9, 9, 1500, 6, 2 ** 32 + 1), (5, 3, 300, 6, 5), (0, 0, 333, 5, 1), (10, 11, 100, 5, 0)]
    spec += [(int(g.integers(0, 12)), 7, int(g.integers(1, 400)), 5, int(g.integers(0, 10 ** 6))) for _ in range(20)]    # more than 16 jobs of one modulus
    layers, in0s, acts, out0s, outs, tables, host = [], [], [], [], [], [], []
    for pi, qi, n, lid, base in spec:
        p, q = orc.primes[pi], orc.primes[qi]
        in0 = workloads.uniform_labels(g, n, orc.lam(p), p)
        phi = workloads.proj_phi(g, max(n, 1), p, q)[:n]
        a = g.integers(0, p, n)
        act = ((in0.astype(np.int64) + a[:, None] * orc.delta(p).astype(np.int64)[None, :]) % p).astype(np.uint8)
        tin0, tact = Labels(ctx, n, only=[pi]), Labels(ctx, n, only=[pi])
        if n:
            tin0.from_numpy(pi, in0)
            tact.from_numpy(pi, act)
        phid = torch.as_tensor(phi.reshape(-1, p) if n else np.zeros((1, p), np.uint8)).to(ctx.device)
        lay = Layer(PROJ, lid, n, elem_base=base, p_index=pi, q_index=qi, phi=phid, phi_stride=p)
        oe, tb, sb = ctx.layer_sizes(lay)
        layers.append(lay); in0s.append(tin0); acts.append(tact)
        out0s.append(Labels(ctx, n, only=[qi], zero=True)); outs.append(Labels(ctx, n, only=[qi], zero=True))
        tables.append(torch.zeros(max(tb, 4), dtype=torch.uint8, device=ctx.device)[:tb])
        host.append((in0, phi, act))
    ctx.garble_layers(layers, in0s, out0s, tables)
    ctx.eval_layers(layers, acts, tables, outs)
    torch.cuda.synchronize()
    for i, (pi, qi, n, lid, base) in enumerate(spec):
        if n == 0:
            continue
        p, q = orc.primes[pi], orc.primes[qi]
        in0, phi, act = host[i]
        rout0, rtable = orc.proj_garble(p, q, in0, phi, lid, 0, base)
        rout = orc.proj_eval(p, q, act, rtable, lid, 0, base)
        assert (out0s[i].to_numpy(qi) == rout0).all(), ("zero labels", i)
        assert_tables_equal(tables[i], rtable.reshape(-1), "group %d" % i)
        assert (outs[i].to_numpy(qi) == rout).all(), ("evaluated labels", i)
        assert outs[i].pad_is_zero(qi) and out0s[i].pad_is_zero(qi)
