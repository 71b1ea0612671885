"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times.  Where the oracle cannot run the whole size in seconds it runs a sample from the seeds alone (one
batch element, runs of consecutive gates) and the rest is covered by properties that hold at any size:
decoded outputs equal the plain integer evaluation, and active = zero + value * R_p on every boundary
(Sec. Arithmetic Garbled Circuits, label invariant)."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import both
from oracle import capi, plain
from oracle import net as onet
from sampled import SampledOracle, segment_sizes, table_slices

pytestmark = pytest.mark.gpu


def check_invariant(ctx, zero, act, ring_values, what):
    """act == zero + (value mod p) * R_p, digit by digit, for every residue (device-side comparison of
    buffers; the values come from the plain evaluation)."""
    v = torch.as_tensor(np.asarray(ring_values, dtype=np.int64)).to(ctx.device)
    for i, p in enumerate(ctx.primes):
        if zero.tensors[i] is None:
            continue
        nch = zero.tensors[i].shape[0]
        R = np.zeros(nch * 16, np.int16)
        R[:ctx.lam(p)] = ctx.offset(p)
        Rt = torch.as_tensor(R).to(ctx.device).view(nch, 1, 16)
        n = zero.n_elem
        z = zero.tensors[i][:, :n, :].to(torch.int16)
        want = (z + (v % p).to(torch.int16).view(1, n, 1) * Rt) % p
        bad = (want != act.tensors[i][:, :n, :].to(torch.int16)).any(dim=2).any(dim=0)
        assert not bool(bad.any().item()), "%s residue %d: invariant broken at element %d" % (
            what, i, int(torch.nonzero(bad)[0].item()))


def test_config2_lenet_batch16_full():
    """Config 2 at full size.  Batch element 11 of 16 is recomputed by the oracle from the seeds: its
    labels on every boundary and its slice of every table segment must agree byte for byte.  All 16
    decoded outputs against the plain evaluation; the label invariant on every boundary."""
    from paper_2302_06361_amd import Context, GarbledNetwork
    net = workloads.lenet(seed=2, batch=16)
    b = 11
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = GarbledNetwork(ctx, net)
    g.garble()
    g.encode(torch.as_tensor(net["x"]).to(ctx.device))
    g.evaluate()
    values, valid = g.decode()
    torch.cuda.synchronize()
    P = int(np.prod(net["primes"]))
    pv = plain.run_network(net["layers"], net["x"], P, 16)
    assert valid.cpu().numpy().all()
    assert (values.cpu().numpy() == plain.to_signed(pv[-1], P)).all()
    for i in range(len(g.zero)):
        check_invariant(ctx, g.zero[i], g.act[i], pv[i], "boundary %d" % i)

    print("oracle: batch element %d" % b, flush=True)
    ref = onet.run(net, 1, b, 0, keep=True)
    orc = onet.make_oracle(net)
    for i in range(len(g.zero)):
        n = g.sizes[i] // 16
        for r in range(ctx.k):
            assert (g.zero[i].slice(b * n, (b + 1) * n).to_numpy(r) == ref["gb"]["zero"][i][r]).all(), ("zero", i, r)
            assert (g.act[i].slice(b * n, (b + 1) * n).to_numpy(r) == ref["acts"][i][r]).all(), ("act", i, r)
    for li, L in enumerate(net["layers"]):
        if L["id"] not in ref["gb"]["tables"]:
            continue
        want = ref["gb"]["tables"][L["id"]]
        n = L["n"]
        E = 16 * n
        before = 0
        for sz in segment_sizes(orc, L["kind"], L.get("repeat", 1)):
            got = g.tables[li][E * before + b * n * sz:E * before + (b + 1) * n * sz].cpu().numpy()
            assert (got == want[n * before:n * (before + sz)]).all(), "layer %d segment at %d" % (L["id"], before)
            before += sz
        assert n * before == want.size
    assert (values.cpu().numpy()[b * 10:(b + 1) * 10] == ref["values"]).all()


def test_config3_projection_microbenchmark_full():
    """Config 3 at full size: 2^24 gates, (p, q) uniform over the 12-prime base, grouped by pair.  Runs of
    consecutive gates in every sixth group are recomputed by the oracle (zero labels, table rows,
    evaluated labels); every gate must evaluate to out0 + phi(a) * R_q."""
    from paper_2302_06361_amd import ProjectionBatch
    mb = workloads.proj_microbench(seed=3)
    ctx, orc = both(12, seed=mb["seed"])
    pb = ProjectionBatch(ctx, mb["pi"], mb["qi"], layer_id=1)
    assert pb.n == 1 << 24 and len(pb.groups) == 144
    a_all = mb["a"][pb.order]
    keep = {}
    for gi, G in enumerate(pb.groups):
        p, q, n = ctx.primes[G["pi"]], ctx.primes[G["qi"]], G["count"]
        gen = workloads.rng(3, 1000 + gi)
        in0 = workloads.uniform_labels(gen, n, ctx.lam(p), p)
        phi = workloads.proj_phi(gen, n, p, q)
        a = a_all[G["start"]:G["start"] + n].astype(np.int64)
        act = ((in0.astype(np.int16) + a[:, None].astype(np.int16) * orc.delta(p).astype(np.int16)[None, :]) % p).astype(np.uint8)
        G["in0"].from_numpy(G["pi"], in0)
        G["act"].from_numpy(G["pi"], act)
        G["phi"].copy_(torch.as_tensor(phi))
        if gi % 6 == 0:
            off = int(gen.integers(0, n - 40))
            keep[gi] = (off, in0[off:off + 40].copy(), act[off:off + 40].copy(), phi[off:off + 40].copy())
        G["f"] = torch.as_tensor(phi[np.arange(n), a].astype(np.int16)).to(ctx.device)
    print("inputs uploaded", flush=True)
    pb.garble()
    pb.evaluate()
    torch.cuda.synchronize()
    for gi, G in enumerate(pb.groups):
        q, j, n = ctx.primes[G["qi"]], G["qi"], G["count"]
        nch = G["out"].tensors[j].shape[0]
        R = np.zeros(nch * 16, np.int16)
        R[:ctx.lam(q)] = orc.delta(q)
        Rt = torch.as_tensor(R).to(ctx.device).view(nch, 1, 16)
        want = (G["out0"].tensors[j].to(torch.int16) + G["f"].view(1, n, 1) * Rt) % q
        assert bool((want == G["out"].tensors[j].to(torch.int16)).all().item()), "group %d: out != out0 + phi(a) R_q" % gi
    for gi, (off, in0, act, phi) in keep.items():
        G = pb.groups[gi]
        p, q = ctx.primes[G["pi"]], ctx.primes[G["qi"]]
        rout0, rtable = orc.proj_garble(p, q, in0, phi, 1, 0, G["start"] + off)
        rout = orc.proj_eval(p, q, act, rtable, 1, 0, G["start"] + off)
        assert (G["out0"].slice(off, off + 40).to_numpy(G["qi"]) == rout0).all(), gi
        assert (G["out"].slice(off, off + 40).to_numpy(G["qi"]) == rout).all(), gi
        rb = p * ctx.pitch(q)
        assert (G["table"][off * rb:(off + 40) * rb].cpu().numpy() == rtable.reshape(-1)).all(), gi


def vgg_check(net, batch, exact, batch_base=0, sample=None, runs=2, count=6):
    """Gb, En, Ev, De layer by layer in the streamed mode (one table buffer, reused by every layer) over the batch
    elements batch_base .. batch_base + batch - 1.  Always: decoded outputs against the plain evaluation and the
    label invariant on every boundary.  exact: every byte against the oracle run over the same batch elements.
    sample = b: in every activation layer, `runs` runs of `count` consecutive values of batch element b are
    recomputed by the oracle from the seeds alone (tests/sampled.py); their zero and active labels on both sides of
    the layer and their rows of every table segment must agree byte for byte."""
    from paper_2302_06361_amd import Context, StreamedNetwork
    ctx = Context(net["primes"], net["seed"], net["digits"])
    g = StreamedNetwork(ctx, net, batch=batch, batch_base=batch_base)
    P = int(np.prod(net["primes"]))
    x = net["x"][batch_base * net["n_in"]:(batch_base + batch) * net["n_in"]]
    pv = plain.run_network(net["layers"], x, P, batch)
    ref = onet.run(net, batch, batch_base, 0, keep=True) if exact else None
    samples = {}
    if sample is not None:
        so = SampledOracle(net, sample)
        gen = np.random.default_rng(55)
        for li, L in enumerate(net["layers"]):
            if L["kind"] in ("relu", "scale", "sign"):
                n = so.n[li]
                c = min(count, n)
                starts = {0, n - c}
                while len(starts) < min(runs, n - c + 1):
                    starts.add(int(gen.integers(0, n - c + 1)))
                starts = sorted(starts)[:runs]
                samples[li] = [(st, c, so.activation(li, st, c)) for st in starts]
                print("oracle: layer %d (%s), values %s of batch element %d" % (L["id"], L["kind"], starts, sample), flush=True)
    compared = [0]

    def same(labels, first, cnt, want, what):
        for r in range(ctx.k):
            got = labels.slice(first, first + cnt).to_numpy(r)
            assert (got == want[r]).all(), (what, "residue", r)

    def boundary(i, zero, act):
        check_invariant(ctx, zero, act, pv[i], "boundary %d" % i)
        if exact:
            for r in range(ctx.k):
                assert (zero.to_numpy(r) == ref["gb"]["zero"][i][r]).all(), ("zero", i, r)
                assert (act.to_numpy(r) == ref["acts"][i][r]).all(), ("act", i, r)
            if i and net["layers"][i - 1]["id"] in ref["gb"]["tables"]:
                want = ref["gb"]["tables"][net["layers"][i - 1]["id"]]
                assert (g.table[:want.size].cpu().numpy() == want).all(), ("tables", i)
        n = g.sizes[i] // batch
        base = (sample - batch_base) * n if sample is not None else 0
        for st, c, r in samples.get(i, []):              # input side of layer i
            same(zero, base + st, c, r["zero_in"], "layer %d zero labels in" % i)
            same(act, base + st, c, r["act_in"], "layer %d active labels in" % i)
        for st, c, r in samples.get(i - 1, []):          # output side of layer i - 1, and its tables
            same(zero, base + st, c, r["zero_out"], "layer %d zero labels out" % (i - 1))
            same(act, base + st, c, r["act_out"], "layer %d active labels out" % (i - 1))
            for off_gpu, off_run, nbytes in table_slices(so.orc, net["layers"][i - 1], g.sizes[i], base + st, c):
                got = g.table[off_gpu:off_gpu + nbytes].cpu().numpy()
                assert (got == r["tables"][off_run:off_run + nbytes]).all(), ("layer %d tables" % (i - 1), off_gpu)
            compared[0] += 1
    values, valid = g.run(torch.as_tensor(x).to(ctx.device), boundary)
    torch.cuda.synchronize()
    assert valid.cpu().numpy().all()
    assert (values.cpu().numpy() == plain.to_signed(pv[-1], P)).all()
    assert compared[0] == sum(len(v) for v in samples.values())
    return g


def test_config5_vgg_shape_reduced_exact():
    """The VGG-shaped network of config 5 (12 primes, 3x3 convolutions with padding, three pooled blocks,
    scale 2^5) at reduced width and image size, every byte against the oracle, layer by layer in the
    streamed mode config 5 needs."""
    vgg_check(workloads.vgg(seed=5, batch=2, width=(3, 4, 5), hw=8), 2, exact=True)


def test_config5_vgg_full_width_sampled():
    """Config 5 at its real layer shapes: images 36 and 37 of the batch of 64 in one streamed call (the tables of one
    image's largest layer already take 30 GB, so the batch is streamed in chunks and layer by layer; element and
    wire indices of this call start at image 36, not at 0).  In each of the 14 activation layers three runs of values
    of image 37 (first, last and a random position) are recomputed by the oracle: labels on both sides and every
    table byte of those values.  All decoded outputs against the plain evaluation and the label invariant on every
    boundary."""
    g = vgg_check(workloads.vgg(seed=5, batch=64), 2, exact=False, batch_base=36, sample=37, runs=3)
    print("config 5: %.1f GB of tables per image" % (g.table_bytes / 2 / 1e9))


def test_config5_vgg_batch64_streamed():
    """Config 5 as stated: all 64 images, streamed in 32 chunks of 2 images through one set of buffers (garble, encode,
    evaluate, decode per chunk; element and wire indices of a chunk start at its first image).  Every decoded output of
    every image against the plain evaluation, all labels valid, and the label invariant on the output boundary of
    every chunk.  (Labels and table bytes of sampled values: test_config5_vgg_full_width_sampled.)"""
    from paper_2302_06361_amd import Context, StreamedNetwork
    net = workloads.vgg(seed=5, batch=64)
    ctx = Context(net["primes"], net["seed"], net["digits"])
    chunk = 2
    g = StreamedNetwork(ctx, net, batch=chunk)
    P = int(np.prod(net["primes"]))
    n_in, n_out = net["n_in"], 10
    pv = plain.run_network(net["layers"], net["x"], P, 64)[-1].reshape(64, n_out)
    last = len(net["layers"])
    for b in range(0, 64, chunk):
        g.batch_base = b
        g.rebase()
        x = torch.as_tensor(net["x"][b * n_in:(b + chunk) * n_in]).to(ctx.device)

        def boundary(i, zero, act, b=b):
            if i == last:
                check_invariant(ctx, zero, act, pv[b:b + chunk].reshape(-1), "images %d-%d, output boundary" % (b, b + chunk - 1))
        values, valid = g.run(x, boundary)
        torch.cuda.synchronize()
        assert valid.cpu().numpy().all(), b
        assert (values.cpu().numpy() == plain.to_signed(pv[b:b + chunk].reshape(-1), P)).all(), b
        if b % 16 == 0:
            print("images %d-%d ok" % (b, b + chunk - 1), flush=True)


@pytest.mark.parametrize("name", ["f", "F"])
def test_paper_cifar_model_shapes(name):
    """the CIFAR-sized models f and F of the paper's table (7-prime base, rescaling by 2^5 after every ReLU): one
    image; sampled values of every activation layer against the oracle (labels and table bytes), decoded outputs
    against the plain evaluation and the label invariant on every boundary"""
    vgg_check(workloads.paper_model(name, seed=6), 1, exact=False, sample=0, runs=3)


def test_config4_dense_full_size_sampled():
    """Config 4 at full size (dense 4096 x 4096, batch 128, 12 primes) in the launch configuration bench.py times (the
    256 x 256 tile of the MFMA kernel).  The labels are uploaded from the host generator; the oracle recomputes sampled
    outputs one by one: for a few batch elements, a few rows of every row block position, all digits of every prime."""
    from paper_2302_06361_amd import Context, Labels, Layer, DENSE
    mb = workloads.gemm_microbench(seed=4)
    M, K, B = mb["M"], mb["K"], mb["batch"]
    ctx, orc = both(12, seed=mb["seed"])
    wp = ctx.weights_prepare(mb["W"])
    x = Labels(ctx, B * K)
    host = []
    for i, p in enumerate(ctx.primes):
        lab = workloads.uniform_labels(mb["gen"], B * K, ctx.lam(p), p)
        host.append(lab)
        x.from_numpy(i, lab)
    y = Labels(ctx, B * M, zero=True)
    lay = Layer(DENSE, 1, B, in_c=K, out_c=M, weights=wp)
    print("inputs uploaded", flush=True)
    ctx.eval_layer(lay, x, None, y)
    torch.cuda.synchronize()
    g = np.random.default_rng(44)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, M - 1], g.integers(0, M, 26)]))     # tile edges and random rows
    for b in (0, 77, B - 1):
        for i, p in enumerate(ctx.primes):
            want = orc.dense(i, host[i][b * K:(b + 1) * K], 1, K, len(rows), mb["W"][rows])
            got = y.slice(b * M, (b + 1) * M).to_numpy(i)[rows]
            assert (got == want).all(), (b, p)
    for i in range(ctx.k):
        assert y.pad_is_zero(i)
