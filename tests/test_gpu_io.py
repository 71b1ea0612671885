"""GPU parity: context constants, input labels, En, De (through the C ABI, against the oracle)."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import both, upload_bundle, assert_bundle_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k,rule", [(3, 0), (5, 1), (8, 0), (12, 0), (12, 1)])
def test_context_constants(k, rule):
    ctx, orc = both(k, rule)
    assert ctx.digits == list(workloads.DIGITS[k])
    moduli = set(ctx.primes) | {2} | {orc.mj(j) for j in range(1, orc.n + 1)}
    for m in sorted(moduli):
        assert ctx.lam(m) == orc.lam(m)
        assert (ctx.offset(m) == orc.delta(m)).all(), m
    for i in range(k):
        assert (ctx.one(i, 0) == orc.one0(i)).all()
        assert (ctx.one(i, 1) == orc.one(i)).all()


@pytest.mark.parametrize("n", [0, 1, 255, 256, 1000])
def test_input_labels_encode_decode(n):
    from paper_2302_06361_amd import Labels
    ctx, orc = both(8)
    zero, act = Labels(ctx, n, zero=True), Labels(ctx, n, zero=True)
    ctx.input_labels(12345, zero)
    g = np.random.default_rng(n)
    x = g.integers(-2 ** 40, 2 ** 40, n)
    xd = torch.as_tensor(x).to(ctx.device)
    ctx.encode(xd, zero, act)
    values = torch.zeros(n, dtype=torch.int64, device=ctx.device)
    valid = torch.zeros(n, dtype=torch.uint8, device=ctx.device)
    ctx.decode(act, zero, values, valid)
    torch.cuda.synchronize()
    if n == 0:
        return
    ref0 = [orc.input_labels(12345, n, i) for i in range(8)]
    ref1 = [orc.encode(i, x, ref0[i]) for i in range(8)]
    assert_bundle_equal(zero, ref0, "input zero labels")
    assert_bundle_equal(act, ref1, "encoded labels")
    rv, rok = orc.decode(ref1, ref0)
    assert (values.cpu().numpy() == rv).all() and (valid.cpu().numpy() == rok).all() and rok.all()


def test_input_labels_count_argument():
    """dash_input_labels draws the first n labels of the tensor and leaves the rest alone; n beyond the tensor is refused"""
    from paper_2302_06361_amd import Labels
    from paper_2302_06361_amd.binding import DashError
    ctx, orc = both(5)
    zero = Labels(ctx, 300, zero=True)
    ctx.input_labels(77, zero, n=130)
    torch.cuda.synchronize()
    for i in range(5):
        got = zero.to_numpy(i)
        assert (got[:130] == orc.input_labels(77, 130, i)).all()
        assert (got[130:] == 0).all()
    with pytest.raises(DashError):
        ctx.input_labels(0, zero, n=301)
    with pytest.raises(DashError):
        ctx.input_labels(0, zero, n=-1)


def test_decode_flags_forged_labels():
    ctx, orc = both(5)
    n = 300
    g = np.random.default_rng(1)
    x = g.integers(0, orc.P, n)
    ref0 = [orc.input_labels(0, n, i) for i in range(5)]
    ref1 = [orc.encode(i, x, ref0[i]) for i in range(5)]
    forged = [a.copy() for a in ref1]
    for e, i, j in [(3, 0, 127), (77, 2, 0), (299, 4, 10), (150, 1, 80)]:
        p = orc.primes[i]
        forged[i][e, j] = (forged[i][e, j] + 1) % p
    zero, act = upload_bundle(ctx, ref0), upload_bundle(ctx, forged)
    values = torch.zeros(n, dtype=torch.int64, device=ctx.device)
    valid = torch.zeros(n, dtype=torch.uint8, device=ctx.device)
    ctx.decode(act, zero, values, valid)
    rv, rok = orc.decode(forged, ref0)
    assert (valid.cpu().numpy() == rok).all() and rok.sum() == n - 4
    assert (values.cpu().numpy() == rv).all()


def test_bad_arguments_are_refused():
    from paper_2302_06361_amd import Labels, DashError, Context
    ctx, _ = both(3)
    zero = Labels(ctx, 10)
    small = Labels(ctx, 4)
    x = torch.zeros(10, dtype=torch.int64, device=ctx.device)
    with pytest.raises(DashError):
        ctx.encode(x, zero, small)          # output tensor too small
    with pytest.raises(DashError):
        Context([2, 4, 5], bytes(16))       # 4 is not prime
    with pytest.raises(DashError):
        Context([2, 3, 5], bytes(16), digits=[3, 5, 9])    # d_1 must be even


@pytest.mark.parametrize("k,n", [(8, 0), (8, 1), (8, 700), (12, 300)])
def test_labels_pack_unpack_wire_format(k, n):
    """the 128-bit wire format (Sec. Evaluation, online communication; compress of Sec. Implementation) under the
    floor rule: pack == the oracle's compress label by label, unpack == its decompress, on uniform labels that
    include the largest one (all digits p - 1) and on bytes the GPU never produced"""
    from paper_2302_06361_amd import Labels
    from oracle import capi
    ctx, orc = both(k, rule=1)
    g = np.random.default_rng(100 + n)
    lab = [workloads.uniform_labels(g, n, orc.lam(p), p) for p in orc.primes]
    if n > 1:
        for i, p in enumerate(orc.primes):
            lab[i][0, :] = p - 1
            lab[i][1, :] = 0
    t = upload_bundle(ctx, lab) if n else Labels(ctx, 0)
    packed = torch.full((k, n, 16), 0xEE, dtype=torch.uint8, device=ctx.device)
    ctx.labels_pack(t, packed)
    back = Labels(ctx, n)
    for i in range(k):
        if n:
            back.tensors[i].fill_(0xEE)
    ctx.labels_unpack(packed, back)
    torch.cuda.synchronize()
    if n == 0:
        return
    got = packed.cpu().numpy()
    foreign = np.zeros((k, n, 16), np.uint8)
    for i, p in enumerate(orc.primes):
        for e in range(n):
            want = np.frombuffer(capi.compress(lab[i][e], p).to_bytes(16, "little"), np.uint8)
            assert (got[i, e] == want).all(), (i, e)
            # bytes the GPU did not write: the oracle's packing of another label
            foreign[i, e] = np.frombuffer(capi.compress(lab[i][n - 1 - e], p).to_bytes(16, "little"), np.uint8)
    assert_bundle_equal(back, lab, "unpack(pack(labels))")
    ctx.labels_unpack(torch.as_tensor(foreign).to(ctx.device), back)
    torch.cuda.synchronize()
    for i, p in enumerate(orc.primes):
        for e in (0, n // 2, n - 1):
            h = int.from_bytes(foreign[i, e].tobytes(), "little")
            assert (back.to_numpy(i)[e] == capi.decompress(h, p, orc.lam(p))).all(), (i, e)
    assert_bundle_equal(back, [a[::-1] for a in lab], "unpack of the oracle's bytes")


def test_labels_pack_needs_the_floor_rule():
    """with the ceil rule a label can exceed 128 bits: both calls refuse and leave the buffers alone"""
    from paper_2302_06361_amd import Labels
    from paper_2302_06361_amd.binding import DashError
    ctx, _ = both(8, rule=0)
    t = Labels(ctx, 4, zero=True)
    packed = torch.full((8, 4, 16), 7, dtype=torch.uint8, device=ctx.device)
    with pytest.raises(DashError):
        ctx.labels_pack(t, packed)
    with pytest.raises(DashError):
        ctx.labels_unpack(packed, t)
    torch.cuda.synchronize()
    assert bool((packed == 7).all().item())


@pytest.mark.parametrize("k,kind,repeat", [(8, "relu", 1), (8, "scale", 2), (5, "sign", 1), (12, "relu", 1)])
def test_tables_pack_unpack(k, kind, repeat):
    """the packed storage format of a layer's ciphertext tables (16 bytes per row, the row compressed like a label;
    floor-rule contexts): packed bytes against the oracle's packing of the oracle's tables, unpacking gives the
    tables back, and the layer evaluates from the unpacked copy"""
    from paper_2302_06361_amd import Labels, Layer, RELU, SCALE, SIGN
    ctx, orc = both(k, rule=1)
    P = orc.P
    n = 333
    X = np.random.default_rng(k).integers(0, P, n)
    zero = [orc.input_labels(9, n, i) for i in range(k)]
    act = [orc.encode(i, X, zero[i]) for i in range(k)]
    lay = Layer(dict(relu=RELU, scale=SCALE, sign=SIGN)[kind], 3, n, elem_base=50, repeat=repeat)
    if kind == "relu":
        r0, rt = orc.relu_garble(3, zero, 50)
        r = orc.relu_eval(3, act, rt, 50)
    elif kind == "scale":
        r0, rt = orc.scale_garble(3, zero, repeat, 50)
        r = orc.scale_eval(3, act, rt, repeat, 50)
    else:
        r0, rt = orc.signact_garble(3, zero, 50)
        r = orc.signact_eval(3, act, rt, 50)
    want_packed = orc.tables_pack(kind, n, rt, repeat)
    oe, tb, sb = ctx.layer_sizes(lay)
    pb = ctx.tables_packed_bytes(lay)
    assert tb == rt.size and pb == want_packed.size and pb < tb
    tz, ta = upload_bundle(ctx, zero), upload_bundle(ctx, act)
    oz, oa = Labels(ctx, n, zero=True), Labels(ctx, n, zero=True)
    tables = torch.zeros(tb, dtype=torch.uint8, device=ctx.device)
    scratch = torch.zeros(sb + 256, dtype=torch.uint8, device=ctx.device)
    ctx.garble_layer(lay, tz, oz, tables, scratch)
    packed = torch.full((pb,), 0xEE, dtype=torch.uint8, device=ctx.device)
    ctx.tables_pack(lay, tables, packed)
    back = torch.full((tb,), 0xEE, dtype=torch.uint8, device=ctx.device)
    ctx.tables_unpack(lay, packed, back)
    ctx.eval_layer(lay, ta, back, oa, scratch)
    torch.cuda.synchronize()
    assert (packed.cpu().numpy() == want_packed).all(), "packed bytes"
    assert (back.cpu().numpy() == rt).all(), "unpacked tables"
    assert_bundle_equal(oa, r, "evaluated from the unpacked tables")
    print("%s, %d primes: %.1f KB per value unpacked, %.1f KB packed" % (kind, k, tb / n / 1e3, pb / n / 1e3))


def test_tables_pack_needs_rows_below_128_bits():
    from paper_2302_06361_amd import Layer, RELU, DashError
    ctx, orc = both(8)                       # ceil rule: 3^81 > 2^128
    lay = Layer(RELU, 3, 10)
    assert ctx.tables_packed_bytes(lay) == 0
    t = torch.zeros(1 << 20, dtype=torch.uint8, device=ctx.device)
    with pytest.raises(DashError, match="not implemented"):
        ctx.tables_pack(lay, t, t)
    torch.cuda.synchronize()


@pytest.mark.gpu
@pytest.mark.parametrize("variant", [0, 1, 2, 3])
def test_aes_forms_against_the_standard_and_the_oracle(variant):
    """Every form of AES-128 the library holds (4 KB tables, bank-replicated tables, bit planes) on the GPU: FIPS-197
    Appendix B and C.1 vectors, random blocks against the oracle's AES, repeated application, the size rule of the
    bit-plane form."""
    import torch
    from oracle import capi
    from paper_2302_06361_amd import binding
    ctx = binding.Context(workloads.PRIMES[:3], bytes(range(16)), workloads.DIGITS[3])
    n = 4096 + (0 if variant == 2 else 77)
    g = np.random.default_rng(11 + variant)
    blocks = g.integers(0, 256, (n, 16), dtype=np.uint8)
    blocks[5] = np.frombuffer(bytes.fromhex("00112233445566778899aabbccddeeff"), np.uint8)
    blocks[2049] = np.frombuffer(bytes.fromhex("3243f6a8885a308d313198a2e0370734"), np.uint8)
    d_in = torch.from_numpy(blocks).cuda()
    d_out = torch.empty_like(d_in)
    ctx.profile_aes(variant, bytes(range(16)), d_in, d_out)
    out = d_out.cpu().numpy()
    assert out[5].tobytes().hex() == "69c4e0d86a7b0430d8cdb78070b4c55a"
    key_b = bytes.fromhex("2b7e151628aed2a6abf7158809cf4f3c")
    ctx.profile_aes(variant, key_b, d_in, d_out)
    out_b = d_out.cpu().numpy()
    assert out_b[2049].tobytes().hex() == "3925841d02dc09fbdc118597196a0b32"
    key_np = np.frombuffer(key_b, np.uint8)
    for j in list(range(0, n, 97)) + [n - 1]:
        assert (out_b[j] == capi.aes128_encrypt(key_np, blocks[j])).all(), j
    # three applications in one call
    ctx.profile_aes(variant, key_b, d_in, d_out, repeat=3)
    out3 = d_out.cpu().numpy()
    for j in (0, 63, 64, 2047, 2048, n - 1):
        v = blocks[j]
        for _ in range(3):
            v = capi.aes128_encrypt(key_np, v)
        assert (out3[j] == v).all(), j
    if variant == 2:
        with pytest.raises(binding.DashError):
            ctx.profile_aes(2, key_b, d_in[:100], d_out[:100])
