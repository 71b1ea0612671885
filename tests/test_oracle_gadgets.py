"""Pins for the oracle's gates and gadgets: brute force over every input for small moduli,
the comparison [X >= P/2] for every X of small CRT bases, the paper's scaling table for Z_6
and ceil(x/2) for every x of small bases.
"""
import os

import numpy as np
import pytest

import workloads
from oracle import capi, plain

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SEED = bytes(range(32, 48))


def orc_for(k, rule=0):
    return capi.Oracle(workloads.PRIMES[:k], workloads.DIGITS[k], SEED, rule)


def lab(zero, v, delta, m):
    return ((zero.astype(np.int64) + int(v) * delta.astype(np.int64)) % m).astype(np.uint8)


# ---------------------------------------------------------------- projection gate
@pytest.mark.parametrize("p,q", [(2, 2), (2, 37), (3, 5), (5, 3), (7, 60), (13, 2), (37, 37), (60, 4), (96, 26), (125, 60)])
@pytest.mark.parametrize("rule", [0, 1])
def test_projection_gate_every_input(p, q, rule):
    orc = orc_for(5, rule)
    g = np.random.default_rng(p * 1000 + q)
    n = 6
    in0 = workloads.uniform_labels(g, n, orc.lam(p), p)
    phi = workloads.proj_phi(g, n, p, q)
    out0, table = orc.proj_garble(p, q, in0, phi, layer=3, slot=9, elem_base=50)
    dp, dq = orc.delta(p), orc.delta(q)
    assert table.shape == (n, p, capi.pitch(orc.lam(q)))
    assert (table[:, :, orc.lam(q):] == 0).all() and table.max() < q
    for a in range(p):
        act = np.stack([lab(in0[e], a, dp, p) for e in range(n)])
        out = orc.proj_eval(p, q, act, table, layer=3, slot=9, elem_base=50)
        for e in range(n):
            assert (out[e] == lab(out0[e], phi[e, a], dq, q)).all(), (a, e)
    # a different tweak must not decrypt (the hash really depends on layer / slot / element)
    act = np.stack([lab(in0[e], 1, dp, p) for e in range(n)])
    for kw in (dict(layer=4, slot=9, elem_base=50), dict(layer=3, slot=8, elem_base=50), dict(layer=3, slot=9, elem_base=51)):
        bad = orc.proj_eval(p, q, act, table, **kw)
        assert not (bad == np.stack([lab(out0[e], phi[e, 1], dq, q) for e in range(n)])).all()


def test_projection_rows_are_sorted_by_colour():
    """Row c of a table belongs to the input value whose label has colour c (point-and-permute)."""
    orc = orc_for(3)
    p, q = 5, 3
    g = np.random.default_rng(1)
    in0 = workloads.uniform_labels(g, 1, orc.lam(p), p)
    phi = np.array([[0, 1, 2, 1, 0]], np.uint8)
    out0, table = orc.proj_garble(p, q, in0, phi, layer=1)
    for a in range(p):
        la = lab(in0[0], a, orc.delta(p), p)
        h = orc.hash(la, p, 1, 0, 0, q)
        want = (lab(out0[0], phi[0, a], orc.delta(q), q).astype(int) + h) % q
        assert (table[0, la[0], :orc.lam(q)] == want).all()


# ---------------------------------------------------------------- half gate
@pytest.mark.parametrize("p", [2, 3, 5, 7, 11, 37])
def test_half_gate_every_input(p):
    orc = orc_for(5)
    g = np.random.default_rng(p)
    for trial in range(3):
        x0 = workloads.uniform_labels(g, 1, orc.lam(p), p)[0]
        y0 = workloads.uniform_labels(g, 1, orc.lam(2), 2)[0]
        z0, G, E, S = orc.hg_garble(p, x0, y0, layer=2, slotG=40, elem=trial)
        for a in range(p):
            for b in range(2):
                z = orc.hg_eval(p, lab(x0, a, orc.delta(p), p), lab(y0, b, orc.delta(2), 2), 2, 40, trial, G, E, S)
                assert (z == lab(z0, a * b, orc.delta(p), p)).all(), (a, b)


# ---------------------------------------------------------------- sign
def residues(X, primes):
    return [X % p for p in primes]


@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_sign_plain_function_is_exact_for_every_value(k):
    orc = orc_for(k)
    P = orc.P
    assert orc.M >= k * P and orc.digits[0] % 2 == 0
    for X in range(P):
        r = residues(X, orc.primes)
        assert orc.sign_plain(r, 0, 0) == int(2 * X >= P), X
        assert orc.sign_plain(r, 0, 1) == int(2 * X < P), X
        if X % 2 == 0:      # base-extension use: residue 0 is known to be 0 and its gates are left out
            assert orc.sign_plain(r, 1, 0) == int(2 * X >= P), X


@pytest.mark.parametrize("k", [8, 12])
def test_sign_plain_function_boundaries_and_random(k):
    orc = orc_for(k)
    P = orc.P
    assert orc.M >= k * P
    g = np.random.default_rng(k)
    xs = [0, 1, P // 2 - 1, P // 2, P // 2 + 1, P - 1] + [int(v) for v in g.integers(0, P, 300)]
    xs += [P // 2 - 1 - int(v) for v in g.integers(0, 50, 20)] + [P // 2 + int(v) for v in g.integers(0, 50, 20)]
    for X in xs:
        assert orc.sign_plain(residues(X, orc.primes), 0, 0) == int(2 * X >= P), X
    for X in xs:
        X -= X % 2
        assert orc.sign_plain(residues(X, orc.primes), 1, 0) == int(2 * X >= P), X


def test_sign_digit_tables_sum_to_rounded_fraction():
    """sum_j phi_ij(x) * weight_j == ceil(M * (x * (P/p_i)^-1 mod p_i) / p_i)  (big integers)."""
    orc = orc_for(8)
    P, M, n = orc.P, orc.M, orc.n
    w = [1] * (n + 2)
    for j in range(n, 0, -1):
        w[j] = w[j + 1] * orc.digits[j] if j < n else 1
    for i, p in enumerate(orc.primes):
        inv = pow(P // p, -1, p)
        for x in range(p):
            u = (x * inv) % p
            want = -((-M * u) // p)
            got = sum(orc.sign_phi(i, j, x) * w[j] for j in range(1, n + 1))
            assert got == want


def bundle_for(orc, values, first_wire=0):
    """zero labels from the PRG and active labels for the given ring values"""
    n = len(values)
    zero = [orc.input_labels(first_wire, n, i) for i in range(orc.k)]
    act = [orc.encode(i, np.asarray(values), zero[i]) for i in range(orc.k)]
    return zero, act


@pytest.mark.parametrize("k", [2, 3, 4])
def test_relu_layer_every_value(k):
    orc = orc_for(k)
    P = orc.P
    X = np.arange(P)
    zero, act = bundle_for(orc, X)
    out0, tables = orc.relu_garble(5, zero)
    assert tables.size == P * orc.relu_bytes_per_elem()
    out = orc.relu_eval(5, act, tables)
    vals, valid = orc.decode(out, out0)
    assert valid.all()
    assert (vals == plain.to_signed(plain.relu(X, P), P)).all()


@pytest.mark.parametrize("k", [2, 3, 4])
def test_sign_activation_every_value(k):
    orc = orc_for(k)
    P = orc.P
    X = np.arange(P)
    zero, act = bundle_for(orc, X)
    out0, tables = orc.signact_garble(6, zero)
    out = orc.signact_eval(6, act, tables)
    vals, valid = orc.decode(out, out0)
    assert valid.all()
    assert (vals == np.where(2 * X >= P, -1, 1)).all()


def test_relu_internal_wires_keep_the_label_invariant():
    """every gate output inside the sign gadget is zero + value * R_m with the value the plain
    mixed-radix addition predicts"""
    orc = orc_for(4)
    P, k, n = orc.P, orc.k, orc.n
    X = np.array([0, 1, 57, 104, 105, 106, 209])
    zero, act = bundle_for(orc, X)
    out0, tables, w0 = orc.relu_garble(5, zero, want_wires=True)
    out, w = orc.relu_eval(5, act, tables, want_wires=True)
    for e, x in enumerate(X):
        a = {(i, j): orc.sign_phi(i, j, int(x) % orc.primes[i]) for i in range(k) for j in range(1, n + 1)}
        val = {}
        carry = 0
        for i in range(k):
            for j in range(1, n + 1):
                val[i * n + j - 1] = (a[i, j], orc.mj(j))
        for j in range(n, 1, -1):
            s = sum(a[i, j] for i in range(k)) + carry
            assert s < orc.mj(j)
            carry = s // orc.digits[j - 1]
            val[k * n + j - 2] = (carry % orc.mj(j - 1), orc.mj(j - 1))
        s1 = (sum(a[i, 1] for i in range(k)) + carry) % orc.digits[0]
        val[k * n + n - 1] = (int(2 * s1 < orc.digits[0]), 2)
        for s, (v, m) in val.items():
            lam = orc.lam(m)
            assert (w[e, s, :lam] == lab(w0[e, s, :lam], v, orc.delta(m), m)).all(), (x, s)


# ---------------------------------------------------------------- scaling
def _table_rows():
    rows = []
    for line in open(os.path.join(GOLD, "scaling_table_Z6.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            t = line.split()
            pair = lambda s: tuple(int(v) for v in s.split(","))
            rows.append(dict(x=int(t[0]), xs=int(t[1]), phix=pair(t[2]), up=int(t[3]), ups=int(t[4]), phiup=pair(t[5]),
                             alpha=pair(t[6]), crt=int(t[7]), crts=int(t[8]), y=int(t[9]), phiy=pair(t[10]),
                             phiyd=pair(t[11]), yd=int(t[12]), yds=int(t[13])))
    return rows


def test_scaling_table_of_the_paper_plain_steps():
    """the plain definition reproduces every column of the paper's table for Z_6"""
    rows = _table_rows()
    assert len(rows) == 6
    P = 6
    crt = {(X % 2, X % 3): X for X in range(6)}
    for r in rows:
        x = r["x"]
        assert plain.to_signed(x, P) == r["xs"] and (x % 2, x % 3) == r["phix"]
        up = (x + P // 2) % P
        assert up == r["up"] and plain.to_signed(up, P) == r["ups"] and (up % 2, up % 3) == r["phiup"]
        b = ((up % 3 - up % 2) * 2) % 3          # (x_i - x_0) * 2^-1 mod 3, 2^-1 = 2
        assert (0, b) == r["alpha"]
        assert crt[(0, b)] == r["crt"] and plain.to_signed(crt[(0, b)], P) == r["crts"]
        y = up // 2
        assert y == r["y"] and (y % 2, y % 3) == r["phiy"]
        yd = int(plain.scale2(x, P))
        assert yd == r["yd"] and (yd % 2, yd % 3) == r["phiyd"] and plain.to_signed(yd, P) == r["yds"]
        # the base extension recovers the mod-2 residue of y as [crt(alpha) >= P/2]
        assert int(2 * crt[(0, b)] >= P) == y % 2


def test_scaling_table_of_the_paper_garbled():
    rows = _table_rows()
    orc = orc_for(2)
    X = np.array([r["x"] for r in rows])
    zero, act = bundle_for(orc, X)
    out0, tables = orc.scale_garble(4, zero, 1)
    out = orc.scale_eval(4, act, tables, 1)
    vals, valid = orc.decode(out, out0)
    assert valid.all()
    assert vals.tolist() == [r["yds"] for r in rows]
    # residues of the active output labels are the table's phi(y_down) column
    for i, p in enumerate(orc.primes):
        got = (out[i][:, 0].astype(int) - out0[i][:, 0]) % p
        assert got.tolist() == [r["phiyd"][i] for r in rows]


@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_plain_scale_is_ceil_half_of_signed_value(k):
    P = int(np.prod(workloads.PRIMES[:k]))
    X = np.arange(P)
    s = plain.to_signed(X, P)
    assert (plain.to_signed(plain.scale2(X, P), P) == -((-s) // 2)).all()


@pytest.mark.parametrize("k,repeat", [(2, 1), (3, 1), (3, 2), (4, 1), (4, 3)])
def test_scale_layer_every_value(k, repeat):
    orc = orc_for(k)
    P = orc.P
    X = np.arange(P)
    zero, act = bundle_for(orc, X)
    out0, tables = orc.scale_garble(9, zero, repeat)
    assert tables.size == P * repeat * orc.scale_bytes_per_elem()
    out = orc.scale_eval(9, act, tables, repeat)
    vals, valid = orc.decode(out, out0)
    assert valid.all()
    want = plain.to_signed(plain.scale(X, P, repeat), P)
    assert (vals == want).all()
    s = plain.to_signed(X, P)
    assert (want == -((-s) // (2 ** repeat))).all()        # ceil(s / 2^repeat)


def test_scale_and_relu_random_values_base8():
    orc = orc_for(8)
    P = orc.P
    g = np.random.default_rng(3)
    X = np.concatenate([[0, 1, P // 2 - 1, P // 2, P - 1], g.integers(0, P, 12)])
    zero, act = bundle_for(orc, X, first_wire=77)
    r0, rt = orc.relu_garble(2, zero, elem_base=1000)
    r = orc.relu_eval(2, act, rt, elem_base=1000)
    s0, st = orc.scale_garble(3, r0, 6, elem_base=1000)
    s = orc.scale_eval(3, r, st, 6, elem_base=1000)
    vals, valid = orc.decode(s, s0)
    assert valid.all()
    assert (vals == plain.to_signed(plain.scale(plain.relu(X, P), P, 6), P)).all()


# ---------------------------------------------------------------- table sizes
def test_ciphertext_counts_base8_and_base12():
    """Ciphertexts per value, counted as the hashes the garbler spends (one per ciphertext), against the numbers
    worked out by hand.  With the digit and cast gates of the mixed-radix addition merged into one projection per
    (residue, digit), a sign gadget with digits (d_1; d_2..d_n) over k primes has
        n * sum(p) digit rows + k * (d_2 + .. + d_n) carry rows + d_1 final rows:
        base 8, (26; 12 x 6): 7 * 77 + 8 * 72 + 26 = 1141;  base 12, (46; 17 x 10): 11 * 197 + 12 * 170 + 46 = 4253.
    The paper's count for the same digits (Sec. The Scaling Operation, Garbling: alpha = t sum(p) + 2k sum_{i>=2} m_i +
    2n(k-1) + m_1, with separate cast gates) is 539 + 1152 + 98 + 26 = 1815 and 2167 + 4080 + 242 + 46 = 6535.
    ReLU adds sum(p) + 2k rows and 2k one-digit rows (half gates); one scaling step is the sign gadget without
    residue 0 (n * 2 rows fewer) plus 2(k-1) cast rows, as in the paper's alpha + 2(k-1)."""
    for k, sign, relu, scale_step, paper_alpha in ((8, 1141, 1141 + 77 + 16 + 16, 1141 - 7 * 2 + 14, 1815),
                                                   (12, 4253, 4253 + 197 + 24 + 24, 4253 - 11 * 2 + 22, 6535)):
        orc = orc_for(k)
        zero = [orc.input_labels(0, 1, i) for i in range(k)]
        h0 = capi.hash_calls()
        orc.signact_garble(3, zero)
        h1 = capi.hash_calls()
        orc.relu_garble(4, zero)
        h2 = capi.hash_calls()
        orc.scale_garble(5, zero, 3)
        h3 = capi.hash_calls()
        assert h1 - h0 == sign + 2 * k              # the sign activation: the gadget and k two-row gates
        assert h2 - h1 == relu
        assert h3 - h2 == 3 * scale_step
        assert sign < paper_alpha
        n, d = orc.n, orc.digits
        assert paper_alpha == n * sum(orc.primes) + 2 * k * sum(d[1:]) + 2 * n * (k - 1) + d[0]
    # and the evaluator spends one hash per gate: 63 gates per base-8 sign gadget, 143 per base-12 one
    for k, gates in ((8, 8 * 7 + 7), (12, 12 * 11 + 11)):
        orc = orc_for(k)
        zero = [orc.input_labels(0, 1, i) for i in range(k)]
        out0, tab = orc.signact_garble(3, zero)
        h0 = capi.hash_calls()
        orc.signact_eval(3, zero, tab)
        assert capi.hash_calls() - h0 == gates + k


# ---------------------------------------------------------------- decode
def test_decode_flags_forged_labels():
    orc = orc_for(3)
    X = np.array([0, 7, 29, 15, 14])
    zero, act = bundle_for(orc, X)
    vals, valid = orc.decode(act, zero)
    assert valid.all() and (vals == plain.to_signed(X, orc.P)).all()
    act[1][2, 5] = (act[1][2, 5] + 1) % 3           # one digit of one residue of element 2
    vals, valid = orc.decode(act, zero)
    assert valid.tolist() == [1, 1, 0, 1, 1] and vals[2] == 0


# ---- reduced-accuracy sign (Appendix, Approximated Garbled Sign: fewer digits, M < k P) -------------
@pytest.mark.parametrize("k,digits", [(4, (4, 15)), (5, (2, 12, 25)), (5, (6, 20))])
def test_reduced_accuracy_sign_errs_only_next_to_the_boundaries(k, digits):
    """With M < k P the k rounded-up terms overestimate the fraction X/P by less than k/M: the approximated sign
    can differ from [X >= P/2] only for fractions within k/M below 1/2 or below 1, and never elsewhere."""
    orc = capi.Oracle(workloads.PRIMES[:k], digits, SEED)
    P, M = orc.P, orc.M
    assert M < k * P
    wrong = 0
    for X in range(P):
        got = orc.sign_plain(residues(X, orc.primes), 0, 0)
        exact = int(2 * X >= P)
        if got != exact:
            wrong += 1
            f = X / P
            assert (0.5 - k / M <= f < 0.5) or (1 - k / M <= f < 1), X
    assert 0 < wrong <= 2 * k * P / M + 2


def test_reduced_accuracy_relu_garbled_equals_its_plain_approximation():
    """the garbled gadget computes exactly the approximated function, wrong values included"""
    k, digits = 4, (4, 15)
    orc = capi.Oracle(workloads.PRIMES[:k], digits, SEED)
    P = orc.P
    X = np.arange(P)
    zero, act = bundle_for(orc, X)
    out0, tables = orc.relu_garble(5, zero)
    out = orc.relu_eval(5, act, tables)
    vals, valid = orc.decode(out, out0)
    assert valid.all()
    pos = np.array([orc.sign_plain(residues(int(x), orc.primes), 0, 1) for x in X])
    assert (vals == plain.to_signed(np.where(pos == 1, X, 0), P)).all()
    assert (pos != (2 * X < P)).any()


def test_packed_tables_are_horner_integers_and_unpack_back():
    """the packed storage format of the tables: every row of every segment is the integer sum_j row[j] q^j (big
    integers here) in 16 little-endian bytes; one-digit rows one byte; unpacking gives the tables back; sizes;
    not defined under the ceil rule (rows can exceed 128 bits)"""
    orc = orc_for(4, rule=1)
    P = orc.P
    X = np.arange(0, P, 7)
    n = len(X)
    zero = [orc.input_labels(0, n, i) for i in range(orc.k)]
    nd, k = len(orc.digits), orc.k
    m = [orc.mj(j) for j in range(1, nd + 1)]
    sign_segs = lambda first: [(orc.primes[i], m[j]) for i in range(first, k) for j in range(nd)] + \
        [(m[j], m[j - 1]) for j in range(1, nd)] + [(m[0], 2)]
    cases = []
    r0, rt = orc.relu_garble(3, zero)
    cases.append(("relu", 1, rt, sign_segs(0) + [s for p in orc.primes for s in ((p, p), (2, p), (2, 0))]))
    s0, st = orc.scale_garble(4, zero, 2)
    cases.append(("scale", 2, st, ([(2, p) for p in orc.primes[1:]] + sign_segs(1)) * 2))
    a0, at = orc.signact_garble(5, zero)
    cases.append(("sign", 1, at, sign_segs(0) + [(2, p) for p in orc.primes]))
    for kind, rep, tab, segs in cases:
        packed = orc.tables_pack(kind, n, tab, rep)
        assert packed.size == orc.tables_packed_bytes(kind, n, rep) == sum(n * r * 16 if q else -(-n * r // 16) * 16 for r, q in segs)
        t_at = p_at = 0
        for rows, q in segs:
            if q == 0:
                assert (packed[p_at:p_at + n * rows] == tab[t_at:t_at + 4 * n * rows:4]).all()
                t_at += 4 * n * rows
                p_at += -(-n * rows // 16) * 16
                continue
            lq = orc.lam(q)
            pitch = capi.pitch(lq)
            for r in (0, 1, n * rows // 2, n * rows - 1):
                row = tab[t_at + r * pitch:t_at + r * pitch + lq]
                want = sum(int(d) * q ** j for j, d in enumerate(row))
                assert want < 1 << 128
                assert int.from_bytes(packed[p_at + 16 * r:p_at + 16 * r + 16].tobytes(), "little") == want, (kind, q, r)
            t_at += n * rows * pitch
            p_at += n * rows * 16
        assert t_at == tab.size and p_at == packed.size
        assert (orc.tables_unpack(kind, n, packed, tab.size, rep) == tab).all(), kind
    in0 = workloads.uniform_labels(np.random.default_rng(1), 50, orc.lam(5), 5)
    o0, t = orc.proj_garble(5, 7, in0, workloads.proj_phi(np.random.default_rng(2), 50, 5, 7), 1)
    pk = orc.tables_pack("proj", 50, t.reshape(-1), p=5, q=7)
    assert pk.size == 50 * 5 * 16 and (orc.tables_unpack("proj", 50, pk, t.size, p=5, q=7) == t.reshape(-1)).all()
    assert orc_for(4, rule=0).tables_packed_bytes("relu", 10) == 0          # ceil rule: 3^81 > 2^128
