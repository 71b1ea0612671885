"""The bodies of the gate kernels (dash_bodies.h), compiled for the host with the address and
undefined-behaviour sanitizers and run lane by lane over exactly-sized buffers, against the oracle:
every access in bounds, every byte equal.  No GPU involved."""
import os
import struct
import subprocess

import numpy as np
import pytest

import workloads
from oracle import capi

HERE = os.path.dirname(os.path.abspath(__file__))
SEED = bytes(range(7, 23))


EMULATIONS = ("gate_emul", "chain_emul", "digits_emul", "mixed_emul", "cast_emul", "aes_sliced_emul")


@pytest.fixture(scope="module")
def built():
    """all emulation programs, compiled side by side (most of this module's time is their compilation)"""
    procs = [(name, subprocess.Popen(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                                      "-o", os.path.join(HERE, name + ".bin"), os.path.join(HERE, name + ".cpp")],
                                     stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)) for name in EMULATIONS]
    for name, pr in procs:
        out, _ = pr.communicate()
        assert pr.returncode == 0, (name, out[-3000:])
    return {name: os.path.join(HERE, name + ".bin") for name in EMULATIONS}


@pytest.fixture(scope="module")
def emul(built):
    return built["gate_emul"]


def run_case(emul, tmp_path, p, q, n, rule=0, shared=False, elem_base=2 ** 33 + 11, layer=9, slot=3):
    orc = capi.Oracle(workloads.PRIMES[:12], workloads.DIGITS[12], SEED, rule)
    g = np.random.default_rng(p * 1000 + q + n)
    lp, lq = orc.lam(p), orc.lam(q)
    in0 = workloads.uniform_labels(g, n, lp, p)
    phi = workloads.proj_phi(g, 1 if shared else n, p, q)
    a = g.integers(0, p, n)
    act = ((in0.astype(np.int64) + a[:, None] * orc.delta(p).astype(np.int64)[None, :]) % p).astype(np.uint8)
    blob = struct.pack("<8iQ", p, q, rule, n, layer, slot, 0 if shared else p, 0, elem_base) + SEED
    blob += orc.delta(p).tobytes() + orc.delta(q).tobytes() + in0.tobytes() + act.tobytes() + phi.tobytes()
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([emul, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    out = np.fromfile(fout, np.uint8)
    pitch = capi.pitch(lq)
    o0, tab, o = np.split(out, [n * lq, n * lq + n * p * pitch])
    r0, rt = orc.proj_garble(p, q, in0, phi[0] if shared else phi, layer, slot, elem_base)
    ro = orc.proj_eval(p, q, act, rt, layer, slot, elem_base)
    assert (o0.reshape(n, lq) == r0).all()
    assert (tab == rt.reshape(-1)).all()
    assert (o.reshape(n, lq) == ro).all()


@pytest.mark.parametrize("p,q", [(2, 2), (2, 37), (3, 3), (37, 2), (19, 96), (96, 96), (96, 26), (26, 2), (204, 46), (46, 204),
                                 (13, 204), (5, 7), (100, 60), (255, 3)])
def test_gate_bodies_under_sanitizers(emul, tmp_path, p, q):
    run_case(emul, tmp_path, p, q, 300)


def test_gate_bodies_sizes_and_rules(emul, tmp_path):
    for n in (1, 255, 256, 257, 777):
        run_case(emul, tmp_path, 2, 2, n)
        run_case(emul, tmp_path, 7, 96, n)
    run_case(emul, tmp_path, 11, 13, 100, rule=1)
    run_case(emul, tmp_path, 3, 5, 100, shared=True)


# ---- the evaluator's fused carry chain ------------------------------------------------------------


@pytest.fixture(scope="module")
def chain_emul(built):
    return built["chain_emul"]


def run_chain(chain_emul, tmp_path, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 5, layer=4, slot0=70, lam2=0, quad=False):
    """m[0..n-1] = accumulation moduli of digits 1..n.  The tables are random bytes below the output modulus:
    the evaluator's result is defined by them alone, C_{j-1} = row[colour(S_j)] - H(S_j), S_j = sum_j + C_j
    (Appendix, Garbled Mixed-Radix Addition), recomputed here with the oracle's hash."""
    orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule)
    if lam2:        # an explicit label length for modulus 2 (the output wire of the chain)
        orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule, lam=[lam2] + [orc.lam(p) for p in workloads.PRIMES[1:8]])
    n = len(m)
    g = np.random.default_rng(sum(m) + n_elem)
    slots = [slot0 + n - 1] + [slot0 + (j - 2) for j in range(2, n + 1)]          # digit 1 feeds the final gate
    sums = [g.integers(0, mj, (n_elem, orc.lam(mj))).astype(np.uint8) for mj in m]
    outm = [2] + m[:-1]                                                           # output modulus of the gate fed by digit j
    tabs = []
    for j in range(n):
        lam_o = orc.lam(outm[j])
        pitch = capi.pitch(lam_o)
        t = np.zeros((n_elem, m[j], pitch), np.uint8)
        t[:, :, :lam_o] = g.integers(0, outm[j], (n_elem, m[j], lam_o))
        tabs.append(t)
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, lam2, 1 if quad else 0, 0, elem_base)
    blob += struct.pack("<%di" % n, *m) + struct.pack("<%di" % n, *slots)
    blob += b"".join(s.tobytes() for s in sums) + b"".join(t.tobytes() for t in tabs)
    fin, fout = str(tmp_path / "cin.bin"), str(tmp_path / "cout.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([chain_emul, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    got = np.fromfile(fout, np.uint8).reshape(n_elem, orc.lam(2))
    for e in range(n_elem):
        carry = None
        for j in range(n - 1, -1, -1):
            S = sums[j][e].astype(np.int64)
            if carry is not None:
                S = (S + carry) % m[j]
            S = S.astype(np.uint8)
            h = orc.hash(S, m[j], layer, slots[j], elem_base + e, outm[j]).astype(np.int64)
            lam_o = orc.lam(outm[j])
            carry = (tabs[j][e, int(S[0]), :lam_o].astype(np.int64) - h) % outm[j]
        assert (got[e] == carry).all(), (e, variant)


def test_chain_bodies_under_sanitizers(chain_emul, tmp_path):
    run_chain(chain_emul, tmp_path, [26] + [96] * 6, 1, 300)
    run_chain(chain_emul, tmp_path, [26] + [96] * 6, 0, 70)
    run_chain(chain_emul, tmp_path, [46] + [204] * 10, 2, 260)
    run_chain(chain_emul, tmp_path, [46] + [204] * 10, 0, 40)
    run_chain(chain_emul, tmp_path, [10] + [91] * 5, 3, 130)            # the default sets of the 7- and 9-prime bases
    run_chain(chain_emul, tmp_path, [26] + [96] * 6, 1, 301, quad=True)    # four lanes per element (indexing and stores)
    run_chain(chain_emul, tmp_path, [46] + [204] * 10, 2, 65, quad=True)
    run_chain(chain_emul, tmp_path, [22] + [90] * 8, 4, 130)
    run_chain(chain_emul, tmp_path, [2, 6], 0, 257)                 # small bases: generic body, a 128-digit first label
    run_chain(chain_emul, tmp_path, [2, 15, 27], 0, 65)
    run_chain(chain_emul, tmp_path, [4, 60, 56], 0, 33, rule=1)
    run_chain(chain_emul, tmp_path, [26, 96], 1, 5)                 # n = 2: no same-modulus step
    run_chain(chain_emul, tmp_path, [26] + [96] * 6, 0, 70, lam2=64)    # label length of modulus 2 given explicitly
    run_chain(chain_emul, tmp_path, [4, 60], 0, 300, lam2=100)


# ---- the evaluator's fused digit gates --------------------------------------------------------------


@pytest.fixture(scope="module")
def digits_emul(built):
    return built["digits_emul"]


def run_digits(digits_emul, tmp_path, primes, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 9, layer=6, slot0=40, wide=False):
    """the n digit gates of every residue in one pass over its label: gate (t, j) is an ordinary projection gate
    p_t -> m_j with slot slot0 + t n + (j - 1) (Appendix, approximated sign), so every output must equal the
    oracle's evaluation of that gate on the same table segment"""
    orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule)
    n = len(m)
    g = np.random.default_rng(sum(m) + n_elem + len(primes))
    acts = [workloads.uniform_labels(g, n_elem, orc.lam(p), p) for p in primes]
    tabs = []
    for p in primes:
        row = []
        for mj in m:
            lam_o = orc.lam(mj)
            t = np.zeros((n_elem, p, capi.pitch(lam_o)), np.uint8)
            t[:, :, :lam_o] = g.integers(0, mj, (n_elem, p, lam_o))
            row.append(t)
        tabs.append(row)
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, len(primes), slot0, 2 if wide else 0, elem_base)
    blob += struct.pack("<%di" % n, *m) + struct.pack("<%di" % len(primes), *primes)
    blob += b"".join(a.tobytes() for a in acts)
    blob += b"".join(t.tobytes() for row in tabs for t in row)
    fin, fout = str(tmp_path / "din.bin"), str(tmp_path / "dout.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([digits_emul, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    got = np.fromfile(fout, np.uint8)
    at = 0
    for t, p in enumerate(primes):
        for j, mj in enumerate(m):
            lam_o = orc.lam(mj)
            want = orc.proj_eval(p, mj, acts[t], tabs[t][j], layer, slot0 + t * n + j, elem_base)
            assert (got[at:at + n_elem * lam_o].reshape(n_elem, lam_o) == want).all(), (p, mj)
            at += n_elem * lam_o
    assert at == got.size


def test_digit_gate_bodies_under_sanitizers(digits_emul, tmp_path):
    run_digits(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17, 19], [26] + [96] * 6, 1, 300)
    run_digits(digits_emul, tmp_path, [3, 19], [26] + [96] * 6, 0, 70)
    run_digits(digits_emul, tmp_path, [2, 23, 37], [46] + [204] * 10, 2, 260)
    run_digits(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17], [10] + [91] * 5, 3, 130)
    run_digits(digits_emul, tmp_path, [2, 11, 23], [22] + [90] * 8, 4, 130)
    run_digits(digits_emul, tmp_path, [2, 3], [2, 6], 0, 257)
    run_digits(digits_emul, tmp_path, [3, 5, 7], [4, 60, 56], 0, 33, rule=1)
    run_digits(digits_emul, tmp_path, [13], [26], 0, 5)                 # one digit, one residue
    run_digits(digits_emul, tmp_path, [5, 7], [26, 12, 12], 0, 100)      # a reduced-accuracy set


def test_digit_gates_one_per_lane_under_sanitizers(digits_emul, tmp_path):
    """the form for gadgets over few elements: a lane per (element, residue, digit)"""
    run_digits(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17, 19], [26] + [96] * 6, 1, 300, wide=True)
    run_digits(digits_emul, tmp_path, [2, 23, 37], [46] + [204] * 10, 2, 260, wide=True)
    run_digits(digits_emul, tmp_path, [3, 17], [10] + [91] * 5, 3, 70, wide=True)
    run_digits(digits_emul, tmp_path, [5, 23], [22] + [90] * 8, 4, 70, wide=True)
    run_digits(digits_emul, tmp_path, [3, 5, 7], [4, 60, 56], 0, 33, rule=1, wide=True)
    run_digits(digits_emul, tmp_path, [13], [26], 0, 5, wide=True)


def run_digits_sums(digits_emul, tmp_path, primes, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 9, layer=6, slot0=40):
    """the form for few elements in which the digit gates add up their outputs themselves: wire S_j must be the sum over
    the residues of the oracle's gate outputs (t, j), mod m_j (Appendix, Garbled Mixed-Radix Addition: the free sums)"""
    orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule)
    n = len(m)
    g = np.random.default_rng(3 * sum(m) + n_elem + len(primes))
    acts = [workloads.uniform_labels(g, n_elem, orc.lam(p), p) for p in primes]
    tabs = []
    for p in primes:
        row = []
        for mj in m:
            lam_o = orc.lam(mj)
            t = np.zeros((n_elem, p, capi.pitch(lam_o)), np.uint8)
            t[:, :, :lam_o] = g.integers(0, mj, (n_elem, p, lam_o))
            row.append(t)
        tabs.append(row)
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, len(primes), slot0, 4, elem_base)
    blob += struct.pack("<%di" % n, *m) + struct.pack("<%di" % len(primes), *primes)
    blob += b"".join(a.tobytes() for a in acts)
    blob += b"".join(t.tobytes() for row in tabs for t in row)
    fin, fout = str(tmp_path / "sin.bin"), str(tmp_path / "sout.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([digits_emul, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    got = np.fromfile(fout, np.uint8)
    at = 0
    for j, mj in enumerate(m):
        lam_o = orc.lam(mj)
        want = np.zeros((n_elem, lam_o), np.int64)
        for t, p in enumerate(primes):
            want += orc.proj_eval(p, mj, acts[t], tabs[t][j], layer, slot0 + t * n + j, elem_base)
        assert (got[at:at + n_elem * lam_o].reshape(n_elem, lam_o) == want % mj).all(), mj
        at += n_elem * lam_o
    assert at == got.size


def test_digit_gates_with_their_sums_under_sanitizers(digits_emul, tmp_path):
    run_digits_sums(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17, 19], [26] + [96] * 6, 1, 150)
    run_digits_sums(digits_emul, tmp_path, [3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37], [46] + [204] * 10, 2, 70)      # the scaling gadget's 11 residues
    run_digits_sums(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17], [10] + [91] * 5, 3, 65)
    run_digits_sums(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17, 19, 23], [22] + [90] * 8, 4, 1)


def run_digits_garble(digits_emul, tmp_path, primes, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 9, layer=6, slot0=40, wide=False):
    """the garbler's side of the same gates: rows[colour(l0 + a R_p)] = out0 + phi_j(a) R_{m_j} + H(l0 + a R_p), every
    table segment against the oracle's projection gate with the same zero labels and function table"""
    orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule)
    n = len(m)
    g = np.random.default_rng(7 * sum(m) + n_elem + len(primes))
    in0 = [workloads.uniform_labels(g, n_elem, orc.lam(p), p) for p in primes]
    phis = [np.stack([g.integers(0, mj, p).astype(np.uint8) for mj in m]) for p in primes]
    want = [[orc.proj_garble(p, mj, in0[t], phis[t][j], layer, slot0 + t * n + j, elem_base) for j, mj in enumerate(m)]
            for t, p in enumerate(primes)]
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, len(primes), slot0, 3 if wide else 1, elem_base)
    blob += struct.pack("<%di" % n, *m) + struct.pack("<%di" % len(primes), *primes)
    blob += b"".join(a.tobytes() for a in in0)
    blob += b"".join(orc.delta(p).tobytes() for p in primes) + b"".join(orc.delta(mj).tobytes() for mj in m)
    blob += b"".join(want[t][j][0].tobytes() for t in range(len(primes)) for j in range(n))
    blob += b"".join(ph.tobytes() for ph in phis)
    fin, fout = str(tmp_path / "gin.bin"), str(tmp_path / "gout.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([digits_emul, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr[-3000:])
    got = np.fromfile(fout, np.uint8)
    at = 0
    for t, p in enumerate(primes):
        for j, mj in enumerate(m):
            size = n_elem * p * capi.pitch(orc.lam(mj))
            assert (got[at:at + size] == want[t][j][1].reshape(-1)).all(), (p, mj)
            at += size
    assert at == got.size


def test_digit_row_bodies_under_sanitizers(digits_emul, tmp_path):
    run_digits_garble(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17, 19], [26] + [96] * 6, 1, 150)
    run_digits_garble(digits_emul, tmp_path, [3, 19], [26] + [96] * 6, 0, 70)
    run_digits_garble(digits_emul, tmp_path, [2, 23, 37], [46] + [204] * 10, 2, 130)
    run_digits_garble(digits_emul, tmp_path, [2, 7, 17], [10] + [91] * 5, 3, 70)
    run_digits_garble(digits_emul, tmp_path, [3, 23], [22] + [90] * 8, 4, 70)
    run_digits_garble(digits_emul, tmp_path, [2, 3], [2, 6], 0, 257)
    run_digits_garble(digits_emul, tmp_path, [3, 5, 7], [4, 60, 56], 0, 33, rule=1)
    run_digits_garble(digits_emul, tmp_path, [13], [26], 0, 5)


def test_digit_rows_one_per_lane_under_sanitizers(digits_emul, tmp_path):
    """the garbler's form for gadgets over few elements: a lane per ciphertext row (element, value, digit)"""
    run_digits_garble(digits_emul, tmp_path, [2, 3, 5, 7, 11, 13, 17, 19], [26] + [96] * 6, 1, 150, wide=True)
    run_digits_garble(digits_emul, tmp_path, [2, 23, 37], [46] + [204] * 10, 2, 130, wide=True)
    run_digits_garble(digits_emul, tmp_path, [5, 13], [10] + [91] * 5, 3, 40, wide=True)
    run_digits_garble(digits_emul, tmp_path, [2, 19], [22] + [90] * 8, 4, 40, wide=True)
    run_digits_garble(digits_emul, tmp_path, [3, 5, 7], [4, 60, 56], 0, 33, rule=1, wide=True)
    run_digits_garble(digits_emul, tmp_path, [13], [26], 0, 5, wide=True)


# ---- one evaluator launch that mixes output moduli -------------------------------------------------
def test_mixed_output_moduli_in_one_eval_launch_under_sanitizers(built, tmp_path):
    """the evaluator's any-modulus instantiation picks a compile-time description of the output modulus per job:
    16 jobs with 16 of the 20 described moduli as outputs in ONE launch (two lists, so that each of the 20 occurs),
    exactly-sized buffers, address sanitizer; same results as the single-modulus instantiations"""
    exe = built["mixed_emul"]
    for n, seed, which in ((1, 1, 0), (257, 2, 0), (300, 3, 0), (130, 4, 1)):
        r = subprocess.run([exe, str(n), str(seed), str(which)], capture_output=True, text=True)
        assert r.returncode == 0 and r.stdout.strip() == "ok", r.stderr[-3000:]


# ---- evaluator kernels that read a wire of modulus 2 ------------------------------------------------
def run_cast(tmp_path, exe, p, n, addc, rule=0, lam2=0, lam_p=0, elem_base=2 ** 34 + 1, layer=12, slot=200):
    """cast-and-halve of the scaling gadget, b = (x + addc one - cast) / 2 with cast = rows[colour(y)] - H_p(y)
    (Sec. The Scaling Operation), and the evaluator's half-gate step z = V + beta x - U with
    beta = S[colour(y)] - H_p(y)[0] (Appendix), from random tables, recomputed here with the oracle's hash"""
    primes = workloads.PRIMES[:8]
    base = capi.Oracle(primes, workloads.DIGITS[8], SEED, rule)
    lam = [base.lam(q) for q in primes]
    if lam2:
        lam[0] = lam2
    if lam_p:
        lam[primes.index(p)] = lam_p
    orc = capi.Oracle(primes, workloads.DIGITS[8], SEED, rule, lam=lam)
    l2, lp = orc.lam(2), orc.lam(p)
    pitch = capi.pitch(lp)
    g = np.random.default_rng(p * 100 + n + lam2)
    y = g.integers(0, 2, (n, l2)).astype(np.uint8)
    x, U, V = (g.integers(0, p, (n, lp)).astype(np.uint8) for _ in range(3))
    one = g.integers(0, p, lp).astype(np.uint8)
    table = np.zeros((n, 2, pitch), np.uint8)
    table[:, :, :lp] = g.integers(0, p, (n, 2, lp))
    S = np.zeros((n, 2, 4), np.uint8)
    S[:, :, 0] = g.integers(0, p, (n, 2))
    blob = struct.pack("<8iQ", p, n, rule, layer, slot, addc, lam2, lam_p, elem_base)
    blob += b"".join(a.tobytes() for a in (y, x, one, table, U, V, S))
    fin, fout = str(tmp_path / "kin.bin"), str(tmp_path / "kout.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([exe, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    b, z = np.split(np.fromfile(fout, np.uint8), 2)
    b, z = b.reshape(n, lp), z.reshape(n, lp)
    inv2 = (p + 1) // 2
    for e in range(n):
        colour = int(y[e, 0])
        cast = (table[e, colour, :lp].astype(np.int64) - orc.hash(y[e], 2, layer, slot, elem_base + e, p)) % p
        assert (b[e] == ((x[e].astype(np.int64) + addc * one.astype(np.int64) - cast) * inv2) % p).all(), ("cast", e)
        beta = (int(S[e, colour, 0]) - int(orc.hash(y[e], 2, layer, slot + 2, elem_base + e, p)[0])) % p
        assert (z[e] == (V[e].astype(np.int64) + beta * x[e].astype(np.int64) - U[e]) % p).all(), ("half gate", e)


def test_cast_and_half_gate_bodies_under_sanitizers(built, tmp_path):
    exe = built["cast_emul"]
    run_cast(tmp_path, exe, 3, 300, 0)
    run_cast(tmp_path, exe, 19, 257, 7)
    run_cast(tmp_path, exe, 7, 40, 3, rule=1)
    run_cast(tmp_path, exe, 5, 70, 2, lam2=64)                   # label lengths given explicitly: modulus 2 shorter than 128
    run_cast(tmp_path, exe, 13, 33, 0, lam2=100, lam_p=9)


def test_bitsliced_aes_against_the_standard_and_the_oracle(built, tmp_path):
    """dash_aes_sliced.h (32 blocks per lane on bit planes, generated S-box circuit) on the host under the
    sanitizers: FIPS-197 Appendix B and C.1 vectors, and random blocks under random keys against the oracle's AES."""
    exe = built["aes_sliced_emul"]

    def run(key, blocks):
        fin, fout = str(tmp_path / "aes_in.bin"), str(tmp_path / "aes_out.bin")
        open(fin, "wb").write(bytes(key) + blocks.tobytes())
        r = subprocess.run([exe, fin, fout], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        return np.fromfile(fout, np.uint8).reshape(-1, 16)

    # Appendix C.1: key 00..0f, plaintext 00 11 .. ff
    pt = np.zeros((32, 16), np.uint8)
    pt[5] = np.frombuffer(bytes.fromhex("00112233445566778899aabbccddeeff"), np.uint8)
    out = run(bytes(range(16)), pt)
    assert out[5].tobytes().hex() == "69c4e0d86a7b0430d8cdb78070b4c55a"
    # Appendix B: key 2b7e..., input 3243...
    pt[31] = np.frombuffer(bytes.fromhex("3243f6a8885a308d313198a2e0370734"), np.uint8)
    out = run(bytes.fromhex("2b7e151628aed2a6abf7158809cf4f3c"), pt)
    assert out[31].tobytes().hex() == "3925841d02dc09fbdc118597196a0b32"
    g = np.random.default_rng(5)
    for _ in range(3):
        key = g.integers(0, 256, 16, dtype=np.uint8)
        blocks = g.integers(0, 256, (96, 16), dtype=np.uint8)
        out = run(key.tobytes(), blocks)
        for j in range(96):
            assert (out[j] == capi.aes128_encrypt(key, blocks[j])).all(), j
