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
EXE = os.path.join(HERE, "gate_emul.bin")
SEED = bytes(range(7, 23))


@pytest.fixture(scope="module")
def emul():
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-o", EXE, os.path.join(HERE, "gate_emul.cpp")])
    return EXE


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
CHAIN_EXE = os.path.join(HERE, "chain_emul.bin")


@pytest.fixture(scope="module")
def chain_emul():
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-o", CHAIN_EXE, os.path.join(HERE, "chain_emul.cpp")])
    return CHAIN_EXE


def run_chain(chain_emul, tmp_path, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 5, layer=4, slot0=70):
    """m[0..n-1] = accumulation moduli of digits 1..n.  The tables are random bytes below the output modulus:
    the evaluator's result is defined by them alone, C_{j-1} = row[colour(S_j)] - H(S_j), S_j = sum_j + C_j
    (Appendix, Garbled Mixed-Radix Addition), recomputed here with the oracle's hash."""
    orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule)
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
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, 0, 0, 0, elem_base)
    blob += struct.pack("<%di" % n, *m) + struct.pack("<%di" % n, *slots)
    blob += b"".join(s.tobytes() for s in sums) + b"".join(t.tobytes() for t in tabs)
    fin, fout = str(tmp_path / "cin.bin"), str(tmp_path / "cout.bin")
    open(fin, "wb").write(blob)
    r = subprocess.run([chain_emul, fin, fout], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    got = np.fromfile(fout, np.uint8).reshape(n_elem, 128)
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
    run_chain(chain_emul, tmp_path, [2, 6], 0, 257)                 # small bases: generic body, a 128-digit first label
    run_chain(chain_emul, tmp_path, [2, 15, 27], 0, 65)
    run_chain(chain_emul, tmp_path, [4, 60, 56], 0, 33, rule=1)
    run_chain(chain_emul, tmp_path, [26, 96], 1, 5)                 # n = 2: no same-modulus step


# ---- the evaluator's fused digit gates --------------------------------------------------------------
DIGITS_EXE = os.path.join(HERE, "digits_emul.bin")


@pytest.fixture(scope="module")
def digits_emul():
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-o", DIGITS_EXE, os.path.join(HERE, "digits_emul.cpp")])
    return DIGITS_EXE


def run_digits(digits_emul, tmp_path, primes, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 9, layer=6, slot0=40):
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
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, len(primes), slot0, 0, elem_base)
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
    run_digits(digits_emul, tmp_path, [2, 3], [2, 6], 0, 257)
    run_digits(digits_emul, tmp_path, [3, 5, 7], [4, 60, 56], 0, 33, rule=1)
    run_digits(digits_emul, tmp_path, [13], [26], 0, 5)                 # one digit, one residue
    run_digits(digits_emul, tmp_path, [5, 7], [26, 12, 12], 0, 100)      # a reduced-accuracy set


def run_digits_garble(digits_emul, tmp_path, primes, m, variant, n_elem, rule=0, elem_base=2 ** 32 + 9, layer=6, slot0=40):
    """the garbler's side of the same gates: rows[colour(l0 + a R_p)] = out0 + phi_j(a) R_{m_j} + H(l0 + a R_p), every
    table segment against the oracle's projection gate with the same zero labels and function table"""
    orc = capi.Oracle(workloads.PRIMES[:8], workloads.DIGITS[8], SEED, rule)
    n = len(m)
    g = np.random.default_rng(7 * sum(m) + n_elem + len(primes))
    in0 = [workloads.uniform_labels(g, n_elem, orc.lam(p), p) for p in primes]
    phis = [np.stack([g.integers(0, mj, p).astype(np.uint8) for mj in m]) for p in primes]
    want = [[orc.proj_garble(p, mj, in0[t], phis[t][j], layer, slot0 + t * n + j, elem_base) for j, mj in enumerate(m)]
            for t, p in enumerate(primes)]
    blob = struct.pack("<8iQ", n, n_elem, rule, layer, variant, len(primes), slot0, 1, elem_base)
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
    run_digits_garble(digits_emul, tmp_path, [2, 3], [2, 6], 0, 257)
    run_digits_garble(digits_emul, tmp_path, [3, 5, 7], [4, 60, 56], 0, 33, rule=1)
    run_digits_garble(digits_emul, tmp_path, [13], [26], 0, 5)
