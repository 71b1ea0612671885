"""Pins for the oracle's primitives: AES, label length, compress / decompress, hash, PRG.

None of these compares the oracle with itself: AES against the standard's vectors and the
openssl binary, the integer routines against Python big integers, the hash and PRG against
a recomputation from AES (openssl) + big integers written here.
"""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import capi

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _vectors():
    out = []
    for line in open(os.path.join(GOLD, "aes128_fips197.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            out.append([bytes.fromhex(t) for t in line.split()])
    return out


def test_aes_fips197_vectors():
    vecs = _vectors()
    assert len(vecs) == 2
    for key, pt, ct in vecs:
        got = capi.aes128_encrypt(np.frombuffer(key, np.uint8), np.frombuffer(pt, np.uint8))
        assert got.tobytes() == ct


def _openssl_ecb(key, blocks):
    exe = shutil.which("openssl")
    if exe is None:
        pytest.skip("openssl CLI not present")
    r = subprocess.run([exe, "enc", "-aes-128-ecb", "-nopad", "-K", key.hex()], input=blocks,
                       capture_output=True, check=True)
    return r.stdout


def test_aes_against_openssl_random_blocks():
    g = np.random.default_rng(11)
    for _ in range(4):
        key = g.integers(0, 256, 16, dtype=np.uint8)
        blocks = g.integers(0, 256, (32, 16), dtype=np.uint8)
        ref = _openssl_ecb(key.tobytes(), blocks.tobytes())
        for b in range(32):
            assert capi.aes128_encrypt(key, blocks[b]).tobytes() == ref[16 * b:16 * b + 16]


def test_label_length_rules_all_moduli():
    two128 = 1 << 128
    for m in range(2, 256):
        ceil_l = capi.lam(m, 0)
        floor_l = capi.lam(m, 1)
        assert m ** ceil_l >= two128 and m ** (ceil_l - 1) < two128
        assert m ** floor_l <= two128 and m ** (floor_l + 1) > two128
    # the values the 12-prime base must give under the two rules
    want_ceil = {2: 128, 3: 81, 5: 56, 7: 46, 11: 38, 13: 35, 17: 32, 19: 31, 23: 29, 29: 27, 31: 26, 37: 25}
    want_floor = {2: 128, 3: 80, 5: 55, 7: 45, 11: 37, 13: 34, 17: 31, 19: 30, 23: 28, 29: 26, 31: 25, 37: 24}
    for p in want_ceil:
        assert capi.lam(p, 0) == want_ceil[p]
        assert capi.lam(p, 1) == want_floor[p]
    assert sum(want_ceil[p] for p in list(want_ceil)[:8]) == 447
    assert sum(want_ceil.values()) == 554


@pytest.mark.parametrize("q", [2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 26, 46, 96, 204, 255])
def test_compress_is_horner_mod_2_128(q):
    g = np.random.default_rng(q)
    for rule in (0, 1):
        L = capi.lam(q, rule)
        for _ in range(20):
            lab = g.integers(0, q, L, dtype=np.uint8)
            want = sum(int(lab[j]) * q ** j for j in range(L)) % (1 << 128)
            assert capi.compress(lab, q) == want
        # extreme labels: all q-1 (wraps mod 2^128 under the ceil rule) and a single top digit
        lab = np.full(L, q - 1, np.uint8)
        assert capi.compress(lab, q) == (q ** L - 1) % (1 << 128)
        lab = np.zeros(L, np.uint8)
        lab[L - 1] = q - 1
        assert capi.compress(lab, q) == ((q - 1) * q ** (L - 1)) % (1 << 128)


@pytest.mark.parametrize("q", [2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 26, 46, 96, 204, 255])
def test_decompress_is_base_q_digits(q):
    g = np.random.default_rng(100 + q)
    for rule in (0, 1):
        L = capi.lam(q, rule)
        hs = [0, 1, (1 << 128) - 1, 1 << 127] + [int.from_bytes(g.bytes(16), "little") for _ in range(20)]
        for h in hs:
            got = capi.decompress(h, q, L)
            want = [(h // q ** j) % q for j in range(L)]
            assert got.tolist() == want
            if rule == 1:   # floor rule: compress inverts decompress on h mod q^L
                assert capi.compress(got, q) == h % (q ** L)


def _orc(primes=(2, 3, 5), digits=(2, 5, 9), seed=bytes(range(16, 32)), rule=0):
    return capi.Oracle(primes, digits, seed, rule)


def test_hash_is_compress_aes_feedforward_decompress():
    """H_q(L, T) recomputed here from big integers and the openssl binary."""
    orc = _orc()
    g = np.random.default_rng(5)
    fixed_key = bytes(range(16))
    for (p, q) in [(2, 3), (3, 2), (5, 15), (27, 2), (5, 5), (37, 204)]:
        lp, lq = orc.lam(p), orc.lam(q)
        lab = g.integers(0, p, lp, dtype=np.uint8)
        layer, slot, elem = 7, 0x01020304, 0x1122334455667788
        K = sum(int(lab[j]) * p ** j for j in range(lp)) % (1 << 128)
        T = elem | (slot << 64) | (layer << 96)
        X = K ^ T
        enc = int.from_bytes(_openssl_ecb(fixed_key, X.to_bytes(16, "little")), "little")
        h = enc ^ X
        want = [(h // q ** j) % q for j in range(lq)]
        assert orc.hash(lab, p, layer, slot, elem, q).tolist() == want


def test_prg_draw_is_aes_of_counter_block():
    seed = bytes(range(16, 32))
    orc = _orc(seed=seed)
    for (domain, layer, slot, elem, m) in [(2, 3, 5, 9, 7), (1, 0, 0, 12345678901, 2), (3, 65535, 2 ** 32 - 1, 2 ** 63, 37)]:
        blk = elem.to_bytes(8, "little") + slot.to_bytes(4, "little") + layer.to_bytes(2, "little") + bytes([domain, m])
        enc = int.from_bytes(_openssl_ecb(seed, blk), "little")
        lam = orc.lam(m)
        assert orc.draw(domain, layer, slot, elem, m).tolist() == [(enc // m ** j) % m for j in range(lam)]


def test_offsets_have_colour_one_and_inputs_differ():
    orc = _orc()
    for m in (2, 3, 5, 15, 27, 255):
        d = orc.delta(m)
        assert d[0] == 1 and d.max() < m and len(d) == orc.lam(m)
    a = orc.input_labels(0, 8, 1)
    b = orc.input_labels(4, 4, 1)
    assert (a[4:] == b).all()                      # counter based: any wire alone
    assert len({r.tobytes() for r in a}) == 8      # and distinct


def test_explicit_label_lengths_per_prime():
    """label lengths given per prime (instead of the rule): lengths, hash and PRG recomputed from big integers and
    openssl; digits past the 128-bit hash are zero; every projection-gate input still evaluates to its payload"""
    primes, lam = (2, 3, 5, 7), (64, 90, 17, 46)
    orc = capi.Oracle(primes, (4, 15, 14), bytes(range(16, 32)), 0, lam=lam)
    ref = capi.Oracle(primes, (4, 15, 14), bytes(range(16, 32)), 0)
    for p, l in zip(primes, lam):
        assert orc.lam(p) == l and len(orc.delta(p)) == l and orc.delta(p)[0] == 1
    assert orc.lam(60) == ref.lam(60)            # the accumulation moduli keep the rule
    g = np.random.default_rng(6)
    fixed_key = bytes(range(16))
    for p, q in [(2, 3), (3, 5), (5, 2), (7, 3)]:
        lp, lq = orc.lam(p), orc.lam(q)
        lab = g.integers(0, p, lp, dtype=np.uint8)
        K = sum(int(lab[j]) * p ** j for j in range(lp)) % (1 << 128)
        X = K ^ (9 | (3 << 64) | (5 << 96))
        h = int.from_bytes(_openssl_ecb(fixed_key, X.to_bytes(16, "little")), "little") ^ X
        assert orc.hash(lab, p, 5, 3, 9, q).tolist() == [(h // q ** j) % q for j in range(lq)]
    assert (orc.hash(np.zeros(64, np.uint8), 2, 1, 1, 1, 3)[81:] == 0).all()      # 3^81 > 2^128
    for p, q in [(3, 5), (5, 2), (2, 7), (7, 3)]:
        in0 = g.integers(0, p, (1, orc.lam(p)), dtype=np.uint8)
        phi = g.integers(0, q, p, dtype=np.uint8)
        out0, table = orc.proj_garble(p, q, in0, phi, 2, 4, 77)
        for a in range(p):
            act = ((in0.astype(np.int64) + a * orc.delta(p)) % p).astype(np.uint8)
            out = orc.proj_eval(p, q, act, table, 2, 4, 77)
            assert (out == (out0.astype(np.int64) + int(phi[a]) * orc.delta(q)) % q).all()
