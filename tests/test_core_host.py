"""The per-lane arithmetic of the HIP kernels (dash_core.h), compiled for the host, against the
oracle and against plain Python integers.  No GPU involved."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

from oracle import capi

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "core_check.cpp")
SO = os.path.join(HERE, "libcore_check.so")
MODULI = [2, 3, 4, 5, 7, 11, 13, 16, 17, 19, 23, 29, 31, 37, 12, 15, 26, 27, 46, 56, 60, 96, 100, 125, 128, 129, 181, 182, 204, 255]


@pytest.fixture(scope="module")
def cc():
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-o", SO, SRC])
    lib = C.CDLL(SO)
    for f in ("cc_addmod4", "cc_submod4", "cc_axpymod4", "cc_mod_m"):
        getattr(lib, f).restype = C.c_uint32
    return lib


def test_label_lengths(cc):
    for m in range(2, 256):
        for rule in (0, 1):
            assert cc.cc_lambda(m, rule) == capi.lam(m, rule)


@pytest.mark.parametrize("rule", [0, 1])
def test_hash_matches_oracle(cc, rule):
    orc = capi.Oracle([2, 3, 5], [2, 5, 9], bytes(range(16)), rule)
    g = np.random.default_rng(rule)
    for p in MODULI:
        for q, rep in [(q, r) for q in (MODULI if p in (2, 3, 37, 204) else [2, 3, 13, 96, 204]) for r in range(25 if p == 3 else 4)]:
            lp, lq = orc.lam(p), orc.lam(q)
            lab = g.integers(0, p, lp, dtype=np.uint8)
            if g.integers(0, 4) == 0:
                lab[:] = p - 1
            elem, slot, layer = int(g.integers(0, 2 ** 62)), int(g.integers(0, 2 ** 32)), int(g.integers(0, 2 ** 16))
            out = np.zeros(4 * ((lq + 3) // 4), np.uint8)
            col = C.c_uint32()
            want = orc.hash(lab, p, layer, slot, elem, q)
            for fn in (cc.cc_hash, cc.cc_hash_spec):      # run-time and compile-time modulus descriptions
                out[:] = 0xEE
                fn(lab.ctypes.data_as(C.c_void_p), p, q, rule, C.c_uint64(elem), C.c_uint32(slot), C.c_uint32(layer),
                   out.ctypes.data_as(C.c_void_p), C.byref(col))
                assert (out[:lq] == want).all(), (p, q)
                assert (out[lq:] == 0).all() and col.value == lab[0]


def test_draw_matches_oracle(cc):
    seed = bytes(range(100, 116))
    orc = capi.Oracle([2, 3, 5], [2, 5, 9], seed, 0)
    sb = np.frombuffer(seed, np.uint8).copy()
    for m in MODULI:
        lam = orc.lam(m)
        out = np.zeros(4 * ((lam + 3) // 4), np.uint8)
        d0 = C.c_uint32()
        cc.cc_draw(sb.ctypes.data_as(C.c_void_p), 2, 513, 77, C.c_uint64(2 ** 40 + m), m, 0, out.ctypes.data_as(C.c_void_p), C.byref(d0))
        want = orc.draw(2, 513, 77, 2 ** 40 + m, m)
        assert (out[:lam] == want).all() and d0.value == want[0]


def test_packed_digit_arithmetic(cc):
    g = np.random.default_rng(9)
    for m in MODULI:
        for _ in range(200):
            a = g.integers(0, m, 4)
            b = g.integers(0, m, 4)
            c = int(g.integers(0, m))
            pa = int(a[0] | a[1] << 8 | a[2] << 16 | a[3] << 24)
            pb = int(b[0] | b[1] << 8 | b[2] << 16 | b[3] << 24)
            unpack = lambda w: [(w >> (8 * i)) & 255 for i in range(4)]
            assert unpack(cc.cc_addmod4(pa, pb, m)) == ((a + b) % m).tolist()
            assert unpack(cc.cc_submod4(pa, pb, m)) == ((a - b) % m).tolist()
            assert unpack(cc.cc_axpymod4(pa, c, pb, m)) == ((a + c * b) % m).tolist()
        for n in [0, 1, m - 1, m, 2 ** 24 - 1] + g.integers(0, 2 ** 24, 50).tolist():
            assert cc.cc_mod_m(int(n), m) == n % m


def test_aes_two_table_formulation(cc):
    """T2 = rot16(T0), T3 = rot16(T1): the two-table rounds against the FIPS-197 example and against the
    four-table rounds on random blocks"""
    key = np.arange(16, dtype=np.uint8)
    pt = np.frombuffer(bytes.fromhex("00112233445566778899aabbccddeeff"), np.uint8).copy()
    o4, o2 = np.zeros(16, np.uint8), np.zeros(16, np.uint8)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    cc.cc_aes_both(p(key), p(pt), p(o4), p(o2))
    assert o4.tobytes().hex() == o2.tobytes().hex() == "69c4e0d86a7b0430d8cdb78070b4c55a"
    g = np.random.default_rng(5)
    for _ in range(200):
        key, pt = g.integers(0, 256, 16, dtype=np.uint8), g.integers(0, 256, 16, dtype=np.uint8)
        cc.cc_aes_both(p(key), p(pt), p(o4), p(o2))
        assert (o4 == o2).all()
