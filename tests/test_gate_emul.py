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
