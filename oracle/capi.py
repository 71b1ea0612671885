"""ctypes wrapper around oracle/dash_oracle.c -- TEST INFRASTRUCTURE ONLY.

Marshalling only: every number comes out of the C file.  Label tensors are numpy
uint8 arrays [elem][lambda_m]; tables are flat uint8 arrays in the layout documented
at the top of the C file.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dash_oracle.c")
_SO = os.path.join(_HERE, "libdash_oracle.so")
_lib = None

MAXLAM = 128


def build(force=False):
    """Compile the oracle with gcc (no GPU involved)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-shared", "-fPIC", "-o", _SO, _SRC])
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        _lib.orc_ctx_create.restype = C.c_void_p
        _lib.orc_relu_bytes_per_elem.restype = C.c_size_t
        _lib.orc_scale_bytes_per_elem.restype = C.c_size_t
        _lib.orc_signact_bytes_per_elem.restype = C.c_size_t
        _lib.orc_tables_packed_bytes.restype = C.c_size_t
        _lib.orc_hash_calls.restype = C.c_ulonglong
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _ptrs(arrs):
    return (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def hash_calls():
    """hash evaluations made by the calling thread so far (a garbler spends exactly one per ciphertext)"""
    return lib().orc_hash_calls()


def aes128_encrypt(key, block):
    out = np.zeros(16, np.uint8)
    lib().orc_aes128_encrypt(_p(_u8(key)), _p(_u8(block)), _p(out))
    return out


def lam(m, rule=0):
    return lib().orc_lambda(int(m), int(rule))


def pitch(lam_):
    return 4 * ((lam_ + 3) // 4)


def compress(label, q):
    label = _u8(label)
    out = np.zeros(16, np.uint8)
    lib().orc_compress(_p(label), len(label), int(q), _p(out))
    return int.from_bytes(out.tobytes(), "little")


def decompress(h, q, lam_):
    hb = np.frombuffer(int(h).to_bytes(16, "little"), np.uint8).copy()
    out = np.zeros(lam_, np.uint8)
    lib().orc_decompress(_p(hb), int(q), int(lam_), _p(out))
    return out


class Oracle:
    """One garbling context: CRT base, label-length rule, seed, mixed-radix digits."""

    def __init__(self, primes, digits, seed, rule=0, lam=None):
        self.primes = [int(p) for p in primes]
        self.k = len(self.primes)
        self.digits = [int(d) for d in digits]
        self.n = len(self.digits)
        self.rule = rule
        seed = _u8(np.frombuffer(bytes(seed), np.uint8))
        assert seed.size == 16
        pr = (C.c_int * self.k)(*self.primes)
        dg = (C.c_int * self.n)(*self.digits)
        self.L = lib()
        la = None if lam is None else (C.c_int * self.k)(*[int(v) for v in lam])
        self.h = C.c_void_p(self.L.orc_ctx_create(pr, self.k, rule, la, _p(seed), dg, self.n))
        assert self.h, "orc_ctx_create failed"
        self.P = 1
        for p in self.primes:
            self.P *= p
        self.M = 1
        for d in self.digits:
            self.M *= d

    def __del__(self):
        try:
            self.L.orc_ctx_free(self.h)
        except Exception:
            pass

    # -- context data -------------------------------------------------------
    def lam(self, m):
        return self.L.orc_ctx_lambda(self.h, int(m))

    def delta(self, m):
        out = np.zeros(self.lam(m), np.uint8)
        self.L.orc_ctx_delta(self.h, int(m), _p(out))
        return out

    def one0(self, i):
        out = np.zeros(self.lam(self.primes[i]), np.uint8)
        self.L.orc_ctx_one0(self.h, int(i), _p(out))
        return out

    def one(self, i):
        p = self.primes[i]
        return ((self.one0(i).astype(np.int64) + self.delta(p)) % p).astype(np.uint8)

    def mj(self, j):
        return self.L.orc_ctx_mj(self.h, int(j))

    def hash(self, label, p, layer, slot, elem, q):
        out = np.zeros(self.lam(q), np.uint8)
        self.L.orc_hash(self.h, _p(_u8(label)), int(p), int(layer), C.c_uint32(slot), C.c_uint64(elem), int(q), _p(out))
        return out

    def draw(self, domain, layer, slot, elem, m):
        out = np.zeros(self.lam(m), np.uint8)
        self.L.orc_draw(self.h, int(domain), int(layer), C.c_uint32(slot), C.c_uint64(elem), int(m), _p(out))
        return out

    def input_labels(self, first_wire, n, i):
        out = np.zeros((n, self.lam(self.primes[i])), np.uint8)
        self.L.orc_input_labels(self.h, C.c_uint64(first_wire), C.c_long(n), int(i), _p(out))
        return out

    # -- projection gates ---------------------------------------------------
    def proj_garble(self, p, q, in0, phi, layer, slot=0, elem_base=0):
        """in0 [n][lam_p]; phi [n][p] (per gate) or [p] (shared).  -> out0 [n][lam_q], table [n][p][pitch_q]"""
        in0 = _u8(in0)
        n = in0.shape[0]
        phi = _u8(phi)
        stride = p if phi.ndim == 2 else 0
        out0 = np.zeros((n, self.lam(q)), np.uint8)
        table = np.zeros((n, p, pitch(self.lam(q))), np.uint8)
        self.L.orc_proj_garble(self.h, int(p), int(q), C.c_long(n), C.c_uint64(elem_base), int(layer),
                               C.c_uint32(slot), _p(in0), _p(phi), C.c_long(stride), _p(out0), _p(table))
        return out0, table

    def proj_eval(self, p, q, act, table, layer, slot=0, elem_base=0):
        act = _u8(act)
        table = _u8(table)
        n = act.shape[0]
        out = np.zeros((n, self.lam(q)), np.uint8)
        self.L.orc_proj_eval(self.h, int(p), int(q), C.c_long(n), C.c_uint64(elem_base), int(layer),
                             C.c_uint32(slot), _p(act), _p(table), _p(out))
        return out

    # -- half gate (one gate; used by the brute-force pins) -------------------
    def hg_garble(self, p, x0, y0, layer, slotG, elem):
        lp = self.lam(p)
        z0 = np.zeros(lp, np.uint8)
        G = np.zeros((p, pitch(lp)), np.uint8)
        E = np.zeros((2, pitch(lp)), np.uint8)
        S = np.zeros((2, 4), np.uint8)
        self.L.orc_hg_garble(self.h, int(p), _p(_u8(x0)), _p(_u8(y0)), int(layer), C.c_uint32(slotG),
                             C.c_uint64(elem), _p(z0), _p(G), _p(E), _p(S))
        return z0, G, E, S

    def hg_eval(self, p, x, y, layer, slotG, elem, G, E, S):
        z = np.zeros(self.lam(p), np.uint8)
        self.L.orc_hg_eval(self.h, int(p), _p(_u8(x)), _p(_u8(y)), int(layer), C.c_uint32(slotG),
                           C.c_uint64(elem), _p(_u8(G)), _p(_u8(E)), _p(_u8(S)), _p(z))
        return z

    # -- sign gadget as a plain function --------------------------------------
    def sign_phi(self, i, j, x):
        return self.L.orc_sign_phi(self.h, int(i), int(j), int(x))

    def sign_plain(self, residues, first_res=0, negate=0):
        r = (C.c_int * self.k)(*[int(v) for v in residues])
        return self.L.orc_sign_plain(self.h, r, int(first_res), int(negate))

    def sign_nslots(self):
        return self.L.orc_sign_nslots(self.h)

    # -- activation layers ----------------------------------------------------
    def _bundle_out(self, n):
        return [np.zeros((n, self.lam(p)), np.uint8) for p in self.primes]

    def relu_bytes_per_elem(self):
        return self.L.orc_relu_bytes_per_elem(self.h)

    def scale_bytes_per_elem(self):
        return self.L.orc_scale_bytes_per_elem(self.h)

    def signact_bytes_per_elem(self):
        return self.L.orc_signact_bytes_per_elem(self.h)

    def relu_garble(self, layer, in0, elem_base=0, want_wires=False, zero_only=False):
        """zero_only: the output zero labels alone (no ciphertexts are computed) -> out0"""
        in0 = [_u8(a) for a in in0]
        n = in0[0].shape[0]
        out0 = self._bundle_out(n)
        if zero_only:
            self.L.orc_relu_garble(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), _ptrs(in0), _ptrs(out0), None, None)
            return out0
        tables = np.zeros(n * self.relu_bytes_per_elem(), np.uint8)
        wires = np.zeros((n, self.sign_nslots(), MAXLAM), np.uint8) if want_wires else None
        self.L.orc_relu_garble(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), _ptrs(in0), _ptrs(out0),
                               _p(tables), _p(wires) if want_wires else None)
        return (out0, tables, wires) if want_wires else (out0, tables)

    def relu_eval(self, layer, act, tables, elem_base=0, want_wires=False):
        act = [_u8(a) for a in act]
        tables = _u8(tables)
        n = act[0].shape[0]
        out = self._bundle_out(n)
        wires = np.zeros((n, self.sign_nslots(), MAXLAM), np.uint8) if want_wires else None
        self.L.orc_relu_eval(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), _ptrs(act), _p(tables),
                             _ptrs(out), _p(wires) if want_wires else None)
        return (out, wires) if want_wires else out

    def scale_garble(self, layer, in0, repeat, elem_base=0, zero_only=False):
        """zero_only: the output zero labels alone (no ciphertexts are computed) -> out0"""
        in0 = [_u8(a) for a in in0]
        n = in0[0].shape[0]
        out0 = self._bundle_out(n)
        if zero_only:
            self.L.orc_scale_garble(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), int(repeat), _ptrs(in0), None,
                                    _ptrs(out0))
            return out0
        tables = np.zeros(n * repeat * self.scale_bytes_per_elem(), np.uint8)
        self.L.orc_scale_garble(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), int(repeat), _ptrs(in0),
                                _p(tables), _ptrs(out0))
        return out0, tables

    def scale_eval(self, layer, act, tables, repeat, elem_base=0):
        act = [_u8(a) for a in act]
        tables = _u8(tables)
        n = act[0].shape[0]
        out = self._bundle_out(n)
        self.L.orc_scale_eval(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), int(repeat), _ptrs(act),
                              _p(tables), _ptrs(out))
        return out

    def signact_garble(self, layer, in0, elem_base=0):
        in0 = [_u8(a) for a in in0]
        n = in0[0].shape[0]
        out0 = self._bundle_out(n)
        tables = np.zeros(n * self.signact_bytes_per_elem(), np.uint8)
        self.L.orc_signact_garble(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), _ptrs(in0), _p(tables),
                                  _ptrs(out0))
        return out0, tables

    def signact_eval(self, layer, act, tables, elem_base=0):
        act = [_u8(a) for a in act]
        tables = _u8(tables)
        n = act[0].shape[0]
        out = self._bundle_out(n)
        self.L.orc_signact_eval(self.h, int(layer), C.c_uint64(elem_base), C.c_long(n), _ptrs(act), _p(tables),
                                _ptrs(out))
        return out

    # -- packed storage format of the tables ----------------------------------------
    KIND = dict(relu=4, scale=5, sign=6, proj=7)

    def tables_packed_bytes(self, kind, n, repeat=1, p=0, q=0):
        return self.L.orc_tables_packed_bytes(self.h, self.KIND[kind], C.c_long(n), int(repeat), int(p), int(q))

    def tables_pack(self, kind, n, tables, repeat=1, p=0, q=0):
        """tables of a layer over n elements (working format) -> packed format (uint8 array)"""
        tables = _u8(tables).copy()
        out = np.zeros(self.tables_packed_bytes(kind, n, repeat, p, q), np.uint8)
        ok = self.L.orc_tables_repack(self.h, self.KIND[kind], C.c_long(n), int(repeat), int(p), int(q), 1, _p(tables), _p(out))
        assert ok, "packed format not defined for these label lengths"
        return out

    def tables_unpack(self, kind, n, packed, nbytes, repeat=1, p=0, q=0):
        packed = _u8(packed).copy()
        out = np.full(nbytes, 0xEE, np.uint8)
        ok = self.L.orc_tables_repack(self.h, self.KIND[kind], C.c_long(n), int(repeat), int(p), int(q), 0, _p(out), _p(packed))
        assert ok
        return out

    # -- linear layers ----------------------------------------------------------
    def conv2d(self, i, x, batch, in_h, in_w, in_c, out_c, kh, kw, stride, pad, W, bias=None, one=None):
        """x [batch*in_h*in_w*in_c][lam]; W int32 [out_c][kh][kw][in_c].  one: constant-wire label for the bias."""
        x = _u8(x)
        W = np.ascontiguousarray(W, dtype=np.int32)
        oh = (in_h + 2 * pad - kh) // stride + 1
        ow = (in_w + 2 * pad - kw) // stride + 1
        out = np.zeros((batch * oh * ow * out_c, x.shape[1]), np.uint8)
        b = np.ascontiguousarray(bias, dtype=np.int32) if bias is not None else None
        o = _u8(one) if bias is not None else None
        self.L.orc_conv2d(self.h, int(i), C.c_long(batch), in_h, in_w, in_c, out_c, kh, kw, stride, pad, _p(W),
                          _p(b) if b is not None else None, _p(o) if o is not None else None, _p(x), _p(out))
        return out

    def dense(self, i, x, batch, K, M, W, bias=None, one=None):
        return self.conv2d(i, x, batch, 1, 1, K, M, 1, 1, 1, 0, np.asarray(W).reshape(M, 1, 1, K), bias, one)

    def sumpool2(self, i, x, batch, in_h, in_w, ch):
        x = _u8(x)
        out = np.zeros((batch * (in_h // 2) * (in_w // 2) * ch, x.shape[1]), np.uint8)
        self.L.orc_sumpool2(self.h, int(i), C.c_long(batch), in_h, in_w, ch, _p(x), _p(out))
        return out

    # -- En / De ------------------------------------------------------------------
    def encode(self, i, values, zero):
        values = np.ascontiguousarray(values, dtype=np.int64)
        zero = _u8(zero)
        out = np.zeros_like(zero)
        self.L.orc_encode(self.h, int(i), C.c_long(len(values)), _p(values), _p(zero), _p(out))
        return out

    def decode(self, act, zero):
        act = [_u8(a) for a in act]
        zero = [_u8(a) for a in zero]
        n = act[0].shape[0]
        values = np.zeros(n, np.int64)
        valid = np.zeros(n, np.uint8)
        self.L.orc_decode(self.h, C.c_long(n), _ptrs(act), _ptrs(zero), _p(values), _p(valid))
        return values, valid
