"""ctypes binding of include/dash.h: same names, argument marshalling only.

torch is used for device memory (torch.empty(device="cuda")) and for the current HIP stream; no
arithmetic of the method happens here.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libdash.so")

MAX_PRIMES = 16
MAX_DIGITS = 16
DENSE, CONV2D, SUMPOOL, RELU, SCALE, SIGN, PROJ = 1, 2, 3, 4, 5, 6, 7
LAMBDA_CEIL, LAMBDA_FLOOR = 0, 1
NOALLOC_SCRATCH_BYTES = 32 << 20

SYMBOLS = ["dash_ctx_create", "dash_ctx_destroy", "dash_lambda", "dash_ctx_offset", "dash_ctx_one", "dash_ctx_digits",
           "dash_layer_sizes", "dash_weights_bytes", "dash_weights_prepare", "dash_garble_layer", "dash_eval_layer",
           "dash_garble_layers", "dash_eval_layers", "dash_eval_layer_noalloc", "dash_input_labels", "dash_encode", "dash_decode", "dash_labels_pack", "dash_labels_unpack", "dash_tables_packed_bytes", "dash_tables_pack", "dash_tables_unpack", "dash_strerror", "dash_profile_enable", "dash_profile_read", "dash_profile_aes"]


class DashError(RuntimeError):
    pass


class CLabels(C.Structure):
    _fields_ = [("data", C.c_void_p * MAX_PRIMES), ("chunk_stride", C.c_int64 * MAX_PRIMES), ("n_elem", C.c_int64)]


class CLayer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("layer_id", C.c_int32), ("elem_base", C.c_int64), ("n_elem", C.c_int64),
                ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32), ("out_c", C.c_int32),
                ("kh", C.c_int32), ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32),
                ("weights", C.c_void_p), ("bias", C.c_void_p), ("repeat", C.c_int32),
                ("p_index", C.c_int32), ("q_index", C.c_int32), ("phi", C.c_void_p), ("phi_stride", C.c_int64)]


_lib = None


def lib_path():
    return _SO


def lib():
    """Load libdash.so; fail loudly if it has not been built (python -m paper_2302_06361_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise DashError("libdash.so is missing: build it with `python -m paper_2302_06361_amd.build` "
                            "(there is no CPU fallback)")
        L = C.CDLL(_SO)
        L.dash_strerror.restype = C.c_char_p
        L.dash_weights_bytes.restype = C.c_size_t
        L.dash_tables_packed_bytes.restype = C.c_size_t
        L.dash_ctx_destroy.restype = None
        _lib = L
    return _lib


def _check(st, what):
    if st != 0:
        raise DashError("%s: %s (%d)" % (what, lib().dash_strerror(st).decode(), st))


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Labels:
    """One LabelTensor per CRT residue on the GPU: tensors[i] is uint8 [nchunk_i][n_elem][16]."""

    def __init__(self, ctx, n_elem, only=None, zero=False):
        import torch
        self.ctx, self.n_elem = ctx, int(n_elem)
        self.tensors = [None] * ctx.k
        for i, p in enumerate(ctx.primes):
            if only is not None and i not in only:
                continue
            nch = (ctx.lam(p) + 15) // 16
            shape = (nch, max(self.n_elem, 1), 16)
            self.tensors[i] = (torch.zeros if zero else torch.empty)(shape, dtype=torch.uint8, device=ctx.device)

    def c(self):
        s = CLabels()
        s.n_elem = self.n_elem
        for i, t in enumerate(self.tensors):
            if t is not None:
                s.data[i] = t.data_ptr()
                s.chunk_stride[i] = t.stride(0)
        return s

    def slice(self, e0, e1):
        """View of the elements [e0, e1) (same storage)."""
        v = Labels.__new__(Labels)
        v.ctx, v.n_elem = self.ctx, e1 - e0
        v.tensors = [None if t is None else t[:, e0:e1, :] for t in self.tensors]
        return v

    def to_numpy(self, i):
        """Compact host copy [n_elem][lambda] of residue i (layout conversion only)."""
        lam = self.ctx.lam(self.ctx.primes[i])
        t = self.tensors[i][:, :self.n_elem, :].permute(1, 0, 2).reshape(self.n_elem, -1)
        return t[:, :lam].contiguous().cpu().numpy()

    def pad_is_zero(self, i):
        lam = self.ctx.lam(self.ctx.primes[i])
        t = self.tensors[i][:, :self.n_elem, :].permute(1, 0, 2).reshape(self.n_elem, -1)
        return bool((t[:, lam:] == 0).all().item())

    def from_numpy(self, i, arr):
        """Upload compact labels [n_elem][lambda] into residue i (layout conversion only)."""
        import torch
        lam = self.ctx.lam(self.ctx.primes[i])
        nch = (lam + 15) // 16
        a = np.zeros((self.n_elem, nch * 16), np.uint8)
        a[:, :lam] = arr
        t = torch.from_numpy(a).to(self.ctx.device).reshape(self.n_elem, nch, 16).permute(1, 0, 2)
        self.tensors[i][:, :self.n_elem, :].copy_(t)


class Layer:
    """A dash_layer descriptor plus the Python objects that keep its device buffers alive."""

    def __init__(self, kind, layer_id=0, n_elem=0, elem_base=0, **kw):
        self.c = CLayer()
        self.c.kind, self.c.layer_id, self.c.n_elem, self.c.elem_base = kind, layer_id, n_elem, elem_base
        self.keep = []
        for k, v in kw.items():
            if k in ("weights", "bias", "phi"):
                if v is not None:
                    self.keep.append(v)
                    setattr(self.c, k, v.data_ptr())
            else:
                setattr(self.c, k, v)


class Context:
    def __init__(self, primes, seed, digits=None, rule=LAMBDA_CEIL, device=0, lam=None):
        import torch
        if not torch.cuda.is_available():
            raise DashError("no GPU visible: libdash has no CPU path")
        self.L = lib()
        self.primes = [int(p) for p in primes]
        self.k = len(self.primes)
        self.device = torch.device("cuda", device)
        pr = (C.c_uint16 * self.k)(*self.primes)
        sd = (C.c_uint8 * 16)(*bytes(seed))
        h = C.c_void_p()
        la = None if lam is None else (C.c_uint16 * self.k)(*[int(v) for v in lam])
        dg = None if digits is None else (C.c_uint16 * len(digits))(*[int(d) for d in digits])
        st = self.L.dash_ctx_create(C.byref(h), pr, self.k, rule, la, sd, dg, 0 if digits is None else len(digits), device)
        _check(st, "dash_ctx_create")
        self.h = h
        buf = (C.c_uint16 * MAX_DIGITS)()
        n = self.L.dash_ctx_digits(self.h, buf)
        self.digits = [int(buf[j]) for j in range(n)]
        self._lam = {}

    def close(self):
        if getattr(self, "h", None):
            self.L.dash_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def lam(self, m):
        if m not in self._lam:
            self._lam[m] = self.L.dash_lambda(self.h, int(m))
        return self._lam[m]

    def pitch(self, m):
        return 4 * ((self.lam(m) + 3) // 4)

    def offset(self, m):
        out = np.zeros(self.lam(m), np.uint8)
        _check(self.L.dash_ctx_offset(self.h, int(m), out.ctypes.data_as(C.c_void_p)), "dash_ctx_offset")
        return out

    def one(self, i, which):
        out = np.zeros(self.lam(self.primes[i]), np.uint8)
        _check(self.L.dash_ctx_one(self.h, int(i), int(which), out.ctypes.data_as(C.c_void_p)), "dash_ctx_one")
        return out

    def profile_enable(self, on):
        _check(self.L.dash_profile_enable(self.h, int(on)), "dash_profile_enable")

    def profile_read(self, kind):
        """-> dict(ms, launches, units, bytes) summed over the launches since the last read"""
        ms, n, u, b = C.c_double(), C.c_int64(), C.c_double(), C.c_double()
        _check(self.L.dash_profile_read(self.h, int(kind), C.byref(ms), C.byref(n), C.byref(u), C.byref(b)), "dash_profile_read")
        return dict(ms=ms.value, launches=n.value, units=u.value, bytes=b.value)

    def profile_aes(self, variant, key, blocks_in, blocks_out, repeat=1):
        """AES-128 alone (variant 0: 4 KB tables, 1: bank-replicated tables T0/T1, 2: bit planes, 3: bank-replicated T0..T3) on device byte tensors
        [n][16]; out = AES_key^repeat(in)"""
        import torch
        key = bytes(key)
        assert len(key) == 16 and blocks_in.dtype == torch.uint8 and blocks_out.dtype == torch.uint8
        assert blocks_in.is_cuda and blocks_out.is_cuda and blocks_in.is_contiguous() and blocks_out.is_contiguous()
        assert blocks_in.numel() % 16 == 0 and blocks_out.numel() == blocks_in.numel()
        kb = (C.c_uint8 * 16).from_buffer_copy(key)
        _check(self.L.dash_profile_aes(self.h, int(variant), kb, C.c_void_p(blocks_in.data_ptr()), C.c_void_p(blocks_out.data_ptr()),
                                       C.c_uint64(blocks_in.numel() // 16), int(repeat), _stream()), "dash_profile_aes")

    # ---- the ABI calls, same names -------------------------------------------------------------
    def layer_sizes(self, layer):
        oe, tb, sb = C.c_int64(), C.c_size_t(), C.c_size_t()
        _check(self.L.dash_layer_sizes(self.h, C.byref(layer.c), C.byref(oe), C.byref(tb), C.byref(sb)), "dash_layer_sizes")
        return oe.value, tb.value, sb.value

    def weights_prepare(self, w):
        """w: int32 array/tensor [out_c][K] -> prepared device buffer (torch uint8)."""
        import torch
        wt = torch.as_tensor(np.ascontiguousarray(w, dtype=np.int32)).to(self.device)
        out_c, K = wt.shape
        nbytes = self.L.dash_weights_bytes(self.h, out_c, K)
        buf = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        _check(self.L.dash_weights_prepare(self.h, C.c_void_p(wt.data_ptr()), out_c, K, C.c_void_p(buf.data_ptr()), _stream()),
               "dash_weights_prepare")
        torch.cuda.current_stream().synchronize()     # wt may be freed after return
        return buf

    def input_labels(self, first_wire, zero, n=None):
        """zero labels of the input wires first_wire .. first_wire + n - 1 (n: all elements of `zero` by default)"""
        cz = zero.c()
        n = cz.n_elem if n is None else n
        _check(self.L.dash_input_labels(self.h, C.c_int64(first_wire), C.c_int64(n), C.byref(cz), _stream()), "dash_input_labels")

    def encode(self, values, zero, out):
        cz, co = zero.c(), out.c()
        _check(self.L.dash_encode(self.h, C.c_void_p(values.data_ptr()), C.c_int64(values.numel()), C.byref(cz), C.byref(co),
                                  _stream()), "dash_encode")

    def decode(self, act, zero, values, valid):
        ca, cz = act.c(), zero.c()
        _check(self.L.dash_decode(self.h, C.byref(ca), C.byref(cz), C.c_int64(values.numel()), C.c_void_p(values.data_ptr()),
                                  C.c_void_p(valid.data_ptr()), _stream()), "dash_decode")

    def labels_pack(self, labels, packed):
        """labels -> packed (uint8 tensor [k][n][16]): the 128-bit wire format; floor-rule contexts only"""
        cl = labels.c()
        _check(self.L.dash_labels_pack(self.h, C.byref(cl), C.c_int64(labels.n_elem), C.c_void_p(packed.data_ptr()), _stream()),
               "dash_labels_pack")

    def labels_unpack(self, packed, labels):
        cl = labels.c()
        _check(self.L.dash_labels_unpack(self.h, C.c_void_p(packed.data_ptr()), C.c_int64(labels.n_elem), C.byref(cl), _stream()),
               "dash_labels_unpack")

    def tables_packed_bytes(self, layer):
        """bytes of the layer's tables in the packed storage format (0: not available under this context's label lengths)"""
        return self.L.dash_tables_packed_bytes(self.h, C.byref(layer.c))

    def tables_pack(self, layer, tables, packed):
        _check(self.L.dash_tables_pack(self.h, C.byref(layer.c), C.c_void_p(tables.data_ptr()), C.c_void_p(packed.data_ptr()), _stream()),
               "dash_tables_pack")

    def tables_unpack(self, layer, packed, tables):
        _check(self.L.dash_tables_unpack(self.h, C.byref(layer.c), C.c_void_p(packed.data_ptr()), C.c_void_p(tables.data_ptr()), _stream()),
               "dash_tables_unpack")

    def garble_layer(self, layer, in_zero, out_zero, tables=None, scratch=None):
        ci, co = in_zero.c(), out_zero.c()
        _check(self.L.dash_garble_layer(self.h, C.byref(layer.c), C.byref(ci), C.byref(co),
                                        C.c_void_p(tables.data_ptr() if tables is not None else 0),
                                        C.c_void_p(scratch.data_ptr() if scratch is not None else 0), _stream()),
               "dash_garble_layer")

    def _layer_lists(self, layers, ins, outs, tables, scratch):
        n = len(layers)
        cl = (CLayer * n)(*[l.c for l in layers])
        ci = (CLabels * n)(*[t.c() for t in ins])
        co = (CLabels * n)(*[t.c() for t in outs])
        ct = (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in tables])
        cs = None if scratch is None else (C.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in scratch])
        return n, cl, ci, co, ct, cs

    def garble_layers(self, layers, in_zero, out_zero, tables, scratch=None):
        """n independent layer calls in one ABI call (lists of equal length)"""
        n, cl, ci, co, ct, cs = self._layer_lists(layers, in_zero, out_zero, tables, scratch)
        _check(self.L.dash_garble_layers(self.h, n, cl, ci, co, ct, cs, _stream()), "dash_garble_layers")

    def eval_layers(self, layers, in_act, tables, out_act, scratch=None):
        n, cl, ci, co, ct, cs = self._layer_lists(layers, in_act, out_act, tables, scratch)
        _check(self.L.dash_eval_layers(self.h, n, cl, ci, ct, co, cs, _stream()), "dash_eval_layers")

    def eval_layer_noalloc(self, layer, in_act, tables, out_act):
        """dash_eval_layer with the library's own fixed scratch array (NOALLOC_SCRATCH_BYTES): allocates nothing"""
        ci, co = in_act.c(), out_act.c()
        _check(self.L.dash_eval_layer_noalloc(self.h, C.byref(layer.c), C.byref(ci),
                                              C.c_void_p(tables.data_ptr() if tables is not None else 0), C.byref(co), _stream()),
               "dash_eval_layer_noalloc")

    def eval_layer(self, layer, in_act, tables, out_act, scratch=None):
        ci, co = in_act.c(), out_act.c()
        _check(self.L.dash_eval_layer(self.h, C.byref(layer.c), C.byref(ci),
                                      C.c_void_p(tables.data_ptr() if tables is not None else 0), C.byref(co),
                                      C.c_void_p(scratch.data_ptr() if scratch is not None else 0), _stream()),
               "dash_eval_layer")
