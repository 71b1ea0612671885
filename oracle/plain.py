"""Plain integer definitions of what the garbled layers compute -- TEST INFRASTRUCTURE ONLY.

Everything here works on ordinary integers in the ring Z_P (P = product of the CRT
primes, P even), with no labels, residues or gadgets: it is the definition the
decoded output of a garbled network must equal.

  Sec. Quantization and Encoding : Encode(x) = x mod P, negatives in the upper half
  Sec. Arithmetic Garbled Circuits (Sign Gadget) : ReLU(a) = a * sgn_{0,1}(a)
  Sec. The Scaling Operation, High-Level Steps : ShiftUp, Scale, ShiftDown
"""
import numpy as np


def to_ring(x, P):
    return np.mod(np.asarray(x, dtype=np.int64), P)


def to_signed(X, P):
    """Upper half of the ring (X >= P/2) holds the negative numbers."""
    X = np.asarray(X, dtype=np.int64)
    return np.where(2 * X >= P, X - P, X)


def relu(X, P):
    """X for the lower half (zero included), 0 for the upper half."""
    X = np.asarray(X, dtype=np.int64)
    return np.where(2 * X >= P, 0, X)


def sign_act(X, P):
    """sgn_{-1,1}: +1 on the lower half, -1 (= P-1) on the upper half."""
    X = np.asarray(X, dtype=np.int64)
    return np.where(2 * X >= P, P - 1, 1)


def scale2(X, P):
    """ShiftDown(Scale(ShiftUp(X))): ((X + P/2) mod P) div 2 - floor(P/4)  (mod P)."""
    X = np.asarray(X, dtype=np.int64)
    up = np.mod(X + P // 2, P)
    return np.mod(up // 2 - P // 4, P)


def scale(X, P, repeat):
    for _ in range(repeat):
        X = scale2(X, P)
    return X


def conv2d(X, P, batch, in_h, in_w, in_c, out_c, kh, kw, stride, pad, W, bias=None):
    """X [batch][in_h][in_w][in_c] ring values; W int [out_c][kh][kw][in_c]; -> [batch][oh][ow][out_c]."""
    X = np.asarray(X, dtype=np.int64).reshape(batch, in_h, in_w, in_c)
    W = np.asarray(W, dtype=np.int64).reshape(out_c, kh, kw, in_c)
    oh = (in_h + 2 * pad - kh) // stride + 1
    ow = (in_w + 2 * pad - kw) // stride + 1
    Xp = np.zeros((batch, in_h + 2 * pad, in_w + 2 * pad, in_c), np.int64)
    Xp[:, pad:pad + in_h, pad:pad + in_w, :] = X
    out = np.zeros((batch, oh, ow, out_c), np.int64)
    # |W| small, X < 2^43: reduce mod P after every kernel tap so int64 never overflows
    assert np.abs(W).max(initial=0) < 2 ** 15 and P < 2 ** 44
    for ky in range(kh):
        for kx in range(kw):
            patch = Xp[:, ky:ky + stride * oh:stride, kx:kx + stride * ow:stride, :]  # [b][oh][ow][ci]
            # in_c up to 4096 terms of < 2^58 would overflow: split the channel sum
            for c0 in range(0, in_c, 16):
                out += np.mod(np.einsum("bhwc,oc->bhwo", patch[..., c0:c0 + 16], W[:, ky, kx, c0:c0 + 16]), P)
                out = np.mod(out, P)
    if bias is not None:
        out = np.mod(out + np.asarray(bias, dtype=np.int64).reshape(1, 1, 1, out_c), P)
    return out.reshape(-1)


def dense(X, P, batch, K, M, W, bias=None):
    return conv2d(X, P, batch, 1, 1, K, M, 1, 1, 1, 0, np.asarray(W).reshape(M, 1, 1, K), bias)


def sumpool2(X, P, batch, in_h, in_w, ch):
    X = np.asarray(X, dtype=np.int64).reshape(batch, in_h // 2, 2, in_w // 2, 2, ch)
    return np.mod(X.sum(axis=(2, 4)), P).reshape(-1)


def run_network(layers, x, P, batch):
    """Evaluate a layer list (see workloads.py for the format) on ring values; returns the
    value on every layer boundary (list, entry 0 = the encoded input)."""
    vals = [to_ring(x, P).reshape(-1)]
    for L in layers:
        X = vals[-1]
        kind = L["kind"]
        if kind == "conv":
            Y = conv2d(X, P, batch, L["in_h"], L["in_w"], L["in_c"], L["out_c"], L["kh"], L["kw"],
                       L["stride"], L["pad"], L["W"], L.get("bias"))
        elif kind == "sumpool":
            Y = sumpool2(X, P, batch, L["in_h"], L["in_w"], L["ch"])
        elif kind == "relu":
            Y = relu(X, P)
        elif kind == "scale":
            Y = scale(X, P, L["repeat"])
        elif kind == "sign":
            Y = sign_act(X, P)
        else:
            raise ValueError(kind)
        vals.append(np.asarray(Y, dtype=np.int64).reshape(-1))
    return vals
