"""Seeded synthetic workloads shared by the tests, the oracle runs and bench.py.

This module holds shapes and random draws only: none of the garbling arithmetic.
The inputs stand in for the MNIST / CIFAR-10 images and trained weights of the paper's
evaluation (Sec. Model Benchmarks), which are not needed: the cost of garbling and of
evaluating a garbled network does not depend on the data.

Network format: a dict with
  primes, digits : CRT base and the mixed-radix digits of the sign gadget
  batch, n_in    : batch size, inputs per batch element
  x              : int64 [batch * n_in] input values (uniform uint8 range)
  layers         : list of dicts, executed in order; every layer has "kind" and "id"
     conv    : in_h in_w in_c out_c kh kw stride pad, W int32 [out_c][kh][kw][in_c], bias (opt.)
               (a dense layer K -> M is a conv with in_h = in_w = kh = kw = 1, in_c = K, out_c = M)
     sumpool : in_h in_w ch   (2x2 sum, stride 2)
     relu    : n (values per batch element)
     scale   : n, repeat      (repeat halvings = division by 2**repeat)
     sign    : n
Tensors of one batch element are ordered [y][x][channel].
"""
import numpy as np

PRIMES = [2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37]

# mixed-radix digits (d_1 most significant, even) with prod(d) >= k * P_k and k*d_j <= 255
DIGITS = {
    2: (2, 6),
    3: (2, 5, 9),
    4: (4, 15, 14),
    5: (2, 12, 25, 20),
    7: (10,) + (13,) * 5,
    8: (26, 12, 12, 12, 12, 12, 12),
    9: (22,) + (10,) * 8,
    12: (46,) + (17,) * 10,
}
# (7 and 9: the sets (d_1; d, .., d) with the fewest table bytes per sign gadget, found by exhaustive search)

# Reduced-accuracy sign (Appendix, Approximated Garbled Sign): fewer digits, prod(d) < k * P_k.  The k-term sum
# of fractions rounded up to 1/M overestimates by less than k/M, so the sign is wrong only for values whose
# fraction X/P lies within k/M below 1/2 or below 1: at most a share 2k/M of all values.
DIGITS_REDUCED = {
    8: (26, 12, 12),          # M = 3744: wrong for at most 0.43 % of the values, 27 gates per sign instead of 63
}


def rng(seed, stream=0):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def seed_bytes(seed):
    return bytes(rng(seed, 999).integers(0, 256, 16, dtype=np.uint8).tolist())


def _conv(lid, g, in_h, in_w, in_c, out_c, k, stride, pad, lo, hi, bias=False):
    L = dict(kind="conv", id=lid, in_h=in_h, in_w=in_w, in_c=in_c, out_c=out_c, kh=k, kw=k,
             stride=stride, pad=pad, W=g.integers(lo, hi + 1, (out_c, k, k, in_c)).astype(np.int32))
    if bias:
        L["bias"] = g.integers(lo * 16, hi * 16 + 1, out_c).astype(np.int32)
    L["out_h"] = (in_h + 2 * pad - k) // stride + 1
    L["out_w"] = (in_w + 2 * pad - k) // stride + 1
    L["n_out"] = L["out_h"] * L["out_w"] * out_c
    return L


def _dense(lid, g, K, M, lo, hi, bias=False):
    return _conv(lid, g, 1, 1, K, M, 1, 1, 0, lo, hi, bias)


class _Builder:
    def __init__(self, seed, k, batch, n_in, lo, hi, digits=None):
        self.g = rng(seed)
        self.net = dict(primes=PRIMES[:k], digits=list(digits or DIGITS[k]), batch=batch, n_in=n_in,
                        seed=seed_bytes(seed), layers=[])
        self.net["x"] = self.g.integers(0, 256, batch * n_in).astype(np.int64)
        self.lo, self.hi = lo, hi
        self.n = n_in

    def _add(self, L):
        self.net["layers"].append(L)

    def lid(self):
        return len(self.net["layers"]) + 1

    def conv(self, in_h, in_w, in_c, out_c, k, stride=1, pad=0, bias=False):
        assert in_h * in_w * in_c == self.n
        L = _conv(self.lid(), self.g, in_h, in_w, in_c, out_c, k, stride, pad, self.lo, self.hi, bias)
        self._add(L)
        self.n = L["n_out"]
        return L

    def dense(self, M, bias=False):
        L = _dense(self.lid(), self.g, self.n, M, self.lo, self.hi, bias)
        self._add(L)
        self.n = M

    def relu(self):
        self._add(dict(kind="relu", id=self.lid(), n=self.n))

    def sign(self):
        self._add(dict(kind="sign", id=self.lid(), n=self.n))

    def scale(self, repeat):
        self._add(dict(kind="scale", id=self.lid(), n=self.n, repeat=repeat))

    def sumpool(self, in_h, in_w, ch):
        assert in_h * in_w * ch == self.n
        self._add(dict(kind="sumpool", id=self.lid(), in_h=in_h, in_w=in_w, ch=ch))
        self.n = (in_h // 2) * (in_w // 2) * ch


def mlp(seed=1, batch=1, centered=False, k=8, n_in=784, hidden=128, n_out=10, repeat=6):
    """Config 1: dense 784->128, ReLU, scale 2^6, dense 128->10; weights in [-8,7].
    centered=True uses [-7,7] so that both ReLU branches occur (parity variant)."""
    b = _Builder(seed, k, batch, n_in, -7 if centered else -8, 7)
    b.dense(hidden)
    b.relu()
    b.scale(repeat)
    b.dense(n_out)
    return b.net


def lenet(seed=2, batch=16, centered=False, k=8, repeat=6):
    """Config 2: LeNet-5 shape on 1x28x28: conv5x5(6, pad 2) ReLU scale pool conv5x5(16) ReLU scale
    pool dense 400->120->84->10, ReLU + scale after every conv/dense but the last."""
    b = _Builder(seed, k, batch, 28 * 28, -7 if centered else -8, 7)
    b.conv(28, 28, 1, 6, 5, pad=2); b.relu(); b.scale(repeat); b.sumpool(28, 28, 6)
    b.conv(14, 14, 6, 16, 5); b.relu(); b.scale(repeat); b.sumpool(10, 10, 16)
    b.dense(120); b.relu(); b.scale(repeat)
    b.dense(84); b.relu(); b.scale(repeat)
    b.dense(10)
    return b.net


def vgg(seed=5, batch=64, centered=False, k=12, repeat=5, width=(64, 128, 256), hw=32):
    """Config 5: VGG-style CIFAR shape on 3x32x32, 3x3 convs pad 1, weights in [-16,15]."""
    b = _Builder(seed, k, batch, hw * hw * 3, -15 if centered else -16, 15)
    c_in, s = 3, hw
    for c_out in width:
        for _ in range(2):
            b.conv(s, s, c_in, c_out, 3, pad=1); b.relu(); b.scale(repeat)
            c_in = c_out
        b.sumpool(s, s, c_out)
        s //= 2
    b.dense(256); b.relu(); b.scale(repeat)
    b.dense(10)
    return b.net


def tiny(seed=7, k=3, batch=2, n_in=6, hidden=5, n_out=3, repeat=1, sign=False, bias=True, wmax=2):
    """A very small dense network for small CRT bases (exhaustive / fast oracle tests)."""
    b = _Builder(seed, k, batch, n_in, -wmax, wmax)
    b.net["x"] = b.g.integers(0, 4, batch * n_in).astype(np.int64)
    b.dense(hidden, bias=bias)
    if sign:
        b.sign()
    else:
        b.relu()
        if repeat:
            b.scale(repeat)
    b.dense(n_out, bias=bias)
    return b.net


def tiny_cnn(seed=8, k=4, batch=2, repeat=1):
    """Small conv net exercising padding, stride, pooling and flatten order."""
    b = _Builder(seed, k, batch, 6 * 6 * 2, -1, 1)
    b.net["x"] = b.g.integers(0, 3, batch * 72).astype(np.int64)
    b.conv(6, 6, 2, 3, 3, stride=1, pad=1, bias=True); b.relu(); b.sumpool(6, 6, 3)
    b.conv(3, 3, 3, 2, 2, stride=1, pad=0); b.relu()
    if repeat:
        b.scale(repeat)
    b.dense(3)
    return b.net


# Sec. Model architectures, the table of models: (in, out, filter, stride) convolutions without padding, R = ReLU,
# (a) = dense layer.  CRT bases per model as in the text; models f and F rescale by 2^5 after every ReLU.
PAPER_MODELS = {
    "A": dict(k=8, hw=28, c=1, scale=0, layers=[("d", 128), "R", ("d", 128), "R", ("d", 10)]),
    "B": dict(k=9, hw=28, c=1, scale=0, layers=[("c", 5, 5, 1), "R", ("c", 5, 3, 3), "R", ("c", 10, 3, 1), "R", ("c", 10, 3, 3), "R",
                                                  ("d", 100), "R", ("d", 10)]),
    "C": dict(k=9, hw=28, c=1, scale=0, layers=[("c", 5, 4, 2), "R", ("d", 100), "R", ("d", 10)]),
    "D": dict(k=8, hw=28, c=1, scale=0, layers=[("c", 16, 6, 2), "R", ("c", 16, 6, 2), "R", ("d", 100), "R", ("d", 10)]),
    "f": dict(k=7, hw=32, c=3, scale=5, layers=[("c", 32, 3, 1), "R", ("c", 32, 3, 1), "R", ("c", 32, 2, 2), ("c", 64, 3, 1), "R",
                                                  ("c", 64, 3, 1), "R", ("c", 64, 2, 2), ("c", 128, 3, 1), "R", ("c", 128, 3, 1), "R", ("d", 10)]),
    "F": dict(k=7, hw=32, c=3, scale=5, layers=[("c", 64, 3, 1), "R", ("c", 64, 3, 1), "R", ("c", 64, 2, 2), ("c", 64, 3, 1), "R",
                                                  ("c", 64, 3, 1), "R", ("c", 64, 2, 2), ("c", 64, 3, 1), "R", ("c", 64, 1, 1), "R",
                                                  ("c", 16, 1, 1), "R", ("d", 10)]),
}


def paper_model(name, seed=6, batch=1, centered=True):
    """The SHAPE of one of the paper's models A, B, C, D, f, F with random integer weights and biases (the trained
    weights are not available; run time does not depend on them)."""
    spec = PAPER_MODELS[name]
    hw, ch = spec["hw"], spec["c"]
    b = _Builder(seed, spec["k"], batch, hw * hw * ch, -7 if centered else -8, 7)
    h = w = hw
    for L in spec["layers"]:
        if L == "R":
            b.relu()
            if spec["scale"]:
                b.scale(spec["scale"])
        elif L[0] == "c":
            _, out_c, ks, stride = L
            b.conv(h, w, ch, out_c, ks, stride=stride, pad=0, bias=True)
            h, w, ch = (h - ks) // stride + 1, (w - ks) // stride + 1, out_c
        else:
            b.dense(L[1], bias=True)
            h = w = 1
            ch = L[1]
    return b.net


def proj_microbench(seed=3, n_gates=1 << 24, k=12):
    """Config 3: n independent unary gates Z_p -> Z_q with (p, q) uniform over the CRT base,
    a random function table per gate and a uniform input value per gate.
    Returns dict(pi, qi, a, phi) with phi [n][37] (entries beyond p unused, < q)."""
    g = rng(seed)
    pi = g.integers(0, k, n_gates).astype(np.int8)
    qi = g.integers(0, k, n_gates).astype(np.int8)
    pr = np.array(PRIMES[:k])
    u = g.integers(0, 1 << 30, n_gates)
    a = (u % pr[pi]).astype(np.uint8)
    return dict(pi=pi, qi=qi, a=a, seed=seed_bytes(seed), primes=PRIMES[:k], gen=g)


def proj_phi(g, n, p, q):
    """Random function tables [n][p] with values in Z_q."""
    return g.integers(0, q, (n, p)).astype(np.uint8)


def gemm_microbench(seed=4, M=4096, K=4096, batch=128, k=12, lo=-64, hi=63):
    """Config 4: dense M x K, weights uniform in [lo, hi]; label tensors are drawn by the caller
    with uniform_labels()."""
    g = rng(seed)
    return dict(W=g.integers(lo, hi + 1, (M, K)).astype(np.int32), M=M, K=K, batch=batch,
                primes=PRIMES[:k], seed=seed_bytes(seed), gen=g)


def uniform_labels(g, n, lam, p):
    """[n][lam] label components uniform in Z_p."""
    return g.integers(0, p, (n, lam)).astype(np.uint8)
