"""Oracle values for a SAMPLE of the wires of a network that is too large for the oracle to garble whole.

Everything here comes from the seeds, the weights and the oracle (oracle/): nothing the GPU computed is read.
What makes single wires computable alone (Sec. Arithmetic Garbled Circuits; Appendix, half gates):
  * fresh zero labels come from the counter-based PRG, addressed by (layer, slot, element), so the zero label
    of any wire depends only on the zero labels of the wires in its receptive field, never on a ciphertext:
    the oracle's garblers are run in their zero-labels-only mode (no tables) over that receptive field;
  * the active label of a wire is En of its plain value on that zero label (the label invariant
    active = zero + value * R_p, which the CPU tests pin on every boundary of whole networks): the oracle's
    own encode is applied to the plain evaluation (oracle/plain.py) of the same network.
For the sampled values themselves the oracle then garbles and evaluates the activation layer in full:
zero labels, every ciphertext row and the evaluated labels.

Index bookkeeping only; all arithmetic is in oracle/.
"""
import numpy as np

from oracle import plain
from oracle import net as onet


def _runs(idx):
    """sorted unique indices -> list of (start, count) of consecutive runs"""
    idx = np.asarray(idx, dtype=np.int64)
    if idx.size == 0:
        return []
    cut = np.flatnonzero(np.diff(idx) != 1) + 1
    starts = np.concatenate([[0], cut])
    ends = np.concatenate([cut, [idx.size]])
    return [(int(idx[s]), int(e - s)) for s, e in zip(starts, ends)]


class SampledOracle:
    """net: a workloads.py network; b: the batch element whose wires are sampled."""

    def __init__(self, net, b):
        self.net, self.b = net, b
        self.orc = onet.make_oracle(net)
        self.layers = net["layers"]
        self.P = int(np.prod(net["primes"], dtype=object))
        n_in = net["n_in"]
        x = np.asarray(net["x"][b * n_in:(b + 1) * n_in])
        self.pv = plain.run_network(self.layers, x, self.P, 1)     # ring values on every boundary of element b
        self.n = [len(v) for v in self.pv]                         # values per batch element on every boundary
        self.ones0 = [self.orc.one0(i) for i in range(self.orc.k)]
        self.memo = {}

    # ---- zero labels of arbitrary wires -----------------------------------------------------------
    def zero_at(self, boundary, idx):
        """zero labels of the values idx (any order, may repeat) on `boundary` (0 = network input) of batch
        element b -> bundle: per residue [len(idx)][lambda]"""
        idx = np.asarray(idx, dtype=np.int64)
        uniq = np.unique(idx)
        key = boundary
        have = self.memo.setdefault(key, {})
        todo = np.array([e for e in uniq.tolist() if e not in have], dtype=np.int64)
        if todo.size:
            got = self._compute(boundary, todo)
            for j, e in enumerate(todo.tolist()):
                have[e] = [g[j] for g in got]
        return [np.stack([have[e][i] for e in idx.tolist()]) for i in range(self.orc.k)]

    def _by_runs(self, todo, fn):
        """fn(start, count) -> bundle for consecutive elements; concatenated over the runs of todo (sorted unique)"""
        parts = [fn(s, c) for s, c in _runs(todo)]
        return [np.concatenate([p[i] for p in parts]) for i in range(self.orc.k)]

    def _compute(self, boundary, todo):
        orc, b = self.orc, self.b
        if boundary == 0:
            n_in = self.net["n_in"]
            return self._by_runs(todo, lambda s, c: [orc.input_labels(b * n_in + s, c, i) for i in range(orc.k)])
        L = self.layers[boundary - 1]
        kind = L["kind"]
        if kind == "relu":
            # the product wire's zero label is drawn (Appendix, half gate): it does not depend on the input wire
            def f(s, c):
                dummy = [np.zeros((c, orc.lam(p)), np.uint8) for p in orc.primes]
                return orc.relu_garble(L["id"], dummy, elem_base=b * L["n"] + s, zero_only=True)
            return self._by_runs(todo, f)
        if kind == "scale":
            def f(s, c):
                in0 = self.zero_at(boundary - 1, np.arange(s, s + c))
                return orc.scale_garble(L["id"], in0, L["repeat"], elem_base=b * L["n"] + s, zero_only=True)
            return self._by_runs(todo, f)
        if kind == "sumpool":
            in_h, in_w, ch = L["in_h"], L["in_w"], L["ch"]
            ow = in_w // 2
            c_ = todo % ch
            ox = (todo // ch) % ow
            oy = todo // (ch * ow)
            src = np.stack([((2 * oy + dy) * in_w + 2 * ox + dx) * ch + c_ for dy in range(2) for dx in range(2)], axis=1)
            x = self.zero_at(boundary - 1, src.reshape(-1))       # [len(todo) * 4]: one 2 x 2 x 1 image per value
            return [orc.sumpool2(i, x[i], len(todo), 2, 2, 1) for i in range(orc.k)]
        if kind == "conv":
            in_h, in_w, in_c, out_c = L["in_h"], L["in_w"], L["in_c"], L["out_c"]
            kh, kw, st, pad = L["kh"], L["kw"], L["stride"], L["pad"]
            ow = L["out_w"]
            co = todo % out_c
            pix = todo // out_c
            out = [np.zeros((len(todo), orc.lam(p)), np.uint8) for p in orc.primes]
            W = np.asarray(L["W"]).reshape(out_c, kh, kw, in_c)
            for px in np.unique(pix).tolist():
                sel = np.flatnonzero(pix == px)
                oy, ox = divmod(px, ow)
                # the kh x kw x in_c patch under this output pixel; taps outside the image contribute nothing
                # (an all-zero label times any weight adds nothing)
                src, inside = [], []
                for ky in range(kh):
                    for kx in range(kw):
                        iy, ix = oy * st + ky - pad, ox * st + kx - pad
                        ok = 0 <= iy < in_h and 0 <= ix < in_w
                        inside.append(ok)
                        if ok:
                            src.append((iy * in_w + ix) * in_c + np.arange(in_c))
                z = self.zero_at(boundary - 1, np.concatenate(src))
                bias = None if L.get("bias") is None else np.asarray(L["bias"])[co[sel]]
                for i, p in enumerate(orc.primes):
                    patch = np.zeros((kh * kw, in_c, orc.lam(p)), np.uint8)
                    patch[np.array(inside)] = z[i].reshape(-1, in_c, orc.lam(p))
                    out[i][sel] = orc.conv2d(i, patch.reshape(kh * kw * in_c, -1), 1, kh, kw, in_c, len(sel), kh, kw, 1, 0,
                                             W[co[sel]], bias, self.ones0[i])
            return out
        raise ValueError(kind)

    # ---- one activation layer on a run of consecutive values ----------------------------------------
    def activation(self, li, start, count):
        """Layer li (relu / scale / sign) on the values start .. start+count-1 of batch element b, garbled and
        evaluated by the oracle -> dict(zero_in, act_in, zero_out, act_out, tables) (tables in the oracle's layout
        for `count` elements)."""
        orc, L = self.orc, self.layers[li]
        idx = np.arange(start, start + count)
        zin = self.zero_at(li, idx)
        ain = [orc.encode(i, self.pv[li][idx], zin[i]) for i in range(orc.k)]
        eb = self.b * L["n"] + start
        if L["kind"] == "relu":
            zout, tab = orc.relu_garble(L["id"], zin, elem_base=eb)
            aout = orc.relu_eval(L["id"], ain, tab, elem_base=eb)
        elif L["kind"] == "scale":
            zout, tab = orc.scale_garble(L["id"], zin, L["repeat"], elem_base=eb)
            aout = orc.scale_eval(L["id"], ain, tab, L["repeat"], elem_base=eb)
        elif L["kind"] == "sign":
            zout, tab = orc.signact_garble(L["id"], zin, elem_base=eb)
            aout = orc.signact_eval(L["id"], ain, tab, elem_base=eb)
        else:
            raise ValueError(L["kind"])
        # the evaluated labels must carry the plain values of the next boundary (the invariant, on the oracle's side)
        vals, valid = orc.decode(aout, zout)
        assert valid.all() and (vals == plain.to_signed(self.pv[li + 1][idx], self.P)).all()
        return dict(zero_in=zin, act_in=ain, zero_out=zout, act_out=aout, tables=tab)


def segment_sizes(orc, kind, repeat=1):
    """bytes per element of every table segment of an activation layer, in slot order (the table format:
    segment = [gate][row][pitch], rows = input modulus, pitch = 4 * ceil(lambda_out / 4))"""
    k, n = orc.k, len(orc.digits)
    m = [orc.mj(j) for j in range(1, n + 1)]
    pitch = lambda q: 4 * ((orc.lam(q) + 3) // 4)

    def sign(first):
        out = [orc.primes[i] * pitch(m[j]) for i in range(first, k) for j in range(n)]
        out += [m[j] * pitch(m[j - 1]) for j in range(1, n)]
        out.append(m[0] * pitch(2))
        return out
    if kind == "relu":
        out = sign(0)
        for i in range(k):
            p = orc.primes[i]
            out += [p * pitch(p), 2 * pitch(p), 2 * 4]
        assert sum(out) == orc.relu_bytes_per_elem()
        return out
    if kind == "sign":
        out = sign(0) + [2 * pitch(orc.primes[i]) for i in range(k)]
        assert sum(out) == orc.signact_bytes_per_elem()
        return out
    out = []
    for _ in range(repeat):
        out += [2 * pitch(orc.primes[i]) for i in range(1, k)] + sign(1)
    assert sum(out) == repeat * orc.scale_bytes_per_elem()
    return out


def table_slices(orc, L, E, first, count):
    """(offset in a table buffer laid out for E elements, offset in one laid out for `count` elements, bytes) of
    the rows of elements first .. first+count-1 (positions inside the E elements), one entry per segment"""
    out, before = [], 0
    for sz in segment_sizes(orc, L["kind"], L.get("repeat", 1)):
        out.append((E * before + first * sz, count * before, count * sz))
        before += sz
    return out
