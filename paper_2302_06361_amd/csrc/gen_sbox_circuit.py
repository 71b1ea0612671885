"""Writes dash_sbox_circuit.h: the AES S-box (FIPS-197, Sec. 5.1.1) as a straight-line Boolean circuit for
bitsliced evaluation, in 2- and 3-input operations (gfx950 has a 3-input bit operation with any truth table).

Construction, all derived here from the field arithmetic, nothing tabulated:
  * GF(2^8) of the standard (x^8 + x^4 + x^3 + x + 1) is mapped to the tower GF(((2^2)^2)^2) with polynomial bases
    W^2 = W + 1, Z^2 = Z + N, Y^2 = Y + nu; inversion there needs one GF(2^4) inversion and three GF(2^4)
    products (A = A1 Y + A0: D = A1^2 nu + A1 A0 + A0^2, A^-1 = (A1 D^-1) Y + (A1 + A0) D^-1), and likewise one
    level down.  The S-box's affine map is merged with the map back; its constant 0x63 is left to the caller
    (it commutes with ShiftRows and MixColumns and is folded into the round keys).
  * every exclusive-or is kept lazy (a signal is a set of "atoms": inputs and AND outputs) and only the operands
    of AND gates and the outputs are materialised, all together, with a greedy common-pair elimination
    (repeatedly: the pair of atoms that occurs in most targets becomes a new atom);
  * all choices of N, nu and of the root that defines the field isomorphism are tried; the smallest circuit wins;
  * pairs of 2-input gates are then merged into 3-input operations where the inner gate has one use.
The result is checked against the S-box computed from the field definition for all 256 inputs.

Run:  python gen_sbox_circuit.py  (writes dash_sbox_circuit.h beside itself; not needed at build time)
"""
import itertools
import os
import sys


# ---------------- GF(2^8), the S-box from its definition ----------------
def gmul(a, b, poly=0x11b):
    r = 0
    while b:
        if b & 1:
            r ^= a
        a <<= 1
        if a & 0x100:
            a ^= poly
        b >>= 1
    return r


def ginv(a):
    if a == 0:
        return 0
    r = 1
    for _ in range(254):
        r = gmul(r, a)
    return r


def sbox_linear_part(x):
    """affine map of the S-box without its constant"""
    r = 0
    for i in range(8):
        b = 0
        for j in (0, 4, 5, 6, 7):
            b ^= (x >> ((i + j) % 8)) & 1
        r |= b << i
    return r


SBOX = [sbox_linear_part(ginv(x)) ^ 0x63 for x in range(256)]


# ---------------- tower field on integers (to find the isomorphism) ----------------
class Tower:
    """elements: 8-bit ints, bit layout (Y1: (Z1: (W1 W0), Z0: (W1 W0)), Y0: ...) most significant first"""

    def __init__(self, N, nu):
        self.N, self.nu = N, nu

    @staticmethod
    def m2(a, b):
        a1, a0, b1, b0 = a >> 1, a & 1, b >> 1, b & 1
        p, q, m = a1 & b1, a0 & b0, (a1 ^ a0) & (b1 ^ b0)
        return ((m ^ q) << 1) | (p ^ q)

    def m4(self, a, b):
        a1, a0, b1, b0 = a >> 2, a & 3, b >> 2, b & 3
        p, q, m = self.m2(a1, b1), self.m2(a0, b0), self.m2(a1 ^ a0, b1 ^ b0)
        return ((m ^ q) << 2) | (self.m2(p, self.N) ^ q)

    def m8(self, a, b):
        a1, a0, b1, b0 = a >> 4, a & 15, b >> 4, b & 15
        p, q, m = self.m4(a1, b1), self.m4(a0, b0), self.m4(a1 ^ a0, b1 ^ b0)
        return ((m ^ q) << 4) | (self.m4(p, self.nu) ^ q)

    def irreducible(self):
        # Z^2 + Z + N over GF(4), Y^2 + Y + nu over GF(16): no root
        if any(self.m2(z, z) ^ z ^ self.N == 0 for z in range(4)):
            return False
        return not any(self.m4(y, y) ^ y ^ self.nu == 0 for y in range(16))


def isomorphisms(T):
    """all 8x8 bit matrices (as lists of 8 images of the standard basis x^i) mapping GF(2^8) standard -> tower"""
    out = []
    for beta in range(2, 256):
        # beta must satisfy x^8 + x^4 + x^3 + x + 1 in the tower
        pw = [1]
        for _ in range(8):
            pw.append(T.m8(pw[-1], beta))
        if pw[8] ^ pw[4] ^ pw[3] ^ pw[1] ^ pw[0] == 0:
            out.append(pw[:8])
    return out


# ---------------- lazy-xor circuit ----------------
class Circ:
    def __init__(self, n_in):
        self.n_in = n_in
        self.n_atoms = n_in
        self.ands = []          # (atom id, frozenset a, frozenset b); b is None for a cut (atom = xor of the set a)
        self.cache = {}
        self.cuts = set()       # names of the places where a lazy signal is turned into an atom

    def inputs(self):
        return [frozenset([i]) for i in range(self.n_in)]

    def AND(self, a, b):
        if not a or not b:
            return frozenset()
        key = (a, b) if sorted(a) <= sorted(b) else (b, a)
        if key not in self.cache:
            self.cache[key] = self.n_atoms
            self.ands.append((self.n_atoms, key[0], key[1]))
            self.n_atoms += 1
        return frozenset([self.cache[key]])


    def cut(self, where, sigs):
        """materialise the signals here (they become atoms) if `where` is among the chosen cut points"""
        if where not in self.cuts:
            return sigs
        out = []
        for sg in sigs:
            if len(sg) < 2:
                out.append(sg)
                continue
            key = (sg, None)
            if key not in self.cache:
                self.cache[key] = self.n_atoms
                self.ands.append((self.n_atoms, sg, None))
                self.n_atoms += 1
            out.append(frozenset([self.cache[key]]))
        return out


def X(a, b):
    return a ^ b


class SymTower:
    """the same tower arithmetic on lazy-xor signals; an element of GF(2^(2k)) is a list of bits, least first"""

    def __init__(self, C, N, nu):
        self.C, self.N, self.nu = C, N, nu

    def add(self, a, b):
        return [X(x, y) for x, y in zip(a, b)]

    def m2(self, a, b):
        C = self.C
        p, q, m = C.AND(a[1], b[1]), C.AND(a[0], b[0]), C.AND(X(a[1], a[0]), X(b[1], b[0]))
        return [X(p, q), X(m, q)]

    def const_mul(self, a, c, mulfn, width):
        """a (symbolic, `width` bits) times the constant c: linear, so a bit matrix applied lazily"""
        out = [frozenset() for _ in range(width)]
        for i in range(width):
            img = mulfn(1 << i, c)
            for j in range(width):
                if (img >> j) & 1:
                    out[j] = X(out[j], a[i])
        return out

    def sq2(self, a):
        return [X(a[1], a[0]), a[1]]          # (a1 W + a0)^2 = a1 W + (a1 + a0)

    def inv2(self, a):
        return self.sq2(a)                    # a^-1 = a^2 in GF(4)

    def m4(self, a, b):
        a1, a0, b1, b0 = a[2:], a[:2], b[2:], b[:2]
        p, q, m = self.m2(a1, b1), self.m2(a0, b0), self.m2(self.add(a1, a0), self.add(b1, b0))
        lo = self.add(self.const_mul(p, self.N, Tower.m2, 2), q)
        return self.C.cut("m4", lo + self.add(m, q))

    def inv4(self, T, a):
        a1, a0 = a[2:], a[:2]
        s = self.add(a1, a0)
        d = self.add(self.add(self.const_mul(self.sq2(a1), self.N, Tower.m2, 2), self.m2(a1, a0)), self.sq2(a0))
        d = self.C.cut("d4", d)
        di = self.C.cut("di4", self.inv2(d))
        return self.C.cut("inv4", self.m2(s, di) + self.m2(a1, di))

    def sq4_lin(self, T, a, c):
        """(a^2) * c in GF(16): linear in a"""
        out = [frozenset() for _ in range(4)]
        for i in range(4):
            img = T.m4(T.m4(1 << i, 1 << i), c)
            for j in range(4):
                if (img >> j) & 1:
                    out[j] = X(out[j], a[i])
        return out

    def inv8(self, T, a):
        a1, a0 = a[4:], a[:4]
        s = self.C.cut("s8", self.add(a1, a0))
        d = self.add(self.add(self.sq4_lin(T, a1, self.nu), self.m4(a1, a0)), self.sq4_lin(T, a0, 1))
        d = self.C.cut("d8", d)
        di = self.inv4(T, d)
        return self.m4(s, di) + self.m4(a1, di)


def apply_matrix(cols, vec):
    """cols[i] = image (int) of basis vector i; vec = list of lazy signals -> list of 8 lazy signals"""
    out = [frozenset() for _ in range(8)]
    for i in range(8):
        for j in range(8):
            if (cols[i] >> j) & 1:
                out[j] = X(out[j], vec[i])
    return out


def invert_matrix(cols):
    """inverse of the 8x8 GF(2) matrix given by column images, as column images"""
    # solve by brute force over the 256 vectors
    fwd = {}
    for v in range(256):
        r = 0
        for i in range(8):
            if (v >> i) & 1:
                r ^= cols[i]
        fwd[r] = v
    return [fwd[1 << i] for i in range(8)]


def build(N, nu, iso, cuts=()):
    T = Tower(N, nu)
    C = Circ(8)
    C.cuts = set(cuts)
    S = SymTower(C, N, nu)
    x = C.inputs()
    t = C.cut("t", apply_matrix(iso, x))
    ti = C.cut("ti", S.inv8(T, t))
    back = invert_matrix(iso)
    # tower -> standard, then the S-box's linear map
    lin = [sbox_linear_part(b) for b in back]
    y = apply_matrix(lin, ti)
    return C, y


# ---------------- materialise xors: greedy common-pair elimination ----------------
def materialise(C, outs):
    """returns a list of 2-input gates ('x'|'a', dst, s1, s2) in an order that respects dependencies, and the names
    of the outputs.  Targets: both operands of every AND (in creation order) and the outputs."""
    targets = []                                  # [set of atoms], owner
    for (aid, a, b) in C.ands:
        targets.append(set(a))
        targets.append(set(b) if b is not None else set())
    for o in outs:
        targets.append(set(o))
    n_atoms = C.n_atoms
    # an atom may be used by a target only if it exists before the target's owner; pair atoms are defined when both
    # members exist, which is always before any target that holds both.
    pair_def = {}
    while True:
        cnt = {}
        for t in targets:
            if len(t) < 2:
                continue
            for p in itertools.combinations(sorted(t), 2):
                cnt[p] = cnt.get(p, 0) + 1
        if not cnt:
            break
        best = max(cnt.items(), key=lambda kv: (kv[1], -kv[0][0], -kv[0][1]))
        (i, j), c = best
        if c < 2:
            break
        new = n_atoms
        n_atoms += 1
        pair_def[new] = (i, j)
        for t in targets:
            if i in t and j in t:
                t.discard(i)
                t.discard(j)
                t.add(new)
    # emit
    gates = []
    ready = set(range(C.n_in))
    alias = {}

    def need(atom):
        if atom in ready:
            return
        if atom in pair_def:
            i, j = pair_def[atom]
            need(i)
            need(j)
            gates.append(('x', atom, i, j))
            ready.add(atom)
            return
        raise KeyError(atom)

    def realise(t):
        t = sorted(t)
        for a in t:
            need(a)
        if len(t) == 1:
            return t[0]
        nonlocal n_atoms
        acc = t[0]
        for a in t[1:]:
            new = n_atoms
            n_atoms += 1
            gates.append(('x', new, acc, a))
            ready.add(new)
            acc = new
        return acc

    ti = 0
    for (aid, a, b) in C.ands:
        ra = realise(targets[ti])
        if b is None:                       # a cut: the atom is the materialised xor itself
            ti += 2
            alias[aid] = ra
            ready.add(aid)
            continue
        rb = realise(targets[ti + 1])
        ti += 2
        gates.append(('a', aid, ra, rb))
        ready.add(aid)
    outs_named = []
    for o in outs:
        outs_named.append(realise(targets[ti]))
        ti += 1

    def res(a):
        while a in alias:
            a = alias[a]
        return a
    gates = [(k, d, res(a), res(b)) for (k, d, a, b) in gates]
    return gates, [res(o) for o in outs_named]


# ---------------- 3-input fusion ----------------
def fuse(gates, outs, trials=24, seed=1):
    """Merge 2-input gates into their users: a gate x = a . b disappears when EVERY user u = x . c takes it in as the
    3-input operation (a . b) . c (a user can take in one operand only, and a merged user cannot be taken in itself).
    Which gates go is a matching problem; several random orders are tried.  Result: ops (dst, table | 'x' | 'a', a, b, c)
    in the v_bitop3 convention (table = f(0xF0, 0xCC, 0xAA)); 2-input gates keep c = None."""
    import random
    rnd = random.Random(seed)
    f2 = {'x': lambda p, q: p ^ q, 'a': lambda p, q: p & q}
    users = {}
    for (k, d, a, b) in gates:
        users.setdefault(a, []).append(d)
        users.setdefault(b, []).append(d)
    defs = {d: (k, a, b) for (k, d, a, b) in gates}
    outset = set(outs)
    cands = [d for (k, d, a, b) in gates if d not in outset and d in users]
    best = None
    for t in range(trials):
        order = sorted(cands, key=lambda d: (len(users[d]), rnd.random())) if t else sorted(cands, key=lambda d: len(users[d]))
        if t > trials // 2:
            rnd.shuffle(order)
        absorbed = {}          # user -> inner it took in
        gone = set()
        for x in order:
            us = users[x]
            if len(set(us)) != len(us):
                continue       # x . x does not occur, but be safe
            if any(u in absorbed or u in gone for u in us):
                continue
            if x in absorbed:  # x is already a 3-input operation
                continue
            for u in us:
                absorbed[u] = x
            gone.add(x)
        n = len(gates) - len(gone)
        if best is None or n < best[0]:
            best = (n, dict(absorbed), set(gone))
    n, absorbed, gone = best
    ops = []
    for (k, d, a, b) in gates:
        if d in gone:
            continue
        if d in absorbed:
            x = absorbed[d]
            other = b if a == x else a
            ik, ia, ib = defs[x]
            tt = f2[k](f2[ik](0xF0, 0xCC), 0xAA) & 0xff
            ops.append((d, tt, ia, ib, other))
        else:
            ops.append((d, k, a, b, None))
    return ops


def evaluate(ops, outs, x):
    v = {i: (x >> i) & 1 for i in range(8)}
    for (d, k, a, b, c) in ops:
        if c is None:
            v[d] = (v[a] ^ v[b]) if k == 'x' else (v[a] & v[b])
        else:
            v[d] = (k >> (v[a] * 4 + v[b] * 2 + v[c])) & 1
    return sum(v[o] << i for i, o in enumerate(outs))


CUTS = ("d8", "d4", "inv4", "s8", "ti")


def main():
    best = None
    for N in (2, 3):
        for nu in range(16):
            T = Tower(N, nu)
            if not T.irreducible():
                continue
            for iso in isomorphisms(T):
                for nc in range(len(CUTS) + 1):
                    for cuts in itertools.combinations(CUTS, nc):
                        C, y = build(N, nu, iso, cuts)
                        gates, outs = materialise(C, y)
                        ops = fuse(gates, outs)
                        key = (len(ops), len(gates))
                        if best is None or key < best[0]:
                            best = (key, N, nu, iso, gates, outs, ops)
                            print(key, N, nu, cuts, file=sys.stderr)
    key, N, nu, iso, gates, outs, ops = best
    for x in range(256):
        assert evaluate(ops, outs, x) == SBOX[x] ^ 0x63, x
    n_and = sum(1 for g in gates if g[0] == 'a')
    print("N=%d nu=%d: %d two-input gates (%d and, %d xor) -> %d operations of up to three inputs" %
          (N, nu, len(gates), n_and, len(gates) - n_and, len(ops)), file=sys.stderr)
    # emit
    name = {i: "x%d" % i for i in range(8)}
    lines = []
    for (d, k, a, b, c) in ops:
        name[d] = "t%d" % d
        if c is None:
            lines.append("    const W t%d = %s %s %s;" % (d, name[a], '^' if k == 'x' else '&', name[b]))
        else:
            lines.append("    const W t%d = bop3<0x%02x>(%s, %s, %s);" % (d, k, name[a], name[b], name[c]))
    hdr = []
    hdr.append("// GENERATED by gen_sbox_circuit.py -- do not edit.  The AES S-box WITHOUT its constant 0x63 (FIPS-197 Sec. 5.1.1:")
    hdr.append("// inverse in GF(2^8), then the affine map's linear part) on bit planes: x0..x7 = planes of the input byte, least")
    hdr.append("// significant first; y likewise.  %d operations (%d two-input gates before merging; tower N=%d, nu=%d)." %
               (len(ops), len(gates), N, nu))
    hdr.append("#pragma once")
    hdr.append("namespace dash {")
    hdr.append("constexpr int kSboxCircuitOps = %d;" % len(ops))
    hdr.append("template <class W, class B3>")
    hdr.append("DASH_HD void sbox_planes(const W& x0, const W& x1, const W& x2, const W& x3, const W& x4, const W& x5, const W& x6, const W& x7,")
    hdr.append("                         W& y0, W& y1, W& y2, W& y3, W& y4, W& y5, W& y6, W& y7, B3) {")
    body = [l.replace("bop3<", "B3::template op<") for l in lines]
    hdr += body
    for i, o in enumerate(outs):
        hdr.append("    y%d = %s;" % (i, name[o]))
    hdr.append("}")
    hdr.append("}  // namespace dash")
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "dash_sbox_circuit.h")
    with open(path, "w") as f:
        f.write("\n".join(hdr) + "\n")


if __name__ == "__main__":
    main()
