"""Whole-network garble / encode / evaluate / decode with the CPU oracle -- TEST
INFRASTRUCTURE ONLY.  (Sec. Garbled Circuits: Gb, En, Ev, De; Sec. System-level Architecture.)

A bundle is a list of k label tensors [n][lambda_{p_i}], one per CRT residue.
Element index of a value inside a layer: batch_index * values_per_batch_element + index.
Input wire index: batch_index * n_in + index.
"""
import numpy as np

from .capi import Oracle


def make_oracle(net, rule=0):
    return Oracle(net["primes"], net["digits"], net["seed"], rule)


def _linear(orc, L, batch, bundle, ones):
    out = []
    for i in range(orc.k):
        if L["kind"] == "conv":
            out.append(orc.conv2d(i, bundle[i], batch, L["in_h"], L["in_w"], L["in_c"], L["out_c"], L["kh"],
                                  L["kw"], L["stride"], L["pad"], L["W"], L.get("bias"), ones[i]))
        else:
            out.append(orc.sumpool2(i, bundle[i], batch, L["in_h"], L["in_w"], L["ch"]))
    return out


def garble(orc, net, batch=None, batch_base=0, keep=False):
    """Gb: returns dict(e = input zero labels, d = output zero labels, tables = per-layer tables,
    zero = zero labels on every layer boundary if keep)."""
    batch = net["batch"] if batch is None else batch
    n_in = net["n_in"]
    cur = [orc.input_labels(batch_base * n_in, batch * n_in, i) for i in range(orc.k)]
    e = cur
    ones0 = [orc.one0(i) for i in range(orc.k)]
    tables, zeros = {}, [cur]
    for L in net["layers"]:
        kind = L["kind"]
        if kind in ("conv", "sumpool"):
            cur = _linear(orc, L, batch, cur, ones0)
        elif kind == "relu":
            cur, tables[L["id"]] = orc.relu_garble(L["id"], cur, elem_base=batch_base * L["n"])
        elif kind == "scale":
            cur, tables[L["id"]] = orc.scale_garble(L["id"], cur, L["repeat"], elem_base=batch_base * L["n"])
        elif kind == "sign":
            cur, tables[L["id"]] = orc.signact_garble(L["id"], cur, elem_base=batch_base * L["n"])
        else:
            raise ValueError(kind)
        if keep:
            zeros.append(cur)
    return dict(e=e, d=cur, tables=tables, zero=zeros)


def encode(orc, net, e, x):
    """En: active input labels."""
    return [orc.encode(i, x, e[i]) for i in range(orc.k)]


def evaluate(orc, net, act, tables, batch=None, batch_base=0, keep=False):
    """Ev: active output labels (and every boundary if keep)."""
    batch = net["batch"] if batch is None else batch
    ones = [orc.one(i) for i in range(orc.k)]
    cur, acts = act, [act]
    for L in net["layers"]:
        kind = L["kind"]
        if kind in ("conv", "sumpool"):
            cur = _linear(orc, L, batch, cur, ones)
        elif kind == "relu":
            cur = orc.relu_eval(L["id"], cur, tables[L["id"]], elem_base=batch_base * L["n"])
        elif kind == "scale":
            cur = orc.scale_eval(L["id"], cur, tables[L["id"]], L["repeat"], elem_base=batch_base * L["n"])
        elif kind == "sign":
            cur = orc.signact_eval(L["id"], cur, tables[L["id"]], elem_base=batch_base * L["n"])
        if keep:
            acts.append(cur)
    return (cur, acts) if keep else cur


def run(net, batch=None, batch_base=0, rule=0, keep=False):
    """Garble, encode, evaluate and decode `batch` batch elements starting at batch_base."""
    orc = make_oracle(net, rule)
    batch = net["batch"] if batch is None else batch
    n_in = net["n_in"]
    x = np.asarray(net["x"][batch_base * n_in:(batch_base + batch) * n_in])
    gb = garble(orc, net, batch, batch_base, keep)
    act_in = encode(orc, net, gb["e"], x)
    ev = evaluate(orc, net, act_in, gb["tables"], batch, batch_base, keep)
    act_out, acts = (ev if keep else (ev, None))
    values, valid = orc.decode(act_out, gb["d"])
    return dict(orc=orc, gb=gb, act_in=act_in, act_out=act_out, acts=acts, values=values, valid=valid)
