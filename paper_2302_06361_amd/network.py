"""Layer sequencing for a whole network (Gb, En, Ev, De of Sec. Garbled Circuits) on top of the ABI
calls: buffer allocation and call order only."""
import numpy as np

from . import binding as B


class GarbledNetwork:
    """net: the dict format of workloads.py.  Buffers (labels on every boundary, tables, scratch) are
    allocated once; garble() / evaluate() only enqueue kernels."""

    def __init__(self, ctx, net, batch=None, batch_base=0):
        import torch
        self.ctx, self.net = ctx, net
        self.batch = net["batch"] if batch is None else batch
        self.batch_base = batch_base
        b = self.batch
        self.n_in = net["n_in"]
        self.layers, self.tables = [], []
        n = self.n_in
        scratch_max = 0
        self.sizes = [n * b]
        for L in net["layers"]:
            kind = L["kind"]
            if kind == "conv":
                dense = L["in_h"] == 1 and L["in_w"] == 1 and L["kh"] == 1 and L["kw"] == 1
                K = L["kh"] * L["kw"] * L["in_c"]
                w = ctx.weights_prepare(np.asarray(L["W"]).reshape(L["out_c"], K))
                bias = None
                if L.get("bias") is not None:
                    bias = torch.as_tensor(np.asarray(L["bias"], dtype=np.int32)).to(ctx.device)
                lay = B.Layer(B.DENSE if dense else B.CONV2D, L["id"], b, in_h=L["in_h"], in_w=L["in_w"], in_c=L["in_c"],
                              out_c=L["out_c"], kh=L["kh"], kw=L["kw"], stride=L["stride"], pad=L["pad"], weights=w, bias=bias)
            elif kind == "sumpool":
                lay = B.Layer(B.SUMPOOL, L["id"], b, in_h=L["in_h"], in_w=L["in_w"], in_c=L["ch"])
            elif kind in ("relu", "sign"):
                lay = B.Layer(B.RELU if kind == "relu" else B.SIGN, L["id"], n * b, elem_base=batch_base * n)
            elif kind == "scale":
                lay = B.Layer(B.SCALE, L["id"], n * b, elem_base=batch_base * n, repeat=L["repeat"])
            else:
                raise ValueError(kind)
            oe, tb, sb = ctx.layer_sizes(lay)
            if kind in ("conv", "sumpool"):
                n = oe
            self.layers.append(lay)
            self.tables.append(torch.empty(tb, dtype=torch.uint8, device=ctx.device) if tb else None)
            scratch_max = max(scratch_max, sb)
            self.sizes.append(n * b)
        self.n_out = n
        self.scratch = torch.empty(max(scratch_max, 256), dtype=torch.uint8, device=ctx.device)
        self.zero = [B.Labels(ctx, s) for s in self.sizes]
        self.act = [B.Labels(ctx, s) for s in self.sizes]
        self.values = torch.empty(self.sizes[-1], dtype=torch.int64, device=ctx.device)
        self.valid = torch.empty(self.sizes[-1], dtype=torch.uint8, device=ctx.device)
        self.table_bytes = sum(t.numel() for t in self.tables if t is not None)

    def garble(self):
        c = self.ctx
        c.input_labels(self.batch_base * self.n_in, self.zero[0])
        for i, lay in enumerate(self.layers):
            c.garble_layer(lay, self.zero[i], self.zero[i + 1], self.tables[i], self.scratch)

    def encode(self, x_dev):
        self.ctx.encode(x_dev, self.zero[0], self.act[0])

    def evaluate(self):
        c = self.ctx
        for i, lay in enumerate(self.layers):
            c.eval_layer(lay, self.act[i], self.tables[i], self.act[i + 1], self.scratch)

    def decode(self):
        self.ctx.decode(self.act[-1], self.zero[-1], self.values, self.valid)
        return self.values, self.valid
