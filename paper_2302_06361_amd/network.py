"""Layer sequencing for a whole network (Gb, En, Ev, De of Sec. Garbled Circuits) on top of the ABI
calls: buffer allocation and call order only."""
import numpy as np

from . import binding as B


def build_layers(ctx, net, b, batch_base):
    """-> (layer descriptors, values on every boundary, table bytes per layer, scratch bytes) for b batch elements"""
    import torch
    layers, table_bytes = [], []
    n = net["n_in"]
    scratch_max = 0
    sizes = [n * b]
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
            lay.per_batch_element = n
        elif kind == "scale":
            lay = B.Layer(B.SCALE, L["id"], n * b, elem_base=batch_base * n, repeat=L["repeat"])
            lay.per_batch_element = n
        else:
            raise ValueError(kind)
        oe, tb, sb = ctx.layer_sizes(lay)
        if kind in ("conv", "sumpool"):
            n = oe
        layers.append(lay)
        table_bytes.append(tb)
        scratch_max = max(scratch_max, sb)
        sizes.append(n * b)
    return layers, sizes, table_bytes, scratch_max


class GarbledNetwork:
    """net: the dict format of workloads.py.  Buffers (labels on every boundary, tables, scratch) are
    allocated once; garble() / evaluate() only enqueue kernels."""

    def __init__(self, ctx, net, batch=None, batch_base=0):
        import torch
        self.ctx, self.net = ctx, net
        self.batch = net["batch"] if batch is None else batch
        self.batch_base = batch_base
        self.n_in = net["n_in"]
        self.layers, self.sizes, tbytes, scratch_max = build_layers(ctx, net, self.batch, batch_base)
        self.tables = [torch.empty(tb, dtype=torch.uint8, device=ctx.device) if tb else None for tb in tbytes]
        self.n_out = self.sizes[-1] // max(self.batch, 1)
        self.scratch = torch.empty(max(scratch_max, 256), dtype=torch.uint8, device=ctx.device)
        self.zero = [B.Labels(ctx, s) for s in self.sizes]
        self.act = [B.Labels(ctx, s) for s in self.sizes]
        self.values = torch.empty(self.sizes[-1], dtype=torch.int64, device=ctx.device)
        self.valid = torch.empty(self.sizes[-1], dtype=torch.uint8, device=ctx.device)
        self.table_bytes = sum(tbytes)

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


class StreamedNetwork:
    """The same call sequence for networks whose tables do not fit in memory at once: layer by layer,
    garble then evaluate, with one table buffer (the size of the largest layer) that the next layer
    overwrites, and two label bundles per side.  In the two-party setting this is the point where the
    garbler would ship each layer's tables to the evaluator."""

    def __init__(self, ctx, net, batch=None, batch_base=0):
        import torch
        self.ctx, self.net = ctx, net
        self.batch = net["batch"] if batch is None else batch
        self.batch_base = batch_base
        self.n_in = net["n_in"]
        self.layers, self.sizes, self.layer_table_bytes, scratch_max = build_layers(ctx, net, self.batch, batch_base)
        self.table = torch.empty(max(max(self.layer_table_bytes), 256), dtype=torch.uint8, device=ctx.device)
        self.scratch = torch.empty(max(scratch_max, 256), dtype=torch.uint8, device=ctx.device)
        big = max(self.sizes)
        self.zero = [B.Labels(ctx, big), B.Labels(ctx, big)]
        self.act = [B.Labels(ctx, big), B.Labels(ctx, big)]
        self.values = torch.empty(self.sizes[-1], dtype=torch.int64, device=ctx.device)
        self.valid = torch.empty(self.sizes[-1], dtype=torch.uint8, device=ctx.device)
        self.table_bytes = sum(self.layer_table_bytes)

    def rebase(self):
        """after a change of self.batch_base: the same buffers and descriptors serve the next chunk of the batch (element
        and wire indices of a chunk start at its first batch element)"""
        for lay in self.layers:
            n = getattr(lay, "per_batch_element", None)
            if n is not None:
                lay.c.elem_base = self.batch_base * n

    def run(self, x_dev, on_boundary=None):
        """Gb, En, Ev, De over the whole network.  on_boundary(b, zero, act) sees the label bundles of
        boundary b (0 = network input) before the next layer overwrites them."""
        c = self.ctx
        z = [self.zero[0].slice(0, self.sizes[0]), None]
        a = [self.act[0].slice(0, self.sizes[0]), None]
        c.input_labels(self.batch_base * self.n_in, z[0])
        c.encode(x_dev, z[0], a[0])
        if on_boundary:
            on_boundary(0, z[0], a[0])
        for i, lay in enumerate(self.layers):
            s, d = i & 1, (i + 1) & 1
            z[d] = self.zero[d].slice(0, self.sizes[i + 1])
            a[d] = self.act[d].slice(0, self.sizes[i + 1])
            tab = self.table[:self.layer_table_bytes[i]] if self.layer_table_bytes[i] else None
            c.garble_layer(lay, z[s], z[d], tab, self.scratch)
            c.eval_layer(lay, a[s], tab, a[d], self.scratch)
            if on_boundary:
                on_boundary(i + 1, z[d], a[d])
        last = len(self.layers) & 1
        c.decode(a[last], z[last], self.values, self.valid)
        return self.values, self.valid
