"""Independent projection gates with mixed moduli (Sec. Arithmetic Garbled Circuits, projection gates):
the gates are grouped by their (input modulus, output modulus) pair, every group is one PROJ layer
descriptor, and all descriptors go to the library in one call.  Buffer allocation and grouping only; the gates
themselves run in the library."""
import numpy as np

from . import binding as B


class ProjectionBatch:
    """n gates, gate g maps Z_{primes[pi[g]]} -> Z_{primes[qi[g]]}.

    Gates are renumbered in grouped order: `order[j]` is the caller's index of the gate at position j,
    and position j is the gate's element index (its tweak).  Per group the buffers are
    in0 / act (input zero and active labels), out0 / out (output labels), phi [count][p], table.
    garble() and evaluate() hand all groups to the library in ONE call (dash_garble_layers / dash_eval_layers),
    which serves the groups that share an output modulus with one kernel launch."""

    def __init__(self, ctx, pi, qi, layer_id=1):
        import torch
        self.ctx = ctx
        k = ctx.k
        key = np.asarray(pi, np.int64) * k + np.asarray(qi, np.int64)
        self.order = np.argsort(key, kind="stable")
        counts = np.bincount(key, minlength=k * k)
        self.groups = []
        start = 0
        for pair in range(k * k):
            n = int(counts[pair])
            if n == 0:
                continue
            i, j = divmod(pair, k)
            p = ctx.primes[i]
            phi = torch.empty((n, p), dtype=torch.uint8, device=ctx.device)
            lay = B.Layer(B.PROJ, layer_id, n, elem_base=start, p_index=i, q_index=j, phi=phi, phi_stride=p)
            oe, tb, sb = ctx.layer_sizes(lay)
            self.groups.append(dict(
                pi=i, qi=j, start=start, count=n, layer=lay, phi=phi,
                in0=B.Labels(ctx, n, only=[i]), act=B.Labels(ctx, n, only=[i]),
                out0=B.Labels(ctx, n, only=[j], zero=True), out=B.Labels(ctx, n, only=[j], zero=True),
                table=torch.empty(tb, dtype=torch.uint8, device=ctx.device)))
            start += n
        self.n = start
        self.table_bytes = sum(g["table"].numel() for g in self.groups)
        self.rows = sum(g["count"] * ctx.primes[g["pi"]] for g in self.groups)

    def _lists(self, a, b):
        G = self.groups
        return [g["layer"] for g in G], [g[a] for g in G], [g[b] for g in G], [g["table"] for g in G]

    def garble(self, one_call_per_group=False):
        """one_call_per_group: a dash_garble_layer call (and its own kernel launches) per (p, q) group instead"""
        if one_call_per_group:
            for g in self.groups:
                self.ctx.garble_layer(g["layer"], g["in0"], g["out0"], g["table"])
            return
        layers, ins, outs, tables = self._lists("in0", "out0")
        self.ctx.garble_layers(layers, ins, outs, tables)

    def evaluate(self, one_call_per_group=False):
        if one_call_per_group:
            for g in self.groups:
                self.ctx.eval_layer(g["layer"], g["act"], g["table"], g["out"])
            return
        layers, ins, outs, tables = self._lists("act", "out")
        self.ctx.eval_layers(layers, ins, tables, outs)
