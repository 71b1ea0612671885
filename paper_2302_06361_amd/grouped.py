"""Independent projection gates with mixed moduli (Sec. Arithmetic Garbled Circuits, projection gates):
the gates are grouped by their (input modulus, output modulus) pair and every group is one PROJ layer
call.  Buffer allocation, grouping and call order only; the gates themselves run in the library."""
import numpy as np

from . import binding as B


class ProjectionBatch:
    """n gates, gate g maps Z_{primes[pi[g]]} -> Z_{primes[qi[g]]}.

    Gates are renumbered in grouped order: `order[j]` is the caller's index of the gate at position j,
    and position j is the gate's element index (its tweak).  Per group the buffers are
    in0 / act (input zero and active labels), out0 / out (output labels), phi [count][p], table."""

    def __init__(self, ctx, pi, qi, layer_id=1, streams=4):
        import torch
        self.ctx = ctx
        # the groups are independent: their calls go round-robin to a few streams (default priority), so that the
        # ramp-up and tail of one group's kernels overlap with its neighbours'
        self._streams = [torch.cuda.Stream(device=ctx.device) for _ in range(max(1, streams))] if streams > 1 else []
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

    def _each_group(self, call, serial=False):
        import torch
        if serial or not self._streams:
            for g in self.groups:
                call(g)
            return
        cur = torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(cur)
        for s in self._streams:
            s.wait_event(start)                       # after everything already queued on the caller's stream
        for idx, g in enumerate(self.groups):
            with torch.cuda.stream(self._streams[idx % len(self._streams)]):
                call(g)
        for s in self._streams:                       # the caller's stream continues when all groups are done
            done = torch.cuda.Event()
            done.record(s)
            cur.wait_event(done)

    def garble(self, serial=False):
        """serial: all groups on the caller's stream, one after the other (per-kernel timing)"""
        self._each_group(lambda g: self.ctx.garble_layer(g["layer"], g["in0"], g["out0"], g["table"]), serial)

    def evaluate(self, serial=False):
        self._each_group(lambda g: self.ctx.eval_layer(g["layer"], g["act"], g["table"], g["out"]), serial)
