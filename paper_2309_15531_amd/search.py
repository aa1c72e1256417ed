"""The per-layer AdaDim search as a sequence of library calls (Sec. 3.3, App. B).

Allocation and call order only; all arithmetic happens in libadadim.so.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def clip_grid(n: int = 20, lo: float = 0.5, hi: float = 1.0):
    """n clip ratios in [lo, hi], ends included, fp64 then one rounding to fp32."""
    if n == 1:
        return [float(np.float32(hi))]
    return [float(np.float32(lo + (hi - lo) * i / (n - 1))) for i in range(n)]


class PreparedHessian:
    """H = X^T X on the device plus the fp16 form the scoring kernel consumes."""

    def __init__(self, ctx: B.Context, in_f: int, device="cuda"):
        self.ctx = ctx
        self.in_f = in_f
        self.H = torch.empty((in_f, in_f), dtype=torch.float32, device=device)
        self.Hs = ctx.alloc_score(in_f, in_f, device)      # scoring layout, flat
        self.hmeta = torch.empty((2, in_f), dtype=torch.float32, device=device)
        self.tokens = 0

    def update(self, X, accumulate: bool = False):
        self.ctx.adadim_hessian(X, self.H, accumulate=accumulate)
        self.tokens = X.shape[0] + (self.tokens if accumulate else 0)
        return self

    def prepare(self):
        self.ctx.adadim_hessian_prepare(self.H, self.Hs, self.hmeta)
        return self

    def update_prepared(self, X):
        """update(X) and prepare() in one call (adadim_hessian_prepared): for a calibration set that comes whole."""
        self.ctx.adadim_hessian_prepared(X, self.H, self.Hs, self.hmeta)
        self.tokens = X.shape[0]
        return self

    @property
    def colscale(self):
        return self.hmeta[0]


class LayerSearch:
    """Buffers for searching layers of one shape; reused across layers and candidates.

    Candidates are scored in batches of up to `batch` (one adadim_layer_error_batch call each).
    With at most `batch` candidates and keep_winner, every candidate's packed codes, scales and
    zeros are written while it is scored, so the winner needs no second quantization.

    meta16: candidates are quantized into the b + 16/g storage format (adadim_quantize_meta16), so
    the losses are those of the weights that will be stored; the winner's group words are in
    self.meta (uint16 bits in an int16 tensor) and self.scales / self.zeros stay None."""

    def __init__(self, ctx: B.Context, out_f: int, in_f: int, bits: int, group: int, clips=(1.0,),
                 keep_winner: bool = True, batch: int = 8, device="cuda", meta16: bool = False):
        self.ctx, self.out_f, self.in_f, self.bits, self.group = ctx, out_f, in_f, bits, group
        self.meta16 = meta16
        self.clips = [float(np.float32(c)) for c in clips]
        self.cands = [(d, c) for d in (B.DIM_OC, B.DIM_IC) for c in self.clips]
        self.batch = max(1, min(batch, 8, len(self.cands)))
        self.dWs = [ctx.alloc_score(out_f, in_f, device) for _ in range(self.batch)]   # scoring layout, flat
        self.losses = torch.empty(len(self.cands), dtype=torch.float32, device=device)
        self.best = torch.empty(1, dtype=torch.int32, device=device)
        self.keep_winner = keep_winner
        g_oc = in_f if group == 0 else group
        g_ic = out_f if group == 0 else group
        self.meta_shape = {B.DIM_OC: (out_f, in_f // g_oc), B.DIM_IC: (out_f // g_ic, in_f)}
        self.scales = self.zeros = self.packed = self.meta = None
        if keep_winner:
            n_meta = max(out_f * (in_f // g_oc), (out_f // g_ic) * in_f)
            words = max(out_f * ((in_f * bits + 31) // 32), in_f * ((out_f * bits + 31) // 32))
            # one output set per candidate when they all fit in one batch, else one set for the winner
            self.inline = len(self.cands) <= self.batch
            n_sets = len(self.cands) if self.inline else 1
            if meta16:
                self._meta = [torch.empty(n_meta, dtype=torch.int16, device=device) for _ in range(n_sets)]
            else:
                self._scales = [torch.empty(n_meta, dtype=torch.float32, device=device) for _ in range(n_sets)]
                self._zeros = [torch.empty(n_meta, dtype=torch.uint8, device=device) for _ in range(n_sets)]
            self._packed = [torch.empty(words, dtype=torch.int32, device=device) for _ in range(n_sets)]
        else:
            self.inline = False

    def score_all(self, W, hp: PreparedHessian, select: bool = False):
        """Quantizes and scores every candidate; losses stay on the device.  select: also leave the winning
        index in self.best (taken by the scoring call itself when the candidates fit one batch)."""
        for c0 in range(0, len(self.cands), self.batch):
            chunk = self.cands[c0:c0 + self.batch]
            if len(self.cands) == 2 and self.inline:
                # the plain search: its two candidates in one call (one launch where the shape allows)
                key = "meta" if self.meta16 else "scales"
                sets = [{"dW": self.dWs[k], "packed": self._packed[k], key: (self._meta if self.meta16 else self._scales)[k],
                         "zeros": None if self.meta16 else self._zeros[k]} for k in (0, 1)]
                self.ctx.adadim_quantize_both(W, self.bits, self.group, hp.colscale, sets[0], sets[1], clip=chunk[0][1],
                                              meta16=self.meta16)
            else:
                for k, (dim, clip) in enumerate(chunk):
                    self._quantize(W, dim, clip, c0 + k if self.inline else None, dW=self.dWs[k],
                                   dW_dtype=B.DW_F16_SCALED, colscale=hp.colscale)
            if select and len(chunk) == len(self.cands):
                self.ctx.adadim_layer_error_batch_select(self.dWs[:len(chunk)], B.DW_F16_SCALED, hp.Hs, hp.hmeta,
                                                         self.losses, self.best, shape=(self.out_f, self.in_f))
                return
            self.ctx.adadim_layer_error_batch(self.dWs[:len(chunk)], B.DW_F16_SCALED, hp.Hs, hp.hmeta,
                                              self.losses[c0:c0 + len(chunk)], shape=(self.out_f, self.in_f))
        if select:
            self.ctx.adadim_select(self.losses, best_dev=self.best, to_host=False)

    def _quantize(self, W, dim, clip, out_set, **kw):
        """One candidate; out_set names the output set that receives its parameters and packed codes."""
        if self.meta16:
            if out_set is not None:
                kw.update(meta=self._meta[out_set], packed=self._packed[out_set])
            self.ctx.adadim_quantize_meta16(W, dim, self.bits, self.group, clip, **kw)
        else:
            if out_set is not None:
                kw.update(scales=self._scales[out_set], zeros=self._zeros[out_set], packed=self._packed[out_set])
            self.ctx.adadim_quantize(W, dim, self.bits, self.group, clip, **kw)

    def launch(self, W, hp: PreparedHessian):
        """Queues the whole search for one layer and returns at once: the losses and the winning index stay on
        the device until `result` asks for them, so a driver can queue the next layer meanwhile."""
        self.score_all(W, hp, select=True)
        self._W = W

    def result(self):
        """Waits for the last `launch`: returns (best index, dim, clip); with keep_winner the winner's packed
        codes, scales and zeros are in self.packed / self.scales / self.zeros."""
        torch.cuda.synchronize()
        return self._finish(int(self.best.item()), self._W)

    def run(self, W, hp: PreparedHessian):
        """launch + result with the library's own wait (one synchronisation of the context's stream)."""
        self.score_all(W, hp)
        best = self.ctx.adadim_select(self.losses, best_dev=self.best, to_host=True)
        return self._finish(best, W)

    def _finish(self, best, W):
        dim, clip = self.cands[best]
        if self.keep_winner:
            k = best if self.inline else 0
            self.packed = self._packed[k]
            if self.meta16:
                self.meta = self._meta[k]
            else:
                self.scales, self.zeros = self._scales[k], self._zeros[k]
            if not self.inline:
                self._quantize(W, dim, clip, 0)
        return best, dim, clip


class GraphedSearch:
    """One layer's whole step (Gram matrix, preparation, every candidate, selection) recorded once as a HIP graph
    and replayed per layer: the layers of a model that share a shape reuse the graph, their weights and
    activations are copied into (or produced in) the buffers the graph was recorded with.

    The context must live on a stream of its own (not the default stream); torch work that feeds the buffers must
    be ordered before the launch by the caller (same stream, or an event)."""

    def __init__(self, ctx: B.Context, ls: LayerSearch, hp: PreparedHessian, W, X):
        if not (ls.inline or not ls.keep_winner):
            raise ValueError("GraphedSearch needs every candidate's outputs kept while scored (candidates <= batch)")
        self.ctx, self.ls, self.hp, self.W, self.X = ctx, ls, hp, W, X
        self._step()                      # sizes the context's scratch; recording may not allocate
        torch.cuda.synchronize()
        ctx.adadim_capture_begin()
        try:
            self._step()
        finally:
            self.graph = ctx.adadim_capture_end()

    def _step(self):
        self.hp.update_prepared(self.X)
        self.ls.score_all(self.W, self.hp, select=True)

    def launch(self):
        """Queues one replay on the current contents of W and X."""
        self.ctx.adadim_graph_launch(self.graph)

    def run(self):
        """Replays the step on the current contents of W and X; returns (best index, dim, clip)."""
        self.launch()
        return self.result()

    def result(self):
        ls = self.ls
        torch.cuda.synchronize()          # the one synchronisation of the step (whatever stream torch is on)
        best = int(ls.best.item())
        dim, clip = ls.cands[best]
        if ls.keep_winner:
            ls.packed = ls._packed[best]
            if ls.meta16:
                ls.meta = ls._meta[best]
            else:
                ls.scales, ls.zeros = ls._scales[best], ls._zeros[best]
        return best, dim, clip

    def close(self):
        self.ctx.adadim_graph_destroy(getattr(self, "graph", None))
        self.graph = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SharedSearch:
    """The same search for several layers of one shape that see the same input (q/k/v, or
    gate/up, of a decoder block): H is formed once and every (layer, dimension) candidate is
    scored by a single adadim_layer_error_batch launch, which fetches the prepared H once for
    all of them.  At most four layers (eight candidates, the batch limit)."""

    def __init__(self, ctx: B.Context, n_layers: int, out_f: int, in_f: int, bits: int, group: int, device="cuda"):
        if not 1 <= n_layers <= 4:
            raise ValueError("SharedSearch takes 1..4 layers")
        self.ctx, self.n_layers, self.out_f, self.in_f, self.bits, self.group = ctx, n_layers, out_f, in_f, bits, group
        n_c = 2 * n_layers
        self.dWs = [ctx.alloc_score(out_f, in_f, device) for _ in range(n_c)]
        self.losses = torch.empty(n_c, dtype=torch.float32, device=device)      # [layer][oc, ic]
        self.best = torch.empty(n_layers, dtype=torch.int32, device=device)
        g_oc = in_f if group == 0 else group
        g_ic = out_f if group == 0 else group
        n_meta = max(out_f * (in_f // g_oc), (out_f // g_ic) * in_f)
        words = max(out_f * ((in_f * bits + 31) // 32), in_f * ((out_f * bits + 31) // 32))
        self._scales = [torch.empty(n_meta, dtype=torch.float32, device=device) for _ in range(n_c)]
        self._zeros = [torch.empty(n_meta, dtype=torch.uint8, device=device) for _ in range(n_c)]
        self._packed = [torch.empty(words, dtype=torch.int32, device=device) for _ in range(n_c)]
        self.scales = self.zeros = self.packed = None

    def run(self, Ws, hp: PreparedHessian):
        """Ws: the layers' weights.  Returns the list of chosen dimensions (one host sync); the
        winners' packed codes, scales and zeros are in self.packed[l] / self.scales[l] / self.zeros[l]."""
        self.launch(Ws, hp)
        return self.result()

    def launch(self, Ws, hp: PreparedHessian):
        """Queues the search of all the layers; nothing waits."""
        assert len(Ws) == self.n_layers
        for l, W in enumerate(Ws):
            sets = [{"dW": self.dWs[k], "scales": self._scales[k], "zeros": self._zeros[k], "packed": self._packed[k]}
                    for k in (2 * l, 2 * l + 1)]                   # k = 2 l + dim
            self.ctx.adadim_quantize_both(W, self.bits, self.group, hp.colscale, sets[0], sets[1])
        self.ctx.adadim_layer_error_batch(self.dWs, B.DW_F16_SCALED, hp.Hs, hp.hmeta, self.losses,
                                          shape=(self.out_f, self.in_f))
        for l in range(self.n_layers):
            self.ctx.adadim_select(self.losses[2 * l:2 * l + 2], best_dev=self.best[l:l + 1], to_host=False)

    def result(self):
        torch.cuda.synchronize()
        dims = self.best.cpu().tolist()          # the one synchronisation
        self.scales = [self._scales[2 * l + d] for l, d in enumerate(dims)]
        self.zeros = [self._zeros[2 * l + d] for l, d in enumerate(dims)]
        self.packed = [self._packed[2 * l + d] for l, d in enumerate(dims)]
        return dims


class GptqFactor:
    """Visiting order, dead-channel flags and the factor U of the inverse Hessian (adadim_gptq_prepare);
    depends on H only, so one is shared by every layer that sees that input."""

    def __init__(self, ctx: B.Context, hp: PreparedHessian, percdamp: float = 0.01, act_order: bool = True,
                 device="cuda"):
        n = hp.in_f
        self.ctx, self.in_f = ctx, n
        self.perm = torch.empty(n, dtype=torch.int32, device=device)
        self.dead = torch.empty(n, dtype=torch.uint8, device=device)
        self.U = torch.empty((n, n), dtype=torch.float32, device=device)
        self.percdamp, self.act_order = percdamp, act_order
        self.update(hp)

    def update(self, hp: PreparedHessian):
        self.ctx.adadim_gptq_prepare(hp.H, self.perm, self.dead, self.U, self.percdamp, self.act_order)
        return self


class GptqAda:
    """`gptq_ada` of App. B: the RTN search picks the dimension, GPTQ then quantizes in it.
    Per-OC uses the RTN winner's parameters as static groups; per-IC (group 64 or 128) recomputes
    them channel by channel.  Results: codes u8 [out, in], scales, zeros, packed; `loss_rtn` and
    `loss_gptq` (device scalars) are the layer errors before and after.  meta16: search and sweep in
    the b + 16/g storage format; the parameters are then the group words in `meta`."""

    def __init__(self, ctx: B.Context, out_f: int, in_f: int, bits: int, group: int, device="cuda", meta16: bool = False):
        self.ctx, self.out_f, self.in_f, self.bits, self.group = ctx, out_f, in_f, bits, group
        self.meta16 = meta16
        self.search = LayerSearch(ctx, out_f, in_f, bits, group, clips=(1.0,), meta16=meta16)
        self.codes = torch.empty((out_f, in_f), dtype=torch.uint8, device=device)
        self.dW = torch.empty((out_f, in_f), dtype=torch.float32, device=device)
        self.loss_gptq = torch.empty(1, dtype=torch.float32, device=device)
        g_ic = out_f if group == 0 else group
        self.ic_scales = torch.empty((out_f // g_ic, in_f), dtype=torch.float32, device=device)
        self.ic_zeros = torch.empty((out_f // g_ic, in_f), dtype=torch.uint8, device=device)
        self.ic_meta = torch.empty((out_f // g_ic, in_f), dtype=torch.int16, device=device) if meta16 else None
        self.scales = self.zeros = self.meta = None
        self.packed = self.search._packed[0]

    def run(self, W, hp: PreparedHessian, fac: GptqFactor):
        best, dim, _ = self.search.run(W, hp)
        self.loss_rtn = self.search.losses[best:best + 1]
        if self.meta16:
            self.meta = self.search.meta if dim == B.DIM_OC else self.ic_meta
            self.ctx.adadim_gptq_quantize_meta16(W, dim, self.bits, self.group, fac.U, fac.perm, fac.dead, self.codes,
                                                 static_meta=self.meta if dim == B.DIM_OC else None,
                                                 meta=None if dim == B.DIM_OC else self.meta, dW=self.dW,
                                                 packed=self.packed)
        elif dim == B.DIM_OC:
            # static groups: the search's per-OC parameters (of the weight as given; a layer with dead
            # input channels should be passed with those columns already zero)
            self.scales, self.zeros = self.search.scales, self.search.zeros
            self.ctx.adadim_gptq_quantize(W, dim, self.bits, self.group, fac.U, fac.perm, fac.dead, self.codes,
                                          static_scales=self.scales, static_zeros=self.zeros, dW=self.dW,
                                          packed=self.packed)
        else:
            self.scales, self.zeros = self.ic_scales, self.ic_zeros
            self.ctx.adadim_gptq_quantize(W, dim, self.bits, self.group, fac.U, fac.perm, fac.dead, self.codes,
                                          scales=self.scales, zeros=self.zeros, dW=self.dW, packed=self.packed)
        self.ctx.adadim_layer_error_prepared(self.dW, B.DW_F32, hp.Hs, hp.hmeta, self.loss_gptq)
        return dim
