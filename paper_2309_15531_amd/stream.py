"""The search applied to every linear layer of a model, one decoder block after the other
(Sec. 3.3: the dimension is chosen per layer; App. C uses 256 x 512 calibration tokens).

Call order and bookkeeping only; all arithmetic happens in libadadim.so.

* `ResultsLog`: the per-layer results file.  One JSON line per (seed, block, layer name, bits, group);
  a rerun skips the keys that are present, so a 40-block run that was interrupted resumes where it
  stopped.  Pure Python, no GPU needed.
* `BlockSearch`: the buffers and the call sequence for the layers of one decoder block: one Gram matrix
  per distinct input width, layers of one shape that see the same input scored in one launch, every
  result left on the device until the block is collected, so block b + 1 is queued while block b's
  answers are on their way to the host.
* `run_stream`: the loop over blocks with the log.
"""
from __future__ import annotations

import json
import math
import os


from . import binding as B

KEY_FIELDS = ("seed", "block", "layer", "bits", "group")


class ResultsLog:
    """JSON-lines file of per-layer results keyed by (seed, block, layer, bits, group).

    Opening an existing file loads its records; a last line that was cut off (the process died while writing it) is
    dropped and the file truncated back to the last whole record.  `append` writes one line and flushes it to the
    file system before it returns, so a record that `has` reports is on disk."""

    def __init__(self, path: str):
        self.path = path
        self.records: dict[tuple, dict] = {}
        good_end = 0
        if os.path.exists(path):
            with open(path, "rb") as f:
                data = f.read()
            pos = 0
            while pos < len(data):
                nl = data.find(b"\n", pos)
                if nl < 0:
                    break                                  # no newline: an unfinished record
                line = data[pos:nl].strip()
                if line:
                    try:
                        rec = json.loads(line)
                        self.records[self.key_of(rec)] = rec
                    except (ValueError, KeyError):
                        break                              # a damaged record: keep what came before it
                pos = nl + 1
                good_end = pos
            if good_end != len(data):
                with open(path, "r+b") as f:
                    f.truncate(good_end)
        self._f = open(path, "ab")

    @staticmethod
    def key(seed: int, block: int, layer: str, bits: int, group: int) -> tuple:
        return (int(seed), int(block), str(layer), int(bits), int(group))

    @classmethod
    def key_of(cls, rec: dict) -> tuple:
        return cls.key(*(rec[k] for k in KEY_FIELDS))

    def has(self, key: tuple) -> bool:
        return key in self.records

    def get(self, key: tuple):
        return self.records.get(key)

    def append(self, rec: dict) -> None:
        self.append_many([rec])

    def append_many(self, recs) -> None:
        """Writes the records (one line each) and flushes them to the file system once, for all of them: a block's
        seven records cost one fsync, not seven."""
        keys = [self.key_of(r) for r in recs]              # raises KeyError if a key field is missing
        for k in keys:
            if k in self.records or keys.count(k) > 1:
                raise ValueError(f"record {k} is already in {self.path}")
        self._f.write("".join(json.dumps(r, sort_keys=True) + "\n" for r in recs).encode())
        self._f.flush()
        os.fsync(self._f.fileno())
        self.records.update(zip(keys, recs))

    def __len__(self) -> int:
        return len(self.records)

    def close(self) -> None:
        if self._f:
            self._f.close()
            self._f = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def pending_layers(log: ResultsLog, seed: int, blocks, layer_names, bits_list, group: int):
    """[(block, [(layer, bits), ...])] still to be searched, in running order; blocks with nothing left are left out."""
    todo = []
    for b in blocks:
        rest = [(name, bits) for bits in bits_list for name in layer_names
                if not log.has(ResultsLog.key(seed, b, name, bits, group))]
        if rest:
            todo.append((b, rest))
    return todo


class _Group:
    """Up to four layers of one shape that see the same input: two candidates each, scored by one launch."""

    def __init__(self, ctx, names, out_f, in_f, bits_max, group, device):
        import torch
        self.names, self.out_f, self.in_f = list(names), out_f, in_f
        n_c = 2 * len(self.names)
        g_oc = in_f if group == 0 else group
        g_ic = out_f if group == 0 else group
        n_meta = max(out_f * (in_f // g_oc), (out_f // g_ic) * in_f)
        words = max(out_f * ((in_f * bits_max + 31) // 32), in_f * ((out_f * bits_max + 31) // 32))
        self.dWs = [ctx.alloc_score(out_f, in_f, device) for _ in range(n_c)]
        self.scales = [torch.empty(n_meta, dtype=torch.float32, device=device) for _ in range(n_c)]
        self.zeros = [torch.empty(n_meta, dtype=torch.uint8, device=device) for _ in range(n_c)]
        self.packed = [torch.empty(words, dtype=torch.int32, device=device) for _ in range(n_c)]


class BlockSearch:
    """The search over the linear layers of one decoder block shape (plain two-candidate search, clip 1).

    layers: {name: (out, in)}; layers with the same shape are taken to see the same input (q/k/v/o, gate/up: one
    activation matrix per input width, as the workloads here provide them).  Results of a launched block stay on the
    device in one of two result slots, so the next block can be queued before the last one is collected.  The
    winner's packed codes, scales and zeros of each (layer, bits) are in `outputs(name)` until the next block's
    launch overwrites them."""

    def __init__(self, ctx: B.Context, layers: dict, bits_list, group: int, device="cuda"):
        import torch
        self.ctx, self.group, self.device = ctx, group, device
        self.bits_list = tuple(bits_list)
        self.layers = dict(layers)
        self.names = list(layers)
        by_shape: dict[tuple, list] = {}
        for name, shape in layers.items():
            by_shape.setdefault(tuple(shape), []).append(name)
        self.groups = []
        for (out_f, in_f), names in by_shape.items():
            for i in range(0, len(names), 4):
                self.groups.append(_Group(ctx, names[i:i + 4], out_f, in_f, max(self.bits_list), group, device))
        self.widths = sorted({in_f for _, in_f in layers.values()})
        self.H = {w: torch.empty((w, w), dtype=torch.float32, device=device) for w in self.widths}
        self.Hs = {w: ctx.alloc_score(w, w, device) for w in self.widths}
        self.hmeta = {w: torch.empty((2, w), dtype=torch.float32, device=device) for w in self.widths}
        n_l, n_b = len(self.names), len(self.bits_list)
        self.slot_of = {(name, bits): bi * n_l + li for bi, bits in enumerate(self.bits_list)
                        for li, name in enumerate(self.names)}
        # two result slots: losses [n_bits * n_layers, 2] and winners [n_bits * n_layers], with pinned host mirrors
        self.losses = [torch.zeros((n_b * n_l, 2), dtype=torch.float32, device=device) for _ in range(2)]
        self.best = [torch.zeros(n_b * n_l, dtype=torch.int32, device=device) for _ in range(2)]
        self.h_losses = [torch.zeros((n_b * n_l, 2), dtype=torch.float32, pin_memory=True) for _ in range(2)]
        self.h_best = [torch.zeros(n_b * n_l, dtype=torch.int32, pin_memory=True) for _ in range(2)]
        self.done = [torch.cuda.Event() for _ in range(2)]
        self.copied = [torch.cuda.Event() for _ in range(2)]
        self.copy_stream = torch.cuda.Stream()
        self._launched = [None, None]

    def hessians(self, X: dict):
        """H, its prepared form and the column scales for every input width, from X[width] (fp16 [tokens, width])."""
        for w in self.widths:
            self.ctx.adadim_hessian_prepared(X[w], self.H[w], self.Hs[w], self.hmeta[w])

    def launch(self, slot: int, weights: dict, only=None):
        """Queues the search of every (layer, bits) of the block (or of the pairs in `only`) on the weights
        {name: fp16 [out, in] device tensor}; the Gram matrices must have been queued before (`hessians`).
        Nothing waits."""
        import torch
        ctx, want = self.ctx, (None if only is None else set(only))
        launched = []
        for bits in self.bits_list:
            for g in self.groups:
                names = [n for n in g.names if want is None or (n, bits) in want]
                if not names:
                    continue
                for k, name in enumerate(names):
                    sets = [{"dW": g.dWs[2 * k + d], "scales": g.scales[2 * k + d], "zeros": g.zeros[2 * k + d],
                             "packed": g.packed[2 * k + d]} for d in (0, 1)]
                    ctx.adadim_quantize_both(weights[name], bits, self.group, self.hmeta[g.in_f][0], sets[0], sets[1])
                rows = [self.slot_of[(n, bits)] for n in names]
                contiguous = rows == list(range(rows[0], rows[0] + len(rows)))
                dst = self.losses[slot][rows[0]:rows[0] + len(rows)] if contiguous else \
                    torch.empty((len(rows), 2), dtype=torch.float32, device=self.device)
                ctx.adadim_layer_error_batch(g.dWs[:2 * len(names)], B.DW_F16_SCALED, self.Hs[g.in_f], self.hmeta[g.in_f],
                                             dst, shape=(g.out_f, g.in_f))
                for k, r in enumerate(rows):
                    if not contiguous:
                        self.losses[slot][r].copy_(dst[k])
                    ctx.adadim_select(self.losses[slot][r], n=2, best_dev=self.best[slot][r:r + 1], to_host=False)
                launched += [(n, bits) for n in names]
        self.done[slot].record()
        self._launched[slot] = launched

    def collect(self, slot: int):
        """Waits for the block launched into `slot` (and for nothing queued after it) and returns
        [{layer, bits, dim, L_oc, L_ic}] in launch order."""
        import torch
        with torch.cuda.stream(self.copy_stream):
            self.copy_stream.wait_event(self.done[slot])
            self.h_losses[slot].copy_(self.losses[slot], non_blocking=True)
            self.h_best[slot].copy_(self.best[slot], non_blocking=True)
            self.copied[slot].record()
        self.copied[slot].synchronize()
        out = []
        for name, bits in self._launched[slot]:
            r = self.slot_of[(name, bits)]
            l = self.h_losses[slot][r].tolist()
            rec = {"layer": name, "bits": int(bits), "dim": "ic" if int(self.h_best[slot][r]) == 1 else "oc",
                   "L_oc": float(l[0]), "L_ic": float(l[1])}
            if not (math.isfinite(l[0]) and math.isfinite(l[1])):
                # |dW| sqrt(H_jj) left fp16's range for some column (the header of adadim_hessian_prepare gives the
                # range): the choice between the two dimensions is then not to be trusted
                rec["nonfinite_loss"] = True
            out.append(rec)
        return out

    def outputs(self, name: str, dim: int):
        """(packed, scales, zeros) buffers of candidate `dim` of layer `name` as the last launch left them (the
        last bit-width of bits_list)."""
        for g in self.groups:
            if name in g.names:
                k = 2 * g.names.index(name) + dim
                return g.packed[k], g.scales[k], g.zeros[k]
        raise KeyError(name)


def run_stream(bs: BlockSearch, log: ResultsLog, seed: int, blocks, weights_of, activations_of, on_block=None):
    """Searches every layer of every block in `blocks` that the log does not hold yet and appends the results.

    weights_of(block, slot) -> {name: W}: the block's weights, produced into buffers that belong to `slot` (0 or
    1: the buffers of block b are still being read while block b + 1 is produced); activations_of(block) ->
    {width: X}.  Block b + 1 is queued before block b is collected.  Returns the number of records written."""
    todo = pending_layers(log, seed, blocks, bs.names, bs.bits_list, bs.group)
    written = 0

    def finish(entry):
        nonlocal written
        b, slot = entry
        recs = bs.collect(slot)
        for rec in recs:
            rec.update(seed=int(seed), block=int(b), group=int(bs.group))
        log.append_many(recs)
        written += len(recs)
        if on_block:
            on_block(b)

    in_flight = None
    for i, (b, rest) in enumerate(todo):
        slot = i & 1
        bs.hessians(activations_of(b))
        bs.launch(slot, weights_of(b, slot), only=rest)
        if in_flight is not None:
            finish(in_flight)
        in_flight = (b, slot)
    if in_flight is not None:
        finish(in_flight)
    return written
