"""Seeded synthetic inputs: LLaMA-shaped linear weights and calibration activations.

These stand in for the LLaMA-family checkpoints and the calibration text the
paper uses (Sec. 4.1), neither of which is available here.  The module only
draws random numbers and applies the outlier structure; it contains none of
the method's arithmetic, and it is the one module that both the tests of the
CPU oracle and the GPU path use, so that both see identical fp16 bits.

Structure reproduced (paper Sec. 2.2 / 3.1): a few hidden dimensions of the
activations carry outliers that are tens of times larger than the rest and are
the same dimensions for every token; a small share of the weight's input
channels is heavier than the rest.
"""
from __future__ import annotations

import numpy as np

_CHUNK_ROWS = 4096


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([int(seed), int(stream)]))


def make_weight(out_f: int, in_f: int, seed: int, heavy_cols, heavy_scale: float,
                sigma: float = 0.02) -> np.ndarray:
    """W fp16 [out, in] ~ N(0, sigma^2); `heavy_cols` input columns (a count, or a
    fraction of `in` if < 1) are multiplied by `heavy_scale`."""
    rng = _rng(seed, 1)
    n_heavy = int(round(heavy_cols * in_f)) if 0 < heavy_cols < 1 else int(heavy_cols)
    cols = np.sort(rng.choice(in_f, size=n_heavy, replace=False)) if n_heavy else np.zeros(0, np.int64)
    col_scale = np.ones(in_f, dtype=np.float32)
    col_scale[cols] = np.float32(heavy_scale)
    W = np.empty((out_f, in_f), dtype=np.float16)
    for r0 in range(0, out_f, _CHUNK_ROWS):
        r1 = min(out_f, r0 + _CHUNK_ROWS)
        blk = rng.standard_normal((r1 - r0, in_f), dtype=np.float32)
        blk *= np.float32(sigma)
        blk *= col_scale[None, :]
        W[r0:r1] = blk.astype(np.float16)
    return W


def make_activations(tokens: int, in_f: int, seed: int, n_outliers: int,
                     scale_lo: float, scale_hi: float, relu: bool = False) -> np.ndarray:
    """X fp16 [tokens, in] ~ N(0,1) (or max(0, N(0,1)) if `relu`); `n_outliers`
    channels, shared by all tokens, are multiplied by a per-channel factor drawn
    uniformly from [scale_lo, scale_hi]."""
    rng = _rng(seed, 2)
    ch = np.sort(rng.choice(in_f, size=n_outliers, replace=False)) if n_outliers else np.zeros(0, np.int64)
    ch_scale = np.ones(in_f, dtype=np.float32)
    ch_scale[ch] = rng.uniform(scale_lo, scale_hi, size=n_outliers).astype(np.float32)
    X = np.empty((tokens, in_f), dtype=np.float16)
    for r0 in range(0, tokens, _CHUNK_ROWS):
        r1 = min(tokens, r0 + _CHUNK_ROWS)
        blk = rng.standard_normal((r1 - r0, in_f), dtype=np.float32)
        if relu:
            np.maximum(blk, np.float32(0), out=blk)
        blk *= ch_scale[None, :]
        X[r0:r1] = blk.astype(np.float16)
    return X


def on_grid_weight(out_f: int, in_f: int, dim: int, bits: int, group: int, seed: int):
    """A weight that already lies on a quantization grid: W = s*(q - z) with a
    power-of-two s per group, every group containing codes 0 and qmax.  Returns
    (W fp16, q u8, z u8, s f32) with q in W's index space and z, s in the
    group-parameter layout of `dim` (0: [out, in/g], 1: [out/g, in])."""
    rng = _rng(seed, 3)
    qmax = (1 << bits) - 1
    if dim == 0:
        n_ch, n_ax = out_f, in_f
    else:
        n_ch, n_ax = in_f, out_f
    g = n_ax if group == 0 else group
    n_g = n_ax // g
    q = rng.integers(0, qmax + 1, size=(n_ch, n_g, g), dtype=np.int64)
    pos = rng.integers(0, g, size=(n_ch, n_g))
    pos2 = (pos + 1 + rng.integers(0, g - 1, size=(n_ch, n_g))) % g
    np.put_along_axis(q, pos[:, :, None], 0, axis=2)
    np.put_along_axis(q, pos2[:, :, None], qmax, axis=2)
    z = rng.integers(0, qmax + 1, size=(n_ch, n_g), dtype=np.int64)
    e = rng.integers(-9, -3, size=(n_ch, n_g))
    s = np.ldexp(np.float32(1.0), e).astype(np.float32)
    Wt = (s[:, :, None] * (q - z[:, :, None]).astype(np.float32)).reshape(n_ch, n_ax)
    qt = q.reshape(n_ch, n_ax)
    if dim == 0:
        return Wt.astype(np.float16), qt.astype(np.uint8), z.astype(np.uint8), s
    return (np.ascontiguousarray(Wt.T).astype(np.float16), np.ascontiguousarray(qt.T).astype(np.uint8),
            np.ascontiguousarray(z.T).astype(np.uint8), np.ascontiguousarray(s.T))


# The five workloads.  `layers` maps a name to (out, in); `x` gives the
# activation recipe per input width.
CONFIGS = {
    0: dict(name="toy-512", tokens=256, bits=(3,), group=64, clips=1,
            layers={"fc": (512, 512)}, heavy_cols=4, heavy_scale=8.0,
            outliers={512: (3, 60.0, 60.0)}, relu_widths=(), seed=0),
    1: dict(name="llama7b-q_proj", tokens=65536, bits=(3,), group=128, clips=1,
            layers={"q_proj": (4096, 4096)}, heavy_cols=0.01, heavy_scale=5.0,
            outliers={4096: (8, 50.0, 100.0)}, relu_widths=(), seed=1),
    2: dict(name="llama7b-block", tokens=65536, bits=(4, 3), group=128, clips=1,
            layers={"q_proj": (4096, 4096), "k_proj": (4096, 4096), "v_proj": (4096, 4096),
                    "o_proj": (4096, 4096), "gate_proj": (11008, 4096), "up_proj": (11008, 4096),
                    "down_proj": (4096, 11008)},
            heavy_cols=0.01, heavy_scale=5.0,
            outliers={4096: (8, 50.0, 100.0), 11008: (8, 50.0, 100.0)}, relu_widths=(11008,), seed=2),
    3: dict(name="llama13b-stream", tokens=131072, bits=(3,), group=128, clips=1, blocks=40,
            layers={"q_proj": (5120, 5120), "k_proj": (5120, 5120), "v_proj": (5120, 5120),
                    "o_proj": (5120, 5120), "gate_proj": (13824, 5120), "up_proj": (13824, 5120),
                    "down_proj": (5120, 13824)},
            heavy_cols=0.01, heavy_scale=5.0,
            outliers={5120: (10, 80.0, 80.0), 13824: (28, 80.0, 80.0)}, relu_widths=(13824,), seed=3),
    4: dict(name="llama70b-gqa-clipgrid", tokens=65536, bits=(2, 3), group=64, clips=20,
            layers={"q_proj": (8192, 8192), "k_proj": (1024, 8192), "v_proj": (1024, 8192),
                    "o_proj": (8192, 8192), "gate_proj": (28672, 8192), "up_proj": (28672, 8192),
                    "down_proj": (8192, 28672)},
            heavy_cols=0.01, heavy_scale=5.0,
            outliers={8192: (8, 100.0, 100.0), 28672: (8, 100.0, 100.0)}, relu_widths=(28672,), seed=4),
}


def config_weight(cfg_id: int, layer: str, block: int = 0) -> np.ndarray:
    cfg = CONFIGS[cfg_id]
    out_f, in_f = cfg["layers"][layer]
    return make_weight(out_f, in_f, layer_seed(cfg_id, layer, block), cfg["heavy_cols"], cfg["heavy_scale"])


def config_activations(cfg_id: int, in_f: int, tokens: int | None = None) -> np.ndarray:
    cfg = CONFIGS[cfg_id]
    n, lo, hi = cfg["outliers"][in_f]
    t = cfg["tokens"] if tokens is None else tokens
    return make_activations(t, in_f, cfg["seed"] * 100003 + 7 * in_f, n, lo, hi,
                            relu=in_f in cfg["relu_widths"])


# ---------------------------------------------------------------------------------------------
# The same recipes drawn on the device, for inputs too large to draw on the host per use (the
# streamed 40-block workload regenerates 317 M weights per block; its 131072 x 13824 activation
# matrix is 3.6 GB).  torch's seeded device generator replaces numpy's; the structure (which
# channels are heavy, their factors) is still drawn on the host from the same seeded streams as
# above (for weights, on the device as well).  A test that needs the values on the host copies the tensor back: the bits the oracle
# sees are the bits the device holds.

def device_weight(out_f: int, in_f: int, seed: int, heavy_cols, heavy_scale: float, sigma: float = 0.02,
                  out=None, scratch=None, device="cuda"):
    """W fp16 [out, in] on the device, same law as make_weight (different random bits).  `out` (fp16
    [out, in]) and `scratch` (fp32 [out, in]) let a streaming caller reuse its buffers."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    buf = scratch if scratch is not None else torch.empty((out_f, in_f), dtype=torch.float32, device=device)
    buf.normal_(0.0, float(sigma), generator=g)
    # the heavy columns are drawn on the device too (a host-drawn scale vector would cost a blocking copy per
    # layer, and the streaming driver must be able to queue a block without waiting for the GPU)
    n_heavy = int(round(heavy_cols * in_f)) if 0 < heavy_cols < 1 else int(heavy_cols)
    if n_heavy:
        cols = torch.randperm(in_f, generator=g, device=device)[:n_heavy]
        buf[:, cols] *= float(heavy_scale)
    if out is None:
        return buf.to(torch.float16)
    out.copy_(buf)
    return out


def device_activations(tokens: int, in_f: int, seed: int, n_outliers: int, scale_lo: float, scale_hi: float,
                       relu: bool = False, device="cuda", chunk_rows: int = 16384):
    """X fp16 [tokens, in] on the device, same law as make_activations (different random bits)."""
    import torch
    rng = _rng(seed, 2)
    ch = np.sort(rng.choice(in_f, size=n_outliers, replace=False)) if n_outliers else np.zeros(0, np.int64)
    ch_scale = np.ones(in_f, dtype=np.float32)
    ch_scale[ch] = rng.uniform(scale_lo, scale_hi, size=n_outliers).astype(np.float32)
    cs = torch.from_numpy(ch_scale).to(device)[None, :]
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    X = torch.empty((tokens, in_f), dtype=torch.float16, device=device)
    buf = torch.empty((min(chunk_rows, tokens), in_f), dtype=torch.float32, device=device)
    for r0 in range(0, tokens, chunk_rows):
        r1 = min(tokens, r0 + chunk_rows)
        b = buf[:r1 - r0]
        b.normal_(0.0, 1.0, generator=g)
        if relu:
            b.clamp_(min=0.0)
        b.mul_(cs)
        X[r0:r1].copy_(b)
    return X


def layer_seed(cfg_id: int, layer: str, block: int = 0) -> int:
    """Seed of one layer's weight: the workload's seed plus the layer's id within the model."""
    cfg = CONFIGS[cfg_id]
    return cfg["seed"] * 100003 + block * 101 + sorted(cfg["layers"]).index(layer)


def config_weight_device(cfg_id: int, layer: str, block: int = 0, out=None, scratch=None):
    cfg = CONFIGS[cfg_id]
    out_f, in_f = cfg["layers"][layer]
    return device_weight(out_f, in_f, layer_seed(cfg_id, layer, block), cfg["heavy_cols"], cfg["heavy_scale"],
                         out=out, scratch=scratch)


def config_activations_device(cfg_id: int, in_f: int, tokens: int | None = None):
    cfg = CONFIGS[cfg_id]
    n, lo, hi = cfg["outliers"][in_f]
    t = cfg["tokens"] if tokens is None else tokens
    return device_activations(t, in_f, cfg["seed"] * 100003 + 7 * in_f, n, lo, hi, relu=in_f in cfg["relu_widths"])
