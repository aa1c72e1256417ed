"""CPU oracle for the AdaDim per-layer adaptive-dimension search.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the
GPU library is checked against.  Only the tests, the smoke check and the
benchmark's `cpu_baseline` leg may import it; the product path never does.
It shares no code, table or constant with the HIP sources and imports nothing
from the product package.

What it computes (paper citations):

* group-wise asymmetric b-bit round-to-nearest of a linear weight, with the
  groups taken either inside each output channel ("per-OC", the conventional
  layout) or inside each input channel ("per-IC", the paper's proposal):
  Sec. 2.1 (group-wise per-channel quantization: consecutive weights inside a
  channel share parameters), Sec. 3.2 (per-IC grouping), Sec. 4.1 (uniform
  asymmetric setting, group size 128);
* the reconstruction error of a quantized layer on calibration activations,
  Eq. 1 (Sec. 3.3), both straight from the definition and through the Gram
  matrix H = X^T X (||X dW^T||_F^2 = tr(dW H dW^T));
* the binary choice of the dimension with the lower error, Eq. 1 and the
  `rtn_ada` procedure of App. B (candidates visited in the order oc, ic;
  a later candidate replaces the incumbent only when strictly better).

Precision: the quantizer works in IEEE fp32 one operation at a time (numpy
ufuncs never fuse a multiply into an add), the error in fp64.

Readings taken where the paper is silent (each is listed in the design notes):
the quantization range always contains 0; an all-zero group gets scale 1;
rounding is half-to-even; code = rint(w / scale) + zero with a true division;
scales and de-quantized weights stay fp32; the returned error is the squared
Frobenius sum (Eq. 1's norm squared; the listing's mean times T*out); a clip
ratio c multiplies both ends of the range.

Parity status: the quantizer formula is pinned by closed forms, fixed points,
hand-worked groups, nearest-grid-point brute force and the transpose identity
(tests/test_oracle_pins.py).  That it is *the authors'* formula is
"parity unpinned": the paper prints no worked quantizer example and no
per-layer error value.  The clip ratio is not part of the paper's method and
is likewise "parity unpinned" with respect to the paper.
"""
from __future__ import annotations

import numpy as np

OC = 0  # groups of `group` consecutive input channels inside each output row
IC = 1  # groups of `group` consecutive output channels inside each input column

_F32 = np.float32


def _as_f32_weight(W) -> np.ndarray:
    W = np.asarray(W)
    if W.ndim != 2:
        raise ValueError("W must be 2-D [out, in]")
    return W.astype(_F32)  # fp16 -> fp32 is exact


def quantize(W, dim: int, bits: int, group: int, clip: float = 1.0, scale_round=None) -> dict:
    """Group-wise asymmetric RTN of W[out, in] (Sec. 2.1, 3.2, 4.1).

    dim=OC: group (o, k) is W[o, k*g:(k+1)*g];  dim=IC: group (r, j) is
    W[r*g:(r+1)*g, j].  group == 0 means one group per whole channel.

    Returns codes u8 [out, in]; scales f32 and zeros u8 of shape
    [out, in/g] (OC) or [out/g, in] (IC); What f32 (de-quantized weight);
    dW f32 = W - What.

    scale_round, if given, maps the fp32 scales of step 3 to the values a
    storage format can hold (see meta16_oracle); the zero-point, the codes and
    dW are then computed from the rounded scales.
    """
    w = _as_f32_weight(W)
    out_f, in_f = w.shape
    if dim not in (OC, IC):
        raise ValueError("dim must be OC (0) or IC (1)")
    if not (2 <= bits <= 8):
        raise ValueError("bits must be in [2, 8]")
    c = _F32(clip)
    if not (c > 0 and c <= 1):
        raise ValueError("clip must be in (0, 1]")
    axis_len = in_f if dim == OC else out_f
    g = axis_len if group == 0 else int(group)
    if g <= 0 or axis_len % g != 0:
        raise ValueError("group must divide the grouped axis")
    qmax = _F32((1 << bits) - 1)
    zero_f = _F32(0.0)

    # View the weight as [..., groups, g] with the group axis last.  Per-IC is
    # the same quantizer applied to columns, i.e. to the rows of W^T.
    wt = w if dim == OC else w.T
    n_ch = wt.shape[0]
    grp = np.ascontiguousarray(wt).reshape(n_ch, axis_len // g, g)

    # 1. range that always contains zero
    mx = np.maximum(grp.max(axis=2), zero_f)
    mn = np.minimum(grp.min(axis=2), zero_f)
    # 2. clip ratio shrinks both ends toward zero
    mx = (c * mx).astype(_F32)
    mn = (c * mn).astype(_F32)
    # 3. scale; an empty range (all-zero group) gets scale 1
    rng = (mx - mn).astype(_F32)
    scale = (rng / qmax).astype(_F32)
    scale = np.where(rng == zero_f, _F32(1.0), scale).astype(_F32)
    if scale_round is not None:
        scale = np.asarray(scale_round(scale), dtype=_F32)
    # 4. zero-point
    z = np.rint(((-mn) / scale).astype(_F32)).astype(_F32)
    z = np.minimum(np.maximum(z, zero_f), qmax).astype(_F32)
    # 5. codes
    s3 = scale[:, :, None]
    z3 = z[:, :, None]
    q = (np.rint((grp / s3).astype(_F32)).astype(_F32) + z3).astype(_F32)
    q = np.minimum(np.maximum(q, zero_f), qmax).astype(_F32)
    # 6. de-quantize: exact integer difference, then one multiply
    what = (s3 * (q - z3).astype(_F32)).astype(_F32)
    # 7. weight error
    dw = (grp - what).astype(_F32)

    def back(a3):  # [..., groups, g] -> [out, in]
        a = a3.reshape(n_ch, axis_len)
        return np.ascontiguousarray(a if dim == OC else a.T)

    def back_meta(a2):  # [channels, groups] -> [out, in/g] or [out/g, in]
        return np.ascontiguousarray(a2 if dim == OC else a2.T)

    return {
        "codes": back(q).astype(np.uint8),
        "scales": back_meta(scale).astype(_F32),
        "zeros": back_meta(z).astype(np.uint8),
        "What": back(what),
        "dW": back(dw),
    }


def pack(codes, dim: int, bits: int) -> np.ndarray:
    """Little-endian bitstream of b-bit codes along the grouped axis.

    The stream of one channel (an output row for OC, an input column for IC,
    i.e. a row of the (C_in, C_out) view drawn in the paper's App. A.1 figure)
    is the concatenation of its codes, code k occupying bits [k*b, (k+1)*b) of
    the stream, the stream cut into little-endian uint32 words and padded with
    zero bits to a whole word.  Output: uint32 [channels, ceil(len*b/32)].
    The format is this build's own; the paper does not describe one.
    """
    cd = np.asarray(codes, dtype=np.uint8)
    ch = cd if dim == OC else cd.T
    n_ch, n = ch.shape
    n_words = (n * bits + 31) // 32
    out = np.zeros((n_ch, n_words), dtype=np.uint64)
    for k in range(n):
        bit = k * bits
        wd, sh = divmod(bit, 32)
        v = ch[:, k].astype(np.uint64) << np.uint64(sh)
        out[:, wd] |= v & np.uint64(0xFFFFFFFF)
        if sh + bits > 32:
            out[:, wd + 1] |= v >> np.uint64(32)
    return out.astype(np.uint32)


def unpack(packed, n: int, bits: int) -> np.ndarray:
    """Inverse of `pack` for one orientation: uint32 [channels, words] -> u8 [channels, n]."""
    pk = np.asarray(packed, dtype=np.uint32).astype(np.uint64)
    n_ch = pk.shape[0]
    out = np.zeros((n_ch, n), dtype=np.uint8)
    mask = np.uint64((1 << bits) - 1)
    for k in range(n):
        bit = k * bits
        wd, sh = divmod(bit, 32)
        v = pk[:, wd] >> np.uint64(sh)
        if sh + bits > 32:
            v = v | (pk[:, wd + 1] << np.uint64(32 - sh))
        out[:, k] = (v & mask).astype(np.uint8)
    return out


def bits_per_weight(bits: int, group: int, meta_bits: int = 16) -> float:
    """Average storage per weight when each group carries `meta_bits` of
    parameters.  With 16 bits per group this is the accounting behind the
    "Avg Bits" columns of the SpQR comparison tables (App. C)."""
    return bits + meta_bits / group


def hessian(X) -> np.ndarray:
    """H = X^T X in fp64 for calibration activations X[tokens, in]."""
    x = np.asarray(X).astype(np.float64)
    return x.T @ x


def layer_error_direct(X, W, What) -> float:
    """Eq. 1 squared, straight from the definition: the two layer outputs are
    formed separately in fp64 and their difference is squared and summed."""
    x = np.asarray(X).astype(np.float64)
    y_ref = x @ np.asarray(W).astype(np.float64).T
    y_q = x @ np.asarray(What).astype(np.float64).T
    d = y_q - y_ref
    return float(np.sum(d * d))


def layer_error_rows(dW, H) -> np.ndarray:
    """L_o = dW_o H dW_o^T for every output row o, in fp64."""
    d = np.asarray(dW).astype(np.float64)
    return np.einsum("oj,oj->o", d @ np.asarray(H, dtype=np.float64), d)


def layer_error(dW, H) -> float:
    """L = tr(dW H dW^T) = sum_o L_o in fp64 (equals Eq. 1 squared)."""
    return float(np.sum(layer_error_rows(dW, H)))


def layer_error_rows_from_X(X, dW_rows) -> np.ndarray:
    """L_o = ||X dW_o||^2 in fp64 for a few given rows of dW; used where the
    fp64 Gram matrix is too large to form."""
    x = np.asarray(X).astype(np.float64)
    y = x @ np.asarray(dW_rows).astype(np.float64).T
    return np.sum(y * y, axis=0)


def select(losses) -> int:
    """Index of the first minimum: a later candidate wins only if strictly
    lower (App. B procedure, candidates ordered oc then ic).  The procedure starts
    from a best error of +infinity and replaces it on `err < best_err`, so a NaN loss
    never becomes the best (every comparison with it is false) and an infinite one
    never replaces anything; if no candidate ever wins (all NaN or +inf) the first
    candidate is returned."""
    best, best_err = 0, float("inf")
    for i in range(len(losses)):
        if losses[i] < best_err:
            best, best_err = i, losses[i]
    return best


def clip_grid(n: int = 20, lo: float = 0.5, hi: float = 1.0) -> np.ndarray:
    """n evenly spaced clip ratios in [lo, hi], both ends included, each
    computed in fp64 and rounded once to fp32."""
    if n == 1:
        return np.array([hi], dtype=_F32)
    return np.array([lo + (hi - lo) * i / (n - 1) for i in range(n)], dtype=np.float64).astype(_F32)


def search(W, X, bits: int, group: int, clips=(1.0,), H=None) -> dict:
    """The whole per-layer search: every (dim, clip) candidate in the order
    `for dim in (oc, ic): for clip in clips`, scored through H, first minimum
    kept.  Returns losses, the winning index, dim and clip, and the winner's
    quantization."""
    if H is None:
        H = hessian(X)
    losses, cands = [], []
    for dim in (OC, IC):
        for c in clips:
            qz = quantize(W, dim, bits, group, c)
            losses.append(layer_error(qz["dW"], H))
            cands.append((dim, float(_F32(c))))
    best = select(losses)
    dim, c = cands[best]
    return {
        "losses": losses,
        "best": best,
        "dim": dim,
        "clip": c,
        "quant": quantize(W, dim, bits, group, c),
    }
