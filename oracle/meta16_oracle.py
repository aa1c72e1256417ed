"""CPU oracle for the 16-bit-per-group storage format.

TEST INFRASTRUCTURE ONLY (see adadim_oracle.py for the rules): imported by the
tests, the smoke check and the benchmark's cpu_baseline leg, never by the
product, and it shares no code with the HIP sources.

The paper counts the storage of a group-wise quantized weight as b + 16/g bits
per weight (Sec. 4.1 states INT3/INT4 with group size 128; the "Avg Bits"
columns of the SpQR comparison in App. C print 4.125 for b = 4, g = 128 and
4.00 / 3.50 / 3.25 for b = 3, g = 16 / 32 / 64): sixteen bits of parameters per
group.  The paper does not say how a scale and a zero-point share those sixteen
bits; the format below is this build's own reading and is "parity unpinned"
with respect to the authors' code:

    word = pattern << b | zero          one uint16 per group, b in {2, 3, 4}
    zero     the b-bit zero-point
    pattern  the leading 16-b bits of the 15-bit fp16 pattern of the scale (the
             sign bit is always 0): an unsigned float with fp16's exponent
             field and 11-b fraction bits; scale = fp16(pattern << (b-1)).

Rounding of the fp32 scale into the format: to fp16, nearest even; then to the
nearest pattern, ties to the even pattern (the fp16 encoding is monotone, so
this is nearest-even in value as well, inside a binade and across binades); a
pattern of 0 is replaced by 1, the smallest positive value, so that the scale
never vanishes.  The zero-point, the codes and dW are computed from the rounded
scale with the quantizer's own formulas (adadim_oracle.quantize), which makes
the stored word de-quantize to exactly the weights that were scored.
"""
from __future__ import annotations

import numpy as np

from . import adadim_oracle as _q
from . import gemv_oracle as _g
from . import gptq_oracle as _gq


def _check_bits(bits: int) -> int:
    if bits not in (2, 3, 4):
        raise ValueError("the 16-bit group word holds 2-, 3- or 4-bit zero-points")
    return bits - 1


def scale_pattern(scale, bits: int) -> np.ndarray:
    """(16-b)-bit pattern of each fp32 scale (> 0), rounded as the module text states."""
    d = _check_bits(bits)
    h = np.asarray(scale, dtype=np.float32).astype(np.float16).view(np.uint16).astype(np.int64)
    kept, dropped = h >> d, h & ((1 << d) - 1)
    half = 1 << (d - 1)
    up = (dropped > half) | ((dropped == half) & ((kept & 1) == 1))
    return np.maximum(kept + up.astype(np.int64), 1).astype(np.uint16)


def pattern_value(pattern, bits: int) -> np.ndarray:
    """fp32 value of a pattern."""
    d = _check_bits(bits)
    return (np.asarray(pattern, dtype=np.uint16).astype(np.uint32) << d).astype(np.uint16).view(np.float16).astype(np.float32)


def round_scale(scale, bits: int) -> np.ndarray:
    """fp32 scales rounded to the values the group word can hold."""
    return pattern_value(scale_pattern(scale, bits), bits)


def encode(scales, zeros, bits: int) -> np.ndarray:
    """uint16 words from scales that are already values of the format and b-bit zero-points."""
    pat = scale_pattern(scales, bits).astype(np.uint32)
    if not np.array_equal(pattern_value(pat, bits), np.asarray(scales, dtype=np.float32)):
        raise ValueError("scales are not values of the 16-bit group format")
    z = np.asarray(zeros).astype(np.uint32)
    if (z >> bits).any():
        raise ValueError("zero-point does not fit in b bits")
    return ((pat << bits) | z).astype(np.uint16)


def decode(meta, bits: int):
    """(scales f32, zeros u8) from uint16 group words."""
    m = np.asarray(meta, dtype=np.uint16).astype(np.uint32)
    return pattern_value(m >> bits, bits), (m & ((1 << bits) - 1)).astype(np.uint8)


def quantize(W, dim: int, bits: int, group: int, clip: float = 1.0) -> dict:
    """adadim_oracle.quantize with the scale rounded into the group word; adds "meta" (uint16, the
    shape of scales)."""
    _check_bits(bits)
    r = _q.quantize(W, dim, bits, group, clip, scale_round=lambda s: round_scale(s, bits))
    r["meta"] = encode(r["scales"], r["zeros"], bits)
    return r


def stored_bits_per_weight(out_f: int, in_f: int, dim: int, bits: int, group: int) -> float:
    """Bits per weight of the packed code stream plus the group words, counted on the arrays themselves."""
    axis = in_f if dim == _q.OC else out_f
    g = axis if group == 0 else group
    n_ch = out_f if dim == _q.OC else in_f
    code_bits = n_ch * ((axis * bits + 31) // 32) * 32
    meta_bits = n_ch * (axis // g) * 16
    return (code_bits + meta_bits) / (out_f * in_f)


def gemv_ic(packed, meta, x, out_f: int, bits: int, group: int) -> np.ndarray:
    """y fp64 [out] for a per-IC weight stored as code stream + group words (paper Sec. 4.5, App. D)."""
    scales, zeros = decode(meta, bits)
    return _g.gemv_ic(packed, scales, zeros, x, out_f, bits, group)


def abs_terms(packed, meta, x, out_f: int, bits: int, group: int) -> np.ndarray:
    scales, zeros = decode(meta, bits)
    return _g.abs_terms(packed, scales, zeros, x, out_f, bits, group)


def gptq_sweep(W, U, perm, dead, dim: int, bits: int, group: int) -> dict:
    """gptq_oracle.sweep (GPTQ in the selected dimension, paper Sec. 3.3 / App. A.1) with every scale rounded into
    the group word before it is used; adds "meta" (uint16, the shape of scales)."""
    _check_bits(bits)
    r = _gq.sweep(W, U, perm, dead, dim, bits, group, scale_round=lambda s: round_scale(s, bits))
    r["meta"] = encode(r["scales"], r["zeros"], bits)
    return r
