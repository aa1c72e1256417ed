"""CPU oracle for the per-IC de-quantizing matrix-vector product.

TEST INFRASTRUCTURE ONLY (see adadim_oracle.py for the rules): imported by the
tests, the smoke check and the benchmark's cpu_baseline leg, never by the
product, and it shares no code with the HIP sources.

What it computes (paper Sec. 4.5 and App. D, "Per-IC Kernel"): the output of a
linear layer whose weight is stored per-IC quantized, for one fp16 activation
vector x (batch 1, the setting of the latency table in App. D):

    y[o] = sum_j What[o, j] * x[j],   What[o, j] = scale[o//g, j] * (code[o, j] - zero[o//g, j])

with the groups of g consecutive output channels inside each input column of
Sec. 3.2.  The paper folds the per-IC scale into the activation when it builds
its look-up tables; that is a re-association of the same sum, so the oracle is
the plain definition: What formed in fp32 exactly as the quantizer defines it
(one fp32 multiply per weight), the sum in fp64, x taken as the exact fp16
values.  The codes come from the packed stream (this build's format, see
adadim_oracle.pack): [in, ceil(out*b/32)] uint32, code o of column j at bits
[o*b, (o+1)*b) of that column's stream.

`abs_terms` returns sum_j |scale*x|*(code + zero), the size of the partial sums
a kernel that accumulates scale*x*code and scale*x*zero separately goes through;
the GPU tolerance is stated against it.
"""
from __future__ import annotations

import numpy as np


def _codes_from_stream(packed, out_f: int, bits: int) -> np.ndarray:
    """uint32 [in, words] -> codes u8 [out, in] (bit k*b.. of column j's stream is code k)."""
    pk = np.asarray(packed, dtype=np.uint32).astype(np.uint64)
    in_f = pk.shape[0]
    codes = np.zeros((out_f, in_f), dtype=np.uint8)
    mask = np.uint64((1 << bits) - 1)
    for o in range(out_f):
        wd, sh = divmod(o * bits, 32)
        v = pk[:, wd] >> np.uint64(sh)
        if sh + bits > 32:
            v = v | (pk[:, wd + 1] << np.uint64(32 - sh))
        codes[o, :] = (v & mask).astype(np.uint8)
    return codes


def dequantize_ic(packed, scales, zeros, out_f: int, bits: int, group: int) -> np.ndarray:
    """fp32 What[out, in] from the per-IC packed stream, scales f32 [out/g, in], zeros u8 [out/g, in]."""
    g = out_f if group == 0 else group
    codes = _codes_from_stream(packed, out_f, bits).astype(np.int32)
    sc = np.repeat(np.asarray(scales, dtype=np.float32), g, axis=0)
    zp = np.repeat(np.asarray(zeros, dtype=np.uint8).astype(np.int32), g, axis=0)
    return sc * (codes - zp).astype(np.float32)          # one fp32 multiply per weight


def gemv_ic(packed, scales, zeros, x, out_f: int, bits: int, group: int) -> np.ndarray:
    """y fp64 [out] = What @ x (What fp32 as the quantizer defines it, x the exact fp16 values)."""
    What = dequantize_ic(packed, scales, zeros, out_f, bits, group).astype(np.float64)
    return What @ np.asarray(x).astype(np.float64)


def abs_terms(packed, scales, zeros, x, out_f: int, bits: int, group: int) -> np.ndarray:
    """sum_j |scale*x| * (code + zero) per output, fp64."""
    g = out_f if group == 0 else group
    codes = _codes_from_stream(packed, out_f, bits).astype(np.float64)
    sc = np.repeat(np.asarray(scales, dtype=np.float64), g, axis=0)
    zp = np.repeat(np.asarray(zeros).astype(np.float64), g, axis=0)
    ax = np.abs(sc * np.asarray(x).astype(np.float64)[None, :])
    return (ax * (codes + zp)).sum(axis=1)
