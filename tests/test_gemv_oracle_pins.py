"""Pins of the per-IC de-quantizing matrix-vector oracle (CPU only).

The oracle is checked against things other than itself: a hand-worked 4x2 case
(tests/golden/gemv_hand_case.txt), unit activation vectors (y is a column of
the de-quantized weight, which the quantizer oracle returns independently),
codes equal to the zero point (y = 0), linearity, a pure-Python triple loop over
the bit stream, and the quantizer's own What on random layers.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import IC

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "gemv_hand_case.txt")


def _layer(out_f, in_f, bits, group, seed):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    q = oracle.quantize(W, IC, bits, group)
    return q, oracle.pack(q["codes"], IC, bits)


def test_hand_worked_case():
    """4 outputs x 2 inputs, 2 bits, groups of 2 outputs: numbers worked by hand in the golden file."""
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = np.array([float(t) for t in v.split()])
    codes = vals["codes"].reshape(4, 2).astype(np.uint8)
    packed = oracle.pack(codes, IC, 2)
    assert packed.shape == (2, 1) and list(packed[:, 0]) == [int(t) for t in vals["words"]]
    scales = vals["scales"].reshape(2, 2).astype(np.float32)
    zeros = vals["zeros"].reshape(2, 2).astype(np.uint8)
    x = vals["x"].astype(np.float16)
    y = oracle.gemv_ic(packed, scales, zeros, x, 4, 2, 2)
    assert np.array_equal(y, vals["y"])
    assert np.array_equal(oracle.abs_terms(packed, scales, zeros, x, 4, 2, 2), vals["abs_terms"])


@pytest.mark.parametrize("bits,group", [(3, 32), (4, 64), (2, 32), (3, 0)])
def test_unit_vectors_give_columns(bits, group):
    q, packed = _layer(128, 40, bits, group, seed=bits * 10 + group)
    for j in (0, 7, 39):
        x = np.zeros(40, dtype=np.float16)
        x[j] = 1.0
        y = oracle.gemv_ic(packed, q["scales"], q["zeros"], x, 128, bits, group)
        assert np.array_equal(y, q["What"][:, j].astype(np.float64))     # the quantizer's own What


def test_codes_at_zero_point_give_zero():
    g, out_f, in_f = 32, 64, 24
    zeros = np.random.default_rng(1).integers(0, 8, size=(out_f // g, in_f)).astype(np.uint8)
    codes = np.repeat(zeros, g, axis=0)
    scales = np.full((out_f // g, in_f), 0.37, dtype=np.float32)
    x = np.random.default_rng(2).standard_normal(in_f).astype(np.float16)
    y = oracle.gemv_ic(oracle.pack(codes, IC, 3), scales, zeros, x, out_f, 3, g)
    assert not y.any()


def test_linearity_and_triple_loop():
    bits, g, out_f, in_f = 3, 32, 64, 20
    q, packed = _layer(out_f, in_f, bits, g, seed=5)
    rng = np.random.default_rng(6)
    x1 = rng.standard_normal(in_f).astype(np.float16)
    x2 = (rng.standard_normal(in_f) * 3).astype(np.float16)
    y1 = oracle.gemv_ic(packed, q["scales"], q["zeros"], x1, out_f, bits, g)
    y2 = oracle.gemv_ic(packed, q["scales"], q["zeros"], x2, out_f, bits, g)
    xs = (x1.astype(np.float32) * 2).astype(np.float16)                   # doubling is exact in fp16
    assert np.array_equal(oracle.gemv_ic(packed, q["scales"], q["zeros"], xs, out_f, bits, g), 2 * y1)
    # pure-Python reading of the bit stream, fp64 accumulation in the same order as a left-to-right sum
    for o in (0, 31, 32, 63):
        acc1 = acc2 = 0.0
        for j in range(in_f):
            stream = 0
            for w, word in enumerate(packed[j]):
                stream |= int(word) << (32 * w)
            code = (stream >> (o * bits)) & ((1 << bits) - 1)
            what = float(np.float32(q["scales"][o // g, j]) * np.float32(code - int(q["zeros"][o // g, j])))
            acc1 += what * float(x1[j])
            acc2 += what * float(x2[j])
        assert y1[o] == pytest.approx(acc1, rel=1e-12, abs=1e-15)
        assert y2[o] == pytest.approx(acc2, rel=1e-12, abs=1e-15)


def test_matches_layer_output_of_quantized_weight():
    """y equals the layer output X What^T of Eq. 1 for a one-token X."""
    bits, g, out_f, in_f = 4, 64, 128, 48
    q, packed = _layer(out_f, in_f, bits, g, seed=9)
    x = np.random.default_rng(10).standard_normal(in_f).astype(np.float16)
    y = oracle.gemv_ic(packed, q["scales"], q["zeros"], x, out_f, bits, g)
    ref = np.zeros(out_f)
    for o in range(out_f):
        ref[o] = sum(float(q["What"][o, j]) * float(x[j]) for j in range(in_f))
    assert y == pytest.approx(ref, rel=1e-12, abs=1e-14)
    assert (oracle.abs_terms(packed, q["scales"], q["zeros"], x, out_f, bits, g) >= np.abs(y) - 1e-12).all()
