"""Pins of the 16-bit-per-group format oracle (CPU only).

Checked against things other than the oracle: hand-worked roundings and one hand-worked group
(tests/golden/meta16_hand_case.txt), the paper's printed average bits (tests/golden/avg_bits.txt,
App. C) counted on the stored arrays, a brute-force nearest-value search over every value the
word can hold, a brute-force nearest-grid-point search for the codes, weights that already lie
on a representable grid, the transpose identity between the two grouping dimensions, and unit
activation vectors through the matrix-vector oracle.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import IC, OC
from oracle import meta16_oracle as m16

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden():
    rounds, vals = [], {}
    for line in open(os.path.join(GOLDEN, "meta16_hand_case.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        k, v = [t.strip() for t in line.split("=")]
        if k == "round":
            rounds.append(v.split())
        else:
            vals[k] = np.array([float(t) for t in v.split()])
    return rounds, vals


def _rand_w(out_f, in_f, seed, outliers=True):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((out_f, in_f)) * 0.02
    if outliers:
        W *= 1 + 20 * (rng.random(in_f) < 0.05)
    return W.astype(np.float16)


def test_hand_worked_roundings():
    rounds, _ = _golden()
    assert len(rounds) == 10
    for b, s, pat, val in rounds:
        b = int(b)
        p = m16.scale_pattern(np.array([np.float32(float(s))]), b)
        assert int(p[0]) == int(pat), (b, s)
        assert float(m16.pattern_value(p, b)[0]) == float(val)
        assert float(m16.round_scale(np.array([np.float32(float(s))]), b)[0]) == float(val)


def test_hand_worked_group():
    _, v = _golden()
    W = v["group_w"].astype(np.float16).reshape(1, 4)
    r = m16.quantize(W, OC, 4, 4)
    assert r["meta"].tolist() == [[int(v["group_word"][0])]]
    assert r["codes"].ravel().tolist() == [int(t) for t in v["group_codes"]]
    assert np.array_equal(r["What"].ravel(), v["group_what"].astype(np.float32))
    assert np.array_equal(r["dW"].ravel(), v["group_dw"].astype(np.float32))
    # the same numbers per-IC, on the transposed weight
    rt = m16.quantize(W.T.copy(), IC, 4, 4)
    assert rt["meta"].tolist() == [[int(v["group_word"][0])]]
    assert np.array_equal(rt["dW"].ravel(), v["group_dw"].astype(np.float32))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_rounding_is_nearest_value_brute_force(bits):
    """The chosen pattern is a nearest value of the format to fp16(scale); of two equally near, the even one."""
    n_pat = 1 << (16 - bits)
    finite = [p for p in range(1, n_pat) if (p << (bits - 1)) < 0x7C00]
    table = np.array([np.array([p << (bits - 1)], dtype=np.uint16).view(np.float16)[0] for p in finite], dtype=np.float64)
    assert (np.diff(table) > 0).all()                           # the encoding is monotone
    rng = np.random.default_rng(bits)
    s = np.exp(rng.uniform(np.log(1e-8), np.log(4e4), size=4000)).astype(np.float32)
    s = np.concatenate([s, table[::37].astype(np.float32), np.float32([6.1e-5, 6.0e-5, 5.96e-8, 2.9e-8, 3.1e-8])])
    got = m16.scale_pattern(s, bits).astype(np.int64)
    h = s.astype(np.float16).astype(np.float64)
    for hv, gp in zip(h, got):
        dist = np.abs(table - hv)
        best = np.flatnonzero(dist == dist.min())
        cands = [finite[i] for i in best]
        if hv == 0.0 or hv < table[0] / 2:
            assert gp == 1
        elif len(cands) == 1:
            assert gp == cands[0], (hv, gp, cands)
        else:
            assert gp in cands and gp % 2 == 0, (hv, gp, cands)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_word_round_trip(bits):
    words = np.arange(1 << 16, dtype=np.uint32)
    pat = words >> bits
    ok = (pat >= 1) & ((pat << (bits - 1)) < 0x7C00)
    words = words[ok].astype(np.uint16)
    s, z = m16.decode(words, bits)
    assert (s > 0).all() and np.isfinite(s).all() and (z < (1 << bits)).all()
    assert np.array_equal(m16.encode(s, z, bits), words)
    with pytest.raises(ValueError):
        m16.encode(np.float32([0.2]), np.uint8([1]), bits)      # 0.2 is not a value of the format
    with pytest.raises(ValueError):
        m16.encode(np.float32([0.25]), np.uint8([1 << bits]), bits)
    with pytest.raises(ValueError):
        m16.scale_pattern(np.float32([0.25]), 5)


def test_paper_average_bits_on_the_arrays():
    """b + 16/g, the 'Avg Bits' printed for RTN-ada in App. C, counted on the stored streams."""
    with open(os.path.join(GOLDEN, "avg_bits.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for b, g, avg in rows:
        for dim in (OC, IC):
            assert m16.stored_bits_per_weight(512, 256, dim, int(b), int(g)) == pytest.approx(float(avg), abs=1e-12)
    # and on real arrays
    W = _rand_w(256, 128, 3)
    r = m16.quantize(W, IC, 4, 128)
    pk = oracle.pack(r["codes"], IC, 4)
    assert (pk.size * 32 + r["meta"].size * 16) / W.size == 4.125
    assert r["meta"].dtype == np.uint16 and r["meta"].shape == (2, 128)


@pytest.mark.parametrize("dim", [OC, IC])
@pytest.mark.parametrize("bits,group", [(4, 32), (3, 16), (2, 64), (4, 0)])
def test_codes_are_nearest_grid_points(dim, bits, group):
    W = _rand_w(64, 128, seed=10 * bits + group + dim)
    r = m16.quantize(W, dim, bits, group)
    qmax = (1 << bits) - 1
    s_dec, z_dec = m16.decode(r["meta"], bits)
    assert np.array_equal(s_dec, r["scales"]) and np.array_equal(z_dec, r["zeros"])
    g = (128 if dim == OC else 64) if group == 0 else group
    rep = (lambda a: np.repeat(a, g, axis=1)) if dim == OC else (lambda a: np.repeat(a, g, axis=0))
    s, z = rep(s_dec).astype(np.float64), rep(z_dec).astype(np.float64)
    w = W.astype(np.float64)
    # the scale is within half a step of the format of the fp32 scale (fp16 normal range here)
    r32 = oracle.quantize(W, dim, bits, group)
    assert (np.abs(r["scales"].astype(np.float64) / r32["scales"] - 1) <= 2.0 ** -(12 - bits) + 2.0 ** -11).all()
    assert (r["scales"] != r32["scales"]).any()                 # and it is really rounded
    # zero-point from the rounded scale
    mn = np.minimum((w.reshape(64, -1, g).min(axis=2) if dim == OC else w.T.reshape(128, -1, g).min(axis=2).T), 0)
    zq = -mn / s_dec.astype(np.float64)
    off_tie = np.abs(zq - np.floor(zq) - 0.5) > 1e-6
    assert np.array_equal(np.clip(np.rint(zq), 0, qmax)[off_tie], z_dec.astype(np.float64)[off_tie])
    # brute force over every code
    ks = np.arange(qmax + 1, dtype=np.float64)
    err = np.abs(w[None] - s[None] * (ks[:, None, None] - z[None]))
    best = err.min(axis=0)
    mine = np.abs(w - s * (r["codes"].astype(np.float64) - z))
    assert (mine <= best * (1 + 1e-6) + 1e-12).all()
    assert np.array_equal(r["dW"], (W.astype(np.float32) - r["What"]).astype(np.float32))
    assert np.array_equal(r["What"].astype(np.float64), s * (r["codes"].astype(np.float64) - z))   # exact product


def test_representable_grid_is_a_fixed_point():
    """Weights s*(k - z) with s a power of two and every group spanning codes 0..qmax: same codes as the fp32-scale
    quantizer, zero error, and the word holds exactly (s, z)."""
    rng = np.random.default_rng(5)
    bits, g = 4, 16
    k = rng.integers(0, 16, size=(32, 64))
    k[:, 0::16] = 0
    k[:, 1::16] = 15
    z = rng.integers(1, 15, size=(32, 4))
    e = rng.integers(-9, -3, size=(32, 4))
    s = np.ldexp(1.0, e)
    W = (np.repeat(s, g, axis=1) * (k - np.repeat(z, g, axis=1))).astype(np.float16)
    r = m16.quantize(W, OC, bits, g)
    r32 = oracle.quantize(W, OC, bits, g)
    assert np.array_equal(r["codes"], k) and np.array_equal(r32["codes"], k)
    assert not r["dW"].any()
    sd, zd = m16.decode(r["meta"], bits)
    assert np.array_equal(sd, s.astype(np.float32)) and np.array_equal(zd, z)


@pytest.mark.parametrize("bits,group", [(4, 16), (3, 32)])
def test_transpose_identity(bits, group):
    W = _rand_w(64, 96, seed=bits)
    a = m16.quantize(W, IC, bits, group)
    b = m16.quantize(np.ascontiguousarray(W.T), OC, bits, group)
    assert np.array_equal(a["codes"], b["codes"].T) and np.array_equal(a["meta"], b["meta"].T)
    assert np.array_equal(a["dW"], b["dW"].T)


def test_tiny_and_empty_groups():
    W = np.zeros((4, 32), dtype=np.float16)
    W[1, :] = np.float16(6e-8)                                   # the smallest subnormal everywhere: range/15 rounds to 0 in fp16
    W[2, 5] = np.float16(3e-5)                                   # fp16-subnormal scale
    W[3, 7] = np.float16(-65504.0)
    W[3, 9] = np.float16(65504.0)                                # the largest possible range
    for bits in (2, 3, 4):
        r = m16.quantize(W, OC, bits, 32)
        s, _ = m16.decode(r["meta"], bits)
        assert s[0, 0] == 1.0 and not r["dW"][0].any() and not r["codes"][0].any()
        assert s[1, 0] == np.ldexp(1.0, bits - 1 - 24)           # pattern 1
        assert np.isfinite(s).all() and (s > 0).all()
        assert np.isfinite(r["dW"]).all()
        assert np.abs(r["dW"][3]).max() <= s[3, 0] * ((1 << bits) - 1)   # clipped at most by the rounding of the scale


@pytest.mark.parametrize("bits,group", [(4, 32), (3, 64), (2, 32)])
def test_gemv_unit_vectors_give_columns(bits, group):
    W = _rand_w(128, 24, seed=bits + group, outliers=False)
    r = m16.quantize(W, IC, bits, group)
    pk = oracle.pack(r["codes"], IC, bits)
    for j in (0, 11, 23):
        x = np.zeros(24, dtype=np.float16)
        x[j] = 1.0
        assert np.array_equal(m16.gemv_ic(pk, r["meta"], x, 128, bits, group), r["What"][:, j].astype(np.float64))
    x = np.random.default_rng(1).standard_normal(24).astype(np.float16)
    y = m16.gemv_ic(pk, r["meta"], x, 128, bits, group)
    assert y == pytest.approx(r["What"].astype(np.float64) @ x.astype(np.float64), rel=1e-12, abs=1e-12)
    assert (m16.abs_terms(pk, r["meta"], x, 128, bits, group) >= np.abs(y) - 1e-12).all()


@pytest.mark.parametrize("dim", [OC, IC])
def test_gptq_sweep_in_the_format(dim):
    """GPTQ in the selected dimension with the scales rounded into the group word: with a diagonal Hessian no error
    is propagated and the sweep must give the plain quantizer of this module; with a full one the sweep's identity
    W - What = E U must hold and What must be exactly what the stored words and codes de-quantize to."""
    from oracle import gptq_oracle as G
    rng = np.random.default_rng(3 + dim)
    out_f, in_f, bits, group = 64, 96, 4, 32
    W = _rand_w(out_f, in_f, seed=11 + dim)
    # diagonal H: act-order still permutes the channels, the result does not depend on it
    d = rng.uniform(0.5, 4.0, size=in_f)
    Hp, perm, dead = G.prepare(np.diag(d), 0.01, True)
    U = G.factor(Hp).astype(np.float32)
    r = m16.gptq_sweep(W, U, perm, dead, dim, bits, group)
    q = m16.quantize(W, dim, bits, group)
    assert np.array_equal(r["codes"], q["codes"]) and np.array_equal(r["meta"], q["meta"])
    assert np.array_equal(r["dW"], q["dW"])
    # full H
    X = rng.standard_normal((300, in_f)) * (1 + 10 * (rng.random(in_f) < 0.05))
    Hp, perm, dead = G.prepare(X.T @ X, 0.01, True)
    U = G.factor(Hp).astype(np.float32)
    r = m16.gptq_sweep(W, U, perm, dead, dim, bits, group)
    s, z = m16.decode(r["meta"], bits)
    g = group
    rep = (lambda a: np.repeat(a, g, axis=1)) if dim == OC else (lambda a: np.repeat(a, g, axis=0))
    assert np.array_equal(r["What"], (rep(s) * (r["codes"].astype(np.float32) - rep(z).astype(np.float32))).astype(np.float32))
    lhs = (W.astype(np.float64) - r["What"].astype(np.float64))[:, perm]
    rhs = r["E"].astype(np.float64) @ U.astype(np.float64)
    assert np.abs(lhs - rhs).max() <= 1e-4 * np.abs(lhs).max() + 1e-7
    # and it is not the fp32-scale sweep in disguise
    r32 = G.sweep(W, U, perm, dead, dim, bits, group)
    assert (r32["scales"] != r["scales"]).any()
