"""Pins of the GPTQ-ada oracle (CPU only): the algorithm is checked against its defining
identities and against a different formulation of the same update, not against itself."""
import os

import numpy as np
import pytest

import oracle
from oracle import OC, IC
from oracle import gptq_oracle as G

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "gptq_hand_case.txt")


def _layer(out_f, in_f, tokens, seed, outliers=2):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    X = rng.standard_normal((tokens, in_f))
    X[:, rng.choice(in_f, outliers, replace=False)] *= 40
    X = X.astype(np.float16).astype(np.float64)
    return W, X.T @ X


def test_hand_worked_case():
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = np.array([float(t) for t in v.split()])
    H = vals["H"].reshape(2, 2)
    U = G.factor(H)
    assert U == pytest.approx(vals["U"].reshape(2, 2), abs=1e-14)
    # one row on the integer grid: emulate scale 1 / zero 0 by a 2-bit OC group [0, 3] -> put 0 and 3 in the row
    w = vals["w"]
    e0 = (w[0] - np.rint(w[0])) / U[0, 0]
    w1 = w[1] - e0 * U[0, 1]
    assert w1 == pytest.approx(vals["w1_after_channel0"][0], abs=1e-14)
    assert [np.rint(w[0]), np.rint(w1)] == list(vals["q"])
    Hinv = np.linalg.inv(H)
    assert w1 == pytest.approx(w[1] - (w[0] - np.rint(w[0])) * Hinv[0, 1] / Hinv[0, 0], abs=1e-14)


@pytest.mark.parametrize("act_order", [False, True])
def test_factor_identity(act_order):
    W, H = _layer(8, 80, 200, seed=1)
    H[7, :] = 0
    H[:, 7] = 0                                   # a dead channel
    Hp, perm, dead = G.prepare(H, 0.01, act_order)
    assert dead[7] and dead.sum() == 1
    d = np.diag(H).copy()
    d[7] = 1.0
    assert np.array_equal(np.diag(Hp), d[perm] + 0.01 * d.mean())
    if act_order:
        assert (np.diff(d[perm]) <= 0).all()
    else:
        assert np.array_equal(perm, np.arange(80))
    U = G.factor(Hp)
    assert np.allclose(np.tril(U, -1), 0) and (np.diag(U) > 0).all()
    assert U.T @ U @ Hp == pytest.approx(np.eye(80), abs=1e-8)


@pytest.mark.parametrize("dim,group", [(OC, 32), (IC, 32), (OC, 0), (IC, 0)])
def test_diagonal_hessian_is_plain_rtn(dim, group):
    """With a diagonal H no error is propagated (U is diagonal): GPTQ returns RTN."""
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((64, 96)) * 0.02).astype(np.float16)
    H = np.diag(rng.uniform(1, 50, 96))
    r = G.gptq(W, H, dim, 3, group, act_order=True)
    rt = oracle.quantize(W, dim, 3, group)
    for k in ("codes", "scales", "zeros", "What"):
        assert np.array_equal(r[k], rt[k]), k


@pytest.mark.parametrize("dim", [OC, IC])
def test_sweep_identity_and_loss(dim):
    """W - What = E U (every channel's total displacement is the propagated errors), and the
    error-feedback lowers the layer error below plain RTN on a correlated H."""
    W, H = _layer(64, 160, 400, seed=5)
    r = G.gptq(W, H, dim, 3, 32)
    perm = r["perm"]
    lhs = (W.astype(np.float64) - r["What"].astype(np.float64))[:, perm]
    rhs = r["E"].astype(np.float64) @ r["U"].astype(np.float64)
    assert lhs == pytest.approx(rhs, abs=2e-6)
    assert r["codes"].max() <= 7
    rt = oracle.quantize(W, dim, 3, 32)
    assert oracle.layer_error(r["dW"], H) < 0.9 * oracle.layer_error(rt["dW"], H)
    if dim == OC:        # static groups: parameters are the plain RTN ones
        assert np.array_equal(r["scales"], rt["scales"]) and np.array_equal(r["zeros"], rt["zeros"])


def test_matches_optimal_brain_surgeon_updates():
    """The Cholesky form is the same procedure as: quantize a channel, then move the channels
    not yet quantized by -(w_i - q_i)/[Hr^-1]_ii * (Hr^-1)_{i,:}, Hr the Hessian of the remaining
    channels, its inverse recomputed from scratch each time (fp64 throughout here)."""
    rng = np.random.default_rng(7)
    out_f, in_f, bits = 6, 24, 3
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    X = rng.standard_normal((60, in_f))
    X[:, 3] *= 20
    H = X.T @ X
    r = G.gptq(W, H, OC, bits, 0)                 # one static group per row: fixed grid per row
    Hp, perm, dead = G.prepare(H, 0.01, True)
    st = oracle.quantize(W, OC, bits, 0)
    s = st["scales"][:, 0].astype(np.float64)
    z = st["zeros"][:, 0].astype(np.float64)
    Wp = W.astype(np.float64)[:, perm]
    codes = np.zeros((out_f, in_f))
    for i in range(in_f):
        Hr_inv = np.linalg.inv(Hp[i:, i:])
        q = np.clip(np.rint(Wp[:, i] / s) + z, 0, 2 ** bits - 1)
        codes[:, perm[i]] = q
        err = (Wp[:, i] - s * (q - z)) / Hr_inv[0, 0]
        Wp[:, i + 1:] -= err[:, None] * Hr_inv[0, 1:][None, :]
    # same decisions except where fp32 vs fp64 lands on the other side of a rounding boundary
    assert (codes != r["codes"]).mean() < 0.03


def test_dead_channels_are_zeroed():
    W, H = _layer(16, 64, 100, seed=9)
    H[:, 10] = 0
    H[10, :] = 0
    r = G.gptq(W, H, IC, 4, 16)
    assert r["dead"][10]
    assert not r["What"][:, 10].any()             # the channel's weights were set to zero before quantizing
