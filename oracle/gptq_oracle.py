"""CPU oracle for GPTQ in the dimension AdaDim selected ("GPTQ-ada").

TEST INFRASTRUCTURE ONLY (see adadim_oracle.py for the rules): imported by the
tests and the benchmark's cpu_baseline leg, never by the product, and it shares
no code with the HIP sources.

What it computes (paper Sec. 3.3, "Augmenting RTN and GPTQ", App. A.1
"Activation reordering for free", App. B `gptq_ada`, Table 2b): once RTN has
chosen the dimension, GPTQ is run in that dimension.  GPTQ (Frantar et al. 2022)
quantizes the input channels of the layer one after the other and, after each,
spreads that channel's rounding error over the channels not yet quantized, using
the inverse of the (damped) Hessian H = X^T X of the layer input; per-IC GPTQ is
the same sweep with each channel's parameters taken per row group when the channel
is visited (Sec. 3.3).  The configuration the paper settles on (green cells of
Table 2b):

* per-IC: activation reordering (channels visited in the order of decreasing
  diag(H)), quantization parameters of each (row group, channel) taken from the
  channel's CURRENT values when it is visited;
* per-OC: activation reordering with static groups: the parameters of each
  (row, channel group) are computed beforehand from the original weight (plain
  per-OC RTN parameters) and only looked up during the sweep.

Steps, in the published algorithm's order and notation:
  1. dead channels (H_jj = 0): H_jj <- 1, W[:, j] <- 0;
  2. damping: H <- H + percdamp * mean(diag H) * I;
  3. act-order: perm = argsort(-diag H) (ties: lower index first); W, H permuted;
  4. U = upper Cholesky factor of H^-1 (H^-1 = U^T U);
  5. for blocks of 128 channels [i1, i2): for each channel i in the block:
        q_i = Q(w_i);  e_i = (w_i - q_i) / U_ii;
        W[:, i+1:i2] -= e_i (x) U[i, i+1:i2];
     then W[:, i2:] -= E[:, i1:i2] @ U[i1:i2, i2:].

Precision.  Step 4 is done in fp64 (`factor`).  The sweep (`sweep`) takes U as an
fp32 matrix and works in fp32 with one rounding per operation, each update
W <- W - e*u being a rounded product followed by a rounded difference, and the
block update of step 5 applied as its 128 rank-one updates in channel order, so
that a kernel that follows the same sequence can be compared bit for bit; the
quantizer is the one of adadim_oracle.quantize (same fp32 formulas).

Parity status: the algorithm is pinned by its defining identities
(tests/test_gptq_oracle_pins.py): U^T U (H + damp I) = I, the sweep's identity
W - What = E U, agreement with the plain optimal-brain-surgeon update computed
from explicit inverses of the trailing Hessian, the diagonal-H case (no error
is propagated: the result is plain RTN), a hand-worked 1 x 2 case.  That the
options chosen here (block 128, percdamp 0.01, parameters as above) are the
authors' settings is "parity unpinned": the paper names the options but prints
no per-layer output.
"""
from __future__ import annotations

import numpy as np

from .adadim_oracle import OC, IC, quantize

_F32 = np.float32
BLOCK = 128


def prepare(H, percdamp: float = 0.01, act_order: bool = True):
    """Steps 1-3 on H alone: returns (Hp fp64 permuted+damped, perm int64, dead bool[in])."""
    H = np.array(H, dtype=np.float64)
    n = H.shape[0]
    d = np.diag(H).copy()
    dead = d == 0
    H[dead, dead] = 1.0
    d = np.diag(H).copy()
    damp = percdamp * d.mean()
    perm = np.argsort(-d, kind="stable") if act_order else np.arange(n)
    Hp = H[np.ix_(perm, perm)] + damp * np.eye(n)
    return Hp, perm.astype(np.int64), dead


def factor(Hp) -> np.ndarray:
    """Step 4 in fp64: U upper triangular with inv(Hp) = U^T U."""
    Hinv = np.linalg.inv(np.asarray(Hp, dtype=np.float64))
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.linalg.cholesky(Hinv).T


def _params_f32(mn, mx, qmax, scale_round=None):
    """Scale and zero of one group from its min/max (the quantizer's steps 1, 3, 4; clip = 1), fp32;
    scale_round as in adadim_oracle.quantize."""
    zero = _F32(0.0)
    mx = np.maximum(mx, zero)
    mn = np.minimum(mn, zero)
    rng = (mx - mn).astype(_F32)
    scale = (rng / qmax).astype(_F32)
    scale = np.where(rng == zero, _F32(1.0), scale).astype(_F32)
    if scale_round is not None:
        scale = np.asarray(scale_round(scale), dtype=_F32)
    z = np.rint(((-mn) / scale).astype(_F32)).astype(_F32)
    z = np.minimum(np.maximum(z, zero), qmax).astype(_F32)
    return scale, z


def sweep(W, U, perm, dead, dim: int, bits: int, group: int, block: int = BLOCK, scale_round=None) -> dict:
    """Step 5 in fp32 (see the module text for the rounding sequence).

    W fp16 [out, in]; U fp32 [in, in] upper, in visiting order; perm[i] = original index of
    the channel visited i-th.  Returns codes u8 [out, in], scales f32 / zeros u8 ([out, in/g]
    static for OC, [out/g, in] for IC), What f32, dW f32 = W - What (all in original order),
    E f32 [out, in] (errors in visiting order).  scale_round: every scale (the static ones and the
    ones computed during the sweep) is rounded into a storage format first, see meta16_oracle."""
    W0 = np.asarray(W).astype(_F32)
    out_f, in_f = W0.shape
    U = np.asarray(U, dtype=_F32)
    qmax = _F32((1 << bits) - 1)
    zero = _F32(0.0)
    W0 = W0.copy()
    W0[:, np.asarray(dead, dtype=bool)] = zero
    Wp = np.ascontiguousarray(W0[:, perm])
    if dim == OC:
        g = in_f if group == 0 else group
        st = quantize(W0, OC, bits, group, scale_round=scale_round)   # static: plain per-OC RTN of the original weight
        s_static, z_static = st["scales"], st["zeros"].astype(_F32)
        scales, zeros = st["scales"], st["zeros"]
    else:
        g = out_f if group == 0 else group
        scales = np.zeros((out_f // g, in_f), dtype=_F32)
        zeros = np.zeros((out_f // g, in_f), dtype=np.uint8)
    codes = np.zeros((out_f, in_f), dtype=np.uint8)
    What = np.zeros((out_f, in_f), dtype=_F32)
    E = np.zeros((out_f, in_f), dtype=_F32)
    for i1 in range(0, in_f, block):
        i2 = min(i1 + block, in_f)
        for i in range(i1, i2):
            j = int(perm[i])                       # original channel
            w = Wp[:, i]
            if dim == OC:
                s = s_static[:, j // g]
                z = z_static[:, j // g]
            else:
                wg = w.reshape(out_f // g, g)
                sg, zg = _params_f32(wg.min(axis=1), wg.max(axis=1), qmax, scale_round)
                scales[:, j] = sg
                zeros[:, j] = zg.astype(np.uint8)
                s = np.repeat(sg, g)
                z = np.repeat(zg, g)
            q = (np.rint((w / s).astype(_F32)).astype(_F32) + z).astype(_F32)
            q = np.minimum(np.maximum(q, zero), qmax).astype(_F32)
            wq = (s * (q - z).astype(_F32)).astype(_F32)
            codes[:, j] = q.astype(np.uint8)
            What[:, j] = wq
            e = ((w - wq).astype(_F32) / U[i, i]).astype(_F32)
            E[:, i] = e
            if i + 1 < i2:
                upd = (e[:, None] * U[i, i + 1:i2][None, :]).astype(_F32)
                Wp[:, i + 1:i2] = (Wp[:, i + 1:i2] - upd).astype(_F32)
        if i2 < in_f:
            for k in range(i1, i2):                # the block update, one channel's error at a time
                upd = (E[:, k][:, None] * U[k, i2:][None, :]).astype(_F32)
                Wp[:, i2:] = (Wp[:, i2:] - upd).astype(_F32)
    return {"codes": codes, "scales": scales, "zeros": zeros, "What": What,
            "dW": (W0 - What).astype(_F32), "E": E}


def gptq(W, H, dim: int, bits: int, group: int, percdamp: float = 0.01, act_order: bool = True) -> dict:
    """Whole procedure: prepare and factor in fp64, U rounded once to fp32, sweep in fp32."""
    Hp, perm, dead = prepare(H, percdamp, act_order)
    U = factor(Hp).astype(_F32)
    r = sweep(W, U, perm, dead, dim, bits, group)
    r.update(perm=perm, dead=dead, U=U)
    return r
