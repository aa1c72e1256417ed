"""Seeded sweep of random shapes through every entry point of the search, against the CPU oracle.

The fixed cases of test_gpu_parity.py are chosen to hit each kernel path once; this sweep draws shapes, group
sizes and precisions at random (seeded, so a failure names its case) to catch what a hand-picked list misses:
ragged tiles in both directions, groups that are not powers of two, widths that are not multiples of 8 or 32."""
import numpy as np
import pytest
import torch

import oracle
from oracle import IC, OC
from oracle import meta16_oracle as m16
from paper_2309_15531_amd import binding as B
from paper_2309_15531_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = B.Context()
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _divisors(n):
    return [d for d in range(1, n + 1) if n % d == 0]


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        out_f = int(rng.choice([rng.integers(1, 40) * 8, rng.integers(1, 20) * 32, rng.integers(8, 300), 256, 384]))
        in_f = int(rng.choice([rng.integers(1, 40) * 8, rng.integers(1, 20) * 32, rng.integers(8, 300), 512, 264]))
        dim = int(rng.integers(0, 2))
        axis = in_f if dim == OC else out_f
        group = int(rng.choice(_divisors(axis) + [0, 0]))
        bits = int(rng.integers(2, 9))
        clip = float(np.float32(rng.choice([1.0, 1.0, rng.uniform(0.5, 1.0)])))
        out.append((out_f, in_f, dim, group, bits, clip))
    return out


@pytest.mark.parametrize("case", _cases(48, seed=2024), ids=lambda c: "o%d_i%d_d%d_g%d_b%d_c%.3f" % c)
def test_quantize_random_case(ctx, case):
    out_f, in_f, dim, group, bits, clip = case
    W = synth.make_weight(out_f, in_f, seed=out_f * 131 + in_f, heavy_cols=max(1, in_f // 50), heavy_scale=6.0)
    g = (in_f if dim == OC else out_f) if group == 0 else group
    shape = (out_f, in_f // g) if dim == OC else (out_f // g, in_f)
    n_ch, ln = (out_f, in_f) if dim == OC else (in_f, out_f)
    for fmt16 in ([False, True] if bits <= 4 else [False]):
        ref = (m16.quantize if fmt16 else oracle.quantize)(W, dim, bits, group, clip)
        codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda")
        dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
        packed = torch.full((n_ch, (ln * bits + 31) // 32), -1, dtype=torch.int32, device="cuda")
        if fmt16:
            meta = torch.full(shape, -1, dtype=torch.int16, device="cuda")
            ctx.adadim_quantize_meta16(dev(W), dim, bits, group, clip, codes=codes, meta=meta, dW=dW, packed=packed)
            torch.cuda.synchronize()
            assert np.array_equal(meta.cpu().numpy().view(np.uint16), ref["meta"])
        else:
            scales = torch.full(shape, -1.0, dtype=torch.float32, device="cuda")
            zeros = torch.full(shape, 255, dtype=torch.uint8, device="cuda")
            ctx.adadim_quantize(dev(W), dim, bits, group, clip, codes=codes, scales=scales, zeros=zeros, dW=dW, packed=packed)
            torch.cuda.synchronize()
            assert np.array_equal(scales.cpu().numpy().view(np.uint32), ref["scales"].view(np.uint32))
            assert np.array_equal(zeros.cpu().numpy(), ref["zeros"])
        assert np.array_equal(codes.cpu().numpy(), ref["codes"])
        assert np.array_equal(dW.cpu().numpy(), ref["dW"])
        assert np.array_equal(packed.cpu().numpy().view(np.uint32), oracle.pack(ref["codes"], dim, bits))


def _search_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        out_f = int(rng.integers(1, 24)) * 32
        in_f = int(rng.integers(1, 40)) * 8
        tokens = int(rng.integers(1, 700))
        bits = int(rng.integers(2, 5))
        group = int(rng.choice([g for g in (8, 16, 32, 64, 0) if g == 0 or (out_f % g == 0 and in_f % g == 0)]))
        out.append((out_f, in_f, tokens, bits, group))
    return out


@pytest.mark.parametrize("case", _search_cases(16, seed=77), ids=lambda c: "o%d_i%d_t%d_b%d_g%d" % c)
def test_search_random_case(ctx, case):
    """Gram matrix, both candidates' losses and the choice for a random layer."""
    from paper_2309_15531_amd import search as S
    out_f, in_f, tokens, bits, group = case
    W = synth.make_weight(out_f, in_f, seed=tokens, heavy_cols=max(1, in_f // 50), heavy_scale=5.0)
    X = synth.make_activations(tokens, in_f, seed=tokens + 1, n_outliers=min(3, in_f), scale_lo=20, scale_hi=80)
    ref = oracle.search(W, X, bits, group)
    hp = S.PreparedHessian(ctx, in_f).update(dev(X)).prepare()
    Href = oracle.hessian(X)
    Hg = hp.H.cpu().numpy().astype(np.float64)
    dg = np.sqrt(np.outer(np.diag(Href), np.diag(Href)))
    assert (np.abs(Hg - Href) <= 2e-5 * dg + 1e-30).all()
    ls = S.LayerSearch(ctx, out_f, in_f, bits, group)
    best, dim, _ = ls.run(dev(W), hp)
    torch.cuda.synchronize()
    got = ls.losses.cpu().numpy()
    assert got == pytest.approx(ref["losses"], rel=1e-3, abs=1e-30)
    lo, hi = min(ref["losses"]), max(ref["losses"])
    if lo > 0 and (hi - lo) / lo > 0.01:
        assert best == ref["best"]


def _gemv_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        group = int(rng.choice([32, 64, 96, 128, 256]))
        out_f = group * int(rng.integers(1, 30))
        in_f = int(rng.integers(1, 300)) * 4
        bits = int(rng.integers(2, 5))
        out.append((out_f, in_f, bits, int(rng.choice([group, group, 0]))))
    return out


@pytest.mark.parametrize("case", _gemv_cases(16, seed=5), ids=lambda c: "o%d_i%d_b%d_g%d" % c)
def test_gemv_random_case(ctx, case):
    out_f, in_f, bits, group = case
    rng = np.random.default_rng(out_f + in_f)
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    x = rng.standard_normal(in_f).astype(np.float16)
    for fmt16 in (False, True):
        q = (m16.quantize if fmt16 else oracle.quantize)(W, IC, bits, group)
        packed = oracle.pack(q["codes"], IC, bits)
        y = torch.full((out_f,), float("nan"), dtype=torch.float16, device="cuda")
        if fmt16:
            ctx.adadim_gemv_ic_meta16(dev(packed.view(np.int32)), dev(q["meta"].view(np.int16)), dev(x), out_f, in_f, bits, group, y)
        else:
            ctx.adadim_gemv_ic(dev(packed.view(np.int32)), dev(q["scales"]), dev(q["zeros"]), dev(x), out_f, in_f, bits, group, y)
        torch.cuda.synchronize()
        ref = oracle.gemv_ic(packed, q["scales"], q["zeros"], x, out_f, bits, group)
        mag = oracle.abs_terms(packed, q["scales"], q["zeros"], x, out_f, bits, group)
        got = y.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        assert (np.abs(got - ref) <= 2.0 ** -10 * np.abs(ref) + 2e-5 * mag).all()
