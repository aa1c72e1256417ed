"""GPU parity of GPTQ in the selected dimension (adadim_gptq_prepare / adadim_gptq_quantize).

Bars.  prepare: dead flags and the visiting order are exact; U is factorized in fp64 and rounded
once, so it must agree with the fp64 oracle factor to fp32 rounding (|dU| <= 2e-6 |U| + 1e-7 max|U|).
quantize: given the same fp32 U, codes, scales, zeros and dW are bit-exact (the sweep's rounding
sequence is part of the definition).  End to end (GPU factor + GPU sweep): a last-bit difference in
U can flip a rounding decision and the difference then propagates, so codes are compared by
agreement rate and the layer error by value (within 2 % of the oracle's, and below plain RTN).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import OC, IC
from oracle import gptq_oracle as G
from paper_2309_15531_amd import binding as B
from paper_2309_15531_amd import search as S
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


def layer(out_f, in_f, tokens, seed, dead=()):
    W = synth.make_weight(out_f, in_f, seed, heavy_cols=max(1, in_f // 100), heavy_scale=5.0)
    X = synth.make_activations(tokens, in_f, seed + 1, n_outliers=3, scale_lo=40, scale_hi=80)
    X[:, list(dead)] = 0
    return W, X


def gpu_prepare(ctx, H32, percdamp=0.01, act_order=True):
    n = H32.shape[0]
    perm = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    dead = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    U = torch.full((n, n), float("nan"), dtype=torch.float32, device="cuda")
    ctx.adadim_gptq_prepare(dev(H32), perm, dead, U, percdamp, act_order)
    torch.cuda.synchronize()
    return perm, dead, U


def gpu_sweep(ctx, W, dim, bits, group, U, perm, dead, want_packed=False):
    out_f, in_f = W.shape
    Wd = dev(W)
    codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda")
    dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
    res = {}
    if dim == OC:
        g = in_f if group == 0 else group
        ss = torch.empty((out_f, in_f // g), dtype=torch.float32, device="cuda")
        sz = torch.empty((out_f, in_f // g), dtype=torch.uint8, device="cuda")
        Wz = Wd.clone()
        Wz[:, dead.bool()] = 0                         # static parameters of the weight with dead channels zeroed
        ctx.adadim_quantize(Wz, OC, bits, group, 1.0, scales=ss, zeros=sz)
        kw = dict(static_scales=ss, static_zeros=sz)
        res["scales"], res["zeros"] = ss, sz
    else:
        sc = torch.full((out_f // group, in_f), -1.0, dtype=torch.float32, device="cuda")
        zr = torch.full((out_f // group, in_f), 255, dtype=torch.uint8, device="cuda")
        kw = dict(scales=sc, zeros=zr)
        res["scales"], res["zeros"] = sc, zr
    packed = None
    if want_packed:
        n_ch, ln = (out_f, in_f) if dim == OC else (in_f, out_f)
        packed = torch.full((n_ch, (ln * bits + 31) // 32), -1, dtype=torch.int32, device="cuda")
    ctx.adadim_gptq_quantize(Wd, dim, bits, group, U, perm, dead, codes, dW=dW, packed=packed, **kw)
    torch.cuda.synchronize()
    out = {k: v.cpu().numpy() for k, v in res.items()}
    out.update(codes=codes.cpu().numpy(), dW=dW.cpu().numpy())
    if want_packed:
        out["packed"] = packed.cpu().numpy().view(np.uint32)
    return out


@pytest.mark.parametrize("in_f,act_order", [(200, True), (512, True), (64, False), (328, True)])
def test_prepare_matches_fp64_factor(ctx, in_f, act_order):
    W, X = layer(8, in_f, 700, seed=in_f, dead=(3, in_f - 2))
    H32 = oracle.hessian(X).astype(np.float32)
    Hp, perm_ref, dead_ref = G.prepare(H32, 0.01, act_order)
    U_ref = G.factor(Hp)
    perm, dead, U = gpu_prepare(ctx, H32, 0.01, act_order)
    assert np.array_equal(dead.cpu().numpy().astype(bool), dead_ref)
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), perm_ref)
    Ug = U.cpu().numpy().astype(np.float64)
    assert not np.tril(Ug, -1).any()
    assert (np.abs(Ug - U_ref) <= 2e-6 * np.abs(U_ref) + 1e-7 * np.abs(U_ref).max()).all()


@pytest.mark.parametrize("out_f,in_f,dim,bits,group", [
    (128, 320, OC, 3, 64),
    (200, 264, OC, 4, 0),        # ragged last block of 8 channels, ragged row tile
    (256, 264, IC, 3, 128),
    (192, 384, IC, 4, 64),
    (64, 96, OC, 2, 32),         # less than one block
    (64, 1280, OC, 3, 128),      # ten blocks: the bulk of each block's trailing update runs on the side stream
    (128, 1160, IC, 4, 128),     # the same per-IC, ragged last block
])
def test_sweep_bit_exact_given_u(ctx, out_f, in_f, dim, bits, group):
    W, X = layer(out_f, in_f, 900, seed=out_f + in_f, dead=(5,))
    H32 = oracle.hessian(X).astype(np.float32)
    Hp, perm, dead = G.prepare(H32, 0.01, True)
    U32 = G.factor(Hp).astype(np.float32)
    ref = G.sweep(W, U32, perm, dead, dim, bits, group)
    got = gpu_sweep(ctx, W, dim, bits, group, dev(U32), dev(perm.astype(np.int32)), dev(dead.astype(np.uint8)),
                    want_packed=True)
    assert np.array_equal(got["codes"], ref["codes"])
    assert np.array_equal(got["scales"].view(np.uint32), ref["scales"].view(np.uint32))
    assert np.array_equal(got["zeros"], ref["zeros"])
    assert np.array_equal(got["dW"], ref["dW"])
    assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, bits))


@pytest.mark.parametrize("dim,group", [(OC, 128), (IC, 128)])
def test_end_to_end_improves_on_rtn(ctx, dim, group):
    out_f, in_f, bits = 256, 768, 3
    W, X = layer(out_f, in_f, 1500, seed=77)
    H = oracle.hessian(X)
    H32 = H.astype(np.float32)
    ref = G.gptq(W, H32, dim, bits, group)
    perm, dead, U = gpu_prepare(ctx, H32)
    got = gpu_sweep(ctx, W, dim, bits, group, U, perm, dead)
    assert (got["codes"] == ref["codes"]).mean() > 0.98
    l_gpu, l_ref = oracle.layer_error(got["dW"], H), oracle.layer_error(ref["dW"], H)
    l_rtn = oracle.layer_error(oracle.quantize(W, dim, bits, group)["dW"], H)
    assert l_gpu == pytest.approx(l_ref, rel=0.02)
    assert l_gpu < 0.9 * l_rtn
    # the library's own scoring of the result agrees with the oracle's
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    ctx.adadim_layer_error(dev(got["dW"]), B.DW_F32, dev(H32), loss)
    torch.cuda.synchronize()
    assert loss.item() == pytest.approx(l_gpu, rel=1e-3)


def test_q_proj_shape_sampled(ctx):
    """LLaMA-7B q_proj shape, 8192 calibration tokens: the fp64 factor of a 4096-wide Hessian to
    fp32 rounding, and the sweep bit-exact on sampled rows (per-OC rows and per-IC row groups are
    independent, so the oracle can sweep them alone)."""
    out_f = in_f = 4096
    W = synth.config_weight(1, "q_proj")
    X = synth.config_activations(1, in_f, tokens=8192)
    H32 = oracle.hessian(X).astype(np.float32)
    Hp, perm_ref, dead_ref = G.prepare(H32, 0.01, True)
    U_ref = G.factor(Hp)
    perm, dead, U = gpu_prepare(ctx, H32)
    assert np.array_equal(perm.cpu().numpy().astype(np.int64), perm_ref)
    Ug = U.cpu().numpy().astype(np.float64)
    assert (np.abs(Ug - U_ref) <= 4e-6 * np.abs(U_ref) + 2e-7 * np.abs(U_ref).max()).all()
    del Ug
    U32 = U_ref.astype(np.float32)
    Ud, pd, dd = dev(U32), dev(perm_ref.astype(np.int32)), dev(dead_ref.astype(np.uint8))
    rng = np.random.default_rng(0)
    got = gpu_sweep(ctx, W, OC, 3, 128, Ud, pd, dd)
    rows = np.sort(rng.choice(out_f, 6, replace=False))
    ref = G.sweep(W[rows], U32, perm_ref, dead_ref, OC, 3, 128)
    assert np.array_equal(got["codes"][rows], ref["codes"])
    assert np.array_equal(got["dW"][rows], ref["dW"])
    got = gpu_sweep(ctx, W, IC, 3, 128, Ud, pd, dd)
    for rg in (0, 17):
        sl = slice(rg * 128, (rg + 1) * 128)
        ref = G.sweep(W[sl], U32, perm_ref, dead_ref, IC, 3, 128)
        assert np.array_equal(got["codes"][sl], ref["codes"])
        assert np.array_equal(got["scales"][rg], ref["scales"][0])
        assert np.array_equal(got["zeros"][rg], ref["zeros"][0])
        assert np.array_equal(got["dW"][sl], ref["dW"])


@pytest.mark.parametrize("out_f,in_f,dim,bits,group", [
    (128, 320, OC, 3, 64),
    (200, 264, OC, 4, 0),
    (256, 264, IC, 3, 128),
    (192, 384, IC, 4, 64),
    (128, 1160, IC, 2, 128),
])
def test_sweep_in_the_storage_format_bit_exact(ctx, out_f, in_f, dim, bits, group):
    """adadim_gptq_quantize_meta16 against the oracle's sweep with every scale rounded into the group word."""
    from oracle import meta16_oracle as m16
    W, X = layer(out_f, in_f, 900, seed=out_f + in_f + 1, dead=(5,))
    H32 = oracle.hessian(X).astype(np.float32)
    Hp, perm, dead = G.prepare(H32, 0.01, True)
    U32 = G.factor(Hp).astype(np.float32)
    ref = m16.gptq_sweep(W, U32, perm, dead, dim, bits, group)
    Wd, Ud, pd, dd = dev(W), dev(U32), dev(perm.astype(np.int32)), dev(dead.astype(np.uint8))
    codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda")
    dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
    n_ch, ln = (out_f, in_f) if dim == OC else (in_f, out_f)
    packed = torch.full((n_ch, (ln * bits + 31) // 32), -1, dtype=torch.int32, device="cuda")
    if dim == OC:
        g = in_f if group == 0 else group
        meta = torch.full((out_f, in_f // g), -1, dtype=torch.int16, device="cuda")
        Wz = Wd.clone()
        Wz[:, dd.bool()] = 0
        ctx.adadim_quantize_meta16(Wz, OC, bits, group, 1.0, meta=meta)
        ctx.adadim_gptq_quantize_meta16(Wd, dim, bits, group, Ud, pd, dd, codes, static_meta=meta, dW=dW, packed=packed)
    else:
        meta = torch.full((out_f // group, in_f), -1, dtype=torch.int16, device="cuda")
        ctx.adadim_gptq_quantize_meta16(Wd, dim, bits, group, Ud, pd, dd, codes, meta=meta, dW=dW, packed=packed)
    torch.cuda.synchronize()
    assert np.array_equal(meta.cpu().numpy().view(np.uint16), ref["meta"])
    assert np.array_equal(codes.cpu().numpy(), ref["codes"])
    assert np.array_equal(dW.cpu().numpy(), ref["dW"])
    assert np.array_equal(packed.cpu().numpy().view(np.uint32), oracle.pack(ref["codes"], dim, bits))


def test_gptq_ada_in_the_storage_format(ctx):
    """GptqAda(meta16=True): search and sweep in the format; the result improves on RTN and its words and codes give
    the dW that was scored."""
    from oracle import meta16_oracle as m16
    out_f, in_f, bits, group = 256, 512, 4, 128
    W, X = layer(out_f, in_f, 2000, seed=77)
    hp = S.PreparedHessian(ctx, in_f).update(dev(X)).prepare()
    fac = S.GptqFactor(ctx, hp)
    ga = S.GptqAda(ctx, out_f, in_f, bits, group, meta16=True)
    dim = ga.run(dev(W), hp, fac)
    torch.cuda.synchronize()
    assert ga.loss_gptq.item() < ga.loss_rtn.item()
    meta = ga.meta.cpu().numpy().view(np.uint16).reshape((out_f, in_f // group) if dim == OC else (out_f // group, in_f))
    s, z = m16.decode(meta, bits)
    rep = (lambda a: np.repeat(a, group, axis=1)) if dim == OC else (lambda a: np.repeat(a, group, axis=0))
    what = (rep(s) * (ga.codes.cpu().numpy().astype(np.float32) - rep(z).astype(np.float32))).astype(np.float32)
    assert np.array_equal(ga.dW.cpu().numpy(), W.astype(np.float32) - what)


@pytest.mark.parametrize("dim,group", [(OC, 128), (IC, 64)])
def test_wide_layer_with_a_diagonal_factor(ctx, dim, group):
    """in = 33280 (a row of W no longer fits the default 64 KB of LDS in the permuting copy; 260 blocks): with a
    diagonal factor nothing propagates, so the sweep in a scrambled visiting order must give the plain quantizer's
    codes, parameters and dW (Sec. 3.3 with a diagonal H; the oracle's quantize is the reference)."""
    out_f, in_f, bits = 64, 33280, 3
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    ref = oracle.quantize(W, dim, bits, group)
    Wd = dev(W)
    U = torch.zeros((in_f, in_f), dtype=torch.float32, device="cuda")
    U.diagonal().copy_(torch.linspace(0.5, 2.0, in_f, device="cuda"))       # any positive diagonal
    perm = torch.from_numpy(rng.permutation(in_f).astype(np.int32)).cuda()
    dead = torch.zeros(in_f, dtype=torch.uint8, device="cuda")
    codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda")
    dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
    if dim == OC:
        sc = torch.empty((out_f, in_f // group), dtype=torch.float32, device="cuda")
        zp = torch.empty((out_f, in_f // group), dtype=torch.uint8, device="cuda")
        ctx.adadim_quantize(Wd, OC, bits, group, 1.0, scales=sc, zeros=zp)
        ctx.adadim_gptq_quantize(Wd, dim, bits, group, U, perm, dead, codes, static_scales=sc, static_zeros=zp, dW=dW)
    else:
        sc = torch.full((out_f // group, in_f), float("nan"), dtype=torch.float32, device="cuda")
        zp = torch.full((out_f // group, in_f), 255, dtype=torch.uint8, device="cuda")
        ctx.adadim_gptq_quantize(Wd, dim, bits, group, U, perm, dead, codes, scales=sc, zeros=zp, dW=dW)
    torch.cuda.synchronize()
    assert np.array_equal(sc.cpu().numpy(), ref["scales"])
    assert np.array_equal(zp.cpu().numpy(), ref["zeros"])
    assert np.array_equal(codes.cpu().numpy(), ref["codes"])
    assert np.array_equal(dW.cpu().numpy(), ref["dW"])


def _random_sweep_cases(n, seed):
    """Seeded shapes for the sweep: odd row counts per-OC (ragged row tiles), every residue of the last block and
    of its last 16-channel sub-block, groups that do and do not line up with the 128-channel blocks."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        bits = int(rng.choice([2, 3, 4, 8]))
        if i % 2 == 0:
            group = int(rng.choice([0, 8, 24, 40, 64, 128]))
            g = group if group else 1
            in_f = g * int(rng.integers(max(1, 40 // g), max(2, 420 // g) + 1))
            out_f = int(rng.integers(1, 150))
            cases.append((out_f, in_f, OC, bits, group))
        else:
            group = int(rng.choice([64, 128]))
            out_f = group * int(rng.integers(1, 4))
            in_f = 4 * int(rng.integers(8, 110))
            cases.append((out_f, in_f, IC, min(bits, 8), group))
    return cases


@pytest.mark.parametrize("out_f,in_f,dim,bits,group", _random_sweep_cases(24, 11))
def test_sweep_bit_exact_random_shapes(ctx, out_f, in_f, dim, bits, group):
    W, X = layer(out_f, in_f, max(2 * in_f, 300), seed=3 * out_f + in_f, dead=(1,) if in_f > 60 else ())
    H32 = oracle.hessian(X).astype(np.float32)
    Hp, perm, dead = G.prepare(H32, 0.01, True)
    U32 = G.factor(Hp).astype(np.float32)
    ref = G.sweep(W, U32, perm, dead, dim, bits, group)
    got = gpu_sweep(ctx, W, dim, bits, group, dev(U32), dev(perm.astype(np.int32)), dev(dead.astype(np.uint8)),
                    want_packed=bits <= 8 and (dim == OC or out_f * bits % 32 == 0))
    assert np.array_equal(got["codes"], ref["codes"])
    assert np.array_equal(got["scales"].view(np.uint32), ref["scales"].view(np.uint32))
    assert np.array_equal(got["zeros"], ref["zeros"])
    assert np.array_equal(got["dW"], ref["dW"])
    if "packed" in got:
        assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, bits))


@pytest.mark.parametrize("out_f,in_f,dim,bits,group",
                         [c for c in _random_sweep_cases(40, 23) if c[3] <= 4 and not (c[2] == OC and c[4] == 0 and c[1] % 2)][:14])
def test_sweep_in_the_storage_format_random_shapes(ctx, out_f, in_f, dim, bits, group):
    """The same in the b + 16/g format (bits 2..4), against the oracle's sweep with rounded scales."""
    from oracle import meta16_oracle as m16
    W, X = layer(out_f, in_f, max(2 * in_f, 300), seed=5 * out_f + in_f, dead=(2,) if in_f > 60 else ())
    H32 = oracle.hessian(X).astype(np.float32)
    Hp, perm, dead = G.prepare(H32, 0.01, True)
    U32 = G.factor(Hp).astype(np.float32)
    ref = m16.gptq_sweep(W, U32, perm, dead, dim, bits, group)
    Wd, Ud, pd, dd = dev(W), dev(U32), dev(perm.astype(np.int32)), dev(dead.astype(np.uint8))
    codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda")
    dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
    if dim == OC:
        g = in_f if group == 0 else group
        meta = torch.full((out_f, in_f // g), -1, dtype=torch.int16, device="cuda")
        Wz = Wd.clone()
        Wz[:, dd.bool()] = 0
        ctx.adadim_quantize_meta16(Wz, OC, bits, group, 1.0, meta=meta)
        ctx.adadim_gptq_quantize_meta16(Wd, dim, bits, group, Ud, pd, dd, codes, static_meta=meta, dW=dW)
    else:
        meta = torch.full((out_f // group, in_f), -1, dtype=torch.int16, device="cuda")
        ctx.adadim_gptq_quantize_meta16(Wd, dim, bits, group, Ud, pd, dd, codes, meta=meta, dW=dW)
    torch.cuda.synchronize()
    assert np.array_equal(meta.cpu().numpy().view(np.uint16), ref["meta"])
    assert np.array_equal(codes.cpu().numpy(), ref["codes"])
    assert np.array_equal(dW.cpu().numpy(), ref["dW"])
