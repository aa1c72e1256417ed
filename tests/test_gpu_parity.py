"""GPU parity: every library call against the CPU oracle on the same seeded inputs.

Bars: codes, zeros, scales, packed streams and the chosen index are bit-exact;
fp32 dW is bit-exact (same formulas, one rounding per operation); fp16 dW is
the round-to-nearest-even of the oracle's fp32 dW; H within 2e-5*sqrt(H_ii H_jj)
(fp32 accumulation of exact fp16 products); the layer error within 1e-3
relative of the fp64 oracle; the winning dimension is compared only where the
two losses differ by more than 1 %.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import OC, IC
from paper_2309_15531_amd import binding as B
from paper_2309_15531_amd import search as S
from paper_2309_15531_amd import synth

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
H_TOL = 2e-5


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = B.Context()
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def gpu_quantize(ctx, W, dim, bits, group, clip=1.0, dW_dtype=B.DW_F32, colscale=None, want_packed=True,
                 want_codes=True):
    out_f, in_f = W.shape
    g = (in_f if dim == OC else out_f) if group == 0 else group
    meta = (out_f, in_f // g) if dim == OC else (out_f // g, in_f)
    Wd = dev(W)
    codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda") if want_codes else None
    scales = torch.full(meta, -1.0, dtype=torch.float32, device="cuda")
    zeros = torch.full(meta, 255, dtype=torch.uint8, device="cuda")
    if dW_dtype == B.DW_F16_SCALED:
        dW = ctx.alloc_score(out_f, in_f).fill_(float("nan"))   # flat, last row tile padded
    else:
        dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32 if dW_dtype == B.DW_F32 else torch.float16,
                        device="cuda")
    n_ch, ln = (out_f, in_f) if dim == OC else (in_f, out_f)
    packed = torch.full((n_ch, (ln * bits + 31) // 32), -1, dtype=torch.int32, device="cuda") if want_packed else None
    ctx.adadim_quantize(Wd, dim, bits, group, clip, codes=codes, scales=scales, zeros=zeros, dW=dW,
                        dW_dtype=dW_dtype, colscale=colscale, packed=packed)
    torch.cuda.synchronize()
    return {
        "codes": codes.cpu().numpy() if want_codes else None,
        "scales": scales.cpu().numpy(), "zeros": zeros.cpu().numpy(), "dW": dW.cpu().numpy(),
        "packed": packed.cpu().numpy().view(np.uint32) if want_packed else None,
    }


def rand_w(out_f, in_f, seed):
    return synth.make_weight(out_f, in_f, seed, heavy_cols=max(1, in_f // 100), heavy_scale=5.0)


QUANT_CASES = [
    # out, in, bits, group      (several tiles, ragged tails, every kernel path)
    (512, 512, 3, 64),          # the toy workload's setting
    (384, 640, 4, 128),
    (256, 1024, 2, 64),
    (640, 264, 3, 8),           # in not a multiple of the 256-column tile
    (520, 328, 4, 0),           # whole-channel groups
    (96, 1536, 8, 512),         # 64 lanes per group
    (768, 768, 5, 256),
    (240, 72, 3, 24),           # group not a power of two -> element-wise path
    (100, 70, 4, 10),           # in % 8 != 0 -> scalar paths for both dims
    (128, 128, 3, 16),
    (64, 4096, 3, 32),
    (72, 1024, 3, 0),           # wide groups: three passes, the per-OC bit stream written by the last
    (64, 2048, 2, 1024),
    (40, 1536, 8, 768),
    (48, 1056, 4, 528),
]


@pytest.mark.parametrize("dim", [OC, IC])
@pytest.mark.parametrize("out_f,in_f,bits,group", QUANT_CASES)
def test_quantize_bit_exact(ctx, dim, out_f, in_f, bits, group):
    axis = in_f if dim == OC else out_f
    if group and axis % group:
        pytest.skip("group does not divide this axis")
    W = rand_w(out_f, in_f, seed=out_f * 7 + in_f + bits)
    ref = oracle.quantize(W, dim, bits, group)
    got = gpu_quantize(ctx, W, dim, bits, group)
    assert np.array_equal(got["scales"].view(np.uint32), ref["scales"].view(np.uint32))
    assert np.array_equal(got["zeros"], ref["zeros"])
    assert np.array_equal(got["codes"], ref["codes"])
    assert np.array_equal(got["dW"], ref["dW"])
    assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, bits))


@pytest.mark.parametrize("seed", range(12))
def test_quantize_random_shapes(ctx, seed):
    """Seeded random shapes, precisions, group lengths and clip ratios, both dimensions: whatever kernel path the
    shape selects, every output bit for bit."""
    rng = np.random.default_rng(1000 + seed)
    out_f, in_f = 8 * int(rng.integers(4, 120)), 8 * int(rng.integers(4, 160))
    bits = int(rng.choice([2, 3, 4, 5, 8]))
    clip = 1.0 if seed % 3 else float(np.float32(rng.uniform(0.6, 1.0)))
    W = rand_w(out_f, in_f, seed=2000 + seed)
    for dim in (OC, IC):
        axis = in_f if dim == OC else out_f
        fits = [g for g in (8, 16, 32, 64, 128, 256) if axis % g == 0]
        group = int(rng.choice(fits + [0]))
        ref = oracle.quantize(W, dim, bits, group, clip)
        got = gpu_quantize(ctx, W, dim, bits, group, clip)
        what = f"out={out_f} in={in_f} bits={bits} group={group} dim={dim} clip={clip}"
        assert np.array_equal(got["scales"].view(np.uint32), ref["scales"].view(np.uint32)), what
        assert np.array_equal(got["zeros"], ref["zeros"]), what
        assert np.array_equal(got["codes"], ref["codes"]), what
        assert np.array_equal(got["dW"], ref["dW"]), what
        assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, bits)), what


@pytest.mark.parametrize("dim", [OC, IC])
@pytest.mark.parametrize("clip", [0.5, 0.7368421, 0.97])
def test_quantize_clip_and_fp16_outputs(ctx, dim, clip):
    W = rand_w(256, 512, seed=77)
    clip = float(np.float32(clip))
    ref = oracle.quantize(W, dim, 3, 64, clip)
    got = gpu_quantize(ctx, W, dim, 3, 64, clip, dW_dtype=B.DW_F16)
    assert np.array_equal(got["scales"].view(np.uint32), ref["scales"].view(np.uint32))
    assert np.array_equal(got["zeros"], ref["zeros"])
    assert np.array_equal(got["codes"], ref["codes"])
    assert np.array_equal(got["dW"], ref["dW"].astype(np.float16))
    # column-scaled fp16 dW: powers of two commute with the rounding
    cs = np.ldexp(np.float32(1.0), np.random.default_rng(3).integers(-2, 9, size=512)).astype(np.float32)
    got = gpu_quantize(ctx, W, dim, 3, 64, clip, dW_dtype=B.DW_F16_SCALED, colscale=dev(cs))
    assert np.array_equal(B.from_score_layout(got["dW"], 256, 512), (ref["dW"] * cs[None, :]).astype(np.float16))
    # the same with row counts that leave the last 256-row tile of the scoring layout ragged
    for (o2, i2, g2) in ((384, 640, 128), (640, 264, 8), (96, 1536, 32)):
        W2 = rand_w(o2, i2, seed=o2 + i2)
        cs2 = np.ldexp(np.float32(1.0), np.random.default_rng(4).integers(-2, 9, size=i2)).astype(np.float32)
        ref2 = oracle.quantize(W2, dim, 4, g2, clip)
        got2 = gpu_quantize(ctx, W2, dim, 4, g2, clip, dW_dtype=B.DW_F16_SCALED, colscale=dev(cs2), want_packed=False)
        assert np.array_equal(B.from_score_layout(got2["dW"], o2, i2), (ref2["dW"] * cs2[None, :]).astype(np.float16))
        assert np.array_equal(got2["codes"], ref2["codes"])
    # packed stream without a caller-side code buffer
    got = gpu_quantize(ctx, W, dim, 3, 64, clip, want_codes=False)
    assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, 3))


@pytest.mark.parametrize("dim", [OC, IC])
def test_quantize_degenerate_groups(ctx, dim):
    """All-zero groups, one-sided groups, on-grid weights (exact fixed point)."""
    W = rand_w(128, 256, seed=5)
    W[:32] = 0
    W[32:64] = np.abs(W[32:64])
    W[64:96] = -np.abs(W[64:96])
    ref = oracle.quantize(W, dim, 3, 32)
    got = gpu_quantize(ctx, W, dim, 3, 32)
    for k in ("scales", "zeros", "codes", "dW"):
        assert np.array_equal(got[k], ref[k]), k
    Wg, q, z, s = synth.on_grid_weight(128, 256, dim, 4, 64, seed=2)
    got = gpu_quantize(ctx, Wg, dim, 4, 64)
    assert np.array_equal(got["codes"], q) and np.array_equal(got["zeros"], z)
    assert np.array_equal(got["scales"], s) and not got["dW"].any()


def gpu_hessian(ctx, X, accumulate_chunks=None, ld_pad=0):
    t, in_f = X.shape
    if ld_pad:
        Xp = torch.zeros((t, in_f + ld_pad), dtype=torch.float16, device="cuda")
        Xp[:, :in_f] = dev(X)
        Xd = Xp[:, :in_f]
    else:
        Xd = dev(X)
    H = torch.full((in_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
    if accumulate_chunks is None:
        ctx.adadim_hessian(Xd, H)
    else:
        bounds = np.linspace(0, t, accumulate_chunks + 1).astype(int)
        for i in range(accumulate_chunks):
            ctx.adadim_hessian(Xd[bounds[i]:bounds[i + 1]], H, accumulate=i > 0)
    torch.cuda.synchronize()
    return H.cpu().numpy()


def check_hessian(Hg, Href):
    d = np.sqrt(np.maximum(np.diag(Href), 1e-30))
    err = np.abs(Hg.astype(np.float64) - Href) / (d[:, None] * d[None, :])
    assert err.max() <= H_TOL, err.max()
    assert np.array_equal(Hg, Hg.T)


@pytest.mark.parametrize("tokens,in_f", [(256, 512), (1000, 264), (77, 1288), (4096, 128), (3000, 2056), (1, 64),
                                         (70, 6144), (200, 6008), (40, 6016),    # 300 tiles, 256 of them stored whole
                                         (12000, 4096), (9999, 3080), (4097, 5128)])   # token ranges cut two and three ways, ragged
def test_hessian(ctx, tokens, in_f):
    X = synth.make_activations(tokens, in_f, seed=tokens + in_f, n_outliers=3, scale_lo=50, scale_hi=100)
    check_hessian(gpu_hessian(ctx, X), oracle.hessian(X))


def test_hessian_accumulate_and_pitch(ctx):
    X = synth.make_activations(1500, 520, seed=9, n_outliers=4, scale_lo=30, scale_hi=60, relu=True)
    Href = oracle.hessian(X)
    check_hessian(gpu_hessian(ctx, X, accumulate_chunks=3), Href)
    check_hessian(gpu_hessian(ctx, X, ld_pad=24), Href)
    # wide enough for whole-tile stores: the first chunk takes them, the accumulating second one may not
    Xw = synth.make_activations(90, 6144, seed=10, n_outliers=4, scale_lo=30, scale_hi=60)
    check_hessian(gpu_hessian(ctx, Xw, accumulate_chunks=2), oracle.hessian(Xw))
    # tokens == 0 clears H
    H = torch.ones((64, 64), dtype=torch.float32, device="cuda")
    ctx.adadim_hessian(torch.empty((0, 64), dtype=torch.float16, device="cuda"), H)
    torch.cuda.synchronize()
    assert not H.cpu().numpy().any()


def test_hessian_with_cut_rests(ctx):
    """A shape whose launch plan cuts the token range three ways (17 tiles per XCD on 32 units: one full piece per
    tile, the rest whole for most tiles and in four short pieces for sixteen of them; tests/host/gram_plan_check
    prints the plan with arguments "8232 4096"), with a ragged last stage: plain, accumulated over two chunks, and
    through the call that also prepares H for scoring."""
    tokens, in_f = 8232, 4096
    X = synth.make_activations(tokens, in_f, seed=77, n_outliers=6, scale_lo=30, scale_hi=80)
    Href = oracle.hessian(X)
    check_hessian(gpu_hessian(ctx, X), Href)
    Xd = dev(X)
    H = torch.zeros((in_f, in_f), dtype=torch.float32, device="cuda")
    ctx.adadim_hessian(Xd[:4000], H)                              # a different plan
    ctx.adadim_hessian(Xd[4000:], H, accumulate=True)
    torch.cuda.synchronize()
    check_hessian(H.cpu().numpy(), Href)
    H1 = torch.full((in_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
    Hs = ctx.alloc_score(in_f, in_f).fill_(float("nan"))
    hmeta = torch.full((2, in_f), float("nan"), dtype=torch.float32, device="cuda")
    ctx.adadim_hessian_prepared(Xd, H1, Hs, hmeta)
    H2 = torch.empty_like(H1)
    ctx.adadim_hessian(Xd, H2)
    torch.cuda.synchronize()
    assert np.array_equal(H1.cpu().numpy().view(np.uint32), H2.cpu().numpy().view(np.uint32))
    check_hessian(H1.cpu().numpy(), Href)
    assert np.array_equal(hmeta[1].cpu().numpy(), np.diag(H1.cpu().numpy()))


def test_hessian_reproducible(ctx):
    X = synth.make_activations(5000, 776, seed=4, n_outliers=2, scale_lo=50, scale_hi=50)
    a, b = gpu_hessian(ctx, X), gpu_hessian(ctx, X)
    assert np.array_equal(a, b)


ERR_CASES = [(512, 512, 256), (384, 640, 1000), (264, 328, 300), (1288, 264, 500), (96, 2056, 2048)]


@pytest.mark.parametrize("out_f,in_f,tokens", ERR_CASES)
@pytest.mark.parametrize("dW_dtype", [B.DW_F32, B.DW_F16])
def test_layer_error(ctx, out_f, in_f, tokens, dW_dtype):
    W = rand_w(out_f, in_f, seed=out_f + in_f)
    X = synth.make_activations(tokens, in_f, seed=in_f, n_outliers=4, scale_lo=50, scale_hi=100,
                               relu=(in_f == 2056))
    H64 = oracle.hessian(X)
    Hg = dev(gpu_hessian(ctx, X))
    for dim in (OC, IC):
        group = 8
        dw = oracle.quantize(W, dim, 3, group)["dW"]
        if dW_dtype == B.DW_F16:
            dw = dw.astype(np.float16)
        rows_ref = oracle.layer_error_rows(dw, H64)
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        rows = torch.zeros(out_f, dtype=torch.float32, device="cuda")
        ctx.adadim_layer_error(dev(dw), dW_dtype, Hg, loss, loss_rows=rows)
        torch.cuda.synchronize()
        assert loss.item() == pytest.approx(rows_ref.sum(), rel=LOSS_RTOL)
        r = rows.cpu().numpy().astype(np.float64)
        assert np.abs(r - rows_ref).max() <= LOSS_RTOL * rows_ref.max()
        assert r.sum() == pytest.approx(loss.item(), rel=1e-5)


@pytest.mark.parametrize("in_f", [520, 544])   # row-major and k-blocked scoring layouts
def test_layer_error_prepared_matches_and_scaled_input(ctx, in_f):
    out_f = 640
    W = rand_w(out_f, in_f, seed=1)
    X = synth.make_activations(700, in_f, seed=2, n_outliers=3, scale_lo=60, scale_hi=60)
    hp = S.PreparedHessian(ctx, in_f).update(dev(X)).prepare()
    torch.cuda.synchronize()
    hmeta = hp.hmeta.cpu().numpy()
    Hg = hp.H.cpu().numpy()
    # column scales are powers of two within a factor sqrt(2) of sqrt(H_jj) / 64
    m, e = np.frexp(hmeta[0])
    assert (m == 0.5).all()
    assert np.array_equal(hmeta[1], np.diag(Hg))
    ratio = hmeta[0] * 64.0 / np.sqrt(np.diag(Hg))
    assert (ratio > 0.70).all() and (ratio < 1.42).all()
    Hs = B.from_score_layout(hp.Hs.cpu().numpy(), in_f, in_f).astype(np.float64)
    assert not np.triu(Hs).any() and np.abs(Hs).max() <= 2.0 * 4096.0
    d = hmeta[0].astype(np.float64)
    assert np.allclose(Hs, np.tril(Hg.astype(np.float64) / d[:, None] / d[None, :], -1), rtol=2.0 ** -10, atol=1e-7 * 4096.0)
    ref = oracle.layer_error(oracle.quantize(W, IC, 3, 64)["dW"], oracle.hessian(X))
    Wd = dev(W)
    dW = ctx.alloc_score(out_f, in_f)   # 640 rows: the last 256-row tile of the scoring layout is half empty
    losses = torch.zeros(3, dtype=torch.float32, device="cuda")
    ctx.adadim_quantize(Wd, IC, 3, 64, dW=dW, dW_dtype=B.DW_F16_SCALED, colscale=hp.colscale)
    ctx.adadim_layer_error_prepared(dW, B.DW_F16_SCALED, hp.Hs, hp.hmeta, losses[0:1], shape=(out_f, in_f))
    dW32 = torch.empty((out_f, in_f), dtype=torch.float32, device="cuda")
    ctx.adadim_quantize(Wd, IC, 3, 64, dW=dW32, dW_dtype=B.DW_F32)
    ctx.adadim_layer_error_prepared(dW32, B.DW_F32, hp.Hs, hp.hmeta, losses[1:2])
    ctx.adadim_layer_error(dW32, B.DW_F32, hp.H, losses[2:3])
    torch.cuda.synchronize()
    got = losses.cpu().numpy()
    assert got[1] == got[2]
    assert got == pytest.approx([ref] * 3, rel=LOSS_RTOL)


def test_layer_error_zero_and_identity(ctx):
    """dW = 0 gives exactly 0; H = I gives ||dW||_F^2."""
    n = 256
    H = torch.eye(n, dtype=torch.float32, device="cuda")
    loss = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    ctx.adadim_layer_error(torch.zeros((128, n), dtype=torch.float32, device="cuda"), B.DW_F32, H, loss)
    torch.cuda.synchronize()
    assert loss.item() == 0.0
    d = np.random.default_rng(0).standard_normal((128, n)).astype(np.float32) * 0.01
    ctx.adadim_layer_error(dev(d), B.DW_F32, H, loss)
    torch.cuda.synchronize()
    assert loss.item() == pytest.approx(float(np.sum(d.astype(np.float64) ** 2)), rel=1e-5)


def test_select(ctx):
    for vals, want in [([1.0, 1.0], 0), ([2.0, 1.0], 1), ([3.0, 2.0, 2.0, 5.0], 1),
                       ([float("nan"), 4.0, 3.0], 2), ([5.0] * 40, 0), ([float("nan"), 2.0], 1), ([2.0, float("nan")], 0),
                       ([float("nan"), float("nan")], 0), ([float("inf"), 2.0], 1), ([float("inf"), float("inf")], 0)]:
        t = torch.tensor(vals, dtype=torch.float32, device="cuda")
        best_dev = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        assert ctx.adadim_select(t, best_dev=best_dev) == want
        assert oracle.select(vals) == want
        assert ctx.adadim_select(t) == want
        assert best_dev.item() == want


def run_search(ctx, W, X, bits, group, clips=(1.0,)):
    in_f = W.shape[1]
    hp = S.PreparedHessian(ctx, in_f).update(dev(X)).prepare()
    ls = S.LayerSearch(ctx, W.shape[0], in_f, bits, group, clips)
    best, dim, clip = ls.run(dev(W), hp)
    torch.cuda.synchronize()
    return ls, best, dim, clip


def test_toy_workload_end_to_end(ctx):
    """The 512x512 workload: full search against the full oracle."""
    cfg = synth.CONFIGS[0]
    W, X = synth.config_weight(0, "fc"), synth.config_activations(0, 512)
    ref = oracle.search(W, X, cfg["bits"][0], cfg["group"])
    ls, best, dim, clip = run_search(ctx, W, X, cfg["bits"][0], cfg["group"])
    got = ls.losses.cpu().numpy()
    assert got == pytest.approx(ref["losses"], rel=LOSS_RTOL)
    # direct definition of Eq. 1 on this small case
    assert got[0] == pytest.approx(oracle.layer_error_direct(X, W, oracle.quantize(W, OC, 3, 64)["What"]),
                                   rel=LOSS_RTOL)
    lo, hi = min(ref["losses"]), max(ref["losses"])
    if (hi - lo) / lo > 0.01:
        assert best == ref["best"] and dim == ref["dim"]
    q = ref["quant"] if dim == ref["dim"] else oracle.quantize(W, dim, 3, 64)
    n_meta = q["scales"].size
    assert np.array_equal(ls.scales[:n_meta].cpu().numpy(), q["scales"].ravel())
    assert np.array_equal(ls.zeros[:n_meta].cpu().numpy(), q["zeros"].ravel())
    pk = oracle.pack(q["codes"], dim, 3)
    assert np.array_equal(ls.packed[:pk.size].cpu().numpy().view(np.uint32), pk.ravel())


def test_clip_grid_search(ctx):
    W = rand_w(256, 512, seed=31)
    X = synth.make_activations(512, 512, seed=32, n_outliers=4, scale_lo=100, scale_hi=100)
    clips = oracle.clip_grid(20)
    assert S.clip_grid(20) == [float(c) for c in clips]
    ref = oracle.search(W, X, 2, 64, clips=clips)
    ls, best, dim, clip = run_search(ctx, W, X, 2, 64, clips=S.clip_grid(20))
    got = ls.losses.cpu().numpy()
    assert len(got) == 40
    assert got == pytest.approx(ref["losses"], rel=LOSS_RTOL)
    srt = np.sort(ref["losses"])
    if (srt[1] - srt[0]) / srt[0] > 0.01:
        assert best == ref["best"] and (dim, np.float32(clip)) == (ref["dim"], np.float32(ref["clip"]))
    else:
        assert ref["losses"][best] <= srt[0] * 1.01


def test_choice_flips_under_transpose_gpu(ctx):
    n = 256
    X = np.eye(n, dtype=np.float16)
    rng = np.random.default_rng(13)
    W = rng.standard_normal((n, n)).astype(np.float32) * 0.02
    W[:, rng.choice(n, 8, replace=False)] *= 12.0
    W = W.astype(np.float16)
    _, _, dim_a, _ = run_search(ctx, W, X, 3, 32)
    _, _, dim_b, _ = run_search(ctx, np.ascontiguousarray(W.T), X, 3, 32)
    assert (dim_a, dim_b) == (IC, OC)


def _check_winner(ls_scales, ls_zeros, ls_packed, W, dim, bits, group):
    q = oracle.quantize(W, dim, bits, group)
    n_meta = q["scales"].size
    assert np.array_equal(ls_scales[:n_meta].cpu().numpy(), q["scales"].ravel())
    assert np.array_equal(ls_zeros[:n_meta].cpu().numpy(), q["zeros"].ravel())
    pk = oracle.pack(q["codes"], dim, bits)
    assert np.array_equal(ls_packed[:pk.size].cpu().numpy().view(np.uint32), pk.ravel())


@pytest.mark.parametrize("bits", [3, 4])
@pytest.mark.parametrize("group", [256, 128, 64, 0])
def test_group_size_sweep(ctx, bits, group):
    """The paper's sweep of precisions and group sizes (Sec. 4.4), plus whole-channel groups:
    full search against the oracle, winner's stored outputs bit-exact."""
    out_f, in_f = 768, 1024
    W = rand_w(out_f, in_f, seed=900 + bits + group)
    X = synth.make_activations(1100, in_f, seed=17, n_outliers=4, scale_lo=50, scale_hi=100)
    ref = oracle.search(W, X, bits, group)
    ls, best, dim, clip = run_search(ctx, W, X, bits, group)
    got = ls.losses.cpu().numpy()
    assert got == pytest.approx(ref["losses"], rel=LOSS_RTOL)
    lo, hi = min(ref["losses"]), max(ref["losses"])
    if (hi - lo) / lo > 0.01:
        assert best == ref["best"]
    _check_winner(ls.scales, ls.zeros, ls.packed, W, dim, bits, group)


@pytest.mark.parametrize("seed", range(8))
def test_search_random_shapes(ctx, seed):
    """The whole search on seeded random layer shapes, token counts, precisions and group lengths (ragged tiles of
    every kernel on the path): both losses against the fp64 oracle, the winner when it is clear, and the winner's
    stored outputs bit for bit."""
    rng = np.random.default_rng(3000 + seed)
    group = int(rng.choice([32, 64, 128]))
    out_f, in_f = group * int(rng.integers(2, 1536 // group)), group * int(rng.integers(2, 2560 // group))
    tokens, bits = int(rng.integers(50, 3000)), int(rng.choice([2, 3, 4]))
    W = rand_w(out_f, in_f, seed=4000 + seed)
    X = synth.make_activations(tokens, in_f, seed=5000 + seed, n_outliers=int(rng.integers(0, 6)), scale_lo=30, scale_hi=100,
                               relu=bool(seed & 1))
    ref = oracle.search(W, X, bits, group)
    ls, best, dim, clip = run_search(ctx, W, X, bits, group)
    what = f"out={out_f} in={in_f} tokens={tokens} bits={bits} group={group}"
    assert ls.losses.cpu().numpy() == pytest.approx(ref["losses"], rel=LOSS_RTOL), what
    lo, hi = min(ref["losses"]), max(ref["losses"])
    if (hi - lo) / lo > 0.01:
        assert best == ref["best"], what
    _check_winner(ls.scales, ls.zeros, ls.packed, W, dim, bits, group)


def test_shared_input_search(ctx):
    """Three layers that see the same input (q, k, v): one H, one scoring launch for all six
    candidates; every layer's losses equal the single-layer search's, winners bit-exact."""
    out_f, in_f, bits, group = 512, 768, 3, 128
    Ws = [rand_w(out_f, in_f, seed=700 + l) for l in range(3)]
    X = synth.make_activations(900, in_f, seed=23, n_outliers=3, scale_lo=60, scale_hi=90)
    hp = S.PreparedHessian(ctx, in_f).update(dev(X)).prepare()
    sh = S.SharedSearch(ctx, 3, out_f, in_f, bits, group)
    dims = sh.run([dev(W) for W in Ws], hp)
    torch.cuda.synchronize()
    got = sh.losses.cpu().numpy().reshape(3, 2)
    H = oracle.hessian(X)
    for l, W in enumerate(Ws):
        ref = oracle.search(W, X, bits, group, H=H)
        assert got[l] == pytest.approx(ref["losses"], rel=LOSS_RTOL)
        if abs(ref["losses"][0] - ref["losses"][1]) / min(ref["losses"]) > 0.01:
            assert dims[l] == ref["best"]
        single = S.LayerSearch(ctx, out_f, in_f, bits, group)
        single.run(dev(W), hp)
        torch.cuda.synchronize()
        assert single.losses.cpu().numpy() == pytest.approx(got[l], rel=1e-5)   # same kernels, other chunking
        _check_winner(sh.scales[l], sh.zeros[l], sh.packed[l], W, dims[l], bits, group)


@pytest.mark.parametrize("tokens,in_f", [(300, 512), (2500, 264), (77, 1288), (5000, 2080), (9000, 4096), (1, 64),
                                         (0, 256), (130, 6144), (64, 6008), (50, 6016)])
def test_hessian_prepared_equals_the_two_calls(ctx, tokens, in_f):
    """adadim_hessian_prepared against adadim_hessian + adadim_hessian_prepare: H, hmeta and Hs bit for bit (both
    tile widths, one and several token splits, both scoring layouts, ragged last tiles)."""
    X = synth.make_activations(max(tokens, 1), in_f, seed=tokens + in_f, n_outliers=min(4, in_f), scale_lo=50,
                               scale_hi=100)[:tokens]
    Xd = dev(X) if tokens else torch.empty((0, in_f), dtype=torch.float16, device="cuda")
    outs = []
    for fused in (False, True):
        H = torch.full((in_f, in_f), float("nan"), dtype=torch.float32, device="cuda")
        Hs = ctx.alloc_score(in_f, in_f).fill_(float("nan"))
        hmeta = torch.full((2, in_f), float("nan"), dtype=torch.float32, device="cuda")
        if fused:
            ctx.adadim_hessian_prepared(Xd, H, Hs, hmeta, tokens=tokens)
        else:
            ctx.adadim_hessian(Xd, H, tokens=tokens)
            ctx.adadim_hessian_prepare(H, Hs, hmeta)
        torch.cuda.synchronize()
        outs.append((H.cpu().numpy(), hmeta.cpu().numpy(), B.from_score_layout(Hs.cpu().numpy(), in_f, in_f)))
    (H0, m0, s0), (H1, m1, s1) = outs
    assert np.array_equal(H0.view(np.uint32), H1.view(np.uint32))
    assert np.array_equal(m0.view(np.uint32), m1.view(np.uint32))
    assert np.array_equal(s0.view(np.uint16), s1.view(np.uint16))
    if tokens:
        check_hessian(H1, oracle.hessian(X))
        assert not np.triu(s1.astype(np.float32)).any()          # zero on and above the diagonal


def test_layer_error_batch_select(ctx):
    """The scoring call that also selects: same losses as adadim_layer_error_batch, same index as adadim_select,
    over several calls in a row (its tickets must be back at zero each time), ties and NaN included."""
    out_f, in_f = 512, 520
    X = synth.make_activations(300, in_f, seed=5, n_outliers=3, scale_lo=50, scale_hi=100)
    H = dev(oracle.hessian(X).astype(np.float32))
    Hs = ctx.alloc_score(in_f, in_f)
    hmeta = torch.empty((2, in_f), dtype=torch.float32, device="cuda")
    ctx.adadim_hessian_prepare(H, Hs, hmeta)
    rng = np.random.default_rng(0)
    for n, twin in ((2, None), (5, (1, 3)), (8, (0, 7)), (3, None), (11, (9, 10)), (17, (2, 16))):   # > 8: several batches
        dWs = [(rng.standard_normal((out_f, in_f)) * 1e-3 * (1 + (c * 7) % n)).astype(np.float32) for c in range(n)]
        if twin:
            dWs[twin[1]] = dWs[twin[0]].copy()                    # a tie: the first one wins
        if n == 3:
            dWs[0][7, 9] = np.nan                                 # a NaN loss never wins
        dev_dWs = [dev(d) for d in dWs]
        ref_losses = torch.empty(n, dtype=torch.float32, device="cuda")
        ctx.adadim_layer_error_batch(dev_dWs, B.DW_F32, Hs, hmeta, ref_losses)
        ref_best = ctx.adadim_select(ref_losses)
        losses = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
        best = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        ctx.adadim_layer_error_batch_select(dev_dWs, B.DW_F32, Hs, hmeta, losses, best)
        torch.cuda.synchronize()
        assert torch.equal(losses.cpu().nan_to_num(nan=-1.0), ref_losses.cpu().nan_to_num(nan=-1.0))
        assert int(best.item()) == ref_best
        if n != 3:                                                # the oracle's argmin is not defined for NaN
            assert ref_best == oracle.select(ref_losses.cpu().numpy().astype(np.float64).tolist())
        else:
            assert ref_best == 1


@pytest.mark.parametrize("out_f,in_f,bits,group,meta16", [
    (512, 512, 3, 64, False),       # one launch
    (384, 640, 4, 128, False),      # one launch, ragged row tiles of the scoring layout
    (256, 1024, 2, 32, True),       # one launch, group words
    (768, 768, 4, 128, True),
    (640, 264, 3, 8, False),        # in % 32 != 0: two launches
    (512, 768, 5, 256, False),      # groups of 256, 5 bits: two launches
    (256, 512, 4, 0, False),        # whole channels: two launches
])
def test_quantize_both_equals_the_two_calls(ctx, out_f, in_f, bits, group, meta16):
    """adadim_quantize_both against adadim_quantize(OC) + adadim_quantize(IC) (or the _meta16 pair), every output
    bit for bit, and against the oracle."""
    W = rand_w(out_f, in_f, seed=out_f + 3 * in_f + bits)
    Wd = dev(W)
    clip = float(np.float32(0.9))
    cs = np.ldexp(np.float32(1.0), np.random.default_rng(1).integers(-2, 9, size=in_f)).astype(np.float32)
    csd = dev(cs)
    def bufs(dim):
        g = (in_f if dim == OC else out_f) if group == 0 else group
        shape = (out_f, in_f // g) if dim == OC else (out_f // g, in_f)
        n_ch, ln = (out_f, in_f) if dim == OC else (in_f, out_f)
        d = {"codes": torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda"),
             "dW": ctx.alloc_score(out_f, in_f).fill_(float("nan")),
             "packed": torch.full((n_ch, (ln * bits + 31) // 32), -1, dtype=torch.int32, device="cuda")}
        if meta16:
            d["meta"] = torch.full(shape, -1, dtype=torch.int16, device="cuda")
        else:
            d["scales"] = torch.full(shape, -1.0, dtype=torch.float32, device="cuda")
            d["zeros"] = torch.full(shape, 255, dtype=torch.uint8, device="cuda")
        return d
    one = {OC: bufs(OC), IC: bufs(IC)}
    two = {OC: bufs(OC), IC: bufs(IC)}
    ctx.adadim_quantize_both(Wd, bits, group, csd, one[OC], one[IC], clip=clip, meta16=meta16)
    for dim in (OC, IC):
        if meta16:
            ctx.adadim_quantize_meta16(Wd, dim, bits, group, clip, codes=two[dim]["codes"], meta=two[dim]["meta"],
                                       dW=two[dim]["dW"], dW_dtype=B.DW_F16_SCALED, colscale=csd, packed=two[dim]["packed"])
        else:
            ctx.adadim_quantize(Wd, dim, bits, group, clip, codes=two[dim]["codes"], scales=two[dim]["scales"],
                                zeros=two[dim]["zeros"], dW=two[dim]["dW"], dW_dtype=B.DW_F16_SCALED, colscale=csd,
                                packed=two[dim]["packed"])
    torch.cuda.synchronize()
    for dim in (OC, IC):
        for k in one[dim]:
            a, b = one[dim][k].cpu().numpy(), two[dim][k].cpu().numpy()
            if k == "dW":
                a, b = B.from_score_layout(a, out_f, in_f).view(np.uint16), B.from_score_layout(b, out_f, in_f).view(np.uint16)
            assert np.array_equal(a, b), (dim, k)
        ref = (oracle.meta16_oracle.quantize if meta16 else oracle.quantize)(W, dim, bits, group, clip)
        assert np.array_equal(one[dim]["codes"].cpu().numpy(), ref["codes"])
        assert np.array_equal(B.from_score_layout(one[dim]["dW"].cpu().numpy(), out_f, in_f),
                              (ref["dW"] * cs[None, :]).astype(np.float16))


def test_profile_only_one_kernel(ctx):
    """adadim_profile_only: with a name set only that kernel is bracketed; cleared, every kernel again."""
    out_f, in_f = 256, 512
    W = synth.make_weight(out_f, in_f, 3, heavy_cols=4, heavy_scale=5.0)
    X = synth.make_activations(1024, in_f, 4, n_outliers=2, scale_lo=30, scale_hi=60)
    hp = S.PreparedHessian(ctx, in_f)
    ls = S.LayerSearch(ctx, out_f, in_f, 3, 64)
    Wd, Xd = dev(W), dev(X)

    def step():
        hp.update_prepared(Xd)
        ls.run(Wd, hp)

    ctx.adadim_profile_only("gram_tiles")
    ctx.adadim_profile(True)
    step(); step()
    ctx.adadim_profile(False)
    rec = ctx.adadim_profile_read()
    assert list(rec) == ["gram_tiles"] and rec["gram_tiles"][1] == 2 and rec["gram_tiles"][0] > 0
    total, n, lo, mid, hi = ctx.adadim_profile_read(spread=True)["gram_tiles"]
    assert n == 2 and 0 < lo <= mid <= hi                     # two launches: the median is their mean
    assert lo + hi == pytest.approx(total, rel=1e-5) and mid == pytest.approx(total / 2, rel=1e-5)
    ctx.adadim_profile_only(None)
    ctx.adadim_profile(True)
    step()
    ctx.adadim_profile(False)
    rec = ctx.adadim_profile_read()
    assert "gram_tiles" in rec and "error_tiles" in rec and len(rec) >= 4


@pytest.mark.parametrize("log2_scale", [-5, 0, 7])
def test_search_losses_over_the_activation_range(ctx, log2_scale):
    """The scoring operands are fp16 after the power-of-two column scaling (dW * d, d ~ sqrt(H_jj) / 64), so the loss
    is accurate while |dW| sqrt(H_jj) / 64 stays inside fp16's normal range (the header of adadim_hessian_prepare
    states the range).  Activations 2^-5 and 2^7 times the usual size (the largest the outlier channels leave room
    for in fp16) are inside it at this token count: both losses to 1e-3 of the fp64 oracle, as at the usual size,
    through the calls the search makes."""
    out_f, in_f, tokens, bits, group = 512, 768, 4096, 3, 128
    W = rand_w(out_f, in_f, seed=77)
    X = synth.make_activations(tokens, in_f, seed=78, n_outliers=4, scale_lo=50, scale_hi=100)
    X = (X.astype(np.float32) * np.float32(2.0 ** log2_scale)).astype(np.float16)      # exact: a power of two, no overflow
    assert np.isfinite(X).all()
    H64 = oracle.hessian(X)
    hp = S.PreparedHessian(ctx, in_f).update_prepared(dev(X))
    ls = S.LayerSearch(ctx, out_f, in_f, bits, group)
    ls.launch(dev(W), hp)
    best, dim, _ = ls.result()
    got = ls.losses.cpu().numpy().astype(np.float64)
    ref = [oracle.layer_error(oracle.quantize(W, dm, bits, group)["dW"], H64) for dm in (OC, IC)]
    assert np.isfinite(got).all()
    assert got == pytest.approx(ref, rel=LOSS_RTOL)
    if abs(ref[0] - ref[1]) / min(ref) > 0.01:
        assert best == oracle.select(ref)


def test_search_with_outlier_channels_at_fp16_max(ctx):
    """Three activation channels at +-60000 in every token (fp16 holds nothing larger) beside ordinary ones: with
    weights of ordinary size the scoring operands stay finite, and both losses agree with the fp64 oracle."""
    out_f, in_f, tokens, bits, group = 384, 640, 8192, 4, 128
    W = rand_w(out_f, in_f, seed=91)
    X = synth.make_activations(tokens, in_f, seed=92, n_outliers=0, scale_lo=1, scale_hi=1)
    sign = np.sign(X[:, [5, 300, 639]].astype(np.float32))
    sign[sign == 0] = 1
    X[:, [5, 300, 639]] = (sign * 60000.0).astype(np.float16)
    assert np.isfinite(X).all()
    H64 = oracle.hessian(X)
    hp = S.PreparedHessian(ctx, in_f).update_prepared(dev(X))
    ls = S.LayerSearch(ctx, out_f, in_f, bits, group)
    ls.launch(dev(W), hp)
    best, dim, _ = ls.result()
    got = ls.losses.cpu().numpy().astype(np.float64)
    ref = [oracle.layer_error(oracle.quantize(W, dm, bits, group)["dW"], H64) for dm in (OC, IC)]
    assert np.isfinite(got).all()
    assert got == pytest.approx(ref, rel=LOSS_RTOL)
    if abs(ref[0] - ref[1]) / min(ref) > 0.01:
        assert best == oracle.select(ref)


@pytest.mark.gpu
def test_matrix_core_probes_report_a_rate_below_the_published_peaks(ctx):
    """The two measurement aids run, wait for the stream and return a rate and a clock that make sense for this
    chip: above a tenth of the published dense peaks (fp16 2.5 PFLOP/s, fp64 78.6 TFLOP/s) and not above them."""
    tf16, mhz16 = ctx.adadim_probe_mfma(True, 500)
    tf64, mhz64 = ctx.adadim_probe_mfma_f64(2000)
    assert 250.0 < tf16 <= 2500.0 and 7.8 < tf64 <= 78.6
    assert 500.0 < mhz16 < 3000.0 and 500.0 < mhz64 < 3000.0
    with pytest.raises(B.AdaDimError):
        ctx.adadim_probe_mfma_f64(0)
    # the matrix-vector product's read pattern by itself: runs on a stream of any bit pattern, every width
    for bits in (2, 3, 4):
        out_f, in_f = 4096, 520
        packed = torch.randint(-2 ** 31, 2 ** 31 - 1, (in_f, out_f * bits // 32), dtype=torch.int32, device="cuda")
        assert 0.0 < ctx.adadim_probe_gemv_read(packed, out_f, in_f, bits) < 1e5
    with pytest.raises(B.AdaDimError):
        ctx.adadim_probe_gemv_read(packed, 4096 + 8, 520, 4)


def test_gram_timeline_probe_stamps_every_piece(ctx):
    """The time-stamped launch of the Gram tile kernel (a measurement aid): one record per piece of the plan, each with
    a list, an XCD, a start before its end, and a prologue and main loop that fit inside it; the pieces of a list
    that share a tile's token range order themselves by list; H = X^T X computed afterwards is unharmed by the stamps
    the probe left in the scratch buffer."""
    tokens, in_f = 6000, 2048
    X = synth.make_activations(tokens, in_f, seed=5, n_outliers=3, scale_lo=20, scale_hi=40)
    Xd = dev(X)
    for dispatcher in (False, True):
        rec, plan = ctx.adadim_probe_gram_timeline(Xd, dispatcher=dispatcher)
        n_tiles = (in_f // 256) * (in_f // 256 + 1) // 2
        assert plan[0] == n_tiles and plan[1] >= 0 and plan[7] >= 1
        assert len(rec) >= n_tiles                                # at least one piece per tile
        assert set(np.unique(rec[:, 0])) <= {0.0, 1.0, 2.0} and rec[:, 1].min() >= 0 and rec[:, 1].max() <= 7
        assert (rec[:, 2] >= 0).all() and (rec[:, 3] > rec[:, 2]).all() and rec[:, 2].min() == 0.0
        assert (rec[:, 5] + rec[:, 6] <= rec[:, 3] - rec[:, 2] + 0.05).all()
        assert (rec[:, 4] > 0).all()
    check_hessian(gpu_hessian(ctx, X), oracle.hessian(X))
    with pytest.raises(B.AdaDimError):
        ctx.adadim_probe_gram_timeline(dev(X[:, :1024].copy()))  # the 128-wide kernel's widths carry no stamps
