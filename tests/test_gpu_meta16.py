"""GPU parity of the b + 16/g storage format (adadim_quantize_meta16, adadim_gemv_ic_meta16) against the CPU oracle.

Bar: group words, codes, packed stream and fp32 dW bit-exact; the matrix-vector product within the
bound stated in test_gpu_gemv.py; the search's losses within 1e-3 relative.
"""
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


def gpu_quantize(ctx, W, dim, bits, group, clip=1.0, dW_dtype=B.DW_F32, colscale=None, want_codes=True):
    out_f, in_f = W.shape
    g = (in_f if dim == OC else out_f) if group == 0 else group
    shape = (out_f, in_f // g) if dim == OC else (out_f // g, in_f)
    codes = torch.full((out_f, in_f), 255, dtype=torch.uint8, device="cuda") if want_codes else None
    meta = torch.full(shape, -1, dtype=torch.int16, device="cuda")
    if dW_dtype == B.DW_F16_SCALED:
        dW = ctx.alloc_score(out_f, in_f).fill_(float("nan"))
    else:
        dW = torch.full((out_f, in_f), float("nan"), dtype=torch.float32 if dW_dtype == B.DW_F32 else torch.float16,
                        device="cuda")
    n_ch, ln = (out_f, in_f) if dim == OC else (in_f, out_f)
    packed = torch.full((n_ch, (ln * bits + 31) // 32), -1, dtype=torch.int32, device="cuda")
    ctx.adadim_quantize_meta16(dev(W), dim, bits, group, clip, codes=codes, meta=meta, dW=dW, dW_dtype=dW_dtype,
                               colscale=colscale, packed=packed)
    torch.cuda.synchronize()
    return {"codes": codes.cpu().numpy() if want_codes else None, "meta": meta.cpu().numpy().view(np.uint16),
            "dW": dW.cpu().numpy(), "packed": packed.cpu().numpy().view(np.uint32)}


def rand_w(out_f, in_f, seed):
    return synth.make_weight(out_f, in_f, seed, heavy_cols=max(1, in_f // 100), heavy_scale=5.0)


CASES = [
    # out, in, bits, group: every quantizer kernel path, ragged tiles
    (512, 512, 3, 64),
    (384, 640, 4, 128),
    (256, 1024, 2, 64),
    (640, 264, 3, 8),
    (520, 328, 4, 0),
    (96, 1536, 4, 512),
    (768, 768, 3, 256),
    (240, 72, 3, 24),
    (100, 70, 4, 10),
    (64, 4096, 2, 32),
    (1024, 256, 4, 1024),
]


@pytest.mark.parametrize("dim", [OC, IC])
@pytest.mark.parametrize("out_f,in_f,bits,group", CASES)
def test_quantize_meta16_bit_exact(ctx, dim, out_f, in_f, bits, group):
    axis = in_f if dim == OC else out_f
    if group and axis % group:
        pytest.skip("group does not divide this axis")
    W = rand_w(out_f, in_f, seed=out_f * 5 + in_f + bits)
    ref = m16.quantize(W, dim, bits, group)
    got = gpu_quantize(ctx, W, dim, bits, group)
    assert np.array_equal(got["meta"], ref["meta"])
    assert np.array_equal(got["codes"], ref["codes"])
    assert np.array_equal(got["dW"], ref["dW"])
    assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, bits))


@pytest.mark.parametrize("dim", [OC, IC])
def test_quantize_meta16_clip_scaled_and_degenerate(ctx, dim):
    W = rand_w(256, 512, seed=9)
    W[:64, :128] = 0                                              # all-zero groups: scale 1
    W[64:128, 128:256] = np.float16(6e-8)                         # range/qmax below fp16: the smallest pattern
    W[128:192, 256:384] = (np.random.default_rng(1).standard_normal((64, 128)) * 2e-5).astype(np.float16)   # fp16-subnormal scales
    W[200, 300] = np.float16(65504.0)
    W[201, 300] = np.float16(-65504.0)                            # the largest range
    clip = float(np.float32(0.83))
    for bits in (2, 3, 4):
        ref = m16.quantize(W, dim, bits, 64, clip)
        got = gpu_quantize(ctx, W, dim, bits, 64, clip)
        assert np.array_equal(got["meta"], ref["meta"])
        assert np.array_equal(got["codes"], ref["codes"])
        assert np.array_equal(got["dW"], ref["dW"])
    cs = np.ldexp(np.float32(1.0), np.random.default_rng(3).integers(-2, 9, size=512)).astype(np.float32)
    ref = m16.quantize(W, dim, 4, 64, clip)
    got = gpu_quantize(ctx, W, dim, 4, 64, clip, dW_dtype=B.DW_F16_SCALED, colscale=dev(cs), want_codes=False)
    assert np.array_equal(got["meta"], ref["meta"])
    want = (ref["dW"] * cs[None, :]).astype(np.float32)
    have = B.from_score_layout(got["dW"], 256, 512).astype(np.float32)
    with np.errstate(over="ignore"):                              # the 65504 group times its column factor leaves fp16
        want16 = want.astype(np.float16)
    finite = np.isfinite(want16)
    assert np.array_equal(have[finite], want16.astype(np.float32)[finite])
    assert np.array_equal(got["packed"], oracle.pack(ref["codes"], dim, 4))


def test_plain_quantizer_unchanged_by_the_format_flag(ctx):
    """adadim_quantize after an adadim_quantize_meta16 call still writes fp32 scales (no state carried over)."""
    W = rand_w(256, 256, seed=4)
    gpu_quantize(ctx, W, IC, 4, 64)
    scales = torch.empty((4, 256), dtype=torch.float32, device="cuda")
    zeros = torch.empty((4, 256), dtype=torch.uint8, device="cuda")
    ctx.adadim_quantize(dev(W), IC, 4, 64, 1.0, scales=scales, zeros=zeros)
    torch.cuda.synchronize()
    ref = oracle.quantize(W, IC, 4, 64)
    assert np.array_equal(scales.cpu().numpy(), ref["scales"]) and np.array_equal(zeros.cpu().numpy(), ref["zeros"])


def run_gemv(ctx, packed, meta, x, out_f, in_f, bits, group):
    y = torch.full((out_f,), float("nan"), dtype=torch.float16, device="cuda")
    ctx.adadim_gemv_ic_meta16(dev(packed.view(np.int32)), dev(meta.view(np.int16)), dev(x), out_f, in_f, bits, group, y)
    torch.cuda.synchronize()
    return y.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("out_f,in_f,bits,group", [
    (2048, 256, 4, 128),
    (2560, 520, 3, 128),        # ragged output tile and ragged column chunk
    (4096, 1028, 2, 64),
    (1536, 772, 3, 512),
    (640, 64, 4, 0),
    (96, 12, 3, 32),
])
def test_gemv_meta16(ctx, out_f, in_f, bits, group):
    rng = np.random.default_rng(out_f + in_f + bits)
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    W[:, rng.integers(0, in_f, 3)] *= 6
    q = m16.quantize(W, IC, bits, group)
    packed = oracle.pack(q["codes"], IC, bits)
    x = rng.standard_normal(in_f).astype(np.float16)
    y = run_gemv(ctx, packed, q["meta"], x, out_f, in_f, bits, group)
    ref = m16.gemv_ic(packed, q["meta"], x, out_f, bits, group)
    mag = m16.abs_terms(packed, q["meta"], x, out_f, bits, group)
    assert np.isfinite(y).all()
    assert (np.abs(y - ref) <= 2.0 ** -10 * np.abs(ref) + 2e-5 * mag).all(), np.abs(y - ref).max()


def test_gemv_meta16_every_word(ctx):
    """Random group words over the whole range of patterns (fp16-subnormal scales included) and zero-points."""
    rng = np.random.default_rng(11)
    out_f, in_f, group = 256, 64, 32
    for bits in (2, 3, 4):
        pat = rng.integers(1, (0x7C00 >> (bits - 1)) // 8, size=(out_f // group, in_f)).astype(np.uint32)   # scales up to ~2^-2
        pat[0, :8] = np.arange(1, 9)                              # the smallest values of the format
        meta = ((pat << bits) | rng.integers(0, 1 << bits, size=pat.shape).astype(np.uint32)).astype(np.uint16)
        codes = rng.integers(0, 1 << bits, size=(out_f, in_f)).astype(np.uint8)
        packed = oracle.pack(codes, IC, bits)
        x = rng.standard_normal(in_f).astype(np.float16)
        y = run_gemv(ctx, packed, meta, x, out_f, in_f, bits, group)
        ref = m16.gemv_ic(packed, meta, x, out_f, bits, group)
        mag = m16.abs_terms(packed, meta, x, out_f, bits, group)
        assert (np.abs(y - ref) <= 2.0 ** -10 * np.abs(ref) + 2e-5 * mag + 6e-8).all(), (bits, np.abs(y - ref).max())


def test_quantize_then_gemv_on_device(ctx):
    """The two calls chained on the device: quantize per-IC into the format, multiply from it."""
    out_f, in_f, bits, group = 4096, 1024, 4, 128
    W = rand_w(out_f, in_f, seed=21)
    meta = torch.empty((out_f // group, in_f), dtype=torch.int16, device="cuda")
    packed = torch.empty((in_f, out_f * bits // 32), dtype=torch.int32, device="cuda")
    ctx.adadim_quantize_meta16(dev(W), IC, bits, group, 1.0, meta=meta, packed=packed)
    x = np.random.default_rng(2).standard_normal(in_f).astype(np.float16)
    y = torch.empty(out_f, dtype=torch.float16, device="cuda")
    ctx.adadim_gemv_ic_meta16(packed, meta, dev(x), out_f, in_f, bits, group, y)
    torch.cuda.synchronize()
    q = m16.quantize(W, IC, bits, group)
    ref = q["What"].astype(np.float64) @ x.astype(np.float64)     # the quantizer oracle's own de-quantized weight
    mag = m16.abs_terms(oracle.pack(q["codes"], IC, bits), q["meta"], x, out_f, bits, group)
    got = y.cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= 2.0 ** -10 * np.abs(ref) + 2e-5 * mag).all()


@pytest.mark.parametrize("bits,group,clips", [(4, 128, (1.0,)), (3, 64, (1.0, 0.9, 0.8))])
def test_search_in_the_storage_format(ctx, bits, group, clips):
    """The whole search (Sec. 3.3, Eq. 1) with every candidate quantized into the format: losses against the oracle's
    (its quantizer with the rounded scale, its fp64 error through H), winner's words and packed codes bit-exact."""
    from paper_2309_15531_amd import search as S
    out_f, in_f = 768, 1024
    W = rand_w(out_f, in_f, seed=333 + bits)
    X = synth.make_activations(1100, in_f, seed=17, n_outliers=4, scale_lo=50, scale_hi=100)
    H = oracle.hessian(X)
    clips = [float(np.float32(c)) for c in clips]
    cands = [(d, c) for d in (OC, IC) for c in clips]
    ref_q = [m16.quantize(W, d, bits, group, c) for d, c in cands]
    ref_losses = [oracle.layer_error(q["dW"], H) for q in ref_q]
    ref_best = oracle.select(ref_losses)
    hp = S.PreparedHessian(ctx, in_f).update(dev(X)).prepare()
    ls = S.LayerSearch(ctx, out_f, in_f, bits, group, clips, meta16=True)
    best, dim, clip = ls.run(dev(W), hp)
    torch.cuda.synchronize()
    assert ls.losses.cpu().numpy() == pytest.approx(ref_losses, rel=1e-3)
    srt = sorted(ref_losses)
    if (srt[1] - srt[0]) / srt[0] > 0.01:
        assert best == ref_best
    q = ref_q[best]
    assert ls.scales is None and ls.zeros is None
    assert np.array_equal(ls.meta[:q["meta"].size].cpu().numpy().view(np.uint16), q["meta"].ravel())
    pk = oracle.pack(q["codes"], dim, bits)
    assert np.array_equal(ls.packed[:pk.size].cpu().numpy().view(np.uint32), pk.ravel())
