"""GPU parity of the per-IC de-quantizing matrix-vector product (adadim_gemv_ic) against the CPU oracle.

Bar.  The kernel forms y in fp32 and rounds once to fp16, so with an exact fp32 sum the answer would be within
half an fp16 ulp of the oracle's fp64 value.  The fp32 sum is not exact: the kernel reads code k as code + c_k, c_k a
power of two up to 1024 fixed by the code's bit position, accumulates sum_j a_j (code_j + c_k) (a = scale * x) in one
fma chain per wave and column chunk, and takes c_k * sum_j a_j off again (the header of the call says so).  Every
rounding in such a chain is at most 2^-24 of a partial sum whose terms are t_j = a_j (c_k + code_j) (and a_j zero_j
for the zero-point sum), so

    |y - y_ref| <= half_ulp_fp16(y_ref) + min( LIN * mag,  RSS * 2^-24 * sqrt(sum_j (|a_j| (1024 + code_j + zero_j))^2) )

    mag = sum_j |a_j| (code_j + zero_j).

The second form is the random-walk size of the accumulated roundings (independent roundings of partial sums that
themselves grow like the root of the number of terms); it is what keeps the bound near one fp16 ulp on the long
columns of the App. D shape, where the inputs are random streams and mag is 150 |y|.  The first form caps it on
short columns, where there is no averaging.  Constants: the worst case observed over this file's seeded cases is
(|y - y_ref| - half ulp) = 9.1e-6 mag (printed by every case, with the RSS ratio beside it); LIN = 2e-5 is 2.2 times
that, RSS = 128 is at least 4 times the largest ratio seen on the App. D cases.  The worst-case bound of the same chain
(every rounding at its maximum, all of one sign) is (2 L + 4) * 2^-24 * sum_j |a_j| (1024 + qmax) with L the chain
length, hundreds of times larger than either.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import IC
from paper_2309_15531_amd import binding as B

pytestmark = pytest.mark.gpu

LIN, RSS, C_MAX = 2e-5, 128.0, 1024.0


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = B.Context()
    yield c
    torch.cuda.synchronize()
    c.close()


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_gemv(ctx, packed, scales, zeros, x, out_f, in_f, bits, group):
    y = torch.full((out_f,), float("nan"), dtype=torch.float16, device="cuda")
    ctx.adadim_gemv_ic(dev(packed.view(np.int32)), dev(scales), dev(zeros), dev(x), out_f, in_f, bits, group, y)
    torch.cuda.synchronize()
    return y.cpu().numpy().astype(np.float64)


def check(y, packed, scales, zeros, x, out_f, bits, group, rows=None):
    if rows is None:
        ref = oracle.gemv_ic(packed, scales, zeros, x, out_f, bits, group)
        mag = oracle.abs_terms(packed, scales, zeros, x, out_f, bits, group)
        rss = _rss_terms(oracle.gemv_oracle._codes_from_stream(packed, out_f, bits), scales, zeros, x, group)
        got = y
    else:  # sampled outputs: the oracle on the words that hold them
        ref, mag, rss = _oracle_rows(packed, scales, zeros, x, bits, group, rows)
        got = y[rows]
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    half_ulp = 0.5 * np.spacing(np.abs(ref).astype(np.float16)).astype(np.float64)
    excess = np.maximum(err - half_ulp, 0.0)
    fp32_tol = np.minimum(LIN * mag, RSS * 2.0 ** -24 * rss)
    print(f"gemv: max|y-ref| = {err.max():.3e} (max half fp16 ulp {half_ulp.max():.3e}); max (|y-ref| - half ulp) = "
          f"{(excess / mag).max():.3e} mag (LIN {LIN:.1e}) = {(excess / (2.0 ** -24 * rss)).max():.2f} * 2^-24 rss (RSS {RSS:.0f}); "
          f"fp32 allowance / half ulp: max {(fp32_tol / half_ulp).max():.2f}", flush=True)
    assert (err <= half_ulp + fp32_tol).all(), (err.max(), (excess / mag).max(), (excess / (2.0 ** -24 * rss)).max())


def _rss_terms(codes, scales, zeros, x, group):
    """sqrt(sum_j (|scale x| (C_MAX + code + zero))^2) per output, fp64; codes u8 [out, in]."""
    out_f = codes.shape[0]
    g = out_f if group == 0 else group
    sc = np.repeat(np.asarray(scales, dtype=np.float64), g, axis=0)
    zp = np.repeat(np.asarray(zeros).astype(np.float64), g, axis=0)
    t = np.abs(sc * np.asarray(x).astype(np.float64)[None, :]) * (C_MAX + codes.astype(np.float64) + zp)
    return np.sqrt((t * t).sum(axis=1))


def _oracle_rows(packed, scales, zeros, x, bits, group, rows):
    """Oracle on single outputs: each output's code is cut out of the stream into a 1-output layer."""
    ref, mag, rss = np.zeros(len(rows)), np.zeros(len(rows)), np.zeros(len(rows))
    for i, o in enumerate(rows):
        wd, sh = divmod(int(o) * bits, 32)
        v = packed[:, wd].astype(np.uint64) >> np.uint64(sh)
        if sh + bits > 32:
            v = v | (packed[:, wd + 1].astype(np.uint64) << np.uint64(32 - sh))
        code = (v & np.uint64((1 << bits) - 1)).astype(np.uint32)       # [in]
        one = code.reshape(-1, 1)                                          # stream of a 1-output layer, per column
        s1, z1 = scales[o // group][None, :], zeros[o // group][None, :]
        ref[i] = oracle.gemv_ic(one, s1, z1, x, 1, bits, 1)[0]
        mag[i] = oracle.abs_terms(one, s1, z1, x, 1, bits, 1)[0]
        rss[i] = _rss_terms(code.astype(np.uint8)[None, :], s1, z1, x, 1)[0]
    return ref, mag, rss


@pytest.mark.parametrize("out_f,in_f,bits,group", [
    (2048, 256, 4, 128),        # one block tile, one column chunk
    (2560, 520, 3, 128),        # ragged output tile and ragged column chunk
    (4096, 1028, 2, 64),
    (1536, 772, 3, 512),
    (640, 64, 4, 0),            # whole-channel groups
    (96, 12, 3, 32),            # smaller than every tile
])
def test_gemv_quantized_layer(ctx, out_f, in_f, bits, group):
    """A layer quantized by the oracle: realistic codes, scales and zeros."""
    rng = np.random.default_rng(out_f + in_f + bits)
    W = (rng.standard_normal((out_f, in_f)) * 0.02).astype(np.float16)
    W[:, rng.integers(0, in_f, 3)] *= 6
    q = oracle.quantize(W, IC, bits, group)
    packed = oracle.pack(q["codes"], IC, bits)
    x = rng.standard_normal(in_f).astype(np.float16)
    x[rng.integers(0, in_f, 2)] *= 40
    y = run_gemv(ctx, packed, q["scales"], q["zeros"], x, out_f, in_f, bits, group)
    check(y, packed, q["scales"], q["zeros"], x, out_f, bits, group)


def test_gemv_reproducible_and_zero_input(ctx):
    rng = np.random.default_rng(3)
    out_f, in_f, bits, g = 4096, 1024, 4, 128
    packed = rng.integers(0, 2 ** 32, size=(in_f, out_f * bits // 32), dtype=np.uint64).astype(np.uint32)
    scales = rng.uniform(0.005, 0.015, size=(out_f // g, in_f)).astype(np.float32)
    zeros = rng.integers(0, 16, size=(out_f // g, in_f)).astype(np.uint8)
    x = rng.standard_normal(in_f).astype(np.float16)
    y1 = run_gemv(ctx, packed, scales, zeros, x, out_f, in_f, bits, g)
    y2 = run_gemv(ctx, packed, scales, zeros, x, out_f, in_f, bits, g)
    assert np.array_equal(y1, y2)
    assert not run_gemv(ctx, packed, scales, zeros, np.zeros(in_f, np.float16), out_f, in_f, bits, g).any()


@pytest.mark.parametrize("bits,group", [(4, 128), (3, 128), (3, 2048), (2, 128)])
def test_gemv_appendix_shape_sampled(ctx, bits, group):
    """The shape of the paper's latency table (App. D): weight [4m x m], m = 12288, batch 1.
    Inputs are seeded random streams (every bit pattern is a valid code for 2, 3 and 4 bits),
    scales and zeros; 64 sampled outputs are checked against the oracle one by one."""
    m = 12288
    out_f, in_f = 4 * m, m
    rng = np.random.default_rng(100 + bits + group)
    packed = rng.integers(0, 2 ** 32, size=(in_f, out_f * bits // 32), dtype=np.uint64).astype(np.uint32)
    scales = rng.uniform(0.004, 0.02, size=(out_f // group, in_f)).astype(np.float32)
    zeros = rng.integers(0, 2 ** bits, size=(out_f // group, in_f)).astype(np.uint8)
    x = rng.standard_normal(in_f).astype(np.float16)
    y = run_gemv(ctx, packed, scales, zeros, x, out_f, in_f, bits, group)
    rows = np.sort(rng.choice(out_f, 64, replace=False))
    rows[0], rows[-1] = 0, out_f - 1
    check(y, packed, scales, zeros, x, out_f, bits, group, rows=rows)
