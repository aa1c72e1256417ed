"""The scoring entry point that allocates nothing (adadim_layer_error_batch_select_noalloc) against the
entry point it is a variant of (adadim_layer_error_batch_select), through the C ABI: two calls in a row on
one context, the second on a smaller layer, so that the second call finds the first call's contents in the
fixed scratch array.  Same kernels and launch shape, so losses, row losses and the winner are compared
bit for bit (the bar of the existing entry point against the oracle is 1e-3 relative; it is checked too,
on the oracle's fp64 losses, for the first layer)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from oracle import OC, IC
from paper_2309_15531_amd import binding as B
from paper_2309_15531_amd import synth

pytestmark = pytest.mark.gpu


def _layer(ctx, out_f, in_f, tokens, bits, group, seed):
    W = synth.make_weight(out_f, in_f, seed, 0.01, 5.0)
    X = synth.make_activations(tokens, in_f, seed + 1, 4, 50.0, 100.0)
    Wd, Xd = torch.from_numpy(W).cuda(), torch.from_numpy(X).cuda()
    H = torch.empty((in_f, in_f), dtype=torch.float32, device="cuda")
    Hs = ctx.alloc_score(in_f, in_f)
    hmeta = torch.empty((2, in_f), dtype=torch.float32, device="cuda")
    ctx.adadim_hessian_prepared(Xd, H, Hs, hmeta)
    dWs = [ctx.alloc_score(out_f, in_f) for _ in range(2)]
    ctx.adadim_quantize_both(Wd, bits, group, hmeta[0], {"dW": dWs[0]}, {"dW": dWs[1]})
    return W, X, dWs, Hs, hmeta


def _both_ways(ctx, lib, out_f, in_f, dWs, Hs, hmeta):
    n = len(dWs)
    res = []
    arr = (ctypes.c_void_p * n)(*[t.data_ptr() for t in dWs])
    for noalloc in (False, True):
        losses = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
        rows = torch.full((n, out_f), -1.0, dtype=torch.float32, device="cuda")
        best = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        if noalloc:
            rc = lib.adadim_layer_error_batch_select_noalloc(ctx._h, n, arr, out_f, in_f, Hs.data_ptr(), hmeta.data_ptr(),
                                                             rows.data_ptr(), losses.data_ptr(), best.data_ptr())
        else:
            rc = lib.adadim_layer_error_batch_select(ctx._h, n, arr, B.DW_F16_SCALED, out_f, in_f, Hs.data_ptr(),
                                                     hmeta.data_ptr(), rows.data_ptr(), losses.data_ptr(), best.data_ptr())
        assert rc == B.OK, ctx.last_error()
        torch.cuda.synchronize()
        res.append((losses.cpu().numpy(), rows.cpu().numpy(), int(best.item())))
    return res


def test_noalloc_matches_allocating_entry_point_twice():
    lib = B.load_library()
    ctx = B.Context()
    try:
        # first call: 3 x 2 row blocks, ragged 640-wide contraction (2.5 column blocks)
        shapes = [(768, 640, 1536, 3, 128, 11), (256, 384, 512, 4, 64, 23)]
        for k, (out_f, in_f, tokens, bits, group, seed) in enumerate(shapes):
            print("case", k, out_f, in_f, tokens, bits, group, seed, flush=True)
            W, X, dWs, Hs, hmeta = _layer(ctx, out_f, in_f, tokens, bits, group, seed)
            assert 0 < lib.adadim_noalloc_scratch_bytes(2, out_f, in_f) <= 16 << 20
            (l0, r0, b0), (l1, r1, b1) = _both_ways(ctx, lib, out_f, in_f, dWs, Hs, hmeta)
            assert np.array_equal(l0, l1) and np.array_equal(r0, r1) and b0 == b1
            assert (l1 > 0).all() and b1 in (0, 1)
            if k == 0:
                H64 = oracle.hessian(X)
                ref = [oracle.layer_error(oracle.quantize(W, dm, bits, group)["dW"], H64) for dm in (OC, IC)]
                assert l1 == pytest.approx(ref, rel=1e-3)
                if abs(ref[0] - ref[1]) / min(ref) > 0.01:
                    assert b1 == oracle.select(ref)
    finally:
        torch.cuda.synchronize()
        ctx.close()


def test_noalloc_rejects_sizes_beyond_the_array():
    lib = B.load_library()
    ctx = B.Context()
    try:
        out_f, in_f = 8192, 28672          # 8 candidates: 8 * 112 * 8192 * 4 bytes of row partials
        assert lib.adadim_noalloc_scratch_bytes(8, out_f, in_f) > 16 << 20
        dummy = torch.zeros(64, dtype=torch.float32, device="cuda")     # never read: the call is rejected first
        arr = (ctypes.c_void_p * 8)(*[dummy.data_ptr()] * 8)
        rc = lib.adadim_layer_error_batch_select_noalloc(ctx._h, 8, arr, out_f, in_f, dummy.data_ptr(), dummy.data_ptr(),
                                                         None, dummy.data_ptr(), dummy.data_ptr())
        assert rc == B.EINVAL and "scratch" in ctx.last_error()
    finally:
        ctx.close()
