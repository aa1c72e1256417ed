"""GPU test of the recorded step (adadim_capture_begin / _end / adadim_graph_launch): every replay of the graph,
with new weights and activations in the recorded buffers and the program's own eager work and synchronisations
between the replays, must give what the same calls give when launched one by one, and the first must agree with
the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_15531_amd import binding as B
from paper_2309_15531_amd import search as S
from paper_2309_15531_amd import synth

pytestmark = pytest.mark.gpu


def _inputs(seed, out_f, in_f, tokens):
    W = synth.make_weight(out_f, in_f, seed, heavy_cols=max(1, in_f // 100), heavy_scale=5.0)
    X = synth.make_activations(tokens, in_f, seed=seed + 1, n_outliers=4, scale_lo=50, scale_hi=100)
    return W, X


@pytest.mark.parametrize("meta16", [False, True])
def test_graph_replays_match_eager(meta16):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    out_f, in_f, tokens, bits, group = 768, 1024, 1500, 4, 128
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = B.Context()                                   # bound to `side`: a stream that can be recorded
        eager_ctx = B.Context()
        Wd = torch.empty((out_f, in_f), dtype=torch.float16, device="cuda")
        Xd = torch.empty((tokens, in_f), dtype=torch.float16, device="cuda")
        hp, ls = S.PreparedHessian(ctx, in_f), S.LayerSearch(ctx, out_f, in_f, bits, group, meta16=meta16)
        hp2, ls2 = S.PreparedHessian(eager_ctx, in_f), S.LayerSearch(eager_ctx, out_f, in_f, bits, group, meta16=meta16)
        W, X = _inputs(0, out_f, in_f, tokens)
        Wd.copy_(torch.from_numpy(W)); Xd.copy_(torch.from_numpy(X))
        torch.cuda.synchronize()
        gs = S.GraphedSearch(ctx, ls, hp, Wd, Xd)
        for rep in range(4):
            W, X = _inputs(10 * rep, out_f, in_f, tokens)
            Wd.copy_(torch.from_numpy(W)); Xd.copy_(torch.from_numpy(X))
            # eager work of the program's own between the replays, and a synchronisation
            hp2.update(Xd).prepare()
            best2, dim2, _ = ls2.run(Wd, hp2)
            torch.cuda.synchronize()
            ls.losses.fill_(float("nan")); ls.best.fill_(-1)
            best, dim, _ = gs.run()
            assert (best, dim) == (best2, dim2)
            assert torch.equal(ls.losses, ls2.losses)
            assert torch.equal(hp.H, hp2.H) and torch.equal(hp.Hs, hp2.Hs)
            assert torch.equal(ls.packed, ls2.packed)
            if meta16:
                assert torch.equal(ls.meta, ls2.meta)
            else:
                assert torch.equal(ls.scales, ls2.scales) and torch.equal(ls.zeros, ls2.zeros)
            if rep == 0:
                quant = oracle.meta16_oracle.quantize if meta16 else oracle.quantize
                H = oracle.hessian(X)
                ref = [oracle.layer_error(quant(W, d, bits, group)["dW"], H) for d in (oracle.OC, oracle.IC)]
                assert ls.losses.cpu().numpy() == pytest.approx(ref, rel=1e-3)
        gs.close()
        torch.cuda.synchronize()
        ctx.close(); eager_ctx.close()


def test_capture_refuses_what_it_cannot_record():
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = B.Context()
        X = torch.zeros((64, 256), dtype=torch.float16, device="cuda")
        H = torch.empty((256, 256), dtype=torch.float32, device="cuda")
        losses = torch.zeros(2, device="cuda")
        X2 = torch.zeros((64, 4096), dtype=torch.float16, device="cuda")
        H2 = torch.empty((4096, 4096), dtype=torch.float32, device="cuda")
        ctx.adadim_hessian(X, H)                             # sizes the scratch for this shape
        torch.cuda.synchronize()
        ctx.adadim_capture_begin()                           # from here to capture_end: library calls only
        with pytest.raises(B.AdaDimError):                    # already recording
            ctx.adadim_capture_begin()
        with pytest.raises(B.AdaDimError):                    # host output needs a synchronisation
            ctx.adadim_select(losses, to_host=True)
        with pytest.raises(B.AdaDimError) as e:               # larger scratch than the warm-up call sized
            ctx.adadim_hessian(X2, H2)
        assert "recorded" in str(e.value)
        ctx.adadim_hessian(X, H)                             # the recorded call
        g = ctx.adadim_capture_end()
        H.fill_(-1.0)
        ctx.adadim_graph_launch(g)
        torch.cuda.synchronize()
        assert not H.any()                                    # X = 0 gives H = 0
        ctx.adadim_graph_destroy(g)
        ctx.close()
