#!/usr/bin/env python3
"""Benchmark of the AdaDim layer search on one MI355X.

A step is one pass of the whole hot path over one layer: Gram matrix of the
calibration activations, its preparation, quantize + score for both grouping
dimensions, selection, and the winner's packed codes / scales / zeros.
Prints ONE JSON line: metric, value, unit, ms_per_step, config, and the roofline / cpu_baseline objects.

    python bench.py [--steps K] [--warmup W]
                    [--workload down_proj|gate_proj|q_proj|qkv|clip_grid|toy|block7b|stream13b|block70b|gemv_ic|gptq|mfma_ceiling|gram_timeline]
                    [--bits B] [--group G] [--meta16]

The default workload is the layer the targets are stated on: W[4096, 11008] (the FFN down projection of the
LLaMA-7B-shaped block) with 65536 calibration tokens.  block7b / block70b run a whole decoder block (every layer,
every precision of the workload, one Gram matrix per input width); stream13b streams blocks of the 40-block
13B-shaped model, weights regenerated per block, results appended to a JSON-lines file.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # B/s, MI355X HBM3E
MFMA_F16_PEAK = 2.5e15     # flop/s, dense fp16 with fp32 accumulate

WORKLOADS = {
    # name: (config id in synth.CONFIGS, layer name)
    "toy": (0, "fc"),
    "q_proj": (1, "q_proj"),
    "gate_proj": (2, "gate_proj"),
    "down_proj": (2, "down_proj"),     # the workload the targets are stated on: W[4096, 11008], 65536 tokens
    # q, k and v of one decoder block: three layers that share X, one H, one scoring launch
    "qkv": (2, ("q_proj", "k_proj", "v_proj")),
    # the 70B-shaped block's q_proj with the clip-ratio grid: 20 ratios x both dims = 40 candidates per layer
    "clip_grid": (4, "q_proj"),
}


def gram_tiling(in_f: int):
    bt = 128 if in_f <= 1024 else 256
    nb = (in_f + bt - 1) // bt
    return bt, nb * (nb + 1) // 2


def copy_calibration():
    """One plain elementwise kernel that reads 256 MiB and writes 256 MiB (one vectorized_elementwise_kernel dispatch
    with a MulFunctor in a counter file): the dispatch of known size that scales rocprofv3's FETCH_SIZE / WRITE_SIZE."""
    import torch
    src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    torch.mul(src, 2.0, out=dst)
    torch.cuda.synchronize()
    del src, dst


def gram_issued_flops(in_f: int, tokens: int) -> float:
    """MFMA flops the Gram kernel issues: upper-triangular tiles (full diagonal tiles) x 2*BT*BT*tokens."""
    bt, n_tiles = gram_tiling(in_f)
    return 2.0 * n_tiles * bt * bt * tokens


def error_issued_flops(out_f: int, in_f: int) -> float:
    """MFMA flops the error GEMM issues per candidate: 256x256 tiles, column block nb contracts over (nb+1)*256."""
    bn = 256
    nbk, mbk = (in_f + bn - 1) // bn, (out_f + bn - 1) // bn
    return 2.0 * (mbk * bn) * bn * bn * nbk * (nbk + 1) / 2


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` on `workload` from profiles/traffic.txt ("<kernel>/<workload> <bytes>
    <commit the counters were read at>" per line; FETCH_SIZE and WRITE_SIZE of two rocprofv3 --pmc runs of this
    command, scaled by a plain copy's readings): (bytes, commit) or (None, None) when not measured."""
    tpath = os.path.join(ROOT, "profiles", "traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) >= 2 and f[0] == f"{kernel}/{workload}":
                return float(f[1]), (f[2] if len(f) > 2 else None)
    return None, None


def _blas_threads() -> int:
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(layer_list, X_of, tokens, bits_list, group, n_clips=1, budget_flops=5.0e11, quant_budget=48_000_000):
    """Times the CPU oracle, as it stands, on a bounded sample of the workload and scales to the whole of it, twice:
    with the BLAS threads the box gives (`cores`) and single-threaded.

    layer_list: [(W fp16 host array, count)]: one layer per distinct shape and how many layers of that shape (times
    precisions are counted through bits_list); X_of(width, t) -> the first t tokens of that width's activations.
    Sampled: the fp64 Gram matrix on as many tokens as cost `budget_flops`, scaled to `tokens`; the fp64 loss on as
    many output rows as cost `budget_flops`, scaled to all rows (extrapolated); both quantizations of each distinct
    shape on the first whole row groups that hold at most `quant_budget` weights (all rows of the 7B shapes), for the
    first precision (numpy, one thread whatever the setting), scaled to all rows, layers, precisions and clip ratios.  Returns the cpu_baseline object."""
    import oracle
    from threadpoolctl import threadpool_limits
    widths = sorted({W.shape[1] for W, _ in layer_list})
    n_weights = sum(W.size * c for W, c in layer_list)
    t_quant, quant_done = 0.0, {}
    legs = {}
    for label, limit, scale in (("all", None, 1.0), ("single", 1, 1.0 / 8)):
        with threadpool_limits(limits=limit):
            t_h, H = 0.0, {}
            for w in widths:
                t_s = int(max(64, min(tokens, budget_flops * scale / (2.0 * w * w))))
                Xs = X_of(w, t_s)
                t0 = time.perf_counter()
                H[w] = oracle.hessian(Xs)
                t_h += (time.perf_counter() - t0) * tokens / t_s
            t_l = 0.0
            for W, count in layer_list:
                out_f, in_f = W.shape
                g_rows = group if group else out_f
                q_rows = int(min(out_f, max(g_rows, (quant_budget // in_f) // g_rows * g_rows)))
                if label == "all":
                    t0 = time.perf_counter()
                    quant_done[W.shape] = [oracle.quantize(W[:q_rows], dim, bits_list[0], group)["dW"]
                                           for dim in (oracle.OC, oracle.IC)]
                    t_quant += (time.perf_counter() - t0) * (out_f / q_rows) * count * len(bits_list) * n_clips
                rows = int(max(8, min(q_rows, budget_flops * scale / (2.0 * in_f * in_f) / 2)))
                t0 = time.perf_counter()
                losses = [float(oracle.layer_error_rows(dW[:rows], H[in_f]).sum()) for dW in quant_done[W.shape]]
                oracle.select(losses)
                t_l += (time.perf_counter() - t0) * (out_f / rows) * count * len(bits_list) * n_clips
            legs[label] = {"gram_s": t_h, "loss_s": t_l}
    out = {}
    for label in ("all", "single"):
        total = legs[label]["gram_s"] + legs[label]["loss_s"] + t_quant
        out[label] = {"value": n_weights * len(bits_list) / total, "seconds_extrapolated": total,
                      "gram_s": legs[label]["gram_s"], "loss_s": legs[label]["loss_s"], "quantize_s": t_quant}
    cores = _blas_threads()
    return {
        "value": out["all"]["value"], "unit": "weights/s", "cores": int(cores), "kind": "oracle",
        "sample": ("per input width the fp64 Gram matrix on the first tokens worth %.0e flop, scaled to %d tokens; per "
                   "distinct layer shape both quantizations of the first row groups holding up to %d weights (numpy, one "
                   "thread) and both fp64 losses on the first rows worth %.0e flop, scaled to all rows, layers, "
                   "precisions and clip ratios; repeated with one BLAS thread on an eighth of the sample"
                   % (budget_flops, tokens, quant_budget, budget_flops)),
        "seconds_extrapolated": out["all"]["seconds_extrapolated"],
        "parts_s": {k: out["all"][k] for k in ("gram_s", "loss_s", "quantize_s")},
        "single_thread": {"value": out["single"]["value"], "cores": 1,
                          "seconds_extrapolated": out["single"]["seconds_extrapolated"],
                          "parts_s": {k: out["single"][k] for k in ("gram_s", "loss_s", "quantize_s")}},
        "host_cpus": os.cpu_count(),
    }


def gemv_bench(args):
    """The per-IC de-quantizing matrix-vector product on the shape of the paper's latency table
    (App. D): weight [4m x m], m = 12288, batch 1.  One step = one adadim_gemv_ic call."""
    import torch
    from paper_2309_15531_amd import binding as B
    B.load_library()
    m = 12288
    out_f, in_f = 4 * m, m
    bits = 4 if args.bits is None else args.bits
    group = 128 if args.group is None else args.group
    g = torch.Generator(device="cuda").manual_seed(7)
    n_words = out_f * bits // 32
    # seeded random streams (every bit pattern is a valid code), scales and zeros
    # two copies of the weight stream, used alternately, so that the 256 MB Infinity Cache cannot
    # hold what the next call reads (weights of a model that does not fit the cache)
    packs = [torch.randint(-2 ** 31, 2 ** 31 - 1, (in_f, n_words), dtype=torch.int32, device="cuda", generator=g)
             for _ in range(2)]
    scales = torch.empty((out_f // group, in_f), dtype=torch.float32, device="cuda").uniform_(0.004, 0.02, generator=g)
    zeros = torch.randint(0, 2 ** bits, (out_f // group, in_f), dtype=torch.uint8, device="cuda", generator=g)
    x = torch.randn(in_f, dtype=torch.float32, device="cuda", generator=g).half()
    y = torch.empty(out_f, dtype=torch.float16, device="cuda")
    packed = packs[0]
    # the same parameters as 16-bit group words: random patterns of scales in about [0.004, 0.02]
    meta = ((torch.randint(0x1C19 >> (bits - 1), 0x251F >> (bits - 1), (out_f // group, in_f), dtype=torch.int32,
                           device="cuda", generator=g) << bits) | zeros.int()).to(torch.int16)
    ctx = B.Context()

    def call(i):
        if args.meta16:
            ctx.adadim_gemv_ic_meta16(packs[i & 1], meta, x, out_f, in_f, bits, group, y)
        else:
            ctx.adadim_gemv_ic(packs[i & 1], scales, zeros, x, out_f, in_f, bits, group, y)

    for i in range(args.warmup):
        call(i)
    torch.cuda.synchronize()
    # the timed region brackets the dominant kernel only (an event pair costs the stream about 7 us, a tenth of this
    # step); the small second kernel is timed in a pass of its own afterwards
    ctx.adadim_profile_only("gemv_ic_tiles")
    ctx.adadim_profile(True)
    t0 = time.perf_counter()
    for i in range(args.steps):
        call(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ctx.adadim_profile(False)
    kern = {k: v[0] / max(v[1], 1) * 1e3 for k, v in ctx.adadim_profile_read().items()}
    ctx.adadim_profile_only(None)
    ctx.adadim_profile(True)
    for i in range(min(args.steps, 200)):
        call(i)
    torch.cuda.synchronize()
    ctx.adadim_profile(False)
    kern = dict({k: v[0] / max(v[1], 1) * 1e3 for k, v in ctx.adadim_profile_read().items()}, **kern)
    # what reading the code stream in the kernel's pattern costs by itself, the two buffers taken in turn
    for i in range(4):
        ctx.adadim_probe_gemv_read(packs[i & 1], out_f, in_f, bits)
    bare = [ctx.adadim_probe_gemv_read(packs[i & 1], out_f, in_f, bits) for i in range(10)]
    bare_us = float(np.mean(bare))
    alg_bytes = out_f * in_f * bits / 8 + (2.0 if args.meta16 else 5.0) * (out_f // group) * in_f + 2 * in_f + 2 * out_f
    sec = kern["gemv_ic_tiles"] * 1e-6
    result = {
        "metric": "per-IC dequant matrix-vector product, weights/s", "value": out_f * in_f / (elapsed / args.steps),
        "unit": "weights/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"per-IC kernel W[{out_f},{in_f}] int{bits} g{group} x[{in_f}] batch 1 (App. D shape)"
                               + (", 16-bit group words" if args.meta16 else ""),
                   "bits": bits, "group": group},
        "roofline": {"kernel": "gemv_ic_tiles", "bound": "hbm", "achieved": alg_bytes / sec / 1e9, "peak": HBM_PEAK / 1e9,
                     "unit": "GB/s", "frac": alg_bytes / sec / HBM_PEAK, "traffic": None,
                     "bare_read": {"us": bare_us, "frac_hbm": out_f * in_f * bits / 8 / (bare_us * 1e-6) / HBM_PEAK,
                                   "note": "the code words alone, read by the same grid and column ranges with one xor "
                                           "per word (adadim_probe_gemv_read); event-timed launch by launch"}},
        "kernels_us": kern,
    }
    if not args.no_cpu_baseline:
        import oracle
        rows = 4
        pk = packed[:, :max(1, rows * bits // 32 + 1)].cpu().numpy().view(np.uint32)
        t0 = time.perf_counter()
        oracle.gemv_ic(pk[:, :1], scales[:1].cpu().numpy(), zeros[:1].cpu().numpy(), x.cpu().numpy(), 32 // bits if bits != 3 else 10, bits, 0)
        t = time.perf_counter() - t0
        n_o = 32 // bits if bits != 3 else 10
        result["cpu_baseline"] = {"value": n_o * in_f / t, "unit": "weights/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{n_o} outputs x {in_f} inputs"}
    print(json.dumps(result))


def gptq_bench(args):
    """GPTQ-ada on the q_proj workload: H and its preparation are already there; one step = the RTN
    search for the dimension plus GPTQ in that dimension and the scoring of its result; the factor
    of the inverse Hessian (once per distinct input) is timed on its own."""
    import torch
    from paper_2309_15531_amd import binding as B
    from paper_2309_15531_amd import search as S
    from paper_2309_15531_amd import synth
    B.load_library()
    cfg = synth.CONFIGS[1]
    out_f, in_f = cfg["layers"]["q_proj"]
    bits = 3 if args.bits is None else args.bits
    group = cfg["group"] if args.group is None else args.group
    Wd = torch.from_numpy(synth.config_weight(1, "q_proj")).cuda()
    Xd = torch.from_numpy(synth.config_activations(1, in_f)).cuda()
    ctx = B.Context()
    hp = S.PreparedHessian(ctx, in_f).update(Xd).prepare()
    del Xd
    fac = S.GptqFactor(ctx, hp)
    ga = S.GptqAda(ctx, out_f, in_f, bits, group)
    for _ in range(max(1, args.warmup)):
        dim = ga.run(Wd, hp, fac)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fac.update(hp)
    torch.cuda.synchronize()
    t_factor = time.perf_counter() - t0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dim = ga.run(Wd, hp, fac)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # per-kernel durations from a second pass: with the library's events on, the sweep keeps its two streams'
    # work on one stream (so that the events bracket single kernels), which the timed pass above does not
    ctx.adadim_profile(True)
    for _ in range(args.steps):
        ga.run(Wd, hp, fac)
    torch.cuda.synchronize()
    ctx.adadim_profile(False)
    prof = ctx.adadim_profile_read()
    kern = {k: v[0] / max(v[1], 1) * 1e3 for k, v in prof.items()}
    print(json.dumps({
        "metric": "weight params searched + GPTQ-quantized /s", "value": out_f * in_f / (elapsed / args.steps),
        "unit": "weights/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"gptq-ada llama7b-q_proj W[{out_f},{in_f}] int{bits} g{group}", "bits": bits, "group": group},
        "result": {"dim": "oc" if dim == 0 else "ic", "loss_rtn": float(ga.loss_rtn.item()),
                   "loss_gptq": float(ga.loss_gptq.item())},
        "factor_ms": t_factor * 1e3, "kernels_us": kern,
    }))


def block_bench(args):
    """Whole decoder blocks.  block7b: the seven layers of the LLaMA-7B-shaped block, INT4 and INT3, per step two Gram
    matrices (one per input width) and 14 searches; stream13b: blocks of the 40-block 13B-shaped model, weights of
    every layer regenerated on the device per block from seed + layer id, results appended to a JSON-lines file,
    block b + 1 queued while block b's answers travel to the host; block70b: the 70B-shaped GQA block with the
    20-ratio clip grid (40 candidates per layer and precision).  One step = one block.  The activation matrices are
    drawn once per input width and shared by the layers of that width and by every block (each block still forms
    its own Gram matrices from them)."""
    import tempfile

    import torch
    from paper_2309_15531_amd import binding as B
    from paper_2309_15531_amd import search as S
    from paper_2309_15531_amd import stream as ST
    from paper_2309_15531_amd import synth
    B.load_library()
    cfg_id = BLOCK_WORKLOADS[args.workload]
    cfg = synth.CONFIGS[cfg_id]
    layers, tokens = cfg["layers"], cfg["tokens"]
    group = cfg["group"] if args.group is None else args.group
    bits_list = (args.bits,) if args.bits is not None else tuple(cfg["bits"])
    clips = tuple(S.clip_grid(cfg["clips"])) if cfg["clips"] > 1 else (1.0,)
    n_blocks_model = cfg.get("blocks", 1)
    streaming = n_blocks_model > 1
    if streaming and args.warmup + args.steps > n_blocks_model:
        print(f"bench.py: {args.workload} has {n_blocks_model} blocks; --warmup + --steps must not exceed that", file=sys.stderr)
        sys.exit(2)
    widths = sorted({i for _, i in layers.values()})
    Xd = {w: synth.config_activations_device(cfg_id, w) for w in widths}
    block_weights = sum(o * i for o, i in layers.values())
    ctx = B.Context()
    shapes = sorted(set(layers.values()))

    # weights: two buffer sets when they are regenerated per block (block b's are read while block b + 1's are drawn)
    n_sets = 2 if streaming else 1
    bufs = [{n: torch.empty(sh, dtype=torch.float16, device="cuda") for n, sh in layers.items()} for _ in range(n_sets)]
    scratch = {sh: torch.empty(sh, dtype=torch.float32, device="cuda") for sh in shapes}
    for n in layers:
        synth.config_weight_device(cfg_id, n, block=0, out=bufs[0][n], scratch=scratch[layers[n]])

    # A streamed model's next block is drawn on a stream of its own, under the Gram kernels just queued for it on the
    # context's stream (in a real job the block's weights arrive by DMA meanwhile).  The draw may start once the
    # kernels that read this slot's buffers two blocks ago are done: everything queued before the previous draw.
    gen_stream = torch.cuda.Stream() if streaming else None
    queued_before = [None, None]

    def weights_of(b, slot):
        if not streaming:
            return bufs[0]
        main = torch.cuda.current_stream()
        mark = torch.cuda.Event()
        mark.record(main)
        with torch.cuda.stream(gen_stream):
            if queued_before[slot ^ 1] is not None:
                gen_stream.wait_event(queued_before[slot ^ 1])
            for n in layers:
                synth.config_weight_device(cfg_id, n, block=b, out=bufs[slot][n], scratch=scratch[layers[n]])
            drawn = torch.cuda.Event()
            drawn.record(gen_stream)
        queued_before[slot] = mark
        main.wait_event(drawn)
        return bufs[slot]

    if len(clips) == 1:
        bs = ST.BlockSearch(ctx, layers, bits_list, group)
        tmp = None
        if args.log is None:
            tmp = tempfile.NamedTemporaryFile(prefix="adadim_stream_", suffix=".jsonl", delete=False)
            tmp.close()
            log_path = tmp.name
        else:
            log_path = args.log
            if not args.resume and os.path.exists(log_path):
                os.remove(log_path)
        log = ST.ResultsLog(log_path)
        next_block = [max([k[1] for k in log.records] + [-1]) + 1 if args.resume else 0]

        def run(n):
            """Searches the next n blocks (a streamed model: its next blocks; a single block: the same block again
            under a new step number); returns the records written."""
            b0 = next_block[0]
            next_block[0] += n
            return ST.run_stream(bs, log, cfg["seed"], range(b0, b0 + n), weights_of, lambda b: Xd)
    else:
        # clip grid: 2 x 20 candidates per layer and precision, scored in batches of eight; the winner is quantized
        # again once it is known, so every layer waits for its answer
        hps = {w: S.PreparedHessian(ctx, w) for w in widths}
        searches = {(sh, b): S.LayerSearch(ctx, sh[0], sh[1], b, group, clips=clips) for sh in shapes for b in bits_list}
        results = []

        def run(n):
            for _ in range(n):
                for w in widths:
                    hps[w].update_prepared(Xd[w])
                for b in bits_list:
                    for name, sh in layers.items():
                        best, dim, clip = searches[(sh, b)].run(bufs[0][name], hps[sh[1]])
                        results.append({"layer": name, "bits": b, "dim": "ic" if dim == 1 else "oc", "clip": clip})
            return n * len(layers) * len(bits_list)
        log = None

    def profiled(n, only=None):
        ctx.adadim_profile_only(only)
        ctx.adadim_profile(True)
        t_begin = time.perf_counter()
        run(n)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t_begin
        ctx.adadim_profile(False)
        ctx.adadim_profile_only(None)
        return dt, {k: {"total_us": v[0] * 1e3, "launches": v[1], "steps": n} for k, v in ctx.adadim_profile_read().items()}

    run(max(1, args.warmup))
    torch.cuda.synchronize()
    if args.copy_calibration:
        copy_calibration()
    # the timed region brackets the dominant kernel only (see the single-layer path); the others from a second pass
    elapsed, live = profiled(args.steps, only="gram_tiles" if len(clips) == 1 else "error_tiles")
    recs = list(log.records.values()) if log is not None else []
    if streaming and args.log is None:
        # the per-kernel pass re-runs one block of the model; the log would skip a block it holds, so it starts afresh
        log.close()
        os.remove(log_path)
        log = ST.ResultsLog(log_path)
        next_block[0] %= n_blocks_model
    _, kern = profiled(1)
    kern.update(live)

    def per_step(k):
        return kern[k]["total_us"] / kern[k]["steps"] * 1e-6 if k in kern else 0.0

    gram_flops = sum(gram_issued_flops(w, tokens) for w in widths)
    err_flops = sum(error_issued_flops(o, i) for o, i in layers.values()) * 2 * len(clips) * len(bits_list)
    gram_s, err_s = per_step("gram_tiles"), per_step("error_tiles")
    comps = {k: {"us_per_step": v["total_us"] / v["steps"], "launches_per_step": v["launches"] / v["steps"]} for k, v in kern.items()}
    comps["gram_tiles"].update(tflops_issued=gram_flops / gram_s / 1e12, frac_mfma=gram_flops / gram_s / MFMA_F16_PEAK)
    comps["error_tiles"].update(tflops_issued=err_flops / err_s / 1e12, frac_mfma=err_flops / err_s / MFMA_F16_PEAK)
    dom = "gram_tiles" if gram_s >= err_s else "error_tiles"
    traffic, traffic_at = read_traffic(dom, args.workload)
    roofline = {"kernel": dom, "bound": "mfma", "achieved": comps[dom]["tflops_issued"], "peak": MFMA_F16_PEAK / 1e12,
                "unit": "TFLOP/s", "frac": comps[dom]["frac_mfma"], "traffic": traffic, "traffic_measured_at": traffic_at,
                "note": "issued flops of all the kernel's launches in a step over their summed durations (a step holds "
                        "launches of several sizes); traffic likewise summed over a step"}
    # quantizer: bytes both dimensions move per weight (W read for each, two fp16 dW, packed codes, scale + zero)
    q_s = per_step("quant_both") + per_step("quant_oc") + per_step("quant_ic")
    q_bytes = sum(block_weights * (2 * (2 + 2 + b / 8.0) + 2 * 5.0 / group) for b in bits_list) * len(clips)
    if q_s > 0:
        comps["quantizers"] = {"us_per_step": q_s * 1e6, "GBps_algorithmic": q_bytes / q_s / 1e9, "frac_hbm": q_bytes / q_s / HBM_PEAK,
                               "note": "in-step launches, the bytes of the two dimensions added up (W read for each)"}
    searched = block_weights * len(bits_list)
    sec_per_step = elapsed / args.steps
    result = {
        "metric": "weight params quantized+scored (both dims)/s", "value": searched / sec_per_step, "unit": "weights/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{cfg['name']}: one step = one decoder block, {len(layers)} layers "
                               f"({', '.join(f'{n}[{o},{i}]' for n, (o, i) in layers.items())}), X[{tokens},w] per input width "
                               f"w in {widths}, int{'/int'.join(str(b) for b in bits_list)} g{group} both dims"
                               + (f" x {len(clips)} clip ratios" if len(clips) > 1 else "") + " + selection"
                               + (f"; blocks streamed, weights regenerated per block ({n_blocks_model}-block model)" if streaming else ""),
                   "bits": list(bits_list), "group": group, "tokens": tokens, "weights_per_block": block_weights,
                   "searches_per_step": len(layers) * len(bits_list)},
        "roofline": roofline, "kernels": comps,
        "gram_share_of_step": gram_s / sec_per_step,
        "weights_per_s_without_gram": searched / max(sec_per_step - gram_s - per_step("gram_reduce"), 1e-9),
    }
    if log is not None:
        result["results_log"] = {"records": len(recs), "sample": recs[-2:], "ic_chosen": sum(r["dim"] == "ic" for r in recs),
                                 "note": "one JSON line per (seed, block, layer, bits, group), warm-up blocks included; a "
                                         "rerun with --log PATH --resume skips the keys the file holds"}
        log.close()
        if args.log is None:
            os.remove(log_path)
    else:
        result["results_sample"] = results[-2:]
    if not args.no_cpu_baseline:
        by_shape = {}
        for n, sh in layers.items():
            by_shape.setdefault(sh, []).append(n)
        host_layers = [(bufs[0][names[0]].cpu().numpy(), len(names)) for sh, names in by_shape.items()]
        Xs = {}

        def X_of(w, t):
            if w not in Xs or Xs[w].shape[0] < t:
                Xs[w] = Xd[w][:t].cpu().numpy()
            return Xs[w][:t]
        result["cpu_baseline"] = cpu_baseline(host_layers, X_of, tokens, bits_list, group, n_clips=len(clips), budget_flops=2.0e11)
    print(json.dumps(result))


def timeline_bench(args):
    """Where the Gram tile kernel's time goes on the narrow layers, piece by piece (adadim_probe_gram_timeline): the
    4096-wide input of the q_proj workload and the 5120-wide one of the streamed model at 65536 tokens, once with the fixed
    order the library uses for plans with short pieces and once with one workgroup per piece left to the hardware's
    dispatcher.  Per run: the plan, the span from the first start to the last end, the mean duration and shader
    clock of each list's pieces, when the last piece of each XCD's lists ends, and how many short pieces started
    more than 20 us after the first short piece of their XCD.  One JSON line."""
    import torch
    from paper_2309_15531_amd import binding as B
    from paper_2309_15531_amd import synth
    B.load_library()
    ctx = B.Context()
    runs = []
    for cfg_id, width in ((1, 4096), (3, 5120)):
        X = synth.config_activations_device(cfg_id, width, tokens=65536)
        for dispatcher in (False, True, False, True):
            rec, plan = ctx.adadim_probe_gram_timeline(X, dispatcher=dispatcher)
            lists = {}
            for name, c in (("full", 0), ("rest", 1), ("short", 2)):
                r = rec[rec[:, 0] == c]
                if len(r):
                    dur = r[:, 3] - r[:, 2]
                    lists[name] = {"pieces": int(len(r)), "mean_us": round(float(dur.mean()), 1),
                                   "clock_mhz": round(float((r[:, 4] / dur).mean()))}
            xcd_end = [round(float(rec[rec[:, 1] == x][:, 3].max()), 1) for x in range(8)]
            late = 0
            short = rec[rec[:, 0] == 2]
            for x in range(8):
                sx = short[short[:, 1] == x]
                if len(sx):
                    late += int((sx[:, 2] > sx[:, 2].min() + 20.0).sum())
            runs.append({"in": width, "order": "dispatcher" if dispatcher else ("fixed" if plan[6] else "dispatcher (plan has no short pieces)"),
                         "plan": {"tiles": plan[0], "full_pieces_per_tile": plan[1], "full_piece_stages": plan[2],
                                  "tiles_with_cut_rest": plan[3], "short_pieces_per_cut_rest": plan[4],
                                  "short_piece_stages": plan[5], "places_per_xcd": plan[7]},
                         "span_us": round(float(rec[:, 3].max()), 1), "lists": lists, "last_end_per_xcd_us": xcd_end,
                         "short_pieces_started_late": late})
        del X
    print(json.dumps({
        "metric": "span of one Gram tile launch, first start to last end", "value": runs[0]["span_us"], "unit": "us",
        "n_gpus": 1, "steps": 1, "warmup": 2, "ms_per_step": runs[0]["span_us"] / 1e3, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "time-stamped Gram tile launches, X[65536, 4096] and X[65536, 5120]"}, "runs": runs}))


def ceiling_bench(args):
    """What the matrix cores sustain on this chip, beside the published peak: (a) a register-resident loop of the MFMA
    instruction the two matrix kernels use, on all-zero and on random fp16 operands (adadim_probe_mfma); (b) the Gram
    kernel itself on [65536, in] inputs of zeros, of positive parts of normal deviates (half the entries zero, as the
    FFN-down input) and of normal deviates.  Same instruction streams, different operand bits: the rates differ
    because the chip lowers its clock to hold its power limit.  One JSON line."""
    import torch
    from paper_2309_15531_amd import binding as B
    B.load_library()
    ctx = B.Context()
    probe = {}
    for name, rnd in (("zeros", False), ("random", True), ("zeros_again", False), ("random_again", True)):
        runs = [ctx.adadim_probe_mfma(rnd, 4000) for _ in range(3)]
        probe[name] = {"tflops": [round(r[0], 1) for r in runs], "clock_mhz": [round(r[1]) for r in runs]}
    runs64 = [ctx.adadim_probe_mfma_f64(20000) for _ in range(3)]
    probe64 = {"tflops": [round(r[0], 1) for r in runs64], "clock_mhz": [round(r[1]) for r in runs64],
               "published_peak_tflops": 78.6}
    T = 65536
    gram = {}
    for n in (11008, 4096):
        H = torch.empty(n, n, dtype=torch.float32, device="cuda")
        g = torch.Generator(device="cuda").manual_seed(n)
        Xn = torch.randn(T, n, device="cuda", generator=g).half()
        for kind in ("normal", "relu", "zeros", "normal_again"):
            X = Xn if kind.startswith("normal") else (torch.relu(Xn) if kind == "relu" else torch.zeros_like(Xn))
            for _ in range(30 if n == 4096 else 8):
                ctx.adadim_hessian(X, H)
            torch.cuda.synchronize()
            ctx.adadim_profile_only("gram_tiles")
            ctx.adadim_profile(True)
            for _ in range(10):
                ctx.adadim_hessian(X, H)
            torch.cuda.synchronize()
            ctx.adadim_profile(False)
            ctx.adadim_profile_only(None)
            tot_ms, launches = ctx.adadim_profile_read()["gram_tiles"]
            us = tot_ms / launches * 1e3
            gram[f"in{n}_{kind}"] = {"gram_tiles_us": round(us, 1), "tflops_issued": round(gram_issued_flops(n, T) / us / 1e6, 1),
                                     "frac_of_published_peak": round(gram_issued_flops(n, T) / (us * 1e-6) / MFMA_F16_PEAK, 4)}
            del X
        del Xn, H
    worst = min(probe["random"]["tflops"] + probe["random_again"]["tflops"])
    print(json.dumps({
        "metric": "sustained fp16 MFMA rate (register-resident loop, random operands)", "value": worst, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": 3, "warmup": 0, "ms_per_step": None, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "matrix-core ceiling probe: v_mfma_f32_32x32x16_f16 loop on zero / random operands; Gram kernel on "
                               "[65536, 11008] and [65536, 4096] inputs of zeros / relu(normal) / normal"},
        "published_peak_tflops": MFMA_F16_PEAK / 1e12, "mfma_loop": probe, "mfma_f64_loop": probe64,
        "gram_kernel_by_input": gram}))


# (warm-up, timed) steps when the flags are absent.  The chip needs some tens of milliseconds of load before its
# clocks settle (the first 20 q_proj steps of a process run 5 % slower than the 200 after them), so the defaults
# time a few tenths of a second of sustained work; clip_grid has 50 launches per step and stays within the
# library's 8192 timed launches.
SETTLE_SECONDS = 0.15
DEFAULT_STEPS = {"toy": (20, 200), "q_proj": (20, 200), "gate_proj": (20, 200), "down_proj": (10, 100), "qkv": (20, 200),
                 "clip_grid": (5, 50), "gemv_ic": (100, 2000), "gptq": (3, 30), "block7b": (2, 10), "stream13b": (1, 4),
                 "block70b": (1, 2)}
BLOCK_WORKLOADS = {"block7b": 2, "stream13b": 3, "block70b": 4}      # name: config id in synth.CONFIGS


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: by workload, see DEFAULT_STEPS)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them")
    ap.add_argument("--workload", default="down_proj",
                    choices=sorted(WORKLOADS) + sorted(BLOCK_WORKLOADS) + ["gemv_ic", "gptq", "mfma_ceiling", "gram_timeline"])
    ap.add_argument("--log", default=None, help="stream13b: the JSON-lines results file (default: a fresh temporary file)")
    ap.add_argument("--resume", action="store_true", help="stream13b: keep the records --log already holds and skip their layers")
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--group", type=int, default=None, help="group size (0 = whole channel); default: the config's")
    ap.add_argument("--meta16", action="store_true",
                    help="quantize into / multiply from the b + 16/g storage format (one 16-bit word per group)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step as one recorded HIP graph in the timed region (single layer, at most 8 "
                         "candidates); per-kernel durations then come from a second pass of the same steps launched "
                         "one by one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy, the reference dispatch that scales "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    d_warm, d_steps = DEFAULT_STEPS.get(args.workload, DEFAULT_STEPS["q_proj"])
    args.steps = d_steps if args.steps is None else args.steps
    args.warmup = d_warm if args.warmup is None else args.warmup
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (layers are independent, so a multi-GPU run would "
              "deal whole layers to ranks); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2309_15531_amd import binding as B
    from paper_2309_15531_amd import search as S
    from paper_2309_15531_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.workload == "gemv_ic":
        gemv_bench(args)
        return
    if args.workload == "gptq":
        gptq_bench(args)
        return
    if args.workload in BLOCK_WORKLOADS:
        block_bench(args)
        return
    if args.workload == "gram_timeline":
        timeline_bench(args)
        return
    if args.workload == "mfma_ceiling":
        ceiling_bench(args)
        return
    B.load_library()  # fails loudly if the HIP library has not been built

    cfg_id, layer = WORKLOADS[args.workload]
    cfg = synth.CONFIGS[cfg_id]
    layers = layer if isinstance(layer, tuple) else (layer,)
    layer = layers[0]
    out_f, in_f = cfg["layers"][layer]
    bits = args.bits if args.bits is not None else (3 if 3 in cfg["bits"] else cfg["bits"][0])
    group = cfg["group"] if args.group is None else args.group
    tokens = cfg["tokens"]
    clips = tuple(S.clip_grid(cfg["clips"])) if cfg["clips"] > 1 else (1.0,)

    W = synth.config_weight(cfg_id, layer)
    X = synth.config_activations(cfg_id, in_f)
    Wd = torch.from_numpy(W).cuda()
    Xd = torch.from_numpy(X).cuda()

    use_graph = args.graph and len(layers) == 1 and 2 * len(clips) <= 8
    if use_graph:
        # a stream of its own for everything: the default stream cannot be recorded
        torch.cuda.set_stream(torch.cuda.Stream())
    ctx = B.Context()
    hp = S.PreparedHessian(ctx, in_f)
    if len(layers) == 1:
        ls = S.LayerSearch(ctx, out_f, in_f, bits, group, clips=clips, meta16=args.meta16)

        # Steps are queued back to back and the winners read after the loop, as a model driver would queue
        # the next layer while the last one's answer is on its way (layers do not depend on each other).
        # With more candidates than one scoring batch the winner is quantized again once it is known, so
        # that case waits for the answer inside every step.
        def step():
            hp.update_prepared(Xd)
            if ls.inline:
                ls.launch(Wd, hp)
            else:
                ls.run(Wd, hp)

        def finish():
            return ls.result() if ls.inline else (int(ls.best.item()),) + ls.cands[int(ls.best.item())]
    else:
        Wds = [Wd] + [torch.from_numpy(synth.config_weight(cfg_id, l)).cuda() for l in layers[1:]]
        ls = S.SharedSearch(ctx, len(layers), out_f, in_f, bits, group)
        ls.cands = [(d, 1.0) for _ in layers for d in (B.DIM_OC, B.DIM_IC)]

        def step():
            hp.update_prepared(Xd)
            ls.launch(Wds, hp)

        def finish():
            dims = ls.result()
            return dims[0], dims[0], 1.0

    timed_step = step
    if use_graph:
        torch.cuda.synchronize()
        gs = S.GraphedSearch(ctx, ls, hp, Wd, Xd)
        timed_step, finish = gs.launch, gs.result
    # Before the W warm-up steps: untimed steps until the chip has been under load for SETTLE_SECONDS, so that a
    # short run (--steps 5 --warmup 1) times the clocks a long job sees and not their ramp.  Skipped under the
    # counter runs (--copy-calibration), which want few dispatches.
    settle_steps = 0
    if not args.copy_calibration:
        t_settle = time.perf_counter()
        while time.perf_counter() - t_settle < SETTLE_SECONDS:
            for _ in range(4):
                timed_step()
            torch.cuda.synchronize()
            settle_steps += 4
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        copy_calibration()
    # Per-kernel durations come from the library's event pair around each launch, and a pair costs the stream about
    # 7 us: bracketing all five kernels of a q_proj step takes 3 % off the figure being measured.  So the timed
    # region brackets one kernel, the dominant one (found in one untimed step with every kernel bracketed), which
    # is the one the roofline object describes; the other kernels are timed in a second, untimed pass of the same
    # steps.
    def profiled(n, fn, only=None):
        ctx.adadim_profile_only(only)
        ctx.adadim_profile(True)
        t_begin = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t_begin
        ctx.adadim_profile(False)
        ctx.adadim_profile_only(None)
        return dt, {k: {"avg_us": v[0] / max(v[1], 1) * 1e3, "launches": v[1], "steps": n,
                        "min_us": v[2] * 1e3, "median_us": v[3] * 1e3, "max_us": v[4] * 1e3}
                    for k, v in ctx.adadim_profile_read(spread=True).items()}

    _, probe = profiled(1, step)
    dominant = max(probe, key=lambda k: probe[k]["avg_us"] * probe[k]["launches"])
    if use_graph:
        # the recorded graph carries no events at all
        t0 = time.perf_counter()
        for _ in range(args.steps):
            timed_step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        live = {}
    else:
        elapsed, live = profiled(args.steps, timed_step, only=dominant)
    best, dim, clip = finish()
    # What the chip's matrix cores sustain right now on nothing but the MFMA instruction, random operands: the
    # ceiling the two matrix kernels work under on this machine (power-limited clock), beside the published peak.
    loop = [ctx.adadim_probe_mfma(1, 4000) for _ in range(2)][-1]
    _, kern = profiled(min(args.steps, 50), step)
    kern.update(live)                                         # the dominant kernel: as measured in the timed region
    losses = ls.losses.cpu().numpy().tolist()

    ms_per_step = elapsed / args.steps * 1e3

    # roofline of the dominant kernel: the Gram-matrix tiles.  MFMA flops actually issued = upper-triangular
    # tiles x 2*BT*BT*tokens.  HBM bytes per launch of that kernel from profiles/traffic.txt (null when not measured).
    gram_flops = gram_issued_flops(in_f, tokens)
    gram_s = kern["gram_tiles"]["avg_us"] * 1e-6
    traffic, traffic_at = read_traffic("gram_tiles", args.workload)
    roofline = {
        "kernel": "gram_tiles", "bound": "mfma", "achieved": gram_flops / gram_s / 1e12, "peak": MFMA_F16_PEAK / 1e12,
        "unit": "TFLOP/s", "frac": gram_flops / gram_s / MFMA_F16_PEAK, "traffic": traffic, "traffic_measured_at": traffic_at,
        "must_move_bytes": 2.0 * tokens * in_f + 4.0 * in_f * in_f,
        "dense_equivalent": 2.0 * tokens * in_f * in_f / gram_s / 1e12,
    }
    spread = {k: kern["gram_tiles"][k] for k in ("min_us", "median_us", "max_us") if k in kern["gram_tiles"]}

    # the error GEMM (MFMA) and the quantizers (HBM)
    comps = {}
    if "error_tiles" in kern:
        s = kern["error_tiles"]["avg_us"] * 1e-6
        per_launch = len(ls.cands) * kern["error_tiles"]["steps"] / kern["error_tiles"]["launches"]   # candidates per launch
        issued = per_launch * error_issued_flops(out_f, in_f)
        comps["error_tiles"] = {
            "avg_us": s * 1e6, "candidates_per_launch": per_launch, "tflops_issued": issued / s / 1e12,
            "frac_mfma": issued / s / MFMA_F16_PEAK,
            "tflops_dense_equivalent": per_launch * 2.0 * out_f * in_f * in_f / s / 1e12,
        }
    # with many candidates per layer (clip grid) the error GEMM, not the Gram matrix, is the dominant kernel
    et = comps.get("error_tiles")
    if et and dominant == "error_tiles":
        traffic, traffic_at = read_traffic("error_tiles", args.workload)
        roofline = {"kernel": "error_tiles", "bound": "mfma", "achieved": et["tflops_issued"], "peak": MFMA_F16_PEAK / 1e12,
                    "unit": "TFLOP/s", "frac": et["frac_mfma"], "traffic": traffic, "traffic_measured_at": traffic_at,
                    "dense_equivalent": et["tflops_dense_equivalent"]}
        spread = {k: kern["error_tiles"][k] for k in ("min_us", "median_us", "max_us") if k in kern["error_tiles"]}
    roofline.update(spread)                                   # of the same launches `achieved` averages over
    roofline["chip_mfma_loop"] = {"tflops": round(loop[0], 1), "clock_mhz": round(loop[1]),
                                  "frac_of_peak": round(loop[0] * 1e12 / MFMA_F16_PEAK, 3),
                                  "note": "v_mfma_f32_32x32x16_f16 alone, register-resident random fp16 operands, right "
                                          "after the timed region"}
    if et:
        et["traffic"], et["traffic_measured_at"] = read_traffic("error_tiles", args.workload)
    # W read + fp16 dW written + scale/zero (one pair per group of the larger of the two group counts)
    qbytes = out_f * in_f * (2 + 2) + 5.0 * (out_f * in_f / group if group else max(out_f, in_f))
    for k in ("quant_oc", "quant_ic"):
        if k in kern:
            s = kern[k]["avg_us"] * 1e-6
            comps[k] = {"avg_us": s * 1e6,
                        "note": "in-step launches (inputs mostly cache resident; event pairs add ~3 us to "
                                "each short kernel); see quantizer_hbm for the HBM-resident rate"}
    for k, v in kern.items():
        comps.setdefault(k, {"avg_us": v["avg_us"]})
        comps[k]["launches_per_step"] = v["launches"] / v["steps"]
        for f in ("min_us", "median_us"):
            if f in v:
                comps[k][f] = v[f]

    # The quantizer on its own, with HBM-resident inputs: back-to-back launches between two events
    # while rotating over enough weight / dW buffers (> 512 MB) that the 256 MB Infinity Cache
    # cannot serve them.  Bytes per launch: W read + fp16 dW written + scales and zeros.
    quant = {}
    n_rot = max(2, int(np.ceil(600e6 / (out_f * in_f * 2))))
    Ws = [Wd] + [Wd.clone() for _ in range(n_rot - 1)]
    dWs = [ctx.alloc_score(out_f, in_f) for _ in range(n_rot)]
    def kernel_seconds(sweep):
        """Average duration of the launches of three sweeps, from the library's event pair around each launch (as
        for every other kernel here; an interval over back-to-back launches would add the launch gaps, which for
        these short kernels are a quarter of the kernel)."""
        sweep()
        torch.cuda.synchronize()
        ctx.adadim_profile(True)
        for _ in range(3):
            sweep()
        torch.cuda.synchronize()
        ctx.adadim_profile(False)
        tot = [v for k, v in ctx.adadim_profile_read().items() if k.startswith("quant")]
        return sum(v[0] for v in tot) * 1e-3 / (3 * n_rot)

    for dim, name in ((B.DIM_OC, "quant_oc"), (B.DIM_IC, "quant_ic")):
        def sweep():
            for i in range(n_rot):
                ctx.adadim_quantize(Ws[i], dim, bits, group, 1.0, dW=dWs[i], dW_dtype=B.DW_F16_SCALED,
                                    colscale=hp.colscale)
        sec = kernel_seconds(sweep)
        quant[name] = {"us_per_launch": sec * 1e6, "GBps_algorithmic": qbytes / sec / 1e9,
                       "frac_hbm": qbytes / sec / HBM_PEAK, "rotating_buffers": n_rot}
    # both dimensions in one call, as the search issues them (one launch where both fast kernels take the shape):
    # W read twice, two fp16 dW written
    if group == 0 or (out_f % group == 0 and in_f % group == 0):
        dW2 = [ctx.alloc_score(out_f, in_f) for _ in range(n_rot)]

        def sweep_both():
            for i in range(n_rot):
                ctx.adadim_quantize_both(Ws[i], bits, group, hp.colscale, {"dW": dWs[i]}, {"dW": dW2[i]})
        sec = kernel_seconds(sweep_both)
        once = 2 * qbytes - out_f * in_f * 2          # W counted once: what one pass over W would have to move
        quant["quant_both"] = {"us_per_launch": sec * 1e6, "GBps_algorithmic": 2 * qbytes / sec / 1e9,
                               "frac_hbm": 2 * qbytes / sec / HBM_PEAK, "frac_hbm_w_counted_once": once / sec / HBM_PEAK,
                               "rotating_buffers": n_rot,
                               "note": "bytes of the two dimensions added up (W read for each), as for the single launches"}
        del dW2
    # For scale: what a plain device copy of one weight matrix reaches on this machine in the same arrangement
    # (torch's elementwise copy of W into a buffer of the same size, the same rotation; bytes = read + written).
    # The quantizers read W and write as many bytes again, so this is the rate to hold their fractions against.
    dsts = [torch.empty_like(Wd) for _ in range(n_rot)]
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for rep in range(2):                                      # the first sweep warms up
        ev0.record()
        for _ in range(3 if rep else 1):
            for i in range(n_rot):
                dsts[i].copy_(Ws[i])
        ev1.record()
        torch.cuda.synchronize()
    copy_sec = ev0.elapsed_time(ev1) * 1e-3 / (3 * n_rot)
    quant["plain_copy"] = {"us_per_launch": copy_sec * 1e6, "GBps": 4.0 * out_f * in_f / copy_sec / 1e9,
                           "frac_hbm": 4.0 * out_f * in_f / copy_sec / HBM_PEAK, "rotating_buffers": n_rot,
                           "note": "back-to-back copies between two events: includes the gaps between launches"}
    del Ws, dWs, dsts

    result = {
        "metric": "weight params quantized+scored (both dims)/s",
        "value": len(layers) * out_f * in_f / (elapsed / args.steps),
        "unit": "weights/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": settle_steps, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{cfg['name']}/{'+'.join(layers)} W[{out_f},{in_f}] X[{tokens},{in_f}] int{bits} "
                               f"g{group} both dims" + (f" x {len(clips)} clip ratios" if len(clips) > 1 else "") + " + selection"
                               + (", 16-bit group words" if args.meta16 else ""),
                   "bits": bits, "group": group, "tokens": tokens},
        "result": {"losses": losses, "best": int(best), "dim": "oc" if dim == 0 else "ic"},
        "roofline": roofline,
        "launch": ("one recorded HIP graph per step; kernel durations from a second pass of the same steps launched "
                   "one by one" if use_graph else
                   "kernel by kernel; the duration of %s (the dominant kernel, which roofline describes) from HIP events in "
                   "the timed region, the other kernels' from a second pass of the same steps" % dominant),
        "quantizer_hbm": dict(quant, note=("each launch moves %.0f MB: below some 150 MB a launch is mostly ramp and tail, the "
                                           "HBM-bound rate shows on the gate_proj / down_proj / clip_grid workloads" % (qbytes / 1e6))),
        "kernels": comps,
    }
    if not args.no_cpu_baseline:
        Ws_host = [(W, 1)] + [(synth.config_weight(cfg_id, l), 1) for l in layers[1:]]
        result["cpu_baseline"] = cpu_baseline(Ws_host, lambda w, t: X[:t], tokens, (bits,), group, n_clips=len(clips))
    print(json.dumps(result))


if __name__ == "__main__":
    main()
