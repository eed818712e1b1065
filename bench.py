#!/usr/bin/env python3
"""Benchmark of the small-batch GeMM hot path on one MI355X.

A step is one pass of the whole hot path over one batch sweep: for every batch size B of
the workload, the four linear layers of one transformer layer (QKV, attention output,
FFN1 + bias + GeLU, FFN2 + bias + residual) through sbi_layer_gemms.  The default workload
is the h=4096 layer at B in {1, 2, 4, 8} (W shapes [4096,12288], [4096,4096], [4096,16384],
[16384,4096], 384 MiB of fp16 weights).  Steps rotate over several device copies of the
laid-out weights so that every pass streams them from HBM rather than from the 256 MB
last-level cache.  All inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: whole-job weight-streaming throughput (algorithmic bytes / time), the
roofline figure of the dominant kernel measured with events around each of its launches,
and the CPU oracle timed on the host cores for the same GeMMs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2,
                    help="workload configuration: 1-4 time the four-GeMM layer (2 = h=4096, the headline); 5 is the "
                         "batch crossover sweep of the h=8192 FFN1 GeMM (per batch: every forced path and the dispatcher's pick)")
    ap.add_argument("--no-tune", action="store_true",
                    help="keep the cost model's launch plans instead of measuring the candidates once at set-up "
                         "(sbi_layer_tune / sbi_gemm_tune, untimed, as a serving engine does at model load)")
    ap.add_argument("--no-extra", action="store_true",
                    help="default run only: skip the rows beyond the headline workload (single-GeMM launches, B=16, "
                         "the h=12288 configurations 3 and 4)")
    ap.add_argument("--batches", type=str, default="", help="comma list overriding the batch sweep")
    ap.add_argument("--copies", type=int, default=0, help="weight copies to rotate over (0 = auto)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-gemm", action="store_true", help="also time every GeMM as a launch of its own")
    ap.add_argument("--path", type=str, default="auto", choices=["auto", "stream", "mfma", "streamk"])
    ap.add_argument("--graph", type=int, default=0, metavar="N",
                    help="capture N consecutive steps into one HIP graph and time replays of it "
                         "(removes host launch overhead; steps is rounded to a multiple of N)")
    ap.add_argument("--layernorm", action="store_true",
                    help="fuse a layer-norm in front of QKV and FFN1 (sbi_layer's ln1/ln2); also times the "
                         "same layer with the two norms as separate torch kernels, for comparison")
    ap.add_argument("--int8", action="store_true",
                    help="INT8 layer: weights quantised per output channel and laid out as int8, activations "
                         "quantised inside the kernel (sbi_layer's scales); algorithmic bytes count one byte per weight")
    ap.add_argument("--attention", type=str, default=None, metavar="B:H:d:ctx[:r][,...]", nargs="?",
                    const="1:32:128:136,8:32:128:136,64:32:128:136,8:32:128:2048,64:32:128:2048,1:32:128:8192,8:32:128:8192",
                    help="time the single-token attention with a KV cache (sbi_attn_decode) instead of the GeMMs: "
                         "ctx = positions attended to, the new token's included; a shape ending in :r is a ragged batch "
                         "(sbi_attn_decode_ragged, lengths spread evenly from ctx/8 to ctx); value = KV-cache streaming GB/s")
    ap.add_argument("--decoder-layer", type=str, default=None, metavar="B:ctx[,...]", nargs="?", const="1:136,4:136,8:136,8:2048",
                    help="time one token-generation step of a whole h=4096 layer (32 heads): layer-norm + QKV, attention "
                         "over the KV cache, attention output + residual, layer-norm + FFN1 + GeLU, FFN2 + residual as five "
                         "dependent launches replayed from a HIP graph; value = algorithmic bytes of the step / time")
    ap.add_argument("--read-ceiling", action="store_true",
                    help="time pure streaming reads of the layer's bytes (sbi_calib_read: the weight stream's access shape, "
                         "nothing else) over block shapes, cold, and exit: the ceiling the GeMM launch is measured against")
    ap.add_argument("--timeline", action="store_true",
                    help="measurement build only (python paper_2207_00032_amd/csrc/build.py --dev): per-block timestamps of "
                         "the layer launch - start, X staged, first k-step, end of stream, end of block - as percentiles")
    ap.add_argument("--ablate", action="store_true",
                    help="measurement build only: time the layer launch with parts of the kernel switched off "
                         "(matrix-core work, operand reads, X staging, reduction + epilogue)")
    ap.add_argument("--split-cost", action="store_true",
                    help="measurement build only: the same 384 MiB of weights as one GeMM without split-K ([4096,49152]) and "
                         "with it ([16384,12288] split 2 and 4), identical block streams: time per launch, span of the blocks "
                         "and what a block spends between the end of its stream and its own end (the split-K hand-over)")
    ap.add_argument("--single-timeline", action="store_true",
                    help="measurement build only: each of the configuration's four GeMMs as a launch of its own at B = 1 "
                         "(the dispatcher's plan): time per launch, span of the blocks, per-block timestamps as percentiles, "
                         "and what lies between two such launches")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="run a few copy-kernel and layer launches and exit (for rocprofv3 --pmc runs)")
    return ap.parse_args()


def measured_traffic(args, batches):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary (FETCH_SIZE and WRITE_SIZE
    runs scaled against the copy kernel), if it covers exactly this workload; else None."""
    if args.config != 2 or tuple(batches) != (1, 2, 4, 8) or args.path != "auto" or args.layernorm or args.int8:
        return None
    path = os.path.join(ROOT, "profiles", "sbi_mfma_kernel_config2_pmc_traffic.md")
    try:
        for line in open(path):
            if line.strip().startswith("traffic_bytes_per_launch"):
                return int(line.split("=")[1])
    except OSError:
        pass
    return None


def attention_bytes(B, H, d, ctx):
    """HBM bytes one decode-attention call must move: ctx-1 cached rows of K and of V per
    (sequence, head), q/k/v of the new token in, its k and v rows out to the caches, the context out."""
    return 2 * (2 * B * H * (ctx - 1) * d) + 2 * (3 * B * H * d) + 2 * (2 * B * H * d) + 2 * B * H * d


def attention_main(args):
    """--attention: one JSON line; a step is one call per listed shape."""
    import numpy as np
    import torch
    from paper_2207_00032_amd import binding as sb
    from paper_2207_00032_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sb.load()
    dev = torch.device("cuda:0")
    # B:H:d:ctx, or B:H:d:ctx:r for a ragged batch (sbi_attn_decode_ragged): sequence b attends to
    # ctx/8 + b (ctx - ctx/8) / max(B-1, 1) positions, i.e. lengths spread evenly up to ctx, bound ctx - 1
    shapes = [(tuple(int(v) for v in item.split(":")[:4]), item.split(":")[4:] == ["r"]) for item in args.attention.split(",")]
    cases = []
    for (B, H, d, ctx), ragged in shapes:
        lens = [ctx // 8 + b * (ctx - ctx // 8) // max(B - 1, 1) for b in range(B)] if ragged else [ctx] * B
        qkv, K, V = wl.make_attention_inputs(B, H, d, ctx, seed=0, config_id=600)
        cache_bytes = 2 * K.nbytes
        copies = max(2, -(-3 * 256 * 1000 * 1000 // cache_bytes))      # rotate so the cache comes from HBM
        Kd = [torch.from_numpy(K).to(dev) for _ in range(copies)]
        Vd = [torch.from_numpy(V).to(dev) for _ in range(copies)]
        cases.append({"shape": (B, H, d, ctx), "lens": lens,
                      "pos": torch.tensor([n - 1 for n in lens], dtype=torch.int32, device=dev) if ragged else None,
                      "host": (qkv, K, V), "qkv": torch.from_numpy(qkv).to(dev), "K": Kd, "V": Vd,
                      "out": torch.empty((B, H * d), dtype=torch.float16, device=dev), "n": 0,
                      "ws": sb.new_workspace(max(256, sb.attn_workspace_bytes(B, H, d, ctx)), dev)})

    def call(c):
        j = c["n"] % len(c["K"])
        c["n"] += 1
        B, H, d, ctx = c["shape"]
        if c["pos"] is not None:
            sb.attn_decode_ragged(c["qkv"], c["K"][j], c["V"][j], c["pos"], ctx - 1, out=c["out"], workspace=c["ws"])
        else:
            sb.attn_decode(c["qkv"], c["K"][j], c["V"][j], ctx - 1, out=c["out"], workspace=c["ws"])

    def step():
        for c in cases:
            call(c)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec_per_step = (time.perf_counter() - t0) / args.steps
    def case_bytes(c):                                          # every sequence moves what its own length asks for
        B, H, d, ctx = c["shape"]
        return sum(attention_bytes(1, H, d, n) for n in c["lens"])

    bytes_per_step = sum(case_bytes(c) for c in cases)

    per_call = []
    for c in cases:
        us = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                call(c)
            e1.record()
            torch.cuda.synchronize()
            us.append(e0.elapsed_time(e1) * 1e2)
        med = sorted(us)[2]
        nb = case_bytes(c)
        B, H, d, ctx = c["shape"]
        per_call.append({"B": B, "heads": H, "head_dim": d, "ctx": ctx, "ragged": c["pos"] is not None,
                         "us_median": round(med, 2),
                         "GBps": round(nb / med / 1e3, 1), "hbm_frac": round(nb / med / 1e3 / HBM_PEAK_GBPS, 4),
                         "bytes": nb})
    big = max(per_call, key=lambda r: r["bytes"])
    roofline = {"bound": "hbm", "achieved": big["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": big["hbm_frac"],
                "traffic": None, "kernel": f"sbi_attn_decode_kernel<{big['head_dim']}>",
                "avg_launch_us": big["us_median"], "avg_bytes_per_launch": big["bytes"],
                "shape": f"B={big['B']} H={big['heads']} d={big['head_dim']} ctx={big['ctx']}"}

    cpu = parity = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        t_cpu, nbytes, n_bad, max_abs = 0.0, 0, 0, 0.0
        for c in cases:
            B, H, d, ctx = c["shape"]
            if attention_bytes(B, H, d, ctx) > (64 << 20) or c["pos"] is not None:
                continue
            qkv, K, V = c["host"]
            c0 = time.perf_counter()
            want, _, _ = orc.attn_decode(qkv, K, V, ctx - 1)
            t_cpu += time.perf_counter() - c0
            nbytes += attention_bytes(B, H, d, ctx)
            call(c)
            torch.cuda.synchronize()
            ok, rep = orc.check_close(c["out"].cpu().numpy(), want)
            n_bad += rep["n_bad"]
            max_abs = max(max_abs, rep["max_abs"])
        if t_cpu > 0:
            cpu = {"value": round(nbytes / t_cpu / 1e9, 3), "unit": "GB/s", "cores": orc.max_threads(), "kind": "oracle",
                   "sample": f"the listed shapes of at most 64 MiB, {t_cpu:.1f} s of CPU time"}
            parity = {"ok": n_bad == 0, "n_bad": n_bad, "max_abs": max_abs, "tolerance": "max(2 ulp16, 1e-3)"}
    print(json.dumps({
        "metric": "KV-cache HBM GB/s (algorithmic bytes of single-token attention / time)",
        "value": round(bytes_per_step / sec_per_step / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(sec_per_step * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "single-token attention over a KV cache, one call per shape "
                               "(B:heads:head_dim:context) " + args.attention},
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity, "per_call": per_call}))


def decoder_main(args):
    """--decoder-layer: one JSON line; a step is one token-generation step per listed (B, context)."""
    import numpy as np
    import torch
    from paper_2207_00032_amd import binding as sb
    from paper_2207_00032_amd import decoder
    from paper_2207_00032_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sb.load()
    dev = torch.device("cuda:0")
    h, heads, f = 4096, 32, 16384
    d = h // heads
    cases = [tuple(int(v) for v in item.split(":")) for item in args.decoder_layer.split(",")]
    Bmax = max(B for B, _ in cases)
    hw = {}
    for gi, (name, K, N) in enumerate((("qkv", h, 3 * h), ("out", h, h), ("ffn1", h, f), ("ffn2", f, h))):
        W, bias, _, _ = wl.make_gemm_inputs(K, N, 1, seed=0, config_id=2, gemm_id=gi)
        hw["W" + name], hw["b" + name] = torch.from_numpy(W).to(dev), torch.from_numpy(bias).to(dev)
    g1, be1, x_host = wl.make_layernorm_inputs(h, Bmax, seed=0, config_id=2, gemm_id=0)
    g2, be2, _ = wl.make_layernorm_inputs(h, Bmax, seed=0, config_id=2, gemm_id=2)
    g1, be1, g2, be2 = (torch.from_numpy(a).to(dev) for a in (g1, be1, g2, be2))
    copies = 3                                                    # 3 x 384 MiB of weights: every step streams from HBM
    layers = [decoder.DecoderLayer(h, heads, hw["Wqkv"], hw["bqkv"], hw["Wout"], hw["bout"], hw["Wffn1"], hw["bffn1"],
                                   hw["Wffn2"], hw["bffn2"], g1, be1, g2, be2) for _ in range(copies)]
    del hw["Wqkv"], hw["Wout"], hw["Wffn1"], hw["Wffn2"]
    weight_bytes = 2 * (3 * h * h + h * h + 2 * h * f)
    results = []
    tuned = {}
    total_bytes = total_sec = 0.0
    for B, ctx in cases:
        _, Kc, Vc = wl.make_attention_inputs(B, heads, d, ctx, seed=0, config_id=2)
        x = torch.from_numpy(np.ascontiguousarray(x_host[:B])).to(dev)
        states = [layers[c].new_state(B, ctx, dev, torch.from_numpy(Kc).to(dev), torch.from_numpy(Vc).to(dev))
                  for c in range(copies)]
        nbytes = weight_bytes + attention_bytes(B, heads, d, ctx) + 2 * B * (3 * h + 4 * h + f) * 2

        # every layer copy gets the same input x; its row moments stand in for what the previous
        # layer's FFN2 epilogue leaves (each FFN2 here emits its own output's moments inside the timed
        # region, as in a real stack), so the input layer-norm starts from moments like the second one
        xp = x.float().view(B, h // 64, 64)
        x_moments = torch.stack((xp.mean(-1), ((xp - xp.mean(-1, keepdim=True)) ** 2).sum(-1)), dim=-1).contiguous()

        def run():
            for c in range(copies):
                layers[c].step(x, ctx - 1, states[c], x_moments=x_moments)

        if not args.no_tune:
            # the two plain GeMMs of the step (attention output, FFN2) get their launch plans measured, within the
            # workspace the states were given; the layer-norm launches keep the model's plans
            st0 = states[0]
            st0.ctx.zero_()
            st0.f.zero_()
            tuned[f"out B={B}"] = sb.gemm_tune([l.Wout for l in layers], h, h, st0.ctx, layers[0].bout, x, "bias_residual",
                                               out=st0.x2, workspace=st0.workspace)
            tuned[f"ffn2 B={B}"] = sb.gemm_tune([l.Wffn2 for l in layers], f, h, st0.f, layers[0].bffn2, st0.x2,
                                                "bias_residual", out=st0.y, workspace=st0.workspace)
        run()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                run()
        torch.cuda.synchronize()
        reps = max(1, args.steps // copies)
        us = {}
        for label, fn in (("graph", graph.replay), ("eager", run)):
            for _ in range(max(1, args.warmup // copies)):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            us[label] = (time.perf_counter() - t0) / (reps * copies) * 1e6
        total_bytes += nbytes
        total_sec += us["graph"] * 1e-6
        results.append({"B": B, "ctx": ctx, "us_per_layer_step_graph": round(us["graph"], 2),
                        "us_per_layer_step_eager": round(us["eager"], 2), "GBps": round(nbytes / us["graph"] / 1e3, 1),
                        "bytes": nbytes})
        del states
        torch.cuda.empty_cache()
    print(json.dumps({
        "metric": "HBM GB/s of a whole layer's token-generation step (algorithmic bytes of its five dependent launches / time)",
        "value": round(total_bytes / total_sec / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(total_sec * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": "h=4096 layer (32 heads of 128, FFN 16384), one generated token per step, "
                               "(B:context) " + args.decoder_layer + ", HIP-graph replay, 3 weight copies"},
        "roofline": None, "cpu_baseline": None, "per_case": results,
        "tuned_plans": {k: {"waves": v["waves"], "depth": v["depth"], "block_ksteps": v["block_ksteps"],
                            "us_best": round(v["us_best"], 2), "us_model": round(v["us_model"], 2)} for k, v in tuned.items()}}))


MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X dense fp16 matrix-core peak, published


def _median_us(torch, fn, reps=10, runs=5):
    """Median over `runs` of the time per call of `reps` back-to-back calls (events on the current stream)."""
    us = []
    for _ in range(runs):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us.append(e0.elapsed_time(e1) * 1e3 / reps)
    return sorted(us)[len(us) // 2]


def crossover_main(args):
    """--config 5: the batch crossover sweep on the h=8192 FFN1 GeMM [8192,32768] + bias + GeLU with
    outlier input channels.  Per batch size: the time under every forced path (vector-ALU stream
    kernel up to 8 rows, matrix-core block kernel, work-balanced kernel) and under the dispatcher's own
    pick with the plan it made, weights cold (three copies in rotation, 1.5 GiB); then, for the
    matrix-core rate at the large-batch end, a 128 MiB slice of the same matrix cold (six copies in
    rotation) and warm (one copy, resident in the 256 MB last-level cache), with the ceiling
    B x achieved bytes/s beside it.  One JSON line; value = algorithmic bytes / time of the
    dispatcher's picks over the whole sweep."""
    import numpy as np
    import torch
    from oracle import oracle as orc
    from paper_2207_00032_amd import binding as sb
    from paper_2207_00032_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sb.load()
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[5]
    spec = cfg.gemms[0]
    K, N = spec.K, spec.N
    batches = tuple(int(b) for b in args.batches.split(",")) if args.batches else cfg.batches
    Bmax = max(batches)
    W, bias, X, R = wl.make_gemm_inputs(K, N, Bmax, 0, 5, 0, cfg.outlier_channels, cfg.outlier_scale)
    Wd = torch.from_numpy(W).to(dev)
    Wl0 = sb.layout_weights(Wd)
    Wl = [Wl0, Wl0.clone(), Wl0.clone()]
    bias_d = torch.from_numpy(bias).to(dev)
    paths = [("auto", sb.PATH_AUTO), ("mfma", sb.PATH_MFMA), ("stream", sb.PATH_STREAM), ("streamk", sb.PATH_STREAMK)]
    need = max(sb.plan(B, K, N, p)["workspace_bytes"] for B in batches for _, p in paths
               if not (p == sb.PATH_STREAM and B > 8))
    ws = sb.new_workspace(max(need, 256), dev)
    n = [0]
    rows = []
    auto_us = {}
    if args.pmc_probe:                  # a few launches of the dispatcher's pick per batch, for rocprofv3 --pmc runs
        for B in batches:
            Xd = torch.from_numpy(np.ascontiguousarray(X[:B])).to(dev)
            Yd = torch.empty((B, N), dtype=torch.float16, device=dev)
            for i in range(4):
                sb.gemm(Wl[i % 3], K, N, Xd, bias_d, None, "bias_gelu", out=Yd, workspace=ws)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "config": 5, "batches": list(batches), "launches_per_batch": 4,
                          "bytes": {str(B): spec.algorithmic_bytes(B) for B in batches},
                          "plans": {str(B): sb.plan(B, K, N) for B in batches}}))
        return
    for B in batches:
        Xd = torch.from_numpy(np.ascontiguousarray(X[:B])).to(dev)
        Yd = torch.empty((B, N), dtype=torch.float16, device=dev)
        want = None if args.no_cpu_baseline else orc.gemm(X[:B], W, bias, None, epi=orc.EPI_BIAS | orc.EPI_GELU)
        for name, path in paths:
            if path == sb.PATH_STREAM and B > 8:
                continue
            pl = sb.plan(B, K, N, path)

            def call():
                sb.gemm(Wl[n[0] % 3], K, N, Xd, bias_d, None, "bias_gelu", out=Yd, workspace=ws, path=path)
                n[0] += 1

            for _ in range(3):
                call()
            us = _median_us(torch, call)
            torch.cuda.synchronize()
            ok = None
            if want is not None:
                ok, _rep = orc.check_close(Yd.cpu().numpy(), want)
            nbytes, nflops = spec.algorithmic_bytes(B), spec.flops(B)
            rows.append({"B": B, "path": name, "kernel": sb.PATH_NAMES[pl["path"]], "waves": pl["waves"], "depth": pl["depth"],
                         "split_k": pl["split_k"], "panels": pl["panels"], "us": round(us, 2),
                         "GBps": round(nbytes / us / 1e3, 1), "hbm_frac": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4),
                         "TFLOPs": round(nflops / us / 1e6, 2),
                         "mfma_frac": round(nflops / us / 1e6 / MFMA_F16_PEAK_TFLOPS, 4),
                         "hbm_ceiling_mfma_frac": round(nflops / nbytes * HBM_PEAK_GBPS / 1e3 / MFMA_F16_PEAK_TFLOPS, 4),
                         "parity_ok": ok})
            if name == "auto":
                auto_us[B] = us
    del Wl, Wl0, Wd
    torch.cuda.empty_cache()

    # matrix-core rate with the weights in the last-level cache: a 128 MiB column slice of the same matrix
    Ns = 8192
    Ws = np.ascontiguousarray(W[:, :Ns])
    Wls0 = sb.layout_weights(torch.from_numpy(Ws).to(dev))
    Wls = [Wls0] + [Wls0.clone() for _ in range(5)]
    bs_d = torch.from_numpy(np.ascontiguousarray(bias[:Ns])).to(dev)
    sspec = wl.GemmSpec("ffn1_slice", K, Ns, wl.BIAS_GELU)
    warm = []
    for B in [b for b in (1, 16, 32, 64) if b <= Bmax]:
        Xd = torch.from_numpy(np.ascontiguousarray(X[:B])).to(dev)
        Yd = torch.empty((B, Ns), dtype=torch.float16, device=dev)
        ws2 = sb.new_workspace(max(sb.workspace_bytes(B, K, Ns), 256), dev)
        res = {}
        for label, ncopy in (("cold", 6), ("warm", 1)):
            def call():
                sb.gemm(Wls[n[0] % ncopy], K, Ns, Xd, bs_d, None, "bias_gelu", out=Yd, workspace=ws2)
                n[0] += 1
            for _ in range(5):
                call()
            res[label] = _median_us(torch, call, reps=20)
        nbytes, nflops = sspec.algorithmic_bytes(B), sspec.flops(B)
        warm.append({"B": B, "us_cold": round(res["cold"], 2), "us_warm": round(res["warm"], 2),
                     "GBps_cold": round(nbytes / res["cold"] / 1e3, 1), "GBps_warm": round(nbytes / res["warm"] / 1e3, 1),
                     "TFLOPs_cold": round(nflops / res["cold"] / 1e6, 1), "TFLOPs_warm": round(nflops / res["warm"] / 1e6, 1),
                     "mfma_frac_cold": round(nflops / res["cold"] / 1e6 / MFMA_F16_PEAK_TFLOPS, 4),
                     "mfma_frac_warm": round(nflops / res["warm"] / 1e6 / MFMA_F16_PEAK_TFLOPS, 4),
                     # what HBM alone allows at this batch: flops per algorithmic byte x the 8 TB/s peak
                     "hbm_ceiling_TFLOPs": round(nflops / nbytes * HBM_PEAK_GBPS / 1e3, 1),
                     "hbm_ceiling_mfma_frac": round(nflops / nbytes * HBM_PEAK_GBPS / 1e3 / MFMA_F16_PEAK_TFLOPS, 4)})
    total_bytes = sum(spec.algorithmic_bytes(B) for B in batches)
    total_us = sum(auto_us[B] for B in batches)
    dom = max(batches)
    print(json.dumps({
        "metric": "weight-stream HBM GB/s over the batch crossover sweep (dispatcher's picks) and us per GeMM per path",
        "value": round(total_bytes / total_us / 1e3, 1), "unit": "GB/s", "n_gpus": 1, "steps": 50, "warmup": 3,
        "ms_per_step": round(total_us / 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"config5:{cfg.name} [8192,32768] + bias + GeLU, 1 % of input channels x 50, B in {list(batches)}, "
                               "3 weight copies in rotation (1.5 GiB); every path per batch"},
        "roofline": {"bound": "hbm", "achieved": round(spec.algorithmic_bytes(dom) / auto_us[dom] / 1e3, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(spec.algorithmic_bytes(dom) / auto_us[dom] / 1e3 / HBM_PEAK_GBPS, 4),
                     "traffic": None, "kernel": f"dispatcher's pick at B={dom}", "avg_launch_us": round(auto_us[dom], 2)},
        "cpu_baseline": None, "per_case": rows, "cache_resident_slice_8192x8192": warm}))


def split_cost_main(args):
    """--split-cost: what the cross-block split-K hand-over costs.  One JSON line."""
    import numpy as np
    dev_lib = os.path.join(ROOT, "paper_2207_00032_amd", "libsbi_gemm_dev.so")
    assert os.path.exists(dev_lib), "build the measurement library first: python paper_2207_00032_amd/csrc/build.py --dev"
    os.environ["SBI_GEMM_LIB"] = dev_lib
    import torch
    from paper_2207_00032_amd import binding as sb
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev).manual_seed(0)
    ws = sb.new_workspace(64 << 20, dev)
    trace = torch.zeros(8 * 16384, dtype=torch.int64, device=dev)
    pct = lambda a: [round(float(np.percentile(a, q)), 2) for q in (0, 10, 50, 90, 100)]
    rows = []
    for K, N, S in ((4096, 49152, 1), (16384, 12288, 2), (16384, 12288, 4)):
        W = (torch.randn(K, N, device=dev, generator=g) * 0.02).half()
        Wl = [sb.layout_weights(W)]
        del W
        Wl += [Wl[0].clone() for _ in range(2)]
        X = torch.randn(1, K, device=dev, generator=g).half()
        Y = torch.empty(1, N, dtype=torch.float16, device=dev)
        for waves, depth in ((4, 4), (8, 2)):
            n = [0]

            def call():
                sb.gemm(Wl[n[0] % 3], K, N, X, None, None, "none", out=Y, workspace=ws, path=sb.PATH_MFMA,
                        split_k=S, waves=waves, depth=depth)
                n[0] += 1
            pl = sb.plan(1, K, N, sb.PATH_MFMA, split_k=S, waves=waves, depth=depth)
            for _ in range(5):
                call()
            us = _median_us(torch, call, reps=20)
            os.environ["SBI_TRACE_PTR"] = hex(trace.data_ptr())
            call()
            torch.cuda.synchronize()
            os.environ.pop("SBI_TRACE_PTR", None)
            t = trace.cpu().numpy().reshape(-1, 8)[:pl["grid"]].astype(np.int64)
            t0 = t[:, 0].min()
            col = lambda c: (t[:, c] - t0) / 100.0                  # 100 MHz counter -> microseconds
            rows.append({"K": K, "N": N, "split_k": S, "waves": waves, "depth": depth, "grid": pl["grid"],
                         "ksteps_per_block": pl["ksteps_per_split"], "us_per_launch": round(us, 2),
                         "span_us": round(float(col(2).max()), 2), "percentiles": "min p10 p50 p90 max",
                         "x_staged": pct(col(5)), "last_wave_stream_done": pct(col(4)), "block_end": pct(col(2)),
                         "end_minus_last_wave": pct(col(2) - col(4))})
        del Wl
    print(json.dumps({"split_cost": rows, "workload": "384 MiB of fp16 weights as one GeMM, B = 1, no epilogue, 3 copies in rotation"}))


def single_timeline_main(args):
    """--single-timeline: where the time of a single sbi_gemm launch goes.  One JSON line."""
    import numpy as np
    dev_lib = os.path.join(ROOT, "paper_2207_00032_amd", "libsbi_gemm_dev.so")
    assert os.path.exists(dev_lib), "build the measurement library first: python paper_2207_00032_amd/csrc/build.py --dev"
    os.environ["SBI_GEMM_LIB"] = dev_lib
    import torch
    from paper_2207_00032_amd import binding as sb
    from paper_2207_00032_amd import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    g = torch.Generator(device=dev).manual_seed(0)
    ws = sb.new_workspace(64 << 20, dev)
    pct = lambda a: [round(float(np.percentile(a, q)), 2) for q in (0, 10, 50, 90, 100)]
    B = 1
    rows = []
    for spec in cfg.gemms:
        K, N = spec.K, spec.N
        W = (torch.randn(K, N, device=dev, generator=g) * 0.02).half()
        Wl = [sb.layout_weights(W)]
        del W
        copies = max(3, -(-(768 << 20) // spec.weight_bytes))        # at least 768 MiB in rotation: cold
        Wl += [Wl[0].clone() for _ in range(copies - 1)]
        X = torch.randn(B, K, device=dev, generator=g).half()
        bias = (torch.randn(N, device=dev, generator=g) * 0.02).half() if "bias" in spec.epilogue else None
        R = torch.randn(B, N, device=dev, generator=g).half() if "residual" in spec.epilogue else None
        Y = torch.empty(B, N, dtype=torch.float16, device=dev)
        n = [0]

        def call():
            sb.gemm(Wl[n[0] % copies], K, N, X, bias, R, spec.epilogue, out=Y, workspace=ws)
            n[0] += 1
        pl = sb.plan(B, K, N)
        for _ in range(2 * copies):
            call()
        us = _median_us(torch, call, reps=20)
        traces = [torch.zeros(8 * pl["grid"], dtype=torch.int64, device=dev) for _ in range(6)]
        for tb in traces:
            os.environ["SBI_TRACE_PTR"] = hex(tb.data_ptr())
            call()
        torch.cuda.synchronize()
        os.environ.pop("SBI_TRACE_PTR", None)
        tm = [tb.cpu().numpy().reshape(-1, 8).astype(np.int64) for tb in traces]
        t = tm[3]
        t0 = t[:, 0].min()
        col = lambda c: (t[:, c] - t0) / 100.0                      # 100 MHz counter -> microseconds
        rows.append({"gemm": spec.name, "K": K, "N": N, "weight_MiB": spec.weight_bytes >> 20, "plan": {k: pl[k] for k in (
                         "waves", "depth", "split_k", "ksteps_per_split", "grid")},
                     "us_per_launch": round(us, 2), "read_time_at_7_TBps_us": round(spec.weight_bytes / 7.0e6, 2),
                     "span_us": [round(float(x[:, 2].max() - x[:, 0].min()) / 100.0, 2) for x in tm],
                     "last_end_to_next_first_start_us": [round(float(b[:, 0].min() - a[:, 2].max()) / 100.0, 2)
                                                         for a, b in zip(tm, tm[1:])],
                     "percentiles": "min p10 p50 p90 max", "block_start": pct(col(0)), "x_staged": pct(col(5)),
                     # (no such mark in a block whose waves take a single round of k-steps)
                     "first_kstep_done": pct(col(6)) if (t[:, 6] > 0).all() else None,
                     "last_wave_stream_done": pct(col(4)), "block_end": pct(col(2)),
                     "end_minus_last_wave": pct(col(2) - col(4))})
        del Wl
    print(json.dumps({"single_timeline": rows, "workload": f"config{args.config}:{cfg.name}, each GeMM a launch of its own, B = 1, "
                      "weights cold (at least 768 MiB of copies in rotation)"}))


def measure_main(args):
    """--read-ceiling, --timeline, --ablate: where the time of the layer launch goes.  One JSON line each."""
    import numpy as np
    if args.timeline or args.ablate:
        dev_lib = os.path.join(ROOT, "paper_2207_00032_amd", "libsbi_gemm_dev.so")
        assert os.path.exists(dev_lib), "build the measurement library first: python paper_2207_00032_amd/csrc/build.py --dev"
        os.environ["SBI_GEMM_LIB"] = dev_lib
    import torch
    from paper_2207_00032_amd import binding as sb
    from paper_2207_00032_amd import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    specs = cfg.gemms
    batches = tuple(int(b) for b in args.batches.split(",")) if args.batches else (1, 8)
    copies = 3
    layer_bytes = sum(s.weight_bytes for s in specs)

    if args.read_ceiling:
        sink = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
        bufs = [torch.randint(0, 255, (layer_bytes,), dtype=torch.uint8, device=dev) for _ in range(copies)]
        n = [0]
        rows = []
        for blocks, waves, depth in ((256, 8, 4), (256, 8, 8), (256, 16, 4), (512, 8, 4), (768, 4, 4), (768, 4, 8), (768, 8, 4),
                                     (1024, 4, 4), (1536, 4, 4)):
            for nt in (1, 0):
                def call():
                    sb.calib_read(bufs[n[0] % copies], sink, blocks, waves, depth, bool(nt))
                    n[0] += 1
                for _ in range(3):
                    call()
                us = _median_us(torch, call, reps=20)
                rows.append({"blocks": blocks, "waves": waves, "depth": depth, "nontemporal": nt, "us": round(us, 2),
                             "GBps": round(layer_bytes / us / 1e3, 1), "hbm_frac": round(layer_bytes / us / 1e3 / HBM_PEAK_GBPS, 4)})
        best = min(rows, key=lambda r: r["us"])
        # the same read from the last-level cache: one buffer read again and again ("same") against buffers in
        # rotation (at least 1 GiB of them), 768 blocks x 8 waves x 4 deep, non-temporal and ordinary loads
        del bufs
        sizes = []
        for mib in (64, 128, 256, 384):
            many = [torch.randint(0, 255, (mib << 20,), dtype=torch.uint8, device=dev) for _ in range(max(2, -(-1024 // mib)))]
            for nt in (1, 0):
                us = {}
                for mode in ("same", "rotating"):
                    def call():
                        sb.calib_read(many[n[0] % len(many)] if mode == "rotating" else many[0], sink, 768, 8, 4, bool(nt))
                        n[0] += 1
                    for _ in range(3):
                        call()
                    us[mode] = _median_us(torch, call, reps=20)
                sizes.append({"MiB": mib, "nontemporal": nt, "us_same_buffer": round(us["same"], 2),
                              "GBps_same_buffer": round((mib << 20) / us["same"] / 1e3, 1),
                              "us_rotating": round(us["rotating"], 2), "GBps_rotating": round((mib << 20) / us["rotating"] / 1e3, 1)})
            del many
        print(json.dumps({"read_ceiling": {"bytes": layer_bytes, "copies_in_rotation": copies, "best": best, "rows": rows,
                                           "cache_resident_against_rotating": sizes}}))
        return

    # seeded random weights of the configuration's shapes (values do not matter for timing; parity is not checked here)
    g = torch.Generator(device=dev).manual_seed(0)
    Wl0 = [sb.layout_weights((torch.randn(s.K, s.N, device=dev, generator=g) * 0.02).half()) for s in specs]
    Wl = [Wl0] + [[w.clone() for w in Wl0] for _ in range(copies - 1)]
    bias = [(torch.randn(s.N, device=dev, generator=g) * 0.02).half() for s in specs]
    use_bias = [s.epilogue in (wl.BIAS, wl.BIAS_GELU, wl.BIAS_RESIDUAL) for s in specs]
    layers = [sb.make_layer(*Wl[c], specs[0].K, specs[0].N, specs[1].K, specs[2].N, specs[3].K,
                            bqkv=bias[0] if use_bias[0] else None, bout=bias[1] if use_bias[1] else None,
                            bffn1=bias[2] if use_bias[2] else None, bffn2=bias[3] if use_bias[3] else None,
                            ffn1_gelu=specs[2].epilogue in (wl.BIAS_GELU, wl.GELU)) for c in range(copies)]
    ws = sb.new_workspace(64 << 20, dev)
    trace = torch.zeros(8 * 16384, dtype=torch.int64, device=dev)
    out = []
    for B in batches:
        X = [torch.randn(B, s.K, device=dev, generator=g).half() for s in specs]
        R = torch.randn(B, specs[3].N, device=dev, generator=g).half() if specs[3].epilogue in (wl.BIAS_RESIDUAL, wl.RESIDUAL) else None
        Y = [torch.empty(B, s.N, dtype=torch.float16, device=dev) for s in specs]
        n = [0]

        def call():
            sb.layer_gemms(layers[n[0] % copies], B, X[0], X[1], X[2], X[3], R, Y[0], Y[1], Y[2], Y[3], ws)
            n[0] += 1

        plans, grid = sb.layer_plan(layers[0], B)
        plan = {"grid": grid, "waves": plans[0]["waves"], "depth": plans[0]["depth"],
                "split_k": [p["split_k"] for p in plans], "ksteps_per_block": [p["ksteps_per_split"] for p in plans]}
        if args.ablate:
            res = {}
            for mask, name in ((0, "full kernel"), (1, "no matrix-core work"), (8, "no operand reads from LDS"), (2, "no X staging"),
                               (4, "no reduction, no epilogue"), (6, "no X staging, no reduction, no epilogue"),
                               (15, "weight stream only")):
                os.environ["SBI_ABLATE"] = str(mask)
                for _ in range(3):
                    call()
                res[name] = round(_median_us(torch, call, reps=20), 2)
            os.environ.pop("SBI_ABLATE", None)
            out.append({"B": B, "plan": plan, "us": res})
            continue
        for _ in range(5):
            call()
        us = _median_us(torch, call, reps=20)
        os.environ["SBI_TRACE_PTR"] = hex(trace.data_ptr())
        call()
        torch.cuda.synchronize()
        os.environ.pop("SBI_TRACE_PTR", None)
        t = trace.cpu().numpy().reshape(-1, 8)[:grid].astype(np.int64)
        # six launches back to back, each into a trace buffer of its own: how far apart they run
        more = [torch.zeros(8 * grid, dtype=torch.int64, device=dev) for _ in range(6)]
        for tb in more:
            os.environ["SBI_TRACE_PTR"] = hex(tb.data_ptr())
            call()
        torch.cuda.synchronize()
        os.environ.pop("SBI_TRACE_PTR", None)
        tm = [tb.cpu().numpy().reshape(-1, 8).astype(np.int64) for tb in more]
        back_to_back = {"span_us": [round(float(x[:, 2].max() - x[:, 0].min()) / 100.0, 2) for x in tm],
                        "last_end_to_next_first_start_us": [round(float(b[:, 0].min() - a[:, 2].max()) / 100.0, 2)
                                                            for a, b in zip(tm, tm[1:])],
                        "first_start_to_next_first_start_us": [round(float(b[:, 0].min() - a[:, 0].min()) / 100.0, 2)
                                                               for a, b in zip(tm, tm[1:])]}
        t0 = t[:, 0].min()
        col = lambda c: (t[:, c] - t0) / 100.0                      # 100 MHz counter -> microseconds
        start, stream0, end, last, xst, first = col(0), col(1), col(2), col(4), col(5), col(6)
        slot = t[:, 3] >> 32
        pct = lambda a: [round(float(np.percentile(a, q)), 2) for q in (0, 10, 50, 90, 100)]
        out.append({"B": B, "plan": plan, "us_per_launch_untraced": round(us, 2), "span_us": round(float(end.max()), 2),
                    "back_to_back": back_to_back,
                    "percentiles": "min p10 p50 p90 max",
                    "block_start": pct(start), "x_staged": pct(xst), "first_kstep_done": pct(first),
                    "wave0_stream_done": pct(stream0), "last_wave_stream_done": pct(last), "block_end": pct(end),
                    "end_minus_last_wave": pct(end - last),
                    "per_problem_slot": [{"slot": int(k), "blocks": int((slot == k).sum()),
                                          "last_wave_stream_done_p50": round(float(np.median(last[slot == k])), 2),
                                          "last_wave_stream_done_max": round(float(last[slot == k].max()), 2),
                                          "block_end_max": round(float(end[slot == k].max()), 2)}
                                         for k in sorted(set(slot.tolist()))],
                    "blocks_done_streaming_by_us": {str(q): round(float(np.quantile(last, q / 100)), 2) for q in (50, 80, 90, 95, 99)}})
    print(json.dumps({"ablation" if args.ablate else "timeline": out, "workload": f"config{args.config}:{cfg.name} layer launch, "
                      f"{copies} weight copies in rotation"}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.attention:
        return attention_main(args)
    if args.decoder_layer:
        return decoder_main(args)
    if args.config == 5:
        return crossover_main(args)
    if args.split_cost:
        return split_cost_main(args)
    if args.single_timeline:
        return single_timeline_main(args)
    if args.read_ceiling or args.timeline or args.ablate:
        return measure_main(args)

    import numpy as np
    import torch
    from paper_2207_00032_amd import binding as sb
    from paper_2207_00032_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sb.load()
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    assert len(cfg.gemms) == 4, "bench.py times a four-GeMM layer configuration"
    batches = tuple(int(b) for b in args.batches.split(",")) if args.batches else cfg.batches
    # the rows beyond the headline workload: only with the default command (config 2, automatic dispatch)
    extras = (not args.no_extra and args.config == 2 and not args.batches and args.path == "auto"
              and not args.layernorm and not args.int8 and not args.graph and not args.pmc_probe)
    row_batches = batches + ((16,) if extras else ())          # batches that get a per-launch row
    Bmax = max(row_batches)
    specs = cfg.gemms
    layer_weight_bytes = sum(s.weight_bytes for s in specs) // (2 if args.int8 else 1)
    copies = args.copies or max(3, -(-3 * 256 * 1000 * 1000 // layer_weight_bytes))

    # ---- seeded synthetic inputs (host), uploaded and laid out once ------------------------
    # (drawn for the largest batch of THIS run: --batches may go beyond the configuration's own sweep)
    host = []
    for gi, s in enumerate(specs):
        W, bias, X, R = wl.make_gemm_inputs(s.K, s.N, Bmax, 0, args.config, gi, cfg.outlier_channels,
                                            cfg.outlier_scale)
        assert X.shape == (Bmax, s.K) and R.shape == (Bmax, s.N)
        host.append((W, bias, X, R))
    LN_EPS = 1e-5
    ln_host = None
    if args.layernorm:
        assert args.path == "auto", "--layernorm runs through sbi_layer_gemms"
        # the inputs of QKV and FFN1 become residual-stream rows (own mean and spread per row)
        ln_host = {gi: wl.make_layernorm_inputs(specs[gi].K, Bmax, seed=0, config_id=args.config, gemm_id=gi)
                   for gi in (0, 2)}
        for gi in (0, 2):
            W, bias, _, R = host[gi]
            host[gi] = (W, bias, ln_host[gi][2], R)
    use_bias = [s.epilogue in (wl.BIAS, wl.BIAS_GELU, wl.BIAS_RESIDUAL) for s in specs]
    use_res = specs[3].epilogue in (wl.BIAS_RESIDUAL, wl.RESIDUAL)
    gelu = specs[2].epilogue in (wl.BIAS_GELU, wl.GELU)

    scales_d = None
    if args.int8:
        assert args.path == "auto", "--int8 runs through sbi_layer_gemms"
        prepared = [sb.i8_quantize_weights(torch.from_numpy(h[0]).to(dev)) for h in host]
        Wl0 = [sb.i8_layout_weights(q) for q, _ in prepared]
        scales_d = [sc for _, sc in prepared]
        Wq_host = [q.cpu().numpy() for q, _ in prepared]          # codes and scales for the oracle leg
        sw_host = [sc.cpu().numpy() for sc in scales_d]
        del prepared
        for w, s in zip(Wl0, specs):
            assert sb.i8_layout_check(w, s.K, s.N) == 0
    else:
        Wl0 = [sb.layout_weights(torch.from_numpy(h[0]).to(dev)) for h in host]
        for w, s in zip(Wl0, specs):
            assert sb.layout_check(w, s.K, s.N) == 0
    Wl = [Wl0] + [[w.clone() for w in Wl0] for _ in range(copies - 1)]
    bias_d = [torch.from_numpy(h[1]).to(dev) if ub else None for h, ub in zip(host, use_bias)]
    X_d = {B: [torch.from_numpy(np.ascontiguousarray(h[2][:B])).to(dev) for h in host] for B in row_batches}
    R_d = {B: torch.from_numpy(np.ascontiguousarray(host[3][3][:B])).to(dev) if use_res else None for B in row_batches}
    Y_d = {B: [torch.empty((B, s.N), dtype=torch.float16, device=dev) for s in specs] for B in row_batches}
    h_dim = specs[0].K
    layers = [sb.make_layer(*Wl[c], h_dim, specs[0].N, specs[1].K, specs[2].N, specs[3].K,
                            bqkv=bias_d[0], bout=bias_d[1], bffn1=bias_d[2], bffn2=bias_d[3], ffn1_gelu=gelu,
                            scales=scales_d)
              for c in range(copies)]
    plain_layers = layers
    if args.layernorm:
        ln_d = {gi: (torch.from_numpy(ln_host[gi][0]).to(dev), torch.from_numpy(ln_host[gi][1]).to(dev))
                for gi in (0, 2)}
        layers = [sb.make_layer(*Wl[c], h_dim, specs[0].N, specs[1].K, specs[2].N, specs[3].K,
                                bqkv=bias_d[0], bout=bias_d[1], bffn1=bias_d[2], bffn2=bias_d[3], ffn1_gelu=gelu,
                                ln1=ln_d[0], ln2=ln_d[2], ln_eps=LN_EPS, scales=scales_d) for c in range(copies)]
    ws = sb.new_workspace(max([64 << 20] + [sb.layer_workspace_bytes(layers[0], B) for B in row_batches] +
                              [sb.layer_workspace_bytes(plain_layers[0], B) for B in row_batches] +
                              [sb.plan(B, s.K, s.N, int8=args.int8)["workspace_bytes"] for B in row_batches for s in specs]),
                          dev)
    path = {"auto": sb.PATH_AUTO, "stream": sb.PATH_STREAM, "mfma": sb.PATH_MFMA,
            "streamk": sb.PATH_STREAMK}[args.path]

    # ---- launch plans measured once at set-up (untimed), as at model load ---------------------
    tuned = {}
    if not args.no_tune and path == sb.PATH_AUTO and not args.pmc_probe:
        for B in row_batches:
            x, y = X_d[B], Y_d[B]
            tuned[f"layer B={B}"] = sb.layer_tune(layers, B, x[0], x[1], x[2], x[3], R_d[B], y[0], y[1], y[2], y[3], ws)
        if (args.per_gemm or extras) and not args.int8 and not args.layernorm:
            for B in (batches if args.per_gemm else (1, 8)):
                for gi, s in enumerate(specs):
                    tuned[f"single:{s.name} B={B}"] = sb.gemm_tune(
                        [Wl[c][gi] for c in range(copies)], s.K, s.N, X_d[B][gi], bias_d[gi], R_d[B] if gi == 3 else None,
                        s.epilogue, out=Y_d[B][gi], workspace=ws)

    launch_no = [0]

    def next_copy():
        """Every launch streams a different weight copy than the one before it."""
        c = launch_no[0] % copies
        launch_no[0] += 1
        return c

    def launch_layer(B):
        x, y = X_d[B], Y_d[B]
        c = next_copy()
        if path == sb.PATH_AUTO:
            sb.layer_gemms(layers[c], B, x[0], x[1], x[2], x[3], R_d[B], y[0], y[1], y[2], y[3], ws)
        else:
            for gi, s in enumerate(specs):
                sb.gemm(Wl[c][gi], s.K, s.N, x[gi], bias_d[gi], R_d[B] if gi == 3 else None, s.epilogue,
                        out=y[gi], workspace=ws, path=path)

    def eager_step(i):
        for B in batches:
            launch_layer(B)

    step = eager_step

    if args.pmc_probe:
        # known-traffic reference (reads 256 MiB, writes 256 MiB), then the layer launches
        src = torch.randint(0, 255, (256 << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            sb.calib_copy(src, dst)
        for i in range(4):
            step(i)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "copy_bytes": 256 << 20, "batches": list(batches),
                          "layer_bytes": {str(B): sum(s.algorithmic_bytes(B, args.int8) for s in specs) for B in batches}}))
        return

    # ---- timed region: K steps, one event per step boundary on the launch stream -------------
    for i in range(args.warmup):
        step(i)
    per_mark = 1                               # steps between two event marks
    if args.graph:
        per_mark = args.graph
        args.steps = max(per_mark, args.steps // per_mark * per_mark)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for j in range(per_mark):
                    eager_step(j)
        torch.cuda.synchronize()
        for _ in range(2):
            graph.replay()
    nmarks = args.steps // per_mark
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(nmarks + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(nmarks):
        if args.graph:
            graph.replay()
        else:
            step(args.warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps
    bytes_per_step = sum(s.algorithmic_bytes(B, args.int8) for B in batches for s in specs)
    flops_per_step = sum(s.flops(B) for B in batches for s in specs)
    value = bytes_per_step / sec_per_step / 1e9
    # dominant kernel: with the automatic dispatch a step is len(batches) launches of it, back to back
    step_us = [marks[i].elapsed_time(marks[i + 1]) * 1e3 / per_mark for i in range(nmarks)]
    launches_per_step = len(batches) * (1 if path == sb.PATH_AUTO else len(specs))
    avg_launch_us = sum(step_us) / len(step_us) / launches_per_step

    # ---- per-batch launch times: events around runs of 10 back-to-back launches of one B ------
    per_launch = []
    def timed_run(label, B, nbytes, nflops, fn, reps=10, runs=5):
        us = []
        for _ in range(runs):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us.append(e0.elapsed_time(e1) * 1e3 / reps)
        med = sorted(us)[len(us) // 2]
        per_launch.append({"launch": label, "B": B, "us_median": round(med, 2),
                           "GBps": round(nbytes / (med * 1e-6) / 1e9, 1),
                           "hbm_frac": round(nbytes / (med * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                           "TFLOPs": round(nflops / (med * 1e-6) / 1e12, 3)})

    for B in row_batches:
        timed_run("layer", B, sum(s.algorithmic_bytes(B, args.int8) for s in specs), sum(s.flops(B) for s in specs),
                  lambda: launch_layer(B))
    if args.layernorm:
        # the unfused alternative: the two norms as kernels of their own (torch's), then the plain layer
        Xn_d = {B: [torch.empty_like(X_d[B][0]), torch.empty_like(X_d[B][2])] for B in batches}

        def launch_unfused(B):
            x, y = X_d[B], Y_d[B]
            c = next_copy()
            for j, gi in enumerate((0, 2)):
                Xn_d[B][j].copy_(torch.nn.functional.layer_norm(x[gi], (h_dim,), ln_d[gi][0], ln_d[gi][1], LN_EPS))
            sb.layer_gemms(plain_layers[c], B, Xn_d[B][0], x[1], Xn_d[B][1], x[3], R_d[B],
                           y[0], y[1], y[2], y[3], ws)

        for B in batches:
            timed_run("layer, norms as separate torch kernels", B, sum(s.algorithmic_bytes(B, args.int8) for s in specs),
                      sum(s.flops(B) for s in specs), lambda: launch_unfused(B))
    ceiling = None
    if extras:
        # the same weights on every launch ("warm"): 384 MiB do not fit the 256 MB last-level cache, so this
        # row says how much of the rotation's effect is cache and how much is address translation
        B0 = batches[0]
        x, y = X_d[B0], Y_d[B0]
        timed_run("layer, same weight copy every launch (warm)", B0, sum(s.algorithmic_bytes(B0) for s in specs),
                  sum(s.flops(B0) for s in specs),
                  lambda: sb.layer_gemms(layers[0], B0, x[0], x[1], x[2], x[3], R_d[B0], y[0], y[1], y[2], y[3], ws))
        # pure streaming read of the layer's weight bytes with the weight stream's access shape (non-temporal
        # 128-bit loads, 768 blocks x 8 waves x 4 deep, the best shape of bench.py --read-ceiling), rotating over
        # the same copies: the calibrated ceiling beside the 8 TB/s data-sheet peak
        sink = torch.zeros(1 << 16, dtype=torch.uint8, device=dev)
        flat = [torch.cat([w.view(torch.uint8).reshape(-1)[256:256 + sp.weight_bytes] for w, sp in zip(Wl[c], specs)])
                for c in range(copies)]
        k = [0]

        def read_once():
            sb.calib_read(flat[k[0] % copies], sink, 768, 8, 4, True)
            k[0] += 1
        for _ in range(3):
            read_once()
        r_us = _median_us(torch, read_once, reps=20)
        nb = flat[0].numel()
        ceiling = {"us": round(r_us, 2), "bytes": nb, "GBps": round(nb / r_us / 1e3, 1),
                   "frac_of_peak": round(nb / r_us / 1e3 / HBM_PEAK_GBPS, 4), "shape": "768 blocks x 8 waves x 4 deep, non-temporal"}
        del flat
    if (args.per_gemm or extras) and not args.int8:
        # every GeMM as a launch of its own (sbi_gemm): what a caller with dependent GeMMs gets
        for B in (batches if args.per_gemm else (1, 8)):
            for gi, s in enumerate(specs):
                timed_run("single:" + s.name, B, s.algorithmic_bytes(B, args.int8), s.flops(B),
                          lambda: sb.gemm(Wl[next_copy()][gi], s.K, s.N, X_d[B][gi], bias_d[gi],
                                          R_d[B] if gi == 3 else None, s.epilogue, out=Y_d[B][gi],
                                          workspace=ws, path=path))
    Bk = max(batches)                  # the timed region's largest batch names the kernel variant
    pl0 = sb.plan(Bk, specs[0].K, specs[0].N, path)
    if path == sb.PATH_AUTO:
        lp, _ = sb.layer_plan(layers[0], Bk)
        pl0 = lp[0]
    kname = {sb.PATH_STREAMK: "sbi_streamk_kernel", sb.PATH_MFMA: "sbi_mfma_kernel",
             sb.PATH_STREAM: "sbi_stream_kernel"}[pl0["path"]]
    if args.int8:
        kname = "sbi_i8_kernel"
    bytes_per_launch = bytes_per_step / launches_per_step
    achieved = bytes_per_launch / (avg_launch_us * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(args, batches),
                "kernel": f"{kname}<{(Bk + 15) // 16 if pl0['path'] != sb.PATH_STREAM else Bk},"
                          f"{pl0['waves']},{pl0['depth']}>",
                "launches": args.steps * launches_per_step, "avg_launch_us": round(avg_launch_us, 2),
                "avg_bytes_per_launch": round(bytes_per_launch)}

    # ---- CPU oracle on the host cores, same GeMMs (a reported baseline, not a target) -------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        epi_map = {wl.NONE: 0, wl.BIAS: orc.EPI_BIAS, wl.BIAS_GELU: orc.EPI_BIAS | orc.EPI_GELU,
                   wl.BIAS_RESIDUAL: orc.EPI_BIAS | orc.EPI_RES, wl.GELU: orc.EPI_GELU, wl.RESIDUAL: orc.EPI_RES}
        torch.cuda.synchronize()
        for B in row_batches:        # outputs of one more launch per batch for the parity check below
            launch_layer(B)
        torch.cuda.synchronize()
        t_cpu = 0.0
        cpu_bytes = 0
        worst = {"max_abs": 0.0, "n_bad": 0}
        sample_batches = row_batches if layer_weight_bytes < (1 << 30) else (Bmax,)
        for B in sample_batches:
            for gi, s in enumerate(specs):
                W, bias, X, R = host[gi]
                xin = X[:B]
                if gi == 3 and path == sb.PATH_AUTO:
                    xin = X[:B]      # sbi_layer_gemms was given FFN2's own input, not chained
                c0 = time.perf_counter()
                if args.layernorm and gi in (0, 2):
                    xin = orc.layernorm(xin, ln_host[gi][0], ln_host[gi][1], LN_EPS)
                if args.int8:
                    want = orc.gemm_i8_from_fp16(xin, Wq_host[gi], sw_host[gi], bias, R[:B], epi_map[s.epilogue])
                else:
                    want = orc.gemm(xin, W, bias, R[:B], epi=epi_map[s.epilogue])
                t_cpu += time.perf_counter() - c0
                cpu_bytes += s.algorithmic_bytes(B, args.int8)
                ok, rep = orc.check_close(Y_d[B][gi].cpu().numpy(), want)
                worst["max_abs"] = max(worst["max_abs"], rep["max_abs"])
                worst["n_bad"] += rep["n_bad"]
        # the same oracle on ONE host thread, on one GeMM of the sample (QKV at the largest sampled batch)
        W0, b0, X0, R0 = host[0]
        c0 = time.perf_counter()
        if not args.int8:
            orc.gemm(X0[:Bmax], W0, b0, R0[:Bmax], epi=epi_map[specs[0].epilogue], threads=1)
        t_one = time.perf_counter() - c0
        cpu = {"value": round(cpu_bytes / t_cpu / 1e9, 3), "unit": "GB/s", "cores": orc.max_threads(),
               "kind": "oracle",
               "sample": f"{len(sample_batches) * len(specs)} GeMMs (config {args.config}, B in "
                         f"{list(sample_batches)}), {t_cpu:.1f} s of CPU time",
               "value_1_thread": None if args.int8 else round(specs[0].algorithmic_bytes(Bmax) / t_one / 1e9, 3),
               "sample_1_thread": None if args.int8 else f"{specs[0].name} at B={Bmax}, {t_one:.1f} s"}
        parity = {"ok": worst["n_bad"] == 0, "n_bad": worst["n_bad"], "max_abs": worst["max_abs"],
                  "tolerance": "max(2 ulp16, 1e-3)"}

    # ---- the rest of the metric's range (h = 12288): configurations 3 and 4 as layer launches ------
    if extras:
        del Wl, Wl0, layers, plain_layers
        torch.cuda.empty_cache()
        for cid in (3, 4):
            xcfg = wl.CONFIGS[cid]
            xs_ = xcfg.gemms
            xB = max(xcfg.batches)
            xhost = [wl.make_gemm_inputs(s.K, s.N, xB, 0, cid, gi) for gi, s in enumerate(xs_)]
            xbytes = sum(s.weight_bytes for s in xs_)
            ncopy = 1 if xbytes > (1 << 30) else 3            # 3.6 GB of weights are cold by themselves
            xWl0 = [sb.layout_weights(torch.from_numpy(h[0]).to(dev)) for h in xhost]
            xWl = [xWl0] + [[w.clone() for w in xWl0] for _ in range(ncopy - 1)]
            xbias = [torch.from_numpy(h[1]).to(dev) if s.epilogue in (wl.BIAS, wl.BIAS_GELU, wl.BIAS_RESIDUAL) else None
                     for h, s in zip(xhost, xs_)]
            xlayers = [sb.make_layer(*xWl[c], xs_[0].K, xs_[0].N, xs_[1].K, xs_[2].N, xs_[3].K, bqkv=xbias[0], bout=xbias[1],
                                     bffn1=xbias[2], bffn2=xbias[3], ffn1_gelu=xs_[2].epilogue in (wl.BIAS_GELU, wl.GELU))
                       for c in range(ncopy)]
            for B in xcfg.batches:
                xws = sb.new_workspace(max(sb.layer_workspace_bytes(xlayers[0], B), 64 << 20), dev)
                xX = [torch.from_numpy(np.ascontiguousarray(h[2][:B])).to(dev) for h in xhost]
                xY = [torch.empty((B, s.N), dtype=torch.float16, device=dev) for s in xs_]
                k = [0]

                def launch_x():
                    sb.layer_gemms(xlayers[k[0] % ncopy], B, xX[0], xX[1], xX[2], xX[3], None, xY[0], xY[1], xY[2], xY[3], xws)
                    k[0] += 1

                if not args.no_tune:
                    tuned[f"layer config{cid} B={B}"] = sb.layer_tune(xlayers, B, xX[0], xX[1], xX[2], xX[3], None,
                                                                      xY[0], xY[1], xY[2], xY[3], xws)
                for _ in range(2):
                    launch_x()
                timed_run(f"layer config{cid}:{xcfg.name}", B, sum(s.algorithmic_bytes(B) for s in xs_),
                          sum(s.flops(B) for s in xs_), launch_x, reps=5 if ncopy == 1 else 10)
                if not args.no_cpu_baseline:
                    torch.cuda.synchronize()
                    bad = 0
                    for gi, s in enumerate(xs_):
                        want = orc.gemm(xhost[gi][2][:B], xhost[gi][0], xhost[gi][1] if xbias[gi] is not None else None, None,
                                        epi=epi_map[s.epilogue])
                        bad += orc.check_close(xY[gi].cpu().numpy(), want)[1]["n_bad"]
                    per_launch[-1]["parity_ok"] = bad == 0
                    parity["n_bad"] += bad
                    parity["ok"] = parity["n_bad"] == 0
            del xWl, xWl0, xlayers, xhost
            torch.cuda.empty_cache()

    out = {
        "metric": "weight-stream HBM GB/s (algorithmic bytes of the layer's four GeMMs / time)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "i8" if args.int8 else "f16", "data": "synthetic",
        "config": {"workload": f"config{args.config}:{cfg.name} four-GeMM layer, B in {list(batches)}, "
                               f"rotating over {copies} weight copies ({copies * layer_weight_bytes >> 20} MiB)",
                   "batches": list(batches), "weight_copies": copies,
                   "dispatch": args.path + (", plans measured at set-up (sbi_layer_tune / sbi_gemm_tune)" if tuned else ""),
                   "fused_layernorm": bool(args.layernorm), "int8": bool(args.int8),
                   "graph_replay_steps": args.graph},
        "hbm_frac": round(value / HBM_PEAK_GBPS, 4),
        "us_per_gemm_mean": round(sec_per_step * 1e6 / (len(batches) * len(specs)), 2),
        "TFLOPs": round(flops_per_step / sec_per_step / 1e12, 3),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
        "calibrated_read_ceiling": None if ceiling is None else dict(
            ceiling, value_as_frac_of_ceiling=round(value / ceiling["GBps"], 4),
            dominant_kernel_as_frac_of_ceiling=round(roofline["achieved"] / ceiling["GBps"], 4)),
        "per_launch": per_launch,
        "tuned_plans": {k: {"waves": v["waves"], "depth": v["depth"], "panels": v["panels"], "block_ksteps": v["block_ksteps"],
                            "candidates": v["candidates"], "us_best": round(v["us_best"], 2), "us_model": round(v["us_model"], 2)}
                        for k, v in tuned.items()},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
