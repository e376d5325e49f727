#!/usr/bin/env python3
"""Headline benchmark: fused fp16 GEMM C = ReLU(A.B + bias), M = N = K = 4096, on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--dtype f16|bf16] [--k 4096|1024] [--no-cpu-baseline]

One step = one pass of the whole hot path over one batch of synthetic input: block-level task mapping,
cooperative predicated loads, double-buffered LDS staging, MFMA contraction, fused bias+ReLU epilogue and
store -- a single hidet_gemm call.  Inputs are resident in HBM before the timed region.  Tuning (one
enumeration of the schedule space) happens before the warm-up and is reported separately.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f16": 2516.6, "bf16": 2516.6, "f32": 157.3}  # 256 CUs x 4 SIMDs x FLOP/clk x 2.4 GHz (dense MFMA)

# HBM bytes per launch of the dominant kernel, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this very
# command line, each scaled by what the same counter reads for a plain copy of known size (`--copy-calibration`).  The
# counters cannot be read inside a timed run, so the bench line carries the figure of the committed profile together
# with where it came from; shapes without a committed counter run report null.
MEASURED_TRAFFIC = {
    # (dtype, M, N, K): (bytes per launch, profile that holds the counter run)
    ("f16", 4096, 4096, 4096): (235409564, "profiles/gemm_pingpong_f16_4096.md"),
    ("f16", 4096, 4096, 1024): (84428443, "profiles/gemm_pingpong_f16_4096x4096x1024.md"),
    ("bf16", 4096, 4096, 4096): (235411612, "profiles/gemm_pingpong_bf16_4096_and_1024.md"),
    ("bf16", 4096, 4096, 1024): (84430490, "profiles/gemm_pingpong_bf16_4096_and_1024.md"),
}


def graph_time(torch, fn, reps=20, replays=10):
    """Microseconds per call of fn, replayed from a HIP graph (reps calls per graph, `replays` replays)."""
    fn()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for _ in range(reps):
                fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1000.0 / (reps * replays)


def side_report(torch, hb, wl, steps=200):
    """Time the other workloads with the tuner (every configuration of the space, `steps` launches each, winner reported):
    list of dicts with us, TFLOP/s, % of peak MFMA and algorithmic GB/s."""
    import numpy as np
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}

    def dev(stored, dt):
        if stored is None:
            return None
        if dt == "bf16":
            return torch.from_numpy(np.ascontiguousarray(stored).view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(np.ascontiguousarray(stored)).cuda()

    ws = torch.empty(16 << 20, dtype=torch.float32, device="cuda")  # 64 MiB: 16 K-slices of a 2^20-element output

    def timed(fn, tune, tune_sliced=None, out_elems=0):
        # timed inside the library (a tight C++ launch loop between two HIP events): a Python call per
        # launch costs more than these small kernels run
        t0 = time.perf_counter()
        cfg, us = tune()
        tune_s = time.perf_counter() - t0
        sliced = None
        if tune_sliced is not None and out_elems <= (1 << 20):
            # parallel reduction on K pays only when the output has few tiles; both kernels (partial sums and
            # reduce + epilogue) are inside the timed launches
            sliced = tune_sliced()
        return us, cfg, tune_s, sliced

    rows = [{"workload": "empty_kernel_launch_floor", "dtype": "-", "us": round(hb.hidet_probe_launch_floor(2000), 2)}]

    def cold(call, tensors, nbytes):
        """Microseconds per call when every call finds its operands in HBM only: the call walks over enough copies of
        its operand set to exceed the 256 MB Infinity Cache twice (unsliced kernel, tuned tile, replayed from a graph)."""
        n = max(2, min(256, int(600e6 // max(nbytes, 1)) + 1))
        sets = [[t.clone() for t in tensors] for _ in range(n)]

        def sweep():
            for ts in sets:
                call(*ts)
        return graph_time(torch, sweep, reps=1, replays=10) / n

    def add(name, dt, flops, nbytes, us, cfg, tune_s, sliced=None, us_cold=None):
        unsliced_us = us
        slices = 1
        if sliced is not None and sliced[2] < us:
            cfg, slices, us = sliced
        info = hb.hidet_config_info(cfg)
        rows.append({"workload": name, "dtype": dt, "us": round(us, 2), "k_slices": slices,
                     "us_unsliced": round(unsliced_us, 2), "TFLOPs": round(flops / us * 1e-6, 2),
                     "pct_peak_mfma": round(100 * flops / us * 1e-6 / PEAK_TFLOPS[dt], 2),
                     "algorithmic_GBps": round(nbytes / us * 1e-3, 1), "pct_of_8TBps": round(100 * nbytes / us * 1e-3 / 8000, 2),
                     "tile_config": cfg, "tile": "%dx%dx%d/%dx%d/mfma%d" % (info["block_m"], info["block_n"], info["block_k"],
                                                                            info["waves_m"], info["waves_n"], info["mfma"]),
                     "tuning_seconds": round(tune_s, 3)})
        if us_cold is not None:
            rows[-1]["us_cold_unsliced"] = round(us_cold, 2)

    def gemm_row(c):
        dt = c["dtype"]
        es = 4 if dt == "f32" else 2
        A, B = dev(c["A"], dt), dev(c["B"], dt)
        bias, res = dev(c["bias"], dt), dev(c["residual"], dt)
        C = torch.empty((c["M"], c["N"]), dtype=tdt[dt], device="cuda")
        axis = {None: hb.HIDET_BIAS_NONE, "col": hb.HIDET_BIAS_PER_COL, "row": hb.HIDET_BIAS_PER_ROW}[c["bias_axis"]]
        epi = hb.make_epilogue(alpha=c.get("alpha", 1.0), bias=bias, bias_axis=axis, residual=res, relu=c.get("relu", False))
        us, cfg, ts, sl = timed(lambda cfg: hb.hidet_gemm(A, B, C, epilogue=epi, config=cfg),
                                lambda: hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=steps),
                                lambda: hb.hidet_tune_gemm_splitk(A, B, C, ws, epilogue=epi, iters=steps), c["M"] * c["N"])
        nbytes = (c["M"] * c["K"] + c["K"] * c["N"] + c["M"] * c["N"] * (2 if res is not None else 1)) * es
        uc = None
        if nbytes < (64 << 20):  # the small, bandwidth- or latency-bound workloads
            uc = cold(lambda a, b_, c_: hb.hidet_gemm(a, b_, c_, epilogue=epi, config=cfg), [A, B, C], nbytes)
        add(c["name"], dt, 2.0 * c["M"] * c["N"] * c["K"], nbytes, us, cfg, ts, sl, uc)

    for c in wl.config1():
        gemm_row(c)
    for dt in ("f16", "bf16"):
        for c in wl.config2(dt):
            gemm_row(c)
    for c in wl.config3("f16"):
        x, w, b = dev(c["x"], "f16"), dev(c["w"], "f16"), dev(c["bias"], "f16")
        y = torch.empty((c["Nb"], c["OC"], c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(bias=b, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
        sp = dict(stride=(c["stride"], c["stride"]), pad=(c["pad"], c["pad"]))
        us, cfg, ts, sl = timed(lambda cfg: hb.hidet_conv2d_implicit_gemm(x, w, y, epilogue=epi, config=cfg, **sp),
                                lambda: hb.hidet_tune_conv2d(x, w, y, epilogue=epi, iters=steps, **sp),
                                lambda: hb.hidet_tune_conv2d_splitk(x, w, y, ws, epilogue=epi, iters=steps, **sp), y.numel())
        flops = 2.0 * c["Nb"] * c["OC"] * c["OH"] * c["OW"] * c["IC"] * c["KH"] * c["KW"]
        nbytes = (x.numel() + w.numel() + y.numel()) * 2
        # (no configuration named: the call runs what the tuner remembered, which for the 1x1 layers may be the
        # batched-GEMM form)
        uc = cold(lambda x_, w_, y_: hb.hidet_conv2d_implicit_gemm(x_, w_, y_, epilogue=epi, **sp), [x, w, y], nbytes)
        add(c["name"], "f16", flops, nbytes, us, cfg, ts, sl, uc)
    for c in wl.config4("f16"):
        Q, Kt, V, S = (dev(c[k], "f16") for k in ("Q", "K", "V", "S"))
        b, s, d = c["batch"], c["seq"], c["d"]
        scores = torch.empty((b, s, s), dtype=torch.float16, device="cuda")
        ctx = torch.empty((b, s, d), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(alpha=c["alpha"])
        us, cfg, ts, _ = timed(lambda cfg: hb.hidet_batched_gemm(Q, Kt, scores, transB=True, epilogue=epi, config=cfg),
                               lambda: hb.hidet_tune_gemm(Q, Kt, scores, transB=True, epilogue=epi, iters=steps))
        nbytes = (2 * b * s * d + b * s * s) * 2
        uc = cold(lambda q_, k_, o_: hb.hidet_batched_gemm(q_, k_, o_, transB=True, epilogue=epi, config=cfg),
                  [Q, Kt, scores], nbytes)
        add(c["name"] + "_QKt", "f16", 2.0 * b * s * s * d, nbytes, us, cfg, ts, None, uc)
        us, cfg, ts, _ = timed(lambda cfg: hb.hidet_batched_gemm(S, V, ctx, config=cfg),
                               lambda: hb.hidet_tune_gemm(S, V, ctx, iters=steps))
        uc = cold(lambda s_, v_, o_: hb.hidet_batched_gemm(s_, v_, o_, config=cfg), [S, V, ctx], nbytes)
        add(c["name"] + "_SV", "f16", 2.0 * b * s * s * d, nbytes, us, cfg, ts, None, uc)
    for dt in ("f16", "bf16"):
        for K in (4096, 1024):
            gemm_row(wl.config5(dt, K=K))

    # reduction template: row softmax over the attention scores (memory bound: one read, one write), then the
    # whole attention chain (scaled Q.K^T, softmax in place, S.V).  Launches are replayed from a HIP graph so that
    # the Python call overhead stays out of the timing.
    for c in wl.config4("f16"):
        Q, Kt, V = (dev(c[k], "f16") for k in ("Q", "K", "V"))
        b, s, d = c["batch"], c["seq"], c["d"]
        scores = torch.empty((b, s, s), dtype=torch.float16, device="cuda")
        ctx = torch.empty((b, s, d), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(alpha=c["alpha"])
        hb.hidet_batched_gemm(Q, Kt, scores, transB=True, epilogue=epi)
        us = graph_time(torch, lambda: hb.hidet_softmax_rows(scores, scores))
        nbytes = 2 * scores.numel() * 2
        rows.append({"workload": c["name"] + "_softmax", "dtype": "f16", "us": round(us, 2), "bound": "hbm",
                     "algorithmic_GBps": round(nbytes / us * 1e-3, 1), "pct_of_8TBps": round(100 * nbytes / us * 1e-3 / 8000, 2)})

        def chain():
            hb.hidet_batched_gemm(Q, Kt, scores, transB=True, epilogue=epi)
            hb.hidet_softmax_rows(scores, scores)
            hb.hidet_batched_gemm(scores, V, ctx)
        us = graph_time(torch, chain)
        flops = 4.0 * b * s * s * d
        rows.append({"workload": c["name"] + "_attention_3_kernels", "dtype": "f16", "us": round(us, 2),
                     "TFLOPs": round(flops / us * 1e-6, 2), "pct_peak_mfma": round(100 * flops / us * 1e-6 / PEAK_TFLOPS["f16"], 2)})
    return rows


def other_workload(torch, hb, wl, which, steps, warmup, graph_replay=False, cold=False):
    """One of the secondary kernels on its own, K steps after W warm-up steps, so that a profiler sees nothing else:
    "softmax" = row softmax over the scores of the largest attention case (memory bound), "conv" = the case-study
    convolution with its tuned (tile, K-slice) choice (two kernels per step when K is sliced), "conv64" = a
    bottleneck convolution at batch 64 (throughput-sized, one kernel), "mlp" = the 128 x 768 x 3072 GEMM of the
    transformer MLP (latency-bound, one kernel), "gemm32" = the headline shape in fp32 (bound by the fp32
    matrix-core rate)."""
    import numpy as np

    def dev(stored):
        return torch.from_numpy(np.ascontiguousarray(stored)).cuda()

    if which in ("qkt", "sv"):
        # the two attention products at batch x heads = 192, seq = 512 (the memory-bound members of the benchmark
        # configurations): scores = Q.K^T / 8 writes 100 MB, context = S.V reads 100 MB
        c = wl.config4("f16")[3]
        b, sq, d = c["batch"], c["seq"], c["d"]
        n_sets = 4 if cold else 1  # 4 x 126 MB > 256 MB
        if which == "qkt":
            sets = [(dev(c["Q"]), dev(c["K"]), torch.empty((b, sq, sq), dtype=torch.float16, device="cuda")) for _ in range(n_sets)]
            epi = hb.make_epilogue(alpha=c["alpha"])
            cfg, _ = hb.hidet_tune_gemm(*sets[0], transB=True, epilogue=epi, iters=50)
            call = lambda t: hb.hidet_batched_gemm(t[0], t[1], t[2], transB=True, epilogue=epi, config=cfg)
            name = "batched f16 GEMM scores = Q.K^T / 8, batch x heads = 192, seq 512, d 64 (%s)" % c["name"]
        else:
            sets = [(dev(c["S"]), dev(c["V"]), torch.empty((b, sq, d), dtype=torch.float16, device="cuda")) for _ in range(n_sets)]
            cfg, _ = hb.hidet_tune_gemm(*sets[0], iters=50)
            call = lambda t: hb.hidet_batched_gemm(t[0], t[1], t[2], config=cfg)
            name = "batched f16 GEMM context = S.V, batch x heads = 192, seq 512, d 64 (%s)" % c["name"]
        name += ", operands rotated over %d sets (HBM only)" % n_sets if cold else ", same buffers every launch"
        counter = [0]

        def step():
            call(sets[counter[0] % n_sets])
            counter[0] += 1
        unit_bytes = (2 * b * sq * d + b * sq * sq) * 2
        extra = {"tile_config": cfg, "k_slices": 1, "flops": 2.0 * b * sq * sq * d}
    elif which == "softmax":
        b, s = 192, 512
        g = wl.rng(6300)
        x = dev(wl.to_storage(g.standard_normal((b * s, s)).astype(np.float32), "f16"))
        y = torch.empty_like(x)
        step = lambda: hb.hidet_softmax_rows(x, y)
        name = "row softmax, f16, %d rows x %d columns (scores of attention batch*heads=192, seq=512), N(0,1)" % (b * s, s)
        unit_bytes = 2 * x.numel() * 2
        extra = {}
    elif which == "mlp":
        # the latency-bound GEMM of the transformer MLP: 128 x 768 x 3072 with a residual (few output tiles, long K)
        c = wl.config2("f16")[1]
        A, B, res = dev(c["A"]), dev(c["B"]), dev(c["residual"])
        C = torch.empty((c["M"], c["N"]), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(residual=res)
        cfg, _ = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=100)
        step = lambda: hb.hidet_gemm(A, B, C, epilogue=epi, config=cfg)
        name = "fused f16 GEMM C = A.B + residual, M=128, N=768, K=3072 (%s), seed %d" % (c["name"], c["seed"])
        unit_bytes = (A.numel() + B.numel() + 2 * C.numel()) * 2
        extra = {"tile_config": cfg, "k_slices": 1, "flops": 2.0 * c["M"] * c["N"] * c["K"]}
    elif which == "gemm32":
        # the headline shape in fp32: bound by the fp32 matrix-core rate (157.3 TFLOP/s), not by memory
        c = wl.gemm_case(5200, 4096, 4096, 4096, "f32", bias="col")
        A, B, bias = dev(c["A"]), dev(c["B"]), dev(c["bias"])
        C = torch.empty((4096, 4096), dtype=torch.float32, device="cuda")
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
        cfg, _ = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=5)
        step = lambda: hb.hidet_gemm(A, B, C, epilogue=epi, config=cfg)
        name = "fused f32 GEMM C = ReLU(A.B + bias), M=N=K=4096, U(-1,1), seed 5200"
        unit_bytes = (A.numel() + B.numel() + C.numel() + bias.numel()) * 4
        extra = {"tile_config": cfg, "k_slices": 1, "flops": 2.0 * 4096 ** 3}
    elif which == "conv64":
        # a throughput-sized convolution: the 28x28, 128 -> 128, 3x3 bottleneck layer at batch 64 (single kernel)
        c = wl.conv_case(6400, 64, 128, 28, 28, 128, 3, 3, 1, 1, "f16")
        x, w, bias = dev(c["x"]), dev(c["w"]), dev(c["bias"])
        y = torch.empty((64, 128, c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
        sp = dict(stride=(1, 1), pad=(1, 1))
        cfg, _ = hb.hidet_tune_conv2d(x, w, y, epilogue=epi, iters=20, **sp)
        step = lambda: hb.hidet_conv2d_implicit_gemm(x, w, y, config=cfg, epilogue=epi, **sp)
        name = "conv2d 64x128x28x28 -> 128, 3x3, stride 1, pad 1, f16, bias + ReLU, He-init weights, seed 6400"
        unit_bytes = (x.numel() + w.numel() + y.numel() + bias.numel()) * 2
        extra = {"tile_config": cfg, "k_slices": 1, "flops": 2.0 * 64 * 128 * c["OH"] * c["OW"] * 128 * 9}
    else:
        c = wl.conv_case(6100, 1, 256, 28, 28, 256, 3, 3, 2, 1, "f16")
        x, w, bias = dev(c["x"]), dev(c["w"]), dev(c["bias"])
        y = torch.empty((1, 256, c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
        ws = torch.empty(16 << 20, dtype=torch.float32, device="cuda")
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
        sp = dict(stride=(2, 2), pad=(1, 1))
        cfg, slices, _ = hb.hidet_tune_conv2d_splitk(x, w, y, ws, epilogue=epi, iters=50, **sp)
        step = lambda: hb.hidet_conv2d_implicit_gemm_splitk(x, w, y, ws, k_slices=slices, config=cfg, epilogue=epi, **sp)
        name = "conv2d 1x256x28x28 -> 256, 3x3, stride 2, pad 1, f16, bias + ReLU, He-init weights, seed 6100"
        unit_bytes = (x.numel() + w.numel() + y.numel() + bias.numel()) * 2
        extra = {"tile_config": cfg, "k_slices": slices,
                 "flops": 2.0 * 256 * c["OH"] * c["OW"] * 256 * 9}
    for _ in range(warmup):
        step()
    # The K timed steps are captured into one HIP graph and replayed once between the two events: kernels of a few
    # tens of microseconds are otherwise launched more slowly from Python than they run.  (The library only launches
    # kernels, so a call may be captured; the graph is replayed once untimed first.)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            for _ in range(steps):
                step()
    g.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    g.replay()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    gbps = unit_bytes / (ms * 1e-3) / 1e9
    out = {"metric": "algorithmic GB/s of one secondary kernel, 1 GPU", "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": round(ms, 6), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f16", "data": "synthetic", "config": dict(workload=name, **extra),
           "roofline": {"bound": "hbm", "achieved": round(gbps, 1), "peak": 8000.0, "unit": "GB/s",
                        "frac": round(gbps / 8000.0, 4), "traffic": None}}
    if "flops" in extra:
        out["config"]["TFLOPs"] = round(extra["flops"] / (ms * 1e-3) / 1e12, 2)
    if which in ("qkt", "sv", "softmax"):
        # what plain read / write / copy kernels sustain on this machine on memory that no cache holds: the ceiling a
        # memory-bound kernel can be held against (the 8 TB/s of the roofline is the datasheet's figure)
        ring = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        out["config"]["streaming_kernel_GBps"] = {k: round(hb.hidet_probe_stream_bandwidth(ring, m), 1)
                                                  for m, k in enumerate(("read", "write", "copy"))}
        del ring
    if which == "gemm32":
        tf = extra["flops"] / (ms * 1e-3) / 1e12
        out.update(metric="TFLOP/s of one secondary kernel, 1 GPU", value=round(tf, 2), unit="TFLOP/s", dtype="f32")
        out["roofline"] = {"bound": "mfma", "achieved": round(tf, 2), "peak": 157.3, "unit": "TFLOP/s",
                           "frac": round(tf / 157.3, 4), "traffic": None}
    if graph_replay:
        out["config"]["us_per_call_graph_replay"] = round(graph_time(torch, step), 2)
    return out


def studies(torch, hb, wl, steps=100):
    """Schedule-space studies in the manner of Section 6.3.1 (latency of every schedule of the space on one
    convolution) and Section 6.3.2 (consecutive problem sizes, among them the prime 2039)."""
    import numpy as np

    def dev(stored):
        return None if stored is None else torch.from_numpy(np.ascontiguousarray(stored)).cuda()

    def tile(cfg):
        i = hb.hidet_config_info(cfg)
        return "%dx%dx%d/%dx%d/mfma%d/%s" % (i["block_m"], i["block_n"], i["block_k"], i["waves_m"], i["waves_n"], i["mfma"],
                                            ("2stage", "ring", "2stage-ahead", "2stage-ksplit")[i["schedule"]])

    out = {}
    ws = torch.empty(16 << 20, dtype=torch.float32, device="cuda")
    c = wl.conv_case(6100, 1, 256, 28, 28, 256, 3, 3, 2, 1, "f16")
    x, w, b = dev(c["x"]), dev(c["w"]), dev(c["bias"])
    y = torch.empty((1, 256, c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(bias=b, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
    sp = dict(stride=(2, 2), pad=(1, 1))
    t0 = time.perf_counter()
    best, us = hb.hidet_tune_conv2d(x, w, y, epilogue=epi, iters=steps, **sp)
    secs = time.perf_counter() - t0
    plain = hb.hidet_tune_last_times()
    best_s, slices, us_s = hb.hidet_tune_conv2d_splitk(x, w, y, ws, epilogue=epi, iters=steps, **sp)
    sliced = hb.hidet_tune_last_times()
    out["conv_28x28x256_k3_s2_p1_f16"] = {
        "best": {"config": best, "tile": tile(best), "us": round(us, 2)},
        "best_with_k_slices": {"config": best_s, "tile": tile(best_s), "k_slices": slices, "us": round(us_s, 2)},
        "tuning_seconds_unsliced": round(secs, 3),
        "schedules": [{"config": i, "tile": tile(i), "us": round(t, 2), "us_best_over_k_slices": round(sliced[i], 2)}
                      for i, t in enumerate(plain) if t > 0]}

    g = wl.config5("f16")
    A, B, bias = dev(g["A"]), dev(g["B"]), dev(g["bias"])
    C = torch.empty((g["M"], g["N"]), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
    t0 = time.perf_counter()
    best, us = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=20)
    secs = time.perf_counter() - t0
    out["gemm_4096_f16"] = {"best": {"config": best, "tile": tile(best), "us": round(us, 2)}, "tuning_seconds": round(secs, 3),
                            "schedules": [{"config": i, "tile": tile(i), "us": round(t, 2),
                                           "TFLOPs": round(2.0 * 4096 ** 3 / t * 1e-6, 1)}
                                          for i, t in enumerate(hb.hidet_tune_last_times()) if t > 0]}
    del A, B, C

    sweep = []
    for n in range(2032, 2049):
        g = wl.gemm_case(6200 + n, n, n, n, "f16", bias="col")
        A, B, bias = dev(g["A"]), dev(g["B"]), dev(g["bias"])
        C = torch.empty((n, n), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
        best, us = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=20)
        sweep.append({"n": n, "config": best, "tile": tile(best), "us": round(us, 2),
                      "TFLOPs": round(2.0 * n ** 3 / us * 1e-6, 1)})
    out["gemm_square_sizes_2032_2048_f16"] = sweep

    # batch sizes 1, 4, 8 on the four bottleneck convolutions (after Section 6.3.3)
    batches = []
    for i, (IC, H, W, OC, KH, KW, s_, p_) in enumerate(wl.RESNET50_CONVS):
        for nb in (1, 4, 8):
            c = wl.conv_case(6400 + 10 * i + nb, nb, IC, H, W, OC, KH, KW, s_, p_, "f16")
            x, w, b = dev(c["x"]), dev(c["w"]), dev(c["bias"])
            y = torch.empty((nb, OC, c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
            epi = hb.make_epilogue(bias=b, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
            sp = dict(stride=(s_, s_), pad=(p_, p_))
            best, slices, us = hb.hidet_tune_conv2d_splitk(x, w, y, ws, epilogue=epi, iters=steps, **sp)
            flops = 2.0 * nb * OC * c["OH"] * c["OW"] * IC * KH * KW
            batches.append({"layer": "%dx%d %d->%d k%d" % (H, W, IC, OC, KH), "batch": nb, "config": best, "tile": tile(best),
                            "k_slices": slices, "us": round(us, 2), "TFLOPs": round(flops / us * 1e-6, 2)})
    out["conv_batch_1_4_8_f16"] = batches

    # post-scheduling fusion (after Section 6.3.4): the fused call against the same anchor kernel with an identity
    # epilogue followed by separate elementwise kernels (PyTorch's add and relu) for the bias and the activation
    fusion = []
    for c in wl.config3("f16"):
        x, w, b = dev(c["x"]), dev(c["w"]), dev(c["bias"])
        y = torch.empty((c["Nb"], c["OC"], c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
        sp = dict(stride=(c["stride"], c["stride"]), pad=(c["pad"], c["pad"]))
        epi = hb.make_epilogue(bias=b, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
        # both anchors tuned; no configuration named, so each call runs what the tuner remembered for it
        hb.hidet_tune_conv2d(x, w, y, epilogue=epi, iters=steps, **sp)
        hb.hidet_tune_conv2d(x, w, y, iters=steps, **sp)
        bias4 = b.view(1, -1, 1, 1)

        def unfused():
            hb.hidet_conv2d_implicit_gemm(x, w, y, **sp)
            y.add_(bias4)
            y.relu_()
        fused_us = graph_time(torch, lambda: hb.hidet_conv2d_implicit_gemm(x, w, y, epilogue=epi, **sp))
        fusion.append({"workload": c["name"], "fused_us": round(fused_us, 2), "unfused_3_kernels_us": round(graph_time(torch, unfused), 2)})
    for c in wl.config2("f16"):
        A, B, bias = dev(c["A"]), dev(c["B"]), dev(c["bias"])
        res = dev(c["residual"]) if c["residual"] is not None else None
        C = torch.empty((c["M"], c["N"]), dtype=torch.float16, device="cuda")
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, residual=res, relu=c.get("relu", False))
        cfg, _ = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=steps)

        def unfused():
            hb.hidet_gemm(A, B, C, config=cfg)
            if bias is not None:
                C.add_(bias)
            if res is not None:
                C.add_(res)
            if c.get("relu", False):
                C.relu_()
        fused_us = graph_time(torch, lambda: hb.hidet_gemm(A, B, C, epilogue=epi, config=cfg))
        fusion.append({"workload": c["name"], "fused_us": round(fused_us, 2), "unfused_us": round(graph_time(torch, unfused), 2)})
    out["fused_vs_separate_elementwise_kernels_f16"] = fusion

    # 1x1 convolutions (two thirds of the bottleneck network's layers): the gather form against the batched-GEMM form
    # that a call without an explicit configuration takes; best configuration of each form, HIP-graph replays
    pointwise = []
    hb.hidet_tune_clear()
    for nb in (1, 64):
        for IC, OC, HW in ((64, 256, 56), (256, 64, 56), (128, 512, 28), (512, 128, 28), (256, 1024, 14), (1024, 256, 14),
                           (512, 2048, 7), (2048, 512, 7)):
            c = wl.conv_case(6500 + nb + HW, nb, IC, HW, HW, OC, 1, 1, 1, 0, "f16")
            x, w, b = dev(c["x"]), dev(c["w"]), dev(c["bias"])
            y = torch.empty((nb, OC, HW, HW), dtype=torch.float16, device="cuda")
            epi = hb.make_epilogue(bias=b, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
            untuned = graph_time(torch, lambda: hb.hidet_conv2d_implicit_gemm(x, w, y, epilogue=epi))
            gather = min((graph_time(torch, lambda: hb.hidet_conv2d_implicit_gemm(x, w, y, epilogue=epi, config=i), 10, 5), i)
                         for i in range(hb.hidet_config_count()) if not hb.hidet_config_info(i)["is_f32"])
            A, B, C = w.view(1, OC, IC).expand(nb, OC, IC), x.view(nb, IC, HW * HW), y.view(nb, OC, HW * HW)
            g_cfg, _ = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=steps if nb == 1 else 20)
            gemm_form = graph_time(torch, lambda: hb.hidet_batched_gemm(A, B, C, epilogue=epi, config=g_cfg))
            flops = 2.0 * nb * OC * IC * HW * HW
            pointwise.append({"layer": "%dx%d %d->%d k1" % (HW, HW, IC, OC), "batch": nb,
                              "gather_form_us": round(gather[0], 2), "gather_form_tile": tile(gather[1]),
                              "gemm_form_us": round(gemm_form, 2), "gemm_form_tile": tile(g_cfg),
                              "untuned_call_us": round(untuned, 2),
                              "TFLOPs_best": round(flops / min(gather[0], gemm_form) * 1e-6, 2)})
    out["pointwise_conv_forms_f16"] = pointwise

    # 3x3 convolutions: the (ic, kh, kw) K order over OIHW weights against the tap-major order over repacked weights
    # (one filter tap per K tile); both tuned over tiles and K-slice counts, HIP-graph replays
    packed = []
    for nb in (1, 8, 64):
        for IC, HW, OC, s_ in ((64, 56, 64, 1), (128, 28, 128, 1), (256, 14, 256, 1), (512, 7, 512, 1), (256, 28, 256, 2)):
            c = wl.conv_case(6600 + nb + HW + s_, nb, IC, HW, HW, OC, 3, 3, s_, 1, "f16")
            x, w, b = dev(c["x"]), dev(c["w"]), dev(c["bias"])
            y = torch.empty((nb, OC, c["OH"], c["OW"]), dtype=torch.float16, device="cuda")
            epi = hb.make_epilogue(bias=b, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
            sp = dict(stride=(s_, s_), pad=(1, 1))
            wp = hb.hidet_conv2d_pack_weights(w)
            c0, s0, _ = hb.hidet_tune_conv2d_splitk(x, w, y, ws, epilogue=epi, iters=20, **sp)
            t0 = graph_time(torch, lambda: hb.hidet_conv2d_implicit_gemm_splitk(x, w, y, ws, k_slices=s0, epilogue=epi, config=c0, **sp))
            c1, s1, _ = hb.hidet_tune_conv2d_packed(x, wp, y, ws, epilogue=epi, iters=20, **sp)
            t1 = graph_time(torch, lambda: hb.hidet_conv2d_implicit_gemm_packed(x, wp, y, epilogue=epi, config=c1, k_slices=s1,
                                                                                workspace=ws, **sp))
            flops = 2.0 * nb * OC * c["OH"] * c["OW"] * IC * 9
            packed.append({"layer": "%dx%d %d->%d k3 s%d" % (HW, HW, IC, OC, s_), "batch": nb,
                           "oihw_us": round(t0, 2), "oihw_tile": tile(c0), "oihw_k_slices": s0,
                           "packed_us": round(t1, 2), "packed_tile": tile(c1), "packed_k_slices": s1,
                           "TFLOPs_best": round(flops / min(t0, t1) * 1e-6, 2)})
    out["conv3x3_weight_orders_f16"] = packed
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--dtype", default="f16", choices=["f16", "bf16"])
    ap.add_argument("--k", type=int, default=4096)
    ap.add_argument("--config", type=int, default=None, help="force a tile configuration instead of tuning")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--report", default=None, metavar="PATH",
                    help="also time every parity configuration (configs 1-4 and both config-5 shapes, fp16 and bf16) "
                         "and write the table to PATH as JSON; the headline line is printed as usual")
    ap.add_argument("--cold", action="store_true",
                    help="with --workload qkt / sv: rotate over enough copies of the operands to exceed the 256 MB Infinity "
                         "Cache, so that every launch finds them in HBM only")
    ap.add_argument("--workload", default="gemm", choices=["gemm", "softmax", "conv", "conv64", "mlp", "gemm32", "qkt", "sv"],
                    help="gemm (default): the headline benchmark; softmax / conv: one secondary kernel alone (for profiling)")
    ap.add_argument("--graph-replay", action="store_true",
                    help="with --workload other than gemm: also time the call replayed from a HIP graph "
                         "(the device-side time of kernels shorter than a Python launch)")
    ap.add_argument("--studies", default=None, metavar="PATH",
                    help="instead of the benchmark, run the schedule-space studies (latency of every schedule on the "
                         "case-study convolution and on the headline GEMM; square sizes 2032..2048) and write them to PATH")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, run 10 plain device-to-device copies of MIB mebibytes "
                         "(known traffic, used to scale the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards by output tiles without any exchange); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2210_09603_amd import binding as hb
    from paper_2210_09603_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    hb.lib()  # raises if the HIP extension has not been built

    if args.studies:
        with open(args.studies, "w") as fh:
            json.dump(studies(torch, hb, wl), fh, indent=1)
        print(json.dumps({"studies_written_to": args.studies}))
        return

    if args.workload != "gemm":
        print(json.dumps(other_workload(torch, hb, wl, args.workload, args.steps, args.warmup, args.graph_replay, args.cold)))
        return

    if args.copy_calibration > 0:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 10}))
        return

    dt = args.dtype
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[dt]
    c = wl.config5(dt, K=args.k)
    M, N, K = c["M"], c["N"], c["K"]

    def dev(stored):
        import numpy as np
        if dt == "bf16":
            return torch.from_numpy(np.ascontiguousarray(stored).view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(np.ascontiguousarray(stored)).cuda()

    A, B, bias = dev(c["A"]), dev(c["B"]), dev(c["bias"])
    C = torch.empty((M, N), dtype=tdt, device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)

    t0 = time.perf_counter()
    if args.config is None:
        best_cfg, best_us = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=10)
    else:
        best_cfg, best_us = args.config, float("nan")
    tune_s = time.perf_counter() - t0
    cfg_info = hb.hidet_config_info(best_cfg)

    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        hb.hidet_gemm(A, B, C, epilogue=epi, stream=stream, config=best_cfg)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(args.steps):
        hb.hidet_gemm(A, B, C, epilogue=epi, stream=stream, config=best_cfg)
    e1.record(stream)
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    flops = 2.0 * M * N * K
    tflops = flops / (ms_per_step * 1e-3) / 1e12

    # Spread of the per-launch time: a second pass of the same K launches cut into groups of consecutive launches, one
    # HIP event between groups (an event after every single launch would add its own few microseconds to each of
    # them); median, min and max are taken over the groups' means.
    n_groups = min(20, args.steps)
    per_group = max(1, args.steps // n_groups)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_groups + 1)]
    marks[0].record(stream)
    for g in range(n_groups):
        for _ in range(per_group):
            hb.hidet_gemm(A, B, C, epilogue=epi, stream=stream, config=best_cfg)
        marks[g + 1].record(stream)
    torch.cuda.synchronize()
    groups = sorted(marks[g].elapsed_time(marks[g + 1]) * 1000.0 / per_group for g in range(n_groups))
    launch_stats = {"groups": n_groups, "launches_per_group": per_group, "median_us": round(groups[n_groups // 2], 2),
                    "min_us": round(groups[0], 2), "max_us": round(groups[-1], 2),
                    "mean_us": round(sum(groups) / n_groups, 2),
                    "method": "second pass, one HIP event between groups of consecutive launches"}

    # what the matrix cores alone sustain on these operand values (clock is power-limited and data-dependent)
    ceil_tflops, ceil_mhz = hb.hidet_probe_mfma_peak(A, mfma=cfg_info["mfma"])
    algo_bytes = (M * K + K * N + M * N + N) * 2  # every operand and the output once
    out = {
        "metric": "fused GEMM/implicit-GEMM conv TFLOP/s and % of MI355X peak MFMA, 1 GPU",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dt,
        "data": "synthetic",
        "config": {
            "workload": "cfg5: fused %s GEMM C=ReLU(A.B+bias), M=N=%d, K=%d, row-major, U(-1,1), seed %d" % (dt, M, K, c["seed"]),
            "tile_config": best_cfg,
            "tile": "%dx%dx%d, %dx%d waves, mfma %d" % (cfg_info["block_m"], cfg_info["block_n"], cfg_info["block_k"],
                                                         cfg_info["waves_m"], cfg_info["waves_n"], cfg_info["mfma"]),
            "tuning_seconds": round(tune_s, 3),
            "pct_of_peak_mfma": round(100.0 * tflops / PEAK_TFLOPS[dt], 2),
            "algorithmic_hbm_GBps": round(algo_bytes / (ms_per_step * 1e-3) / 1e9, 1),
            "mfma_only_ceiling_TFLOPs_same_data": round(ceil_tflops, 1),
            "mfma_only_ceiling_sclk_MHz": round(ceil_mhz),
            "pct_of_mfma_only_ceiling": round(100.0 * tflops / ceil_tflops, 2) if ceil_tflops > 0 else None,
            "per_launch": launch_stats,
        },
        "roofline": {
            "bound": "mfma",
            "achieved": round(tflops, 2),
            "peak": PEAK_TFLOPS[dt],
            "unit": "TFLOP/s",
            "frac": round(tflops / PEAK_TFLOPS[dt], 4),
            "traffic": MEASURED_TRAFFIC.get((dt, M, N, K), (None, None))[0],
            "traffic_source": MEASURED_TRAFFIC.get((dt, M, N, K), (None, None))[1],
            "algorithmic_bytes": algo_bytes,
        },
    }

    if args.report:
        out_report = side_report(torch, hb, wl)
        with open(args.report, "w") as fh:
            json.dump(out_report, fh, indent=1)

    if not args.no_cpu_baseline:
        import oracle
        A64, B64, b64 = wl.widen(c["A"], dt), wl.widen(c["B"], dt), wl.widen(c["bias"], dt)
        rows, t = 32, 0.0
        while True:  # grow the row sample until the oracle has worked for about 10 s
            t0 = time.perf_counter()
            oracle.gemm(A64, B64, bias=b64, relu=True, rows=(0, rows))
            t = time.perf_counter() - t0
            if t >= 8.0 or rows >= M:
                break
            rows = min(M, max(rows * 2, int(rows * 10.0 / max(t, 1e-3))))
        out["cpu_baseline"] = {
            "value": round(2.0 * rows * N * K / t / 1e12, 6),
            "unit": "TFLOP/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "first %d of %d rows of C (all %d columns, full K=%d), fp64, %.1f s" % (rows, M, N, K, t),
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
