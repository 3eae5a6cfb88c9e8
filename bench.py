#!/usr/bin/env python3
"""Benchmark of the 4-bit linear-layer hot path on one MI355X.

Primary workload (the one `value` is quoted on): the four W4A16 linears of a
Llama-2-7B decoder layer at M = 1 (fused QKV 4096->12288, out 4096->4096, fused
gate+up 4096->22016, down 11008->4096; group 128, asymmetric uint4).  One step
= one decoder layer's four GEMVs through qail_w4a16_linear_batch.  The steps
rotate through `--layers` independently seeded layers (default 32: the whole
decode stack of the full-stack configuration, 3.36 GB of packed weights) so that neither L2 nor the 256 MB last-level cache can serve the
reads.  Throughput = algorithmic bytes (packed weights + scales + zero-points +
x + y) per second, with everything resident in HBM before the timed region.

Secondary workloads (reported under "extra", never in `value`): prefill GEMM
at M = 288 / 1024, the 35 W4A4 convolutions of a ResNet-34 body at batch 32,
and a decode stack walk at M in {1, 4, 16}.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the decode kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (profiles/w4a16_gemv_decode_layer_pmc.txt), and the sha256 of the kernel source the
# counters were taken on; reported as null once the kernel has changed.
GEMV_TRAFFIC_BYTES = 106030306
GEMV_TRAFFIC_SOURCE_SHA256 = "46c8a68ba336220dc6951ea77e255a605ea0dc66a533767f30505c97b0f63c86"

HBM_PEAK_GBS = 8000.0         # MI355X HBM3E, published
BF16_PEAK_TFLOPS = 2500.0     # dense bf16 MFMA, published
INT8_PEAK_TOPS = 5000.0       # dense int8 MFMA, published
GROUP = 128


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=2000)
    p.add_argument("--warmup", type=int, default=100)
    p.add_argument("--settle-ms", type=float, default=200.0,
                   help="how long a matrix-core-bound extra line repeats its work before it is timed")
    p.add_argument("--layers", type=int, default=32,
                   help="independently seeded layers to rotate through (32 = the full decode stack, 3.36 GB packed)")
    p.add_argument("--no-extra", action="store_true", help="skip the secondary workloads")
    p.add_argument("--only", type=str, default="",
                   help="comma-separated names of the secondary workloads to run (default: all): spread, singles, "
                        "stack, lora, prefill, conv32, conv32_fused, conv256, w8, train, cpu_extra")
    p.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    p.add_argument("--calibrate-copy", action="store_true",
                   help="also run a few 256 MiB device copies (a kernel of known traffic, for scaling "
                        "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return p.parse_args()


def gemv_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_2412_01034_amd", "csrc", "w4a16_gemv.hip")
    try:
        sha = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    return GEMV_TRAFFIC_BYTES if sha == GEMV_TRAFFIC_SOURCE_SHA256 else None


def linear_bytes(N, K, M, g=GROUP):
    G = K // g
    return N * K // 2 + N * G * 2 + N * ((G + 7) // 8) * 4 + M * K * 2 + M * N * 2


def main():
    args = parse()
    if args.gpus != 1:
        log("bench.py: the library runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2412_01034_amd import binding as B
    from paper_2412_01034_amd import synth

    if not os.path.exists(B.LIB_PATH):
        from paper_2412_01034_amd import build
        build.build_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint32:
            a = a.view(np.int32)
        elif a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).cuda()

    # ---------------------------------------------------------------- weights
    t0 = time.time()
    shapes = synth.LLAMA7B_LINEARS
    L = args.layers

    def gen(job):
        layer, i = job
        _, N, K = shapes[i]
        return job, synth.llm_weight(N, K, synth.seed_for(4, layer * 4 + i, 0), outlier_frac=0.01)

    layers = [[None] * 4 for _ in range(L)]
    jobs = [(l, i) for l in range(L) for i in range(4)]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        for (l, i), w in ex.map(gen, jobs):
            _, N, K = shapes[i]
            qb, sb, zb = B.qail_packed_sizes(N, K, GROUP, B.QAIL_W4_ASYM_GROUP)
            qw = torch.empty(qb // 4, dtype=torch.int32, device="cuda")
            sc = torch.empty(sb // 2, dtype=torch.int16, device="cuda")
            zr = torch.empty(zb // 4, dtype=torch.int32, device="cuda")
            wd = torch.from_numpy(w).cuda()
            B.qail_quantize_weights(wd, GROUP, B.QAIL_W4_ASYM_GROUP, qw, sc, zr)
            torch.cuda.synchronize()
            del wd, w
            layers[l][i] = dict(N=N, K=K, group_size=GROUP, qweight=qw, scales=sc, zeros=zr)
    log(f"[bench] {L} layers generated and quantised in {time.time() - t0:.1f} s")

    def with_io(M):
        """Attach x / y buffers for batch M to every layer; returns per-layer item arrays."""
        xs = [dev(synth.llm_activation_bf16(M, K, synth.seed_for(1, i, 1))) for i, (_, N, K) in enumerate(shapes)]
        out = []
        for l in range(L):
            ents = []
            for i, (_, N, K) in enumerate(shapes):
                e = dict(layers[l][i])
                e["x"] = xs[i]
                e["y"] = torch.empty(M * N, dtype=torch.int16, device="cuda")
                ents.append(e)
            out.append((B.make_w4a16_items(ents, M), ents))
        return out

    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    if args.calibrate_copy:
        src = torch.ones(256 << 18, dtype=torch.int32, device="cuda")   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------- primary: decode GEMVs
    dec = with_io(1)
    bytes_per_step = sum(linear_bytes(N, K, 1) for _, N, K in shapes)

    def step(i):
        items, _ = dec[i % L]
        B.qail_w4a16_linear_batch(items, 4, 1, None, sh)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_begin = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    gpu_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / args.steps
    value = bytes_per_step / (wall / args.steps) / 1e9
    # one launch per step: the batched call serves the four linears in one kernel
    launches = args.steps
    kern_us = gpu_ms * 1e3 / launches
    achieved = bytes_per_step / (kern_us * 1e-6) / 1e9
    log(f"[bench] decode: {ms_per_step * 1e3:.2f} us/step wall, {kern_us:.2f} us/launch by events, "
        f"{value:.0f} GB/s ({100 * value / HBM_PEAK_GBS:.1f}% of HBM peak)")

    result = {
        "metric": "W4A16 decode GEMV GB/s at Llama-2-7B shapes (M=1)",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: four Llama-2-7B decode linears (12288x4096, 4096x4096, 22016x4096, "
                        "4096x11008), W4A16 group 128 asymmetric uint4, M=1, one decoder layer per step",
            "layers_rotated": L,
            "bytes_per_step": bytes_per_step,
            "pct_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "w4a16_gemv_kernel (one launch = one decoder layer, 4 linears)",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": gemv_traffic(),
            "traffic_source": "profiles/w4a16_gemv_decode_layer_pmc.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, "
                              "not re-measured in this run; null when the kernel source has changed since)",
            "avg_launch_us": round(kern_us, 3),
        },
    }
    # spread of single launches of the headline step: an event pair around each of 300 launches
    # (the pair's own gap is inside each reading, so the median sits above avg_launch_us)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(300)]
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs)
    result["us_per_step_p10_p50_p90"] = [round(us[len(us) // 10], 2), round(us[len(us) // 2], 2),
                                         round(us[len(us) * 9 // 10], 2)]

    # --------------------------------------------------------------- extras
    extra = {}
    only = [w for w in args.only.split(",") if w]

    def want(name):
        return not args.no_extra and (not only or name in only)

    def timed(fn, iters, warm=5, settle=False):
        # settle: matrix-core-bound work is timed at the clock the chip sustains under it.  Coming
        # from idle (or from memory-bound work) the first milliseconds run at a lower clock, so
        # such a line first repeats its work for --settle-ms (0.2 s) and is then timed over half of that or more.
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        if settle:
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(3):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            once = max(a.elapsed_time(b) * 1e-3 / 3, 1e-6)
            for _ in range(min(20000, int(args.settle_ms * 1e-3 / once) + 1)):
                fn()
            iters = max(iters, min(20000, int(args.settle_ms * 0.5e-3 / once) + 1))
            torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(iters):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / iters

    if want("spread"):
        # the headline layer launched over and over, labelled as what it is: its 105 MB stay in the last-level cache
        tcr = timed(lambda: step(0), 400)
        extra["decode_layer_cache_resident"] = {"us": round(tcr * 1e6, 2), "GBps": round(bytes_per_step / tcr / 1e9, 1),
                                                "note": "one layer repeated: served by the last-level cache, not HBM"}

    if want("singles"):
        # single-linear decode launches (cold weights: rotate layers)
        per = {}
        for i, (name, N, K) in enumerate(shapes):
            singles = [B.make_w4a16_items([dec[l][1][i]], 1) for l in range(L)]
            cnt = [0]

            def one():
                B.qail_w4a16_linear_batch(singles[cnt[0] % L], 1, 1, None, sh)
                cnt[0] += 1
            t = timed(one, 400)
            gbps = linear_bytes(N, K, 1) / t / 1e9
            per[name] = {"us": round(t * 1e6, 2), "GBps": round(gbps, 1), "frac_hbm_peak": round(gbps / HBM_PEAK_GBS, 4)}
        extra["decode_single_linear"] = per

    if want("stack"):
        # the full decode stack: 32 layers x 4 linears per token-step, 7 token-steps per timing;
        # with the default --layers 32 every layer has its own seeded weights (3.36 GB per token-step)
        stack = {}
        stack_bytes_w = 32 * sum(linear_bytes(N, K, 0) for _, N, K in shapes)
        for M in (1, 4, 16, 32, 64):
            io = dec if M == 1 else with_io(M)
            nws = B.qail_w4a16_batch_workspace(io[0][0], 4, M)   # M > 32: the matrix-core GEMM's
            wsk = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None

            def walk():
                for l in range(32):
                    B.qail_w4a16_linear_batch(io[l % L][0], 4, M, wsk, sh)
            t = timed(walk, 7, warm=1)
            gbps = 32 * sum(linear_bytes(N, K, M) for _, N, K in shapes) / t / 1e9
            stack[f"M={M}"] = {"ms_per_token_step": round(t * 1e3, 4), "tokens_per_s": round(M / t, 1),
                               "GBps": round(gbps, 1), "frac_hbm_peak": round(gbps / HBM_PEAK_GBS, 4)}
            if M == 1:
                # the same walk with real dependences, as a decoder has them (each linear may read what the
                # one before it wrote), in one launch per 32 linears: the blocks meet between two linears
                # through counters while the next linear's first weights are already on their way
                ents_all = [io[l % L][1][i] for l in range(32) for i in range(4)]
                chain_items = B.make_w4a16_items(ents_all, 1)
                wsc = torch.zeros(B.qail_w4a16_chain_workspace(chain_items, len(ents_all)), dtype=torch.uint8, device="cuda")
                t = timed(lambda: B.qail_w4a16_linear_chain(chain_items, len(ents_all), wsc, sh), 7, warm=1)
                torch.cuda.synchronize()
                gbps1 = 32 * sum(linear_bytes(N, K, M) for _, N, K in shapes) / t / 1e9
                stack["M=1, dependent linears chained in one launch per 32"] = {
                    "ms_per_token_step": round(t * 1e3, 4), "tokens_per_s": round(M / t, 1), "GBps": round(gbps1, 1),
                    "frac_hbm_peak": round(gbps1 / HBM_PEAK_GBS, 4), "status_word": int(wsc[:4].view(torch.int32)[0].item())}
                del ents_all, chain_items, wsc
            if M in (1, 16):
                # the same walk with one launch per linear: stream order then makes every linear wait for
                # the one before it, as the data dependences of a real decoder layer would
                ones = [[B.make_w4a16_items([io[l][1][i]], M) for i in range(4)] for l in range(L)]

                def walk_dep():
                    for l in range(32):
                        for i in range(4):
                            B.qail_w4a16_linear_batch(ones[l % L][i], 1, M, wsk, sh)
                t = timed(walk_dep, 7, warm=1)
                gbps1 = 32 * sum(linear_bytes(N, K, M) for _, N, K in shapes) / t / 1e9
                stack[f"M={M}, one launch per linear"] = {"ms_per_token_step": round(t * 1e3, 4),
                                                          "tokens_per_s": round(M / t, 1), "GBps": round(gbps1, 1),
                                                          "frac_hbm_peak": round(gbps1 / HBM_PEAK_GBS, 4)}
                if M == 1:
                    # the same 128 launches recorded once into a graph and replayed
                    gs = torch.cuda.Stream()
                    with torch.cuda.stream(gs):
                        graph = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(graph, stream=gs):
                            for l in range(32):
                                for i in range(4):
                                    B.qail_w4a16_linear_batch(ones[l % L][i], 1, M, None, gs.cuda_stream)
                    torch.cuda.synchronize()
                    tg = timed(graph.replay, 7, warm=1)
                    del graph
                    stack["M=1, one launch per linear, graph replay"] = {"ms_per_token_step": round(tg * 1e3, 4),
                                                                         "tokens_per_s": round(M / tg, 1)}
                del ones
            if M != 1:
                del io
        stack["note"] = (f"32 layer-steps per token over {L} distinct layers"
                         + ("" if L >= 32 else " cycled") + f"; packed weights per token-step {stack_bytes_w} B; "
                         "the bound at 8 TB/s is 2378 token-steps/s")
        extra["decode_stack"] = stack

    if want("lora"):
        # the same decode layer with a rank-32 adapter beside each linear (unmerged, as the
        # fine-tuned 4-bit policy runs): down-projections in one small launch, up-projections
        # inside the streaming kernel's final store
        R = 32
        LL = min(L, 8)
        lora_io = []
        for l in range(LL):
            lents = []
            for i, (_, N, K) in enumerate(shapes):
                ab, bb = synth.lora_factors(N, K, R, synth.seed_for(4, l * 4 + i, 5))
                lents.append(dict(A=dev(ab), B=dev(bb), r=R, scaling=2.0, N=N, K=K))
            lora_io.append((B.make_loras(lents), lents))
        wsl = torch.empty(B.qail_w4a16_lora_workspace(dec[0][0], lora_io[0][0], 4, 1), dtype=torch.uint8, device="cuda")
        cntl = [0]

        def lora_step():
            l = cntl[0] % LL
            B.qail_w4a16_linear_lora_batch(dec[l][0], lora_io[l][0], 4, 1, wsl, sh)
            cntl[0] += 1
        tl = timed(lora_step, 400)
        lbytes = sum(R * (N + K) * 2 for _, N, K in shapes)
        extra["decode_layer_lora_r32"] = {"us_per_layer": round(tl * 1e6, 2),
                                          "GBps": round((bytes_per_step + lbytes) / tl / 1e9, 1),
                                          "adapter_bytes": lbytes,
                                          "launches_per_layer": 2}
        del lora_io, wsl

    if want("prefill"):
        pre = {}
        for M in (288, 1024):
            io = with_io(M)
            for i, (name, N, K) in enumerate(shapes):
                it = B.make_w4a16_items([io[0][1][i]], M)
                nws = B.qail_w4a16_batch_workspace(it, 1, M)
                ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
                t = timed(lambda: B.qail_w4a16_linear_batch(it, 1, M, ws, sh), 20, settle=True)
                tf = 2.0 * M * N * K / t / 1e12
                pre[f"{name}_M{M}"] = {"us": round(t * 1e6, 1), "TFLOPs": round(tf, 1),
                                       "frac_bf16_peak": round(tf / BF16_PEAK_TFLOPS, 4)}
            # the same four linears as one batched call: they share launches, each on a share of the blocks
            nws = B.qail_w4a16_batch_workspace(io[0][0], 4, M)
            ws = torch.empty(nws, dtype=torch.uint8, device="cuda") if nws else None
            t = timed(lambda: B.qail_w4a16_linear_batch(io[0][0], 4, M, ws, sh), 20, settle=True)
            tf = sum(2.0 * M * N * K for _, N, K in shapes) / t / 1e12
            pre[f"layer_batched_M{M}"] = {"us": round(t * 1e6, 1), "TFLOPs": round(tf, 1),
                                          "frac_bf16_peak": round(tf / BF16_PEAK_TFLOPS, 4)}
            del io
        extra["prefill_gemm"] = pre

    # ---- W4A4 ResNet-34 body.  Roof of a layer: max(ops / int8 peak, algorithmic bytes / HBM peak) with the
    # input tensor counted once (for a stride-2 1x1 only the sampled pixels), the packed weights, and 4 B
    # (int32 / fp32 output) or 0.5 B (fused 4-bit output) per output element.
    def conv_bytes(s, out_bytes):
        a_pix = s.B * s.H * s.W if s.KH > 1 else s.M
        return a_pix * s.Cin // 2 + s.Cout * s.K // 2 + int(s.M * s.Cout * out_bytes) + 8 * s.Cout

    def conv_roof_us(s, out_bytes):
        return max(s.ops / (INT8_PEAK_TOPS * 1e12), conv_bytes(s, out_bytes) / (HBM_PEAK_GBS * 1e9)) * 1e6

    def mfma_bound(s, out_bytes):
        return s.ops / (INT8_PEAK_TOPS * 1e12) >= conv_bytes(s, out_bytes) / (HBM_PEAK_GBS * 1e9)

    def conv_key(s):
        return f"{s.KH}x{s.KW}_{s.Cin}to{s.Cout}_s{s.stride}"

    def conv_summary(convs_, per_shape, t_pass, out_bytes):
        """Aggregates over all calls and over the layers whose roof is the matrix pipe, from the per-shape
        times (a sum of single-call times: no gaps between calls) and from the back-to-back pass."""
        tot_ops_ = sum(s.ops for s in convs_)
        sub = [s for s in convs_ if mfma_bound(s, out_bytes)]
        t_sum = sum(per_shape[conv_key(s)]["us"] for s in convs_) * 1e-6
        t_sub = sum(per_shape[conv_key(s)]["us"] for s in sub) * 1e-6
        roof = sum(conv_roof_us(s, out_bytes) for s in convs_) * 1e-6
        return {
            "all_calls": {"calls": len(convs_), "GOP": round(tot_ops_ / 1e9, 1),
                          "TOPs_back_to_back": round(tot_ops_ / t_pass / 1e12, 1),
                          "frac_int8_peak_back_to_back": round(tot_ops_ / t_pass / 1e12 / INT8_PEAK_TOPS, 4),
                          "TOPs_sum_of_calls": round(tot_ops_ / t_sum / 1e12, 1),
                          "roof_us": round(roof * 1e6, 1), "frac_of_roof": round(roof / t_pass, 4)},
            "mfma_bound_subset": {"calls": len(sub), "shapes": sorted({conv_key(s) for s in sub}),
                                  "GOP": round(sum(s.ops for s in sub) / 1e9, 1),
                                  "us_sum_of_calls": round(t_sub * 1e6, 1),
                                  "TOPs": round(sum(s.ops for s in sub) / max(t_sub, 1e-12) / 1e12, 1),
                                  "frac_int8_peak": round(sum(s.ops for s in sub) / max(t_sub, 1e-12) / 1e12 / INT8_PEAK_TOPS, 4)},
        }

    conv_state = {}

    def conv32_calls():
        if "calls" not in conv_state:
            convs = synth.resnet34_convs(32)
            rng = np.random.default_rng(synth.seed_for(3, 0, 0))
            calls, cache = [], {}
            for li, s in enumerate(convs):
                key = (s.H, s.Cin)
                if key not in cache:   # one code tensor per input shape (values do not affect timing)
                    cache[key] = dev(rng.integers(0, 2 ** 32, size=s.B * s.H * s.W * s.Cin // 8,
                                                  dtype=np.uint64).astype(np.uint32))
                ww = dev(rng.integers(0, 2 ** 32, size=s.Cout * s.K // 8, dtype=np.uint64).astype(np.uint32))
                scale = torch.full((s.Cout,), 1e-3, dtype=torch.float32, device="cuda")
                bias = torch.zeros(s.Cout, dtype=torch.float32, device="cuda")
                y = torch.empty(s.M * s.Cout, dtype=torch.float32, device="cuda")
                calls.append((s, cache[key], ww, scale, bias, y))
            conv_state["calls"] = calls
            conv_state["rng"] = rng
        return conv_state["calls"]

    def shape_line(s, tt, out_bytes):
        roof = conv_roof_us(s, out_bytes)
        return {"us": round(tt * 1e6, 2), "TOPs": round(s.ops / tt / 1e12, 1), "roof_us": round(roof, 2),
                "roof": "mfma" if mfma_bound(s, out_bytes) else "hbm", "frac_of_roof": round(roof / (tt * 1e6), 4)}

    if want("conv32"):
        calls = conv32_calls()
        tot_ops = sum(c[0].ops for c in calls)

        def body():
            for s, a, ww, scale, bias, y in calls:
                B.qail_w4a4_gemm(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww,
                                 scale=scale, bias=bias, y_out=y, stream=sh)
        t = timed(body, 20, settle=True)
        per_shape = {}
        for s, a, ww, scale, bias, y in calls:
            if conv_key(s) in per_shape:
                continue
            tt = timed(lambda: B.qail_w4a4_gemm(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad,
                                                a, ww, scale=scale, bias=bias, y_out=y, stream=sh), 50, settle=True)
            per_shape[conv_key(s)] = shape_line(s, tt, 4)
        # the same 35 calls captured once into a graph and replayed (the library only launches kernels)
        gs = torch.cuda.Stream()
        with torch.cuda.stream(gs):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=gs):
                for s, a, ww, scale, bias, y in calls:
                    B.qail_w4a4_gemm(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww,
                                     scale=scale, bias=bias, y_out=y, stream=gs.cuda_stream)
        torch.cuda.synchronize()
        tg = timed(graph.replay, 20, settle=True)
        del graph
        extra["w4a4_resnet34_b32"] = {"ms_per_pass": round(t * 1e3, 4), "TOPs": round(tot_ops / t / 1e12, 1),
                                      "frac_int8_peak": round(tot_ops / t / 1e12 / INT8_PEAK_TOPS, 4),
                                      "calls": len(calls), "ms_per_pass_graph_replay": round(tg * 1e3, 4),
                                      "per_shape": per_shape,
                                      "aggregate": conv_summary([c[0] for c in calls], per_shape, t, 4)}

    if want("conv32_fused"):
        # the same 35 calls with the fused 4-bit output (ReLU + shortcut + quantise for the next
        # layer): every call writes 0.5 B per output instead of 4 B
        calls = conv32_calls()
        tot_ops = sum(c[0].ops for c in calls)
        fcalls = []
        for s, a, ww, scale, bias, y in calls:
            out = torch.empty(s.M * s.Cout // 8, dtype=torch.int32, device="cuda")
            res = a if (s.Cin == s.Cout and s.stride == 1) else None   # identity shortcut: same shape as the output
            fcalls.append((s, a, ww, scale, bias, out, res))

        def fused_body():
            for s, a, ww, scale, bias, out, res in fcalls:
                B.qail_w4a4_conv_u4(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww, scale, bias,
                                    0.37, out, res_u4=res, res_scale=0.11, stream=sh)
        tf_ = timed(fused_body, 20, settle=True)
        fper = {}
        for s, a, ww, scale, bias, out, res in fcalls:
            if conv_key(s) in fper:
                continue
            tt = timed(lambda: B.qail_w4a4_conv_u4(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww,
                                                   scale, bias, 0.37, out, res_u4=res, res_scale=0.11, stream=sh), 50, settle=True)
            fper[conv_key(s)] = shape_line(s, tt, 0.5)
        gs = torch.cuda.Stream()
        with torch.cuda.stream(gs):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=gs):
                for s, a, ww, scale, bias, out, res in fcalls:
                    B.qail_w4a4_conv_u4(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww, scale, bias,
                                        0.37, out, res_u4=res, res_scale=0.11, stream=gs.cuda_stream)
        torch.cuda.synchronize()
        tgf = timed(graph.replay, 20, settle=True)
        del graph
        # the same body with the two convolutions that open each down-sampling block (3x3 stride 2 and the
        # 1x1 projection: same input, no dependence) in one qail_w4a4_conv_batch launch: 32 launches
        plan, i = [], 0
        while i < len(fcalls):
            s = fcalls[i][0]
            nxt = fcalls[i + 1][0] if i + 1 < len(fcalls) else None
            if nxt is not None and s.KH == 3 and s.stride == 2 and nxt.KH == 1 and nxt.stride == 2 and nxt.Cin == s.Cin:
                ents = []
                for s_, a_, ww_, scale_, bias_, out_, res_ in fcalls[i:i + 2]:
                    ents.append(dict(B=s_.B, H=s_.H, W=s_.W, Cin=s_.Cin, Cout=s_.Cout, KH=s_.KH, KW=s_.KW, stride=s_.stride,
                                     pad=s_.pad, a_u4=a_, w_s4=ww_, scale=scale_, bias=bias_, out_u4=out_, s_out=0.37))
                plan.append(("pair", B.make_conv_items(ents)))
                i += 2
            else:
                plan.append(("one", fcalls[i]))
                i += 1

        def paired_body():
            for kind, v in plan:
                if kind == "pair":
                    B.qail_w4a4_conv_batch(v, 2, stream=sh)
                else:
                    s, a, ww, scale, bias, out, res = v
                    B.qail_w4a4_conv_u4(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a, ww, scale, bias,
                                        0.37, out, res_u4=res, res_scale=0.11, stream=sh)
        tp_ = timed(paired_body, 20, settle=True)
        extra["w4a4_resnet34_b32_fused_u4"] = {"ms_per_pass": round(tf_ * 1e3, 4),
                                               "TOPs": round(tot_ops / tf_ / 1e12, 1),
                                               "frac_int8_peak": round(tot_ops / tf_ / 1e12 / INT8_PEAK_TOPS, 4),
                                               "calls": len(fcalls), "ms_per_pass_graph_replay": round(tgf * 1e3, 4),
                                               "ms_per_pass_paired_launches": round(tp_ * 1e3, 4),
                                               "launches_paired": len(plan),
                                               "per_shape": fper,
                                               "aggregate": conv_summary([c[0] for c in fcalls], fper, tf_, 0.5)}
        del fcalls

    if want("conv256"):
        # the same body at batch 256 with the fused 4-bit output: the matrix-core-bound regime of the
        # same kernels (batch 32 above is bound by per-call fixed cost); NOT the configuration's batch.
        # One code tensor per input shape, one output tensor per output shape.
        rng = np.random.default_rng(synth.seed_for(3, 0, 7))
        convs256 = synth.resnet34_convs(256)
        big, ops256, cache_a, cache_o = [], 0, {}, {}
        for s2 in convs256:
            ka, ko = (s2.H, s2.Cin), (s2.M, s2.Cout)
            if ka not in cache_a:
                cache_a[ka] = dev(rng.integers(0, 2 ** 32, size=s2.B * s2.H * s2.W * s2.Cin // 8,
                                               dtype=np.uint64).astype(np.uint32))
            if ko not in cache_o:
                cache_o[ko] = torch.empty(s2.M * s2.Cout // 8, dtype=torch.int32, device="cuda")
            w2 = dev(rng.integers(0, 2 ** 32, size=s2.Cout * s2.K // 8, dtype=np.uint64).astype(np.uint32))
            sc2 = torch.full((s2.Cout,), 1e-3, dtype=torch.float32, device="cuda")
            bi2 = torch.zeros(s2.Cout, dtype=torch.float32, device="cuda")
            big.append((s2, cache_a[ka], w2, sc2, bi2, cache_o[ko]))
            ops256 += s2.ops

        def body256():
            for s2, a2, w2, sc2, bi2, o2 in big:
                B.qail_w4a4_conv_u4(s2.B, s2.H, s2.W, s2.Cin, s2.Cout, s2.KH, s2.KW, s2.stride, s2.pad, a2, w2, sc2, bi2,
                                    0.37, o2, stream=sh)
        t256 = timed(body256, 5, settle=True)
        per256 = {}
        for s2, a2, w2, sc2, bi2, o2 in big:
            if conv_key(s2) in per256:
                continue
            tt = timed(lambda: B.qail_w4a4_conv_u4(s2.B, s2.H, s2.W, s2.Cin, s2.Cout, s2.KH, s2.KW, s2.stride, s2.pad,
                                                   a2, w2, sc2, bi2, 0.37, o2, stream=sh), 10, settle=True)
            per256[conv_key(s2)] = shape_line(s2, tt, 0.5)
        extra["w4a4_resnet34_b256_fused_u4"] = {"ms_per_pass": round(t256 * 1e3, 4),
                                                "TOPs": round(ops256 / t256 / 1e12, 1),
                                                "frac_int8_peak": round(ops256 / t256 / 1e12 / INT8_PEAK_TOPS, 4),
                                                "calls": len(big), "per_shape": per256,
                                                "aggregate": conv_summary([c[0] for c in big], per256, t256, 0.5),
                                                "note": "saturating batch, not the configuration's batch of 32"}
        del big, cache_a, cache_o

    if want("w8"):
        # 8-bit variants: the same 35 conv calls as W8A8, and the decode layer with 8-bit weights only
        calls = conv32_calls()
        tot_ops = sum(c[0].ops for c in calls)
        rng = np.random.default_rng(synth.seed_for(3, 0, 8))
        c8 = []
        for s, a, ww, scale, bias, y in calls:
            a8 = dev(rng.integers(0, 2 ** 32, size=s.B * s.H * s.W * s.Cin // 4, dtype=np.uint64).astype(np.uint32))
            w8 = dev(rng.integers(0, 2 ** 32, size=s.Cout * s.K // 4, dtype=np.uint64).astype(np.uint32))
            c8.append((s, a8, w8, scale, bias, y))

        def body8():
            for s, a8, w8, scale, bias, y in c8:
                B.qail_w8a8_gemm(s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, a8, w8,
                                 scale=scale, bias=bias, y_out=y, stream=sh)
        t8 = timed(body8, 20, settle=True)
        extra["w8a8_resnet34_b32"] = {"ms_per_pass": round(t8 * 1e3, 4), "TOPs": round(tot_ops / t8 / 1e12, 1),
                                      "frac_int8_peak": round(tot_ops / t8 / 1e12 / INT8_PEAK_TOPS, 4), "calls": len(c8)}
        del c8
        # four distinct layers of random codes (0.8 GB), cycled, so the last-level cache cannot serve the weights
        L8 = 4
        w8ls = []
        for l in range(L8):
            w8l = []
            for i, (name, N, K) in enumerate(shapes):
                q8 = torch.randint(-2 ** 31, 2 ** 31 - 1, (N * K // 4,), dtype=torch.int32, device="cuda")
                s8 = torch.full((N * (K // GROUP),), 0x1C00, dtype=torch.int16, device="cuda")
                w8l.append((N, K, q8, s8, dec[0][1][i]["x"], torch.empty(N, dtype=torch.int16, device="cuda")))
            w8ls.append(w8l)
        c8l = [0]

        def layer8():
            for N, K, q8, s8, x8, y8 in w8ls[c8l[0] % L8]:
                B.qail_w8a16_linear(N, K, GROUP, q8, s8, x8, y8, 1, stream=sh)
            c8l[0] += 1
        tl8 = timed(layer8, 200)
        b8 = sum(N * K + N * (K // GROUP) * 2 + 2 * (N + K) for N, K, *_ in w8ls[0])
        it8 = [B.make_w8a16_items([dict(N=N, K=K, group_size=GROUP, qweight=q8, scales=s8, x=x8, y=y8)
                                   for N, K, q8, s8, x8, y8 in w8l], 1) for w8l in w8ls]

        def layer8b():
            B.qail_w8a16_linear_batch(it8[c8l[0] % L8], 4, 1, None, sh)
            c8l[0] += 1
        tb8 = timed(layer8b, 200)
        extra["w8a16_decode_layer"] = {"us_per_layer": round(tb8 * 1e6, 2), "GBps": round(b8 / tb8 / 1e9, 1),
                                       "bytes": b8, "launches_per_layer": 1,
                                       "us_per_layer_one_launch_per_linear": round(tl8 * 1e6, 2),
                                       "note": f"{L8} distinct layers cycled"}
        # the same layer at M > 1, one batched call per layer: the small-batch streaming kernel with byte
        # weights up to M = 16, the byte-code instantiation of the matrix-core GEMM above
        w8m = {}
        for M8 in (4, 16, 288, 1024):
            xs8 = [dev(synth.llm_activation_bf16(M8, K, synth.seed_for(1, i, 1))) for i, (_, N, K) in enumerate(shapes)]
            its = []
            for w8l in w8ls:
                its.append(B.make_w8a16_items([dict(N=N, K=K, group_size=GROUP, qweight=q8, scales=s8, x=xs8[i],
                                                    y=torch.empty(M8 * N, dtype=torch.int16, device="cuda"))
                                               for i, (N, K, q8, s8, x8, y8) in enumerate(w8l)], M8))
            nws8 = B.qail_w8a16_batch_workspace(its[0], 4, M8)
            ws8 = torch.empty(nws8, dtype=torch.uint8, device="cuda") if nws8 else None
            c8m = [0]

            def layer8m():
                B.qail_w8a16_linear_batch(its[c8m[0] % L8], 4, M8, ws8, sh)
                c8m[0] += 1
            tm = timed(layer8m, 20, settle=M8 > 16)
            tf8 = sum(2.0 * M8 * N * K for _, N, K in shapes) / tm / 1e12
            w8m[f"M={M8}"] = {"us_per_layer": round(tm * 1e6, 1), "TFLOPs": round(tf8, 1),
                              "frac_f16_peak": round(tf8 / BF16_PEAK_TFLOPS, 4),
                              "GBps_weights": round((b8 - sum(2 * (N + K) for _, N, K in shapes)) / tm / 1e9, 1),
                              "kernel": "small-batch stream" if M8 <= 16 else "matrix-core GEMM"}
            del its, xs8, ws8
        extra["w8a16_layer_batched"] = w8m
        del w8ls, it8

    if want("train"):
        # training-side operators (HBM-bound elementwise / reduction kernels): GB/s of bytes touched
        tr = {}
        Nq, Kq = shapes[0][1], shapes[0][2]
        wq_ = torch.randn(Nq, Kq, dtype=torch.float32, device="cuda") * 0.02
        wh_ = torch.empty_like(wq_)
        tt = timed(lambda: B.qail_fake_quant_w4(wq_, GROUP, wh_), 20)
        tr["fake_quant_w4_12288x4096"] = {"us": round(tt * 1e6, 1), "GBps": round(2 * wq_.numel() * 4 / tt / 1e9, 1)}
        # the offline quantise-and-pack of the same matrix: 4 B read, 0.52 B written per weight
        qb_, sb_, zb_ = B.qail_packed_sizes(Nq, Kq, GROUP, B.QAIL_W4_ASYM_GROUP)
        qq_ = torch.empty(qb_ // 4, dtype=torch.int32, device="cuda")
        sq_ = torch.empty(sb_ // 2, dtype=torch.int16, device="cuda")
        zq_ = torch.empty(zb_ // 4, dtype=torch.int32, device="cuda")
        tt = timed(lambda: B.qail_quantize_weights(wq_, GROUP, B.QAIL_W4_ASYM_GROUP, qq_, sq_, zq_), 20)
        tr["quantize_pack_w4_12288x4096"] = {"us": round(tt * 1e6, 1),
                                             "GBps": round((wq_.numel() * 4 + qb_ + sb_ + zb_) / tt / 1e9, 1)}
        del qq_, sq_, zq_
        sdev = torch.full((1,), 0.01, dtype=torch.float32, device="cuda")
        dsd = torch.zeros(1, dtype=torch.float32, device="cuda")
        wsl_ = torch.empty(B.qail_lsq_backward_workspace(), dtype=torch.uint8, device="cuda")
        tt = timed(lambda: B.qail_lsq_forward(wq_, sdev, -8, 7, wh_), 20)
        tr["lsq_forward_50M"] = {"us": round(tt * 1e6, 1), "GBps": round(2 * wq_.numel() * 4 / tt / 1e9, 1)}
        dv_ = torch.empty_like(wq_)
        tt = timed(lambda: B.qail_lsq_backward(wq_, wh_, sdev, -8, 7, 1e-4, dv_, dsd, wsl_), 20)
        tr["lsq_backward_50M"] = {"us": round(tt * 1e6, 1), "GBps": round(3 * wq_.numel() * 4 / tt / 1e9, 1)}
        lq_ = torch.randn(1024, 32000, dtype=torch.float32, device="cuda")
        lf_ = torch.randn(1024, 32000, dtype=torch.float32, device="cuda")
        gq_ = torch.empty_like(lq_)
        wsq_ = torch.empty(1024, dtype=torch.float32, device="cuda")
        tt = timed(lambda: B.qail_qbc_loss(lq_, lf_, dsd, gq_, wsq_), 20)
        tr["qbc_loss_grad_1024x32000"] = {"us": round(tt * 1e6, 1), "GBps": round(3 * lq_.numel() * 4 / tt / 1e9, 1)}
        extra["train_ops"] = tr
        del wq_, wh_, dv_, lq_, lf_, gq_

    if want("cpu_extra") and not args.no_cpu:
        # The oracle timed on this machine's host cores for the other two hot paths, in their own units, on
        # bounded samples (the headline's cpu_baseline below stays the decode layer): one convolution
        # shape per encoder stage (16 images each, exact integer GEMM through float64 BLAS, im2col
        # included) and one prefill linear (out projection, M = 288: unpack + dequantise + fp64 matmul).
        from oracle import qail_oracle as O
        cpu = {}
        rng = np.random.default_rng(synth.seed_for(3, 0, 9))
        for s in synth.resnet34_convs(16):
            if not (s.KH == 3 and s.stride == 1 and s.Cin == s.Cout) or conv_key(s) in cpu:
                continue
            aw = rng.integers(0, 2 ** 32, size=(s.B, s.H, s.W, s.Cin // 8), dtype=np.uint64).astype(np.uint32)
            ww = rng.integers(0, 2 ** 32, size=(s.Cout, s.K // 8), dtype=np.uint64).astype(np.uint32)
            c0, w0 = time.process_time(), time.perf_counter()
            O.w4a4_conv_acc(aw, ww, s.B, s.H, s.W, s.Cin, s.Cout, s.KH, s.KW, s.stride, s.pad, use_blas=True)
            cs, ws_ = time.process_time() - c0, time.perf_counter() - w0
            cpu[conv_key(s)] = {"TOPs": round(s.ops / ws_ / 1e12, 5), "s": round(ws_, 3), "images": s.B,
                                "cores": max(1, int(round(cs / ws_)))}
        name, N, K = shapes[1]
        e = dec[0][1][1]
        xb = synth.llm_activation_bf16(288, K, synth.seed_for(2, 1, 1), outlier_frac=0.005)
        qw_h = e["qweight"].cpu().numpy().view(np.uint32).reshape(N, K // 8)
        sc_h = e["scales"].cpu().numpy().view(np.float16).reshape(N, K // GROUP)
        zr_h = e["zeros"].cpu().numpy().view(np.uint32).reshape(N, -1)
        c0, w0 = time.process_time(), time.perf_counter()
        O.w4a16_linear(xb, qw_h, sc_h, zr_h, GROUP)
        cs, ws_ = time.process_time() - c0, time.perf_counter() - w0
        cpu[f"{name}_M288"] = {"TFLOPs": round(2.0 * 288 * N * K / ws_ / 1e12, 5), "s": round(ws_, 3),
                               "cores": max(1, int(round(cs / ws_)))}
        cpu["note"] = f"numpy oracle on the host ({os.cpu_count()} logical CPUs), kind = oracle, not tuned"
        extra["cpu_oracle_other_paths"] = cpu

    if extra:
        # what a decoder actually gets, beside the headline (whose four linears share one launch as
        # independent items): each linear launched alone, and the 32-layer walk with every linear
        # waiting for the one before it
        beside = {}
        if "decode_single_linear" in extra:
            beside["single_linear_frac_hbm_peak"] = {k: v["frac_hbm_peak"] for k, v in extra["decode_single_linear"].items()}
        if "decode_stack" in extra:
            st_ = extra["decode_stack"]
            beside["decode_stack_tokens_per_s_M1"] = {
                "one call per layer (independent linears)": st_["M=1"]["tokens_per_s"],
                "one launch per linear (dependent)": st_["M=1, one launch per linear"]["tokens_per_s"],
                "chained in one launch per 32 linears (dependent)":
                    st_["M=1, dependent linears chained in one launch per 32"]["tokens_per_s"],
                "bound at 8 TB/s": 2378}
        if beside:
            result["beside_the_headline"] = beside
        result["extra"] = extra
        log("[bench] extra:", json.dumps(extra))

    # ---------------------------------------------------------- CPU baseline
    if not args.no_cpu:
        from oracle import qail_oracle as O
        host = []
        for l in range(min(L, 8)):
            for i, (_, N, K) in enumerate(shapes):
                e = dec[l][1][i]
                host.append((e["qweight"].cpu().numpy().view(np.uint32).reshape(N, K // 8),
                             e["scales"].cpu().numpy().view(np.float16).reshape(N, K // GROUP),
                             e["zeros"].cpu().numpy().view(np.uint32).reshape(N, -1),
                             e["x"].cpu().numpy().view(np.uint16).reshape(1, K)))
        # bounded sample: whole layers until about 15 s of wall time have been spent
        done, c0, w0 = 0, time.process_time(), time.perf_counter()
        while done < 64 and time.perf_counter() - w0 < 15.0:
            for qw, sc, zr, xb in host[(done % min(L, 8)) * 4:(done % min(L, 8)) * 4 + 4]:
                O.w4a16_linear(xb, qw, sc, zr, GROUP)
            done += 1
        cpu_s, wall_s = time.process_time() - c0, time.perf_counter() - w0
        result["cpu_baseline"] = {
            "value": round(done * bytes_per_step / wall_s / 1e9, 4),
            "unit": "GB/s",
            "cores": max(1, int(round(cpu_s / wall_s))),
            "kind": "oracle",
            "sample": f"{done} decoder layers (the same four linears each, M=1) through the numpy oracle: "
                      f"unpack + dequantise + fp64 matmul, {wall_s:.1f} s wall; host has {os.cpu_count()} logical CPUs",
        }

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
