#!/usr/bin/env python3
"""Benchmark of the fused-subgraph hot path on one MI355X.

A "step" is one pass of the whole hot path: the five benchmark subgraphs (two inverted
residuals, the 3x3 -> 3x3 chain, the FFN chain, the attention chain) each run once as its fused
kernel, inputs already resident in HBM.  The subgraphs are independent of one another, so each is
launched on a HIP stream of its own (--streams, default one per subgraph) and the GPU overlaps them:
the small inverted-residual launches fill compute units the others leave idle.  --streams 1 runs
the step back to back on one stream; that figure is reported too (one_stream).  The timed region is
exactly --steps steps between two torch.cuda.synchronize() calls.  One JSON line is printed:

  value        algorithmic TFLOP/s of a step (multiply-adds of the complex operators only)
  per_config   fused / un-fused (one kernel per operator, and epilogue-fused) microseconds,
               TFLOP/s, roofline fraction and speed-ups for each of the five configurations
  roofline     dominant kernel (the fused FFN kernel): algorithmic FLOPs per launch divided by its
               average duration, measured with HIP events recorded around that kernel on its
               launch stream during the timed region, against the dense bf16 MFMA peak
  cpu_baseline the fp64 CPU oracle timed on the host cores on the same step
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3       # fp32 MFMA / vector
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch at the benchmark shape: FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc, scaled by a 256 MiB
# copy (profiles/bench_all_fused_subgraphs.md): the fused FFN streaming kernel alone, and the whole entry point
# (streaming kernel + partial-sum reduction).  Counters cannot be read inside this run; the two figures are
# re-measured whenever the kernels change.
FFN_TRAFFIC_BYTES = 85078851
FFN_TRAFFIC_BYTES_PER_CALL = 138463115


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--detail-iters", type=int, default=100, help="launches per variant in the per-config table")
    ap.add_argument("--streams", type=int, default=5,
                    help="HIP streams (default priority) the subgraphs of a step are spread over; 1 = back to back")
    ap.add_argument("--no-one-stream", action="store_true",
                    help="skip the second, back-to-back pass on one stream (profiling aid: a kernel trace then "
                         "holds the timed region only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-detail", action="store_true")
    ap.add_argument("--only", type=int, default=-1, help="run only this configuration in the timed step (profiling aid)")
    ap.add_argument("--copy-bytes", type=int, default=0,
                    help="calibration aid: instead of the benchmark, run the library's plain elementwise kernel "
                         "(ago_scale, alpha = 1, fp32) over this many bytes --steps times; it reads and writes "
                         "exactly that many bytes, which scales the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the cold-cache timings and launch floors of the per-config table (profiling aid)")
    ap.add_argument("--variants", default="fused,u1,u2,packed",
                    help="which variants the per-config table runs (profiling aid: counters of one variant alone)")
    ap.add_argument("--vendor-context", action="store_true",
                    help="also time the complex operators of the configurations as PyTorch reaches them in the vendor "
                         "libraries (matmul, conv2d, scaled_dot_product_attention), each captured ten times into a HIP "
                         "graph so that no framework dispatch time is included; context for how good the un-fused "
                         "baselines are, reported under 'vendor_context', never part of 'value'")
    ap.add_argument("--tile-config", default="",
                    help="tile-size sweep aid: comma-separated op=id pairs (op: invres, chain, ffn, attn) passed to "
                         "ago_set_tile_config before anything runs; the default is the library's built-in choice")
    return ap.parse_args()


def vendor_context(torch):
    """The benchmark's complex operators through PyTorch's vendor-library calls, us per call (HIP-graph replays)."""
    F = torch.nn.functional
    bf = torch.bfloat16
    torch.backends.cudnn.benchmark = True        # let the convolution library time its own candidates first

    def us(fn):
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            for _ in range(5):
                fn()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                for _ in range(10):
                    fn()
        torch.cuda.synchronize()
        for _ in range(3):
            g.replay()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(20):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        return round(a.elapsed_time(b) / 200 * 1e3, 2)

    res = {"how": "torch %s; each operator captured 10x into a HIP graph, 20 replays timed" % torch.__version__}
    for m, k, n in [(2048, 768, 3072), (2048, 3072, 768), (196, 192, 32), (3136, 24, 144), (784, 144, 32)]:
        a, b = torch.randn(m, k, device="cuda", dtype=bf), torch.randn(k, n, device="cuda", dtype=bf)
        c = torch.empty(m, n, device="cuda", dtype=bf)
        res["matmul_%dx%dx%d_us" % (m, k, n)] = us(lambda: torch.matmul(a, b, out=c))
    x = torch.randn(2048, 768, device="cuda", dtype=bf)
    w1, b1 = torch.randn(3072, 768, device="cuda", dtype=bf), torch.randn(3072, device="cuda", dtype=bf)
    w2, b2 = torch.randn(768, 3072, device="cuda", dtype=bf), torch.randn(768, device="cuda", dtype=bf)
    res["linear_gelu_linear_2048x768x3072_us"] = us(lambda: F.linear(F.gelu(F.linear(x, w1, b1), approximate="tanh"), w2, b2))
    q = torch.randn(8, 12, 384, 64, device="cuda", dtype=bf)
    kk, v = torch.randn_like(q), torch.randn_like(q)
    res["sdpa_8x12x384x64_us"] = us(lambda: F.scaled_dot_product_attention(q, kk, v))
    xc = torch.randn(8, 64, 56, 56, device="cuda", dtype=bf).contiguous(memory_format=torch.channels_last)
    wc = torch.randn(64, 64, 3, 3, device="cuda", dtype=bf).contiguous(memory_format=torch.channels_last)
    res["conv3x3_8x56x56x64_nhwc_us"] = us(lambda: F.conv2d(xc, wc, padding=1))
    xd = torch.randn(1, 144, 56, 56, device="cuda", dtype=bf).contiguous(memory_format=torch.channels_last)
    wd = torch.randn(144, 1, 3, 3, device="cuda", dtype=bf)
    res["dwconv3x3_s2_56x56x144_us"] = us(lambda: F.conv2d(xd, wd, padding=1, stride=2, groups=144))
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2212_01005_amd import binding as ago, runner

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)

    if args.copy_bytes > 0:
        n = args.copy_bytes // 4 // 8 * 8
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            ago.ago_scale(src, dst, 1.0)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": n * 4, "copy_bytes_written": n * 4, "launches": args.steps}))
        return

    tile_cfg = {}
    for item in filter(None, args.tile_config.split(",")):
        name, cid = item.split("=")
        op = {"invres": ago.OP_FUSED_INVRES, "chain": ago.OP_FUSED_CONV_CHAIN, "ffn": ago.OP_FUSED_FFN,
              "attn": ago.OP_FUSED_ATTN}[name]
        if ago.set_tile_config(op, int(cid)) != 0:
            sys.exit("bench.py: unknown tile configuration %s" % item)
        tile_cfg[name] = int(cid)

    idxs = list(range(5)) if args.only < 0 else [args.only]
    cases = [wl.baseline_case(i) for i in idxs]
    state = []
    for c in cases:
        t = runner.to_device(c)
        state.append((c, t, runner.alloc_output(c), runner.alloc_workspace(c, fused=True)))

    # arguments (stream included) are marshalled once: a step is five C calls on resident buffers
    def prepare_step(n_streams):
        if n_streams <= 1:
            return [runner.prepare_fused(c, t, y, ws) for c, t, y, ws in state]
        streams = [torch.cuda.Stream() for _ in range(min(n_streams, len(state)))]     # default priority
        out = []
        for i, (c, t, y, ws) in enumerate(state):
            with torch.cuda.stream(streams[i % len(streams)]):
                out.append((c.flops(), runner.prepare_fused(c, t, y, ws)))
        # largest subgraph first: the launch that needs every compute unit goes out before the small
        # ones have spread over the chip (worth about 4% of the step against the listed order)
        out.sort(key=lambda p: -p[0])
        return [launch for _, launch in out]

    def timed(launches, steps, sample_mask):
        """steps passes; the library brackets the kernels in sample_mask with an event pair on every
        EVENT_EVERY-th step.  Returns milliseconds per step."""
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for i in range(steps):
            if i % EVENT_EVERY == 0:
                ago.profile_select(sample_mask)
                for launch in launches:
                    launch()
                ago.profile_select(0)
            else:
                for launch in launches:
                    launch()
        torch.cuda.synchronize()
        return (time.perf_counter() - t_start) * 1e3 / steps

    launches = prepare_step(args.streams)
    for _ in range(args.warmup):
        for launch in launches:
            launch()
    torch.cuda.synchronize()

    # The roofline needs the dominant kernel's duration from inside the timed region: the library
    # records a HIP event pair around that kernel on every EVENT_EVERY-th step (a pair costs about
    # 4.5 us of stream time, so bracketing every launch would inflate the step it measures).
    EVENT_EVERY = 10
    ago.profile_enable(min(args.steps // EVENT_EVERY + 1, 4096))
    ago.profile_select(0)
    ffn_mask = 1 << ago.OP_FUSED_FFN
    ms_per_step = timed(launches, args.steps, ffn_mask)

    first_kernel_ms = {}

    def read_kernel_ms():
        out = {}
        for op in range(4):
            tot, first, n = ago.profile_read_split(op)
            if n:
                out[op] = tot / n
                first_kernel_ms[op] = first / n
        return out

    kernel_ms = read_kernel_ms()
    ffn_first_ms = first_kernel_ms.get(ago.OP_FUSED_FFN)
    # the same steps back to back on one stream (not the headline: what the overlap is worth, and the
    # dominant kernel's duration with the chip to itself)
    one_stream = None
    if args.streams > 1 and not args.no_one_stream:
        serial = prepare_step(1)
        for _ in range(args.warmup):
            for launch in serial:
                launch()
        ago.profile_enable(min(args.steps // EVENT_EVERY + 1, 4096))
        ago.profile_select(0)
        ms_serial = timed(serial, args.steps, ffn_mask)
        one_stream = {"ms_per_step": round(ms_serial, 5), "kernel_ms": read_kernel_ms()}
        if ago.OP_FUSED_FFN in first_kernel_ms:
            one_stream["first_ms"] = first_kernel_ms[ago.OP_FUSED_FFN]
    ago.profile_enable(0)
    ago.profile_select(0xF)
    ev_overhead_ms = ago.profile_event_overhead_ms(64)   # what an empty event pair reads

    # ---- measured peaks of this GPU (outside the timed region): a plain copy of 2 x 512 MiB (the library's
    # elementwise kernel with alpha = 1) and matrix-instruction-only kernels, timed with events
    def ev_ms(fn, iters):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    n_peak = 512 * 1024 * 1024 // 4
    pk_src = torch.ones(n_peak, dtype=torch.float32, device="cuda")
    pk_dst = torch.empty_like(pk_src)
    copy_ms = ev_ms(ago.prepare(ago.ago_scale, pk_src, pk_dst, 1.0), 5)
    del pk_src, pk_dst
    mf_out = torch.empty(1024 * 1024, dtype=torch.float32, device="cuda")
    fl_bf16 = ago.bench_mfma_kernel(ago.BF16, 4096, mf_out)
    mfma_bf16_ms = ev_ms(lambda: ago.bench_mfma_kernel(ago.BF16, 4096, mf_out), 5)
    fl_f32 = ago.bench_mfma_kernel(ago.F32, 2048, mf_out)
    mfma_f32_ms = ev_ms(lambda: ago.bench_mfma_kernel(ago.F32, 2048, mf_out), 5)
    measured = {"hbm_copy_gbs": round(2 * n_peak * 4 / (copy_ms * 1e-3) / 1e9, 1),
                "mfma_bf16_tflops": round(fl_bf16 / (mfma_bf16_ms * 1e-3) / 1e12, 1),
                "mfma_f32_tflops": round(fl_f32 / (mfma_f32_ms * 1e-3) / 1e12, 1),
                "how": "1 GiB copy (512 MiB read + 512 MiB written) by the library's elementwise kernel; "
                       "matrix-instruction-only kernels, 8 waves x 6 accumulators per compute unit"}

    flops_step = sum(c.flops() for c in cases)
    value = flops_step / (ms_per_step * 1e-3) / 1e12

    # ---- roofline of the dominant kernel (fused FFN) -----------------------------------
    roofline = None
    ffn = [c for c in cases if type(c).__name__ == "FfnCase"]
    if ffn and ago.OP_FUSED_FFN in kernel_ms:
        # The library records events before the streaming kernel, between it and the partial-sum reduction, and
        # after the reduction.  An event pair reads the bracketed work plus the fixed cost of the pair itself.
        call_s = (kernel_ms[ago.OP_FUSED_FFN] - ev_overhead_ms) * 1e-3
        dur_s = ((ffn_first_ms if ffn_first_ms else kernel_ms[ago.OP_FUSED_FFN]) - ev_overhead_ms) * 1e-3
        ach = ffn[0].flops() / dur_s / 1e12
        ach_call = ffn[0].flops() / call_s / 1e12
        roofline = {"bound": "mfma", "kernel": "fused_ffn_stream_kernel", "achieved": round(ach, 2),
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                    "measured_peak": measured["mfma_bf16_tflops"],
                    "frac_measured": round(ach / measured["mfma_bf16_tflops"], 4),
                    "avg_kernel_us": round(dur_s * 1e6, 2),
                    "per_call": {"what": "the whole ago_fused_ffn call: streaming kernel + partial-sum reduction kernel",
                                 "avg_us": round(call_s * 1e6, 2), "achieved": round(ach_call, 2),
                                 "frac": round(ach_call / PEAK_BF16_TFLOPS, 4),
                                 "frac_measured": round(ach_call / measured["mfma_bf16_tflops"], 4),
                                 "traffic": FFN_TRAFFIC_BYTES_PER_CALL},
                    "event_overhead_us": round(ev_overhead_ms * 1e3, 2),
                    "event_sampling": "every %dth step of the timed region" % EVENT_EVERY,
                    "traffic": FFN_TRAFFIC_BYTES}
        if one_stream and ago.OP_FUSED_FFN in one_stream["kernel_ms"]:
            # the same kernel with the chip to itself (steps back to back on one stream)
            d1 = (one_stream.get("first_ms", one_stream["kernel_ms"][ago.OP_FUSED_FFN]) - ev_overhead_ms) * 1e-3
            a1 = ffn[0].flops() / d1 / 1e12
            roofline["one_stream"] = {"avg_kernel_us": round(d1 * 1e6, 2), "achieved": round(a1, 2),
                                      "frac": round(a1 / PEAK_BF16_TFLOPS, 4)}
    if one_stream:
        one_stream = {"ms_per_step": one_stream["ms_per_step"],
                      "value": round(flops_step / (one_stream["ms_per_step"] * 1e-3) / 1e12, 3)}

    # ---- per-configuration table: fused vs un-fused, device time by events ----------------
    per_config = []
    if not args.no_detail:
        def time_us(fn, iters):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(iters):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / iters

        # cold timing: evict the L2s and the 256 MB Infinity Cache with a 2 x 768 MiB copy before every
        # launch, then time that one launch with an event pair (minus what an empty pair reads)
        flush_n = 768 * 1024 * 1024 // 4
        flush_src = torch.ones(flush_n, dtype=torch.float32, device="cuda")
        flush_dst = torch.empty_like(flush_src)

        def cold_us(fn, iters=12, flush=True):
            tot, best = 0.0, 1e30
            for _ in range(iters):
                if flush:
                    ago.ago_scale(flush_src, flush_dst, 1.0)
                else:
                    torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                torch.cuda.synchronize()
                us = (e0.elapsed_time(e1) - ev_overhead_ms) * 1e3
                tot += us
                best = min(best, us)
            return tot / iters, best

        fused_ops = {"InvresCase": ago.OP_FUSED_INVRES, "ChainCase": ago.OP_FUSED_CONV_CHAIN,
                     "FfnCase": ago.OP_FUSED_FFN, "AttnCase": ago.OP_FUSED_ATTN}
        for (c, t, y, ws) in state:
            wsu = runner.alloc_workspace(c, fused=False)
            yu = runner.alloc_output(c)
            variants = args.variants.split(",")
            fused_us = time_us(runner.prepare_fused(c, t, y, ws), args.detail_iters) if "fused" in variants else float("nan")
            u1_us = time_us(runner.prepare_unfused(c, t, yu, wsu, 0), args.detail_iters) if "u1" in variants else float("nan")
            u2_us = time_us(runner.prepare_unfused(c, t, yu, wsu, 1), args.detail_iters) if "u2" in variants else float("nan")
            launch = runner.prepare_fused(c, t, y, ws)
            nan = float("nan")
            cold_avg, cold_min = (nan, nan) if args.no_cold else cold_us(launch)
            warm_avg, _ = (nan, nan) if args.no_cold else cold_us(launch, flush=False)   # same method, caches warm
            # launch floors: an empty kernel with the fused kernel's grid and workgroup size, and a plain
            # copy kernel moving the configuration's algorithmic bytes (half read, half written)
            grid, block = ago.profile_last_launch(fused_ops[type(c).__name__])
            stream = torch.cuda.current_stream().cuda_stream
            empty_us = copy_us = nan
            if not args.no_cold:
                empty_us = time_us(lambda: ago.lib.ago_bench_empty_kernel(grid, block, stream), args.detail_iters)
                n_copy = max(8, c.alg_bytes() // 8 // 8 * 8)
                cp_src = torch.ones(n_copy, dtype=torch.float32, device="cuda")
                cp_dst = torch.empty_like(cp_src)
                copy_us = time_us(ago.prepare(ago.ago_scale, cp_src, cp_dst, 1.0), args.detail_iters)
            tf = c.flops() / (fused_us * 1e-6) / 1e12
            peak = PEAK_F32_TFLOPS if c.dtype == "f32" else PEAK_BF16_TFLOPS
            t_mfma = c.flops() / (peak * 1e12)
            t_hbm = c.alg_bytes() / (PEAK_HBM_GBS * 1e9)
            bound = "mfma" if t_mfma >= t_hbm else "hbm"
            peak_m = measured["mfma_f32_tflops"] if c.dtype == "f32" else measured["mfma_bf16_tflops"]
            t_meas = max(c.flops() / (peak_m * 1e12), c.alg_bytes() / (measured["hbm_copy_gbs"] * 1e9))
            per_config.append({
                "name": c.name, "dtype": c.dtype, "fused_us": round(fused_us, 2),
                "unfused_per_op_us": round(u1_us, 2), "unfused_epilogue_us": round(u2_us, 2),
                "tflops": round(tf, 3), "gbs": round(c.alg_bytes() / (fused_us * 1e-6) / 1e9, 1),
                "bound": bound, "roofline_frac": round(max(t_mfma, t_hbm) / (fused_us * 1e-6), 4),
                "roofline_frac_measured_peak": round(t_meas / (fused_us * 1e-6), 4),
                "fused_single_launch_warm_us": round(warm_avg, 2),
                "fused_cold_us": round(cold_avg, 2), "fused_cold_min_us": round(cold_min, 2),
                "roofline_frac_cold": round(max(t_mfma, t_hbm) / (cold_avg * 1e-6), 4),
                "launch": {"grid": grid, "block": block},
                "floor_empty_kernel_us": round(empty_us, 2), "floor_copy_kernel_us": round(copy_us, 2),
                "speedup_vs_per_op": round(u1_us / fused_us, 2),
                "speedup_vs_epilogue": round(u2_us / fused_us, 2),
            })

    # ---- the FFN chain on pre-packed weights (not part of the step: the step keeps the row-major weights the
    # configurations name).  Packing is a separate call, once per weight tensor; its cost is reported.
    packed = None
    packed_y = None
    if not args.no_detail and "packed" in args.variants.split(","):
        for (c, t, y, ws) in state:
            if type(c).__name__ != "FfnCase":
                continue
            w1p = torch.empty(ago.packed_weight_shape(c.K, c.F), device="cuda", dtype=torch.bfloat16)
            w2p = torch.empty(ago.packed_weight_shape(c.F, c.K2), device="cuda", dtype=torch.bfloat16)
            pk1, pk2 = ago.prepare(ago.ago_pack_weight, t["w1"], w1p), ago.prepare(ago.ago_pack_weight, t["w2"], w2p)
            pack_us = time_us(lambda: (pk1(), pk2()), 20)
            wsp = torch.empty(ago.workspace_bytes(ago.OP_FUSED_FFN_PACKED, [c.M, c.K, c.F, c.K2], ago.BF16),
                              dtype=torch.uint8, device="cuda")
            packed_y = runner.alloc_output(c)
            fp = ago.prepare(ago.ago_fused_ffn_packed, t["x"], w1p, t["b1"], w2p, t["b2"], packed_y, ago.ACT_GELU_TANH, wsp)
            f_us = time_us(fp, args.detail_iters)
            # the streaming kernel alone and the whole call, from the library's event pairs around single calls
            ago.profile_enable(64)
            ago.profile_select(1 << ago.OP_FUSED_FFN)
            for _ in range(32):
                fp()
            torch.cuda.synchronize()
            tot, first, n = ago.profile_read_split(ago.OP_FUSED_FFN)
            ago.profile_enable(0)
            ago.profile_select(0xF)
            k_us = (first / max(n, 1) - ev_overhead_ms) * 1e3
            yu = runner.alloc_output(c)
            wsu = runner.alloc_workspace(c, fused=False)
            u_us = time_us(ago.prepare(ago.ago_unfused_ffn_packed, t["x"], w1p, t["b1"], w2p, t["b2"], yu,
                                       ago.ACT_GELU_TANH, wsu), args.detail_iters)
            hid = torch.empty((c.M, c.F), device="cuda", dtype=torch.bfloat16)
            g1_us = time_us(ago.prepare(ago.ago_gemm_packed, t["x"], w1p, t["b1"], hid, ago.ACT_GELU_TANH), args.detail_iters)
            g2_us = time_us(ago.prepare(ago.ago_gemm_packed, hid, w2p, t["b2"], yu, ago.ACT_NONE), args.detail_iters)
            fp()                                   # leave the fused result in packed_y for the oracle check
            torch.cuda.synchronize()
            packed = {"name": c.name, "what": "the same chain with w1, w2 pre-packed into matrix-instruction fragments "
                                              "(ago_pack_weight, once per weight tensor)",
                      "fused_us": round(f_us, 2), "fused_kernel_us": round(k_us, 2),
                      "fused_kernel_tflops": round(c.flops() / (k_us * 1e-6) / 1e12, 1),
                      "fused_kernel_frac": round(c.flops() / (k_us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
                      "fused_call_frac": round(c.flops() / (f_us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
                      "unfused_epilogue_us": round(u_us, 2),
                      "gemm1_us": round(g1_us, 2), "gemm1_frac": round(2.0 * c.M * c.K * c.F / (g1_us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
                      "gemm2_us": round(g2_us, 2), "gemm2_frac": round(2.0 * c.M * c.F * c.K2 / (g2_us * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
                      "pack_once_us": round(pack_us, 2), "speedup_vs_epilogue": round(u_us / f_us, 2)}

    # ---- the two-operator pairs (not part of the step): fused vs operator by operator --------------
    pairs = []
    if not args.no_detail and not args.no_cold and args.only < 0:
        for c in wl.pair_cases():
            if "ragged" in c.name:
                continue
            t = runner.to_device(c)
            y, ws = runner.alloc_output(c), runner.alloc_workspace(c, fused=True)
            scratch = runner.alloc_pair_scratch(c)
            f_us = time_us(runner.prepare_fused(c, t, y, ws), args.detail_iters)
            u_us = time_us(runner.prepare_pair_unfused(c, t, y, scratch), args.detail_iters)
            pairs.append({"name": c.name, "fused_us": round(f_us, 2), "unfused_epilogue_us": round(u_us, 2),
                          "speedup": round(u_us / f_us, 2),
                          "tflops": round(c.flops() / (f_us * 1e-6) / 1e12, 3)})

    # ---- inverted-residual blocks at the layer shapes of a whole network, batch 1 (not part of the step) ----
    blocks = []
    if not args.no_detail and not args.no_cold and args.only < 0:
        for c in wl.network_block_cases(1):
            t = runner.to_device(c)
            y, ws = runner.alloc_output(c), runner.alloc_workspace(c, fused=True)
            wsu = runner.alloc_workspace(c, fused=False)
            f_us = time_us(runner.prepare_fused(c, t, y, ws), args.detail_iters)
            u_us = time_us(runner.prepare_unfused(c, t, y, wsu, True), args.detail_iters)
            plan = ago.fused_invres_plan(c.N, c.H, c.W, c.Cin, c.Cexp, c.Cout, c.stride, c.ksize, ago.BF16,
                                         ws.numel() if ws is not None else 0)
            blocks.append({"name": c.name, "fused_us": round(f_us, 2), "unfused_epilogue_us": round(u_us, 2),
                           "speedup": round(u_us / f_us, 2), "tile": [plan["tile_h"], plan["tile_w"]],
                           "channel_split": plan["split"]})

    # ---- a whole network body through the graph layer (not part of the step): the 16 inverted-residual
    # blocks of a MobileNetV2-style network at batch 1 (112 x 112 x 16 in, 7 x 7 x 320 out), partitioned and
    # lowered to one launch per block, against the same graph run operator by operator; each plan is
    # recorded into a HIP graph, so the figures are kernel time, not Python launch overhead
    network = None
    if not args.no_detail and not args.no_cold and args.only < 0:
        try:                                   # an auxiliary figure must never cost the headline line
            import numpy as np
            from paper_2212_01005_amd import lowering as L
            g = L.Graph([], {}, "bf16")
            cur, cin, seed = g.add("input", name="x", shape=(1, 112, 112, 16)), 16, 22120100 + 5000

            def dev_param(name, shape, sigma, bias=False):
                nonlocal seed
                seed += 1
                v = torch.from_numpy(np.ascontiguousarray(wl.normal(seed, shape, sigma), dtype=np.float32)).to("cuda:0")
                g.params[name] = v if bias else v.to(torch.bfloat16)
                return name

            bi = 0
            for cout, reps, stride in ((24, 2, 2), (32, 3, 2), (64, 4, 2), (96, 3, 1), (160, 3, 2), (320, 1, 1)):
                for r in range(reps):
                    st, cexp, src = (stride if r == 0 else 1), 6 * cin, cur
                    cur = g.add("conv1x1", [cur], w=dev_param("w1_%d" % bi, (cin, cexp), cin ** -0.5))
                    cur = g.add("bias", [cur], b=dev_param("b1_%d" % bi, (cexp,), 0.1, True))
                    cur = g.add("relu6", [cur])
                    cur = g.add("dwconv", [cur], w=dev_param("wd_%d" % bi, (3, 3, cexp), 1.0 / 3), stride=st)
                    cur = g.add("bias", [cur], b=dev_param("bd_%d" % bi, (cexp,), 0.1, True))
                    cur = g.add("relu6", [cur])
                    cur = g.add("conv1x1", [cur], w=dev_param("w2_%d" % bi, (cexp, cout), cexp ** -0.5))
                    cur = g.add("bias", [cur], b=dev_param("b2_%d" % bi, (cout,), 0.1, True))
                    if st == 1 and cin == cout:
                        cur = g.add("add", [cur, src])
                    cin, bi = cout, bi + 1
            x = torch.from_numpy(np.ascontiguousarray(wl.uniform(seed + 1, (1, 112, 112, 16), -1.0, 1.0),
                                                      dtype=np.float32)).to("cuda:0").to(torch.bfloat16)
            network = {"blocks": bi, "operators": len(g.nodes) - 1}
            for key, part in (("fused", L.partition(g, ago)[0]), ("per_op", list(range(len(g.nodes))))):
                ex = L.Executor(g, L.lower(g, part), ago, torch)
                replay, _, _ = ex.capture({"x": x})
                network[key + "_launches"] = len(ex.plan)
                network[key + "_graph_us"] = round(time_us(replay, args.detail_iters), 1)
            network["speedup"] = round(network["per_op_graph_us"] / network["fused_graph_us"], 2)
        except Exception as e:                 # noqa: BLE001
            network = {"error": "%s: %s" % (type(e).__name__, e)}

    # ---- CPU baseline: the oracle as it stands, on the host cores ---------------------------
    cpu = None
    checks = []
    if not args.no_cpu_baseline:
        from oracle import ago_oracle
        ago_oracle.lib()
        # full steps (all configurations once each), repeated until about ten seconds of CPU work or 25
        # passes; run_case regenerates its inputs, so the generation time is measured and subtracted
        # untimed first pass (library load, page faults); its results check what the timed launches left in
        # their output buffers: max |gpu - oracle| / max(|oracle|, rms(oracle)) against the benchmark's bars
        import numpy as np
        for (c, t, y, ws) in state:
            ref = ago_oracle.run_case(c)
            got = runner.to_numpy64(y)
            rms = float(np.sqrt(np.mean(ref ** 2)))
            err = float((np.abs(got - ref) / np.maximum(np.abs(ref), rms if rms > 0 else 1.0)).max())
            checks.append({"name": c.name, "max_rel_err": float("%.3e" % err),
                           "ok": bool(np.all(np.isfinite(got)) and err <= (1e-4 if c.dtype == "f32" else 2e-2))})
            if packed_y is not None and type(c).__name__ == "FfnCase":
                got = runner.to_numpy64(packed_y)
                err = float((np.abs(got - ref) / np.maximum(np.abs(ref), rms if rms > 0 else 1.0)).max())
                checks.append({"name": c.name + " (packed weights)", "max_rel_err": float("%.3e" % err),
                               "ok": bool(np.all(np.isfinite(got)) and err <= 2e-2)})
        gen0 = time.perf_counter()
        for c in cases:
            c.tensors()
        gen = time.perf_counter() - gen0
        passes, spent = 0, 0.0
        while passes < 25 and spent < 10.0:
            tc0 = time.perf_counter()
            for c in cases:
                ago_oracle.run_case(c)
            spent += time.perf_counter() - tc0
            passes += 1
        secs = max(spent / passes - gen, 1e-9)
        cpu = {"value": round(flops_step / secs / 1e12, 5), "unit": "TFLOP/s",
               "cores": ago_oracle.num_threads(), "kind": "oracle",
               "sample": "%d full steps (all %d configurations once each, fp64; %.2f s per step, %.1f s in all)"
                         % (passes, len(cases), secs, spent)}

    vendor = vendor_context(torch) if args.vendor_context else None

    out = {
        "metric": "fused-block TFLOP/s (algorithmic, one pass over the 5 fused subgraphs)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "all 5 BASELINE configs, one fused launch each per step"
                   if args.only < 0 else cases[0].name,
                   "configs": [c.name for c in cases],
                   "streams": max(1, min(args.streams, len(cases))),
                   "tile_config": tile_cfg or "built-in",
                   "note": "config 0 is fp32 storage, configs 1-4 bf16 storage with fp32 accumulation"},
        "roofline": roofline, "measured_peaks": measured, "cpu_baseline": cpu, "one_stream": one_stream,
        "checked_against_oracle": checks,
        "per_config": per_config, "ffn_packed_weights": packed, "pairs": pairs, "network_blocks": blocks, "network_body": network,
        "vendor_context": vendor,
        "fused_kernel_us": {str(k): round(v * 1e3, 2) for k, v in kernel_ms.items()},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
