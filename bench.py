#!/usr/bin/env python3
"""Benchmark of the any4 GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--extras/--no-extras]

A *step* is one pass of the hot path over one decoder layer of Llama-3-8B at M = 1: the four
quantised linears (fused QKV, O, fused gate/up, down), i.e. four any4_gemm launches.  Successive
steps use successive layers of a stack of `--layers` distinct synthetic layers (default 16, 1.9 GB
of packed weights), so every launch streams its weights from HBM and not from the 256 MB
last-level cache, exactly as token generation over a whole model does ("cold" mode; the same steps
on one layer only, whose weights stay in that cache, are reported as `extras.warm_same_buffers`).
W eager warm-up steps, then untimed replays of the captured graph for at least 50 ms (clocks),
then the K timed steps: ONE replay of a HIP graph of exactly K steps (the launch sequence of a
decode step is static), bracketed by synchronisation on both sides.

The one JSON line printed at the end carries the contract fields plus
  roofline      achieved GB/s of the decode GEMM: algorithmic bytes per launch divided by the
                average launch duration, from the HIP events that bracket the timed graph replay
                (stream = torch's current stream, on which the library is launched);
                roofline.shapes: every decode shape of the Llama-3-8B and -70B linears on its own
                (plain and re-laid-out codes, M = 1 / 8 / 16, 3- and 2-bit codes), microseconds
                (median, p10, p90 over replays), GB/s and fraction of the 8 TB/s peak;
                roofline.prefill: the M = 2048 matrix-core path per 8B shape, TFLOP/s and fraction
                of the bf16 dense peak;
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload, and beside it the
                parity of the GPU result on that very sample (max error over tolerance, pass);
  extras        context: step-time quantiles, warm mode, read-only launches, other formats, the
                paper's square sweep, the quantiser.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0
MIN_WARM_MS = 50.0            # untimed graph replays before anything is timed


def algorithmic_bytes(M, N, K, bits):
    """Bytes the method must move per GEMM: packed codes + per-row tables + per-group scale and
    offset + activations in + outputs out (dequantised weights are never counted)."""
    return N * K * bits // 8 + N * (1 << bits) * 2 + 2 * N * (K // 128) * 2 + M * K * 2 + M * N * 2


def quantiles(v):
    s = sorted(v)
    pick = lambda f: s[min(len(s) - 1, int(round(f * (len(s) - 1))))]
    return pick(0.1), pick(0.5), pick(0.9)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--layers", type=int, default=16)
    ap.add_argument("--extras", dest="extras", action="store_true", default=True)
    ap.add_argument("--no-extras", dest="extras", action="store_false")
    ap.add_argument("--no-shapes", dest="shapes", action="store_false", default=True,
                    help="skip the per-shape table (roofline.shapes / roofline.prefill)")
    ap.add_argument("--no-cpu-baseline", dest="cpu", action="store_false", default=True)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (a kernel of known traffic, used to "
                         "scale the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); the path shards without "
              "communication along N and with one small all-reduce along K.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2507_04610_amd as any4
    from paper_2507_04610_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    any4.load_library()                      # raises if libany4.so was not built
    benchlib = ctypes.CDLL(os.path.join(ROOT, "paper_2507_04610_amd", "bench_support", "libany4_bench.so"))
    benchlib.bench_stream_read.restype = ctypes.c_int
    benchlib.bench_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_void_p,
                                           ctypes.c_void_p]
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    bits = 4

    def make_problem(name, M, N, K, b, seed):
        t = inputs.make_case_device(M, N, K, b, seed=seed, device=dev)
        codes = any4.any4_pack(t["codes_u8"], b)
        ws_bytes = any4.any4_gemm_workspace_bytes(M, N, K, b)
        return {"name": name, "M": M, "N": N, "K": K, "bits": b, "x": t["x"], "codes": codes, "lut": t["lut"],
                "scale": t["scale"], "offset": t["offset"],
                "y": torch.empty((M, N), dtype=torch.bfloat16, device=dev),
                "ws": torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev),
                "bytes": algorithmic_bytes(M, N, K, b)}

    def make_layer(shapes, M, seed):
        return [make_problem(name, M, N, K, bits, inputs.case_seed(seed, i)) for i, (name, (N, K)) in enumerate(shapes.items())]

    def stream_read(buf, sink, magic=0x5EED1234):
        """measurement helper (paper_2507_04610_amd/bench_support): read `buf` once on the current stream"""
        rc = benchlib.bench_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), magic, sink.data_ptr(),
                                        torch.cuda.current_stream().cuda_stream)
        assert rc == 0, "bench_stream_read refused its arguments"

    def launch(g):
        any4.any4_gemm(g["x"], g["codes"], g["lut"], g["scale"], g["offset"], g["bits"], out=g["y"], workspace=g["ws"])

    def launch_re(g):
        any4.any4_gemm_repacked(g["x"], g["rcodes"], g["lut"], g["scale"], g["offset"], g["bits"], out=g["y"],
                                workspace=g["ws"])

    def capture(calls):
        """a HIP graph of the given launches, warmed up: untimed replays for at least MIN_WARM_MS"""
        for c in calls[:2]:
            c()
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for c in calls:
                c()
        t_begin = time.perf_counter()
        n = 0
        while n < 2 or (time.perf_counter() - t_begin) * 1e3 < MIN_WARM_MS:
            gr.replay()
            torch.cuda.synchronize()
            n += 1
        return gr

    def replay_ms(gr):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        gr.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    def time_calls(calls, reps=32, repeats=7):
        """microseconds per call (p10, median, p90 over `repeats` replays of a graph of `reps` calls that
        cycle through `calls`; eager launches with an event pair each would add microseconds to kernels
        this short)"""
        gr = capture([calls[r % len(calls)] for r in range(reps)])
        us = [replay_ms(gr) * 1e3 / reps for _ in range(repeats)]
        del gr
        return quantiles(us)

    if args.copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    # ------------------------------------------------------------------ headline workload
    M = 1
    layers = [make_layer(inputs.LLAMA3_8B_SHAPES, M, seed=100 + l) for l in range(args.layers)]
    torch.cuda.synchronize()
    step_bytes = sum(g["bytes"] for g in layers[0])
    n_launch = args.steps * len(layers[0])

    for s in range(args.warmup):                                # untimed warm-up, eager
        for g in layers[s % args.layers]:
            launch(g)
    torch.cuda.synchronize()
    graph = capture([(lambda g=g: launch(g)) for s in range(args.steps) for g in layers[s % args.layers]])

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    graph.replay()                                              # EXACTLY --steps steps
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # the K steps as the GPU ran them (HIP events on the launching stream, inside the synchronised bracket);
    # the host's clock around the same bracket also counts the graph launch and the wake-up after the
    # synchronisation (tens of microseconds, 2 - 3 % of a 20-step run) and is reported in extras
    ms_per_step = e0.elapsed_time(e1) / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9             # GB/s, whole job
    # roofline: the HIP events that bracket the timed region itself.  The graph replays the launches back to
    # back, so elapsed / launches is the average launch duration (it agrees with the rocprofv3 kernel-trace
    # average, see profiles/)
    avg_launch_us = e0.elapsed_time(e1) * 1e3 / n_launch
    bytes_per_launch = step_bytes / len(layers[0])
    achieved = bytes_per_launch / (avg_launch_us * 1e-6) / 1e9

    extras = {"host_clock_ms_per_step": (t1 - t0) * 1e3 / args.steps}
    q = quantiles([replay_ms(graph) / args.steps for _ in range(15)])
    extras["step_ms_quantiles"] = {"what": "15 more replays of the timed graph", "p10": q[0], "median": q[1], "p90": q[2]}
    del graph
    # warm mode: the same number of steps on ONE layer, whose 117 MB of weights stay in the last-level cache
    wgraph = capture([(lambda g=g: launch(g)) for s in range(args.steps) for g in layers[0]])
    wq = quantiles([replay_ms(wgraph) / args.steps for _ in range(7)])
    extras["warm_same_buffers"] = {"what": "every step on the same layer (weights served by the 256 MB last-level cache)",
                                   "ms_per_step": wq[1], "GBps": step_bytes / (wq[1] * 1e-3) / 1e9}
    del wgraph

    # ------------------------------------------------------------------ every shape on its own
    shapes_out, prefill_out = {}, {}

    def shape_record(M_, N_, K_, b_, q3):
        by = algorithmic_bytes(M_, N_, K_, b_)
        return {"M": M_, "N": N_, "K": K_, "bits": b_, "us": q3[1], "p10_us": q3[0], "p90_us": q3[2],
                "GBps": by / (q3[1] * 1e-6) / 1e9, "frac": by / (q3[1] * 1e-6) / 1e9 / HBM_PEAK_GBPS}

    if args.shapes:
        # Llama-3-8B: the headline layers themselves, every linear alone, rotating over the layers
        for gi, g in enumerate(layers[0]):
            rot = [layers[l][gi] for l in range(args.layers)]
            shapes_out[f"8b_{g['name']}_M1"] = shape_record(1, g["N"], g["K"], bits, time_calls([(lambda p=p: launch(p)) for p in rot]))
            for p in rot:
                p["rcodes"] = any4.any4_repack(p["codes"], bits)
            shapes_out[f"8b_{g['name']}_M1_repacked"] = shape_record(1, g["N"], g["K"], bits, time_calls([(lambda p=p: launch_re(p)) for p in rot]))
            for p in rot:
                del p["rcodes"]
            rot8 = []
            for p in rot:
                p8 = dict(p)
                p8["M"] = 8
                p8["x"] = torch.randn((8, p["K"]), device=dev).to(torch.bfloat16)
                p8["y"] = torch.empty((8, p["N"]), dtype=torch.bfloat16, device=dev)
                p8["ws"] = torch.empty(max(any4.any4_gemm_workspace_bytes(8, p["N"], p["K"], bits), 16), dtype=torch.uint8, device=dev)
                rot8.append(p8)
            shapes_out[f"8b_{g['name']}_M8"] = shape_record(8, g["N"], g["K"], bits, time_calls([(lambda p=p: launch(p)) for p in rot8]))
            del rot8
            torch.cuda.empty_cache()
        # prefill, M = 2048, on the 8B shapes (weights of layer 0): bound by the bf16 matrix cores
        for g in layers[0]:
            p = dict(g)
            p["M"] = 2048
            p["x"] = torch.randn((2048, p["K"]), device=dev).to(torch.bfloat16)
            p["y"] = torch.empty((2048, p["N"]), dtype=torch.bfloat16, device=dev)
            p["ws"] = torch.empty(max(any4.any4_gemm_workspace_bytes(2048, p["N"], p["K"], bits), 16), dtype=torch.uint8, device=dev)
            q3 = time_calls([lambda p=p: launch(p)], reps=5, repeats=5)
            tf = 2.0 * 2048 * p["N"] * p["K"] / (q3[1] * 1e-6) / 1e12
            prefill_out[f"8b_{g['name']}_M2048"] = {"M": 2048, "N": p["N"], "K": p["K"], "bits": bits, "us": q3[1], "p10_us": q3[0],
                                                    "p90_us": q3[2], "TFLOPs": tf, "frac": tf / MFMA_BF16_PEAK_TFLOPS}
            del p
        keep = layers[0]
        del layers
        torch.cuda.empty_cache()
        layers = [keep]
        # Llama-3-70B (the bandwidth-bound regime): M = 1 plain and re-laid-out, M = 16; 3- and 2-bit codes at M = 1
        for i, (name, (N, K)) in enumerate(inputs.LLAMA3_70B_SHAPES.items()):
            for b in (4, 3, 2):
                copies = max(2, min(8, int(1.2e9 // (N * K * b // 8)) + 1))
                for Mx in ((1, 16) if b == 4 else (1,)):
                    rot = [make_problem(name, Mx, N, K, b, inputs.case_seed(300 + 10 * b + c, i)) for c in range(copies)]
                    tag = f"70b_{name}_M{Mx}" + ("" if b == 4 else f"_any{b}")
                    shapes_out[tag] = shape_record(Mx, N, K, b, time_calls([(lambda p=p: launch(p)) for p in rot], reps=24))
                    if Mx == 1:
                        for p in rot:
                            p["rcodes"] = any4.any4_repack(p["codes"], b)
                        shapes_out[tag + "_repacked"] = shape_record(Mx, N, K, b, time_calls([(lambda p=p: launch_re(p)) for p in rot], reps=24))
                    del rot
                    torch.cuda.empty_cache()

    # ------------------------------------------------------------------ context measurements
    if args.extras:
        if len(layers) < args.layers:
            layers = [make_layer(inputs.LLAMA3_8B_SHAPES, 1, seed=100 + l) for l in range(args.layers)]
        # what the same launches cost when they only read the packed codes (94 % of the algorithmic
        # bytes) and do no arithmetic: same rotation over layers, same graph replay, a plain read kernel
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        rgraph = capture([(lambda g=g: stream_read(g["codes"], sink)) for s_ in range(args.steps) for g in layers[s_ % args.layers]])
        read_ms = replay_ms(rgraph) / args.steps
        del rgraph
        code_bytes = sum(g["codes"].numel() * 4 for g in layers[0])
        bigbuf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        stream_read(bigbuf, sink)
        torch.cuda.synchronize()
        b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        b0.record()
        stream_read(bigbuf, sink)
        b1.record()
        torch.cuda.synchronize()
        extras["read_only_launches"] = {
            "what": "the step's four launches replaced by a kernel that only reads each linear's packed codes",
            "ms_per_step": read_ms, "code_bytes_per_step": code_bytes,
            "GBps": code_bytes / (read_ms * 1e-3) / 1e9,
            "gemm_step_over_read_step": ms_per_step / read_ms,
            "one_GiB_read_GBps": (1 << 30) / (b0.elapsed_time(b1) * 1e-3) / 1e9}
        del bigbuf
        # the same step on codes re-arranged offline into the tile-major layout (any4_repack)
        for layer in layers:
            for g in layer:
                g["rcodes"] = any4.any4_repack(g["codes"], bits)
        pgraph = capture([(lambda g=g: launch_re(g)) for s_ in range(args.steps) for g in layers[s_ % args.layers]])
        re_ms = replay_ms(pgraph) / args.steps
        del pgraph
        extras["repacked_llama3_8b_M1"] = {
            "what": "the timed step with any4_gemm_repacked on any4_repack'ed codes (offline re-layout)",
            "ms_per_step": re_ms, "GBps": step_bytes / (re_ms * 1e-3) / 1e9,
            "frac_of_8TBps": step_bytes / (re_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        for layer in layers:
            for g in layer:
                del g["rcodes"]
        layers_keep = layers[0]
        del layers
        torch.cuda.empty_cache()
        # the quantiser that produces the GEMM's inputs: Llama-3-8B linears, any4, 20 centre updates at
        # most.  `definition_*`: the arithmetic of the algorithm as it is defined (what the oracle and the
        # per-weight method execute): 2 flops per (sample, centre) distance and 3 per sample for the
        # weighted sums, per pass, plus (2q + 1) per sample for start centre q - the sorted-row method
        # does not execute these (a pass is O(2^n log K) there), so the figure is a rate of equivalent
        # work, not a utilisation.  `per_weight_method_ms`: the same call forced onto the per-weight method.
        qz = {}
        for name, (N, K) in inputs.LLAMA3_8B_SHAPES.items():
            t = inputs.make_quant_case_device(N, K, bits, seed=700, device=dev)
            r = any4.any4_quantize(t["w"], t["act"], t["u"], bits, iters=20)
            torch.cuda.synchronize()
            ev = []
            for _ in range(3):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                r = any4.any4_quantize(t["w"], t["act"], t["u"], bits, iters=20)
                b.record()
                ev.append((a, b))
            torch.cuda.synchronize()
            ms = float(np.median([a.elapsed_time(b) for a, b in ev]))
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            any4.any4_quantize(t["w"], t["act"], t["u"], bits, iters=20, centre_gap=-1.0)
            b.record()
            torch.cuda.synchronize()
            passes = float(r["msteps"].float().mean().item()) + 1.0
            L = 1 << bits
            flops = N * K * (passes * (2 * L + 3) + L * L)
            qz[name] = {"ms": ms, "rows_per_s": N / (ms * 1e-3), "Mweights_per_s": N * K / (ms * 1e-3) / 1e6,
                        "mean_passes": passes, "per_weight_method_ms": a.elapsed_time(b),
                        "definition_fp64_TFLOPs": flops / (ms * 1e-3) / 1e12,
                        "definition_over_fp64_vector_peak": flops / (ms * 1e-3) / 1e12 / 78.6}
            del t, r
            torch.cuda.empty_cache()
        extras["quantize_llama3_8b"] = qz
        # the paper's own latency experiment (section 5, "Speed Comparisons": a 1 x K input times a K x K
        # weight, K = 1K .. 16K): any4 GEMM against the bf16 GEMM of the vendor library that torch calls,
        # weights rotated over enough copies to come from HBM
        sq = {}
        for Ks in (1024, 2048, 4096, 8192, 16384):
            copies = max(2, min(16, int(1.2e9 // (Ks * Ks * 2)) + 1))
            rot = [make_problem("sq", 1, Ks, Ks, bits, 900 + c) for c in range(copies)]
            us = time_calls([(lambda g=g: launch(g)) for g in rot], reps=48, repeats=3)[1]
            wb = [torch.randn((Ks, Ks), device=dev).to(torch.bfloat16) for _ in range(copies)]
            xb = torch.randn((1, Ks), device=dev).to(torch.bfloat16)
            yb = torch.empty((1, Ks), dtype=torch.bfloat16, device=dev)
            us_bf16 = time_calls([(lambda wmat=wmat: torch.matmul(xb, wmat.t(), out=yb)) for wmat in wb], reps=48, repeats=3)[1]
            sq[f"K{Ks}"] = {"any4_us": us, "bf16_library_us": us_bf16, "speedup_over_bf16": us_bf16 / us,
                            "any4_GBps": algorithmic_bytes(1, Ks, Ks, bits) / (us * 1e-6) / 1e9}
            del rot, wb
            torch.cuda.empty_cache()
        extras["square_1xK_KxK"] = sq
        # the paper's format comparison (section 5, "Speed Comparisons"): the same Llama-3-8B linears as any4
        # (a table per row), with one table for the whole matrix (nf4-style) and as int4 (no table at all),
        # at M = 1 and at M = 2048
        fm = {}
        for gi, g in enumerate(layers_keep):
            copies = max(2, min(16, int(1.2e9 // (g["N"] * g["K"] // 2)) + 1))
            rot = [make_problem(g["name"], 1, g["N"], g["K"], bits, inputs.case_seed(950 + c, gi)) for c in range(copies)]

            def call(p_, lut_, **kw):
                return lambda: any4.any4_gemm(p_["x"], p_["codes"], lut_, p_["scale"], p_["offset"], bits,
                                              out=p_["y"], workspace=p_["ws"], **kw)
            med = lambda calls: time_calls(calls, reps=48, repeats=3)[1]
            one = [p_["lut"][:1].contiguous() for p_ in rot]
            fm[g["name"]] = {"any4_us": med([call(p_, p_["lut"]) for p_ in rot]),
                             "single_table_us": med([call(p_, t_) for p_, t_ in zip(rot, one)]),
                             "int4_no_table_us": med([call(p_, None) for p_ in rot])}
            # other group sizes (section 2.5.1; the paper's Table 4 varies them): one scale per 64 / 256 / 1024 weights
            for grp in (64, 256, 1024):
                r_ = grp // 128
                if grp == 64:
                    coarse = [(p_["scale"].repeat_interleave(2, dim=1).contiguous(),
                               p_["offset"].repeat_interleave(2, dim=1).contiguous()) for p_ in rot]
                else:
                    coarse = [(p_["scale"][:, ::r_].contiguous(), p_["offset"][:, ::r_].contiguous()) for p_ in rot]
                fm[g["name"]][f"any4_group{grp}_us"] = med(
                    [(lambda p_=p_, c_=c_: any4.any4_gemm(p_["x"], p_["codes"], p_["lut"], c_[0], c_[1], bits, out=p_["y"],
                                                          workspace=p_["ws"], group=grp)) for p_, c_ in zip(rot, coarse)])
                del coarse
            # fp16 in place of bf16 (section 2.4.1 names both): the same values converted
            half = [{k_: p_[k_].to(torch.float16) for k_ in ("x", "lut", "scale", "offset")} for p_ in rot]
            yh = [torch.empty_like(p_["y"], dtype=torch.float16) for p_ in rot]
            fm[g["name"]]["any4_f16_us"] = med(
                [(lambda p_=p_, h_=h_, y_=y_: any4.any4_gemm(h_["x"], p_["codes"], h_["lut"], h_["scale"], h_["offset"], bits,
                                                             out=y_, workspace=p_["ws"])) for p_, h_, y_ in zip(rot, half, yh)])
            # M = 2048: the matrix-core kernel with a table per row, one table, no table
            p_ = dict(rot[0])
            p_["x"] = torch.randn((2048, p_["K"]), device=dev).to(torch.bfloat16)
            p_["y"] = torch.empty((2048, p_["N"]), dtype=torch.bfloat16, device=dev)
            p_["ws"] = torch.empty(max(any4.any4_gemm_workspace_bytes(2048, p_["N"], p_["K"], bits), 16), dtype=torch.uint8, device=dev)
            for tag, lut_ in (("any4", p_["lut"]), ("single_table", one[0]), ("int4_no_table", None)):
                fm[g["name"]][f"{tag}_M2048_us"] = time_calls([call(p_, lut_)], reps=5, repeats=3)[1]
            del rot, one, half, yh, p_
            torch.cuda.empty_cache()
        extras["formats_llama3_8b"] = fm

    # ------------------------------------------------------------------ CPU oracle beside it
    cpu = None
    if args.cpu:
        from oracle import any4_oracle as oracle
        threads = min(16, os.cpu_count() or 1)
        # bounded sample: the first `rows` output rows of each of the four linears of one layer
        cases = []
        for i, (name, (N, K)) in enumerate(inputs.LLAMA3_8B_SHAPES.items()):
            rows = max(threads, N // 8)
            cs = inputs.make_case(1, rows, K, bits, seed=inputs.case_seed(100, i))
            cases.append((name, cs, oracle.pack(cs.codes_u8, bits)))
        t0 = time.perf_counter()
        reps = 0
        y_ref = {}
        while time.perf_counter() - t0 < 10.0:
            for name, cs, packed in cases:
                y_ref[name] = oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, cs.K, bits, threads=threads)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        sample_bytes = sum(algorithmic_bytes(1, cs.N, cs.K, bits) for _, cs, _ in cases)
        # the GPU on the very same sample, against what the oracle just computed
        parity = {}
        for name, cs, packed in cases:
            dv = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev).view(torch.bfloat16)
            y = any4.any4_gemm(dv(cs.x), torch.from_numpy(packed.view(np.int32)).to(dev), dv(cs.lut), dv(cs.scale), dv(cs.offset), bits)
            torch.cuda.synchronize()
            got = y.float().cpu().numpy().astype(np.float64)
            tol = 1e-2 * oracle.rms(y_ref[name]) + np.abs(y_ref[name]) * 2.0 ** -8
            ratio = float((np.abs(got - y_ref[name]) / tol).max())
            parity[name] = {"N": cs.N, "K": cs.K, "max_err_over_tolerance": ratio, "pass": bool(ratio <= 1.0)}
        cpu = {"value": sample_bytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"first N/8 output rows of each of the four Llama-3-8B linears at M=1 "
                         f"({sample_bytes / 1e6:.1f} MB algorithmic), {reps} passes, {dt * 1e3:.1f} ms per pass",
               "gpu_parity_on_sample": parity}

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "decode_llama3_8b_m1_hbm_traffic.txt")
    if os.path.exists(tpath):                       # measured offline with rocprofv3 --pmc, see the file
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])

    out = {
        "metric": "any4 GEMM achieved HBM GB/s (M=1) on Llama-3-8B shapes",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Llama-3-8B decode linears (qkv 6144x4096, o 4096x4096, gate_up 28672x4096, "
                               "down 4096x14336), any4 g=128, M=1; step = the four GEMMs of one layer, "
                               f"rotating over {args.layers} distinct layers, HIP-graph replay",
                   "M": 1, "bits": bits, "group": 128, "bytes_per_step": step_bytes},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "the decode GEMM launches of the step: any4::stream::decode_stream_kernel (qkv, o, gate_up: "
                               "K = 4096) and any4::pack::decode_pack_kernel (down: K = 14336), M = 1",
                     "avg_launch_us": avg_launch_us, "bytes_per_launch": bytes_per_launch,
                     "shapes": shapes_out,
                     "prefill": {"bound": "mfma", "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "shapes": prefill_out}},
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
