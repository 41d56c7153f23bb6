#!/usr/bin/env python3
"""Benchmark of the any4 GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--extras/--no-extras]

A *step* is one pass of the hot path over one decoder layer of Llama-3-8B at M = 1: the four
quantised linears (fused QKV, O, fused gate/up, down), i.e. four any4_gemm launches.  Successive
steps use successive layers of a stack of `--layers` distinct synthetic layers (default 16, 1.9 GB
of packed weights), so every launch streams its weights from HBM and not from the 256 MB
last-level cache, exactly as token generation over a whole model does.  The K timed steps are
replayed from one HIP graph (the launch sequence of a decode step is static), bracketed by
synchronisation on both sides.

The one JSON line printed at the end carries the contract fields plus
  roofline      achieved GB/s of the decode kernel: algorithmic bytes per launch divided by
                the average launch duration, from the HIP events that bracket the timed graph
                replay (stream = torch's current stream, on which the library is launched);
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload;
  extras        per-shape microseconds, other M, the 70B shapes and the M = 2048 matrix-core
                path (context; not part of `value`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0


def algorithmic_bytes(M, N, K, bits):
    """Bytes the method must move per GEMM: packed codes + per-row tables + per-group scale and
    offset + activations in + outputs out (dequantised weights are never counted)."""
    return N * K * bits // 8 + N * (1 << bits) * 2 + 2 * N * (K // 128) * 2 + M * K * 2 + M * N * 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=640)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--layers", type=int, default=16)
    ap.add_argument("--extras", dest="extras", action="store_true", default=True)
    ap.add_argument("--no-extras", dest="extras", action="store_false")
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
    import ctypes
    benchlib = ctypes.CDLL(os.path.join(ROOT, "paper_2507_04610_amd", "bench_support", "libany4_bench.so"))
    benchlib.bench_stream_read.restype = ctypes.c_int
    benchlib.bench_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_void_p,
                                           ctypes.c_void_p]
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    bits = 4

    def make_layer(shapes, M, seed):
        layer = []
        for i, (name, (N, K)) in enumerate(shapes.items()):
            t = inputs.make_case_device(M, N, K, bits, seed=inputs.case_seed(seed, i), device=dev)
            codes = any4.any4_pack(t["codes_u8"], bits)
            ws_bytes = any4.any4_gemm_workspace_bytes(M, N, K, bits)
            layer.append({
                "name": name, "M": M, "N": N, "K": K, "x": t["x"], "codes": codes, "lut": t["lut"],
                "scale": t["scale"], "offset": t["offset"],
                "y": torch.empty((M, N), dtype=torch.bfloat16, device=dev),
                "ws": torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev),
                "bytes": algorithmic_bytes(M, N, K, bits),
            })
            del t["codes_u8"]
        return layer

    def stream_read(buf, sink, magic=0x5EED1234):
        """measurement helper (paper_2507_04610_amd/bench_support): read `buf` once on the current stream"""
        rc = benchlib.bench_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), magic, sink.data_ptr(),
                                        torch.cuda.current_stream().cuda_stream)
        assert rc == 0, "bench_stream_read refused its arguments"

    def launch(g):
        any4.any4_gemm(g["x"], g["codes"], g["lut"], g["scale"], g["offset"], g.get("bits", bits), out=g["y"],
                       workspace=g["ws"])

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

    def run_steps(first, count):
        for s in range(first, first + count):
            for g in layers[s % args.layers]:
                launch(g)

    run_steps(0, args.warmup)                                   # untimed warm-up, eager
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_steps(0, args.steps)
    graph.replay()                                              # untimed: first replay uploads the graph
    torch.cuda.synchronize()

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    graph.replay()                                              # EXACTLY --steps steps
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9             # GB/s, whole job

    # per-launch durations: same steps, eager, one event pair around every launch
    n_launch = args.steps * len(layers[0])
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_launch)]
    i = 0
    for s in range(args.steps):
        for g in layers[s % args.layers]:
            evs[i][0].record()
            launch(g)
            evs[i][1].record()
            i += 1
    torch.cuda.synchronize()
    per_shape_us = {g["name"]: [] for g in layers[0]}
    i = 0
    total_kernel_ms = 0.0
    for s in range(args.steps):
        for g in layers[s % args.layers]:
            dt = evs[i][0].elapsed_time(evs[i][1])
            per_shape_us[g["name"]].append(dt * 1e3)
            total_kernel_ms += dt
            i += 1
    # the roofline figure uses the HIP events that bracket the timed region itself: the graph replays
    # the launches back to back, so elapsed / launches is the average launch duration (it agrees with
    # the rocprofv3 kernel-trace average, see profiles/); the per-launch event pairs above add ~2 us
    # of event overhead each and only feed the per-shape extras
    avg_launch_us = e0.elapsed_time(e1) * 1e3 / n_launch
    bytes_per_launch = step_bytes / len(layers[0])
    achieved = bytes_per_launch / (avg_launch_us * 1e-6) / 1e9

    extras = {
        "graph_event_ms_per_step": e0.elapsed_time(e1) / args.steps,
        "event_pair_avg_launch_us": total_kernel_ms * 1e3 / n_launch,
        "llama3_8b_M1_us": {k: float(np.median(v)) for k, v in per_shape_us.items()},
        "llama3_8b_M1_GBps": {g["name"]: g["bytes"] / (float(np.median(per_shape_us[g["name"]])) * 1e-6) / 1e9
                              for g in layers[0]},
    }

    # ------------------------------------------------------------------ context measurements
    def time_gemm(g, reps, rotate=None, fn=None):
        """microseconds of one launch: `reps` launches, cycling through `rotate` (equivalent problems,
        so that weights come from HBM), captured in one HIP graph and replayed; events around the replay.
        (Eager launches with an event pair each add several microseconds to kernels this short.)"""
        probs = rotate or [g]
        fn = fn or launch
        for p in probs[:2]:
            fn(p)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for r in range(reps):
                fn(probs[r % len(probs)])
        gr.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        gr.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    if args.extras:
        del graph
        # what the same launches cost when they only read the packed codes (94 % of the algorithmic
        # bytes) and do no arithmetic: same rotation over layers, same graph replay, a plain read kernel
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for g in layers[0]:
            stream_read(g["codes"], sink)
        torch.cuda.synchronize()
        rgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(rgraph):
            for s_ in range(args.steps):
                for g in layers[s_ % args.layers]:
                    stream_read(g["codes"], sink)
        rgraph.replay()
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record()
        rgraph.replay()
        r1.record()
        torch.cuda.synchronize()
        read_ms = r0.elapsed_time(r1) / args.steps
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
        del rgraph, bigbuf
        # the same step on codes re-arranged offline into the tile-major layout (any4_repack):
        # same kernels and results, the code stream of a wavefront instruction is one contiguous piece
        for layer in layers:
            for g in layer:
                g["rcodes"] = any4.any4_repack(g["codes"], bits)

        def launch_re(g):
            any4.any4_gemm_repacked(g["x"], g["rcodes"], g["lut"], g["scale"], g["offset"], bits, out=g["y"],
                                    workspace=g["ws"])
        for g in layers[0]:
            launch_re(g)
        torch.cuda.synchronize()
        pgraph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(pgraph):
            for s_ in range(args.steps):
                for g in layers[s_ % args.layers]:
                    launch_re(g)
        pgraph.replay()
        torch.cuda.synchronize()
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        pgraph.replay()
        p1.record()
        torch.cuda.synchronize()
        re_ms = p0.elapsed_time(p1) / args.steps
        extras["repacked_llama3_8b_M1"] = {
            "what": "the timed step with any4_gemm_repacked on any4_repack'ed codes (offline re-layout)",
            "ms_per_step": re_ms, "GBps": step_bytes / (re_ms * 1e-3) / 1e9,
            "frac_of_8TBps": step_bytes / (re_ms * 1e-3) / 1e9 / 8000.0,
            "plain_layout_step_over_this": e0.elapsed_time(e1) / args.steps / re_ms}
        del pgraph
        for layer in layers:
            for g in layer:
                del g["rcodes"]
        torch.cuda.empty_cache()
        m8 = {}
        for gi, g in enumerate(layers[0]):
            rot = []
            for l in range(args.layers):
                p = dict(layers[l][gi])
                p["M"] = 8
                p["x"] = torch.randn((8, p["K"]), device=dev).to(torch.bfloat16)
                p["y"] = torch.empty((8, p["N"]), dtype=torch.bfloat16, device=dev)
                p["ws"] = torch.empty(max(any4.any4_gemm_workspace_bytes(8, p["N"], p["K"], bits), 16),
                                      dtype=torch.uint8, device=dev)
                rot.append(p)
            us = time_gemm(rot[0], 64, rot)
            m8[g["name"]] = {"us": us, "GBps": algorithmic_bytes(8, g["N"], g["K"], bits) / (us * 1e-6) / 1e9}
        extras["llama3_8b_M8"] = m8
        # prefill, M = 2048, on the 8B shapes (weights of layer 0)
        pf = {}
        for g in layers[0]:
            p = dict(g)
            p["M"] = 2048
            p["x"] = torch.randn((2048, p["K"]), device=dev).to(torch.bfloat16)
            p["y"] = torch.empty((2048, p["N"]), dtype=torch.bfloat16, device=dev)
            p["ws"] = torch.empty(max(any4.any4_gemm_workspace_bytes(2048, p["N"], p["K"], bits), 16),
                                  dtype=torch.uint8, device=dev)
            us = time_gemm(p, 5)
            tf = 2.0 * 2048 * p["N"] * p["K"] / (us * 1e-6) / 1e12
            pf[g["name"]] = {"us": us, "TFLOPs": tf, "frac_of_bf16_peak": tf / MFMA_BF16_PEAK_TFLOPS}
            del p
        extras["llama3_8b_M2048"] = pf
        layers_keep = layers[0]
        del layers
        torch.cuda.empty_cache()
        # 70B shapes, M = 1 and 16, rotating over enough copies to exceed the last-level cache
        big = {}
        for i, (name, (N, K)) in enumerate(inputs.LLAMA3_70B_SHAPES.items()):
            copies = max(2, min(8, int(1.2e9 // (N * K // 2)) + 1))
            for Mx in (1, 16):
                rot = [make_layer({name: (N, K)}, Mx, seed=300 + c)[0] for c in range(copies)]
                us = time_gemm(rot[0], 24, rot)
                by = algorithmic_bytes(Mx, N, K, bits)
                big[f"{name}_M{Mx}"] = {"us": us, "GBps": by / (us * 1e-6) / 1e9,
                                        "frac_of_hbm_peak": by / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
                if Mx == 1:                                     # the same launches on re-laid-out codes
                    for p_ in rot:
                        p_["rcodes"] = any4.any4_repack(p_["codes"], bits)
                    us_re = time_gemm(rot[0], 24, rot, fn=launch_re)
                    big[f"{name}_M1_repacked"] = {"us": us_re, "GBps": by / (us_re * 1e-6) / 1e9,
                                                  "frac_of_hbm_peak": by / (us_re * 1e-6) / 1e9 / HBM_PEAK_GBPS}
                del rot
                torch.cuda.empty_cache()
        extras["llama3_70b"] = big
        # config 5: 3- and 2-bit variants on the 70B shapes, M = 1 and 16
        low = {}
        for b in (3, 2):
            for i, (name, (N, K)) in enumerate(inputs.LLAMA3_70B_SHAPES.items()):
                copies = max(2, min(8, int(1.2e9 // (N * K * b // 8)) + 1))
                for Mx in (1, 16):
                    rot = []
                    for c in range(copies):
                        t = inputs.make_case_device(Mx, N, K, b, seed=inputs.case_seed(500 + c, i), device=dev)
                        rot.append({"x": t["x"], "codes": any4.any4_pack(t["codes_u8"], b), "lut": t["lut"],
                                    "scale": t["scale"], "offset": t["offset"], "bits": b,
                                    "y": torch.empty((Mx, N), dtype=torch.bfloat16, device=dev),
                                    "ws": torch.empty(max(any4.any4_gemm_workspace_bytes(Mx, N, K, b), 16),
                                                      dtype=torch.uint8, device=dev)})
                        del t
                    us = time_gemm(rot[0], 24, rot)
                    by = algorithmic_bytes(Mx, N, K, b)
                    low[f"any{b}_{name}_M{Mx}"] = {"us": us, "GBps": by / (us * 1e-6) / 1e9,
                                                   "frac_of_hbm_peak": by / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS}
                    del rot
                    torch.cuda.empty_cache()
        extras["llama3_70b_any3_any2"] = low
        # the quantiser that produces the GEMM's inputs: Llama-3-8B linears, any4, 20 centre updates
        # at most; fp64 vector-ALU bound.  Flops counted: 2 per (sample, centre) distance, 3 per
        # sample for the weighted sums, per pass; (2q + 1) per sample for start centre q.
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
            passes = float(r["msteps"].float().mean().item()) + 1.0
            L = 1 << bits
            flops = N * K * (passes * (2 * L + 3) + L * L)
            qz[name] = {"ms": ms, "rows_per_s": N / (ms * 1e-3), "Mweights_per_s": N * K / (ms * 1e-3) / 1e6,
                        "mean_passes": passes, "fp64_TFLOPs": flops / (ms * 1e-3) / 1e12,
                        "frac_of_fp64_vector_peak": flops / (ms * 1e-3) / 1e12 / 78.6}
            del t, r
            torch.cuda.empty_cache()
        if args.cpu:
            from oracle import any4_quant_oracle as qoracle
            threads_q = min(16, os.cpu_count() or 1)
            qc = inputs.make_quant_case(4 * threads_q, 4096, bits, seed=700)
            t0 = time.perf_counter()
            qoracle.quantize(qc.w, qc.act, qc.u, bits, iters=20, threads=threads_q)
            dtq = time.perf_counter() - t0
            qz["cpu_oracle"] = {"rows_per_s": qc.N / dtq, "cores": threads_q,
                                "sample": f"{qc.N} rows of K = 4096, any4, 20 centre updates at most"}
        extras["quantize_llama3_8b"] = qz
        # the paper's own latency experiment (section 5, "Speed Comparisons": a 1 x K input times a K x K
        # weight, K = 1K .. 16K): any4 GEMM against the bf16 GEMM of the vendor library that torch calls,
        # weights rotated over enough copies to come from HBM
        sq = {}

        def graph_us(calls, reps=48):
            """microseconds per call: `reps` calls (cycling through `calls`) captured in one graph"""
            for c in calls[:2]:
                c()
            torch.cuda.synchronize()
            gsq = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gsq):
                for r_ in range(reps):
                    calls[r_ % len(calls)]()
            gsq.replay()
            torch.cuda.synchronize()
            a_, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a_.record()
            gsq.replay()
            b_.record()
            torch.cuda.synchronize()
            return a_.elapsed_time(b_) * 1e3 / reps

        for Ks in (1024, 2048, 4096, 8192, 16384):
            copies = max(2, min(16, int(1.2e9 // (Ks * Ks * 2)) + 1))
            rot = [make_layer({"sq": (Ks, Ks)}, 1, seed=900 + c)[0] for c in range(copies)]
            us = graph_us([(lambda g=g: launch(g)) for g in rot])
            wb = [torch.randn((Ks, Ks), device=dev).to(torch.bfloat16) for _ in range(copies)]
            xb = torch.randn((1, Ks), device=dev).to(torch.bfloat16)
            yb = torch.empty((1, Ks), dtype=torch.bfloat16, device=dev)
            us_bf16 = graph_us([(lambda wmat=wmat: torch.matmul(xb, wmat.t(), out=yb)) for wmat in wb])
            sq[f"K{Ks}"] = {"any4_us": us, "bf16_library_us": us_bf16, "speedup_over_bf16": us_bf16 / us,
                            "any4_GBps": algorithmic_bytes(1, Ks, Ks, bits) / (us * 1e-6) / 1e9}
            del rot, wb
            torch.cuda.empty_cache()
        extras["square_1xK_KxK"] = sq
        # the paper's format comparison (section 5, "Speed Comparisons"): the same Llama-3-8B linears at
        # M = 1 as any4 (a table per row), with one table shared by all rows (nf4-style: the same
        # kernel, the table rows simply repeat) and as int4 (lut = NULL: no table at all)
        fm = {}
        for gi, g in enumerate(layers_keep):
            copies = max(2, min(16, int(1.2e9 // (g["N"] * g["K"] // 2)) + 1))
            rot = [make_layer({g["name"]: (g["N"], g["K"])}, 1, seed=950 + c)[0] for c in range(copies)]

            def call(p_, lut_):
                return lambda: any4.any4_gemm(p_["x"], p_["codes"], lut_, p_["scale"], p_["offset"], bits,
                                              out=p_["y"], workspace=p_["ws"])
            shared = [p_["lut"][:1].expand(p_["N"], -1).contiguous() for p_ in rot]
            fm[g["name"]] = {"any4_us": graph_us([call(p_, p_["lut"]) for p_ in rot]),
                             "shared_table_us": graph_us([call(p_, sh) for p_, sh in zip(rot, shared)]),
                             "int4_no_table_us": graph_us([call(p_, None) for p_ in rot])}
            # other group sizes (section 2.5.1; the paper's Table 4 varies them): one scale per 64 / 256 / 1024 weights
            for grp in (64, 256, 1024):
                r_ = grp // 128
                if grp == 64:
                    coarse = [(p_["scale"].repeat_interleave(2, dim=1).contiguous(),
                               p_["offset"].repeat_interleave(2, dim=1).contiguous()) for p_ in rot]
                else:
                    coarse = [(p_["scale"][:, ::r_].contiguous(), p_["offset"][:, ::r_].contiguous()) for p_ in rot]
                fm[g["name"]][f"any4_group{grp}_us"] = graph_us(
                    [(lambda p_=p_, c_=c_: any4.any4_gemm(p_["x"], p_["codes"], p_["lut"], c_[0], c_[1], bits, out=p_["y"],
                                                          workspace=p_["ws"], group=grp)) for p_, c_ in zip(rot, coarse)])
                del coarse
            # fp16 in place of bf16 (section 2.4.1 names both): the same values converted
            half = [{k_: p_[k_].to(torch.float16) for k_ in ("x", "lut", "scale", "offset")} for p_ in rot]
            yh = [torch.empty_like(p_["y"], dtype=torch.float16) for p_ in rot]
            fm[g["name"]]["any4_f16_us"] = graph_us(
                [(lambda p_=p_, h_=h_, y_=y_: any4.any4_gemm(h_["x"], p_["codes"], h_["lut"], h_["scale"], h_["offset"], bits,
                                                             out=y_, workspace=p_["ws"])) for p_, h_, y_ in zip(rot, half, yh)])
            del rot, shared, half, yh
            torch.cuda.empty_cache()
        extras["formats_llama3_8b_M1"] = fm
        layers = [layers_keep]

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
            cases.append((cs, oracle.pack(cs.codes_u8, bits)))
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            for cs, packed in cases:
                oracle.gemm(cs.x, packed, cs.lut, cs.scale, cs.offset, cs.K, bits, threads=threads)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        sample_bytes = sum(algorithmic_bytes(1, cs.N, cs.K, bits) for cs, _ in cases)
        cpu = {"value": sample_bytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": f"first N/8 output rows of each of the four Llama-3-8B linears at M=1 "
                         f"({sample_bytes / 1e6:.1f} MB algorithmic), {reps} passes, {dt * 1e3:.1f} ms per pass"}

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "decode_stream_llama3_8b_m1_hbm_traffic.txt")
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
                     "kernel": "any4::stream::decode_stream_kernel (any4 GEMM, M<=16; here M=1)", "avg_launch_us": avg_launch_us,
                     "bytes_per_launch": bytes_per_launch},
        "cpu_baseline": cpu,
        "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
