#!/usr/bin/env python3
"""Benchmark of the BWTA linear hot path on one MI355X.

Default run (`python bench.py`): the headline is the 7B-decoder prefill configuration the metric
and the target are stated on -- ternary activations M=2048 against packed binary weights,
(K,N) in {(4096,4096), (4096,11008), (11008,4096)}.  One step = bwta_gemm (integer product + scale
epilogue, from the packed bit planes) on all three shapes.  Inputs, planes and packed weights are
resident in HBM before the timed region (the paper packs weights before inference; the activation
packer is timed beside it).  `value` is effective TOPS = sum of 2*M*N*K over the step / time (zeros
counted, dense-equivalent work).  `roofline` is for the dominant kernel (the tiled FP4 product on
its longest shape), timed live with HIP events on the launch stream; `cpu_baseline` is the CPU
oracle timed on the host cores of the same box on the same three shapes.  The same JSON line
carries sub-records for the other configurations: `decode_c4` (achieved HBM GB/s, median and best
of 20 grouped launches over 64 distinct weight matrices per case), `ffn_c2` (the encoder FFN step,
whole path from fp16) and `block_c5` (decoder-block latency and the BWTA share of it).

Single workloads (profiling): --workload c1_tiny | c2_ffn | c3_prefill | c4_decode | c5_block | attn |
prep | short_k | copy_probe.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # MI355X dense int8 MFMA, TOP/s
PEAK_FP4_TOPS = 10100.0   # MI355X dense fp4 MFMA, TFLOP/s (the dtype the dominant kernel contracts in)
PEAK_HBM_GBS = 8000.0     # MI355X HBM3E, GB/s
PEAK_VALU_POPC_TOPS = 1258.0  # 256 CU * 64 lanes * 2.4 GHz * 32 MAC per 2 VALU ops * 2 ops/MAC


def _dev(a, torch):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to("cuda:0")


SETTLE_S = 0.03  # load applied before a timed region; see _settle


def _settle(torch, fn, seconds=SETTLE_S):
    """Untimed load in front of a timed region.  An idle MI355X parks its shader clock near
    1.2 GHz and takes some milliseconds of work to reach its working frequency (measured: the
    first 15 ms of a cold loop run about 4 % slow on the FFN step, a 2 ms burst of the
    7B-shape product 10-15 % slow), so a few warm-up launches after host-side set-up time the
    ramp, not the kernel."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()


def _event_ms(torch, fn, reps, warmup):
    """Average duration of fn() in ms, HIP events on the current (launch) stream."""
    _settle(torch, fn)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _launch_times_ms(torch, fn, reps):
    """Durations of `reps` consecutive fn() calls, each between its own pair of HIP events on the
    launch stream (for medians; fn should be long enough that the events do not dominate)."""
    _settle(torch, fn)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ev[0].record()
    for i in range(reps):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    return [ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]


def _traffic_from_profiles(B, kernel, shape):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE runs, copy-probe scaled) of `kernel` on `shape`
    from the tracked table profiles/traffic__hbm_bytes_per_launch.md -- but only if the table was
    measured on this very build of the library (rows carry the build id); otherwise None."""
    path = os.path.join(ROOT, "profiles", "traffic__hbm_bytes_per_launch.md")
    try:
        build = B.build_id()
        for line in open(path):
            cells = [c.strip().strip("`") for c in line.strip().strip("|").split("|")]
            if len(cells) >= 5 and cells[0] == build and cells[1] == kernel and cells[2] == shape:
                return float(cells[3]) + float(cells[4])
    except (OSError, ValueError):
        pass
    return None


def _graph_of(torch, fn, check=None):
    """Capture fn() (launches on the current stream only) into a HIP graph.  The replay is
    checked against the eager result by `check` three times with eager work in between."""
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    torch.cuda.synchronize()
    if check is not None:
        for _ in range(3):
            want = check(None)
            fn()                      # eager
            torch.cuda.synchronize()
            want = check(None)
            g.replay()
            torch.cuda.synchronize()
            check(want)
    return g


def _kernel_path_name(B, M, N, K):
    return {B.PATH_MFMA: "mfma_int8", B.PATH_FP4: "mfma_fp4", B.PATH_POPC: "popc"}[B.auto_path(M, N, K)]


class Layer:
    """One linear layer's device buffers."""

    def __init__(self, cfg, torch, B, from_fp16):
        self.M, self.N, self.K = cfg["M"], cfg["N"], cfg["K"]
        M, N, K = self.M, self.N, self.K
        self.rw = B.plane_row_words(K)
        self.s_w = _dev(cfg["s_w"], torch)
        w = _dev(cfg["w"], torch)
        self.wsign = torch.empty((N, self.rw), dtype=torch.int32, device="cuda:0")
        B.bwta_pack_weights(w, self.wsign, N=N, K=K)
        del w
        self.out = torch.empty((M, N), dtype=torch.float16, device="cuda:0")
        self.ws = torch.empty(max(B.workspace_bytes(M, N, K), 256), dtype=torch.uint8, device="cuda:0")
        self.prep = torch.empty(max(B.prepared_bytes(M, K), 256), dtype=torch.uint8, device="cuda:0")
        self.mask = torch.empty((M, self.rw), dtype=torch.int32, device="cuda:0")
        self.sign = torch.empty_like(self.mask)
        self.from_fp16 = from_fp16
        if from_fp16:
            self.A = _dev(cfg["A"], torch)
            if "s_a" in cfg:
                self.s_a = _dev(cfg["s_a"], torch)
            else:  # the token scales are part of the input recipe: the value training starts them from
                self.s_a = torch.empty((M,), dtype=torch.float16, device="cuda:0")
                B.bwta_act_scale(self.A, self.s_a, M=M, K=K)
            B.bwta_quantize_pack_act(self.A, self.s_a, self.mask, self.sign, None, M=M, K=K)
        else:
            self.s_a = _dev(cfg["s_a"], torch)
            self.A = _dev(cfg["t"], torch)
            B.bwta_quantize_pack_act(self.A, None, self.mask, self.sign, None, M=M, K=K, a_dtype=B.DTYPE_INT8)
        torch.cuda.synchronize()
        self.ops = 2.0 * M * N * K
        self.fmt = None

    def pack(self, B):  # the activation packer (a1 + a2) on this layer's input
        if self.from_fp16:
            B.bwta_quantize_pack_act(self.A, self.s_a, self.mask, self.sign, None, M=self.M, K=self.K)
        else:
            B.bwta_quantize_pack_act(self.A, None, self.mask, self.sign, None, M=self.M, K=self.K, a_dtype=B.DTYPE_INT8)

    def prepare_from_ternary(self, B, torch):
        """Fragments for the tiled kernel alone (bwta_gemm_prepared) from already-ternary input: the
        values +-1 / 0 as fp16 under a unit threshold ternarise to themselves."""
        a16 = self.A.to(torch.float16)
        self.fmt = B.bwta_prepare_act(a16, None, self.prep, M=self.M, K=self.K)
        torch.cuda.synchronize()

    def linear(self, B):
        B.bwta_linear(self.A, self.s_a, self.wsign, self.s_w, self.out, self.ws, M=self.M, N=self.N, K=self.K)

    def quantize(self, B):
        B.bwta_quantize_pack_act(self.A, self.s_a, self.mask, self.sign, None, M=self.M, K=self.K)

    def prepare(self, B):  # first kernel of bwta_linear
        self.fmt = B.bwta_prepare_act(self.A, self.s_a, self.prep, M=self.M, K=self.K)

    def gemm_prepared(self, B):  # second kernel of bwta_linear
        if self.fmt is None:
            self.prepare(B)
        B.bwta_gemm_prepared(self.prep, self.wsign, self.s_a, self.s_w, None, self.out, fmt=self.fmt,
                             M=self.M, N=self.N, K=self.K)

    def gemm(self, B):
        B.bwta_gemm(self.mask, self.sign, self.wsign, self.s_a, self.s_w, None, self.out, self.ws,
                    M=self.M, N=self.N, K=self.K)

    def gemm_prepared_bytes(self):  # second kernel of bwta_linear: E2M1 fragments, weight bits, scales in; fp16 out
        return self.M * self.K // 2 + self.N * self.rw * 4 + 2 * (self.M + self.N) + 2 * self.M * self.N

    def gemm_bytes(self):
        M, N, K = self.M, self.N, self.K
        return N * self.rw * 4 + 2 * M * self.rw * 4 + 2 * (M + N) + 2 * M * N

    def quantize_bytes(self):
        return self.M * self.K * 2 + 2 * self.M * self.rw * 4 + 2 * self.M


def cpu_baseline_c2(cfgs, target_s=12.0):
    """The oracle, as it stands, on the same workload: whole layers, repeated to ~target_s."""
    import oracle
    threads = oracle.num_threads()
    ops_per_pass = sum(2.0 * c["M"] * c["N"] * c["K"] for c in cfgs)
    t0 = time.perf_counter()
    passes = 0
    while True:
        for c in cfgs:
            oracle.linear(c["A"], c["s_a"], c["w"], c["s_w"])  # s_a: oracle.act_scale(A), set by run_c2
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= target_s or passes >= 50:
            break
    out = {"value": round(ops_per_pass * passes / dt / 1e12, 5), "unit": "TOPS", "cores": threads,
           "kind": "oracle", "sample": "%d full passes of the same two layers (all %d tokens), %.1f s"
           % (passes, cfgs[0]["M"], dt)}
    # the same oracle on one thread, on the first 256 tokens of both layers (a few seconds)
    oracle.set_num_threads(1)
    try:
        rows = 256
        t1 = time.perf_counter()
        for c in cfgs:
            oracle.linear(np.ascontiguousarray(c["A"][:rows]), c["s_a"][:rows], c["w"], c["s_w"])
        d1 = time.perf_counter() - t1
        out["single_thread_value"] = round(sum(2.0 * rows * c["N"] * c["K"] for c in cfgs) / d1 / 1e12, 5)
        out["single_thread_sample"] = "one pass over the first %d tokens of both layers, %.1f s" % (rows, d1)
    finally:
        oracle.set_num_threads(threads)
    return out


def run_c2(args, torch, B, synth):
    cfgs = [synth.config2("up"), synth.config2("down")]
    layers = [Layer(c, torch, B, from_fp16=True) for c in cfgs]

    def step():
        for L in layers:
            L.linear(B)

    def check(want):
        got = [L.out.clone() for L in layers]
        if want is not None:
            for a, b in zip(got, want):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "graph replay differs from eager"
        return got

    run = step
    if args.graph:
        graph = _graph_of(torch, step, check)
        run = graph.replay
    _settle(torch, run)  # untimed: brings an idle GPU's clock up, whatever --warmup was asked for
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    ops = sum(L.ops for L in layers)
    value = ops / (ms_per_step * 1e-3) / 1e12

    # per-kernel durations: HIP events on the launch stream.  A layer that bwta_linear runs as one
    # kernel (short K) is timed as such, and its two-kernel form (tuning hook 900) beside it.  The
    # product is timed through its single-kernel entry point (a 10 us kernel keeps the GPU, not the
    # host's launch rate, the bound); a loop over the 3-7 us ternarise kernel alone would time the
    # host (about 8 us per call through Python), so its figure is the two-kernel bwta_linear minus
    # the product.
    kern, contraction_ms = [], []
    for L, c in zip(layers, cfgs):
        launches = B.linear_launches(L.M, L.N, L.K)
        tl = _event_ms(torch, lambda: L.linear(B), args.steps, args.warmup)
        tg = _event_ms(torch, lambda: L.gemm_prepared(B), args.steps, args.warmup)
        k = {"layer": c["name"], "launches": launches, "linear_us": round(tl * 1e3, 2)}
        t2 = tl
        if launches == 1:
            k["kernel"] = "k_linear_fused (ternarise + FP4 MFMA product + scale epilogue)"
            B.set_tile(900)
            try:
                t2 = _event_ms(torch, lambda: L.linear(B), args.steps, args.warmup)
            finally:
                B.set_tile(0)
            k["two_kernel_form_us"] = round(t2 * 1e3, 2)
            contraction_ms.append(tl)
        else:
            k["kernel"] = "k_quantize_to_fp4, then k_gemm_fp4 (FP4 MFMA product + scale epilogue)"
            contraction_ms.append(tg)
        tq = max(t2 - tg, 1e-6)
        k.update({"ternarize_us": round(tq * 1e3, 2), "gemm_us": round(tg * 1e3, 2),
                  "ternarize_GBs": round((L.M * L.K * 2.5 + 2 * L.M) / (tq * 1e-3) / 1e9, 1),
                  "gemm_TOPS": round(L.ops / (tg * 1e-3) / 1e12, 2), "path": _kernel_path_name(B, L.M, L.N, L.K)})
        kern.append(k)
    # the kernels that hold the contraction: per layer, the one-launch linear or the product kernel;
    # the dominant one is the longer of the two (the up layer's: it writes 25 MB of fp16)
    names = ["k_linear_fused" if k["launches"] == 1 else "k_gemm_fp4" for k in kern]
    dom = max(range(len(layers)), key=lambda i: contraction_ms[i])
    L = layers[dom]
    achieved = L.ops / (contraction_ms[dom] * 1e-3) / 1e12
    if kern[dom]["launches"] == 1:  # fp16 activations, weight bits, scales in; fp16 out
        alg_bytes = L.M * L.K * 2 + L.N * L.rw * 4 + 2 * (L.M + L.N) + 2 * L.M * L.N
    else:
        alg_bytes = L.gemm_prepared_bytes()
    other = [{"layer": kern[i]["layer"], "kernel": names[i], "us": round(contraction_ms[i] * 1e3, 2),
              "achieved": round(layers[i].ops / (contraction_ms[i] * 1e-3) / 1e12, 2),
              "frac": round(layers[i].ops / (contraction_ms[i] * 1e-3) / 1e12 / PEAK_FP4_TOPS, 4)}
             for i in range(len(layers)) if i != dom]
    roofline = {"bound": "mfma",
                "kernel": "%s on %s (%s), %.2f us per launch" % (names[dom], kern[dom]["layer"],
                                                                "ternarise + FP4 MFMA product + scale epilogue"
                                                                if kern[dom]["launches"] == 1 else
                                                                "FP4 MFMA product + scale epilogue",
                                                                contraction_ms[dom] * 1e3),
                "achieved": round(achieved, 2), "peak": PEAK_FP4_TOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_FP4_TOPS, 4), "frac_of_int8_peak": round(achieved / PEAK_INT8_TOPS, 4),
                # this layer mostly stores: 25 MB of fp16 out of a 19 Gflop product
                "algorithmic_bytes": alg_bytes,
                "frac_of_hbm_peak": round(alg_bytes / (contraction_ms[dom] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                # HBM/fabric bytes per launch of this kernel from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
                # runs scaled by the copy probe (profiles/traffic_c2_ffn.md)
                "traffic": _traffic_from_profiles(B, names[dom], "M=%d N=%d K=%d" % (L.M, L.N, L.K)),
                "other_contraction_kernels": other}
    out = {"metric": "BWTA linear effective TOPS (ternarize+pack+GEMM+epilogue), encoder FFN shapes",
           "value": round(value, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "fp4 (E2M1 operands, exact integer result in fp32)", "data": "synthetic",
           "config": {"workload": "c2_ffn: M=4096 (32x128 tokens), K=768->N=3072 and K=3072->N=768, fp16 in/out",
                      "path": "full (bwta_linear x2 per step)", "launch": "hip graph replay" if args.graph else "eager",
                      "clock_settle_ms": int(SETTLE_S * 1e3)},
           "roofline": roofline, "kernels": kern}
    if not args.no_cpu:
        import oracle
        for c in cfgs:
            c["s_a"] = oracle.act_scale(c["A"])
        out["cpu_baseline"] = cpu_baseline_c2(cfgs)
    return out


def cpu_baseline_c3(cfgs, target_s=10.0):
    """The oracle as it stands on the headline workload: its triple loop over the unpacked operands
    and its scale epilogue, whole matrices (all tokens of all three shapes), repeated to ~target_s."""
    import oracle
    threads = oracle.num_threads()
    ops_per_pass = sum(2.0 * c["M"] * c["N"] * c["K"] for c in cfgs)
    t0 = time.perf_counter()
    passes = 0
    while True:
        for c in cfgs:
            acc = oracle.gemm_unpacked(c["t"], c["w"])
            oracle.epilogue(acc, c["s_a"], c["s_w"])
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= target_s or passes >= 20:
            break
    return {"value": round(ops_per_pass * passes / dt / 1e12, 5), "unit": "TOPS", "cores": threads, "kind": "oracle",
            "sample": "%d full passes of the same three products and epilogues (all %d tokens), %.1f s"
                      % (passes, cfgs[0]["M"], dt)}


def run_headline(args, torch, B, synth):
    """Headline: the 7B prefill shapes (the configuration the metric and target are stated on), with
    the other configurations as sub-records of the same line."""
    cfgs = [synth.config3(w) for w in ("qkvo", "upgate", "down")]
    layers = [Layer(c, torch, B, from_fp16=False) for c in cfgs]

    def eager_step():
        for L in layers:
            L.gemm(B)

    step = eager_step
    if args.graph:  # the same six launches replayed from a HIP graph; every replay checked against eager below
        def check(want):
            got = [L.out.clone() for L in layers]
            if want is not None:
                for a, b in zip(got, want):
                    assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "graph replay differs from eager"
            for L in layers:
                L.out.fill_(float("nan"))
            return got
        graph = _graph_of(torch, eager_step, check)
        step = graph.replay

    _settle(torch, step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    ops = sum(L.ops for L in layers)
    value = ops / (ms_per_step * 1e-3) / 1e12

    # per shape: the call as benchmarked (planes in: converter + tiled kernel), the tiled kernel alone
    # (fragments prepared, as inside bwta_linear) and the activation packer, HIP events on the launch stream
    reps = max(50, args.steps // 10)
    kern = []
    for L, c in zip(layers, cfgs):
        L.prepare_from_ternary(B, torch)
        tg = _event_ms(torch, lambda: L.gemm(B), reps, 5)
        tk = _event_ms(torch, lambda: L.gemm_prepared(B), reps, 5)
        tp = _event_ms(torch, lambda: L.pack(B), reps, 5)
        kern.append({"layer": c["name"], "M": L.M, "N": L.N, "K": L.K,
                     "kernel_id": B.planned_kernel(0, L.M, L.N, L.K),
                     "bwta_gemm_us": round(tg * 1e3, 2), "bwta_gemm_TOPS": round(L.ops / (tg * 1e-3) / 1e12, 1),
                     "k_gemm_fp4_alone_us": round(tk * 1e3, 2),
                     "k_gemm_fp4_alone_TFLOPs": round(L.ops / (tk * 1e-3) / 1e12, 1),
                     "pack_act_us": round(tp * 1e3, 2),
                     "pack_act_GBs": round((L.M * L.K * 1.25) / (tp * 1e-3) / 1e9, 1),
                     "with_pack_TOPS": round(L.ops / ((tg + tp) * 1e-3) / 1e12, 1)})
    dom = max(range(len(layers)), key=lambda i: kern[i]["k_gemm_fp4_alone_us"])
    L = layers[dom]
    dom_us = kern[dom]["k_gemm_fp4_alone_us"]
    achieved = L.ops / (dom_us * 1e-6) / 1e12
    roofline = {"bound": "mfma",
                "kernel": "k_gemm_fp4_lds (LDS-staged tiled FP4 MFMA product + scale epilogue) on %s, M=%d N=%d K=%d, %.2f us per launch"
                          % (kern[dom]["layer"], L.M, L.N, L.K, dom_us),
                "achieved": round(achieved, 1), "peak": PEAK_FP4_TOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_FP4_TOPS, 4), "frac_of_int8_peak": round(achieved / PEAK_INT8_TOPS, 4),
                "flops_per_launch": L.ops,
                "traffic": _traffic_from_profiles(B, "k_gemm_fp4_lds", "M=%d N=%d K=%d" % (L.M, L.N, L.K)),
                # the same three products on operands already in the kernel's fragment layout (what
                # bwta_linear / bwta_prepare_act feed it): sum of the per-shape kernel times above
                "step_from_prepared_operands_TOPS": round(sum(L_.ops for L_ in layers) / sum(k["k_gemm_fp4_alone_us"] for k in kern) / 1e6, 1),
                "whole_step_frac_of_int8_peak": round(value / PEAK_INT8_TOPS, 4),
                "whole_step_frac_of_fp4_peak": round(value / PEAK_FP4_TOPS, 4)}
    out = {"metric": "BWTA GEMM effective TOPS (prefill) + achieved HBM GB/s (decode), 1 MI355X",
           "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "fp4 (E2M1 operands, exact integer result in fp32)", "data": "synthetic",
           "config": {"workload": "c3_prefill: M=2048 ternary activations P(0)=0.5, (K,N) in {(4096,4096),(4096,11008),"
                                  "(11008,4096)}; one step = bwta_gemm (product + scale epilogue from packed planes) "
                                  "on all three",
                      "launch": "hip graph replay" if args.graph else "eager", "clock_settle_ms": int(SETTLE_S * 1e3),
                      "build_id": B.build_id()},
           "roofline": roofline, "kernels": kern}
    del layers
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline_c3(cfgs)
    del cfgs
    if args.no_sub:
        return out
    torch.cuda.empty_cache()
    # ---- sub-records: the other configurations, each timed the way its own workload does
    dec = decode_cases(args, torch, B, synth)
    gbs = [r["GBs_median"] for r in dec]
    out["decode_c4"] = {"metric": "achieved HBM GB/s, weights streamed once", "unit": "GB/s",
                        "value_median_mean": round(float(np.mean(gbs)), 1),
                        "frac_of_hbm_peak": round(float(np.mean(gbs)) / PEAK_HBM_GBS, 4),
                        "min_case_frac_of_hbm_peak": round(min(gbs) / PEAK_HBM_GBS, 4),
                        "matrices_per_launch": args.decode_matrices, "launches_per_case": max(20, args.decode_reps),
                        "cases": dec}
    torch.cuda.empty_cache()
    sub = argparse.Namespace(**vars(args))
    sub.no_cpu, sub.graph, sub.steps, sub.warmup = True, False, 1000, 500
    c2 = run_c2(sub, torch, B, synth)
    out["ffn_c2"] = {"metric": c2["metric"], "value": c2["value"], "unit": "TOPS", "us_per_step": round(c2["ms_per_step"] * 1e3, 2),
                     "workload": c2["config"]["workload"], "dominant_kernel": c2["roofline"]["kernel"],
                     "dominant_frac_of_fp4_peak": c2["roofline"]["frac"],
                     "dominant_frac_of_hbm_peak": c2["roofline"]["frac_of_hbm_peak"], "kernels": c2["kernels"]}
    torch.cuda.empty_cache()
    sub.steps = 100
    c5 = run_c5(sub, torch, B, synth)
    out["block_c5"] = {"metric": c5["metric"], "block_us": c5["value"], "workload": c5["config"]["workload"], **c5["kernels"]}
    return out


def run_c3(args, torch, B, synth):
    res = []
    tot_ops = tot_ms = 0.0
    for which in ("qkvo", "upgate", "down"):
        c = synth.config3(which)
        L = Layer(c, torch, B, from_fp16=False)
        per = {}
        for name, path in (("fp4", B.PATH_FP4), ("mfma", B.PATH_MFMA), ("popc", B.PATH_POPC)):
            B.set_path(path)
            ms = _event_ms(torch, lambda: L.gemm(B), args.steps, args.warmup)
            per[name + "_us"] = round(ms * 1e3, 1)
            per[name + "_TOPS"] = round(L.ops / (ms * 1e-3) / 1e12, 1)
        B.set_path(B.PATH_AUTO)
        ms = _event_ms(torch, lambda: L.gemm(B), args.steps, args.warmup)
        tot_ops += L.ops
        tot_ms += ms
        res.append(dict(layer=c["name"], M=L.M, N=L.N, K=L.K, auto_us=round(ms * 1e3, 1),
                        auto_TOPS=round(L.ops / (ms * 1e-3) / 1e12, 1), **per))
        del L
    value = tot_ops / (tot_ms * 1e-3) / 1e12
    return {"metric": "BWTA GEMM effective TOPS (prefill linears from packed planes)", "value": round(value, 2),
            "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(tot_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4 (E2M1 operands, exact integer result in fp32)", "data": "synthetic",
            "config": {"workload": "c3_prefill: M=2048, (K,N) in {(4096,4096),(4096,11008),(11008,4096)}"},
            # the dispatcher's kernel contracts in FP4 (k_planes_to_fp4 + k_gemm_fp4, timed together); the
            # int8 dense peak is the bar the target for these shapes is stated against
            "roofline": {"bound": "mfma", "kernel": "k_planes_to_fp4 + k_gemm_fp4 (bwta_gemm from packed planes)",
                         "achieved": round(value, 2), "peak": PEAK_FP4_TOPS, "unit": "TFLOP/s",
                         "frac": round(value / PEAK_FP4_TOPS, 4), "frac_of_int8_peak": round(value / PEAK_INT8_TOPS, 4),
                         "traffic": None},
            "kernels": res}


def decode_cases(args, torch, B, synth, families=False):
    """Decode: stream `nmat` distinct packed weight matrices (more than the Infinity Cache holds) per
    timed region through one grouped call (one kernel launch per 64 matrices).  Every case is timed
    as `reps` (at least 20) grouped launches, each between its own pair of HIP events; the median
    and the best launch are reported, plus the latency of one matrix launched alone."""
    nmat = args.decode_matrices
    reps = max(20, args.decode_reps)
    res = []
    only = getattr(args, "decode_only", None)  # "down:16:fp4": one shape, one token count, one kernel family
    only = only.split(":") if only else None
    for which in ("upgate", "down"):
        for M in (1, 4, 16):
            if only and (which != only[0] or M != int(only[1])):
                continue
            c = synth.config4(which, M)
            L = Layer(c, torch, B, from_fp16=False)
            # distinct weight matrices: rotate the packed rows so the bits differ
            mats = [torch.roll(L.wsign, shifts=i, dims=0).contiguous() for i in range(nmat)]
            outs = [torch.empty_like(L.out) for _ in range(nmat)]
            ws = torch.empty(max(B.workspace_bytes(L.M, L.N, L.K), 256) * nmat, dtype=torch.uint8, device="cuda:0")
            probs = B.make_problems([(L.mask, L.sign, w, L.s_a, L.s_w, None, o) for w, o in zip(mats, outs)])

            def grouped():
                B.bwta_gemm_grouped(probs, ws, M=L.M, N=L.N, K=L.K)

            def case(path):
                B.set_path(path)
                try:
                    _launch_times_ms(torch, grouped, 5)  # first touch of 64 fresh matrices, clock
                    t = sorted(_launch_times_ms(torch, grouped, reps))
                finally:
                    B.set_path(B.PATH_AUTO)
                return t[len(t) // 2] / nmat, t[0] / nmat

            first = {"popc": B.PATH_POPC, "fp4": B.PATH_FP4}[only[2]] if only and len(only) > 2 else B.PATH_AUTO
            med, best = case(first)
            bytes_ = L.gemm_bytes()
            r = dict(layer=c["name"], M=M, N=L.N, K=L.K, path=_kernel_path_name(B, L.M, L.N, L.K),
                     us_per_matrix_median=round(med * 1e3, 3), us_per_matrix_best=round(best * 1e3, 3),
                     GBs_median=round(bytes_ / (med * 1e-3) / 1e9, 1), GBs_best=round(bytes_ / (best * 1e-3) / 1e9, 1),
                     frac_hbm_median=round(bytes_ / (med * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     algorithmic_bytes_per_matrix=bytes_)
            if families and not only:  # the other kernel family on the same case
                r["popc_us_median"] = round(case(B.PATH_POPC)[0] * 1e3, 3)
                r["fp4_us_median"] = round(case(B.PATH_FP4)[0] * 1e3, 3)
                r["single_launch_us"] = round(_event_ms(torch, lambda: L.gemm(B), args.steps, args.warmup) * 1e3, 2)
            res.append(r)
            del mats, outs, ws, L
    return res


def run_c4(args, torch, B, synth):
    res = decode_cases(args, torch, B, synth, families=True)
    nmat = args.decode_matrices
    mean = float(np.mean([r["GBs_median"] for r in res]))
    return {"metric": "BWTA decode GEMM achieved HBM GB/s (weights streamed once)", "value": round(mean, 1),
            "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(float(np.mean([r["us_per_matrix_median"] for r in res])) / 1e3, 6),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4 (E2M1 operands, exact) from 2 tokens, int32 popcount at 1",
            "data": "synthetic",
            "config": {"workload": "c4_decode: M in {1,4,16}, (K,N) in {(4096,11008),(11008,4096)}, %d distinct "
                                   "weight matrices per timed region (bwta_gemm_grouped), median of %d launches"
                                   % (nmat, max(20, args.decode_reps))},
            "roofline": {"bound": "hbm", "achieved": round(mean, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(mean / PEAK_HBM_GBS, 4), "traffic": None},
            "kernels": res}


def run_attn(args, torch, B, synth):
    """The two attention MatMuls at the decoder block's shapes: 32 heads, 2048 tokens, head dim 128.
    Operands are packed once (ternary Q, K, V^T; boolean Att with ~10 % ones, like thresholded
    attention probabilities); the products are timed alone and with their packers."""
    H, S, D = 32, 2048, 128
    dev = "cuda:0"
    rw_d, rw_s = B.plane_row_words(D), B.plane_row_words(S)
    q = _dev(synth.laplace_activations(6, 1, H * S, D), torch)
    k = _dev(synth.laplace_activations(6, 2, H * S, D), torch)
    vt = _dev(synth.laplace_activations(6, 3, H * D, S), torch)
    # one head's |N(0,1)| * 0.3 against a threshold of 0.5: 9.5 % ones; the same head repeated for all heads
    att = _dev((np.abs(synth.gaussian(6, 4, S * S)) * 0.3).astype(np.float16).reshape(S, S), torch).repeat(H, 1)
    one = torch.ones(1, dtype=torch.float16, device=dev)
    s_att = torch.full((1,), 1.0, dtype=torch.float16, device=dev)
    planes = lambda rows, rw: (torch.empty((rows, rw), dtype=torch.int32, device=dev), torch.empty((rows, rw), dtype=torch.int32, device=dev))
    qm, qs = planes(H * S, rw_d)
    km, ks = planes(H * S, rw_d)
    vm, vs = planes(H * D, rw_s)
    am, _ = planes(H * S, rw_s)
    scores = torch.empty((H, S, S), dtype=torch.float16, device=dev)
    ctx = torch.empty((H, S, D), dtype=torch.float16, device=dev)

    def pack_qk():
        B.bwta_quantize_pack_act(q, one, qm, qs, None, M=H * S, K=D)
        B.bwta_quantize_pack_act(k, one, km, ks, None, M=H * S, K=D)

    def pack_att_v():
        B.bwta_quantize_pack_bool(att, s_att, am, M=H * S, K=S)
        B.bwta_quantize_pack_act(vt, one, vm, vs, None, M=H * D, K=S)

    def qk():
        B.bwta_matmul_tt(qm, qs, km, ks, one, one, None, scores, batch=H, M=S, N=S, K=D, alpha=1.0 / D ** 0.5)

    def av():
        B.bwta_matmul_tt(am, None, vm, vs, s_att, one, None, ctx, batch=H, M=S, N=D, K=S)

    pack_qk(); pack_att_v(); torch.cuda.synchronize()
    steps = max(5, args.steps // 10)
    t = {n: _event_ms(torch, f, steps, 2) for n, f in (("pack_qk", pack_qk), ("qk", qk), ("pack_att_v", pack_att_v), ("att_v", av))}
    # the popcount kernels behind the same call, for comparison
    B.set_path(B.PATH_POPC)
    t_popc = {n: _event_ms(torch, f, steps, 2) for n, f in (("qk", qk), ("att_v", av))}
    B.set_path(B.PATH_AUTO)
    # Att V with V^T prepared once as matrix-core fragments (the boolean plane then plays the weights'
    # part in the tiled kernel): same bits, checked here against the planes-in-registers product
    prep_v = torch.empty(B.prepared_bytes(H * D, S), dtype=torch.uint8, device=dev)
    ctx2 = torch.zeros_like(ctx)

    fmt_v = B.prepared_format(H * D, S)

    def prepare_v():
        B.bwta_prepare_act(vt, one, prep_v, M=H * D, K=S)

    def av_prepared():
        B.bwta_matmul_bool_prepared(am, prep_v, s_att, one, ctx2, fmt=fmt_v, batch=H, M=S, N=D, K=S)

    av(); prepare_v(); av_prepared(); torch.cuda.synchronize()
    assert torch.equal(ctx.view(torch.int16), ctx2.view(torch.int16)), "the two Att V products differ"
    t_prep = {n: _event_ms(torch, f, steps, 2) for n, f in (("prepare_v", prepare_v), ("att_v_prepared", av_prepared))}
    ops = 2.0 * H * S * S * D
    total = sum(t.values())
    kern = {n + "_us": round(v * 1e3, 1) for n, v in t.items()}
    kern.update({n + "_us": round(v * 1e3, 1) for n, v in t_prep.items()})
    kern.update(att_v_prepared_TOPS=round(ops / (t_prep["att_v_prepared"] * 1e-3) / 1e12, 1))
    kern.update(qk_TOPS=round(ops / (t["qk"] * 1e-3) / 1e12, 1), att_v_TOPS=round(ops / (t["att_v"] * 1e-3) / 1e12, 1),
                qk_popc_us=round(t_popc["qk"] * 1e3, 1), att_v_popc_us=round(t_popc["att_v"] * 1e3, 1))
    achieved = 2 * ops / ((t["qk"] + t["att_v"]) * 1e-3) / 1e12
    # dominant kernel: the Q K^T product, bound by storing the fp16 score matrix (planes in, scores out)
    qk_bytes = 2.0 * H * S * S + 4 * H * S * rw_d * 4
    qk_gbs = qk_bytes / (t["qk"] * 1e-3) / 1e9
    kern.update(pack_att_v_GBs=round((2.0 * H * S * S + H * S * rw_s * 4 + 2.0 * H * D * S + 2 * H * D * rw_s * 4)
                                     / (t["pack_att_v"] * 1e-3) / 1e9, 1))
    return {"metric": "BWTA attention MatMuls effective TOPS (QK^T and Att V, 32 heads x 2048 x 128)",
            "value": round(achieved, 1), "unit": "TOPS", "n_gpus": 1, "steps": steps, "warmup": 2,
            "ms_per_step": round(total, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "fp4 (E2M1 operands, exact integer result in fp32)", "data": "synthetic",
            "config": {"workload": "attn: BWTA_QK ternary x ternary [2048,128]x[128,2048] and BWTA_Att bool x ternary "
                                   "[2048,2048]x[2048,128], 32 heads"},
            "roofline": {"bound": "hbm", "kernel": "k_matmul_tt_fp4 on Q K^T (fp16 score matrix out)",
                         "achieved": round(qk_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(qk_gbs / PEAK_HBM_GBS, 4), "traffic": None},
            "kernels": kern}


def run_c1(args, torch, B, synth):
    c = synth.config1()
    L = Layer(c, torch, B, from_fp16=False)
    res = {}
    for name, path in (("mfma", B.PATH_MFMA), ("popc", B.PATH_POPC)):
        B.set_path(path)
        res[name + "_us"] = round(_event_ms(torch, lambda: L.gemm(B), args.steps, args.warmup) * 1e3, 2)
    B.set_path(B.PATH_AUTO)
    ms = _event_ms(torch, lambda: L.gemm(B), args.steps, args.warmup)
    return {"metric": "BWTA tiny GEMM latency", "value": round(ms * 1e3, 2), "unit": "us", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 6), "higher_is_better": False,
            "scaling": "weak", "vs_baseline": None, "dtype": "fp4 (E2M1 operands, exact integer result in fp32)",
            "data": "synthetic", "config": {"workload": "c1_tiny: M=64, N=768, K=768",
                                            "path": _kernel_path_name(B, L.M, L.N, L.K)}, "kernels": res}


class Block:
    """One 7B-style decoder block: the seven linears are BWTA layers (ternarise on the fly, one
    ternarisation shared by Q/K/V and by gate/up; the per-token activation scale, the value
    training starts the scale from, is computed in the same pass: bwta_prepare_act_autoscale);
    norms, attention and SiLU are plain torch fp16 ops (the paper keeps nonlinearities in high
    precision)."""

    def __init__(self, cfg, torch, B):
        self.torch, self.B = torch, B
        self.S, self.H, self.F, self.heads = cfg["seq"], cfg["hidden"], cfg["ffn"], cfg["heads"]
        dev = "cuda:0"
        self.x = _dev(cfg["x"], torch)
        self.w, self.sw = {}, {}
        for nm, K, N in [("wq", self.H, self.H), ("wk", self.H, self.H), ("wv", self.H, self.H), ("wo", self.H, self.H),
                         ("wgate", self.H, self.F), ("wup", self.H, self.F), ("wdown", self.F, self.H)]:
            wd = _dev(cfg[nm], torch)
            ws = torch.empty((N, B.plane_row_words(K)), dtype=torch.int32, device=dev)
            B.bwta_pack_weights(wd, ws, N=N, K=K)
            self.w[nm], self.sw[nm] = ws, _dev(cfg["s_" + nm], torch)
            del wd
        S, H, F = self.S, self.H, self.F
        self.prep_h = torch.empty(B.prepared_bytes(S, H), dtype=torch.uint8, device=dev)
        self.prep_f = torch.empty(B.prepared_bytes(S, F), dtype=torch.uint8, device=dev)
        self.q, self.k, self.v, self.o = (torch.empty((S, H), dtype=torch.float16, device=dev) for _ in range(4))
        self.g, self.u = (torch.empty((S, F), dtype=torch.float16, device=dev) for _ in range(2))
        self.d = torch.empty((S, H), dtype=torch.float16, device=dev)
        torch.cuda.synchronize()

    def _norm(self, x):
        xf = x.float()
        return (xf * self.torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + 1e-6)).half()

    def _scale(self, a):  # the value the activation scale is initialised with, per token: 2 mean|a|
        s = self.torch.empty((a.shape[0],), dtype=self.torch.float16, device=a.device)
        self.B.bwta_act_scale(a, s, M=a.shape[0], K=a.shape[1])
        return s

    def _prep(self, a, prep, K):  # token scales and the ternarised operand in one pass over the activations
        s = self.torch.empty((a.shape[0],), dtype=self.torch.float16, device=a.device)
        self.fmt = self.B.bwta_prepare_act_autoscale(a, s, prep, M=a.shape[0], K=K)
        return s

    def _lin(self, prep, s_a, nm, out, K, N):
        self.B.bwta_gemm_prepared(prep, self.w[nm], s_a, self.sw[nm], None, out, fmt=self.fmt, M=self.S, N=N, K=K)

    def _attention_buffers(self):
        torch, B, S, heads, hd = self.torch, self.B, self.S, self.heads, self.H // self.heads
        if hasattr(self, "scores"):
            return
        dev = "cuda:0"
        rw_d, rw_s = B.plane_row_words(hd), B.plane_row_words(S)
        i32 = lambda *shape: torch.empty(shape, dtype=torch.int32, device=dev)
        f16 = lambda *shape: torch.empty(shape, dtype=torch.float16, device=dev)
        self.qm, self.qs, self.km, self.ks = (i32(heads * S, rw_d) for _ in range(4))
        self.am = i32(heads * S, rw_s)
        self.s_q, self.s_k, self.s_p = f16(heads * S), f16(heads * S), f16(heads * S)
        self.s_v = f16(heads * hd)
        self.prep_v = torch.empty(B.prepared_bytes(heads * hd, S), dtype=torch.uint8, device=dev)
        self.scores = f16(heads, S, S)
        self.ctx = f16(heads, S, hd)
        self.causal = torch.ones((S, S), dtype=torch.bool, device=dev).triu_(1)

    def bwta_attention(self):
        """The paper's attention MatMuls in place of fp16 attention: scores = BWTA_QK(ternary(Q),
        ternary(K)) / sqrt(d) (arithmetic Case 3), context = BWTA_Att(bool(softmax), ternary(V))
        (Case 2).  Every operand's scale is the value training starts it from, per row (2 mean|.|),
        computed by the library; the causal mask, the softmax and the head-major / transposed
        layouts are plain tensor ops of the caller."""
        torch, B, S, heads, hd = self.torch, self.B, self.S, self.heads, self.H // self.heads
        self._attention_buffers()
        rows = heads * S
        self.qh = self.q.view(S, heads, hd).transpose(0, 1).contiguous().view(rows, hd)
        self.kh = self.k.view(S, heads, hd).transpose(0, 1).contiguous().view(rows, hd)
        self.vt = self.v.view(S, heads, hd).permute(1, 2, 0).contiguous().view(heads * hd, S)
        for x, s, m, sg in ((self.qh, self.s_q, self.qm, self.qs), (self.kh, self.s_k, self.km, self.ks)):
            B.bwta_act_scale(x, s, M=rows, K=hd)
            B.bwta_quantize_pack_act(x, s, m, sg, None, M=rows, K=hd)
        B.bwta_matmul_tt(self.qm, self.qs, self.km, self.ks, self.s_q, self.s_k, None, self.scores, batch=heads, M=S, N=S,
                         K=hd, alpha=1.0 / hd ** 0.5)
        self.probs = torch.softmax(self.scores.masked_fill(self.causal, float("-inf")), dim=-1, dtype=torch.float32).half()
        pr = self.probs.view(rows, S)
        B.bwta_act_scale(pr, self.s_p, M=rows, K=S)
        B.bwta_quantize_pack_bool(pr, self.s_p, self.am, M=rows, K=S)
        fmt = B.bwta_prepare_act_autoscale(self.vt, self.s_v, self.prep_v, M=heads * hd, K=S)
        B.bwta_matmul_bool_prepared(self.am, self.prep_v, self.s_p, self.s_v, self.ctx, fmt=fmt, batch=heads, M=S, N=hd, K=S)
        return self.ctx.transpose(0, 1).reshape(S, self.H).contiguous()

    def forward(self, bwta_only=False, attention="fp16"):
        """bwta_only: run just the 4 ternarisations and 7 products on whatever the buffers hold.
        attention: "fp16" (plain reference attention) or "bwta" (the paper's two attention MatMuls)."""
        torch, B, S, H, F = self.torch, self.B, self.S, self.H, self.F
        h = self.h if bwta_only else self._norm(self.x)
        s = self.s_h = self._prep(h, self.prep_h, H)
        for nm, out in (("wq", self.q), ("wk", self.k), ("wv", self.v)):
            self._lin(self.prep_h, s, nm, out, H, H)
        if bwta_only:
            att = self.att
        elif attention == "bwta":
            att = self.bwta_attention()
        else:
            hd = H // self.heads
            q, k, v = (t.view(S, self.heads, hd).transpose(0, 1).unsqueeze(0) for t in (self.q, self.k, self.v))
            att = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
            att = att.squeeze(0).transpose(0, 1).reshape(S, H).contiguous()
        s2 = self.s_att = self._prep(att, self.prep_h, H)
        self._lin(self.prep_h, s2, "wo", self.o, H, H)
        if bwta_only:
            h2 = self.h2
        else:
            x1 = self.x + self.o
            h2 = self._norm(x1)
        s3 = self.s_h2 = self._prep(h2, self.prep_h, H)
        self._lin(self.prep_h, s3, "wgate", self.g, H, F)
        self._lin(self.prep_h, s3, "wup", self.u, H, F)
        act = self.act if bwta_only else torch.nn.functional.silu(self.g) * self.u
        s4 = self.s_act = self._prep(act, self.prep_f, F)
        self._lin(self.prep_f, s4, "wdown", self.d, F, H)
        if bwta_only:
            return None
        self.h, self.att, self.h2, self.act = h, att, h2, act
        return x1 + self.d


def run_c5(args, torch, B, synth):
    blk = Block(synth.config5(), torch, B)
    y = blk.forward()
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y).all()), "block output is not finite"
    steps = max(5, args.steps // 10)
    ms_block = _event_ms(torch, blk.forward, steps, 3)
    ms_bwta = _event_ms(torch, lambda: blk.forward(bwta_only=True), steps, 3)
    y2 = blk.forward(attention="bwta")
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y2).all()), "block output is not finite (BWTA attention)"
    ms_block_att = _event_ms(torch, lambda: blk.forward(attention="bwta"), steps, 3)
    ms_att = _event_ms(torch, blk.bwta_attention, steps, 3)
    S, H, F = blk.S, blk.H, blk.F
    ops = 2.0 * S * (4 * H * H + 3 * H * F)
    return {"metric": "BWTA decoder block latency (7 BWTA linears + fp16 attention/norms)", "value": round(ms_block * 1e3, 1),
            "unit": "us", "n_gpus": 1, "steps": steps, "warmup": 3, "ms_per_step": round(ms_block, 5),
            "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "fp4 (E2M1 operands, exact)",
            "data": "synthetic",
            "config": {"workload": "c5_block: hidden 4096, FFN 11008, 32 heads, seq 2048, batch 1; Laplace(0,1) input"},
            "kernels": {"bwta_part_us": round(ms_bwta * 1e3, 1), "bwta_share": round(ms_bwta / ms_block, 3),
                        "bwta_effective_TOPS": round(ops / (ms_bwta * 1e-3) / 1e12, 1),
                        "block_with_bwta_attention_us": round(ms_block_att * 1e3, 1),
                        "bwta_attention_part_us": round(ms_att * 1e3, 1),
                        "note": "bwta part = 4 ternarisations (each computing its per-token scales in the same "
                                "pass) + 7 products; the rest is torch fp16 attention, RMSNorm, SiLU and residuals.  "
                                "block_with_bwta_attention: the same block with the paper's attention MatMuls "
                                "(BWTA_QK ternary x ternary, BWTA_Att bool x ternary; its part = head-major copies, "
                                "scales, packers, both products, causal softmax) in place of fp16 attention"}}


def run_prep(args, torch, B, synth):
    """Weight preparation from an fp16 matrix (centre, sign-pack, per-channel scale) and the per-token
    activation-scale statistic, at the decoder block's largest shapes; both read their input once."""
    dev = "cuda:0"
    N, K, M = 4096, 11008, 2048
    W = _dev((synth.gaussian(7, 1, N * K) * 0.02).astype(np.float16).reshape(N, K), torch)
    A = _dev(synth.laplace_activations(7, 2, M, K), torch)
    wsign = torch.empty((N, B.plane_row_words(K)), dtype=torch.int32, device=dev)
    s_w = torch.empty((N,), dtype=torch.float16, device=dev)
    s_a = torch.empty((M,), dtype=torch.float16, device=dev)
    steps = max(5, args.steps // 10)
    tw = _event_ms(torch, lambda: B.bwta_prepare_weights(W, wsign, s_w, N=N, K=K), steps, 2)
    ta = _event_ms(torch, lambda: B.bwta_act_scale(A, s_a, M=M, K=K), steps, 2)
    prep = torch.empty(B.prepared_bytes(M, K), dtype=torch.uint8, device=dev)
    tp = _event_ms(torch, lambda: B.bwta_prepare_act(A, s_a, prep, M=M, K=K), steps, 2)
    tf = _event_ms(torch, lambda: B.bwta_prepare_act_autoscale(A, s_a, prep, M=M, K=K), steps, 2)
    bw = (2.0 * N * K + N * K / 8 + 2 * N) / (tw * 1e-3) / 1e9
    ba = (2.0 * M * K + 2 * M) / (ta * 1e-3) / 1e9
    return {"metric": "BWTA weight preparation achieved HBM GB/s", "value": round(bw, 1), "unit": "GB/s", "n_gpus": 1,
            "steps": steps, "warmup": 2, "ms_per_step": round(tw, 5), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "int64 (exact row sums of fp16 values)", "data": "synthetic",
            "config": {"workload": "prep: bwta_prepare_weights on fp16 [4096,11008]; bwta_act_scale, bwta_prepare_act and "
                                   "bwta_prepare_act_autoscale on fp16 [2048,11008]"},
            "roofline": {"bound": "hbm", "kernel": "k_prepare_weights", "achieved": round(bw, 1), "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": round(bw / PEAK_HBM_GBS, 4), "traffic": None},
            "kernels": {"prepare_weights_us": round(tw * 1e3, 1), "prepare_weights_GBs": round(bw, 1),
                        "act_scale_us": round(ta * 1e3, 1), "act_scale_GBs": round(ba, 1),
                        "prepare_act_us": round(tp * 1e3, 1), "scale_and_prepare_in_one_pass_us": round(tf * 1e3, 1),
                        "scale_and_prepare_in_one_pass_GBs": round((2.5 * M * K + 2 * M) / (tf * 1e-3) / 1e9, 1)}}


def run_short_k(args, torch, B, synth):
    """bwta_linear on short-K layers (encoder attention projections and the like), as one launch
    (the dispatcher's choice where it pays) and as ternarise + product (forced with the tuning hook)."""
    base = synth.config2("up")
    rows = []
    for (M, N, K) in [(4096, 768, 768), (4096, 768, 256), (4096, 3072, 256), (1024, 768, 768), (4096, 3072, 768),
                      (128, 768, 768), (16, 3072, 768)]:
        A = np.ascontiguousarray(np.tile(base["A"], (1, 2))[:M, :K])
        c = dict(M=M, N=N, K=K, A=A, w=synth.binary_pm1(8, N + K, (N, K)), s_w=synth.scales(8, 4, N), name="short_k")
        L = Layer(c, torch, B, from_fp16=True)
        B.set_tile(900)
        two = _event_ms(torch, lambda: L.linear(B), args.steps, args.warmup)
        B.set_tile(0)
        auto = _event_ms(torch, lambda: L.linear(B), args.steps, args.warmup)
        B.set_tile(901)
        one = _event_ms(torch, lambda: L.linear(B), args.steps, args.warmup)
        B.set_tile(0)
        rows.append({"M": M, "N": N, "K": K, "two_kernels_us": round(two * 1e3, 2), "one_launch_us": round(one * 1e3, 2),
                     "dispatcher_us": round(auto * 1e3, 2), "dispatcher_TOPS": round(L.ops / (auto * 1e-3) / 1e12, 1)})
        del L
    mean = float(np.mean([r["dispatcher_us"] for r in rows]))
    return {"metric": "BWTA linear latency on short-K layers", "value": round(mean, 2), "unit": "us", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(mean / 1e3, 6), "higher_is_better": False,
            "scaling": "weak", "vs_baseline": None, "dtype": "fp4 (E2M1 operands, exact integer result in fp32)",
            "data": "synthetic", "config": {"workload": "short_k: bwta_linear, fp16 in/out, K <= 768"}, "kernels": rows}


def run_copy_probe(args, torch, B, synth):
    """A plain device-to-device copy of known size (256 MiB), used to calibrate the FETCH_SIZE /
    WRITE_SIZE counters that the traffic figures in profiles/ are scaled by."""
    n = 256 << 20
    src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    ms = _event_ms(torch, lambda: dst.copy_(src), max(3, args.steps // 20), 2)
    gbs = 2 * n / (ms * 1e-3) / 1e9
    return {"metric": "device copy bandwidth (counter calibration probe)", "value": round(gbs, 1), "unit": "GB/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "copy_probe: 256 MiB read + 256 MiB written per launch"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 2000 for the headline and c2_ffn, 200 otherwise)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed steps first (default 500 for the headline, 1000 for c2_ffn: the clock ramp of an "
                         "idle GPU; 20 otherwise, where every timed region settles the clock itself)")
    ap.add_argument("--workload", default="headline",
                    choices=["headline", "c2_ffn", "c1_tiny", "c3_prefill", "c4_decode", "c5_block", "attn", "prep",
                             "short_k", "copy_probe"])
    ap.add_argument("--decode-matrices", type=int, default=64)
    ap.add_argument("--decode-reps", type=int, default=20, help="timed grouped launches per decode case (at least 20)")
    ap.add_argument("--decode-only", default=None, metavar="SHAPE:M[:FAMILY]",
                    help="c4_decode: one case only, e.g. down:16:fp4 (upgate|down, 1|4|16, popc|fp4); for counter runs")
    ap.add_argument("--no-sub", action="store_true", help="headline only: skip the c4 / c2 / c5 sub-records")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step from a HIP graph instead of launching eagerly (eager is the default: "
                         "the launch queue stays ahead of the GPU, and a 4-kernel graph replays no faster)")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 2000 if args.workload in ("headline", "c2_ffn") else 200
    if args.warmup is None:
        args.warmup = 500 if args.workload == "headline" else 1000 if args.workload == "c2_ffn" else 20
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the BWTA hot path is a single-GPU kernel "
              "path that uses no collectives). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    from paper_2604_03957_amd import binding as B
    import synth
    torch.cuda.set_device(0)
    run = {"headline": run_headline, "c2_ffn": run_c2, "c1_tiny": run_c1, "c3_prefill": run_c3, "c4_decode": run_c4,
           "c5_block": run_c5, "attn": run_attn, "prep": run_prep, "short_k": run_short_k,
           "copy_probe": run_copy_probe}[args.workload]
    out = run(args, torch, B, synth)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
