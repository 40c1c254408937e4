#!/usr/bin/env python3
"""Benchmark of the W4A8 linear-layer hot path on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input
already resident in HBM: token-wise FP8 quantization of X (plus the LoRC left
factor when the configuration has LoRC) followed by the W4A8 GEMM (with the
fused LoRC epilogue).  The weight packing is offline and not part of a step.

Prints ONE JSON line (see the keys below).  `value` is TFLOP/s of the step,
2*M*K*N / step time; `roofline` prices the GEMM kernel alone against the FP8
matrix-core peak (or HBM for decode-sized M), from HIP-event durations taken
inside the timed loop; `cpu_baseline` is the CPU oracle timed on a bounded
sample of the same workload; `also` lists the other shapes measured in the
same run (decode shapes rotate through weight copies totalling > 512 MB so
that the 256 MB last-level cache cannot serve them).
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2307_09782_amd import inputs, zqfp  # noqa: E402

METRIC = "W4A8 GEMM TFLOPS & HBM GB/s at LLaMA-7B/70B shapes; % FP8 MFMA/HBM roofline"
PEAK_FP8_TFLOPS = 5000.0   # MI355X dense FP8 matrix-core peak
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def f16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.float16).cuda()


def algorithmic_bytes(cfg, M, out_bytes=4):
    """Bytes the GEMM call itself must move once (packed codes + exponent bytes
    + column scales + FP8 activations + token scales + output + LoRC factors)."""
    K, N, G, r = cfg.K, cfg.N, cfg.G, cfg.rank
    w = K * N // 2 + (K // G) * N + 4 * N
    return w + M * K + 4 * M + out_bytes * M * N + (4 * M * r + 2 * r * N if r else 0)


# The GPU's clock takes some 50 ms of uninterrupted work to settle (launch times first rise, then fall below
# where they started): every timed region is preceded by this much of the same work, untimed, on top of
# the warm-up steps asked for on the command line.
SETTLE_S = 0.1


def timed_replays(g, replays, settle_s=0.06):
    """Milliseconds per replay of graph g, after replaying it untimed for `settle_s` seconds (clock settling)."""
    t0 = time.perf_counter()
    while True:
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        if time.perf_counter() - t0 >= settle_s:
            break
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(replays):
        g.replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / replays


class Workload:
    def __init__(self, name, M, accum, copies=1, out_dtype=torch.float32, w8=False):
        self.cfg = cfg = inputs.CONFIGS[name]
        self.name, self.M, self.accum, self.w8 = name, M, accum, w8
        self.X = bf16_dev(inputs.make_x(cfg, M))
        Wd = bf16_dev(inputs.make_w(cfg))
        packed = zqfp.pack_weight_fp8(Wd, cfg.G, cfg.mode) if w8 else zqfp.pack_weight_fp4(Wd, cfg.G, cfg.mode)
        del Wd
        self.packed = [packed] + [packed.clone() for _ in range(copies - 1)]
        self.U = self.V = None
        if cfg.rank:
            U, V = inputs.make_uv(cfg)
            self.U, self.V = f16_dev(U), f16_dev(V)
        self.Y = torch.empty((M, cfg.N), dtype=out_dtype, device="cuda")
        self.flops = 2.0 * M * cfg.K * cfg.N
        self.bytes = algorithmic_bytes(cfg, M, self.Y.element_size())
        self.fused = zqfp.linear_is_fused(M, cfg.K, cfg.rank) and not w8
        if w8:  # E4M3 weights: 1 byte per weight
            self.bytes += cfg.K * cfg.N // 2
        self.i = 0

    def step(self, ev=None):
        cfg = self.cfg
        packed = self.packed[self.i % len(self.packed)]
        self.i += 1
        if self.w8:
            Xq, sx = zqfp.quantize_act_fp8(self.X)
            if ev: ev[0].record()
            zqfp.w8a8_gemm(Xq, sx, packed, cfg.N, cfg.G, accum=self.accum, out=self.Y)
            if ev: ev[1].record()
        elif cfg.rank:
            Xq, sx, T = zqfp.quantize_act_fp8(self.X, self.U)
            if ev: ev[0].record()
            zqfp.w4a8_gemm_lorc(Xq, sx, packed, cfg.N, cfg.G, T, self.V, accum=self.accum, out=self.Y)
            if ev: ev[1].record()
        elif self.fused and not ev:
            # at most 16 tokens, K <= 4096, no LoRC: one kernel (the decode GEMM quantizes in its prologue)
            zqfp.w4a8_linear(self.X, packed, cfg.N, cfg.G, accum=self.accum, out=self.Y)
        else:
            Xq, sx = zqfp.quantize_act_fp8(self.X)
            if ev: ev[0].record()
            zqfp.w4a8_gemm(Xq, sx, packed, cfg.N, cfg.G, accum=self.accum, out=self.Y)
            if ev: ev[1].record()

    def run(self, steps, warmup, settle_s=SETTLE_S):
        # the device first: the same step, untimed, until the clock has settled (see SETTLE_S); then the W
        # warm-up steps that were asked for
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < settle_s:
            for _ in range(32):
                self.step()
            torch.cuda.synchronize()
        for _ in range(warmup):
            self.step()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            self.step(evs[k])
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        times = sorted(a.elapsed_time(b) for a, b in evs)
        self.kernel_ms_median, self.kernel_ms_min = times[len(times) // 2], times[0]
        gemm_ms = float(np.mean(times))
        return dt * 1e3, gemm_ms

    def gemm_graph_ms(self, replays=20):
        """Average GEMM kernel time with launch gaps removed: one HIP graph holding
        one GEMM launch per weight copy, replayed `replays` times."""
        cfg = self.cfg
        if cfg.rank:
            Xq, sx, T = zqfp.quantize_act_fp8(self.X, self.U)
        else:
            Xq, sx = zqfp.quantize_act_fp8(self.X)

        def launches():
            for packed in self.packed:
                if self.w8:
                    zqfp.w8a8_gemm(Xq, sx, packed, cfg.N, cfg.G, accum=self.accum, out=self.Y)
                elif cfg.rank:
                    zqfp.w4a8_gemm_lorc(Xq, sx, packed, cfg.N, cfg.G, T, self.V, accum=self.accum, out=self.Y)
                else:
                    zqfp.w4a8_gemm(Xq, sx, packed, cfg.N, cfg.G, accum=self.accum, out=self.Y)

        launches()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            launches()
        return timed_replays(g, replays) / len(self.packed)

    def step_graph_ms(self, replays=20):
        """Average time of the whole step (quantizer + GEMM) with host launch gaps removed: one HIP
        graph holding one step per weight copy, replayed `replays` times."""
        self.i = 0
        for _ in self.packed:
            self.step()
        torch.cuda.synchronize()
        self.i = 0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in self.packed:
                self.step()
        return timed_replays(g, replays) / len(self.packed)

    def summary(self, steps, warmup):
        ms, gemm_ms = self.run(steps, warmup)
        extra = {}
        if self.M <= 64:  # kernels of a few microseconds: take launch gaps out of the per-kernel figures
            gemm_ms = self.gemm_graph_ms()
            extra["graph_step_us"] = round(self.step_graph_ms() * 1e3, 2)  # quantizer + GEMM as two nodes of a HIP graph
            if self.fused:  # the one-kernel form (w4a8_linear) beside it: one launch instead of two
                extra["graph_step_us_fused"] = extra.pop("graph_step_us")
                self.fused = False
                extra["graph_step_us"] = round(self.step_graph_ms() * 1e3, 2)
                self.fused = True
        tflops = self.flops / (gemm_ms * 1e-3) / 1e12
        gbs = self.bytes / (gemm_ms * 1e-3) / 1e9
        # compact keys (the whole line must stay short): w = workload, acc = accumulation mode, step_us = eager step,
        # gemm_us = GEMM kernel alone, f_mfma / f_hbm = fraction of the FP8 matrix-core peak / of the HBM peak
        row = {"w": f"{self.name} M={self.M}", "acc": "exact" if self.accum == 0 else "fast",
               "step_us": round(ms * 1e3, 1), "gemm_us": round(gemm_ms * 1e3, 2), "tflops": round(tflops, 1),
               "gbs": round(gbs), "f_mfma": round(tflops / PEAK_FP8_TFLOPS, 4), "f_hbm": round(gbs / PEAK_HBM_GBS, 4)}
        if self.Y.dtype != torch.float32:
            row["out"] = "bf16"
        if self.w8:
            row["weights"] = "e4m3"
        if len(self.packed) > 1:
            row["copies"] = len(self.packed)
        row.update(extra)
        return row


def measured_traffic(workload_key):
    """HBM bytes per GEMM launch from the committed rocprofv3 counter runs (profiles/hbm_traffic.json,
    written from FETCH_SIZE / WRITE_SIZE calibrated on a copy of known size); None if not recorded."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    return json.load(open(path)).get(workload_key)


def calibration_copy(nbytes=1 << 30):
    """A plain device-to-device copy of known size: the yardstick for the HBM byte counters."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    torch.cuda.empty_cache()


def quantizer_rows(name="llama7b_qkv", M=4096):
    """The quantizer alone and behind its fused producers, HBM-bound (2 B read + 1 B written per element, plus
    what the producer reads and writes): one HIP graph of calls rotating through input copies that exceed the
    last-level cache."""
    cfg = inputs.CONFIGS[name]
    K = cfg.K
    X = bf16_dev(inputs.make_x(cfg, M))
    copies = max(1, -(-600_000_000 // (2 * M * K)))
    Xs = [X] + [X.clone() for _ in range(copies - 1)]
    gain = torch.ones(K, dtype=torch.bfloat16, device="cuda")
    bias = torch.zeros(K, dtype=torch.bfloat16, device="cuda")
    H = torch.empty_like(X)
    # the gated feed-forward input of the same model: 11008 channels, gate and up halves of one tensor
    Kf = inputs.CONFIGS["llama7b_ffn_up"].N
    GU = torch.randn((M, 2 * Kf), dtype=torch.float32, device="cuda").to(torch.bfloat16)
    GUs = [GU] + [GU.clone() for _ in range(max(1, -(-600_000_000 // (4 * M * Kf))) - 1)]
    rows = []
    for label, fn, ins, kk, nbytes in (
            ("quantize_act_fp8", lambda x: zqfp.quantize_act_fp8(x), Xs, K, 3 * M * K),
            ("rmsnorm_quantize_act_fp8", lambda x: zqfp.rmsnorm_quantize_act_fp8(x, gain, 1e-5), Xs, K, 3 * M * K + 2 * K),
            ("layernorm_quantize_act_fp8", lambda x: zqfp.layernorm_quantize_act_fp8(x, gain, bias, 1e-5), Xs, K,
             3 * M * K + 4 * K),
            ("add_rmsnorm_quantize_act_fp8", lambda xr: zqfp.add_norm_quantize_act_fp8(xr[0], xr[1], gain, 1e-5, H=H),
             list(zip(Xs, Xs[1:] + Xs[:1])), K, 7 * M * K + 2 * K),
            ("relu_quantize_act_fp8", lambda x: zqfp.relu_quantize_act_fp8(x), Xs, K, 3 * M * K),
            ("swiglu_quantize_act_fp8", lambda gu: zqfp.swiglu_quantize_act_fp8(gu[:, :Kf], gu[:, Kf:]), GUs, Kf, 5 * M * Kf)):
        for x in ins[:2]:
            fn(x)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for x in ins:
                fn(x)
        ms = timed_replays(g, 5) / len(ins)
        gbs = (nbytes + 4 * M) / (ms * 1e-3) / 1e9
        rows.append({"call": label, "w": f"{M}x{kk}", "us": round(ms * 1e3, 2), "gbs": round(gbs),
                     "f_hbm": round(gbs / PEAK_HBM_GBS, 4)})
    # with the rank-8 LoRC left factor T = X.U in the same sweep (LLaMA-13B FFN input, 2048 tokens)
    cfg13 = inputs.CONFIGS["llama13b_ffn_lorc"]
    X13 = bf16_dev(inputs.make_x(cfg13, 2048))
    U13 = f16_dev(inputs.make_uv(cfg13)[0])
    ins = [X13] + [X13.clone() for _ in range(max(1, -(-600_000_000 // (2 * 2048 * cfg13.K))) - 1)]
    zqfp.quantize_act_fp8(ins[0], U13)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for x in ins:
            zqfp.quantize_act_fp8(x, U13)
    ms = timed_replays(g, 5) / len(ins)
    nbytes = 3 * 2048 * cfg13.K + 4 * 2048 + 16 * cfg13.K + 32 * 2048
    rows.append({"call": "quantize_act_fp8 + T (rank 8)", "w": f"2048x{cfg13.K}", "us": round(ms * 1e3, 2),
                 "gbs": round(nbytes / (ms * 1e-3) / 1e9), "f_hbm": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})
    return rows


def offline_rows(name="llama7b_qkv", r=8, power_iters=2):
    """The LoRC factorisation of one layer's quantization error (offline step): time, and the rate at which
    it streams the float32 error matrix (one write, 2 + 2 * power_iters reads, plus W and the packed weight)."""
    cfg = inputs.CONFIGS[name]
    W = bf16_dev(inputs.make_w(cfg))
    packed = zqfp.pack_weight_fp4(W, cfg.G, cfg.mode)
    omega = torch.randn((cfg.N, r + 8), dtype=torch.float32, device="cuda")
    zqfp.lorc_factorize(W, packed, cfg.G, r, omega, power_iters)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(3):
        zqfp.lorc_factorize(W, packed, cfg.G, r, omega, power_iters)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / 3
    nbytes = cfg.K * cfg.N * (2 + 0.5 + 4 + 4 * (2 + 2 * power_iters))
    rows = [{"call": "lorc_factorize", "workload": f"{name} K={cfg.K} N={cfg.N} rank {r}, {power_iters} power iterations",
             "ms": round(ms, 4), "gbs": round(nbytes / (ms * 1e-3) / 1e9, 1)}]
    # GPTQ on the same layer: the float32 matrix products behind the row blocks dominate (K^2 N multiply-adds)
    U = torch.triu(torch.randn((cfg.K, cfg.K), dtype=torch.float32, device="cuda")) * 0.01 + torch.eye(cfg.K, device="cuda")
    zqfp.gptq_pack_weight_fp4(W, U, cfg.G, cfg.mode)
    torch.cuda.synchronize()
    a.record()
    zqfp.gptq_pack_weight_fp4(W, U, cfg.G, cfg.mode)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b)
    rows.append({"call": "gptq_pack_weight_fp4", "workload": f"{name} K={cfg.K} N={cfg.N} G={cfg.G}",
                 "ms": round(ms, 3), "tflops_f32": round(float(cfg.K) ** 2 * cfg.N / (ms * 1e-3) / 1e12, 2)})
    return rows


def measured_ceilings():
    """What the device itself sustains right now (measurement probes of the library, timed with HIP
    events): a plain streaming read of 2 GiB, twice the last-level cache eight times over, and a
    register-only loop of the FP8 x FP4 matrix instruction on every compute unit."""
    src = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").fill_(3)
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    ops = torch.randint(0, 2 ** 31 - 1, (1024,), dtype=torch.int32, device="cuda")
    wgs_mfma = 256
    fsink = torch.zeros(512 * wgs_mfma, dtype=torch.float32, device="cuda")

    def timed(fn, reps, warm):
        for _ in range(warm):  # long enough for the clock to settle
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    wgs_read = 2048
    ms_read = timed(lambda: zqfp.probe_stream_read(src, sink, wgs_read), 20, 120)
    read_bytes = (src.numel() // (wgs_read * 4 * 8 * 1024)) * (wgs_read * 4 * 8 * 1024)
    iters = 4000
    flop = [0.0]
    def mf():
        flop[0] = zqfp.probe_mfma(ops, fsink, iters, wgs_mfma)
    ms_mfma = timed(mf, 10, 12)
    del src
    torch.cuda.empty_cache()
    return {"stream_read_gbs": round(read_bytes / (ms_read * 1e-3) / 1e9, 1),
            "mfma_fp8xfp4_tflops": round(flop[0] / (ms_mfma * 1e-3) / 1e12, 1)}


def cpu_baseline(name, M, rows=4096):
    """The CPU oracle on a bounded sample: `rows` tokens of the same workload,
    whole hot path (quantize, LoRC left factor, GEMM over all N)."""
    import oracle
    cfg = inputs.CONFIGS[name]
    rows = min(rows, M)
    X = inputs.make_x(cfg, M)[:rows].copy()
    W = inputs.make_w(cfg)
    codes, exps, c, _ = oracle.pack_weight(W, cfg.G, cfg.mode)  # offline, not timed
    U = V = T = None
    if cfg.rank:
        U, V = inputs.make_uv(cfg)
    t0 = time.perf_counter()
    Xq, sx = oracle.quantize_act(X)
    if cfg.rank:
        T, _ = oracle.lorc_left(X, U)
    oracle.gemm(Xq, sx, codes, exps, c, cfg.G, T=T, V=V, want_abs=False)
    dt = time.perf_counter() - t0
    threads = min(oracle.max_threads(), rows)
    return {"value": round(2.0 * rows * cfg.K * cfg.N / dt / 1e12, 6), "unit": "TFLOP/s", "cores": threads,
            "kind": "oracle", "sample": f"{rows} of {M} tokens, all {cfg.N} outputs, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="llama7b_qkv")
    ap.add_argument("--M", type=int, default=4096)
    ap.add_argument("--accum", choices=["exact", "fast"], default="exact")
    ap.add_argument("--no-also", action="store_true", help="skip the extra shapes")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--only-quantizer", action="store_true",
                    help="run the quantizer rows alone and print them (for profiling the quantizer kernels)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (yardstick for rocprofv3 HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus must be 1 (nothing here uses a second GPU)")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    zqfp.lib()  # fail loudly if the HIP library has not been built
    accum = zqfp.ACCUM_EXACT if args.accum == "exact" else zqfp.ACCUM_FAST

    if args.calib_copy:
        calibration_copy()
    if args.only_quantizer:
        print(json.dumps({"quantizer": quantizer_rows()}), flush=True)
        return
    decode = args.M <= 64
    copies = 1
    if decode:  # HBM-bound: rotate through weight copies that together exceed the 256 MB last-level cache
        cfg0 = inputs.CONFIGS[args.workload]
        copies = min(64, max(1, -(-600_000_000 // (cfg0.K * cfg0.N // 2))))
    main_wl = Workload(args.workload, args.M, accum, copies)
    ms, gemm_ms = main_wl.run(args.steps, args.warmup)
    cfg = main_wl.cfg
    value = main_wl.flops / (ms * 1e-3) / 1e12
    if decode:
        gemm_ms = main_wl.gemm_graph_ms()
        gbs = main_wl.bytes / (gemm_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4),
                    "traffic": measured_traffic(f"{args.workload} M={args.M} {args.accum}"),
                    "kernel": "k_gemm_decode" if args.M <= 16 else "k_gemm_tile", "kernel_ms": round(gemm_ms, 5),
                    "weight_copies_rotated": copies}
    else:
        gemm_tflops = main_wl.flops / (gemm_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(gemm_tflops, 3), "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(gemm_tflops / PEAK_FP8_TFLOPS, 4),
                    "traffic": measured_traffic(f"{args.workload} M={args.M} {args.accum}"),
                    "traffic_source": "profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                      "calibrated on a 1 GiB copy; a stored figure, not counted in this run",
                    "kernel": "k_gemm_tile", "kernel_ms": round(gemm_ms, 5),
                    "kernel_ms_median": round(main_wl.kernel_ms_median, 5), "kernel_ms_min": round(main_wl.kernel_ms_min, 5)}
        if args.accum == "exact":
            # every activation tile is fed to the matrix cores twice (two exponent bands): twice the instructions
            # for the algorithmic FLOPs counted here, so this mode cannot pass half the peak
            roofline["ceiling_frac"] = 0.5
            roofline["matrix_flops_executed_frac"] = round(2 * gemm_tflops / PEAK_FP8_TFLOPS, 4)
    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "settle_ms": int(SETTLE_S * 1e3), "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3 x fp4_e2m1 -> f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload} M={args.M} K={cfg.K} N={cfg.N} G={cfg.G} "
                               f"{'M1' if cfg.mode == 1 else 'M2'} rank={cfg.rank}",
                   "accum": args.accum, "step": "quantize_act_fp8 + w4a8_gemm" + ("_lorc" if cfg.rank else "")},
        "roofline": roofline,
    }
    del main_wl
    torch.cuda.empty_cache()

    if not args.no_also:
        also = []
        plan = [
            ("llama7b_qkv", 4096, zqfp.ACCUM_FAST, 1),
            ("llama7b_qkv", 4096, accum, 1, torch.bfloat16),
            ("llama7b_qkv", 4096, accum, 1, torch.float32, True),   # W8A8: E4M3 weights
            ("llama7b_qkv", 16, accum, 12, torch.float32, True),
            ("llama7b_ffn_up", 4096, accum, 1),
            ("llama13b_ffn_lorc", 2048, accum, 1),
            ("opt1p3b_fc1", 2048, accum, 1),
            ("llama7b_qkv", 256, accum, 1),
            ("llama7b_qkv", 16, accum, 24),
            ("llama7b_qkv", 1, accum, 24),
            ("llama13b_ffn_lorc", 16, accum, 9),
            ("llama70b_ffn_decode", 64, accum, 5),
            ("llama70b_ffn_decode", 16, accum, 5),
            ("llama70b_ffn_decode", 4, accum, 5),
            ("llama70b_ffn_decode", 1, accum, 5),
            ("llama7b_ffn_down", 4096, accum, 1),
            ("llama7b_attn_out", 4096, accum, 1),
            ("llama70b_ffn_down", 16, accum, 5),
        ]
        for name, M, acc, copies, *odt in plan:
            wl = Workload(name, M, acc, copies, *odt)
            also.append(wl.summary(max(10, args.steps), args.warmup))
            del wl
            torch.cuda.empty_cache()
        out["also"] = also
        fast = [r for r in also if r["w"] == f"{args.workload} M={args.M}" and r["acc"] == "fast" and "out" not in r and "weights" not in r]
        if fast and out["roofline"]["bound"] == "mfma":  # the one-pass mode beside the headline: outside the parity tolerance
            out["roofline"]["frac_fast_mode_outside_tolerance"] = fast[0]["f_mfma"]

    if not args.no_also:
        out["quantizer"] = quantizer_rows()
        out["offline"] = offline_rows()
        ceil = measured_ceilings()
        rf = out["roofline"]
        ceil["frac_of_measured"] = round(rf["achieved"] / (ceil["stream_read_gbs"] if rf["bound"] == "hbm" else ceil["mfma_fp8xfp4_tflops"]), 4)
        out["measured_ceilings"] = ceil
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(args.workload, args.M)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
