#!/usr/bin/env python3
"""Benchmark of the W4A4 WUSH layer forward on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
wush_quantize_act (fused transform + MXFP4 quantization of the activations)
followed by wush_linear (MXFP4 GEMM) against weights prepared once, offline,
by wush_prepare_weight.  Inputs are resident in HBM before the timed region.

The default workload is c5, the largest layer (Llama-70B gate+up, 8192 tokens), on which the
GEMM's roofline target is stated; the same line also carries the transform+quantize kernel
on c4 (16384 x 4096 activations, on which its HBM target is stated), once with its working
set resident in the last-level cache and once from HBM (rotating buffer sets).

Prints ONE JSON line:
  value      layer TFLOP/s = 2*M*N*K / (time of one step)
  roofline   the dominant kernel (the GEMM; for the activation-only workload
             the transform+quantize kernel) against the MI355X peak, with its
             average launch duration measured by HIP events on the launch stream
  kernels    per-kernel durations; wush_quantize_act_c4 = {warm, cold} with frac_hbm each and
             the streaming ceilings of this machine for the same byte mix
  cpu_baseline  the CPU oracle's layer forward timed on this machine's host cores
  ceilings   measured on the spot: the GEMM's MFMA instruction alone on all CUs (with the
             workload's own operand bits, and with all-equal operands), the shader clock
             under each, and a plain 1 GiB device copy

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c5|d2|d5|dn2|dn5|di2|di5|n2|n5|i2|i5]

The decode workloads d2/d5 time wush_layer_decode (16 tokens) by replaying a
captured graph of the steps, so that the host's launch cost is not what is
measured; their roofline is HBM (the weights are streamed once per step).
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

import wush_inputs as I  # noqa: E402

PEAK_FP4_TFLOPS = 10100.0   # MI355X dense MXFP4 MFMA
PEAK_F16_TFLOPS = 2500.0    # MI355X dense FP16 / BF16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM traffic per launch of the dominant kernel: (KiB read, KiB written) from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this script, scaled by a plain copy of known size (commands, raw counters and factors:
# profiles/*.md).  A figure belongs to one kernel build: the key holds the library version it was read on,
# and a workload without a figure for the loaded library reports null.
MEASURED_TRAFFIC_KIB = {
    ("c5", "tiled", "0.10"): (2960462, 918738),   # gemm_frag_kernel<false,8,2>: profiles/wush_linear_gemm_frag_c5.md
    ("c2", "tiled", "0.10"): (43802, 27203),      # gemm_frag_kernel<false,4,3>: profiles/wush_linear_gemm_frag_c2.md
    ("c4", "tiled", "0.10"): (134410, 34816),     # transform_quant_kernel, four rotating buffer sets: profiles/transform_quant_c4.md
    ("d5", "tiled", "0.10"): (245616, 1794),      # gemm_skinny_kernel<1,false>: profiles/layer_decode_d2_d5.md
    ("dn5", "tiled", "0.10"): (261307, 1793),     # w4_skinny_kernel<1,2,nvfp4,false>: profiles/w4_skinny_dn5_di5.md
}


def traffic_for(workload, layout, version):
    t = MEASURED_TRAFFIC_KIB.get((workload, layout, version))
    return None if t is None else (t[0] + t[1]) * 1024


WORKLOADS = {
    "c2": "Llama-3.1-8B fused QKV projection, M=2048 K=4096 N=6144, MXFP4 W4A4, 128 WUSH blocks",
    "c3": "Llama-3.1-8B MLP down projection, M=4096 K=14336 N=4096, MXFP4 W4A4, 448 WUSH blocks",
    "c4": "activation path only (wush_quantize_act), M=16384 K=4096",
    "c5": "Llama-70B MLP gate+up projection, M=8192 K=8192 N=57344, MXFP4 W4A4, 256 WUSH blocks",
    "d2": "decode-sized batch on the c2 layer (wush_layer_decode), M=16 K=4096 N=6144",
    "d5": "decode-sized batch on the c5 layer (wush_layer_decode), M=16 K=8192 N=57344",
}
WORKLOADS["n2"] = "the c2 layer in the NVFP4 variant (E4M3 scale per 16, 16 x 16 transforms), M=2048 K=4096 N=6144"
WORKLOADS["n5"] = "the c5 layer in the NVFP4 variant, M=8192 K=8192 N=57344"
WORKLOADS["i2"] = "the c2 layer in the INT4 variant (BF16 scale per 32, Gaussian-MSE step), M=2048 K=4096 N=6144"
WORKLOADS["i5"] = "the c5 layer in the INT4 variant, M=8192 K=8192 N=57344"
WORKLOADS["dn2"] = "decode-sized batch on the c2 layer in the NVFP4 variant, M=16 K=4096 N=6144"
WORKLOADS["dn5"] = "decode-sized batch on the c5 layer in the NVFP4 variant, M=16 K=8192 N=57344"
WORKLOADS["di2"] = "decode-sized batch on the c2 layer in the INT4 variant, M=16 K=4096 N=6144"
WORKLOADS["di5"] = "decode-sized batch on the c5 layer in the INT4 variant, M=16 K=8192 N=57344"
W4_DECODE = {"dn2": ("nvfp4", "c2"), "dn5": ("nvfp4", "c5"), "di2": ("int4", "c2"), "di5": ("int4", "c5")}
NVFP4 = {"n2": "c2", "n5": "c5"}
INT4 = {"i2": "c2", "i5": "c5"}
DECODE = {"d2": "c2", "d5": "c5"}
DECODE_TOKENS = 16


def quant_bytes(M, K):
    """Algorithmic HBM bytes of transform+quantize: 2 B read + 0.5 B codes +
    1/32 B scale per element, plus the transforms once."""
    return M * K * (2 + 0.5 + 1 / 32) + (K // 32) * 2048


def cpu_baseline(cfg, T_bits, L, budget_rows):
    """The oracle's forward (FP64 transform, quantize, dequantize, FP64 GEMM) on
    a slab of the workload's tokens; weights pre-quantized outside the timing,
    as on the GPU."""
    from oracle import wush_oracle as O
    T = O.bf16_bits_to_f64(T_bits)
    rows = min(cfg.M, budget_rows)
    X = O.bf16_bits_to_f64(L["X"][:rows])
    cores = len(os.sched_getaffinity(0))
    n_out = min(cfg.N, 32768)   # c5: 12-13 s of oracle time on 16 cores
    if cfg.N:
        W = O.bf16_bits_to_f64(L["W"][:n_out])
        wc, ws = O.quantize_mxfp4(O.transform_weight(W, T))
        del W
    t0 = time.perf_counter()
    xc, xs = O.quantize_mxfp4(O.transform_act(X, T))
    if cfg.N:
        O.linear_dequant(xc, xs, wc, ws)
    dt = time.perf_counter() - t0
    if cfg.N:
        return {"value": 2.0 * rows * n_out * cfg.K / dt / 1e12, "unit": "TFLOP/s", "cores": cores,
                "kind": "oracle", "seconds": dt,
                "sample": f"oracle layer forward on the first {rows} of {cfg.M} tokens and the first {n_out} of "
                          f"{cfg.N} output channels, full K, weights pre-quantized"}
    return {"value": quant_bytes(rows, cfg.K) / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "seconds": dt, "sample": f"oracle transform+quantize on the first {rows} of {cfg.M} tokens"}


def measured_ceilings(torch, dev, x_bits, w_bits):
    """What this machine sustains, measured now: the GEMM's MFMA instruction in a register-only loop on all
    CUs (the probes library) with the workload's own operand bits and with all-equal operands, the shader
    clock during each, and a plain 1 GiB device copy."""
    from paper_2512_00956_amd import probes
    props = torch.cuda.get_device_properties(dev)
    cus = props.multi_processor_count
    out = {"compute_units": cus}
    ticks = torch.zeros((cus, 2), dtype=torch.int64, device=dev)
    iters = 2000
    flop_per_wg = 4.0 * iters * 64 * 2 * 32 * 32 * 64
    real = torch.cat([x_bits[:8192], w_bits[:8192]]).contiguous()
    equal = torch.full((16384,), 0x22, dtype=torch.uint8, device=dev)
    for name, bits in (("workload_bits", real), ("equal_operands", equal)):
        for _ in range(2):
            probes.mfma_fp4(bits, iters, cus, ticks)
        torch.cuda.synchronize()
        t = ticks.cpu().numpy().astype(np.float64)
        ns = t[:, 1].mean() * 10.0
        out[f"mfma_only_{name}_tflops"] = cus * flop_per_wg / ns / 1e3
        out[f"sclk_ghz_{name}"] = float((t[:, 0] / (t[:, 1] * 10.0)).mean())
        out[f"cycles_per_mfma_{name}"] = float(t[:, 0].mean() / (iters * 64))
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    out["copy_1gib_gbs"] = 5 * 2.0 * (1 << 30) / e0.elapsed_time(e1) / 1e6
    del src, dst
    return out


COLD_WEIGHT_SETS = 4


def cold_weights_ms(torch, replay_ms, weights, launch, steps):
    """The few-token GEMM with the packed weights rotating over COLD_WEIGHT_SETS copies, so that every step streams
    them from HBM (one copy of the c5 weights is about the size of the 256 MB last-level cache and is partly served
    from it when the same buffers are read step after step).  Returns ms per launch, or None if the copies do not
    fit (they do on this part: 4 x 240 MiB)."""
    sets = [weights] + [[w.clone() for w in weights] for _ in range(COLD_WEIGHT_SETS - 1)]
    state = {"i": 0}

    def fn():
        launch(sets[state["i"] % COLD_WEIGHT_SETS])
        state["i"] += 1

    calls = max(COLD_WEIGHT_SETS, steps - steps % COLD_WEIGHT_SETS)
    ms = replay_ms(fn, calls)
    del sets
    return ms


def read_stream_cold_gbs(torch, dev, nbytes):
    """What a read-only linear stream of about nbytes reaches from HBM on this machine, now (probes library: the xor of
    everything read, one small store per wave), over COLD_WEIGHT_SETS rotating buffers."""
    from paper_2512_00956_amd import probes
    n = max(1 << 22, nbytes // (1 << 22) * (1 << 22))
    srcs = [torch.empty(n, dtype=torch.uint8, device=dev).fill_(i + 1) for i in range(COLD_WEIGHT_SETS)]
    dst = torch.empty(256 * 8 * 1024, dtype=torch.uint8, device=dev)
    ms = events_ms(torch, lambda i: probes.stream(srcs[i % COLD_WEIGHT_SETS], n // 4096, 4096, dst, 50, 256), 24, warm=8)
    return n / ms / 1e6


def cold_entry(ms, gemm_bytes):
    return {"ms": ms, "GB/s": gemm_bytes / ms / 1e6, "frac_hbm": gemm_bytes / ms / 1e6 / PEAK_HBM_GBS,
            "weight_sets": COLD_WEIGHT_SETS}


def decode_bench(args, P, torch, dev):
    """d2 / d5: one step = one wush_layer_decode call on M = 16 tokens."""
    base = DECODE[args.workload]
    cfg = I.scaled(I.CONFIGS[base], M=DECODE_TOKENS)
    L = I.make_layer(I.CONFIGS[base])
    M, K, N = cfg.M, cfg.K, cfg.N

    def bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    Td = torch.empty((K // 32, 32, 32), dtype=torch.bfloat16, device=dev)
    bws = torch.empty(P.wush_build_transforms_workspace(K), dtype=torch.uint8, device=dev)
    Wd = bf16(L["W"])
    P.wush_build_transforms(Wd, bf16(L["X_cal"]), 1e-2, Td, bws)
    P.wush_build_transforms_status(bws, K)
    T_bits = Td.view(torch.int16).cpu().numpy().view(np.uint16)
    fmt = P.default_fmt(layout=1)
    wcb, wsb = P.wush_packed_sizes(N, K, fmt)
    Wq = torch.empty(wcb, dtype=torch.uint8, device=dev)
    Ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    wsp = torch.empty(P.wush_prepare_weight_workspace(N, K), dtype=torch.uint8, device=dev)
    P.wush_prepare_weight(Wd, Td, Wq, Ws, wsp, fmt)
    P.wush_workspace_status(wsp, K)
    del Wd, wsp, bws
    Xd = bf16(L["X"][:M])
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    dws = torch.empty(P.wush_layer_decode_workspace(K), dtype=torch.uint8, device=dev)
    P.wush_layer_decode_init(dws, K)
    KT = K // 256
    Xq, Xs = dws[:KT * 8192], dws[KT * 8192:KT * 8192 + KT * 512]   # where the call keeps the quantized activations

    def replay_ms(fn, calls):
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            for _ in range(max(3, args.warmup)):
                fn()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                for _ in range(calls):
                    fn()
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            g.replay()
            e1.record(st)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) / calls

    ms_per_step = replay_ms(lambda: P.wush_layer_decode(Xd, Td, Wq, Ws, Y, dws, fmt), args.steps)
    P.wush_layer_decode_status(dws, K)
    g_ms = replay_ms(lambda: P.wush_linear(Xq, Xs, Wq, Ws, Y, fmt, K=K), args.steps)
    gemm_bytes = N * K * (0.5 + 1 / 32) + M * K * (0.5 + 1 / 32) + M * N * 2
    cold = cold_weights_ms(torch, replay_ms, [Wq, Ws], lambda w: P.wush_linear(Xq, Xs, w[0], w[1], Y, fmt, K=K), args.steps)
    traffic = traffic_for(args.workload, "tiled", P.lib().wush_version().decode())
    layer_bytes = N * K * (0.5 + 1 / 32) + quant_bytes(M, K) + M * K * (0.5 + 1 / 32) + M * N * 2
    flops = 2.0 * M * N * K
    out = {
        "metric": "W4A4 layer TFLOP/s (transform+quant+MXFP4 GEMM); % of MXFP4 MFMA & HBM peak",
        "value": flops / ms_per_step / 1e9, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4 (e2m1 x e8m0), bf16 in/out, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}", **({"debug_set": args.debug_set} if args.debug_set else {}), "M": M, "K": K, "N": N,
                   "launch": "graph replay of the timed steps", "packed_layout": "tiled"},
        "roofline": {"bound": "hbm", "kernel": "wush_linear for M <= 64 (weight-streaming MXFP4 GEMM)",
                     "achieved": gemm_bytes / g_ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gemm_bytes / g_ms / 1e6 / PEAK_HBM_GBS, "traffic": traffic,
                     "algorithmic_bytes": gemm_bytes,
                     "traffic_over_algorithmic": None if traffic is None else traffic / gemm_bytes, "avg_launch_ms": g_ms},
        "kernels": {"wush_layer_decode": {"ms": ms_per_step, "GB/s": layer_bytes / ms_per_step / 1e6,
                                          "algorithmic_bytes": layer_bytes},
                    "wush_linear": {"ms": g_ms, "GB/s": gemm_bytes / g_ms / 1e6, "algorithmic_bytes": gemm_bytes},
                    "wush_linear_cold_weights": cold_entry(cold, gemm_bytes)},
        "read_only_stream_cold_GB/s": read_stream_cold_gbs(torch, dev, int(N * K * (0.5 + 1 / 32))),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, T_bits, L, M)
    print(json.dumps(out))


def w4_decode_bench(args, P, torch, dev):
    """dn2 / dn5 / di2 / di5: one step = activation quantizer + weight-streaming GEMM of the NVFP4 or INT4
    variant on 16 tokens (tiled layout), timed by replaying a captured graph of the steps.  Roofline: the
    GEMM against HBM (the packed weights are read once per step)."""
    fmt_name, base = W4_DECODE[args.workload]
    cfg = I.scaled(I.CONFIGS[base], M=DECODE_TOKENS)
    L = I.make_layer(I.CONFIGS[base])
    M, K, N = cfg.M, cfg.K, cfg.N
    nv = fmt_name == "nvfp4"

    def bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    d = 16 if nv else 32
    Td = torch.empty((K // d, d, d), dtype=torch.bfloat16, device=dev)
    bws = torch.empty(P.wush_build_transforms_workspace(K), dtype=torch.uint8, device=dev)
    Wd = bf16(L["W"])
    (P.wush_build_transforms_nvfp4 if nv else P.wush_build_transforms)(Wd, bf16(L["X_cal"]), 1e-2, Td, bws)
    P.wush_build_transforms_status(bws, K)
    Xd = bf16(L["X"][:M])
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, 1), P.wush_packed_sizes_nvfp4(N, K, 1)
    Xq, Xs = (torch.empty(n, dtype=torch.uint8, device=dev) for n in (xcb, xsb))
    Wq, Ws = (torch.empty(n, dtype=torch.uint8, device=dev) for n in (wcb, wsb))
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    if nv:
        tsx, tsw = (torch.zeros(1, dtype=torch.float32, device=dev) for _ in range(2))
        P.wush_calibrate_act_nvfp4(Xd, Td, tsx)
        wsp = torch.empty(P.wush_prepare_weight_nvfp4_workspace(K), dtype=torch.uint8, device=dev)
        P.wush_prepare_weight_nvfp4(Wd, Td, Wq, Ws, tsw, wsp, layout=1)
        P.wush_prepare_weight_nvfp4_status(wsp, K)
        quant = lambda: P.wush_quantize_act_nvfp4(Xd, Td, tsx, Xq, Xs, layout=1)
        gemm = lambda: P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, layout=1, K=K)
    else:
        wsp = torch.empty(P.wush_prepare_weight_workspace(N, K), dtype=torch.uint8, device=dev)
        P.wush_prepare_weight_int4(Wd, Td, Wq, Ws, wsp, layout=1)
        P.wush_workspace_status(wsp, K)
        quant = lambda: P.wush_quantize_act_int4(Xd, Td, Xq, Xs, layout=1)
        gemm = lambda: P.wush_linear_int4(Xq, Xs, Wq, Ws, Y, layout=1, K=K)
    del Wd, wsp, bws

    def replay_ms(fn, calls):
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            for _ in range(max(3, args.warmup)):
                fn()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                for _ in range(calls):
                    fn()
            g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            g.replay()
            e1.record(st)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) / calls

    def step():
        quant()
        gemm()
    ms_per_step = replay_ms(step, args.steps)
    g_ms = replay_ms(gemm, args.steps)
    gemm_bytes = (N + M) * K * (0.5 + 1 / 16) + M * N * 2
    flops = 2.0 * M * N * K
    traffic = traffic_for(args.workload, "tiled", P.lib().wush_version().decode())
    if nv:
        cold = cold_weights_ms(torch, replay_ms, [Wq, Ws],
                               lambda w: P.wush_linear_nvfp4(Xq, Xs, tsx, w[0], w[1], tsw, Y, layout=1, K=K), args.steps)
    else:
        cold = cold_weights_ms(torch, replay_ms, [Wq, Ws],
                               lambda w: P.wush_linear_int4(Xq, Xs, w[0], w[1], Y, layout=1, K=K), args.steps)
    name = "wush_linear_nvfp4" if nv else "wush_linear_int4"
    out = {
        "metric": f"W4A4 layer TFLOP/s (transform+quant+{fmt_name.upper()} GEMM); % of HBM peak",
        "value": flops / ms_per_step / 1e9, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("nvfp4 (e2m1 x e4m3 per 16 x f32 per tensor)" if nv else "int4 (two's complement x bf16 per 32)") +
                 ", bf16 in/out, f16 MFMA operands, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}", **({"debug_set": args.debug_set} if args.debug_set else {}), "M": M, "K": K, "N": N,
                   "launch": "graph replay of the timed steps", "packed_layout": "tiled"},
        "roofline": {"bound": "hbm", "kernel": f"{name} for M <= 128 (weight-streaming, dequantize in registers)",
                     "achieved": gemm_bytes / g_ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gemm_bytes / g_ms / 1e6 / PEAK_HBM_GBS, "traffic": traffic, "algorithmic_bytes": gemm_bytes,
                     "traffic_over_algorithmic": None if traffic is None else traffic / gemm_bytes,
                     "avg_launch_ms": g_ms},
        "kernels": {name: {"ms": g_ms, "GB/s": gemm_bytes / g_ms / 1e6},
                    name + "_cold_weights": cold_entry(cold, gemm_bytes)},
        "read_only_stream_cold_GB/s": read_stream_cold_gbs(torch, dev, int(N * K * (0.5 + 1 / 16))),
    }
    print(json.dumps(out))


def nvfp4_bench(args, P, torch, dev):
    """The layer forward in the NVFP4 variant: wush_quantize_act_nvfp4 + wush_linear_nvfp4 per step.
    CDNA4 has no scaled-MFMA path for E4M3-per-16 scales; the GEMM dequantizes (exactly) to FP16 and is
    priced against the FP16 MFMA peak."""
    cfg = I.CONFIGS[NVFP4[args.workload]]
    L = I.make_layer(cfg)
    M, K, N = cfg.M, cfg.K, cfg.N

    def bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    # The 16 x 16 transforms come from the library's own offline path (Alg. 1 on the device with d = 16)
    # applied to the workload's weights and calibration tokens.
    Td = torch.empty((K // 16, 16, 16), dtype=torch.bfloat16, device=dev)
    bws = torch.empty(P.wush_build_transforms_workspace(K), dtype=torch.uint8, device=dev)
    P.wush_build_transforms_nvfp4(bf16(L["W"]), bf16(L["X_cal"]), 1e-2, Td, bws)
    P.wush_build_transforms_status(bws, K)
    del bws
    T_bits = Td.view(torch.int16).cpu().numpy().view(np.uint16)
    Xd = bf16(L["X"])
    # The activation tensor scale is an input of the quantizer (a calibrated constant), taken here from
    # the batch itself, once, outside the timed steps.
    tsx = torch.zeros(1, dtype=torch.float32, device=dev)
    P.wush_calibrate_act_nvfp4(Xd, Td, tsx)
    lay = 1 if args.layout == "tiled" else 0
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, lay), P.wush_packed_sizes_nvfp4(N, K, lay)
    Xq = torch.empty(xcb, dtype=torch.uint8, device=dev)
    Xs = torch.empty(xsb, dtype=torch.uint8, device=dev)
    Wq = torch.empty(wcb, dtype=torch.uint8, device=dev)
    Ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    tsw = torch.zeros(1, dtype=torch.float32, device=dev)
    wsp = torch.empty(P.wush_prepare_weight_nvfp4_workspace(K), dtype=torch.uint8, device=dev)
    Wd = bf16(L["W"])
    P.wush_prepare_weight_nvfp4(Wd, Td, Wq, Ws, tsw, wsp, layout=lay)
    P.wush_prepare_weight_nvfp4_status(wsp, K)
    del Wd
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)

    def quant(i):
        P.wush_quantize_act_nvfp4(Xd, Td, tsx, Xq, Xs, layout=lay)

    def gemm(i):
        P.wush_linear_nvfp4(Xq, Xs, tsx, Wq, Ws, tsw, Y, layout=lay, K=K)

    def step(i):
        quant(i)
        gemm(i)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    def kernel_ms(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    q_ms, g_ms = kernel_ms(quant), kernel_ms(gemm)
    qb = M * K * (2 + 0.5 + 1 / 16) + (K // 16) * 512
    flops = 2.0 * M * N * K
    out = {
        "metric": "W4A4 layer TFLOP/s (transform+quant+NVFP4 GEMM); % of FP16 MFMA peak",
        "value": flops / ms_per_step / 1e9, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "nvfp4 (e2m1 x e4m3 per 16 x f32 per tensor), bf16 in/out, f16 MFMA operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}", **({"debug_set": args.debug_set} if args.debug_set else {}), "M": M, "K": K, "N": N,
                   "packed_layout": args.layout, "launch": "host loop"},
        "roofline": {"bound": "mfma", "kernel": "wush_linear_nvfp4 (dequantize to FP16: X through LDS, W in registers; FP16 MFMA)",
                     "achieved": flops / g_ms / 1e9, "peak": PEAK_F16_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / g_ms / 1e9 / PEAK_F16_TFLOPS, "traffic": None, "avg_launch_ms": g_ms},
        "kernels": {"wush_quantize_act_nvfp4": {"ms": q_ms, "GB/s": qb / q_ms / 1e6,
                                                "frac_hbm": qb / q_ms / 1e6 / PEAK_HBM_GBS, "algorithmic_bytes": qb},
                    "wush_linear_nvfp4": {"ms": g_ms, "TFLOP/s": flops / g_ms / 1e9}},
    }
    if not args.no_ceilings:
        # What this machine sustains now: the GEMM's FP16 MFMA in a register-only loop on all CUs, fed with the
        # FP16 images of the workload's own packed operands (first 4096 elements of X and of W) and with
        # all-equal operands; the shader clock during each.
        def f16_image(q, s, rows):
            qc = torch.empty((rows, K // 2), dtype=torch.uint8, device=dev)
            sc = torch.empty((rows, K // 16), dtype=torch.uint8, device=dev)
            if lay:
                P.wush_unpack_tiled_nvfp4(q, s, rows, K, qc, sc)
            else:
                qc, sc = q.view(rows, K // 2), s.view(rows, K // 16)
            b = qc[0, :2048].to(torch.int64)
            codes = torch.stack([b & 15, b >> 4], dim=1).reshape(-1)
            grid = torch.tensor([0, .5, 1, 1.5, 2, 3, 4, 6], device=dev)
            val = grid[codes & 7] * (1.0 - 2.0 * (codes >> 3).float())
            sv = sc[0, :256].view(torch.float8_e4m3fn).float().repeat_interleave(16)
            return (val * sv).half()
        from paper_2512_00956_amd import probes
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        ticks = torch.zeros((cus, 2), dtype=torch.int64, device=dev)
        iters = 4000
        flop_per_wg = 4.0 * iters * 64 * 2 * 32 * 32 * 16
        real = torch.cat([f16_image(Xq, Xs, M), f16_image(Wq, Ws, N)]).contiguous()
        equal = torch.ones(8192, dtype=torch.float16, device=dev)
        ceil = {"compute_units": cus}
        for name, bits in (("workload_bits", real), ("equal_operands", equal)):
            for _ in range(2):
                probes.mfma_f16(bits, iters, cus, ticks)
            torch.cuda.synchronize()
            t = ticks.cpu().numpy().astype(np.float64)
            ns = t[:, 1].mean() * 10.0
            ceil[f"mfma_f16_only_{name}_tflops"] = cus * flop_per_wg / ns / 1e3
            ceil[f"sclk_ghz_{name}"] = float((t[:, 0] / (t[:, 1] * 10.0)).mean())
            ceil[f"cycles_per_mfma_{name}"] = float(t[:, 0].mean() / (iters * 64))
        out["ceilings"] = ceil
        out["roofline"]["frac_of_measured_mfma_ceiling"] = out["roofline"]["achieved"] / ceil["mfma_f16_only_workload_bits_tflops"]
    if not args.no_cpu_baseline:
        from oracle import wush_nvfp4_oracle as NV
        from oracle import wush_oracle as O
        rows, n_out = min(M, {"n2": 1024, "n5": 64}[args.workload]), min(N, 8192)
        T = O.bf16_bits_to_f64(T_bits)
        wc, wsb, tw = NV.prepare_weight(O.bf16_bits_to_f64(L["W"][:n_out]), T)
        X = O.bf16_bits_to_f64(L["X"][:rows])
        ts_host = float(tsx.cpu()[0])
        t0 = time.perf_counter()
        xc, xsb = NV.quantize_nvfp4(NV.transform_act(X, T), ts_host)
        NV.linear_dequant(xc, xsb, ts_host, wc, wsb, tw)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * n_out * K / dt / 1e12, "unit": "TFLOP/s",
                               "cores": len(os.sched_getaffinity(0)), "kind": "oracle", "seconds": dt,
                               "sample": f"NVFP4 oracle layer forward on the first {rows} of {M} tokens and the first "
                                         f"{n_out} of {N} output channels, full K, weights pre-quantized"}
    print(json.dumps(out))


def int4_bench(args, P, torch, dev):
    """The layer forward in the INT4 variant: wush_quantize_act_int4 + wush_linear_int4 per step; the GEMM is the
    NVFP4 one with another dequantization and is priced against the FP16 MFMA peak."""
    cfg = I.CONFIGS[INT4[args.workload]]
    L = I.make_layer(cfg)
    M, K, N = cfg.M, cfg.K, cfg.N

    def bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    Td = torch.empty((K // 32, 32, 32), dtype=torch.bfloat16, device=dev)
    bws = torch.empty(P.wush_build_transforms_workspace(K), dtype=torch.uint8, device=dev)
    Wd = bf16(L["W"])
    P.wush_build_transforms(Wd, bf16(L["X_cal"]), 1e-2, Td, bws)
    P.wush_build_transforms_status(bws, K)
    del bws
    T_bits = Td.view(torch.int16).cpu().numpy().view(np.uint16)
    Xd = bf16(L["X"])
    lay = 1 if args.layout == "tiled" else 0
    (xcb, xsb), (wcb, wsb) = P.wush_packed_sizes_nvfp4(M, K, lay), P.wush_packed_sizes_nvfp4(N, K, lay)
    Xq = torch.empty(xcb, dtype=torch.uint8, device=dev)
    Xs = torch.empty(xsb, dtype=torch.uint8, device=dev)
    Wq = torch.empty(wcb, dtype=torch.uint8, device=dev)
    Ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
    wsp = torch.empty(P.wush_prepare_weight_workspace(N, K), dtype=torch.uint8, device=dev)
    P.wush_prepare_weight_int4(Wd, Td, Wq, Ws, wsp, layout=lay)
    P.wush_workspace_status(wsp, K)
    del Wd
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)

    def quant(i):
        P.wush_quantize_act_int4(Xd, Td, Xq, Xs, layout=lay)

    def gemm(i):
        P.wush_linear_int4(Xq, Xs, Wq, Ws, Y, layout=lay, K=K)

    def step(i):
        quant(i)
        gemm(i)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    def kernel_ms(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    q_ms, g_ms = kernel_ms(quant), kernel_ms(gemm)
    qb = M * K * (2 + 0.5 + 1 / 16) + (K // 32) * 2048
    flops = 2.0 * M * N * K
    out = {
        "metric": "W4A4 layer TFLOP/s (transform+quant+INT4 GEMM); % of FP16 MFMA peak",
        "value": flops / ms_per_step / 1e9, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int4 (two's complement x bf16 per 32), bf16 in/out, f16 MFMA operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}", **({"debug_set": args.debug_set} if args.debug_set else {}), "M": M, "K": K, "N": N,
                   "packed_layout": args.layout, "launch": "host loop"},
        "roofline": {"bound": "mfma", "kernel": "wush_linear_int4 (dequantize to FP16: X through LDS, W in registers; FP16 MFMA)",
                     "achieved": flops / g_ms / 1e9, "peak": PEAK_F16_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / g_ms / 1e9 / PEAK_F16_TFLOPS, "traffic": None, "avg_launch_ms": g_ms},
        "kernels": {"wush_quantize_act_int4": {"ms": q_ms, "GB/s": qb / q_ms / 1e6,
                                               "frac_hbm": qb / q_ms / 1e6 / PEAK_HBM_GBS, "algorithmic_bytes": qb},
                    "wush_linear_int4": {"ms": g_ms, "TFLOP/s": flops / g_ms / 1e9}},
    }
    if not args.no_cpu_baseline:
        from oracle import wush_int4_oracle as Q4
        from oracle import wush_oracle as O
        rows, n_out = min(M, {"i2": 1024, "i5": 64}[args.workload]), min(N, 8192)
        T = O.bf16_bits_to_f64(T_bits)
        wq, wsb_ = Q4.quantize_int4(O.transform_weight(O.bf16_bits_to_f64(L["W"][:n_out]), T))
        X = O.bf16_bits_to_f64(L["X"][:rows])
        t0 = time.perf_counter()
        xq, xsb_ = Q4.quantize_int4(O.transform_act(X, T))
        Q4.linear_dequant(xq, xsb_, wq, wsb_)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * rows * n_out * K / dt / 1e12, "unit": "TFLOP/s",
                               "cores": len(os.sched_getaffinity(0)), "kind": "oracle", "seconds": dt,
                               "sample": f"INT4 oracle layer forward on the first {rows} of {M} tokens and the first "
                                         f"{n_out} of {N} output channels, full K, weights pre-quantized"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=15)   # the c5 GEMM settles after about a dozen launches (power management)
    ap.add_argument("--workload", default="c5", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layout", default="tiled", choices=["tiled", "canonical"],
                    help="layout of the packed codes/scales between the kernels")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (torch) so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured graph of the timed steps instead of launching every step from the host")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the live measurement of the MFMA-only and copy ceilings of this box")
    ap.add_argument("--no-c4", action="store_true",
                    help="workload c5 only: skip the transform+quantize measurement on the c4 activations")
    ap.add_argument("--cold", type=int, default=0,
                    help="rotate over this many input/output buffer sets (>1 defeats the 256 MB last-level cache)")
    ap.add_argument("--debug-set", action="append", default=[], metavar="OPTION=VALUE",
                    help="measurement switch of the library (wush_debug_set), e.g. DECODE_FUSED=1 or GEMM_TILE=0; "
                         "never part of a benchmark line that is reported as the library's own choice")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2512_00956_amd as P
    P.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    for item in args.debug_set:
        name, _, value = item.partition("=")
        P.wush_debug_set(getattr(P, "WUSH_DEBUG_" + name.upper()), int(value))
    if args.workload in DECODE:
        decode_bench(args, P, torch, dev)
        return
    if args.workload in W4_DECODE:
        w4_decode_bench(args, P, torch, dev)
        return
    if args.workload in NVFP4:
        nvfp4_bench(args, P, torch, dev)
        return
    if args.workload in INT4:
        int4_bench(args, P, torch, dev)
        return

    out = layer_bench(args, P, torch, dev)
    print(json.dumps(out))


def events_ms(torch, fn, steps, warm=3):
    """Average duration of fn(i) over `steps` back-to-back launches, HIP events on the launch stream."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def build_transforms_on_device(P, torch, dev, L, K):
    """T_blocks from the library's own offline path (Alg. 1 on the device) applied to the workload's
    weights and calibration tokens."""
    Td = torch.empty((K // 32, 32, 32), dtype=torch.bfloat16, device=dev)
    bws = torch.empty(P.wush_build_transforms_workspace(K), dtype=torch.uint8, device=dev)
    Wcal = torch.from_numpy(L["W"].view(np.int16)).view(torch.bfloat16).to(dev)
    Xcal = torch.from_numpy(L["X_cal"].view(np.int16)).view(torch.bfloat16).to(dev)
    P.wush_build_transforms(Wcal, Xcal, 1e-2, Td, bws)
    P.wush_build_transforms_status(bws, K)
    return Td


def quantizer_c4(args, P, torch, dev, layout, cold_sets=4):
    """wush_quantize_act on the c4 activations (16384 x 4096): `warm` = one buffer set (its 162 MiB
    working set stays in the 256 MB last-level cache between launches), `cold` = `cold_sets` rotating
    buffer sets, so that every byte of a launch comes from and goes to HBM.  Beside them what plain
    streaming kernels with the same byte mix (4 : 1 read : write, non-temporal stores) reach on this
    box from HBM: linear, and in the quantizer's own access pattern without its arithmetic."""
    from paper_2512_00956_amd import probes
    cfg = I.CONFIGS["c4"]
    L = I.make_layer(cfg)
    M, K = cfg.M, cfg.K
    Td = build_transforms_on_device(P, torch, dev, L, K)
    fmt = P.default_fmt(layout=1 if layout == "tiled" else 0)
    xcb, xsb = P.wush_packed_sizes(M, K, fmt)
    X0 = torch.from_numpy(L["X"].view(np.int16)).view(torch.bfloat16).to(dev)
    Xd = [X0] + [X0.clone() for _ in range(cold_sets - 1)]
    Xq = [torch.empty(xcb, dtype=torch.uint8, device=dev) for _ in range(cold_sets)]
    Xs = [torch.empty(xsb, dtype=torch.uint8, device=dev) for _ in range(cold_sets)]
    qb = quant_bytes(M, K)
    steps = max(args.steps, 20)
    res = {"M": M, "K": K, "algorithmic_bytes": qb}
    for name, nset in (("warm", 1), ("cold", cold_sets)):
        ms = events_ms(torch, lambda i: P.wush_quantize_act(Xd[i % nset], Td, Xq[i % nset], Xs[i % nset], fmt),
                       steps, warm=2 * nset)
        res[name] = {"ms": ms, "GB/s": qb / ms / 1e6, "frac_hbm": qb / ms / 1e6 / PEAK_HBM_GBS, "buffer_sets": nset,
                     "working_set_MiB": nset * qb / 2 ** 20}
    # streaming ceilings, cold, same buffers (dst: codes then scales of one set, contiguous)
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    dst = [torch.empty(M * K * 17 // 32 + 4096, dtype=torch.uint8, device=dev) for _ in range(cold_sets)]
    sb = M * K * 2 * (1 + 17 / 64)
    ceil = {}
    for name, mode, blocks in (("linear", 0, cus), ("quantizer_pattern", 1, cus)):
        ms = events_ms(torch, lambda i: probes.stream(Xd[i % cold_sets], M, 2 * K, dst[i % cold_sets], mode, blocks),
                       steps, warm=2 * cold_sets)
        ceil[name + "_GB/s"] = (sb if mode else M * K * 2 * 1.25) / ms / 1e6
    res["same_mix_stream_cold"] = ceil
    res["cold"]["frac_of_same_mix_stream"] = res["cold"]["GB/s"] / max(ceil.values())
    t = traffic_for("c4", layout, P.lib().wush_version().decode())
    res["cold"]["traffic"] = t
    res["cold"]["traffic_over_algorithmic"] = None if t is None else t / qb
    return res


def layer_bench(args, P, torch, dev):
    cfg = I.CONFIGS[args.workload]
    L = I.make_layer(cfg)          # c4 keeps its weights: they are only used to build the transforms
    if args.workload == "c4":
        cfg = I.scaled(cfg, N=0)
    M, K, N = cfg.M, cfg.K, cfg.N
    version = P.lib().wush_version().decode()

    def bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    nset = max(1, args.cold)
    Td = build_transforms_on_device(P, torch, dev, L, K)
    T_bits = Td.view(torch.int16).cpu().numpy().view(np.uint16)
    Xd = [bf16(L["X"]) for _ in range(nset)]
    fmt = P.default_fmt(layout=1 if args.layout == "tiled" else 0)
    xcb, xsb = P.wush_packed_sizes(M, K, fmt)
    Xq = [torch.empty(xcb, dtype=torch.uint8, device=dev) for _ in range(nset)]
    Xs = [torch.empty(xsb, dtype=torch.uint8, device=dev) for _ in range(nset)]
    if N:
        Wd = bf16(L["W"])
        wcb, wsb = P.wush_packed_sizes(N, K, fmt)
        Wq = torch.empty(wcb, dtype=torch.uint8, device=dev)
        Ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
        wsp = torch.empty(P.wush_prepare_weight_workspace(N, K), dtype=torch.uint8, device=dev)
        P.wush_prepare_weight(Wd, Td, Wq, Ws, wsp, fmt)
        P.wush_workspace_status(wsp, K)
        del Wd, wsp
        Y = [torch.empty((M, N), dtype=torch.bfloat16, device=dev) for _ in range(nset)]

    def quant(i):
        P.wush_quantize_act(Xd[i % nset], Td, Xq[i % nset], Xs[i % nset], fmt)

    def gemm(i):
        P.wush_linear(Xq[i % nset], Xs[i % nset], Wq, Ws, Y[i % nset], fmt, K=K)

    def step(i):
        quant(i)
        if N:
            gemm(i)

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if not args.graph:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    else:
        # The K timed steps are captured once into a HIP graph and replayed: the same 2K kernel
        # launches, enqueued by the runtime instead of by 2K calls from Python.
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            step(0)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=st):
                for i in range(args.steps):
                    step(i)
            graph.replay()                      # untimed: first replay uploads the graph
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    q_ms = events_ms(torch, quant, args.steps)
    qb = quant_bytes(M, K)
    kernels = {"wush_quantize_act": {"ms": q_ms, "GB/s": qb / q_ms / 1e6, "frac_hbm": qb / q_ms / 1e6 / PEAK_HBM_GBS,
                                     "algorithmic_bytes": qb}}
    traffic = traffic_for(args.workload, args.layout, version)
    if N:
        g_ms = events_ms(torch, gemm, args.steps)
        flops = 2.0 * M * N * K
        gemm_bytes = (M + N) * K * (0.5 + 1 / 32) + 2.0 * M * N
        kernels["wush_linear"] = {"ms": g_ms, "TFLOP/s": flops / g_ms / 1e9,
                                  "frac_fp4_mfma": flops / g_ms / 1e9 / PEAK_FP4_TFLOPS,
                                  "algorithmic_bytes": gemm_bytes}
        value, unit = flops / ms_per_step / 1e9, "TFLOP/s"
        roof = {"bound": "mfma", "kernel": "wush_linear (MXFP4 scaled-MFMA GEMM)", "achieved": flops / g_ms / 1e9,
                "peak": PEAK_FP4_TFLOPS, "unit": "TFLOP/s", "frac": flops / g_ms / 1e9 / PEAK_FP4_TFLOPS,
                "traffic": traffic, "algorithmic_bytes": gemm_bytes,
                "traffic_over_algorithmic": None if traffic is None else traffic / gemm_bytes, "avg_launch_ms": g_ms}
        kernels["sum_of_kernel_ms"] = q_ms + g_ms
    else:
        value, unit = qb / ms_per_step / 1e6, "GB/s"
        roof = {"bound": "hbm", "kernel": "wush_quantize_act (fused transform+quantize)", "achieved": qb / q_ms / 1e6,
                "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": qb / q_ms / 1e6 / PEAK_HBM_GBS,
                "traffic": traffic, "algorithmic_bytes": qb,
                "traffic_over_algorithmic": None if traffic is None else traffic / qb, "avg_launch_ms": q_ms}

    out = {
        "metric": "W4A4 layer TFLOP/s (transform+quant+MXFP4 GEMM); % of MXFP4 MFMA & HBM peak",
        "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4 (e2m1 x e8m0), bf16 in/out, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {WORKLOADS[args.workload]}", **({"debug_set": args.debug_set} if args.debug_set else {}), "M": M, "K": K, "N": N,
                   "buffer_sets": nset, "packed_layout": args.layout, "library_version": version,
                   "launch": "graph replay of the timed steps" if args.graph else "host loop"},
        "roofline": roof, "kernels": kernels,
    }
    if not args.no_ceilings:
        ceil = measured_ceilings(torch, dev, Xq[0], Wq if N else Xq[0])
        out["ceilings"] = ceil
        if N:
            roof["frac_of_measured_mfma_ceiling"] = roof["achieved"] / ceil["mfma_only_workload_bits_tflops"]
    if not args.no_cpu_baseline:
        rows = {"c2": 2048, "c3": 4096, "c4": 16384, "c5": 8192}[args.workload]
        out["cpu_baseline"] = cpu_baseline(cfg, T_bits, L, rows)
    if args.workload == "c5" and not args.no_c4:
        # free the layer's buffers first: the activation-path measurement gets the GPU to itself
        del Xd, Xq, Xs, Y, Wq, Ws, Td, L
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        kernels["wush_quantize_act_c4"] = quantizer_c4(args, P, torch, dev, args.layout)
    return out


if __name__ == "__main__":
    main()
