#!/usr/bin/env python3
"""Benchmark of the NVFP4 W4A4 prefill linear path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic prefill batch of the headline
workload (Llama-3-8B-shaped linears at M = 8192 tokens): for each of the four layers, quantize
the BF16 activations to NVFP4 on the fly (nvfp4_quantize) and run the block-scaled GEMM against
the offline-quantized weights (nvfp4_gemm_ws, BF16 out).  Inputs are resident in HBM before the
timed region; tensor-level scales and weight quantization are computed once, untimed.

Prints ONE JSON line.  `value` = 2*M*N*K summed over the four layers / step time, in TFLOP/s.
Also measured: the dominant kernel's (NVFP4 GEMM) average launch duration with HIP events on
the launch stream (-> roofline), the quantizer's bandwidth, the in-repo BF16 GEMM on the same
shapes (-> speed-up), and the CPU oracle on a bounded sample (-> cpu_baseline).  Further lines of
the same JSON object, all outside the timed region: the vendor library's BF16 GEMM as context,
the dynamic-alpha pipeline, decode-shape weight streaming, the producer-fused quantizers and
the MLP block as a dependent chain, a tokens-per-batch sweep (64 .. 131072), and the rate an
MFMA-only loop sustains on this machine.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published dense peaks (TFLOP/s) and HBM3E bandwidth (GB/s)
PEAK_MFMA_16BIT = 2516.6
PEAK_MFMA_FP4 = 10066.3
PEAK_HBM_GBS = 8000.0
QUANT_BYTES_PER_ELT = 2.0 + 0.5 + 1.0 / 16.0   # BF16 in, 4-bit code + 1/16 scale byte out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload config id (2 = Llama-3-8B shapes, M=8192)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=4096)
    ap.add_argument("--no-sweep", action="store_true", help="skip the tokens-per-batch sweep (second workload)")
    ap.add_argument("--no-fused", action="store_true", help="skip the producer-fused quantizers and the MLP chain")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path is single-GPU by construction (no collectives are built); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2605_20315_amd as mq
    from paper_2605_20315_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    cfg = wl.configs()[args.config]
    M = cfg.M
    LAYOUT = mq.MQ_LAYOUT_KTILE     # K-step-major NVFP4 bytes: the layout the GEMM streams
    # caller-owned workspace of the NVFP4 product (used only below about 512 tokens, where K is
    # cut into slabs across workgroups); the library's largest request is 16 MiB
    GEMM_WS = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")

    def dev_bf16(bits):
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)

    # ---- inputs resident in HBM, weights quantized offline, scales calibrated once (untimed) ----
    layers = []
    for li, layer in enumerate(cfg.layers):
        x_bits = wl.activation(cfg, li)
        xd, wd = dev_bf16(x_bits), dev_bf16(wl.weight(cfg, li))
        ax, aw = mq.nvfp4_global_scale(xd), mq.nvfp4_global_scale(wd)
        wc, ws = mq.nvfp4_quantize(wd, aw, layout=LAYOUT)
        layers.append(dict(
            layer=layer, x=xd, w=wd, ax=ax, aw=aw, wc=wc, ws=ws,
            xc=torch.empty((M, layer.K // 2), dtype=torch.uint8, device="cuda"),
            xs=torch.empty((M, layer.K // 16), dtype=torch.uint8, device="cuda"),
            y=torch.empty((M, layer.N), dtype=torch.bfloat16, device="cuda"),
            x_bits=x_bits if layer.name in ("gate_up", "linear") else None))
    torch.cuda.synchronize()
    flop_step = sum(wl.layer_flops(M, L["layer"]) for L in layers)
    quant_bytes_step = sum(QUANT_BYTES_PER_ELT * M * L["layer"].K for L in layers)

    def step(events=None):
        for L in layers:
            if events is not None:
                e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                e[0].record()
            mq.nvfp4_quantize(L["x"], L["ax"], L["xc"], L["xs"], LAYOUT)
            if events is not None:
                e[1].record()
            mq.nvfp4_gemm_ws(L["xc"], L["xs"], L["ax"], L["wc"], L["ws"], L["aw"], GEMM_WS, mq.MQ_OUT_BF16, L["y"], LAYOUT)
            if events is not None:
                e[2].record()
                events.append(e)

    if args.copy_calibration:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tflops = flop_step / (ms_per_step * 1e-3) * 1e-12

    nl = len(layers)
    q_ms = [0.0] * nl
    g_ms = [0.0] * nl
    for i, e in enumerate(events):
        q_ms[i % nl] += e[0].elapsed_time(e[1]) / args.steps
        g_ms[i % nl] += e[1].elapsed_time(e[2]) / args.steps
    gemm_ms_step, quant_ms_step = sum(g_ms), sum(q_ms)
    gemm_tflops = flop_step / (gemm_ms_step * 1e-3) * 1e-12
    quant_gbs = quant_bytes_step / (quant_ms_step * 1e-3) * 1e-9

    # ---- same path with the tensor-level scale computed on the fly (amax pass + quantize + GEMM) ----
    def dyn_step():
        for L in layers:
            mq.nvfp4_global_scale(L["x"], L["ax_dyn"])
            mq.nvfp4_quantize(L["x"], L["ax_dyn"], L["xc"], L["xs"], LAYOUT)
            mq.nvfp4_gemm_ws(L["xc"], L["xs"], L["ax_dyn"], L["wc"], L["ws"], L["aw"], GEMM_WS, mq.MQ_OUT_BF16, L["y"], LAYOUT)
    for L in layers:
        L["ax_dyn"] = torch.empty(1, dtype=torch.float32, device="cuda")
    for _ in range(max(1, args.warmup // 2)):
        dyn_step()
    torch.cuda.synchronize()
    d0 = time.perf_counter()
    nd = max(3, args.steps // 2)
    for _ in range(nd):
        dyn_step()
    torch.cuda.synchronize()
    dyn_ms_step = (time.perf_counter() - d0) * 1e3 / nd
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        for L in layers:
            mq.nvfp4_global_scale(L["x"], L["ax_dyn"])
    e1.record()
    torch.cuda.synchronize()
    amax_gbs = 10 * sum(2.0 * M * L["layer"].K for L in layers) / (e0.elapsed_time(e1) * 1e-3) * 1e-9

    # ---- BF16 GEMM on the same shapes (the high-precision baseline) ----
    def bf16_step():
        for L in layers:
            mq.bf16_gemm(L["x"], L["w"], mq.MQ_OUT_BF16, L["y"])
    for _ in range(max(1, args.warmup // 2)):
        bf16_step()
    torch.cuda.synchronize()
    b0 = time.perf_counter()
    nb = max(3, args.steps // 2)
    for _ in range(nb):
        bf16_step()
    torch.cuda.synchronize()
    bf16_ms_step = (time.perf_counter() - b0) * 1e3 / nb
    bf16_tflops = flop_step / (bf16_ms_step * 1e-3) * 1e-12

    # ---- context: the vendor library's BF16 GEMM (hipBLASLt through torch.matmul) on the same shapes ----
    lib_tflops = None
    try:
        def lib_step():
            for L in layers:
                torch.matmul(L["x"], L["w"].t(), out=L["y"])
        for _ in range(3):
            lib_step()
        torch.cuda.synchronize()
        l0 = time.perf_counter()
        for _ in range(nb):
            lib_step()
        torch.cuda.synchronize()
        lib_tflops = flop_step / ((time.perf_counter() - l0) / nb) * 1e-12
    except Exception as exc:  # the library path is context only; never fail the run on it
        print(f"bench.py: torch.matmul reference skipped: {exc}", file=sys.stderr)

    # ---- decode shapes of the high-precision path: a few tokens against the same weights (HBM-bound) ----
    decode = {}
    w_bytes = sum(2.0 * L["layer"].N * L["layer"].K for L in layers)
    for md in (1, 16, 64):
        def dec_step():
            for L in layers:
                mq.bf16_gemm(L["x"][:md], L["w"], mq.MQ_OUT_BF16, L["y"][:md])
        for _ in range(3):
            dec_step()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(20):
            dec_step()
        g1.record()
        torch.cuda.synchronize()
        decode[f"M={md}"] = round(20 * w_bytes / (g0.elapsed_time(g1) * 1e-3) * 1e-9, 1)

    # ---- producer-fused quantizers (the quantizer fused with its neighbour, Section 3.3): the two
    # activations of a decoder block that are quantized, against producer (torch) + nvfp4_quantize ----
    fused = None
    if args.config == 2 and not args.no_fused:
        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            f0.record()
            for _ in range(reps):
                fn()
            f1.record()
            torch.cuda.synchronize()
            return f0.elapsed_time(f1) / reps
        Kd, Kh = 14336, 4096
        gu = torch.randn((M, 2 * Kd), dtype=torch.bfloat16, device="cuda")
        xh = torch.randn((M, Kh), dtype=torch.bfloat16, device="cuda")
        gw = torch.ones(Kh, dtype=torch.bfloat16, device="cuda")
        a1 = torch.full((1,), 30.0 / 2688.0, dtype=torch.float32, device="cuda")
        cd = torch.empty((M, Kd // 2), dtype=torch.uint8, device="cuda")
        sd = torch.empty((M, Kd // 16), dtype=torch.uint8, device="cuda")
        ch = torch.empty((M, Kh // 2), dtype=torch.uint8, device="cuda")
        sh = torch.empty((M, Kh // 16), dtype=torch.uint8, device="cuda")
        t_f1 = timed(lambda: mq.nvfp4_quantize_silu_mul(gu, a1, cd, sd, LAYOUT))
        t_u1 = timed(lambda: mq.nvfp4_quantize(torch.nn.functional.silu(gu[:, :Kd]) * gu[:, Kd:], a1, cd, sd, LAYOUT))
        t_f2 = timed(lambda: mq.nvfp4_quantize_rmsnorm(xh, gw, 1e-6, a1, ch, sh, LAYOUT))
        t_u2 = timed(lambda: mq.nvfp4_quantize(torch.nn.functional.rms_norm(xh, (Kh,), gw, 1e-6), a1, ch, sh, LAYOUT))
        fused = {
            "silu_mul_quantize": {"shape": [M, Kd], "fused_ms": round(t_f1, 4), "producer_then_quantize_ms": round(t_u1, 4),
                                  "fused_gbs": round((4.0 + QUANT_BYTES_PER_ELT - 2.0) * M * Kd / (t_f1 * 1e-3) * 1e-9, 1)},
            "rmsnorm_quantize": {"shape": [M, Kh], "fused_ms": round(t_f2, 4), "producer_then_quantize_ms": round(t_u2, 4),
                                 "fused_gbs": round(QUANT_BYTES_PER_ELT * M * Kh / (t_f2 * 1e-3) * 1e-9, 1)},
        }
        # the MLP half of a decoder block as a dependent chain (each step consumes the previous
        # one's output): RMSNorm -> gate_up -> SiLU*up -> down, NVFP4 with fused quantizers against
        # BF16 with the same in-repo GEMM; tensor-level scales calibrated once, untimed
        by_name = {L["layer"].name: L for L in layers}
        Lg, Ld = by_name["gate_up"], by_name["down"]
        yg = torch.empty((M, 2 * Kd), dtype=torch.bfloat16, device="cuda")
        yo = torch.empty((M, Kh), dtype=torch.bfloat16, device="cuda")
        hn = torch.nn.functional.rms_norm(xh, (Kh,), gw, 1e-6)
        a_n = mq.nvfp4_global_scale(hn)
        mq.bf16_gemm(hn, Lg["w"], mq.MQ_OUT_BF16, yg)
        a_p = mq.nvfp4_global_scale(torch.nn.functional.silu(yg[:, :Kd]) * yg[:, Kd:])
        del hn

        def mlp_nvfp4():
            mq.nvfp4_quantize_rmsnorm(xh, gw, 1e-6, a_n, ch, sh, LAYOUT)
            mq.nvfp4_gemm_ws(ch, sh, a_n, Lg["wc"], Lg["ws"], Lg["aw"], GEMM_WS, mq.MQ_OUT_BF16, yg, LAYOUT)
            mq.nvfp4_quantize_silu_mul(yg, a_p, cd, sd, LAYOUT)
            mq.nvfp4_gemm_ws(cd, sd, a_p, Ld["wc"], Ld["ws"], Ld["aw"], GEMM_WS, mq.MQ_OUT_BF16, yo, LAYOUT)

        def mlp_bf16():
            h = torch.nn.functional.rms_norm(xh, (Kh,), gw, 1e-6)
            mq.bf16_gemm(h, Lg["w"], mq.MQ_OUT_BF16, yg)
            pm = torch.nn.functional.silu(yg[:, :Kd]) * yg[:, Kd:]
            mq.bf16_gemm(pm, Ld["w"], mq.MQ_OUT_BF16, yo)
        t_m4, t_m16 = timed(mlp_nvfp4, 10), timed(mlp_bf16, 10)
        mlp_flop = wl.layer_flops(M, Lg["layer"]) + wl.layer_flops(M, Ld["layer"])
        fused["mlp_block_chain"] = {"nvfp4_ms": round(t_m4, 4), "bf16_ms": round(t_m16, 4),
                                    "nvfp4_tflops": round(mlp_flop / (t_m4 * 1e-3) * 1e-12, 1),
                                    "x_vs_bf16": round(t_m16 / t_m4, 3)}
        del gu, xh, cd, sd, ch, sh, yg, yo
        torch.cuda.empty_cache()

    # ---- second workload: the paper's sweep axis (Section 4.4, Fig. 3: prefill speed-up over BF16
    # against context length / batch), as tokens M per prefill batch on the same layer set.
    # Activations are generated on the device (N(0,1), 0.1 % of the channels scaled by 20: the
    # recipe of the headline workload without its host generator); weights are the headline's. ----
    sweep = None
    if args.config == 2 and not args.no_sweep:
        sweep = {}
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1234)
        for ms in (64, 128, 256, 512, 1024, 2048, 4096, 16384, 32768, 65536, 131072):
            t_q4 = t_b16 = t_ven = 0.0
            small = ms <= 1024
            for L in layers:
                K, N = L["layer"].K, L["layer"].N
                x = torch.randn((ms, K), dtype=torch.bfloat16, device="cuda", generator=gen)
                cols = torch.randperm(K, device="cuda", generator=gen)[:max(1, round(0.001 * K))]
                x[:, cols] *= 20.0
                ax = mq.nvfp4_global_scale(x)
                xc = torch.empty((ms, K // 2), dtype=torch.uint8, device="cuda")
                xs = torch.empty((ms, K // 16), dtype=torch.uint8, device="cuda")
                y = torch.empty((ms, N), dtype=torch.bfloat16, device="cuda")

                def one():
                    mq.nvfp4_quantize(x, ax, xc, xs, LAYOUT)
                    mq.nvfp4_gemm_ws(xc, xs, ax, L["wc"], L["ws"], L["aw"], GEMM_WS, mq.MQ_OUT_BF16, y, LAYOUT)

                def ven():
                    torch.matmul(x, L["w"].t(), out=y)
                for fn, reps in ((one, 20 if small else 3),
                                 (lambda: mq.bf16_gemm(x, L["w"], mq.MQ_OUT_BF16, y), 20 if small else 2),
                                 (ven, 20 if small else 2)):
                    fn()
                    fn()
                    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    s0.record()
                    for _ in range(reps):
                        fn()
                    s1.record()
                    torch.cuda.synchronize()
                    if fn is one:
                        t_q4 += s0.elapsed_time(s1) / reps
                    elif fn is ven:
                        t_ven += s0.elapsed_time(s1) / reps
                    else:
                        t_b16 += s0.elapsed_time(s1) / reps
                del x, xc, xs, y
            fl = sum(wl.layer_flops(ms, L["layer"]) for L in layers)
            sweep[f"M={ms}"] = {"nvfp4_quant_plus_gemm_tflops": round(fl / (t_q4 * 1e-3) * 1e-12, 1),
                                "bf16_gemm_tflops": round(fl / (t_b16 * 1e-3) * 1e-12, 1),
                                "vendor_library_bf16_gemm_tflops": round(fl / (t_ven * 1e-3) * 1e-12, 1),
                                "nvfp4_us": round(t_q4 * 1e3, 1),
                                "x_vs_bf16_gemm": round(t_b16 / t_q4, 3),
                                "x_vs_vendor_library_bf16_gemm": round(t_ven / t_q4, 3)}
            torch.cuda.empty_cache()

    # ---- what the matrix pipe sustains on this machine for random FP16 operands (measured roof) ----
    for _ in range(3):
        mq.mfma_probe(20000)
    torch.cuda.synchronize()
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    p0.record()
    probe_flop = sum(mq.mfma_probe(20000) for _ in range(10))
    p1.record()
    torch.cuda.synchronize()
    mfma_sustained = probe_flop / (p0.elapsed_time(p1) * 1e-3) * 1e-12

    result = {
        "metric": "nvfp4_prefill_gemm_tflops_quant_plus_gemm_m8192",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "nvfp4 (e2m1 x e4m3 block scales) expanded exactly to fp16 MFMA, fp32 accumulate, bf16 out",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: prefill linear layers ({', '.join(L['layer'].name for L in layers)}) "
                               f"at M={M} tokens, NVFP4 W4A4, quantize+GEMM per layer", "M": M,
                   "layers": [[L["layer"].name, L["layer"].K, L["layer"].N] for L in layers]},
        "pct_of_fp4_mfma_peak": round(100.0 * tflops / PEAK_MFMA_FP4, 2),
        "pct_of_16bit_mfma_peak": round(100.0 * tflops / PEAK_MFMA_16BIT, 2),
        "x_vs_bf16_gemm": round(bf16_ms_step / ms_per_step, 3),
        "bf16_gemm_tflops": round(bf16_tflops, 2),
        "vendor_library_bf16_gemm_tflops": None if lib_tflops is None else round(lib_tflops, 2),
        "gemm_only_tflops": round(gemm_tflops, 2),
        "dynamic_alpha_pipeline_tflops": round(flop_step / (dyn_ms_step * 1e-3) * 1e-12, 2),
        "global_scale_gbs": round(amax_gbs, 1),
        "decode_bf16_gemm_weight_gbs": decode,
        "tokens_per_batch_sweep": sweep,
        "fused_producer_quantizers": fused,
        "quantizer_gbs": round(quant_gbs, 1),
        "quantizer_pct_of_hbm_peak": round(100.0 * quant_gbs / PEAK_HBM_GBS, 1),
        "per_layer_ms": {L["layer"].name: {"quantize": round(q_ms[i], 4), "gemm": round(g_ms[i], 4)}
                         for i, L in enumerate(layers)},
        "roofline": {
            "kernel": "nvfp4 gemm (gemm_fp4_direct: 256x256 tile, 4 waves of 128x128, persistent)",
            "bound": "mfma",
            "achieved": round(gemm_tflops, 2),
            "peak": PEAK_MFMA_16BIT,
            "unit": "TFLOP/s",
            "frac": round(gemm_tflops / PEAK_MFMA_16BIT, 4),
            "frac_of_fp4_peak": round(gemm_tflops / PEAK_MFMA_FP4, 4),
            # an MFMA-only loop on random operands, timed in this run: the power-managed clock
            # keeps the matrix pipe well below the published peak on realistic data
            "mfma_only_sustained_tflops": round(mfma_sustained, 1),
            "frac_of_mfma_only_sustained": round(gemm_tflops / mfma_sustained, 4),
            "avg_launch_ms": round(gemm_ms_step / nl, 4),
            "flop_per_launch": flop_step / nl,
            # HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE (x2.0, calibrated on a plain
            # 1 GiB copy) + WRITE_SIZE (x1.0), averaged over the four launches of a step
            # (profiles/nvfp4_gemm_bf16_gemm_quantizer_llama8b_m8192.md)
            "traffic": 0.540 * 2 ** 30 if args.config == 2 else None,
        },
    }

    # ---- the CPU oracle on a bounded sample of the same workload (reported baseline) ----
    if not args.no_cpu_baseline:
        import oracle
        li_sample, L = next((i, l) for i, l in enumerate(layers) if l["x_bits"] is not None)
        rows = min(args.cpu_sample_rows, M)
        xb = L["x_bits"][:rows]
        # everything the oracle sees comes from the seeded generator and the oracle itself
        w_bits = wl.weight(cfg, li_sample)
        ax, aw = oracle.global_scale(L["x_bits"]), oracle.global_scale(w_bits)
        wc, ws = oracle.quantize(w_bits, aw)
        c0 = time.perf_counter()
        xc, xs = oracle.quantize(xb, ax)
        a = oracle.dequantize(xc, xs, ax)
        b = oracle.dequantize(wc, ws, aw)
        y = oracle.gemm_f64(a, b)
        y16 = oracle.bf16_round(y)
        c1 = time.perf_counter()
        flop = 2.0 * rows * L["layer"].N * L["layer"].K
        result["cpu_baseline"] = {
            "value": round(flop / (c1 - c0) * 1e-12, 6),
            "unit": "TFLOP/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "seconds": round(c1 - c0, 2),
            "sample": f"first {rows} of {M} rows of the {L['layer'].name} layer "
                      f"(K={L['layer'].K}, N={L['layer'].N}): quantize + dequantize + FP64 GEMM + BF16 rounding",
        }
        # the sample doubles as an end-of-run parity spot check of what was timed
        got = L["y"][:rows]
        mq.nvfp4_linear(L["x"], L["ax"], L["wc"], L["ws"], L["aw"], mq.MQ_OUT_BF16, L["y"], L["xc"], L["xs"], LAYOUT)
        torch.cuda.synchronize()
        gb = got.contiguous().view(torch.int16).cpu().numpy().view(np.uint16).astype(np.int64)
        rb = y16.astype(np.int64)
        ordv = lambda v: np.where(v & 0x8000, -(v & 0x7FFF), v & 0x7FFF)
        result["parity_spot_check"] = {
            "outputs": int(gb.size),
            "frac_within_1_bf16_ulp_of_oracle": round(float((np.abs(ordv(gb) - ordv(rb)) <= 1).mean()), 6)}

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
