#!/usr/bin/env python3
"""Benchmark of the FGMP hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input:
on-the-fly activation quantization (scoring, FP8/NVFP4 decision, encoding)
followed by the block-mixed-precision GEMM against pre-quantized weights,
issued as one fgmp_quant_gemm_fused call (which hands the quantized
activations to the GEMM as the FP16 values of their codes instead of writing
the packed form; `extra.unfused_ms_per_step` times the same work as
fgmp_quantize_activations + fgmp_gemm through the packed form).  The workload is the Llama-2-7B
fused QKV projection at 4K context: X 4096 x 4096 bf16 with 1% outlier
channels, W 12288 x 4096 pre-quantized with 10% FP8 blocks, 10% FP8
activation blocks.  Inputs are resident in HBM before the timed region.

Prints one JSON line (see the keys below).  `value` is 2*M*N*K divided by the
time of a whole step.  `roofline` is for the dominant kernel (the GEMM);
`extra` carries the standalone activation quantizer's GB/s on 16384 x 8192
and the decode-shape (M <= 32) weight-streaming rates.
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

METRIC = "FGMP GEMM TFLOP/s + act-quant GB/s, Llama-2-7B linear shapes, 10% FP8 blocks"
PEAK_MFMA_F16_TFLOPS = 2500.0   # MI355X dense FP16/BF16 matrix peak
PEAK_HBM_GBPS = 8000.0
P_FP8 = 0.10
PREHEAT_S = 0.08                # untimed load before the warm-up steps (clock ramp)
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemm_mixed_kernel_qkv_prefill_traffic.txt")


def traffic_from_profile() -> int:
    """HBM-side bytes of one gemm_mixed_kernel launch on this workload, read from the committed rocprofv3
    summary (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for a
    copy of known size) -- the line "roofline.traffic: ..." of that file.  Fails loudly when the summary or
    the line is missing, so the benchmark line cannot drift away from the evidence it cites."""
    import re
    with open(TRAFFIC_PROFILE) as fh:
        text = fh.read()
    m = re.search(r"^roofline\.traffic:\s*kernel=gemm_mixed_kernel\s+FETCH_SIZE_KiB=([0-9.eE+]+)\s+fetch_scale=([0-9.]+)"
                  r"\s+WRITE_SIZE_KiB=([0-9.eE+]+)\s+write_scale=([0-9.]+)", text, flags=re.M)
    if m is None:
        raise RuntimeError(f"{TRAFFIC_PROFILE} has no 'roofline.traffic:' line")
    fetch, fs, write, ws_ = (float(g) for g in m.groups())
    return int((fetch * fs + write * ws_) * 1024)


def bytes_per_block(p: float) -> float:
    """Packed bytes per 16-element block: 9 B (FP4 + scale) or 16 B (FP8) + 1 metadata bit (Sec. 5.4.1)."""
    return (1.0 - p) * 9.0 + p * 16.0 + 0.125


def single_case(args, torch, fgmp, synth, dev, dev_bf16, timed) -> int:
    """One kernel, one shape, HBM-cold (the launches rotate over copies that exceed the Infinity Cache)."""
    parts = args.case.split(":")
    if parts[0] == "quantizer":
        Mq, Kq = 16384, 8192
        xqd, xqbits = dev_bf16(synth.activations(Mq, Kq, 0, 11))
        sq = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(xqbits)))
        del xqbits
        fq = torch.from_numpy(synth.fisher_per_channel(Kq, 0, 12)).to(dev)
        _, sc = fgmp.quantize_activations(xqd, fq, float("inf"), sq, want_scores=True)
        Tq = fgmp.threshold_for_fraction(sc, P_FP8)
        del sc
        # three inputs and three outputs in rotation (1 GB in all): nothing of a launch's traffic can come from
        # or stay in the 256 MB Infinity Cache
        xs_pool = [xqd, xqd.clone(), xqd.clone()]
        pq_pool = [fgmp.quantize_activations(xqd, fq, Tq, sq) for _ in range(3)]
        it = [0]

        def call_q():
            fgmp.quantize_activations(xs_pool[it[0] % 3], fq, Tq, sq, out=pq_pool[it[0] % 3])
            it[0] += 1
        ms = timed(call_q, args.steps, args.warmup)
        nbytes = Mq * Kq * 2 + (Mq * Kq // 16) * bytes_per_block(P_FP8)
    elif parts[0] == "decode" and len(parts) == 3:
        shapes = dict(synth.LLAMA2_7B)
        shapes["fc1_70b"] = synth.LLAMA2_70B_FC1
        Kd, Nd = shapes[parts[1]]
        Md = int(parts[2])
        gen = torch.Generator(device=dev)
        gen.manual_seed(20)
        wq = torch.empty((Nd, Kd), dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02, generator=gen)
        swq = float(wq.abs().max().float()) / 448.0
        fwq = torch.from_numpy(synth.fisher_per_channel(Kd, 0, 21)).to(dev)
        _, scq = fgmp.quantize_weights(wq, fwq, float("inf"), swq, want_scores=True)
        Twq = fgmp.threshold_for_fraction(scq, P_FP8)
        del scq
        pWd = fgmp.quantize_weights(wq, fwq, Twq, swq)
        del wq
        ncopies = int(600e6 // pWd.buf.numel()) + 1
        pool = [fgmp.Packed(pWd.buf.clone(), Nd, Kd) for _ in range(ncopies)]
        xk, xkb = dev_bf16(synth.activations(Md, Kd, 0, 23))
        sxk = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(xkb)))
        fxk = torch.from_numpy(synth.fisher_per_channel(Kd, 0, 22)).to(dev)
        Yd = torch.empty((Md, Nd), dtype=torch.float32, device=dev)
        wsd = fgmp.new_workspace(fgmp.workspace_bytes(Md, Nd, Kd), dev)
        it = [0]

        def call():
            fgmp.quant_gemm_fused(xk, fxk, 1e-3, sxk, pool[it[0] % ncopies], out=Yd, workspace=wsd)
            it[0] += 1
        ms = timed(call, args.steps, args.warmup)
        nbytes = Nd * Kd // 16 * bytes_per_block(P_FP8) + Md * Kd * 2 + Md * Nd * 4
    else:
        print(f"bench.py: unknown --case {args.case}", file=sys.stderr)
        return 2
    print(json.dumps({"case": args.case, "us_per_launch": round(ms * 1e3, 2), "algorithmic_bytes": int(nbytes),
                      "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}),
          flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the FP8-fraction sweep at the Llama-2-70B FC1 shape (configs[4]; a few GB, ~1 min)")
    ap.add_argument("--case", default=None,
                    help="run ONE kernel-level case in a loop of --steps launches and print its time (what the profiles/ "
                         "summaries of single kernels are made with): decode:<qkv|o|fc1|fc2|fc1_70b>:<M>, or quantizer")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU; --gpus must be 1 "
              "(the path would shard over rows of X or rows of W without communication)",
              file=sys.stderr)
        return 2

    import torch
    from paper_2504_14152_amd import build as fgmp_build, fgmp, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda"
    fgmp.lib()  # fail loudly if the HIP library is missing
    traffic_bytes = traffic_from_profile()

    def dev_bf16(x32):
        bits = synth.f32_to_bf16_bits(x32)
        return torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16), bits

    def timed(fn, iters, warm, heat_s=0.05):
        t_heat = time.perf_counter()
        while time.perf_counter() - t_heat < heat_s:   # untimed: leave the idle clock state (see below)
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters  # ms per call

    if args.case:
        return single_case(args, torch, fgmp, synth, dev, dev_bf16, timed)

    # ------------------------------------------------------------ workload (configs[1])
    M, K, N = 4096, 4096, 12288
    x32 = synth.activations(M, K, 0, 1)
    w32 = synth.weights(N, K, 0, 2)
    fx = synth.fisher_per_channel(K, 0, 3)
    fw = synth.fisher_per_element(N, K, 0, 4)
    xd, xbits = dev_bf16(x32)
    wd, wbits = dev_bf16(w32)
    xref = synth.bf16_bits_to_f32(xbits)
    sx = float(synth.default_tensor_scale(xref))
    sw = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(wbits)))
    fxd, fwd = torch.from_numpy(fx).to(dev), torch.from_numpy(fw).to(dev)
    del w32

    # offline: weight scores -> threshold for 10% FP8 -> packed weights; activation threshold calibrated the same way
    _, sws = fgmp.quantize_weights(wd, fwd, float("inf"), sw, want_scores=True)
    Tw = fgmp.threshold_for_fraction(sws, P_FP8)
    pW = fgmp.quantize_weights(wd, fwd, Tw, sw)
    del sws
    _, sxs = fgmp.quantize_activations(xd, fxd, float("inf"), sx, want_scores=True)
    Tx = fgmp.threshold_for_fraction(sxs, P_FP8)
    del sxs
    w_info = fgmp.packed_info(pW)

    Y = torch.empty((M, N), dtype=torch.float32, device=dev)
    ws = fgmp.new_workspace(fgmp.workspace_bytes(M, N, K), dev)
    pX = fgmp.quantize_activations(xd, fxd, Tx, sx)
    x_info = fgmp.packed_info(pX)

    def step():
        fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW, out=Y, workspace=ws)

    # ------------------------------------------------------------ timed region: K whole steps
    # After the host-side setup above the GPU sits in a low clock state and needs some tens of
    # milliseconds of load to leave it (the first ~30 steps run about 15% slower than the rest); the
    # pre-heat below is untimed, like the W warm-up steps that follow it.
    t_pre = time.perf_counter()
    while time.perf_counter() - t_pre < PREHEAT_S:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    t_host = (time.perf_counter() - t_host0) * 1e3 / args.steps
    ms_step = max(e0.elapsed_time(e1) / args.steps, 1e-6)
    flops = 2.0 * M * N * K
    value = flops / (ms_step * 1e-3) / 1e12

    # dominant kernel: gemm_mixed_kernel (MFMA kernel that decodes the packed weights itself).  Its
    # duration is measured launch by launch: the library records a pair of events on the launch stream
    # immediately before and after the kernel (fgmp_selftest_time_gemm_kernel), over the same number of
    # whole steps as the timed region, issued back to back right after it.
    n_ev = args.steps
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for ea, eb in pairs:      # torch creates the HIP event on first use
        ea.record()
        eb.record()
    # (the shipped library has no hook: the same sources built with FGMP_MEASUREMENT_HOOKS serve here)
    with fgmp.use_library(fgmp_build.lib_path("hooks")):
        for _ in range(10):
            step()
        for ea, eb in pairs:
            fgmp.selftest_time_gemm_kernel(ea, eb)
            step()
        fgmp.selftest_time_gemm_kernel(None, None)
        torch.cuda.synchronize()
    per_launch = sorted(ea.elapsed_time(eb) for ea, eb in pairs)
    ms_kernel = max(sum(per_launch) / len(per_launch), 1e-6)
    achieved = flops / (ms_kernel * 1e-3) / 1e12
    # cross-check: a step launches two kernels back to back -- the quantizer, which writes the FP16 values
    # of the codes it selects, and this kernel -- so the step time minus the quantizer's (timed on its own
    # through fgmp_quantize_dequantize_f16) should come out the same
    x16 = fgmp.quantize_dequantize_f16(xd, fxd, Tx, sx)
    ms_quant16 = timed(lambda: fgmp.quantize_dequantize_f16(xd, fxd, Tx, sx, out=x16), args.steps, 20)
    del x16
    # the same product from packed activations (fgmp_gemm: expands X to FP16 first), and the packing quantizer
    ms_gemm = timed(lambda: fgmp.gemm(pX, pW, out=Y, workspace=ws), args.steps, 20)
    ms_quant = timed(lambda: fgmp.quantize_activations(xd, fxd, Tx, sx, out=pX), args.steps, 20)

    def unfused():
        fgmp.quantize_activations(xd, fxd, Tx, sx, out=pX)
        fgmp.gemm(pX, pW, out=Y, workspace=ws)
    ms_unfused = timed(unfused, args.steps, 20)
    # reference rates measured on this device: a loop of independent FP16 MFMAs (2 waves per SIMD) and a
    # device-to-device copy (bytes read + written)
    sink = torch.empty(1024 * 256, dtype=torch.float32, device=dev)
    ms_mfma = timed(lambda: fgmp.selftest_mfma_rate(1024, 2000, sink), 20, 5)
    mfma_loop_tflops = 1024 * 4 * 2000 * 8 * 32768.0 / (ms_mfma * 1e-3) / 1e12
    src_c = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev).zero_()
    dst_c = torch.empty_like(src_c)
    ms_copy = timed(lambda: dst_c.copy_(src_c), 20, 5)
    copy_gbps = 2.0 * src_c.numel() / (ms_copy * 1e-3) / 1e9
    del sink, src_c, dst_c
    reference = {"mfma_loop_TFLOPs": round(mfma_loop_tflops, 1), "device_copy_GBps": round(copy_gbps, 1)}
    roofline = {"bound": "mfma", "kernel": "gemm_mixed_kernel", "achieved": round(achieved, 2),
                "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_MFMA_F16_TFLOPS, 4),
                "traffic": traffic_bytes, "ms_per_launch": round(ms_kernel, 4),
                "ms_per_launch_median": round(per_launch[len(per_launch) // 2], 4),
                "ms_step_minus_quantizer": round(ms_step - ms_quant16, 4), "ms_quantize_to_f16": round(ms_quant16, 4),
                "frac_of_measured_mfma_loop": round(achieved / mfma_loop_tflops, 4),
                "gemm_call_alone": {"ms": round(ms_gemm, 4), "TFLOPs": round(flops / (ms_gemm * 1e-3) / 1e12, 2)}}

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic", "preheat_ms": PREHEAT_S * 1e3,
        "config": {"workload": "Llama-2-7B fused QKV prefill (configs[1]): X 4096x4096 bf16, 1% channels x20; "
                               "W 12288x4096 N(0,0.02) packed FGMP; 10% FP8 blocks in weights and activations; "
                               "step = fgmp_quant_gemm_fused",
                   "M": M, "K": K, "N": N, "fp8_fraction_w": round(w_info["n_fp8_blocks"] / w_info["n_blocks"], 4),
                   "fp8_fraction_x": round(x_info["n_fp8_blocks"] / x_info["n_blocks"], 4),
                   "packed_w_bytes": w_info["bytes_used"]},
        "roofline": roofline,
        "reference_rates": reference,
    }

    extra = {"ms_quantize_x": round(ms_quant, 4), "ms_gemm": round(ms_gemm, 4), "host_ms_per_step": round(t_host, 4),
             "unfused_ms_per_step": round(ms_unfused, 4)}
    x_bytes = M * K * 2 + (M * K // 16) * bytes_per_block(P_FP8)
    extra["act_quant_prefill_GBps"] = round(x_bytes / (ms_quant * 1e-3) / 1e9, 1)

    if not args.no_extra:
        # standalone activation quantizer, 16384 x 8192 bf16 (configs[4]); HBM-bound
        Mq, Kq = 16384, 8192
        xq = synth.activations(Mq, Kq, 0, 11)
        xqd, xqbits = dev_bf16(xq)
        sq = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(xqbits)))
        del xq, xqbits
        fq = torch.from_numpy(synth.fisher_per_channel(Kq, 0, 12)).to(dev)
        _, sc = fgmp.quantize_activations(xqd, fq, float("inf"), sq, want_scores=True)
        Tq = fgmp.threshold_for_fraction(sc, P_FP8)
        del sc
        pq = fgmp.quantize_activations(xqd, fq, Tq, sq)
        ms_q = timed(lambda: fgmp.quantize_activations(xqd, fq, Tq, sq, out=pq), 20, 3)
        qbytes = Mq * Kq * 2 + (Mq * Kq // 16) * bytes_per_block(P_FP8)
        gbps = qbytes / (ms_q * 1e-3) / 1e9
        extra["act_quant_16384x8192"] = {"ms": round(ms_q, 4), "GBps": round(gbps, 1),
                                         "frac_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4),
                                         "frac_of_measured_copy": round(gbps / copy_gbps, 4),
                                         "algorithmic_bytes": int(qbytes)}
        # what the memory system alone takes for the kernel's access pattern: the same kernel with its arithmetic
        # taken out (measurement build), and the real kernel from the same build right after it
        with fgmp.use_library(fgmp_build.lib_path("hooks")):
            ms_traffic = timed(lambda: fgmp.selftest_quantizer_traffic(xqd, fq, pq), 20, 3)
            ms_q_again = timed(lambda: fgmp.quantize_activations(xqd, fq, Tq, sq, out=pq), 20, 3)
        extra["act_quant_16384x8192"].update({"ms_traffic_model": round(ms_traffic, 4), "ms_same_run": round(ms_q_again, 4),
                                              "traffic_model_over_kernel": round(ms_traffic / ms_q_again, 4)})
        # the same pass with the Eq. 8 score (error increase of NVFP4 over FP8): threshold recalibrated for 10%
        _, sc = fgmp.quantize_activations(xqd, fq, float("inf"), sq, want_scores=True, score_mode="delta")
        Tqd = fgmp.threshold_for_fraction(sc, P_FP8)
        del sc
        ms_qd = timed(lambda: fgmp.quantize_activations(xqd, fq, Tqd, sq, out=pq, score_mode="delta"), 20, 3)
        extra["act_quant_16384x8192_eq8_score"] = {"ms": round(ms_qd, 4),
                                                   "GBps": round(qbytes / (ms_qd * 1e-3) / 1e9, 1),
                                                   "frac_hbm_peak": round(qbytes / (ms_qd * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                                                   "fp8_fraction": round(fgmp.packed_info(pq)["n_fp8_blocks"] /
                                                                         (Mq * Kq // 16), 4)}
        del xqd, pq
        # offline weight quantization of the workload's W with sensitivity-weighted clipping (Eq. 11):
        # 127 candidate scales per block, about 6 FP32 operations per element and candidate
        pWc = fgmp.quantize_weights_clip(wd, fwd, Tw, sw)
        ms_clip = timed(lambda: fgmp.quantize_weights_clip(wd, fwd, Tw, sw, out=pWc), 5, 1)
        ms_plain = timed(lambda: fgmp.quantize_weights(wd, fwd, Tw, sw, out=pWc), 5, 1)
        clip_flops = 6.0 * 127 * N * K
        extra["weight_quant_clip_12288x4096"] = {"ms": round(ms_clip, 3), "ms_without_clipping": round(ms_plain, 3),
                                                 "fp32_TFLOPs": round(clip_flops / (ms_clip * 1e-3) / 1e12, 1),
                                                 "frac_fp32_vector_peak": round(clip_flops / (ms_clip * 1e-3) / 1e12 / 157.3, 3)}
        del pWc
        # decode shapes (configs[3]): M tokens against packed weights of the four Llama-2-7B linears; a step
        # is fgmp_quant_gemm_fused: ONE kernel that quantizes the M activation rows and streams the weights.
        # HBM-cold: the launches rotate over copies of the packed weights that together exceed the
        # 256 MB Infinity Cache, so every launch streams its weights from HBM.
        dec = {}
        for name, (Kd, Nd) in synth.LLAMA2_7B.items():
            if name == "qkv":
                pWd = pW
            else:
                wq, wqb = dev_bf16(synth.weights(Nd, Kd, 0, 20))
                swq = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(wqb)))
                del wqb
                fwq = torch.from_numpy(synth.fisher_per_channel(Kd, 0, 21)).to(dev)
                _, scq = fgmp.quantize_weights(wq, fwq, float("inf"), swq, want_scores=True)
                Twq = fgmp.threshold_for_fraction(scq, P_FP8)
                del scq
                pWd = fgmp.quantize_weights(wq, fwq, Twq, swq)
                del wq
            used = fgmp.packed_info(pWd)["bytes_used"]
            ncopies = int(600e6 // pWd.buf.numel()) + 1
            pool = [fgmp.Packed(pWd.buf.clone(), Nd, Kd) for _ in range(ncopies)]
            fxk = torch.from_numpy(synth.fisher_per_channel(Kd, 0, 22)).to(dev)
            xk, _ = dev_bf16(synth.activations(32, Kd, 0, 23))
            for Md in (1, 8, 32):
                pXd = fgmp.quantize_activations(xk[:Md].contiguous(), fxk, 1e-3, sx)
                Yd = torch.empty((Md, Nd), dtype=torch.float32, device=dev)
                wsd = fgmp.new_workspace(fgmp.workspace_bytes(Md, Nd, Kd), dev)
                xmd = xk[:Md].contiguous()
                it = [0]

                def call():      # the whole decode step: quantize the M activation rows, multiply
                    fgmp.quant_gemm_fused(xmd, fxk, 1e-3, sx, pool[it[0] % ncopies], out=Yd, workspace=wsd)
                    it[0] += 1

                def call_gemm():  # the product alone, from activations packed earlier
                    fgmp.gemm(pXd, pool[it[0] % ncopies], out=Yd, workspace=wsd)
                    it[0] += 1
                ms_d = timed(call, 40, 5)
                ms_g = timed(call_gemm, 40, 5)
                dbytes = Nd * Kd // 16 * bytes_per_block(P_FP8) + Md * Kd * 2 + Md * Nd * 4
                dec[f"{name}_K{Kd}_N{Nd}_M{Md}"] = {
                    "us_per_step": round(ms_d * 1e3, 2), "GBps": round(dbytes / (ms_d * 1e-3) / 1e9, 1),
                    "frac_hbm_peak": round(dbytes / (ms_d * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                    "frac_of_measured_copy": round(dbytes / (ms_d * 1e-3) / 1e9 / copy_gbps, 4),
                    "us_gemm_from_packed_x": round(ms_g * 1e3, 2), "packed_w_bytes": used}
                # the same steps captured in one HIP graph (a step per weight copy) and replayed: what a serving
                # loop runs that must not be bound by the host's launch path (the eager loop above issues one
                # Python call per step; steps shorter than that call are host-bound there)
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for cpy in pool:
                        fgmp.quant_gemm_fused(xmd, fxk, 1e-3, sx, cpy, out=Yd, workspace=wsd)
                ms_graph = timed(graph.replay, 10, 3) / ncopies
                dec[f"{name}_K{Kd}_N{Nd}_M{Md}"]["us_per_step_in_hip_graph"] = round(ms_graph * 1e3, 2)
                del graph
                if name in ("qkv", "fc1"):
                    # the same step with its results quantized and packed inside the launch (Sec. 4.2), against
                    # the FP32 step followed by the standalone quantizer (10% of the result blocks FP8)
                    fnd = torch.from_numpy(synth.fisher_per_channel(Nd, 0, 24)).to(dev)
                    call()
                    s_yd = float(Yd.abs().max()) / 448.0
                    _, scy = fgmp.quantize_activations(Yd, fnd, float("inf"), s_yd, want_scores=True)
                    T_yd = fgmp.threshold_for_fraction(scy, P_FP8)
                    wsp = fgmp.new_workspace(fgmp.workspace_bytes_packed_out(Md, Nd, Kd), dev)
                    pYd = fgmp.quant_gemm_fused_packed_out(xmd, fxk, 1e-3, sx, pool[0], fnd, T_yd, s_yd, workspace=wsp)
                    pYq = fgmp.quantize_activations(Yd, fnd, T_yd, s_yd)

                    def call_packed():   # one launch: the step quantizes its own results
                        fgmp.quant_gemm_fused_packed_out(xmd, fxk, 1e-3, sx, pool[it[0] % ncopies], fnd, T_yd, s_yd,
                                                         out=pYd, workspace=wsp, epilogue=fgmp.EPILOGUE_ONE_LAUNCH)
                        it[0] += 1

                    def call_then_quantize():   # two launches: FP32 results, then the standalone quantizer
                        call()
                        fgmp.quantize_activations(Yd, fnd, T_yd, s_yd, out=pYq)
                    entry = dec[f"{name}_K{Kd}_N{Nd}_M{Md}"]
                    entry["packed_out"] = {"us_one_launch": round(timed(call_packed, 40, 5) * 1e3, 2),
                                           "us_two_launches": round(timed(call_then_quantize, 40, 5) * 1e3, 2)}
                    for tag, fn in (("us_one_launch_in_hip_graph", call_packed), ("us_two_launches_in_hip_graph", call_then_quantize)):
                        it[0] = 0
                        graph = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(graph):
                            for _ in range(ncopies):
                                fn()
                        entry["packed_out"][tag] = round(timed(graph.replay, 10, 3) / ncopies * 1e3, 2)
                        del graph
            del pool
        extra["decode_hbm_cold"] = dec
        # kernel-level entries beside the dominant kernel's: both are bound by HBM; bytes are the algorithmic
        # ones (packed weights + activations in + results out; input + packed output), time is the launch's
        # share of a run of back-to-back launches on one stream (for the decode step, a single kernel, that
        # includes the gap between launches; the figure inside a HIP graph is given beside it)
        for tag, key in (("decode_qkv_M1", "qkv_K4096_N12288_M1"), ("decode_qkv_M8", "qkv_K4096_N12288_M8"),
                         ("decode_fc1_M8", "fc1_K4096_N22016_M8")):
            d = dec[key]
            roofline[tag] = {"bound": "hbm", "kernel": "gemm_stream_kernel", "achieved": d["GBps"], "peak": PEAK_HBM_GBPS,
                             "unit": "GB/s", "frac": d["frac_hbm_peak"], "us_per_launch": d["us_per_step"],
                             "us_per_launch_in_hip_graph": d.get("us_per_step_in_hip_graph")}
        q = extra["act_quant_16384x8192"]
        roofline["quantizer"] = {"bound": "hbm", "kernel": "quantize_act_kernel", "achieved": q["GBps"], "peak": PEAK_HBM_GBPS,
                                 "unit": "GB/s", "frac": q["frac_hbm_peak"], "us_per_launch": round(q["ms"] * 1e3, 2),
                                 "us_traffic_model": round(q["ms_traffic_model"] * 1e3, 2),
                                 "frac_of_traffic_model": q["traffic_model_over_kernel"],
                                 "workload": "16384 x 8192 bf16 -> packed, 10% FP8 blocks"}
    def prefill_case(Mp_, Kp_, Np_, p_w, p_x, kind, tid):
        """Fused step on another prefill shape; returns ms and TFLOP/s (per-channel weight Fisher)."""
        xp, xpb = dev_bf16(synth.activations(Mp_, Kp_, 0, tid, kind=kind))
        sxp = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(xpb)))
        del xpb
        wp = torch.empty((Np_, Kp_), dtype=torch.bfloat16, device=dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(1000 + tid)
        wp.normal_(0.0, 0.02, generator=gen)       # weights of this size are drawn on the device
        swp = float(wp.abs().max().float()) / 448.0
        fxp = torch.from_numpy(synth.fisher_per_channel(Kp_, 0, tid + 1)).to(dev)
        fwp = torch.from_numpy(synth.fisher_per_channel(Kp_, 0, tid + 2)).to(dev)
        _, sc_w = fgmp.quantize_weights(wp, fwp, float("inf"), swp, want_scores=True)
        Twp = fgmp.threshold_for_fraction(sc_w, p_w)
        del sc_w
        pWp = fgmp.quantize_weights(wp, fwp, Twp, swp)
        del wp
        _, sc_x = fgmp.quantize_activations(xp, fxp, float("inf"), sxp, want_scores=True)
        Txp = fgmp.threshold_for_fraction(sc_x, p_x)
        del sc_x
        Yp = torch.empty((Mp_, Np_), dtype=torch.float32, device=dev)
        wsp = fgmp.new_workspace(fgmp.workspace_bytes(Mp_, Np_, Kp_), dev)
        ms_p = timed(lambda: fgmp.quant_gemm_fused(xp, fxp, Txp, sxp, pWp, out=Yp, workspace=wsp), 50, 10)
        info = fgmp.packed_info(pWp)
        return {"ms_per_step": round(ms_p, 4), "TFLOPs": round(2.0 * Mp_ * Np_ * Kp_ / (ms_p * 1e-3) / 1e12, 1),
                "frac_mfma_peak": round(2.0 * Mp_ * Np_ * Kp_ / (ms_p * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS, 4),
                "fp8_fraction_w": round(info["n_fp8_blocks"] / info["n_blocks"], 4), "packed_w_bytes": info["bytes_used"]}

    if not args.no_extra:
        # MLP prefill shapes (configs[2]); whole fused step, activation quantization included
        extra["prefill_fc1_4096x4096x22016"] = prefill_case(4096, 4096, 22016, P_FP8, P_FP8, "normal", 40)
        extra["prefill_fc2_4096x11008x4096"] = prefill_case(4096, 11008, 4096, P_FP8, P_FP8, "silu_gate", 50)
    def layer_chain():
        """The four linears of one Llama-2-7B layer as a chain of fused steps (QKV -> O -> FC1 -> FC2; the
        attention and the gated activation between them are replaced by taking the leading columns of the
        previous FP32 output), with ONE threshold for all weight tensors and ONE for all activation tensors
        (Eq. 10) instead of one per tensor.  Returns timing and the per-layer FP8 fractions (cf. Fig. 7)."""
        shapes = [("qkv", 4096, 12288), ("o", 4096, 4096), ("fc1", 4096, 22016), ("fc2", 11008, 4096)]
        gen = torch.Generator(device=dev)
        gen.manual_seed(4242)
        Ws, Fws, Sws, w_scores = [], [], [], []
        for li, (_, Kl, Nl) in enumerate(shapes):
            wl = torch.empty((Nl, Kl), dtype=torch.bfloat16, device=dev)
            wl.normal_(0.0, 0.02, generator=gen)
            fwl = torch.from_numpy(synth.fisher_per_channel(Kl, 0, 300 + li)).to(dev)
            swl = float(wl.abs().max().float()) / 448.0
            _, scl = fgmp.quantize_weights(wl, fwl, float("inf"), swl, want_scores=True)
            Ws.append(wl); Fws.append(fwl); Sws.append(swl); w_scores.append(scl)
        T_w = fgmp.threshold_for_fraction_multi(w_scores, P_FP8)
        del w_scores
        pWs = [fgmp.quantize_weights(wl, fwl, T_w, swl) for wl, fwl, swl in zip(Ws, Fws, Sws)]
        del Ws
        Fxs = [torch.from_numpy(synth.fisher_per_channel(Kl, 0, 310 + li)).to(dev) for li, (_, Kl, _) in enumerate(shapes)]
        Ys = [torch.empty((M, Nl), dtype=torch.float32, device=dev) for _, _, Nl in shapes]
        wss = [fgmp.new_workspace(fgmp.workspace_bytes(M, Nl, Kl), dev) for _, Kl, Nl in shapes]

        def layer_input(li):
            return xd if li == 0 else Ys[li - 1][:, :shapes[li][1]]
        # calibration pass: per-tensor thresholds, activation scales and scores of every layer input
        Sxs, x_scores = [], []
        for li in range(4):
            cur = layer_input(li)
            sxl = float(cur.abs().max().float()) / 448.0
            _, scl = fgmp.quantize_activations(cur, Fxs[li], float("inf"), sxl, want_scores=True)
            fgmp.quant_gemm_fused(cur, Fxs[li], fgmp.threshold_for_fraction(scl, P_FP8), sxl, pWs[li], out=Ys[li],
                                  workspace=wss[li])
            Sxs.append(sxl); x_scores.append(scl)
        T_x = fgmp.threshold_for_fraction_multi(x_scores, P_FP8)
        del x_scores

        def chain():
            for li in range(4):
                fgmp.quant_gemm_fused(layer_input(li), Fxs[li], T_x, Sxs[li], pWs[li], out=Ys[li], workspace=wss[li])
        ms_c = timed(chain, 20, 5)
        fl = sum(2.0 * M * Kl * Nl for _, Kl, Nl in shapes)
        frac_w, frac_x = {}, {}
        for li, (name, _, _) in enumerate(shapes):
            iw = fgmp.packed_info(pWs[li])
            frac_w[name] = round(iw["n_fp8_blocks"] / iw["n_blocks"], 4)
            ix = fgmp.packed_info(fgmp.quantize_activations(layer_input(li), Fxs[li], T_x, Sxs[li]))
            frac_x[name] = round(ix["n_fp8_blocks"] / ix["n_blocks"], 4)
        return {"ms_per_layer_pass": round(ms_c, 4), "TFLOPs": round(fl / (ms_c * 1e-3) / 1e12, 1),
                "frac_mfma_peak": round(fl / (ms_c * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS, 4),
                "fp8_fraction_weights_by_layer": frac_w, "fp8_fraction_activations_by_layer": frac_x,
                "target_fraction": P_FP8}

    if not args.no_extra:
        extra["layer_chain_llama2_7b_M4096_global_thresholds"] = layer_chain()
        # output-side quantization (Sec. 4.2) on the workload: the QKV results are scored, quantized and
        # packed in the GEMM epilogue instead of being stored as FP32 and quantized by a second pass
        f_n = torch.from_numpy(synth.fisher_per_channel(N, 0, 40)).to(dev)
        step()
        s_y = float(Y.abs().max()) / 448.0
        _, scy = fgmp.quantize_activations(Y, f_n, float("inf"), s_y, want_scores=True)
        T_y = fgmp.threshold_for_fraction(scy, P_FP8)
        del scy
        pY = fgmp.quantize_activations(Y, f_n, T_y, s_y)
        ws_po = fgmp.new_workspace(fgmp.lib().fgmp_workspace_bytes_packed_out(M, N, K), dev)
        ms_po = timed(lambda: fgmp.quant_gemm_fused_packed_out(xd, fxd, Tx, sx, pW, f_n, T_y, s_y, out=pY,
                                                               workspace=ws_po), 100, 20)

        def two_pass():
            fgmp.quant_gemm_fused(xd, fxd, Tx, sx, pW, out=Y, workspace=ws)
            fgmp.quantize_activations(Y, f_n, T_y, s_y, out=pY)
        ms_tp = timed(two_pass, 100, 20)
        extra["packed_output_qkv_prefill"] = {"ms_per_step": round(ms_po, 4),
                                              "TFLOPs": round(flops / (ms_po * 1e-3) / 1e12, 1),
                                              "ms_fp32_output_then_quantizer": round(ms_tp, 4),
                                              "fp8_fraction_y": round(fgmp.packed_info(pY)["n_fp8_blocks"] /
                                                                      (M * N // 16), 4)}

    def gated_mlp():
        """The gated MLP of a Llama-2-7B layer at M = 4096 (the FC1 / FC2 shapes of configs[2]): FC1 with its
        22016 weight rows in groups of 32 gate + 32 up rows, SiLU(gate) * up and the output quantizer in
        the GEMM epilogue (the 361 MB of FP32 results and the intermediate tensor never reach memory
        unquantized), FC2 from the packed result.  Beside it the same work as two fused steps with FP32
        results in between and the gate as a framework op."""
        Mm, Kh, Nf, Nh = 4096, 4096, 22016, 11008
        xg, xgb = dev_bf16(synth.activations(Mm, Kh, 0, 60))
        sxg = float(synth.default_tensor_scale(synth.bf16_bits_to_f32(xgb)))
        del xgb
        gen = torch.Generator(device=dev)
        gen.manual_seed(1060)
        w1 = torch.empty((Nf, Kh), dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02, generator=gen)
        w2 = torch.empty((Kh, Nh), dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02, generator=gen)
        fx1 = torch.from_numpy(synth.fisher_per_channel(Kh, 0, 61)).to(dev)
        fh = torch.from_numpy(synth.fisher_per_channel(Nh, 0, 62)).to(dev)
        pws = []
        for wt, fw in ((w1, fx1), (w2, fh)):
            sw_ = float(wt.abs().max().float()) / 448.0
            _, scw = fgmp.quantize_weights(wt, fw, float("inf"), sw_, want_scores=True)
            pws.append(fgmp.quantize_weights(wt, fw, fgmp.threshold_for_fraction(scw, P_FP8), sw_))
            del scw
        del w1, w2
        pW1, pW2 = pws
        _, scx = fgmp.quantize_activations(xg, fx1, float("inf"), sxg, want_scores=True)
        Txg = fgmp.threshold_for_fraction(scx, P_FP8)
        del scx
        # calibration of the intermediate tensor (scale, threshold) from one unfused pass
        Y1 = torch.empty((Mm, Nf), dtype=torch.float32, device=dev)
        ws1 = fgmp.new_workspace(fgmp.workspace_bytes(Mm, Nf, Kh), dev)
        ws2 = fgmp.new_workspace(fgmp.workspace_bytes(Mm, Kh, Nh), dev)
        Z = torch.empty((Mm, Kh), dtype=torch.float32, device=dev)

        def framework_gate():
            v = Y1.view(Mm, Nf // 64, 2, 32)
            return (torch.nn.functional.silu(v[:, :, 0, :]) * v[:, :, 1, :]).reshape(Mm, Nh).to(torch.bfloat16)
        fgmp.quant_gemm_fused(xg, fx1, Txg, sxg, pW1, out=Y1, workspace=ws1)
        hb = framework_gate()
        s_h = float(hb.abs().max().float()) / 448.0
        _, sch = fgmp.quantize_activations(hb, fh, float("inf"), s_h, want_scores=True)
        T_h = fgmp.threshold_for_fraction(sch, P_FP8)
        del sch
        pH = fgmp.quantize_activations(hb, fh, T_h, s_h)
        ws_g = fgmp.new_workspace(fgmp.lib().fgmp_workspace_bytes_packed_out_ex(Mm, Nf, Kh, fgmp.EPILOGUE_SILU_GATE), dev)

        def fc1_gated():
            fgmp.quant_gemm_fused_packed_out(xg, fx1, Txg, sxg, pW1, fh, T_h, s_h, out=pH, workspace=ws_g,
                                             epilogue=fgmp.EPILOGUE_SILU_GATE)

        def fc2_packed():
            fgmp.gemm(pH, pW2, out=Z, workspace=ws2)

        def both():
            fc1_gated()
            fc2_packed()

        def unfused():
            fgmp.quant_gemm_fused(xg, fx1, Txg, sxg, pW1, out=Y1, workspace=ws1)
            h = framework_gate()
            fgmp.quant_gemm_fused(h, fh, T_h, s_h, pW2, out=Z, workspace=ws2)
        ms1, ms2, ms12, msu = timed(fc1_gated, 50, 10), timed(fc2_packed, 50, 10), timed(both, 50, 10), timed(unfused, 20, 5)
        fl = 2.0 * Mm * Kh * Nf + 2.0 * Mm * Nh * Kh
        fc1_gated()
        ih = fgmp.packed_info(pH)
        return {"ms_fc1_gate_quantize": round(ms1, 4), "ms_fc2_from_packed": round(ms2, 4), "ms_mlp": round(ms12, 4),
                "TFLOPs": round(fl / (ms12 * 1e-3) / 1e12, 1),
                "ms_mlp_fp32_between_and_framework_gate": round(msu, 4),
                "fp8_fraction_h": round(ih["n_fp8_blocks"] / ih["n_blocks"], 4)}

    if not args.no_extra:
        extra["gated_mlp_llama2_7b_M4096"] = gated_mlp()
        # row counts between the decode and the prefill configurations, on the QKV weights (HBM-cold like the
        # decode steps): 33..256 rows run as 32-row chunks through the weight-streaming kernel or on
        # 256-row tiles split along K, whichever the library's cost model expects to be faster
        ncopies = int(600e6 // pW.buf.numel()) + 1
        pool = [fgmp.Packed(pW.buf.clone(), N, K) for _ in range(ncopies)]
        small = {}
        for Ms in (64, 128, 256):
            xs_ = xd[:Ms].contiguous()
            Ys = torch.empty((Ms, N), dtype=torch.float32, device=dev)
            wss = fgmp.new_workspace(fgmp.workspace_bytes(Ms, N, K), dev)
            it = [0]

            def call_small():
                fgmp.quant_gemm_fused(xs_, fxd, Tx, sx, pool[it[0] % ncopies], out=Ys, workspace=wss)
                it[0] += 1
            ms_s = timed(call_small, 40, 5)
            small[f"M{Ms}"] = {"us_per_step": round(ms_s * 1e3, 1), "TFLOPs": round(2.0 * Ms * N * K / (ms_s * 1e-3) / 1e12, 1)}
        del pool
        extra["qkv_between_decode_and_prefill_hbm_cold"] = small

    if not args.no_sweep and not args.no_extra:
        sw_res = {}
        for frac in (0.0, 0.1, 0.2, 0.3, 1.0):
            sw_res[f"fp8_{int(frac * 100)}pct"] = prefill_case(2048, 8192, 57344, frac, frac, "normal", 60)
        extra["sweep_llama2_70b_fc1_2048x8192x57344"] = sw_res
    out["extra"] = extra

    # ------------------------------------------------------------ CPU baseline: the oracle on a bounded sample
    if not args.no_cpu_baseline:
        from oracle import fgmp_oracle as orc

        def oracle_step(rows, cols):
            wref = synth.bf16_bits_to_f32(wbits[:cols])
            qw = orc.quantize(wref, fw[:cols], Tw, sw)             # offline part, not timed
            aw = orc.dequantize(qw["codes"], qw["scales"], qw["mask"])
            t0 = time.perf_counter()
            qx = orc.quantize(xref[:rows], fx, Tx, sx)
            ax = orc.dequantize(qx["codes"], qx["scales"], qx["mask"])
            orc.gemm(ax, sx, aw, sw)
            return time.perf_counter() - t0

        dt_probe = oracle_step(128, 1024)
        # scale the sample to roughly 15 s of CPU work (cost is proportional to rows * cols)
        budget = 15.0 / max(dt_probe, 1e-4) * 128 * 1024
        cols = int(min(N, max(1024, budget // M)))
        rows = int(min(M, max(128, budget // cols)))
        dt = oracle_step(rows, cols)
        cpu_flops = 2.0 * rows * cols * K
        # the same on one thread, on a sample smaller by the thread count (about the same wall time)
        n_thr = orc.num_threads()
        rows1 = max(8, rows // max(n_thr, 1))
        orc.set_num_threads(1)
        dt1 = oracle_step(rows1, cols)
        orc.set_num_threads(n_thr)
        out["cpu_baseline"] = {"value": round(cpu_flops / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"the same step on the first {rows} rows of X (score, quantize, dequantize) "
                                         f"times the first {cols} weight rows at full K={K}, fp64 dot products; "
                                         f"{dt:.1f} s; rate = 2*rows*cols*K / time",
                               "seconds": round(dt, 2),
                               "one_thread": {"value": round(2.0 * rows1 * cols * K / dt1 / 1e12, 6), "unit": "TFLOP/s",
                                              "sample": f"first {rows1} rows of X times the first {cols} weight rows",
                                              "seconds": round(dt1, 2)}}

    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
