#!/usr/bin/env python3
"""Benchmark of the NVFP4 hot path on one MI355X.

A step is one forward pass of the DiT FFN pair (A[3520,3072] -> up 14336 -> GELU-tanh ->
re-quantize -> down 3072, bf16 out): quantize A (amax + encode), up GEMM with activation and
re-quantization, down GEMM.  Weights are quantized once, outside the timed region.  The value
is the two GEMMs' 2*M*N*K flops over the whole step time.  The other rows of the path (KV
quantize / dequantize, transposed quantize, dgrad / wgrad GEMMs at the training shape) are
measured once each after the timed region and reported under "rows".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0     # MI355X dense f16/bf16 MFMA
PEAK_HBM_GBS = 8000.0
B_PER_ELEM = 2.5625               # quantize: 2 B read + 0.5625 B written; KV dequant the reverse


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step takes ~0.6 ms; the engine clock needs some tens of milliseconds of load to settle
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-rows", action="store_true", help="skip the per-row extras (KV, training triplet)")
    ap.add_argument("--rows-only", default=None, metavar="SECTIONS",
                    help="run only the per-row measurements of the given sections (comma list of kv, lora, train) "
                         "and print them as one JSON line: for per-kernel profiles of the streaming rows")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    from paper_2605_18739_amd import build as hip_build
    if not os.path.exists(hip_build.LIB):           # the library built in-tree is used as it is; compiled only when there is none
        hip_build.build(verbose=False)
    import paper_2605_18739_amd as nv
    from paper_2605_18739_amd import workloads as wl

    torch.cuda.set_device(0)
    dev = "cuda"
    if args.rows_only:
        rows = measure_rows(nv, wl, torch, np, tuple(args.rows_only.split(",")))
        print(json.dumps({"rows_only": args.rows_only, "data": "synthetic", "rows": rows}))
        return
    M, D, F = wl.TOKENS_INFER, wl.D_MODEL, wl.D_FFN
    cfg = wl.config3()
    A = nv.bf16_from_bits(cfg["A"], dev)
    W1 = nv.nvfp4_quantize(nv.bf16_from_bits(cfg["W1"], dev))
    W2 = nv.nvfp4_quantize(nv.bf16_from_bits(cfg["W2"], dev))
    # everything a step touches is allocated up front
    qA = nv.NVFP4Tensor(M, D, dev)
    qH = nv.NVFP4Tensor(M, F, dev)
    Y = torch.empty((M, D), dtype=torch.bfloat16, device=dev)
    ws_q = torch.empty(nv.nvfp4_workspace_bytes(nv.OP_QUANTIZE, M, D), dtype=torch.uint8, device=dev)
    ws_g = torch.empty(nv.nvfp4_workspace_bytes(nv.OP_GEMM_ACT_QUANT, M, F, 0), dtype=torch.uint8, device=dev)

    def step():
        nv.nvfp4_quantize(A, out=qA, workspace=ws_q)
        nv.nvfp4_gemm_act_quant(qA, W1, nv.ACT_GELU_TANH, out=qH, workspace=ws_g)
        nv.nvfp4_gemm(qH, W2, nv.OUT_BF16, Y=Y)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region records HIP events only around the dominant kernel (an event pair idles the
    # stream for a few microseconds); the per-kernel breakdown comes from a second, untimed loop
    nv.nvfp4_set_timing_ops([nv.OP_GEMM_ACT_QUANT_GEMM])
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    n_up, ms_up = nv.nvfp4_timing_read(nv.OP_GEMM_ACT_QUANT_GEMM)
    nv.nvfp4_set_timing_ops([nv.OP_GEMM, nv.OP_GEMM_ACT_QUANT, nv.OP_QUANTIZE])
    for _ in range(min(args.steps, 20)):
        step()
    torch.cuda.synchronize()
    n_gemm, ms_gemm = nv.nvfp4_timing_read(nv.OP_GEMM)
    n_fused, ms_fused = nv.nvfp4_timing_read(nv.OP_GEMM_ACT_QUANT)
    n_q, ms_q = nv.nvfp4_timing_read(nv.OP_QUANTIZE)
    nv.nvfp4_set_timing(False)

    ms_step = (t1 - t0) * 1e3 / args.steps
    flops_gemm = 2.0 * M * F * D
    value = 2 * flops_gemm / (ms_step * 1e-3) / 1e12
    # dominant kernel: the up-projection GEMM (GELU + bf16 H + amax in its epilogue), timed by HIP
    # events on the stream it runs on.  The library launches it as whole waves of 256x256 tiles
    # (768 of the 784) plus a second, small launch (64x64 tiles) for the last 16 tile positions; the events
    # bracket both, and the flops are those of the whole projection.
    up_ms = ms_up / max(n_up, 1)
    achieved = flops_gemm / (up_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "up projection 3520x14336x3072, f16 MFMA: gemm_regdq_kernel<256,256,bf16+gelu> (768 tiles) + gemm_regdq_kernel<64,64,bf16+gelu> (rest)",
                "achieved": round(achieved, 1), "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_MFMA_F16_TFLOPS, 4), "traffic": profile_traffic(),
                "avg_launch_ms": round(up_ms, 4), "launches": n_up}
    gemm_ms = ms_gemm / max(n_gemm, 1)
    fused_ms = ms_fused / max(n_fused, 1)
    q_ms = ms_q / max(n_q, 1)
    kernels = {
        "up_gemm_gelu_h_amax": {"ms": round(up_ms, 4), "tflops": round(achieved, 1)},
        "up_gemm_gelu_requant_total": {"ms": round(fused_ms, 4), "tflops": round(flops_gemm / (fused_ms * 1e-3) / 1e12, 1)},
        "down_gemm_3520x3072x14336": {"ms": round(gemm_ms, 4), "tflops": round(flops_gemm / (gemm_ms * 1e-3) / 1e12, 1),
                                      "frac_mfma": round(flops_gemm / (gemm_ms * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS, 4)},
        "quantize_A_3520x3072": {"ms": round(q_ms, 4),
                                 "GBs": round(B_PER_ELEM * M * D / (q_ms * 1e-3) / 1e9, 1)},
    }
    # the same up projection with the activation scale supplied by the caller: one pass, H never written
    gs_h = qH.global_scale.clone()
    ms1 = _time_op(nv, torch, nv.OP_GEMM_ACT_QUANT,
                   lambda: nv.nvfp4_gemm_act_quant(qA, W1, nv.ACT_GELU_TANH, global_scale_in=gs_h, out=qH, workspace=ws_g), 20)
    kernels["up_gemm_gelu_requant_given_scale"] = {"ms": round(ms1, 4), "tflops": round(flops_gemm / (ms1 * 1e-3) / 1e12, 1)}

    if args.copy_calib:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    rows = None if args.no_rows else measure_rows(nv, wl, torch, np)
    cpu = None if args.no_cpu else cpu_baseline(cfg, wl, np)

    out = {
        "metric": "nvfp4_gemm_tflops_dit_ffn", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "dit_ffn_pair: A[3520,3072] -> W1[14336,3072] -> gelu_tanh -> requantize -> "
                               "W2[3072,14336], W4A4 NVFP4, bf16 out (the DiT FFN pair configuration)",
                   "global_batch": M, "parallelism": "single-gpu"},
        "roofline": roofline, "kernels": kernels, "rows": rows, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


def profile_traffic():
    """HBM bytes per launch of the dominant kernel from the committed counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "gemm_up_projection_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def _time_op(nv, torch, op_id, fn, iters, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    nv.nvfp4_set_timing(True)
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    n, ms = nv.nvfp4_timing_read(op_id)
    nv.nvfp4_set_timing(False)
    return ms / max(n, 1)


def measure_rows(nv, wl, torch, np, sections=("kv", "lora", "train")):
    """One measurement per remaining row of the path, at the sizes of the KV and training configs."""
    dev = "cuda"
    res = {}
    ws = torch.empty(4096, dtype=torch.uint8, device=dev)
    if "kv" in sections:
        _rows_kv(nv, wl, torch, res, ws)
    if "lora" in sections:
        _rows_lora(nv, wl, torch, res)
    if "train" in sections:
        _rows_train(nv, wl, torch, res, ws)
    return res


def _rows_kv(nv, wl, torch, res, ws):
    dev = "cuda"
    # --- KV cache: K [18480, 24, 128] -------------------------------------------------------
    T, H, d = wl.KV_TOKENS, wl.KV_HEADS, wl.KV_DIM
    kv = nv.bf16_from_bits(wl.kv_tensor(T, H, d, 3, 0), dev)
    q = nv.NVFP4Tensor(T * H, d, dev)
    back = torch.empty_like(kv)
    n = T * H * d
    ms = _time_op(nv, torch, nv.OP_KV_QUANT, lambda: nv.nvfp4_kv_quant(kv, out=q, workspace=ws), 20)
    res["kv_quant_18480x24x128"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n / ms / 1e6, 1),
                                    "frac_hbm": round(B_PER_ELEM * n / ms / 1e6 / PEAK_HBM_GBS, 4)}
    # the same cache with the Four-over-Six scale search (the variant the paper applies to the cache)
    ms = _time_op(nv, torch, nv.OP_KV_QUANT_4OVER6, lambda: nv.nvfp4_kv_quant_4over6(kv, out=q, workspace=ws), 20)
    res["kv_quant_4over6_18480x24x128"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n / ms / 1e6, 1),
                                           "frac_hbm": round(B_PER_ELEM * n / ms / 1e6 / PEAK_HBM_GBS, 4)}
    # keys as the paper caches them: row means removed (K-smoothing), then the scale search
    mean = torch.empty(T * H, dtype=torch.bfloat16, device=dev)
    ms = _time_op(nv, torch, nv.OP_KV_QUANT_K, lambda: nv.nvfp4_kv_quant_k(kv, out=q, row_mean=mean, workspace=ws), 20)
    res["kv_quant_k_smooth_4over6_18480x24x128"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n / ms / 1e6, 1),
                                                    "frac_hbm": round(B_PER_ELEM * n / ms / 1e6 / PEAK_HBM_GBS, 4)}
    # gathered reconstruction of a window of 21 chunks of 880 tokens (one launch), plain and smoothed
    Tc = 880
    chunks_v, chunks_k = [], []
    for c in range(T // Tc):
        part = kv[c * Tc:(c + 1) * Tc]
        chunks_v.append((nv.nvfp4_kv_quant(part), None, Tc))
        qk, mk = nv.nvfp4_kv_quant_k(part)
        chunks_k.append((qk, mk, Tc))
    ms = _time_op(nv, torch, nv.OP_KV_DEQUANT_GATHER, lambda: nv.nvfp4_kv_dequant_gather(chunks_v, H, d, out=back), 20)
    res["kv_dequant_gather_21x880x24x128"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n / ms / 1e6, 1),
                                              "frac_hbm": round(B_PER_ELEM * n / ms / 1e6 / PEAK_HBM_GBS, 4)}
    ms = _time_op(nv, torch, nv.OP_KV_DEQUANT_GATHER, lambda: nv.nvfp4_kv_dequant_gather(chunks_k, H, d, out=back), 20)
    res["kv_dequant_gather_smoothed_21x880x24x128"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n / ms / 1e6, 1),
                                                       "frac_hbm": round(B_PER_ELEM * n / ms / 1e6 / PEAK_HBM_GBS, 4)}
    del chunks_v, chunks_k, mean
    nv.nvfp4_kv_quant(kv, out=q, workspace=ws)
    ms = _time_op(nv, torch, nv.OP_KV_DEQUANT, lambda: nv.nvfp4_kv_dequant(q, T, H, d, out=back), 20)
    res["kv_dequant_18480x24x128"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n / ms / 1e6, 1),
                                      "frac_hbm": round(B_PER_ELEM * n / ms / 1e6 / PEAK_HBM_GBS, 4)}
    # send buffers of the NVFP4 all-to-all: one device's share of that window among 4 (L/P = 4620 tokens),
    # cast along d and regrouped into 4 per-destination slabs of 6 heads
    P = 4
    Tl = T // P
    q_a2a = nv.NVFP4Tensor(Tl * H, d, dev)
    ms = _time_op(nv, torch, nv.OP_QUANTIZE_A2A, lambda: nv.nvfp4_quantize_for_all_to_all(kv[:Tl], P, out=q_a2a, workspace=ws), 20)
    n_l = Tl * H * d
    res[f"quantize_for_all_to_all_{Tl}x{H}x{d}_P{P}"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * n_l / ms / 1e6, 1),
                                                        "frac_hbm": round(B_PER_ELEM * n_l / ms / 1e6 / PEAK_HBM_GBS, 4)}
    del kv, back, q, q_a2a


def _rows_lora(nv, wl, torch, res):
    dev = "cuda"
    # --- LoRA side branch on the DiT projection (rank 128, alpha 128): bf16 down projection, then the
    # quantized GEMM with the low-rank update fused in, against the plain quantized GEMM ------------
    c2 = wl.config2()
    Mi, Dm = wl.TOKENS_INFER, wl.D_MODEL
    Xi = nv.bf16_from_bits(c2["A"], dev)
    qXi, qWi = nv.nvfp4_quantize(Xi), nv.nvfp4_quantize(nv.bf16_from_bits(c2["W"], dev))
    La = nv.bf16_from_bits(wl.normal((nv.LORA_RANK, Dm), 0.02, 1, 7), dev)
    Lb = nv.bf16_from_bits(wl.normal((Dm, nv.LORA_RANK), 0.02, 1, 8), dev)
    Tl = torch.empty((Mi, nv.LORA_RANK), dtype=torch.bfloat16, device=dev)
    Yl = torch.empty((Mi, Dm), dtype=torch.bfloat16, device=dev)
    fl = 2.0 * Mi * Dm * Dm
    wsl = torch.empty(nv.nvfp4_workspace_bytes(nv.OP_LORA_DOWN, Mi, Dm), dtype=torch.uint8, device=dev)
    ms = _time_op(nv, torch, nv.OP_LORA_DOWN, lambda: nv.nvfp4_lora_down(Xi, La, out=Tl, workspace=wsl), 20)
    res["lora_down_3520x3072_r128"] = {"ms": round(ms, 4), "tflops": round(2.0 * Mi * Dm * nv.LORA_RANK / ms / 1e9, 1)}
    ms = _time_op(nv, torch, nv.OP_GEMM_LORA, lambda: nv.nvfp4_gemm_lora(qXi, qWi, Tl, Lb, 1.0, nv.OUT_BF16, Y=Yl), 20)
    res["gemm_lora_fused_3520x3072x3072"] = {"ms": round(ms, 4), "tflops": round((fl + 2.0 * Mi * Dm * nv.LORA_RANK) / ms / 1e9, 1)}
    ms = _time_op(nv, torch, nv.OP_GEMM, lambda: nv.nvfp4_gemm(qXi, qWi, nv.OUT_BF16, Y=Yl), 20)
    res["gemm_plain_3520x3072x3072"] = {"ms": round(ms, 4), "tflops": round(fl / ms / 1e9, 1),
                                        "frac_mfma": round(fl / ms / 1e9 / PEAK_MFMA_F16_TFLOPS, 4)}
    del c2, Xi, qXi, qWi, La, Lb, Tl, Yl


def _rows_train(nv, wl, torch, res, ws):
    dev = "cuda"
    # --- training triplet: X[17600,3072], W[14336,3072], dY[17600,14336] ---------------------
    c5 = wl.config5()
    Mt, D, F = wl.TOKENS_TRAIN, wl.D_MODEL, wl.D_FFN
    X, W, dY = (nv.bf16_from_bits(c5[k], dev) for k in ("X", "W", "dY"))
    del c5

    def qtime(x, axis, name):
        R, C = x.shape
        rows, K = (R, C) if axis == 0 else (C, R)
        out = nv.NVFP4Tensor(rows, K, dev)
        ms = _time_op(nv, torch, nv.OP_QUANTIZE, lambda: nv.nvfp4_quantize(x, block_axis=axis, out=out, workspace=ws), 10)
        res[name] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * R * C / ms / 1e6, 1),
                     "frac_hbm": round(B_PER_ELEM * R * C / ms / 1e6 / PEAK_HBM_GBS, 4)}
        return out

    qX = qtime(X, 0, "quantize_X_17600x3072")
    qdY = qtime(dY, 0, "quantize_dY_17600x14336")
    qW = qtime(W, 0, "quantize_W_14336x3072")
    qWt = qtime(W, 1, "quantize_T_W_14336x3072")
    qdYt = qtime(dY, 1, "quantize_T_dY_17600x14336")
    qXt = qtime(X, 1, "quantize_T_X_17600x3072")
    # weight-gradient operand with the random Hadamard transform in front of the transposed quantizer
    qrht = nv.NVFP4Tensor(F, Mt, dev)
    ms = _time_op(nv, torch, nv.OP_QUANTIZE_RHT, lambda: nv.nvfp4_quantize_rht(dY, 0x9A3C, out=qrht, workspace=ws), 5)
    res["quantize_rht_T_dY_17600x14336"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * Mt * F / ms / 1e6, 1),
                                            "frac_hbm": round(B_PER_ELEM * Mt * F / ms / 1e6 / PEAK_HBM_GBS, 4)}
    del qrht
    # weights with one scale per 16x16 tile: W and W^T from one pass (2.5625 B/element per operand written)
    ms = _time_op(nv, torch, nv.OP_QUANTIZE_2D, lambda: nv.nvfp4_quantize_2d(W, workspace=ws), 10)
    res["quantize_2d_W_and_WT_14336x3072"] = {"ms": round(ms, 4), "GBs": round((2.0 + 2 * 0.5625) * F * D / ms / 1e6, 1),
                                              "frac_hbm": round((2.0 + 2 * 0.5625) * F * D / ms / 1e6 / PEAK_HBM_GBS, 4)}
    gs = torch.tensor([float(qdY.global_scale.item())], dtype=torch.float32, device=dev)
    out = nv.NVFP4Tensor(Mt, F, dev)
    ms = _time_op(nv, torch, nv.OP_QUANTIZE, lambda: nv.nvfp4_quantize(dY, global_scale_in=gs, out=out, workspace=ws), 10)
    res["quantize_dY_given_scale"] = {"ms": round(ms, 4), "GBs": round(B_PER_ELEM * Mt * F / ms / 1e6, 1),
                                      "frac_hbm": round(B_PER_ELEM * Mt * F / ms / 1e6 / PEAK_HBM_GBS, 4)}
    # dY along both axes (dgrad needs it along N, wgrad along the tokens): the second call takes the first one's scale
    o_c = nv.NVFP4Tensor(F, Mt, dev)

    def both():
        nv.nvfp4_quantize(dY, out=out, workspace=ws)
        nv.nvfp4_quantize(dY, block_axis=1, global_scale_in=out.global_scale, out=o_c, workspace=ws)

    ms = 2 * _time_op(nv, torch, nv.OP_QUANTIZE, both, 10)          # the timer averages over calls: two per pair
    res["quantize_dY_both_axes_shared_scale"] = {"ms": round(ms, 4), "GBs": round((2 + 2 * 0.5625) * Mt * F / ms / 1e6, 1),
                                                 "frac_hbm": round((2 + 2 * 0.5625) * Mt * F / ms / 1e6 / PEAK_HBM_GBS, 4)}
    del o_c
    del out, X, dY, W

    def gtime(a, w, name, out_dtype=nv.OUT_F32):
        y = torch.empty((a.rows, w.rows), dtype=torch.float32 if out_dtype == nv.OUT_F32 else torch.bfloat16, device=dev)
        ms = _time_op(nv, torch, nv.OP_GEMM, lambda: nv.nvfp4_gemm(a, w, out_dtype, Y=y), 10, warm=3)
        fl = 2.0 * a.rows * w.rows * a.K
        res[name] = {"ms": round(ms, 4), "tflops": round(fl / ms / 1e9, 1),
                     "frac_mfma": round(fl / ms / 1e9 / PEAK_MFMA_F16_TFLOPS, 4)}

    # fp32 outputs (the accumulator as it is); activations and their gradients also as bf16
    gtime(qX, qW, "fprop_17600x14336x3072")
    gtime(qdY, qWt, "dgrad_17600x3072x14336")
    gtime(qdYt, qXt, "wgrad_14336x3072x17600")
    gtime(qX, qW, "fprop_17600x14336x3072_bf16_out", nv.OUT_BF16)
    gtime(qdY, qWt, "dgrad_17600x3072x14336_bf16_out", nv.OUT_BF16)


def cpu_baseline(cfg, wl, np):
    """The CPU oracle, as it stands, on the same workload: the whole FFN pair, once."""
    from oracle import nvfp4_oracle as oracle
    M, D, F = cfg["A"].shape[0], wl.D_MODEL, wl.D_FFN
    t0 = time.perf_counter()
    oa = oracle.quantize(cfg["A"])
    t1 = time.perf_counter()
    ow1, ow2 = oracle.quantize(cfg["W1"]), oracle.quantize(cfg["W2"])      # weights: quantized once, not timed
    t2 = time.perf_counter()
    Y, _ = oracle.gemm(oa, ow1, want_abs=False)
    t3 = time.perf_counter()
    oh = oracle.quantize(oracle.gelu_tanh_bf16(Y))
    t4 = time.perf_counter()
    oracle.gemm(oh, ow2, want_abs=False)
    t5 = time.perf_counter()
    flops = 2.0 * M * F * D
    total = (t1 - t0) + (t5 - t2)
    return {"value": round(2 * flops / total / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"one whole step of the same workload in the oracle (fp64 loops): quantize A {t1 - t0:.2f} s, "
                      f"up GEMM {M}x{F}x{D} {t3 - t2:.2f} s, GELU + requantize {t4 - t3:.2f} s, "
                      f"down GEMM {M}x{D}x{F} {t5 - t4:.2f} s"}


if __name__ == "__main__":
    main()
