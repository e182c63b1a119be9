#!/usr/bin/env python3
"""Benchmark of the NVFP4 hot path on one MI355X.

A step is one forward pass of the DiT FFN pair (A[3520,3072] -> up 14336 -> GELU-tanh ->
re-quantize -> down 3072, bf16 out): quantize A (amax + encode), up GEMM with activation and
re-quantization, down GEMM.  Weights are quantized once, outside the timed region.  The value
is the two GEMMs' 2*M*N*K flops over the whole step time.

Before the warm-up steps the same step runs for a fixed stretch of wall time (--settle-ms, reported
as "settle"): the engine clock needs some hundred milliseconds under load to reach the level it then
holds, and a short timed region right after an idle period would measure that ramp instead.

The other rows of the path (KV quantize / dequantize, transposed quantize, dgrad / wgrad GEMMs at
the training shape, the later variants) are measured after the timed region and reported under
"rows": median and mean of per-call HIP-event durations recorded by the library on the stream it
launches on, with inputs and outputs rotating over enough buffer copies to exceed the 256 MB
Infinity Cache, each next to the seconds the CPU oracle takes for the same operation; "ms_back_to_back" is
the mean over the same calls issued back to back between one pair of events (no event pair per call).  "ceilings"
holds what the same GPU sustains on plain streaming kernels and on back-to-back matrix instructions.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F16_TFLOPS = 2500.0     # MI355X dense f16/bf16 MFMA
PEAK_HBM_GBS = 8000.0
B_PER_ELEM = 2.5625               # quantize: 2 B read + 0.5625 B written; KV dequant the reverse
CACHE_BYTES = 256 << 20           # Infinity Cache: the buffers one row cycles through add up to more than this
TRAFFIC_PROFILE = os.path.join("profiles", "gemm_up_projection_hbm_traffic.txt")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="wall time of untimed, unreported steps before the warm-up (clock settling); 0 = none")
    ap.add_argument("--config", type=int, default=3, choices=(1, 2, 3, 4, 5),
                    help="3 (default): the DiT FFN pair step, the metric's configuration, plus all rows; "
                         "1, 2, 4, 5: only the measurements of that configuration, as one JSON line")
    ap.add_argument("--no-rows", action="store_true", help="skip the per-row extras (KV, training triplet, ceilings)")
    ap.add_argument("--rows-only", default=None, metavar="SECTIONS",
                    help="run only the per-row measurements of the given sections (comma list of tiny, proj, kv, lora, "
                         "train, ceilings) and print them as one JSON line: for per-kernel profiles of the streaming rows")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timings (cpu_baseline and oracle_s)")
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
    ctx = Ctx(nv, wl, torch, np, with_cpu=not args.no_cpu)
    sections_of = {1: ("tiny",), 2: ("proj",), 4: ("kv",), 5: ("train",)}
    if args.rows_only or args.config != 3:
        sections = tuple(args.rows_only.split(",")) if args.rows_only else sections_of[args.config]
        rows = measure_rows(ctx, sections)
        print(json.dumps({"rows_only": ",".join(sections), "data": "synthetic", "cores": ctx.cores(), "rows": rows}))
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

    # clock settling: the same step, untimed, for a fixed stretch of wall time
    settle_steps, t_s0 = 0, time.perf_counter()
    while args.settle_ms > 0 and (time.perf_counter() - t_s0) * 1e3 < args.settle_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
        settle_steps += 20
    settle = {"ms": round((time.perf_counter() - t_s0) * 1e3, 1), "steps": settle_steps,
              "what": "untimed runs of the same step before the warm-up, so that the engine clock has settled"}
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
    up_all = nv.nvfp4_timing_read_all(nv.OP_GEMM_ACT_QUANT_GEMM)
    nv.nvfp4_set_timing_ops([nv.OP_GEMM, nv.OP_GEMM_ACT_QUANT, nv.OP_QUANTIZE])
    for _ in range(max(min(args.steps, 20), 5)):
        step()
    torch.cuda.synchronize()
    gemm_all = nv.nvfp4_timing_read_all(nv.OP_GEMM)
    fused_all = nv.nvfp4_timing_read_all(nv.OP_GEMM_ACT_QUANT)
    q_all = nv.nvfp4_timing_read_all(nv.OP_QUANTIZE)
    nv.nvfp4_set_timing(False)

    ms_step = (t1 - t0) * 1e3 / args.steps
    flops_gemm = 2.0 * M * F * D
    value = 2 * flops_gemm / (ms_step * 1e-3) / 1e12
    # dominant kernel: the up-projection GEMM (GELU + bf16 H + amax in its epilogue), timed by HIP
    # events on the stream it runs on.  The library launches it as whole waves of 256x256 tiles
    # (768 of the 784) plus a second, small launch (64x64 tiles) for the last 16 tile positions; the events
    # bracket both, and the flops are those of the whole projection.
    up_ms = sum(up_all) / max(len(up_all), 1)
    achieved = flops_gemm / (up_ms * 1e-3) / 1e12
    traffic, traffic_note = profile_traffic()
    plan = " + ".join(f"gemm_regdq_kernel<{t},bf16+gelu> ({n} tiles)" for t, n in nv.nvfp4_gemm_plan(M, F, D))
    roofline = {"bound": "mfma", "kernel": f"up projection {M}x{F}x{D}, f16 MFMA: {plan}",
                "achieved": round(achieved, 1), "peak": PEAK_MFMA_F16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_MFMA_F16_TFLOPS, 4), "traffic": traffic, "traffic_source": traffic_note,
                "avg_launch_ms": round(up_ms, 4), "median_launch_ms": round(statistics.median(up_all), 4),
                "launches": len(up_all), "algorithmic_flops_per_launch": flops_gemm}

    def gemm_entry(samples, flops):
        ms = statistics.median(samples)
        return {"ms": round(ms, 4), "ms_mean": round(sum(samples) / len(samples), 4), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                "frac_mfma": round(flops / (ms * 1e-3) / 1e12 / PEAK_MFMA_F16_TFLOPS, 4)}

    kernels = {
        "up_gemm_gelu_h_amax": gemm_entry(up_all, flops_gemm),
        "up_gemm_gelu_requant_total": gemm_entry(fused_all, flops_gemm),
        "down_gemm_3520x3072x14336": gemm_entry(gemm_all, flops_gemm),
        "quantize_A_3520x3072": {"ms": round(statistics.median(q_all), 4),
                                 "GBs": round(B_PER_ELEM * M * D / (statistics.median(q_all) * 1e-3) / 1e9, 1),
                                 "note": "21.6 MB: launch-bound, not a bandwidth figure"},
    }
    # the same up projection with the activation scale supplied by the caller: one pass, H never written
    gs_h = qH.global_scale.clone()
    one = ctx.time_op(nv.OP_GEMM_ACT_QUANT,
                      lambda i: nv.nvfp4_gemm_act_quant(qA, W1, nv.ACT_GELU_TANH, global_scale_in=gs_h, out=qH, workspace=ws_g), 20)
    kernels["up_gemm_gelu_requant_given_scale"] = gemm_entry(one, flops_gemm)

    if args.copy_calib:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    del A, qA, qH, Y, W1, W2
    rows = None if args.no_rows else measure_rows(ctx, ("ceilings", "kv", "lora", "train"))
    cpu = None if args.no_cpu else cpu_baseline(cfg, wl, np)

    out = {
        "metric": "nvfp4_gemm_tflops_dit_ffn", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "dit_ffn_pair: A[3520,3072] -> W1[14336,3072] -> gelu_tanh -> requantize -> "
                               "W2[3072,14336], W4A4 NVFP4, bf16 out (the DiT FFN pair configuration)",
                   "global_batch": M, "parallelism": "single-gpu"},
        "settle": settle,
        "roofline": roofline, "kernels": kernels, "rows": rows, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


def profile_traffic():
    """HBM bytes per launch of the dominant kernel.  Counters cannot be read inside this run (they need
    rocprofv3 around the process): the figure is the one of the committed counter summary, named here."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1]), f"not measured in this run: FETCH_SIZE + WRITE_SIZE of {TRAFFIC_PROFILE}"
    except OSError:
        pass
    return None, "no counter summary found"


class Ctx:
    """What the row measurements share: modules, the timing helper, the oracle clock."""

    def __init__(self, nv, wl, torch, np, with_cpu):
        self.nv, self.wl, self.torch, self.np, self.with_cpu = nv, wl, torch, np, with_cpu
        self._oracle = None

    def oracle(self):
        if self._oracle is None:
            from oracle import nvfp4_oracle
            nvfp4_oracle.build()
            self._oracle = nvfp4_oracle
        return self._oracle

    def cores(self):
        return self.oracle().num_threads() if self.with_cpu else None

    def time_op(self, op_id, fn, iters, warm=3):
        """fn(i) is called warm + iters times with a running index (it picks the buffer copy to work on);
        returns the per-call durations in ms that the library recorded for entry point op_id."""
        nv, torch = self.nv, self.torch
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        nv.nvfp4_set_timing_ops([op_id])
        for i in range(iters):
            fn(warm + i)
        torch.cuda.synchronize()
        samples = Samples(nv.nvfp4_timing_read_all(op_id))
        nv.nvfp4_set_timing(False)
        # the same calls once more, issued back to back between ONE pair of events: what a call costs inside a
        # stream of work, without the event pair of its own around it (a few microseconds on the short kernels)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(warm + i)
        e1.record()
        torch.cuda.synchronize()
        samples.stream_ms = e0.elapsed_time(e1) / iters
        return samples

    def oracle_seconds(self, fn):
        """Wall time of one oracle call on the host cores (None when the oracle legs are switched off)."""
        if not self.with_cpu:
            return None
        t0 = time.perf_counter()
        fn()
        return round(time.perf_counter() - t0, 3)


class Samples(list):
    """Per-call durations (ms) of one entry point, plus .stream_ms: the mean over the same calls issued back to back."""
    stream_ms = None


def copies_for(nbytes):
    """How many buffer copies a row rotates over so that together they exceed the Infinity Cache."""
    return max(2, -(-int(CACHE_BYTES * 1.25) // int(nbytes)))


def bw_row(samples, nbytes, oracle_s=None, copies=None, **extra):
    ms = statistics.median(samples)
    row = {"ms": round(ms, 4), "ms_mean": round(sum(samples) / len(samples), 4), "GBs": round(nbytes / ms / 1e6, 1),
           "frac_hbm": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 4), "calls": len(samples)}
    sm = getattr(samples, "stream_ms", None)
    if sm:
        row["ms_back_to_back"] = round(sm, 4)
        row["frac_hbm_back_to_back"] = round(nbytes / sm / 1e6 / PEAK_HBM_GBS, 4)
    if copies is not None:
        row["buffer_copies"] = copies
    if oracle_s is not None:
        row["oracle_s"] = oracle_s
    row.update(extra)
    return row


def gemm_row(samples, flops, oracle=None):
    ms = statistics.median(samples)
    row = {"ms": round(ms, 4), "ms_mean": round(sum(samples) / len(samples), 4), "tflops": round(flops / ms / 1e9, 1),
           "frac_mfma": round(flops / ms / 1e9 / PEAK_MFMA_F16_TFLOPS, 4), "calls": len(samples)}
    sm = getattr(samples, "stream_ms", None)
    if sm:
        row["ms_back_to_back"] = round(sm, 4)
        row["frac_mfma_back_to_back"] = round(flops / sm / 1e9 / PEAK_MFMA_F16_TFLOPS, 4)
    if oracle is not None:
        row.update(oracle)
    return row


def measure_rows(ctx, sections):
    """One measurement per remaining row of the path, at the sizes of the configurations."""
    res = {}
    ws = ctx.torch.empty(4096, dtype=ctx.torch.uint8, device="cuda")
    table = {"ceilings": _rows_ceilings, "tiny": _rows_tiny, "proj": _rows_proj, "kv": _rows_kv, "lora": _rows_lora,
             "train": _rows_train}
    for name in sections:
        table[name](ctx, res, ws)
        ctx.torch.cuda.empty_cache()
    return res


def _rows_ceilings(ctx, res, ws):
    """What the GPU sustains outside this library's kernels: plain streaming reads, writes and copies of a
    1 GiB buffer (four times the Infinity Cache), and back-to-back MFMAs on register-resident random operands."""
    nv, torch = ctx.nv, ctx.torch
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda")
    b = torch.empty(n, dtype=torch.uint8, device="cuda")
    a.fill_(0x5A)
    for kind, name, moved in ((nv.PROBE_READ, "ceiling_hbm_read_1GiB", n), (nv.PROBE_WRITE, "ceiling_hbm_write_1GiB", n),
                              (nv.PROBE_COPY, "ceiling_hbm_copy_1GiB_read_plus_write", 2 * n)):
        s = ctx.time_op(nv.OP_PROBE, lambda i: nv.nvfp4_probe(kind, a, b, n), 10)
        res[name] = bw_row(s, moved)
    iters = 2000
    for _ in range(3):                                  # the matrix clock settles over a few milliseconds of load
        nv.nvfp4_probe(nv.PROBE_MFMA, None, b, iters=iters)
    s = ctx.time_op(nv.OP_PROBE, lambda i: nv.nvfp4_probe(nv.PROBE_MFMA, None, b, iters=iters), 10)
    res["ceiling_mfma_f16_32x32x16_register_resident_random_operands"] = gemm_row(s, float(iters) * nv.PROBE_MFMA_FLOPS_PER_ITER)
    del a, b


def _rows_tiny(ctx, res, ws):
    """Config 1 (A[128,256], W[256,256]): far too small to time anything but launch latency."""
    nv, wl = ctx.nv, ctx.wl
    cfg = wl.config1()
    a, w = nv.bf16_from_bits(cfg["A"], "cuda"), nv.bf16_from_bits(cfg["W"], "cuda")
    qa, qw = nv.nvfp4_quantize(a), nv.nvfp4_quantize(w)
    s = ctx.time_op(nv.OP_QUANTIZE, lambda i: nv.nvfp4_quantize(a, out=qa, workspace=ws), 20)
    res["quantize_A_128x256"] = bw_row(s, B_PER_ELEM * 128 * 256, ctx.oracle_seconds(lambda: ctx.oracle().quantize(cfg["A"])),
                                       note="launch-bound")
    y = ctx.torch.empty((128, 256), dtype=ctx.torch.float32, device="cuda")
    s = ctx.time_op(nv.OP_GEMM, lambda i: nv.nvfp4_gemm(qa, qw, nv.OUT_F32, Y=y), 20)
    o = None
    if ctx.with_cpu:
        oa, ow = ctx.oracle().quantize(cfg["A"]), ctx.oracle().quantize(cfg["W"])
        o = {"oracle_s": ctx.oracle_seconds(lambda: ctx.oracle().gemm(oa, ow))}
    res["gemm_128x256x256"] = gemm_row(s, 2.0 * 128 * 256 * 256, o)


def _oracle_gemm(ctx, oa, ow, n_rows=512, seed=0):
    """Oracle GEMM on n_rows seeded rows, all columns; the full-size time is that, scaled by M / rows."""
    if not ctx.with_cpu:
        return None
    rows = ctx.np.unique(ctx.np.random.default_rng(seed).integers(0, oa.rows, n_rows)).astype(ctx.np.int64)
    t = ctx.oracle_seconds(lambda: ctx.oracle().gemm(oa, ow, rows=rows, want_abs=False))
    return {"oracle_s_extrapolated": round(t * oa.rows / len(rows), 2), "oracle_rows_timed": int(len(rows)), "oracle_s_rows": t}


def _rows_proj(ctx, res, ws):
    """Config 2: the single DiT projection, activations quantized per call, weights once."""
    nv, wl, torch = ctx.nv, ctx.wl, ctx.torch
    c2 = wl.config2()
    M, D = wl.TOKENS_INFER, wl.D_MODEL
    X = nv.bf16_from_bits(c2["A"], "cuda")
    qW = nv.nvfp4_quantize(nv.bf16_from_bits(c2["W"], "cuda"))
    nc = copies_for(2 * M * D)
    xs = [X.clone() for _ in range(nc)]
    qs = [nv.NVFP4Tensor(M, D, "cuda") for _ in range(nc)]
    s = ctx.time_op(nv.OP_QUANTIZE, lambda i: nv.nvfp4_quantize(xs[i % nc], out=qs[i % nc], workspace=ws), 3 * nc)
    res["quantize_A_3520x3072"] = bw_row(s, B_PER_ELEM * M * D, ctx.oracle_seconds(lambda: ctx.oracle().quantize(c2["A"])), nc)
    Y = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
    o = None
    if ctx.with_cpu:
        oa, ow = ctx.oracle().quantize(c2["A"]), ctx.oracle().quantize(c2["W"])
        o = {"oracle_s": ctx.oracle_seconds(lambda: ctx.oracle().gemm(oa, ow, want_abs=False))}
    s = ctx.time_op(nv.OP_GEMM, lambda i: nv.nvfp4_gemm(qs[0], qW, nv.OUT_BF16, Y=Y), 30, warm=10)
    res["gemm_3520x3072x3072_bf16_out"] = gemm_row(s, 2.0 * M * D * D, o)


def _rows_kv(ctx, res, ws):
    nv, wl, torch, np = ctx.nv, ctx.wl, ctx.torch, ctx.np
    dev = "cuda"
    # --- KV cache: K [18480, 24, 128] -------------------------------------------------------
    T, H, d = wl.KV_TOKENS, wl.KV_HEADS, wl.KV_DIM
    kb = wl.kv_tensor(T, H, d, 3, 0)
    n = T * H * d
    nc = copies_for(2 * n)
    kvs = [nv.bf16_from_bits(kb, dev) for _ in range(nc)]
    qs = [nv.NVFP4Tensor(T * H, d, dev) for _ in range(nc)]
    backs = [torch.empty_like(kvs[0]) for _ in range(nc)]
    means = [torch.empty(T * H, dtype=torch.bfloat16, device=dev) for _ in range(nc)]
    it = 4 * nc
    ora = ctx.oracle() if ctx.with_cpu else None
    k2 = kb.reshape(T * H, d)
    s = ctx.time_op(nv.OP_KV_QUANT, lambda i: nv.nvfp4_kv_quant(kvs[i % nc], out=qs[i % nc], workspace=ws), it)
    res["kv_quant_18480x24x128"] = bw_row(s, B_PER_ELEM * n, ctx.oracle_seconds(lambda: ora.quantize(k2)), nc)
    # values whose tensor scale the producing GEMM already supplied (nvfp4_gemm_scale_out on the V projection): the
    # same bytes through the given-scale quantizer, one streaming pass and no maximum to wait for
    gs = torch.tensor([float(np.float32(np.abs(wl.bf16_bits_to_f32(kb)).max()) / np.float32(2688.0))], dtype=torch.float32, device=dev)
    s = ctx.time_op(nv.OP_QUANTIZE, lambda i: nv.nvfp4_quantize(kvs[i % nc].view(T * H, d), global_scale_in=gs, out=qs[i % nc], workspace=ws), it)
    res["kv_quant_given_scale_18480x24x128"] = bw_row(
        s, B_PER_ELEM * n, ctx.oracle_seconds(lambda: ora.quantize(k2, global_scale_in=float(gs.cpu()[0]))), nc)
    # the same cache with the Four-over-Six scale search (the variant the paper applies to the cache)
    s = ctx.time_op(nv.OP_KV_QUANT_4OVER6, lambda i: nv.nvfp4_kv_quant_4over6(kvs[i % nc], out=qs[i % nc], workspace=ws), it)
    res["kv_quant_4over6_18480x24x128"] = bw_row(s, B_PER_ELEM * n, ctx.oracle_seconds(lambda: ora.quantize(k2, four_over_six=True)), nc)
    # keys as the paper caches them: row means removed (K-smoothing), then the scale search
    s = ctx.time_op(nv.OP_KV_QUANT_K, lambda i: nv.nvfp4_kv_quant_k(kvs[i % nc], out=qs[i % nc], row_mean=means[i % nc], workspace=ws), it)
    res["kv_quant_k_smooth_4over6_18480x24x128"] = bw_row(
        s, B_PER_ELEM * n, ctx.oracle_seconds(lambda: ora.quantize(ora.kv_smooth(k2)[1], four_over_six=True)), nc)
    # plain reconstruction of the whole window
    for i in range(nc):
        nv.nvfp4_kv_quant(kvs[i], out=qs[i], workspace=ws)
    oq = ora.quantize(k2) if ctx.with_cpu else None
    s = ctx.time_op(nv.OP_KV_DEQUANT, lambda i: nv.nvfp4_kv_dequant(qs[i % nc], T, H, d, out=backs[i % nc]), it)
    res["kv_dequant_18480x24x128"] = bw_row(s, B_PER_ELEM * n, ctx.oracle_seconds(lambda: ora.dequant_bf16(oq)), nc)
    # gathered reconstruction of a window of 21 chunks of 880 tokens (one launch), plain and smoothed
    Tc = 880
    sets_v, sets_k = [], []
    for c in range(nc):
        cv, ck = [], []
        for j in range(T // Tc):
            part = kvs[c][j * Tc:(j + 1) * Tc]
            cv.append((nv.nvfp4_kv_quant(part), None, Tc))
            qk, mk = nv.nvfp4_kv_quant_k(part)
            ck.append((qk, mk, Tc))
        sets_v.append(cv)
        sets_k.append(ck)
    s = ctx.time_op(nv.OP_KV_DEQUANT_GATHER, lambda i: nv.nvfp4_kv_dequant_gather(sets_v[i % nc], H, d, out=backs[i % nc]), it)
    res["kv_dequant_gather_21x880x24x128"] = bw_row(s, B_PER_ELEM * n, None, nc)
    s = ctx.time_op(nv.OP_KV_DEQUANT_GATHER, lambda i: nv.nvfp4_kv_dequant_gather(sets_k[i % nc], H, d, out=backs[i % nc]), it)
    om = None
    if ctx.with_cpu:
        m_, xbar = ora.kv_smooth(k2)
        oqk = ora.quantize(xbar, four_over_six=True)
        om = ctx.oracle_seconds(lambda: ora.dequant_bf16(oqk, m_))
    res["kv_dequant_gather_smoothed_21x880x24x128"] = bw_row(s, B_PER_ELEM * n, om, nc)
    del sets_v, sets_k
    # send buffers of the NVFP4 all-to-all: one device's share of that window among 4 (L/P = 4620 tokens),
    # cast along d and regrouped into 4 per-destination slabs of 6 heads
    P = 4
    Tl = T // P
    n_l = Tl * H * d
    nca = copies_for(2 * n_l)
    srcs = [kvs[i % nc][(i // nc % P) * Tl:(i // nc % P + 1) * Tl] for i in range(nca)]
    q_a2a = [nv.NVFP4Tensor(Tl * H, d, dev) for _ in range(nca)]
    s = ctx.time_op(nv.OP_QUANTIZE_A2A, lambda i: nv.nvfp4_quantize_for_all_to_all(srcs[i % nca], P, out=q_a2a[i % nca], workspace=ws), 3 * nca)
    res[f"quantize_for_all_to_all_{Tl}x{H}x{d}_P{P}"] = bw_row(
        s, B_PER_ELEM * n_l, ctx.oracle_seconds(lambda: ora.quantize(k2[:Tl * H])), nca)


def _rows_lora(ctx, res, ws):
    nv, wl, torch = ctx.nv, ctx.wl, ctx.torch
    dev = "cuda"
    # --- LoRA side branch on the DiT projection (rank 128, alpha 128): bf16 down projection, then the
    # quantized GEMM with the low-rank update fused in, against the plain quantized GEMM ------------
    c2 = wl.config2()
    Mi, Dm = wl.TOKENS_INFER, wl.D_MODEL
    Xi = nv.bf16_from_bits(c2["A"], dev)
    qXi, qWi = nv.nvfp4_quantize(Xi), nv.nvfp4_quantize(nv.bf16_from_bits(c2["W"], dev))
    la_bits, lb_bits = wl.normal((nv.LORA_RANK, Dm), 0.02, 1, 7), wl.normal((Dm, nv.LORA_RANK), 0.02, 1, 8)
    La, Lb = nv.bf16_from_bits(la_bits, dev), nv.bf16_from_bits(lb_bits, dev)
    Tl = torch.empty((Mi, nv.LORA_RANK), dtype=torch.bfloat16, device=dev)
    Yl = torch.empty((Mi, Dm), dtype=torch.bfloat16, device=dev)
    fl = 2.0 * Mi * Dm * Dm
    wsl = torch.empty(nv.nvfp4_workspace_bytes(nv.OP_LORA_DOWN, Mi, Dm), dtype=torch.uint8, device=dev)
    s = ctx.time_op(nv.OP_LORA_DOWN, lambda i: nv.nvfp4_lora_down(Xi, La, out=Tl, workspace=wsl), 20)
    o = {"oracle_s": ctx.oracle_seconds(lambda: ctx.oracle().lora_down(c2["A"], la_bits))} if ctx.with_cpu else None
    res["lora_down_3520x3072_r128"] = gemm_row(s, 2.0 * Mi * Dm * nv.LORA_RANK, o)
    s = ctx.time_op(nv.OP_GEMM_LORA, lambda i: nv.nvfp4_gemm_lora(qXi, qWi, Tl, Lb, 1.0, nv.OUT_BF16, Y=Yl), 20, warm=10)
    res["gemm_lora_fused_3520x3072x3072"] = gemm_row(s, fl + 2.0 * Mi * Dm * nv.LORA_RANK)
    s = ctx.time_op(nv.OP_GEMM, lambda i: nv.nvfp4_gemm(qXi, qWi, nv.OUT_BF16, Y=Yl), 20, warm=10)
    res["gemm_plain_3520x3072x3072"] = gemm_row(s, fl)


def _rows_train(ctx, res, ws):
    nv, wl, torch, np = ctx.nv, ctx.wl, ctx.torch, ctx.np
    dev = "cuda"
    # --- training triplet: X[17600,3072], W[14336,3072], dY[17600,14336] ---------------------
    c5 = wl.config5()
    Mt, D, F = wl.TOKENS_TRAIN, wl.D_MODEL, wl.D_FFN
    ora = ctx.oracle() if ctx.with_cpu else None
    host = {"X": c5["X"], "W": c5["W"], "dY": c5["dY"]}
    devs = {}
    for k, bits in host.items():
        nc = copies_for(bits.size * 2)
        devs[k] = [nv.bf16_from_bits(bits, dev) for _ in range(nc)]
    kept, okept = {}, {}

    def qtime(name, axis, row_name):
        xs = devs[name]
        nc = len(xs)
        R, C = xs[0].shape
        rows, K = (R, C) if axis == 0 else (C, R)
        outs = [nv.NVFP4Tensor(rows, K, dev) for _ in range(nc)]
        s = ctx.time_op(nv.OP_QUANTIZE, lambda i: nv.nvfp4_quantize(xs[i % nc], block_axis=axis, out=outs[i % nc], workspace=ws), 4 * nc)
        osec = None
        if ctx.with_cpu:
            t0 = time.perf_counter()
            okept[(name, axis)] = ora.quantize(host[name], block_axis=axis)
            osec = round(time.perf_counter() - t0, 3)
        res[row_name] = bw_row(s, B_PER_ELEM * R * C, osec, nc)
        kept[(name, axis)] = outs[0]

    qtime("X", 0, "quantize_X_17600x3072")
    qtime("dY", 0, "quantize_dY_17600x14336")
    qtime("W", 0, "quantize_W_14336x3072")
    qtime("W", 1, "quantize_T_W_14336x3072")
    qtime("dY", 1, "quantize_T_dY_17600x14336")
    qtime("X", 1, "quantize_T_X_17600x3072")
    dYs, Ws = devs["dY"], devs["W"]
    ncd, ncw = len(dYs), len(Ws)
    # weight-gradient operand with the random Hadamard transform in front of the transposed quantizer
    qrht = [nv.NVFP4Tensor(F, Mt, dev) for _ in range(ncd)]
    ws_rht = ctx.torch.empty(nv.nvfp4_workspace_bytes(nv.OP_QUANTIZE_RHT, Mt, F), dtype=ctx.torch.uint8, device="cuda")
    s = ctx.time_op(nv.OP_QUANTIZE_RHT, lambda i: nv.nvfp4_quantize_rht(dYs[i % ncd], 0x9A3C, out=qrht[i % ncd], workspace=ws_rht), 3 * ncd)
    res["quantize_rht_T_dY_17600x14336"] = bw_row(
        s, B_PER_ELEM * Mt * F, ctx.oracle_seconds(lambda: ora.quantize(ora.rht_rows(host["dY"], 0x9A3C), block_axis=1)), ncd)
    del qrht, ws_rht
    # the scale search on the activations
    q46 = [nv.NVFP4Tensor(Mt, D, dev) for _ in range(len(devs["X"]))]
    ncx = len(q46)
    s = ctx.time_op(nv.OP_QUANTIZE_4OVER6, lambda i: nv.nvfp4_quantize_4over6(devs["X"][i % ncx], out=q46[i % ncx], workspace=ws), 4 * ncx)
    res["quantize_4over6_X_17600x3072"] = bw_row(s, B_PER_ELEM * Mt * D, ctx.oracle_seconds(lambda: ora.quantize(host["X"], four_over_six=True)), ncx)
    del q46
    # weights with one scale per 16x16 tile: W and W^T from one pass (2.5625 B/element per operand written)
    s = ctx.time_op(nv.OP_QUANTIZE_2D, lambda i: nv.nvfp4_quantize_2d(Ws[i % ncw], workspace=ws), 4 * ncw)
    res["quantize_2d_W_and_WT_14336x3072"] = bw_row(s, (2.0 + 2 * 0.5625) * F * D, ctx.oracle_seconds(lambda: ora.quantize_2d(host["W"])), ncw)
    gs = kept[("dY", 0)].global_scale.clone()
    outs = [nv.NVFP4Tensor(Mt, F, dev) for _ in range(ncd)]
    s = ctx.time_op(nv.OP_QUANTIZE, lambda i: nv.nvfp4_quantize(dYs[i % ncd], global_scale_in=gs, out=outs[i % ncd], workspace=ws), 4 * ncd)
    res["quantize_dY_given_scale"] = bw_row(s, B_PER_ELEM * Mt * F, None, ncd)
    # dY along both axes (dgrad needs it along N, wgrad along the tokens): the second call takes the first one's scale
    o_c = [nv.NVFP4Tensor(F, Mt, dev) for _ in range(ncd)]

    def both(i):
        nv.nvfp4_quantize(dYs[i % ncd], out=outs[i % ncd], workspace=ws)
        nv.nvfp4_quantize(dYs[i % ncd], block_axis=1, global_scale_in=outs[i % ncd].global_scale, out=o_c[i % ncd], workspace=ws)

    s = ctx.time_op(nv.OP_QUANTIZE, both, 3 * ncd)
    pairs = [a + b for a, b in zip(s[0::2], s[1::2])]               # two recorded calls per pair
    res["quantize_dY_both_axes_shared_scale"] = bw_row(pairs, (2 + 2 * 0.5625) * Mt * F, None, ncd)
    del o_c, outs, devs, dYs, Ws
    torch.cuda.empty_cache()

    def gtime(a, b, name, out_dtype=nv.OUT_F32, seed=0):
        ga, gb = kept[a], kept[b]
        y = torch.empty((ga.rows, gb.rows), dtype=torch.float32 if out_dtype == nv.OUT_F32 else torch.bfloat16, device=dev)
        s = ctx.time_op(nv.OP_GEMM, lambda i: nv.nvfp4_gemm(ga, gb, out_dtype, Y=y), 12, warm=4)
        o = _oracle_gemm(ctx, okept[a], okept[b], 512, seed) if (ctx.with_cpu and out_dtype == nv.OUT_F32) else None
        res[name] = gemm_row(s, 2.0 * ga.rows * gb.rows * ga.K, o)

    # fp32 outputs (the accumulator as it is); activations and their gradients also as bf16
    gtime(("X", 0), ("W", 0), "fprop_17600x14336x3072")
    gtime(("dY", 0), ("W", 1), "dgrad_17600x3072x14336")
    gtime(("dY", 1), ("X", 1), "wgrad_14336x3072x17600")
    gtime(("X", 0), ("W", 0), "fprop_17600x14336x3072_bf16_out", nv.OUT_BF16)
    gtime(("dY", 0), ("W", 1), "dgrad_17600x3072x14336_bf16_out", nv.OUT_BF16)
    # the same fprop returning the NVFP4 tensor scale of its [17600, 14336] output from the epilogue: what a quantizer
    # of that output then takes as given (row quantize_dY_given_scale is that call at this size), instead of an amax pass
    ga, gb = kept[("X", 0)], kept[("W", 0)]
    y = torch.empty((ga.rows, gb.rows), dtype=torch.bfloat16, device=dev)
    sc = torch.empty(1, dtype=torch.float32, device=dev)
    wsg = torch.empty(nv.nvfp4_workspace_bytes(nv.OP_GEMM_SCALE_OUT, ga.rows, gb.rows), dtype=torch.uint8, device=dev)
    s = ctx.time_op(nv.OP_GEMM_SCALE_OUT, lambda i: nv.nvfp4_gemm_scale_out(ga, gb, Y=y, scale_out=sc, workspace=wsg), 12, warm=4)
    res["fprop_17600x14336x3072_bf16_out_plus_tensor_scale"] = gemm_row(s, 2.0 * ga.rows * gb.rows * ga.K)


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
