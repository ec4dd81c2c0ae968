#!/usr/bin/env python3
"""Benchmark of the SQuat key-quantization hot path on one MI355X.

One step = one pass of the whole path over the long-context workload (32 layers x 8 KV heads
stacked along the head axis, 32768 tokens per layer, d = 128, bf16, r = 32, 2-bit, group 32):
  squat_build_subspace -> squat_prepare -> squat_quantize_keys -> squat_dequantize_keys.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0


def cpu_baseline(wl_args: dict, heads: int = 4, repeats: int = 8):
    """The float64 oracle, as it stands, on a bounded sample of the same workload: `heads` KV heads
    (pooled queries of 4 query heads each, all their tokens)."""
    import numpy as np
    from oracle import squat_oracle as O
    from paper_2503_24358_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    n, r, lam, bits, G, g = (wl_args[k] for k in ("n_tokens", "r", "lam", "bits", "group", "g"))
    qpk = wl_args["q_per_kv"]
    _, qval = synth.store(synth.queries(77, heads * qpk, n), synth.BF16)
    _, kval = synth.store(synth.keys(78, heads, n), synth.BF16)
    t0 = time.perf_counter()
    for _ in range(repeats):
        for h in range(heads):
            Qh, _ = O.subspace(qval[h * qpk:(h + 1) * qpk], r)
            U = O.update_matrix_lemma(Qh, lam, g)
            out = O.quantize_keys(kval[h], U, bits, G, g)
            O.dequantize_keys(out["codes"], out["scale"], out["zero"], G)
    dt = time.perf_counter() - t0

    def one_pass():
        for h in range(heads):
            Qh, _ = O.subspace(qval[h * qpk:(h + 1) * qpk], r)
            U = O.update_matrix_lemma(Qh, lam, g)
            out = O.quantize_keys(kval[h], U, bits, G, g)
            O.dequantize_keys(out["codes"], out["scale"], out["zero"], G)

    single = None
    try:                                            # the same oracle with the BLAS / OpenMP pools held to one thread
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            t1 = time.perf_counter()
            one_pass()
            single = heads * n / (time.perf_counter() - t1)
    except Exception:
        pass
    model = None
    try:
        with open("/proc/cpuinfo") as f:
            model = [ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")][0]
    except Exception:
        pass
    return {"value": repeats * heads * n / dt, "unit": "keys/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d KV heads x %d tokens (pooled queries of %d query heads each), whole path, "
                      "%d passes, %.1f s" % (heads, n, qpk, repeats, dt),
            "value_one_thread": single, "cpu_model": model, "cpu_count": os.cpu_count()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--tokens", type=int, default=32768)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variants", action="store_true",
                    help="also time the quantize and dequantize kernels for the other bit widths / group sizes "
                         "of the long-context configuration (adds a \"variants\" list to the JSON line)")
    ap.add_argument("--decode", action="store_true",
                    help="also time the decode-time flush shape (64 sequences, 32 buffered tokens per head): one "
                         "layer (8 heads) per launch and all 32 layers (256 heads) per launch (adds \"decode_flush\")")
    ap.add_argument("--per-layer", action="store_true",
                    help="also run the whole path with one launch per stage and LAYER (8 KV heads per launch instead of "
                         "all 256 stacked), launched eagerly and replayed from a HIP graph (adds \"per_layer\")")
    ap.add_argument("--with-copy", action="store_true",
                    help="profiling aid: also run one plain device copy of the key tensor (known size) per step, "
                         "to calibrate the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--only", default="", help="profiling aid: time only this stage (e.g. quantize_keys); "
                                               "the other stages run once, untimed, to prepare its inputs")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (heads/layers would shard without communication); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_24358_amd import squat
    from paper_2503_24358_amd.workload import LongContext

    if not torch.cuda.is_available():
        print("bench.py needs the GPU (there is no CPU fallback)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    wl = LongContext(layers=args.layers, n_tokens=args.tokens)
    H, n, d = wl.heads, wl.n_tokens, wl.d
    dev = wl.device

    # every buffer is allocated once, outside the timed region
    qhat = torch.empty((H, wl.r, d), dtype=torch.float32, device=dev)
    eig = torch.empty((H, wl.r), dtype=torch.float32, device=dev)
    ws_sub = torch.empty(squat.build_subspace_workspace(n, H, wl.q_per_kv, d, wl.r), dtype=torch.uint8, device=dev)
    update = torch.empty((H, d, d), dtype=torch.float32, device=dev)
    ws_prep = torch.empty(max(256, squat.prepare_workspace(H, d, wl.r, wl.g)), dtype=torch.uint8, device=dev)
    codes = torch.empty((1, H, n, d * wl.bits // 32), dtype=torch.int32, device=dev)
    scale = torch.empty((1, H, n, d // wl.group), dtype=torch.float16, device=dev)
    zero = torch.empty((1, H, n, d // wl.group), dtype=torch.float16, device=dev)
    back = torch.empty((1, H, n, d), dtype=torch.bfloat16, device=dev)

    stages = ("build_subspace", "prepare", "quantize_keys", "dequantize_keys")

    only = args.only

    def step(ev=None, everything=False):
        run = lambda name: everything or not only or only == name  # noqa: E731
        if ev: ev[0].record()
        if run("build_subspace"):
            squat.build_subspace(wl.q, wl.q_per_kv, wl.r, qhat=qhat, eig=eig, ws=ws_sub)
        if ev: ev[1].record()
        if run("prepare"):
            squat.prepare(qhat, wl.lam, wl.g, update=update, ws=ws_prep)
        if ev: ev[2].record()
        if run("quantize_keys"):
            squat.quantize_keys(wl.k, update, wl.bits, wl.group, wl.g, codes=codes, scale=scale, zero=zero)
        if ev: ev[3].record()
        if run("dequantize_keys"):
            squat.dequantize_keys(codes, scale, zero, wl.bits, wl.group, out=back)
        if ev: ev[4].record()
        if args.with_copy:
            back.copy_(wl.k)          # 2 x keys x 256 B through a plain elementwise copy kernel

    step(everything=True)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {}
    stage_ms_median, stage_ms_min = {}, {}
    for s, name in enumerate(stages):
        ts = sorted(ev[s].elapsed_time(ev[s + 1]) for ev in events)
        stage_ms[name] = sum(ts) / args.steps
        stage_ms_median[name] = ts[len(ts) // 2]
        stage_ms_min[name] = ts[0]

    n_keys = wl.n_keys
    # roofline of the dominant bandwidth kernel, the quantize pass: algorithmic bytes = keys x (256 B in +
    # 32 B codes + 16 B scale/zero); duration = HIP-event time around its single launch
    q_ms = stage_ms["quantize_keys"]
    q_bytes = n_keys * wl.key_bytes()
    achieved = q_bytes / (q_ms * 1e-3) / 1e9
    roofline = {"kernel": "quantize_kernel<2-bit,G32,g32,bf16>", "bound": "hbm", "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                # FETCH_SIZE + WRITE_SIZE of this kernel from rocprofv3 --pmc, scaled by a plain copy of known
                # size (profiles/quantize_kernel_long_context_hbm_traffic.txt); measured at the default workload
                "traffic": 2.5629e9 if (args.layers == 32 and args.tokens == 32768) else None,
                "bytes_per_launch": q_bytes, "ms_per_launch": q_ms,
                # embedded contraction: 12288 flop per key at g = 32, two fp16 passes (update matrix on the fp16 grid)
                "mfma_tflops": n_keys * 12288 * 2 / (q_ms * 1e-3) / 1e12,
                "mfma_frac_of_fp16_peak": n_keys * 12288 * 2 / (q_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    d_ms = stage_ms["dequantize_keys"]
    gram_bytes = wl.q.numel() * 2
    other = {
        "dequantize_keys": {"bound": "hbm", "achieved": q_bytes / (d_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                            "unit": "GB/s", "frac": q_bytes / (d_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "build_subspace": {"ms": stage_ms["build_subspace"], "gram_input_GB": gram_bytes / 1e9,
                           "note": "gram (HBM-bound bf16 MFMA, see profiles/) + fp64 eigen-solver, one workgroup per "
                                   "head (Householder tridiagonalisation, bisection, inverse iteration; latency-bound)"},
        "prepare": {"ms": stage_ms["prepare"]},
    }
    out = {
        "metric": "keys quantized/sec (tokens x KV-heads), whole path, 2-bit d=128",
        "value": n_keys / (ms_per_step * 1e-3), "unit": "keys/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "only_stage": only or None,
        "config": {"workload": "long-context: %d layers x %d KV heads (x%d query heads), %d tokens/layer, d=128, "
                               "bf16 in, r=%d, lambda=%g, %d-bit, group %d, g=%d; layers stacked along the head axis, "
                               "one launch per stage" % (wl.layers, wl.kv_heads, wl.q_per_kv, n, wl.r, wl.lam,
                                                         wl.bits, wl.group, wl.g),
                   "keys_per_step": n_keys},
        "stage_ms": stage_ms, "stage_ms_median": stage_ms_median, "stage_ms_min": stage_ms_min,
        "quantize_keys_per_s": n_keys / (q_ms * 1e-3),
        "roofline": roofline,
        "other_kernels": other,
    }
    def timed(fn, reps=5):
        fn()
        fn()
        torch.cuda.synchronize()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        evs[0].record()
        for i in range(reps):
            fn()
            evs[i + 1].record()
        torch.cuda.synchronize()
        return sum(evs[i].elapsed_time(evs[i + 1]) for i in range(reps)) / reps

    # The machine, and a practical ceiling measured beside the vendor peak: a plain elementwise device copy
    # of the key tensor (reads and writes keys x 256 B each).
    props = torch.cuda.get_device_properties(0)

    def max_clock_mhz():
        # rocminfo's "Max Clock Freq. (MHz)" of the first GPU agent (the torch properties do not carry it)
        try:
            import subprocess
            txt = subprocess.run(["/opt/rocm/bin/rocminfo"], capture_output=True, text=True, timeout=20).stdout
            gpu = txt[txt.index("Device Type:             GPU"):]
            line = [ln for ln in gpu.splitlines() if "Max Clock Freq. (MHz)" in ln][0]
            return int(line.split(":")[1])
        except Exception:
            return None
    t_copy = timed(lambda: back.copy_(wl.k.view_as(back)))
    out["device"] = {"name": props.name, "compute_units": props.multi_processor_count,
                     "max_clock_mhz": max_clock_mhz(),
                     "hbm_GiB": props.total_memory / 2 ** 30,
                     "device_copy_GBps": 2 * n_keys * d * 2 / (t_copy * 1e-3) / 1e9}
    roofline["frac_of_device_copy"] = achieved / out["device"]["device_copy_GBps"]

    # The paper's own grouping (statistics per channel over 32 tokens): same keys, same update matrix, the
    # per-channel entry points; the headline variant always, the others with --variants.
    pc_list = [(2, 32, True)]
    if args.variants:
        pc_list += [(2, 64, True), (4, 32, True), (4, 64, True), (2, 128, False)]
    out["per_channel"] = []
    qdec = wl.q[:, n - 1, :].unsqueeze(0).contiguous()                      # [1, q_heads, d]: the last prompt token's queries
    logits = torch.empty((1, H * wl.q_per_kv, n), dtype=torch.float32, device=dev)
    inv_freq = (10000.0 ** (-torch.arange(64, dtype=torch.float64, device=dev) / 64.0)).float()
    for bits, g, use_update in pc_list:
        upd = (update if g == wl.g else squat.prepare(qhat, wl.lam, g)) if use_update else None
        c = torch.empty((1, H, n // 32, d, bits), dtype=torch.int32, device=dev)
        sc = torch.empty((1, H, n // 32, d), dtype=torch.float16, device=dev)
        ze = torch.empty_like(sc)
        tq = timed(lambda: squat.quantize_keys_per_channel(wl.k, upd, bits, 32, g, codes=c, scale=sc, zero=ze))
        td = timed(lambda: squat.dequantize_keys_per_channel(c, sc, ze, bits, 32, out=back))
        tsc = timed(lambda: squat.key_scores_per_channel(qdec, c, sc, ze, bits, wl.q_per_kv, d ** -0.5, out=logits), reps=10)
        # the same store read as pre-RoPE keys (rotation after dequantization: the paper's SQuat-pre on its own grouping)
        tsr = timed(lambda: squat.key_scores_rope_per_channel(qdec, c, sc, ze, bits, wl.q_per_kv, inv_freq, 0, d ** -0.5,
                                                              out=logits), reps=10)
        nbytes = n_keys * (d * 2 + d * bits // 8 + 4 * (d // 32))
        sb = n_keys * (d * bits // 8 + 4 * (d // 32) + 4 * wl.q_per_kv)
        # the whole path with this grouping in place of the per-token one (subspace and update as in `step`): the
        # kernel's time between the other stages, not back to back with itself
        in_step = None
        if use_update and g == wl.g and not only:
            def step_pc(ev=None):
                squat.build_subspace(wl.q, wl.q_per_kv, wl.r, qhat=qhat, eig=eig, ws=ws_sub)
                squat.prepare(qhat, wl.lam, wl.g, update=update, ws=ws_prep)
                if ev: ev[0].record()
                squat.quantize_keys_per_channel(wl.k, update, bits, 32, g, codes=c, scale=sc, zero=ze)
                if ev: ev[1].record()
                squat.dequantize_keys_per_channel(c, sc, ze, bits, 32, out=back)
                if ev: ev[2].record()
            for _ in range(max(1, args.warmup)):
                step_pc()
            torch.cuda.synchronize()
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
            t0 = time.perf_counter()
            for i in range(args.steps):
                step_pc(evs[i])
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / args.steps
            tq_in = sorted(e[0].elapsed_time(e[1]) for e in evs)
            td_in = sorted(e[1].elapsed_time(e[2]) for e in evs)
            in_step = {"ms_per_step": ms, "keys_per_s": n_keys / (ms * 1e-3),
                       "quantize_us_mean": sum(tq_in) / len(tq_in) * 1e3, "quantize_us_median": tq_in[len(tq_in) // 2] * 1e3,
                       "quantize_frac_of_hbm_peak": nbytes / (sum(tq_in) / len(tq_in) * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "dequantize_us_mean": sum(td_in) / len(td_in) * 1e3}
        out["per_channel"].append({"bits": bits, "token_group": 32, "g": g, "update": use_update,
                                   "bytes_per_key": nbytes // n_keys,
                                   "quantize_us": tq * 1e3, "quantize_frac_of_hbm_peak": nbytes / (tq * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                   "dequantize_us": td * 1e3, "dequantize_frac_of_hbm_peak": nbytes / (td * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                   "key_scores_us": tsc * 1e3, "key_scores_bytes_per_key": sb // n_keys,
                                   "key_scores_frac_of_hbm_peak": sb / (tsc * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                   "whole_path": in_step,
                                   "key_scores_rope_us": tsr * 1e3,
                                   "key_scores_rope_frac_of_hbm_peak": sb / (tsr * 1e-3) / 1e9 / HBM_PEAK_GBS})
    # Decode-side consumer: attention logits of one query token per query head straight from the packed
    # store just written (48 B of codes and metadata in, 4 B per query head out, per key).
    ts = timed(lambda: squat.key_scores(qdec, codes, scale, zero, wl.bits, wl.group, wl.q_per_kv, d ** -0.5, out=logits), reps=10)
    sbytes = n_keys * (d * wl.bits // 8 + 4 * (d // wl.group) + 4 * wl.q_per_kv)
    out["key_scores"] = {"bits": wl.bits, "group": wl.group, "q_per_kv": wl.q_per_kv, "bytes_per_key": sbytes // n_keys,
                         "us": ts * 1e3, "keys_per_s": n_keys / (ts * 1e-3),
                         "frac_of_hbm_peak": sbytes / (ts * 1e-3) / 1e9 / HBM_PEAK_GBS}
    # the pre-RoPE variant of the same consumer: keys dequantized, rotated to their positions and rounded to
    # fp16 in registers before the contraction (bound by vector arithmetic, not by HBM)
    tr = timed(lambda: squat.key_scores_rope(qdec, codes, scale, zero, wl.bits, wl.group, wl.q_per_kv, inv_freq, 0,
                                             d ** -0.5, out=logits), reps=10)
    out["key_scores_rope"] = {"bits": wl.bits, "group": wl.group, "q_per_kv": wl.q_per_kv, "bound": "alu", "us": tr * 1e3,
                              "keys_per_s": n_keys / (tr * 1e-3), "frac_of_hbm_peak": sbytes / (tr * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "valu_instructions_per_16_keys": 300,
                              # 300 wave64 instructions per 16 keys (main loop of the built kernel) = 1200 lane-operations per key; peak: 256 CUs x 4 SIMDs
                              # x 16 lanes x 2.4 GHz (packed fp32 is switched off in this build)
                              "alu_lane_ops_per_s": n_keys / (tr * 1e-3) * 1200,
                              "alu_peak_lane_ops_per_s": 256 * 4 * 16 * 2.4e9,
                              "alu_frac": n_keys / (tr * 1e-3) * 1200 / (256 * 4 * 16 * 2.4e9)}
    if args.variants:
        out["variants"] = []
        for bits, G, g, use_update in [(2, 32, 32, True), (2, 32, 64, True), (4, 32, 32, True), (4, 32, 64, True),
                                       (2, 128, 32, True), (4, 128, 32, True), (2, 128, 64, True),
                                       (2, 32, 128, False), (2, 128, 128, False), (4, 128, 128, False)]:
            upd = squat.prepare(qhat, wl.lam, g) if use_update else None
            c = torch.empty((1, H, n, d * bits // 32), dtype=torch.int32, device=dev)
            sc = torch.empty((1, H, n, d // G), dtype=torch.float16, device=dev)
            ze = torch.empty_like(sc)
            tq = timed(lambda: squat.quantize_keys(wl.k, upd, bits, G, g, codes=c, scale=sc, zero=ze))
            td = timed(lambda: squat.dequantize_keys(c, sc, ze, bits, G, out=back))
            nbytes = n_keys * (d * 2 + d * bits // 8 + 4 * (d // G))
            out["variants"].append({"bits": bits, "group": G, "g": g, "update": use_update,
                                    "bytes_per_key": nbytes // n_keys,
                                    "quantize_us": tq * 1e3, "quantize_frac_of_hbm_peak": nbytes / (tq * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                    "dequantize_us": td * 1e3, "dequantize_frac_of_hbm_peak": nbytes / (td * 1e-3) / 1e9 / HBM_PEAK_GBS})
    if args.decode:
        def timed_us(fn, reps=50):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps
        out["decode_flush"] = []
        for heads in (wl.kv_heads, H):
            kb = torch.randn((64, heads, 32, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
            c = torch.empty((64, heads, 32, d * wl.bits // 32), dtype=torch.int32, device=dev)
            sc = torch.empty((64, heads, 32, d // wl.group), dtype=torch.float16, device=dev)
            ze = torch.empty_like(sc)
            us = timed_us(lambda: squat.quantize_keys(kb, update[:heads], wl.bits, wl.group, wl.g, codes=c, scale=sc, zero=ze))
            nk = 64 * heads * 32
            out["decode_flush"].append({"sequences": 64, "heads_per_launch": heads, "keys_per_flush": nk,
                                        "us_per_flush_back_to_back": us, "keys_per_s": nk / (us * 1e-6)})
        # logits of 64 sequences x all (layer, KV head) slots over 2048 quantized tokens each
        nd = 2048
        cd = torch.randint(-2 ** 31, 2 ** 31 - 1, (64, H, nd, d * wl.bits // 32), dtype=torch.int32, device=dev)
        sd = torch.rand((64, H, nd, d // wl.group), device=dev).half()
        zd = torch.randn((64, H, nd, d // wl.group), device=dev).half()
        qd = torch.randn((64, H * wl.q_per_kv, d), device=dev, dtype=torch.bfloat16)
        ld = torch.empty((64, H * wl.q_per_kv, nd), dtype=torch.float32, device=dev)
        us = timed_us(lambda: squat.key_scores(qd, cd, sd, zd, wl.bits, wl.group, wl.q_per_kv, d ** -0.5, out=ld), reps=10)
        nk = 64 * H * nd
        nb = nk * (d * wl.bits // 8 + 4 * (d // wl.group) + 4 * wl.q_per_kv)
        # the same shape through the cache object: 64 decode steps (append one token per sequence, then
        # logits over everything cached); two of the 64 appends flush a full residual buffer.  Once with
        # keys grouped per token, once per channel over the 32 flushed tokens (the paper's grouping).
        kp = torch.randn((64, H, nd, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
        knew = torch.randn((64, H, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
        lc = torch.empty((64, H * wl.q_per_kv, nd + 64), dtype=torch.float32, device=dev)
        for name, per_channel in (("decode_cache", False), ("decode_cache_per_channel", True)):
            cache = squat.Cache(64, H, wl.q_per_kv, wl.bits, wl.group, wl.g, 32, nd + 64, kv_dtype=torch.bfloat16,
                                update=update, key_per_channel=per_channel)
            cache.prefill(kp)
            torch.cuda.synchronize()
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            t_app = t_sc = 0.0
            for _ in range(64):
                e[0].record()
                cache.append(knew)
                e[1].record()
                cache.key_scores(qd, d ** -0.5, out=lc)
                e[2].record()
                torch.cuda.synchronize()
                t_app += e[0].elapsed_time(e[1])
                t_sc += e[1].elapsed_time(e[2])
            cnt = cache.counts()
            # the same cache read as a store of pre-RoPE keys (rotation after dequantization), at its final state
            rope_us = timed_us(lambda: cache.key_scores_rope(qd, inv_freq, 0, d ** -0.5, out=lc), reps=5)
            out[name] = {"sequences": 64, "heads": H, "tokens_cached": int(cnt.n_tokens), "residual": 32,
                         "us_per_rope_logits_at_end": rope_us,
                         "us_per_append_mean_of_64": t_app / 64 * 1e3, "us_per_logits_mean_of_64": t_sc / 64 * 1e3,
                         "note": "append = copy into the residual buffer, plus every 32nd step one quantize "
                                 "launch over 64 x %d x 32 keys" % H}
            del cache
        del kp
        out["decode_scores"] = {"sequences": 64, "heads": H, "quantized_tokens": nd, "q_per_kv": wl.q_per_kv, "us": us,
                                "keys_per_s": nk / (us * 1e-6), "frac_of_hbm_peak": nb / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    if args.per_layer:
        # The same work as `step`, issued layer by layer: 4 launches-groups x 32 layers.  Eager launches are
        # bound by the host (ctypes marshalling per call); the graph replays the identical launches back to back.
        kvh, qhs = wl.kv_heads, wl.kv_heads * wl.q_per_kv
        ws_l = torch.empty(squat.build_subspace_workspace(n, kvh, wl.q_per_kv, d, wl.r), dtype=torch.uint8, device=dev)
        wp_l = torch.empty(max(256, squat.prepare_workspace(kvh, d, wl.r, wl.g)), dtype=torch.uint8, device=dev)
        codes_b = codes.clone()

        def layer_step():
            for l in range(wl.layers):
                hs = slice(l * kvh, (l + 1) * kvh)
                squat.build_subspace(wl.q[l * qhs:(l + 1) * qhs], wl.q_per_kv, wl.r, qhat=qhat[hs], eig=eig[hs], ws=ws_l)
                squat.prepare(qhat[hs], wl.lam, wl.g, update=update[hs], ws=wp_l)
                squat.quantize_keys(wl.k[:, hs], update[hs], wl.bits, wl.group, wl.g, codes=codes[:, hs],
                                    scale=scale[:, hs], zero=zero[:, hs])
                squat.dequantize_keys(codes[:, hs], scale[:, hs], zero[:, hs], wl.bits, wl.group, out=back[:, hs])

        t_eager = timed(layer_step, reps=5)
        codes_e = codes.clone()

        # the same launches spread over 8 streams (layer l on stream l mod 8, each stream with its own workspaces)
        NS = 8
        streams = [torch.cuda.Stream() for _ in range(NS)]
        ws_s = [torch.empty_like(ws_l) for _ in range(NS)]
        wp_s = [torch.empty_like(wp_l) for _ in range(NS)]

        def streams_step():
            main = torch.cuda.current_stream()
            start = torch.cuda.Event()
            start.record(main)
            for i, st in enumerate(streams):
                st.wait_event(start)
            for l in range(wl.layers):
                i = l % NS
                hs = slice(l * kvh, (l + 1) * kvh)
                with torch.cuda.stream(streams[i]):
                    squat.build_subspace(wl.q[l * qhs:(l + 1) * qhs], wl.q_per_kv, wl.r, qhat=qhat[hs], eig=eig[hs], ws=ws_s[i])
                    squat.prepare(qhat[hs], wl.lam, wl.g, update=update[hs], ws=wp_s[i])
                    squat.quantize_keys(wl.k[:, hs], update[hs], wl.bits, wl.group, wl.g, codes=codes[:, hs],
                                        scale=scale[:, hs], zero=zero[:, hs])
                    squat.dequantize_keys(codes[:, hs], scale[:, hs], zero[:, hs], wl.bits, wl.group, out=back[:, hs])
            for st in streams:
                done = torch.cuda.Event()
                done.record(st)
                main.wait_event(done)

        codes.zero_()
        t_streams = timed(streams_step, reps=5)
        streams_equal = bool(torch.equal(codes, codes_e))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            layer_step()
        codes.zero_()
        t_graph = timed(graph.replay, reps=10)
        out["per_layer"] = {"launch_groups": wl.layers, "heads_per_launch": kvh, "ms_per_step_eager": t_eager,
                            "ms_per_step_graph": t_graph, "keys_per_s_graph": n_keys / (t_graph * 1e-3),
                            "ms_per_step_8_streams": t_streams, "keys_per_s_8_streams": n_keys / (t_streams * 1e-3),
                            "streams_codes_equal_eager": streams_equal,
                            "graph_codes_equal_eager": bool(torch.equal(codes, codes_e)),
                            # the Gram sums are grouped differently (32 workgroups per head instead of 1)
                            "packed_words_differing_from_stacked": float((codes_e != codes_b).float().mean()),
                            "note": "the per-head solvers (eigen-solver 0.37 ms, prepare 0.07 ms per launch whatever the "
                                    "number of heads) run on 8 of 256 CUs here and are serial over the layers: stack the "
                                    "layers, as the headline step does, or give each layer its own stream"}
        del graph
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(dict(n_tokens=n, r=wl.r, lam=wl.lam, bits=wl.bits, group=wl.group,
                                                g=wl.g, q_per_kv=wl.q_per_kv))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
