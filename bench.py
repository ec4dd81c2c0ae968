#!/usr/bin/env python3
"""Benchmark of the SQuat key-quantization hot path on one MI355X.

One step = one pass of the whole path over the long-context workload (32 layers x 8 KV heads
stacked along the head axis, 32768 tokens per layer, d = 128, bf16, r = 32, 2-bit, group 32):
  squat_build_subspace -> squat_prepare -> squat_quantize_keys -> squat_dequantize_keys.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

Beside the headline step the default run also times, each in a bounded number of launches: the four
(bits, group) variants of the long-context configuration, the two storage forms of the update matrix, the
kernels under sustained back-to-back load, the per-channel grouping, the logits kernels, the decode-time
flush, the layer-by-layer schedule with its per-stage split, and the routes to the query subspace.
`--brief` keeps only the headline step (for profiler runs).
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_16BIT_PEAK_TFLOPS = 2500.0
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9      # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz (packed fp32 is off in this build)


def profile_facts() -> dict:
    """Figures that only a profiler run can give (HBM traffic, instruction counts) are read from the tracked
    summaries under profiles/: lines of the form `@bench <name> <number>`.  Nothing is hard-coded here, so a
    summary that is missing or was made for another workload simply leaves the figure out."""
    facts = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        try:
            for line in open(path):
                m = re.match(r"@bench\s+(\S+)\s+([-+0-9.eE]+)\s*$", line)
                if m:
                    facts[m.group(1)] = (float(m.group(2)), os.path.basename(path))
        except OSError:
            pass
    return facts


def cpu_baseline(wl_args: dict, heads: int = 4, repeats: int = 16):
    """The float64 oracle, as it stands, on a bounded sample of the same workload: `heads` KV heads
    (pooled queries of 4 query heads each, all their tokens)."""
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

    def one_pass():
        for h in range(heads):
            Qh, _ = O.subspace(qval[h * qpk:(h + 1) * qpk], r)
            U = O.update_matrix_lemma(Qh, lam, g)
            out = O.quantize_keys(kval[h], U, bits, G, g)
            O.dequantize_keys(out["codes"], out["scale"], out["zero"], G)

    t0 = time.perf_counter()
    for _ in range(repeats):
        one_pass()
    dt = time.perf_counter() - t0
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
    ap.add_argument("--brief", action="store_true", help="headline step only (profiler runs)")
    ap.add_argument("--decode", action="store_true",
                    help="also run the cache object's append + logits loop at the decode shape (64 sequences x 256 "
                         "heads x 2048 tokens) and the logits kernel alone at that shape")
    ap.add_argument("--with-copy", action="store_true",
                    help="profiling aid: also run one plain device copy of the key tensor (known size) per step, "
                         "to calibrate the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--only", default="", help="profiling aid: time only this stage (e.g. quantize_keys); "
                                               "the other stages run once, untimed, to prepare its inputs")
    ap.add_argument("--extra-kernels", action="store_true",
                    help="profiling aid: with --brief, also launch the per-channel and logits kernels once per step")
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
    default_workload = args.layers == 32 and args.tokens == 32768
    facts = profile_facts() if default_workload else {}

    def fact(name):
        return facts[name][0] if name in facts else None

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
    qdec = wl.q[:, n - 1, :].unsqueeze(0).contiguous()                      # [1, q_heads, d]: the last prompt token's queries
    logits = torch.empty((1, H * wl.q_per_kv, n), dtype=torch.float32, device=dev)
    inv_freq = (10000.0 ** (-torch.arange(64, dtype=torch.float64, device=dev) / 64.0)).float()
    pc_codes = torch.empty((1, H, n // 32, d, wl.bits), dtype=torch.int32, device=dev)
    pc_scale = torch.empty((1, H, n // 32, d), dtype=torch.float16, device=dev)
    pc_zero = torch.empty_like(pc_scale)

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
        if args.extra_kernels:
            squat.quantize_keys_per_channel(wl.k, update, wl.bits, 32, wl.g, codes=pc_codes, scale=pc_scale, zero=pc_zero)
            squat.dequantize_keys_per_channel(pc_codes, pc_scale, pc_zero, wl.bits, 32, out=back)
            squat.key_scores(qdec, codes, scale, zero, wl.bits, wl.group, wl.q_per_kv, d ** -0.5, out=logits)
            squat.key_scores_per_channel(qdec, pc_codes, pc_scale, pc_zero, wl.bits, wl.q_per_kv, d ** -0.5, out=logits)
            squat.key_scores_rope(qdec, codes, scale, zero, wl.bits, wl.group, wl.q_per_kv, inv_freq, 0, d ** -0.5, out=logits)
            squat.key_scores_rope_per_channel(qdec, pc_codes, pc_scale, pc_zero, wl.bits, wl.q_per_kv, inv_freq, 0,
                                              d ** -0.5, out=logits)

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
    stage_ms, stage_ms_median, stage_ms_min = {}, {}, {}
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
    # the embedded contraction (Lemma 2's update): 12288 flop per key at g = 32 by the definition; the kernel
    # executes it as two fp16 matrix passes (update matrix on the fp16 grid), i.e. twice that
    alg_tflops = n_keys * 12288 / (q_ms * 1e-3) / 1e12
    traffic_gb = fact("quantize_kernel.traffic_GB_per_launch")
    roofline = {"kernel": "quantize_kernel<2-bit,G32,g32,bf16>", "bound": "hbm", "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                # FETCH_SIZE + WRITE_SIZE of this kernel from rocprofv3 --pmc, scaled by a plain copy of known size:
                # read from the tracked summary, None when there is none for this workload
                "traffic": None if traffic_gb is None else traffic_gb * 1e9,
                "traffic_source": facts["quantize_kernel.traffic_GB_per_launch"][1] if traffic_gb is not None else None,
                "bytes_per_launch": q_bytes, "ms_per_launch": q_ms,
                "contraction": {"algorithmic_flop_per_key": 12288, "algorithmic_tflops": alg_tflops,
                                "algorithmic_frac_of_fp16_mfma_peak": alg_tflops / MFMA_16BIT_PEAK_TFLOPS,
                                "executed_fp16_passes": 2, "executed_tflops": 2 * alg_tflops,
                                "executed_frac_of_fp16_mfma_peak": 2 * alg_tflops / MFMA_16BIT_PEAK_TFLOPS}}
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

    def finish():
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline(dict(n_tokens=n, r=wl.r, lam=wl.lam, bits=wl.bits, group=wl.group,
                                                    g=wl.g, q_per_kv=wl.q_per_kv))
        print(json.dumps(out))

    if args.brief or only:
        finish()
        return

    def series(fn, reps):
        """reps back-to-back launches of fn, each timed by its own pair of events (us)."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        evs[0].record()
        for i in range(reps):
            fn()
            evs[i + 1].record()
        torch.cuda.synchronize()
        return [evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(reps)]

    def timed(fn, reps=5):
        """mean ms of `reps` launches after two untimed ones"""
        fn()
        fn()
        torch.cuda.synchronize()
        return sum(series(fn, reps)) / reps * 1e-3

    def in_path(qfn, dfn, reps=12):
        """A quantize launch timed as it runs in the path: between other kernels (its own dequantize), not back
        to back with itself.  Returns (quantize us, dequantize us), medians over reps after three untimed rounds
        (the first launches after a change of kernel fall into the power controller's transient, see
        `sustained_back_to_back`)."""
        tq, td = [], []
        for i in range(reps + 3):
            e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            e[0].record()
            qfn()
            e[1].record()
            dfn()
            e[2].record()
            torch.cuda.synchronize()
            if i >= 3:
                tq.append(e[0].elapsed_time(e[1]) * 1e3)
                td.append(e[1].elapsed_time(e[2]) * 1e3)
        tq.sort()
        td.sort()
        return tq[len(tq) // 2], td[len(td) // 2]

    def hbm_frac(nbytes, us):
        return nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS

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

    # ---- the long-context configuration's variants: 2 and 4 bits x groups of 32 and 128 channels (g = 32), each
    # quantize launch timed between other kernels as in the path, plus the single-block ceiling (g = G = 128, no
    # update: plain round-to-nearest)
    out["variants"] = []
    var_list = [(2, 32, 32, True), (4, 32, 32, True), (2, 128, 32, True), (4, 128, 32, True), (2, 32, 64, True),
                (2, 128, 128, False)]
    upd64 = squat.prepare(qhat, wl.lam, 64)
    cmax = torch.empty((1, H, n, d * 4 // 32), dtype=torch.int32, device=dev)       # one set of buffers for all variants
    smax = torch.empty((1, H, n, d // 32), dtype=torch.float16, device=dev)
    zmax = torch.empty_like(smax)
    for idx, (bits, G, g, use_update) in enumerate(var_list[:1] + var_list):      # the first entry twice: its first round only warms up
        upd = (update if g == wl.g else upd64) if use_update else None
        c = cmax.view(-1)[:H * n * d * bits // 32].view(1, H, n, d * bits // 32)
        sc = smax.view(-1)[:H * n * d // G].view(1, H, n, d // G)
        ze = zmax.view(-1)[:H * n * d // G].view(1, H, n, d // G)
        tq, td = in_path(lambda: squat.quantize_keys(wl.k, upd, bits, G, g, codes=c, scale=sc, zero=ze),
                         lambda: squat.dequantize_keys(c, sc, ze, bits, G, out=back))
        if idx == 0:
            continue
        nbytes = n_keys * (d * 2 + d * bits // 8 + 4 * (d // G))
        out["variants"].append({"bits": bits, "group": G, "g": g, "update": use_update, "bytes_per_key": nbytes // n_keys,
                                "quantize_us": tq, "quantize_frac_of_hbm_peak": hbm_frac(nbytes, tq),
                                "quantize_keys_per_s": n_keys / (tq * 1e-6),
                                "dequantize_us": td, "dequantize_frac_of_hbm_peak": hbm_frac(nbytes, td)})
    del cmax, smax, zmax, upd64

    # ---- the update matrix's two storage forms (squat_prepare: fp16 grid, two matrix passes in the quantize
    # kernels; squat_prepare_ex full precision: three passes), same keys, same launches
    update_full = squat.prepare(qhat, wl.lam, wl.g, full_precision=True)
    forms = {}
    for name, upd in (("fp16_grid", update), ("full_precision", update_full)):
        tq, _ = in_path(lambda: squat.quantize_keys(wl.k, upd, wl.bits, wl.group, wl.g, codes=codes, scale=scale, zero=zero),
                        lambda: squat.dequantize_keys(codes, scale, zero, wl.bits, wl.group, out=back))
        tp, _ = in_path(lambda: squat.quantize_keys_per_channel(wl.k, upd, wl.bits, 32, wl.g, codes=pc_codes, scale=pc_scale, zero=pc_zero),
                        lambda: squat.dequantize_keys_per_channel(pc_codes, pc_scale, pc_zero, wl.bits, 32, out=back))
        forms[name] = {"quantize_us": tq, "quantize_frac_of_hbm_peak": hbm_frac(q_bytes, tq),
                       "quantize_per_channel_us": tp, "quantize_per_channel_frac_of_hbm_peak": hbm_frac(q_bytes, tp)}
    out["update_matrix_storage"] = forms
    del update_full
    squat.quantize_keys(wl.k, update, wl.bits, wl.group, wl.g, codes=codes, scale=scale, zero=zero)

    # ---- sustained load: 60 launches of one kernel back to back.  The first launch after a pause runs at the
    # boost clock, launches 4-8 are the slowest (the power controller's reaction), then the time settles.
    def board_power_w():
        # the driver's (slowly filtered) board power reading, if the box exposes it
        for path in glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"):
            try:
                return int(open(path).read()) / 1e6
            except (OSError, ValueError):
                pass
        return None

    def sustained(fn):
        torch.cuda.synchronize()
        time.sleep(0.05)
        p0 = board_power_w()
        us = series(fn, 60)
        p1 = board_power_w()
        tail = sorted(us[40:])
        return {"first_us": us[0], "slowest_us": max(us), "slowest_at_launch": us.index(max(us)) + 1,
                "settled_us_median_of_last_20": tail[len(tail) // 2], "first_12_us": [round(x, 1) for x in us[:12]],
                "every_5th_us": [round(x, 1) for x in us[::5]],
                "board_power_W_before_and_after": [p0, p1]}
    sus = {"quantize_keys": sustained(lambda: squat.quantize_keys(wl.k, update, wl.bits, wl.group, wl.g, codes=codes, scale=scale, zero=zero)),
           "dequantize_keys": sustained(lambda: squat.dequantize_keys(codes, scale, zero, wl.bits, wl.group, out=back)),
           "quantize_keys_per_channel": sustained(lambda: squat.quantize_keys_per_channel(wl.k, update, wl.bits, 32, wl.g, codes=pc_codes, scale=pc_scale, zero=pc_zero))}
    for v in sus.values():
        v["settled_frac_of_hbm_peak"] = hbm_frac(q_bytes, v["settled_us_median_of_last_20"])
    out["sustained_back_to_back"] = sus

    # ---- the paper's own grouping (statistics per channel over 32 tokens): same keys, same update matrix
    out["per_channel"] = []
    for bits, g, use_update in [(2, 32, True), (4, 32, True), (2, 64, True)]:
        upd = (update if g == wl.g else squat.prepare(qhat, wl.lam, g)) if use_update else None
        c = pc_codes if bits == wl.bits else torch.empty((1, H, n // 32, d, bits), dtype=torch.int32, device=dev)
        tq, td = in_path(lambda: squat.quantize_keys_per_channel(wl.k, upd, bits, 32, g, codes=c, scale=pc_scale, zero=pc_zero),
                         lambda: squat.dequantize_keys_per_channel(c, pc_scale, pc_zero, bits, 32, out=back))
        tsc = timed(lambda: squat.key_scores_per_channel(qdec, c, pc_scale, pc_zero, bits, wl.q_per_kv, d ** -0.5, out=logits), reps=10) * 1e3
        # the same store read as pre-RoPE keys (rotation after dequantization: the paper's SQuat-pre on its own grouping)
        tsr = timed(lambda: squat.key_scores_rope_per_channel(qdec, c, pc_scale, pc_zero, bits, wl.q_per_kv, inv_freq, 0, d ** -0.5,
                                                              out=logits), reps=10) * 1e3
        nbytes = n_keys * (d * 2 + d * bits // 8 + 4 * (d // 32))
        sb = n_keys * (d * bits // 8 + 4 * (d // 32) + 4 * wl.q_per_kv)
        out["per_channel"].append({"bits": bits, "token_group": 32, "g": g, "update": use_update,
                                   "bytes_per_key": nbytes // n_keys,
                                   "quantize_us": tq, "quantize_frac_of_hbm_peak": hbm_frac(nbytes, tq),
                                   "dequantize_us": td, "dequantize_frac_of_hbm_peak": hbm_frac(nbytes, td),
                                   "key_scores_us": tsc, "key_scores_bytes_per_key": sb // n_keys,
                                   "key_scores_frac_of_hbm_peak": hbm_frac(sb, tsc),
                                   "key_scores_rope_us": tsr, "key_scores_rope_frac_of_hbm_peak": hbm_frac(sb, tsr)})
    # Decode-side consumer: attention logits of one query token per query head straight from the packed
    # store just written (48 B of codes and metadata in, 4 B per query head out, per key).
    ts = timed(lambda: squat.key_scores(qdec, codes, scale, zero, wl.bits, wl.group, wl.q_per_kv, d ** -0.5, out=logits), reps=10) * 1e3
    sbytes = n_keys * (d * wl.bits // 8 + 4 * (d // wl.group) + 4 * wl.q_per_kv)
    out["key_scores"] = {"bits": wl.bits, "group": wl.group, "q_per_kv": wl.q_per_kv, "bytes_per_key": sbytes // n_keys,
                         "us": ts, "keys_per_s": n_keys / (ts * 1e-6), "frac_of_hbm_peak": hbm_frac(sbytes, ts)}
    # the pre-RoPE variant of the same consumer: keys dequantized, rotated to their positions and rounded to
    # fp16 in registers before the contraction (bound by vector arithmetic, not by HBM)
    tr = timed(lambda: squat.key_scores_rope(qdec, codes, scale, zero, wl.bits, wl.group, wl.q_per_kv, inv_freq, 0,
                                             d ** -0.5, out=logits), reps=10) * 1e3
    rope = {"bits": wl.bits, "group": wl.group, "q_per_kv": wl.q_per_kv, "bound": "alu", "us": tr,
            "keys_per_s": n_keys / (tr * 1e-6), "frac_of_hbm_peak": hbm_frac(sbytes, tr)}
    valu = fact("key_scores_rope_kernel.valu_per_16_keys")       # SQ_INSTS_VALU per unit of 16 keys, from the tracked counters
    if valu is not None:
        lane_ops = n_keys / (tr * 1e-6) * valu * 64 / 16
        rope.update({"valu_instructions_per_16_keys": valu, "valu_source": facts["key_scores_rope_kernel.valu_per_16_keys"][1],
                     "alu_lane_ops_per_s": lane_ops, "alu_peak_lane_ops_per_s": ALU_PEAK_LANE_OPS,
                     "alu_frac": lane_ops / ALU_PEAK_LANE_OPS})
    out["key_scores_rope"] = rope

    # ---- decode-time flush (Algorithm 1, decoding phase): 64 sequences x 32 buffered tokens per head, the update
    # matrix shared by the batch; one layer (8 heads) per launch and all 32 layers (256 heads) per launch.  Latency
    # of an isolated flush (host-synchronised) and the rate of flushes issued back to back.
    out["decode_flush"] = []
    for heads in (wl.kv_heads, H):
        kb = torch.randn((64, heads, 32, d), device=dev, dtype=torch.float32).to(torch.bfloat16)
        c = torch.empty((64, heads, 32, d * wl.bits // 32), dtype=torch.int32, device=dev)
        sc = torch.empty((64, heads, 32, d // wl.group), dtype=torch.float16, device=dev)
        ze = torch.empty_like(sc)
        fn = lambda: squat.quantize_keys(kb, update[:heads], wl.bits, wl.group, wl.g, codes=c, scale=sc, zero=ze)  # noqa: E731
        fn()
        torch.cuda.synchronize()
        lat = []
        for _ in range(20):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1) * 1e3)
        lat.sort()
        us = series(fn, 50)
        nk = 64 * heads * 32
        # the same launch 32 times in a captured graph (a decode step flushes layer after layer): the rate the
        # device sustains when the host's per-call cost is out of the way
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(32):
                fn()
        graph.replay()
        torch.cuda.synchronize()
        rep = []
        for _ in range(10):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            rep.append(e0.elapsed_time(e1) * 1e3 / 32)
        rep.sort()
        del graph
        out["decode_flush"].append({"sequences": 64, "heads_per_launch": heads, "keys_per_flush": nk,
                                    "us_per_flush_isolated_median": lat[len(lat) // 2],
                                    "us_per_flush_back_to_back": sum(us) / len(us),
                                    "keys_per_s_back_to_back": nk / (sum(us) / len(us) * 1e-6),
                                    "us_per_flush_in_a_graph_of_32": rep[len(rep) // 2],
                                    "keys_per_s_in_a_graph": nk / (rep[len(rep) // 2] * 1e-6)})

    # ---- the same work issued layer by layer (8 KV heads per launch, as a prefill produces them): one stream,
    # with the per-stage split; then layer l on stream l mod S for S = 2 and 8 (equal priorities), which lets the
    # per-head solvers of one layer (8 of 256 CUs busy) overlap the streaming kernels of others
    kvh, qhs = wl.kv_heads, wl.kv_heads * wl.q_per_kv
    ws_l = torch.empty(squat.build_subspace_workspace(n, kvh, wl.q_per_kv, d, wl.r), dtype=torch.uint8, device=dev)
    wp_l = torch.empty(max(256, squat.prepare_workspace(kvh, d, wl.r, wl.g)), dtype=torch.uint8, device=dev)

    def one_layer(l, ws, wp, ev=None):
        hs = slice(l * kvh, (l + 1) * kvh)
        if ev: ev[0].record()
        squat.build_subspace(wl.q[l * qhs:(l + 1) * qhs], wl.q_per_kv, wl.r, qhat=qhat[hs], eig=eig[hs], ws=ws)
        if ev: ev[1].record()
        squat.prepare(qhat[hs], wl.lam, wl.g, update=update[hs], ws=wp)
        if ev: ev[2].record()
        squat.quantize_keys(wl.k[:, hs], update[hs], wl.bits, wl.group, wl.g, codes=codes[:, hs],
                            scale=scale[:, hs], zero=zero[:, hs])
        if ev: ev[3].record()
        squat.dequantize_keys(codes[:, hs], scale[:, hs], zero[:, hs], wl.bits, wl.group, out=back[:, hs])
        if ev: ev[4].record()

    def layer_step(ev=None):
        for l in range(wl.layers):
            one_layer(l, ws_l, wp_l, ev[l] if ev else None)

    layer_step()
    layer_step()
    torch.cuda.synchronize()
    reps = 4
    evs = [[[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(wl.layers)] for _ in range(reps)]
    t0 = time.perf_counter()
    for i in range(reps):
        layer_step(evs[i])
    torch.cuda.synchronize()
    t_serial = (time.perf_counter() - t0) * 1e3 / reps
    split = {name: sum(evs[i][l][s].elapsed_time(evs[i][l][s + 1]) for i in range(reps) for l in range(wl.layers)) / reps
             for s, name in enumerate(stages)}
    per_layer = {"launch_groups": wl.layers, "heads_per_launch": kvh, "one_stream": {"ms_per_step": t_serial,
                 "keys_per_s": n_keys / (t_serial * 1e-3), "stage_ms_sum_over_layers": split}}
    codes_serial = codes.clone()
    for NS in (2, 8):
        streams = [torch.cuda.Stream() for _ in range(NS)]
        ws_s = [torch.empty_like(ws_l) for _ in range(NS)]
        wp_s = [torch.empty_like(wp_l) for _ in range(NS)]

        def streams_step():
            main = torch.cuda.current_stream()
            start = torch.cuda.Event()
            start.record(main)
            for st in streams:
                st.wait_event(start)
            for l in range(wl.layers):
                with torch.cuda.stream(streams[l % NS]):
                    one_layer(l, ws_s[l % NS], wp_s[l % NS])
            for st in streams:
                done = torch.cuda.Event()
                done.record(st)
                main.wait_event(done)

        codes.zero_()
        streams_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            streams_step()
        torch.cuda.synchronize()
        t_s = (time.perf_counter() - t0) * 1e3 / reps
        per_layer["%d_streams" % NS] = {"ms_per_step": t_s, "keys_per_s": n_keys / (t_s * 1e-3),
                                        "codes_equal_one_stream": bool(torch.equal(codes, codes_serial))}
        del streams, ws_s, wp_s
    out["per_layer"] = per_layer
    del codes_serial

    # ---- routes to the query subspace on 256 heads: the exact solver against block power iteration on the Gram
    # matrix (cold start, and warm start after 64 new queries), on near-isotropic queries and on queries that
    # concentrate in a few directions; error = || Qhat^T Qhat - exact || / || exact ||, worst head
    def subspace_routes(q, n_tok, r, label):
        qpk = wl.q_per_kv
        heads = q.shape[0] // qpk
        n_old = n_tok - 64
        state = torch.zeros((heads, d, d), dtype=torch.float64, device=dev)
        ws = torch.empty(int(squat.lib().squat_refresh_subspace_workspace(n_old, heads, qpk, d, r)), dtype=torch.uint8, device=dev)
        prev, _, _ = squat.refresh_subspace(state, qpk, r, -1, q_new=q[:, :n_old], accumulate=False, ws=ws)
        squat.refresh_subspace(state, qpk, 0, 0, q_new=q[:, n_old:n_tok], accumulate=True, ws=ws)
        exact, ev, _ = squat.refresh_subspace(state, qpk, r, -1, ws=ws)
        ref = torch.bmm(exact.double().transpose(1, 2), exact.double())
        refn = ref.flatten(1).norm(dim=1)
        qh, ei, re = torch.empty_like(exact), torch.empty_like(ev), torch.empty((heads,), dtype=torch.float32, device=dev)

        def err(x):
            m = torch.bmm(x.double().transpose(1, 2), x.double())
            return float(((m - ref).flatten(1).norm(dim=1) / refn).max())
        t_exact = timed(lambda: squat.refresh_subspace(state, qpk, r, -1, qhat=qh, eig=ei, residual=re, ws=ws), reps=5) * 1e3
        rows = {"exact_solver_us": t_exact, "cold": [], "warm_after_64_new_queries": []}
        for k in (0, 1, 2, 4, 8, 16, 32, 64):
            t = timed(lambda: squat.refresh_subspace(state, qpk, r, k, qhat=qh, eig=ei, residual=re, ws=ws), reps=3) * 1e3
            rows["cold"].append({"iterations": k, "us": t, "error": err(qh), "residual": float(re.max()),
                                 "eig_rel_error": float(((ei - ev).abs().max(dim=1).values / ev[:, 0]).max())})
        for k in (0, 1, 2, 3, 5, 8):
            t = timed(lambda: squat.refresh_subspace(state, qpk, r, k, qhat_prev=prev, qhat=qh, eig=ei, residual=re, ws=ws), reps=3) * 1e3
            rows["warm_after_64_new_queries"].append({"iterations": k, "us": t, "error": err(qh), "residual": float(re.max())})
        rows["previous_qhat_error"] = err(prev)
        rows["workload"] = label
        return rows
    routes = []
    n_r = min(n, 4096)
    routes.append(subspace_routes(wl.q, n_r, 32, "near-isotropic N(0,1) queries, %d tokens x 4 query heads per KV head, r = 32" % n_r))
    routes.append(subspace_routes(wl.q, n_r, 8, "near-isotropic N(0,1) queries, %d tokens x 4 query heads per KV head, r = 8" % n_r))
    wlp = LongContext(layers=args.layers, n_tokens=n_r, planted_rank=12, seed=5100)
    routes.append(subspace_routes(wlp.q, n_r, 8, "queries with 12 planted decaying directions, %d tokens, r = 8" % n_r))
    routes.append(subspace_routes(wlp.q, n_r, 16, "queries with 12 planted decaying directions, %d tokens, r = 16" % n_r))
    del wlp
    out["subspace_routes"] = routes

    # ---- the (r, lambda, g) settings the paper reports (Section 4 "Hyper-parameters"): the default of its short-task
    # runs and the ones of its long-context runs, whole path on the same workload, stage by stage
    out["paper_settings"] = []
    for r_s, lam_s, g_s in ((5, 1e-3, 64), (10, 5e-4, 64), (20, 5e-4, 64), (40, 1e-3, 64), (60, 5e-4, 32)):
        qh_s = torch.empty((H, r_s, d), dtype=torch.float32, device=dev)
        eg_s = torch.empty((H, r_s), dtype=torch.float32, device=dev)
        wp_s = torch.empty(max(256, squat.prepare_workspace(H, d, r_s, g_s)), dtype=torch.uint8, device=dev)

        def setting(ev=None):
            if ev: ev[0].record()
            squat.build_subspace(wl.q, wl.q_per_kv, r_s, qhat=qh_s, eig=eg_s, ws=ws_sub)
            if ev: ev[1].record()
            squat.prepare(qh_s, lam_s, g_s, update=update, ws=wp_s)
            if ev: ev[2].record()
            squat.quantize_keys(wl.k, update, wl.bits, wl.group, g_s, codes=codes, scale=scale, zero=zero)
            if ev: ev[3].record()
            squat.dequantize_keys(codes, scale, zero, wl.bits, wl.group, out=back)
            if ev: ev[4].record()

        setting()
        setting()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(4)]
        for e5 in evs:
            setting(e5)
        torch.cuda.synchronize()
        med = lambda k: sorted(e5[k].elapsed_time(e5[k + 1]) for e5 in evs)[2]  # noqa: E731
        tot = sorted(e5[0].elapsed_time(e5[4]) for e5 in evs)[2]
        out["paper_settings"].append({"r": r_s, "lambda": lam_s, "g": g_s, "ms_per_step": tot, "keys_per_s": n_keys / (tot * 1e-3),
                                      "stage_ms": {"build_subspace": med(0), "prepare": med(1), "quantize_keys": med(2),
                                                   "dequantize_keys": med(3)}})
        del qh_s, eg_s, wp_s
    # the headline matrices back in place for what follows
    squat.prepare(qhat, wl.lam, wl.g, update=update, ws=ws_prep)
    squat.quantize_keys(wl.k, update, wl.bits, wl.group, wl.g, codes=codes, scale=scale, zero=zero)

    if args.decode:
        def timed_us(fn, reps=50):
            fn()
            torch.cuda.synchronize()
            return sum(series(fn, reps)) / reps
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
            # one untimed pass first (a kernel's first launch in a process loads its code: ~1 ms), then the timed one
            # from the same starting state
            for timed in (False, True):
                cache.reset()
                cache.prefill(kp)
                torch.cuda.synchronize()
                e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                app, sco = [], []
                for _ in range(64 if timed else 33):
                    e[0].record()
                    cache.append(knew)
                    e[1].record()
                    cache.key_scores(qd, d ** -0.5, out=lc)
                    e[2].record()
                    torch.cuda.synchronize()
                    app.append(e[0].elapsed_time(e[1]))
                    sco.append(e[1].elapsed_time(e[2]))
            t_app, t_sc = sum(app), sum(sco)
            cnt = cache.counts()
            # the same cache read as a store of pre-RoPE keys (rotation after dequantization), at its final state
            rope_us = timed_us(lambda: cache.key_scores_rope(qd, inv_freq, 0, d ** -0.5, out=lc), reps=5)
            out[name] = {"sequences": 64, "heads": H, "tokens_cached": int(cnt.n_tokens), "residual": 32,
                         "us_per_rope_logits_at_end": rope_us,
                         "us_per_append_mean_of_64": t_app / 64 * 1e3, "us_per_logits_mean_of_64": t_sc / 64 * 1e3,
                         "us_per_append_median": sorted(app)[32] * 1e3, "us_per_append_with_flush_max": max(app) * 1e3,
                         "note": "append = copy into the residual buffer, plus every 32nd step one quantize "
                                 "launch over 64 x %d x 32 keys" % H}
            del cache
        del kp
        out["decode_scores"] = {"sequences": 64, "heads": H, "quantized_tokens": nd, "q_per_kv": wl.q_per_kv, "us": us,
                                "keys_per_s": nk / (us * 1e-6), "frac_of_hbm_peak": nb / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    finish()


if __name__ == "__main__":
    main()
