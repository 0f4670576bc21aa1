#!/usr/bin/env python3
"""SPTS prefill benchmark on one MI355X: tokens/s + TTFT of the token-skipped prefill, with the
roofline fraction of the dominant kernel, the library's own dense prefill, and the CPU oracle
timed on the host cores as a reported baseline.

A step is one pass of the whole hot path (every layer of the stack: PAP probe, TopK, reduced
attention, LTP proxy, reduced FFN, MSDP compaction at stage ends) over one batch of seeded
synthetic hidden states that already sit in HBM.  TTFT here = stack-in hidden states -> final
hidden states (no embedding, final norm or LM head).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA (published)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E (published)
# Kernel behind the roofline figure (phase ffn_gate_up of the library's event timer) as rocprofv3 names it.
DOMINANT_KERNEL = "gemm_mfma_kernel<1, 32, false, 8>"
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "c2_ffn_gate_up_hbm_traffic.txt")


def measured_traffic(workload):
    """Bytes per launch that the dominant kernel moves between L2 and the fabric, read from the committed counter
    summary (two rocprofv3 --pmc runs of this script, FETCH_SIZE and WRITE_SIZE, scaled by the readings of a plain
    1 GiB elementwise kernel, --calibrate-copy).  Counters cannot be read inside this process; the summary carries one
    line `bench-table: workload=<w> kernel="<name>" bytes_per_launch=<b>` per workload it covers.  The figure is used only
    if that line names this workload AND the kernel timed here; otherwise None."""
    try:
        with open(TRAFFIC_SUMMARY) as f:
            lines = [l.strip() for l in f if l.startswith("bench-table:")]
    except OSError:
        return None, None
    for l in lines:
        fields = dict(kv.split("=", 1) for kv in __import__("shlex").split(l[len("bench-table:"):]))
        if fields.get("workload") == workload:
            assert fields.get("kernel") == DOMINANT_KERNEL, (
                f"{TRAFFIC_SUMMARY} was measured on {fields.get('kernel')!r}, bench.py times {DOMINANT_KERNEL!r}: regenerate it")
            return float(fields["bytes_per_launch"]), os.path.relpath(TRAFFIC_SUMMARY, ROOT)
    return None, None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(wl, w_host, sample_tokens):
    """Times the oracle (as it stands) on one skip layer of the workload at two prefix lengths, n/2 and n tokens, fits
    t(N) = a*N + b*N^2 through the two timings (projections, proxy and FFN grow with N, the reduced attention with
    N^2 at a fixed keep ratio) and sums the fit over the candidate counts of the stack's layers (the stage pruning
    shrinks them): tokens/s = N_0 / sum_l t(N_l), labelled extrapolated."""
    import numpy as np
    from oracle import spts_oracle as orc
    from paper_2601_13155_amd import synth
    try:
        from threadpoolctl import threadpool_info
    except Exception:
        threadpool_info = None
    shape = wl.shape
    mdl = orc.Model(shape.D, shape.H, shape.Hkv, shape.d, shape.Dff, shape.rms_eps, shape.rope_base)
    plan = wl.layer_plan()
    first_skip = next(it for it in plan if it.get("skip", 1))   # budgets of the first skip layer, scaled to the sample
    ka, kf = first_skip["m_attn"] / first_skip["N"], first_skip["m_ffn"] / first_skip["N"]
    w64 = {k: np.asarray(v, dtype=np.float64) for k, v in w_host.items()}   # conversion is not part of the timing
    x_all = synth.hidden_states(wl.seed, wl.N, shape.D, shape.dtype)
    n2 = min(sample_tokens, wl.N)
    n1 = max(n2 // 2, min(wl.probe_len, n2))
    secs = {}
    for n in sorted({n1, n2}):
        cfg = orc.LayerCfg(1, min(wl.probe_len, n), int(ka * n), int(kf * n), wl.protect_last, 0)
        t0 = time.perf_counter()
        orc.layer_prefill(x_all[:n], synth.positions(n), w64, mdl, cfg,
                          rnd=orc.bf16_prefill if shape.dtype == "bf16" else orc.identity, score_cast=orc.f32_round)
        secs[n] = time.perf_counter() - t0
    if n1 != n2:
        bq = (secs[n2] / n2 - secs[n1] / n1) / (n2 - n1)
        bq = max(bq, 0.0)
        al = secs[n2] / n2 - bq * n2
    else:
        al, bq = secs[n2] / n2, 0.0
    t_stack = sum(al * it["N"] + bq * it["N"] ** 2 for it in plan)
    threads = None
    if threadpool_info is not None:
        ths = [p.get("num_threads") for p in threadpool_info() if p.get("user_api") == "blas"]
        threads = max(ths) if ths else None
    if threads is None:
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    try:
        allowed = len(os.sched_getaffinity(0))
    except AttributeError:
        allowed = os.cpu_count()
    return {
        "value": wl.N / t_stack, "unit": "tokens/s", "cores": int(threads), "nproc": int(os.cpu_count() or 0),
        "cpus_allowed": int(allowed), "kind": "oracle",
        "sample": (f"oracle.layer_prefill (numpy fp64, bf16-faithful rounding) on ONE skip layer over the first {n1} and the first "
                   f"{n2} tokens of the workload input (keep {ka:.3f}/{kf:.3f}, P={wl.probe_len}, r={wl.r}): {secs[n1]:.2f} s and "
                   f"{secs[n2]:.2f} s; t(N) = {al:.3e}*N + {bq:.3e}*N^2 fitted through both and summed over the {len(plan)} "
                   f"layers' candidate counts (extrapolated: {t_stack:.0f} s for the stack)"),
        "seconds_per_sample": {str(k): v for k, v in secs.items()}, "seconds_stack_extrapolated": t_stack,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "p32", "q32"],
                    help="c2 = the configuration the metric is quoted on; p32 / q32 = the paper's own LLaMA / Qwen schedule at 32K")
    ap.add_argument("--length", type=int, default=0, help="override the context length N (0 = the workload's)")
    ap.add_argument("--components", default="full", choices=["full", "pap+ltp", "pap"],
                    help="modules switched on: all three, no stage pruning, or attention skipping only")
    ap.add_argument("--ablation", action="store_true",
                    help="p32 / q32: also time dense, PAP, PAP+LTP and PAP+LTP+MSDP prefills at 8K, 16K, 24K and 32K tokens, "
                         "and the end-to-end latency with 16 decoded tokens (the measurements of Sec. 4.2 / Table "
                         "ablation_main_speed, on synthetic data)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = the workload's)")
    ap.add_argument("--weight-pool", type=int, default=2,
                    help="distinct synthetic weight sets; layers cycle through them (bounds set-up time)")
    ap.add_argument("--row-major-weights", action="store_true",
                    help="do not upload the slab-major weight copies (the prefill GEMMs then read the row-major matrices)")
    ap.add_argument("--dense-steps", type=int, default=1, help="timed steps of the dense (skip=0) prefill; 0 = skip it")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192,
                    help="the oracle is timed on one layer over the first n/2 and the first n tokens (0 = no cpu_baseline leg)")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket phases with events in the timed region")
    ap.add_argument("--topk-batch", type=int, default=2048,
                    help="rows of the batched TopK micro-benchmark (rows x 131072 fp32 scores; 0 = skip it)")
    ap.add_argument("--decode-steps", type=int, default=32,
                    help="greedy decode steps over the caches the prefill leaves (0 = skip the decode leg)")
    ap.add_argument("--vocab", type=int, default=128256, help="rows of the synthetic vocabulary table of the decode leg")
    ap.add_argument("--decode-batch", type=int, default=8,
                    help="sequences of the batched decode leg (copies of the prefill caches decoded together, at most 16; 0 or 1 = skip it)")
    ap.add_argument("--builder-tokens", type=int, default=8192,
                    help="calibration tokens of the offline channel-importance leg (0 = skip it)")
    ap.add_argument("--batch-seqs", type=int, default=4,
                    help="sequences of the batched-layer leg (one skip layer over that many sequences of 8192 tokens, "
                         "as one spts_layer_prefill_batched call and as single calls; 0 = skip it)")
    ap.add_argument("--builder-channels", action="store_true",
                    help="p32 / q32: the proxy's Dlow channels are chosen on the GPU (spts_channel_importance + spts_select_topk "
                         "on synthetic calibration rows) instead of a seeded random subset")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first launch a plain elementwise kernel (dst = src + 1 over 2^28 floats: reads 1 GiB, writes 1 GiB) "
                         "three times; under a counter-collecting profiler its FETCH_SIZE / WRITE_SIZE readings give the "
                         "scale of those counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported (nothing here shards).")
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2601_13155_amd import costmodel as cm
    from paper_2601_13155_amd import runtime, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    wl = synth.WORKLOADS[args.workload]
    if args.length or args.components != "full":
        wl = synth.scaled(wl, N=args.length or wl.N, components=args.components)
    if args.layers:
        ends = tuple(e for e in wl.stage_end_layers if e < args.layers)
        wl = synth.scaled(wl, layers=args.layers, stage_end_layers=ends, stage_cum_keep=wl.stage_cum_keep[:len(ends) + 1])
    shape = wl.shape
    plan = wl.layer_plan()
    Dlow = wl.proxy_dlow

    t_setup = time.perf_counter()
    pool = max(1, min(args.weight_pool, wl.layers))
    host_sets, dev_sets = [], []
    ctx = runtime.make_context(shape, wl.N, wl.probe_len, wl.proxy_r, Dlow)
    for i in range(pool):
        channels = None
        if args.builder_channels and wl.dlow:
            # Sec. 3.3 on the GPU: channel scores over synthetic calibration rows (rho = 0.2), C = TopK(I, Dlow); the
            # SVD of the sliced matrices is harness set-up
            dw0 = runtime.upload_layer(synth.layer_weights(wl.seed, i, shape), shape, 0, pack=False)
            T = min(args.builder_tokens or 2048, wl.N)
            channels, _ = runtime.select_proxy_channels(ctx, dw0, shape, synth.calibration_states(wl.seed + i, T, shape.D, shape.dtype),
                                                        max(1, int(0.2 * T)), wl.dlow)
            del dw0
        w = synth.make_layer(wl.seed, i, shape, wl.r, wl.dlow, wl.r_pad, channels=channels)
        dev_sets.append(runtime.upload_layer(w, shape, wl.proxy_r, pack=not args.row_major_weights))
        host_sets.append(w if i == 0 else None)
        log(f"[setup] weight set {i + 1}/{pool} ready ({time.perf_counter() - t_setup:.1f} s)")
    layers = [dev_sets[l % pool] for l in range(wl.layers)]
    x0 = runtime.to_device(synth.hidden_states(wl.seed, wl.N, shape.D, shape.dtype), shape.dtype)
    pos0 = torch.from_numpy(synth.positions(wl.N)).cuda()
    assert ctx.uses_mfma(), "matrix-core kernels are not serving this workload"
    runner = runtime.StackRunner(ctx, shape, layers, plan, wl.probe_len, wl.protect_last, skip=1)
    log(f"[setup] done in {time.perf_counter() - t_setup:.1f} s; workload {wl.name}: N={wl.N}, layers={wl.layers}")

    def timed(run, steps, warmup, profile):
        for _ in range(warmup):
            run.run(x0, pos0)
        torch.cuda.synchronize()
        if profile:
            ctx.spts_profile_begin()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            run.run(x0, pos0)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        phases = ctx.spts_profile_end() if profile else {}
        return e0.elapsed_time(e1) / steps, wall / steps, phases

    profile = not args.no_profile
    ms, wall_ms, phases = timed(runner, args.steps, args.warmup, profile)
    log(f"[spts] {ms:.2f} ms/step (host wall {wall_ms:.2f} ms)")
    xo, po, n_final = runner.run(x0, pos0)
    torch.cuda.synchronize()
    assert n_final == plan[-1]["N"] if plan[-1]["N_next"] is None else True
    assert bool(torch.isfinite(xo.float()).all()), "non-finite hidden states"

    # ---- algorithmic work of the timed region
    flops_by = {}
    for item in plan:
        if item.get("skip", 1):
            f = cm.layer_flops(shape.D, shape.H, shape.Hkv, shape.d, shape.Dff, item["N"], wl.probe_len,
                               min(item["N"], item["m_attn"]), min(item["N"], item["m_ffn"]), wl.r, Dlow, True)
            if item["m_ffn"] >= item["N"]:
                f["proxy"] = 0.0   # every candidate takes the FFN: the library does not run the proxy
        else:   # dense layer of the schedule: same phases, all tokens, no probe / proxy
            f = cm.layer_flops(shape.D, shape.H, shape.Hkv, shape.d, shape.Dff, item["N"], wl.probe_len,
                               item["N"], item["N"], wl.r, Dlow, False)
            qkv = f.pop("qkv_proj")
            f["k_proj"] = qkv * shape.Hkv / (shape.H + 2 * shape.Hkv)
            f["qv_proj"] = qkv - f["k_proj"]
        for k, v in f.items():
            flops_by[k] = flops_by.get(k, 0.0) + v
    for k in ("probe_q", "probe_attn", "proxy"):
        flops_by.setdefault(k, 0.0)
    total_flops = sum(flops_by.values())
    gate_up_flops = flops_by["ffn"] * 2.0 / 3.0   # gate + up projections of the gathered rows
    roofline = None
    phase_out = {}
    if phases:
        for name, (tot_ms, n) in phases.items():
            phase_out[name] = {"ms_per_step": tot_ms / args.steps, "launches_per_step": n / args.steps}
        gu_ms = phases["ffn_gate_up"][0] / args.steps
        achieved = gate_up_flops / (gu_ms * 1e-3) / 1e12
        traffic, traffic_src = (None, None) if (args.layers or args.length or args.row_major_weights) else measured_traffic(wl.name)
        roofline = {"kernel": f"spts::{DOMINANT_KERNEL} (ffn_gate_up: SiLU(gate)*up GEMM on the gathered rows)", "bound": "mfma",
                    "achieved": achieved,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                    "traffic": traffic, "traffic_source": traffic_src,
                    "traffic_unit": "bytes per launch (L2 <-> fabric, counter-measured offline)",
                    "flops_per_step": gate_up_flops, "ms_per_step": gu_ms,
                    "launches_per_step": phases["ffn_gate_up"][1] / args.steps}
        # add derived rates for the other phases
        phase_flops = {"k_proj": flops_by["k_proj"], "probe_q": flops_by["probe_q"], "probe_attn": flops_by["probe_attn"],
                       "attention": flops_by["attention"], "o_proj": flops_by["o_proj"],
                       "ffn_gate_up": gate_up_flops, "ffn_down": flops_by["ffn"] / 3.0,
                       "qv_proj": flops_by["qv_proj"],
                       "q_proj": flops_by["qv_proj"] * shape.H / (shape.H + shape.Hkv),
                       "v_proj": flops_by["qv_proj"] * shape.Hkv / (shape.H + shape.Hkv)}
        proxy_ms = sum(phase_out[k]["ms_per_step"] for k in ("proxy_in", "proxy_mid", "proxy_z", "proxy_out") if k in phase_out)
        for k, fl in phase_flops.items():
            if k in phase_out and phase_out[k]["ms_per_step"] > 0:
                phase_out[k]["tflops"] = fl / (phase_out[k]["ms_per_step"] * 1e-3) / 1e12
        if proxy_ms > 0:
            phase_out["proxy_total"] = {"ms_per_step": proxy_ms, "tflops": flops_by["proxy"] / (proxy_ms * 1e-3) / 1e12}
        b = 2 if shape.dtype == "bf16" else 4
        norm_bytes = sum(2 * 2.0 * item["N"] * shape.D * b for item in plan)
        if "rmsnorm" in phase_out:
            phase_out["rmsnorm"]["gbs"] = norm_bytes / (phase_out["rmsnorm"]["ms_per_step"] * 1e-3) / 1e9
        probe_bytes = sum(item["N"] * shape.Hkv * shape.d * b + 4.0 * item["N"] for item in plan if item.get("skip", 1))
        if "probe_attn" in phase_out:
            phase_out["probe_attn"]["gbs"] = probe_bytes / (phase_out["probe_attn"]["ms_per_step"] * 1e-3) / 1e9
        # TopK (two per layer): scores in, indices out.  K-hat / position gather: rows read and written.
        topk_bytes = sum(8.0 * item["N"] + 4.0 * (min(item["N"], item["m_attn"]) + min(item["N"], item["m_ffn"]))
                         for item in plan if item.get("skip", 1))
        if "topk" in phase_out:
            phase_out["topk"]["gbs"] = topk_bytes / (phase_out["topk"]["ms_per_step"] * 1e-3) / 1e9
        gather_bytes = sum(min(item["N"], item["m_attn"]) * (2.0 * shape.Hkv * shape.d * b + 12.0) for item in plan
                           if item.get("skip", 1))
        if "gather" in phase_out:
            phase_out["gather"]["gbs"] = gather_bytes / (phase_out["gather"]["ms_per_step"] * 1e-3) / 1e9
        comp_bytes = sum(cm.compact_bytes(shape.D, item["N"], item["N_next"], b) for item in plan if item["N_next"] is not None)
        if "compact" in phase_out and phase_out["compact"]["ms_per_step"] > 0:
            phase_out["compact"]["gbs"] = comp_bytes / (phase_out["compact"]["ms_per_step"] * 1e-3) / 1e9
        for v in phase_out.values():
            if "gbs" in v:
                v["hbm_frac"] = v["gbs"] / PEAK_HBM_GBS
            if "tflops" in v:
                v["mfma_frac"] = v["tflops"] / PEAK_BF16_TFLOPS

    # ---- dense prefill of the same stack through the same library (skip = 0 on every layer)
    dense = None
    if args.dense_steps > 0:
        drunner = runtime.StackRunner(ctx, shape, layers, plan, wl.probe_len, wl.protect_last, skip=0)
        dms, _, _ = timed(drunner, args.dense_steps, 0, False)
        dflops = wl.layers * sum(cm.layer_flops(shape.D, shape.H, shape.Hkv, shape.d, shape.Dff, wl.N, wl.probe_len,
                                                wl.N, wl.N, wl.r, Dlow, False).values())
        dense = {"ms_per_step": dms, "tokens_per_s": wl.N / (dms * 1e-3), "speedup_spts_over_dense": dms / ms,
                 "tflops": dflops / (dms * 1e-3) / 1e12, "steps": args.dense_steps}
        log(f"[dense] {dms:.2f} ms/step -> SPTS speedup {dms / ms:.2f}x")

    # ---- decode leg: the prefill runs once more with per-layer caches attached, then greedy decode steps
    decode = None
    if args.decode_steps > 0:
        steps_d = args.decode_steps
        prof_steps = min(steps_d, 8)
        caches = [runtime.KVCache(shape, (min(it["N"], it["m_attn"]) if it.get("skip", 1) else it["N"]) + steps_d + prof_steps + 1)
                  for it in plan]
        crunner = runtime.StackRunner(ctx, shape, layers, plan, wl.probe_len, wl.protect_last, skip=1, caches=caches)
        crunner.run(x0, pos0)
        torch.cuda.synchronize()
        cached = [c.count for c in caches]
        table = runtime.to_device(synth.vocab_table(wl.seed, args.vocab, shape.D, shape.dtype), shape.dtype)
        gamma_f = runtime.to_device(np.ones(shape.D, dtype=np.float32), shape.dtype)
        dec = runtime.DecodeRunner(ctx, shape, layers, caches, gamma_f, table)
        dec.x.copy_(table[1])
        dec.generate(wl.N, 1)                       # warm-up step (also the first appended pair)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        toks = torch.zeros(steps_d, dtype=torch.int32, device="cuda")
        e0.record()
        dec.generate(wl.N + 1, steps_d, toks)
        e1.record()
        torch.cuda.synchronize()
        dms = e0.elapsed_time(e1) / steps_d
        # phase split from a few more steps with the library's events on (they cost time: not part of dms)
        ctx.spts_profile_begin()
        dec.generate(wl.N + 1 + steps_d, prof_steps)
        torch.cuda.synchronize()
        dphases = ctx.spts_profile_end()
        b = 2 if shape.dtype == "bf16" else 4
        wbytes = wl.layers * b * (shape.D * (shape.H + 2 * shape.Hkv) * shape.d + shape.H * shape.d * shape.D
                                  + 3 * shape.D * shape.Dff)
        kvbytes = sum(2.0 * (cn + 1 + steps_d / 2.0) * shape.Hkv * shape.d * b for cn in cached)
        head_bytes = float(args.vocab) * shape.D * b
        tot = wbytes + kvbytes + head_bytes
        decode = {"steps": steps_d, "ms_per_token": dms, "tokens_per_s": 1e3 / dms,
                  "bytes_per_token": {"layer_weights": wbytes, "kv_cache": kvbytes, "vocab_table": head_bytes},
                  "gbs": tot / (dms * 1e-3) / 1e9, "hbm_frac": tot / (dms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                  "e2e_ms": ms + steps_d * dms,   # prefill (TTFT) + the decode steps: end-to-end latency of the request
                  "cached_pairs_per_layer": cached, "cached_fraction": sum(cached) / float(wl.layers * wl.N),
                  "distinct_tokens": int(torch.unique(toks).numel()),
                  "phases": {k: {"ms_per_token": v[0] / prof_steps, "launches_per_token": v[1] / prof_steps}
                             for k, v in dphases.items() if k.startswith("dec_")}}
        gemv_ms = sum(decode["phases"][k]["ms_per_token"] for k in ("dec_qkv", "dec_o_proj", "dec_gate_up", "dec_down")
                      if k in decode["phases"])
        if gemv_ms > 0:
            decode["gemv_gbs"] = wbytes / (gemv_ms * 1e-3) / 1e9
            decode["gemv_hbm_frac"] = decode["gemv_gbs"] / PEAK_HBM_GBS
        log(f"[decode] {dms:.3f} ms/token ({1e3 / dms:.1f} tokens/s), {decode['gbs']:.0f} GB/s of weights + cache + table")
        # the same step over a batch of sequences (each with its own copy of the caches): the weights are read once per step
        if 2 <= args.decode_batch <= 16:
            nb = args.decode_batch
            bsteps = min(steps_d, 16)
            bc = []
            for _ in range(nb):
                seq = []
                for c0, cn in zip(caches, cached):
                    kc = runtime.KVCache(shape, cn + bsteps + 2)
                    kc.k[:cn].copy_(c0.k[:cn]); kc.v[:cn].copy_(c0.v[:cn]); kc.pos[:cn].copy_(c0.pos[:cn])
                    kc.struct.count = cn
                    seq.append(kc)
                bc.append(seq)
            bdec = runtime.BatchedDecodeRunner(ctx, shape, layers, bc, gamma_f, table)
            bdec.x.copy_(table[1:1 + nb])
            bdec.generate([wl.N] * nb, 1)
            torch.cuda.synchronize()
            e0.record()
            bdec.generate([wl.N + 1] * nb, bsteps)
            e1.record()
            torch.cuda.synchronize()
            bms = e0.elapsed_time(e1) / bsteps
            btot = wbytes + nb * kvbytes + head_bytes
            decode["batched"] = {"sequences": nb, "steps": bsteps, "ms_per_step": bms, "tokens_per_s": nb * 1e3 / bms,
                                 "gbs": btot / (bms * 1e-3) / 1e9, "hbm_frac": btot / (bms * 1e-3) / 1e9 / PEAK_HBM_GBS}
            log(f"[decode, batch of {nb}] {bms:.3f} ms/step = {nb * 1e3 / bms:.0f} tokens/s")
            del bc, bdec
        del caches, crunner, dec
        # the same decode over the full caches of a dense prefill (every layer keeps all N pairs): the library's own
        # baseline for the end-to-end figure
        if dense is not None:
            dsteps = min(steps_d, 16)
            dcaches = [runtime.KVCache(shape, wl.N + dsteps + 2) for _ in plan]
            dr = runtime.StackRunner(ctx, shape, layers, plan, wl.probe_len, wl.protect_last, skip=0, caches=dcaches)
            dr.run(x0, pos0)
            ddec = runtime.DecodeRunner(ctx, shape, layers, dcaches, gamma_f, table)
            ddec.x.copy_(table[1])
            ddec.generate(wl.N, 1)
            torch.cuda.synchronize()
            e0.record()
            ddec.generate(wl.N + 1, dsteps)
            e1.record()
            torch.cuda.synchronize()
            ddms = e0.elapsed_time(e1) / dsteps
            decode["dense_cache"] = {"steps": dsteps, "ms_per_token": ddms,
                                     "e2e_ms": dense["ms_per_step"] + steps_d * ddms,
                                     "e2e_speedup_spts_over_dense": (dense["ms_per_step"] + steps_d * ddms) / decode["e2e_ms"]}
            log(f"[decode, dense caches] {ddms:.3f} ms/token -> end-to-end speedup {decode['dense_cache']['e2e_speedup_spts_over_dense']:.2f}x "
                f"for {steps_d} tokens")
            del dcaches, dr, ddec
        del table

    # ---- component ablation over context lengths (paper schedules only)
    ablation = None
    if args.ablation and wl.stage_budgets:
        lengths = [n for n in (8192, 16384, 24576, 32768) if n <= wl.N]
        variants = ("dense", "pap", "pap+ltp", "full")
        ttft = {v: [] for v in variants}
        e2e = {"dense": [], "full": []}
        nsteps = max(2, min(args.steps, 5))
        table = runtime.to_device(synth.vocab_table(wl.seed, args.vocab, shape.D, shape.dtype), shape.dtype)
        gamma_f = runtime.to_device(np.ones(shape.D, dtype=np.float32), shape.dtype)

        def decode16(pl, skip_flag, n_tok, xs, ps):
            caches_ = [runtime.KVCache(shape, ((min(it["N"], it["m_attn"]) if it.get("skip", 1) else it["N"]) if skip_flag
                                               else n_tok) + 20) for it in pl]
            runtime.StackRunner(ctx, shape, layers, pl, wl.probe_len, wl.protect_last, skip=skip_flag, caches=caches_).run(xs, ps)
            d_ = runtime.DecodeRunner(ctx, shape, layers, caches_, gamma_f, table)
            d_.x.copy_(table[1])
            d_.generate(n_tok, 1)
            torch.cuda.synchronize()
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            d_.generate(n_tok + 1, 16)
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1)

        for n_tok in lengths:
            xs, ps = x0[:n_tok].contiguous(), pos0[:n_tok].contiguous()
            for v in variants:
                pl = synth.scaled(wl, N=n_tok, components="full" if v == "dense" else v).layer_plan()
                rn = runtime.StackRunner(ctx, shape, layers, pl, wl.probe_len, wl.protect_last, skip=0 if v == "dense" else 1)
                rn.run(xs, ps)
                torch.cuda.synchronize()
                a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a0.record()
                for _ in range(nsteps):
                    rn.run(xs, ps)
                a1.record()
                torch.cuda.synchronize()
                ttft[v].append(a0.elapsed_time(a1) / nsteps)
                if v in e2e:
                    e2e[v].append(ttft[v][-1] + decode16(pl, 0 if v == "dense" else 1, n_tok, xs, ps))
            log(f"[ablation] N={n_tok}: " + ", ".join(f"{v} {ttft[v][-1]:.1f} ms" for v in variants)
                + f"; e2e(16) dense {e2e['dense'][-1]:.1f} / full {e2e['full'][-1]:.1f} ms")
        ablation = {"lengths": lengths, "steps": nsteps, "ttft_ms": ttft,
                    "ttft_speedup_over_dense": {v: [d / t for d, t in zip(ttft["dense"], ttft[v])] for v in variants[1:]},
                    "e2e16_ms": e2e, "e2e16_speedup_over_dense": [d / t for d, t in zip(e2e["dense"], e2e["full"])]}
        del table

    # ---- batched TopK: one workgroup per row, so the whole chip streams scores (a single row is latency-bound)
    topk_batched = None
    if args.topk_batch > 0:
        tn, tb = 131072, args.topk_batch
        tk = int(0.4 * tn)
        tctx = runtime.make_context(synth.TINY, tn, 1, 1, synth.TINY.Dff)
        sc = torch.rand((tb, tn), dtype=torch.float32, device="cuda")
        ti = torch.empty((tb, tk), dtype=torch.int32, device="cuda")
        tctx.spts_select_topk_batched(sc, tn, tk, 1, tb, ti)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            tctx.spts_select_topk_batched(sc, tn, tk, 1, tb, ti)
        e1.record()
        torch.cuda.synchronize()
        tms = e0.elapsed_time(e1) / 3
        tbytes = tb * (4.0 * tn + 4.0 * tk)
        topk_batched = {"rows": tb, "N": tn, "k": tk, "ms": tms, "gbs": tbytes / (tms * 1e-3) / 1e9,
                        "hbm_frac": tbytes / (tms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                        "note": "algorithmic bytes (scores once + indices) / time; the kernel sweeps the scores three times (first sweep from HBM, the others from the memory-side cache)"}
        del sc, ti, tctx

    # ---- one skip layer over a batch of sequences: one batched call against one call per sequence
    batched = None
    if args.batch_seqs > 0 and wl.N >= 8192 * args.batch_seqs:
        from paper_2601_13155_amd import binding
        nb, ln = args.batch_seqs, 8192
        offs = [i * ln for i in range(nb + 1)]
        keep_a = wl.attn_keep if wl.attn_keep > 0 else 0.4
        keep_f = wl.ffn_keep if wl.ffn_keep > 0 else 0.4
        ma, mf = [int(keep_a * ln)] * nb, [int(keep_f * ln)] * nb
        xb = x0[:nb * ln].clone()
        pb = torch.cat([pos0[:ln]] * nb).contiguous()
        cfg1 = binding.spts_layer_cfg(1, wl.probe_len, ma[0], mf[0], wl.protect_last, 0)

        def run_batched():
            ctx.spts_layer_prefill_batched(xb, pb, offs, layers[0], wl.probe_len, ma, mf, wl.protect_last)

        def run_single():
            for i in range(nb):
                ctx.spts_layer_prefill(xb[i * ln:(i + 1) * ln], pb[i * ln:(i + 1) * ln], ln, layers[0], cfg1, None, None, None, None)

        res = {}
        for nm, fn in (("batched", run_batched), ("single_calls", run_single)):
            xb.copy_(x0[:nb * ln]); fn(); torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                fn()
            e1.record(); torch.cuda.synchronize()
            res[nm] = e0.elapsed_time(e1) / 3
        batched = {"sequences": nb, "tokens_per_sequence": ln, "ms_batched": res["batched"], "ms_single_calls": res["single_calls"],
                   "tokens_per_s_batched": nb * ln / (res["batched"] * 1e-3)}
        del xb, pb

    # ---- offline proxy construction: channel scores on a synthetic calibration set (rho = 0.2)
    builder = None
    if args.builder_tokens > 0:
        Tc = min(args.builder_tokens, wl.N)
        kc = max(1, int(0.2 * Tc))
        xc = runtime.to_device(synth.calibration_states(wl.seed, Tc, shape.D, shape.dtype), shape.dtype)
        imp = torch.zeros(shape.Dff, dtype=torch.float32, device="cuda")
        ctx.spts_channel_importance(xc, Tc, layers[0], kc, imp)
        torch.cuda.synchronize()
        ctx.spts_profile_begin()
        for _ in range(3):
            ctx.spts_channel_importance(xc, Tc, layers[0], kc, imp)
        torch.cuda.synchronize()
        bph = ctx.spts_profile_end()
        b = 2 if shape.dtype == "bf16" else 4
        sal_ms, top_ms = bph["build_saliency"][0] / 3, bph["build_topmean"][0] / 3
        builder = {"tokens": Tc, "k": kc, "saliency_ms": sal_ms, "saliency_tflops": 4.0 * Tc * shape.D * shape.Dff / (sal_ms * 1e-3) / 1e12,
                   "topmean_ms": top_ms, "topmean_gbs": (float(shape.Dff) * Tc * b + 4.0 * shape.Dff) / (top_ms * 1e-3) / 1e9}
        builder["topmean_hbm_frac"] = builder["topmean_gbs"] / PEAK_HBM_GBS
        del xc, imp

    cpu = None
    if args.cpu_sample_tokens > 0:
        cpu = cpu_baseline(wl, host_sets[0], args.cpu_sample_tokens)
        log(f"[cpu] oracle layer timings {cpu['seconds_per_sample']} s -> stack extrapolated {cpu['seconds_stack_extrapolated']:.0f} s")

    out = {
        "metric": "SPTS prefill tokens/s (TTFT = ms_per_step) at %dK, %s-shaped, 1 GPU%s" % (
            wl.N // 1024, "LLaMA-3.1-8B" if shape.D == 4096 else "Qwen2.5-7B",
            " (the paper's own schedule)" if wl.stage_budgets else ""),
        "value": wl.N / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "ttft_ms": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "seq_len": wl.N, "layers": wl.layers, "probe_len": wl.probe_len,
                   "attn_keep": wl.attn_keep, "ffn_keep": wl.ffn_keep, "proxy_rank": wl.r, "proxy_dlow": Dlow,
                   "dense_layers": wl.dense_layers, "stage_budgets": list(wl.stage_budgets), "stage_prune": wl.stage_prune,
                   "stage_end_layers": list(wl.stage_end_layers), "stage_cum_keep": list(wl.stage_cum_keep),
                   "components": wl.components, "weight_pool": pool, "batch": 1,
                   "proxy_channels": ("all" if not wl.dlow else "TopK of channel scores computed on the GPU" if args.builder_channels else "seeded random subset"),
                   "weight_layout": "row-major" if args.row_major_weights else "row-major + slab-major copies (spts_pack_slab32)"},
        "algorithmic_tflop_per_step": total_flops / 1e12,
        "achieved_tflops_whole_step": total_flops / (ms * 1e-3) / 1e12,
        "roofline": roofline, "cpu_baseline": cpu, "dense": dense, "phases": phase_out, "topk_batched": topk_batched, "decode": decode, "proxy_builder": builder, "ablation": ablation, "batched_layer": batched,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
