#!/usr/bin/env python3
"""Benchmark of the cached denoising step (dLLM-Cache) on one MI355X.

A "step" is one denoising step: one pass of the whole hot path (all layers: V-verify,
selection, partial recompute, cache scatter) over the batch.  Steps follow the workload's
schedule (step index i mod the schedule length), so --steps equal to the schedule length times
one whole generation with its mix of full-refresh, response-refresh and adaptive steps.
Inputs (embedded tokens of every schedule step) and weights are resident in HBM before the
timed region.  Prints one JSON line.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP32_VECTOR_PEAK_TFLOPS = 157.3   # 256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2 (dual issue) x 2.4 GHz
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
FP32_VALU_PEAK_TFLOPS = 157.3
# HBM bytes per launch of the streaming GEMM (reads + writes): NOT measured by this program.  The
# figure comes from separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this benchmark,
# scaled by the counters' reading for a 256 MiB copy (profiles/k_gemm_stream_<workload>_hbm_counters.txt);
# None where no such run has been recorded for the workload.
TRAFFIC_BYTES_PER_LAUNCH = {"llada8b": 114.8e6}
TRAFFIC_SOURCE = "profiles/k_gemm_stream_{name}_hbm_counters.txt (separate rocprofv3 --pmc runs, not this run)"


def make_denoiser(binding, cfg, weights, **over):
    return binding.CachedDenoiser(
        n_layers=cfg.T, d_model=cfg.d, n_q_heads=cfg.H_q, n_kv_heads=cfg.H_kv, head_dim=cfg.d_h,
        d_ffn=cfg.m, batch=cfg.B, dtype=cfg.dtype, weights=weights, L_p=cfg.L_p, L_r=cfg.L_r,
        rho=over.get("rho", cfg.rho), K_p=over.get("K_p", cfg.K_p), K_r=over.get("K_r", cfg.K_r),
        rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta)


def step_kind(cfg, i):
    P, R = i % cfg.K_p == 0, i % cfg.K_r == 0
    return "full" if P and R else "prompt+adaptive" if P else "response" if R else "adaptive"


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, dev_weights, hidden_host, sample_layers=8):
    """The CPU oracle timed on the host cores: one step of each kind on `sample_layers` layers,
    scaled to the full depth and to the schedule's kind counts."""
    import numpy as np
    from oracle import dllm_cache_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    Ls = min(sample_layers, cfg.T)
    ws = [{k: v.float().cpu().numpy().astype(np.float64) for k, v in dev_weights[l].items()}
          for l in range(Ls)]
    model = O.Model(Ls, cfg.d, cfg.H_q, cfg.H_kv, cfg.d_h, cfg.m, cfg.rms_eps, cfg.rope_theta)
    # K_p = 3, K_r = 2 visits the four step kinds in steps 0..3
    ora = O.CachedDenoiser(model, ws, cfg.B, cfg.L_p, cfg.L_r, cfg.rho, 3, 2,
                           storage="bf16" if cfg.dtype == "bf16" else "f64")
    kinds = ["full", "adaptive", "response", "prompt+adaptive"]
    t_kind = {}
    for i, kind in enumerate(kinds):
        t0 = time.perf_counter()
        ora.step(hidden_host[i % len(hidden_host)].astype(np.float64), i)
        t_kind[kind] = time.perf_counter() - t0
    counts = {k: 0 for k in kinds}
    for i in range(cfg.steps):
        counts[step_kind(cfg, i)] += 1
    sched_s = sum(counts[k] * t_kind[k] for k in kinds) * (cfg.T / Ls)
    return {
        "value": cfg.steps / sched_s, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
        "cpu_model": cpu_model(),
        "sample": (f"numpy float64 oracle, {Ls} of {cfg.T} layers, one step of each kind "
                   f"(full/adaptive/response/prompt+adaptive = "
                   f"{t_kind['full']:.2f}/{t_kind['adaptive']:.2f}/{t_kind['response']:.2f}/"
                   f"{t_kind['prompt+adaptive']:.2f} s), scaled by {cfg.T // Ls}x depth and the "
                   f"schedule's kind counts {counts}"),
        "response_tokens_per_s": cfg.B * cfg.L_r / sched_s,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: one schedule)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps (default: one schedule)")
    ap.add_argument("--config", default="llada8b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-uncached", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (reference for HBM counters)")
    ap.add_argument("--no-probes", action="store_true", help="skip the achievable-peak probes")
    ap.add_argument("--no-closed-loop", action="store_true",
                    help="skip the closed-loop generation leg (embedding, head, remasking)")
    ap.add_argument("--rho", type=float, default=None, help="update ratio instead of the workload's")
    ap.add_argument("--layer-rho", default="", help="first,last: update ratio per layer on a straight "
                    "line from the first to the last layer (cross-layer allocation study)")
    ap.add_argument("--policy", default="", help="variant of the paper's ablations, e.g. "
                    "source=k,metric=l2,selection=random,v_update=selected,seed=1")
    ap.add_argument("--tune", default="", help="GEMM tuning knobs, e.g. nw=8,nw_dual=4,force_s=0,target_wg=256")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (sequences would shard across GPUs "
              "with no exchange step; not built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_06295_amd import binding, inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    cfg = I.CONFIGS[args.config]
    if args.rho is not None:
        cfg = cfg.replace(rho=args.rho)
    if args.tune:
        binding.set_gemm_tuning(**{k: int(v) for k, v in (kv.split("=") for kv in args.tune.split(","))})
    K = args.steps if args.steps is not None else cfg.steps
    W = args.warmup if args.warmup is not None else cfg.steps

    if args.calibration_copy:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    weights = I.device_weights(cfg)
    sched = I.TokenSchedule(cfg)
    hidden_host = [sched.hidden_in(i) for i in range(cfg.steps)]
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    hidden = [torch.from_numpy(h).cuda().to(tdt).contiguous() for h in hidden_host]
    out = torch.empty_like(hidden[0])
    den = make_denoiser(binding, cfg, weights)
    variant = {}
    if args.policy:
        variant = {k: (int(v) if k == "seed" else v) for k, v in (kv.split("=") for kv in args.policy.split(","))}
        den.set_policy(**variant)
    if args.layer_rho:
        first, last = (float(v) for v in args.layer_rho.split(","))
        ratios = [first + (last - first) * l / max(cfg.T - 1, 1) for l in range(cfg.T)]
        den.set_layer_rho(ratios)
        variant["layer_rho"] = [first, last]

    def run(count, start=0):
        for s in range(start, start + count):
            i = s % cfg.steps
            den.step(hidden[i], i, out)

    # warm-up, then the timed region: exactly K steps between two device synchronisations
    w_aligned = W
    run(w_aligned)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K, start=w_aligned)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kinds_timed = {}
    for s in range(w_aligned, w_aligned + K):
        kinds_timed[step_kind(cfg, s % cfg.steps)] = kinds_timed.get(step_kind(cfg, s % cfg.steps), 0) + 1

    # Every step kind on its own, whatever slice of the schedule the flags picked: groups of
    # same-kind steps (ascending step indices of that kind; step 0 may be repeated, it starts a
    # new generation) between two synchronisations, median of three groups.  The headline is the
    # whole schedule: its kind counts weighted with these per-kind times.
    KINDS = ("full", "prompt+adaptive", "response", "adaptive")
    counts = {k: 0 for k in KINDS}
    for i in range(cfg.steps):
        counts[step_kind(cfg, i)] += 1
    cursor = [0]

    def indices_of(kind, reps):
        out_idx = []
        for _ in range(reps):
            if kind == "full":
                i = 0
            else:
                i = cursor[0] + 1
                while step_kind(cfg, i) != kind:
                    i += 1
            cursor[0] = i
            out_idx.append(i)
        return out_idx

    def run_indices(idx):
        for i in idx:
            den.step(hidden[i % cfg.steps], i, out)

    group = {"full": 2, "prompt+adaptive": 2, "response": 4, "adaptive": 12}
    den.step(hidden[0], 0, out)
    ms_kind = {}
    for kind in KINDS:
        if counts[kind] == 0:
            continue
        ts = []
        for _ in range(3):
            run_indices(indices_of(kind, 1))   # the kind's kernels warm
            idx = indices_of(kind, group[kind])
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            run_indices(idx)
            torch.cuda.synchronize()
            ts.append(1e3 * (time.perf_counter() - t1) / len(idx))
        ms_kind[kind] = float(np.median(ts))
    sched_ms = sum(counts[k] * ms_kind[k] for k in ms_kind)
    steps_per_s = cfg.steps / (sched_ms * 1e-3)

    result = {
        "metric": "cached denoise steps/s",
        "value": steps_per_s,
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": sched_ms / cfg.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} heads={cfg.H_q}/{cfg.H_kv}x{cfg.d_h} "
                               f"m={cfg.m} B={cfg.B} L_p={cfg.L_p} L_r={cfg.L_r} rho={cfg.rho} "
                               f"K_p={cfg.K_p} K_r={cfg.K_r} schedule={cfg.steps} steps",
                   "seed": cfg.seed, "variant": variant or None},
        "value_is": "whole schedule: the schedule's step-kind counts weighted with the time of each "
                    "kind measured on its own (ms_per_step_kind), so it does not depend on which "
                    "slice --steps/--warmup pick; timed_slice is the literal K-step region",
        "schedule_kind_counts": counts,
        "ms_per_step_kind": ms_kind,
        "ms_per_schedule": sched_ms,
        "timed_slice": {"steps": K, "warmup": W, "ms_per_step": 1e3 * elapsed / K,
                        "steps_per_s": K / elapsed, "step_kinds": kinds_timed},
        "response_tokens_per_s": cfg.B * cfg.L_r / (sched_ms * 1e-3),
        "token_rows_per_s": cfg.B * cfg.L_r * steps_per_s,
    }

    # per-kernel pass over the same K steps with HIP events around every launch
    if not args.no_profile:
        run(w_aligned)   # a fresh generation up to the first timed step (step 0 restarts the schedule)
        den.profile_enable(True)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
        spans_per_step, seen = [], 0
        for j, s in enumerate(range(w_aligned, w_aligned + K)):
            i = s % cfg.steps
            ev[j][0].record()
            den.step(hidden[i], i, out)
            ev[j][1].record()
            # cumulative span count (the read waits for the stream; the totals keep adding up)
            tot = den.profile_read(reset=False)
            n_now = sum(v["launches"] for k, v in tot.items() if k != "k_gemm_stream")
            spans_per_step.append(n_now - seen)
            seen = n_now
        stats = den.profile_read(reset=True)
        den.profile_enable(False)
        # One event record sits between consecutive kernels and lengthens every span.  What it
        # adds per launch is measured on the run itself: the spans of the profiled pass add up to
        # its duration, the timed region above ran the same K steps without events, and the
        # difference divided by the number of spans is the cost of one event.  (The library also
        # reports an empty span per step, two events back to back: an upper bound, since nothing
        # overlaps with them.)
        empty = stats.pop("event_overhead")
        dup = stats["k_gemm_stream"]  # the same spans a second time
        raw_ms = sum(v["ms"] for v in stats.values()) - dup["ms"] + empty["ms"]
        n_spans = sum(v["launches"] for v in stats.values()) - dup["launches"] + empty["launches"]
        ov_ms = max(raw_ms - 1e3 * elapsed, 0.0) / max(n_spans, 1)
        for v in stats.values():
            v["ms_raw"] = v["ms"]
            v["ms"] = max(v["ms"] - ov_ms * v["launches"], 0.0)
        # per step kind, with the events of the step taken out the same way
        per_kind, per_kind_raw = {}, {}
        for j, s in enumerate(range(w_aligned, w_aligned + K)):
            kind = step_kind(cfg, s % cfg.steps)
            raw = ev[j][0].elapsed_time(ev[j][1])
            per_kind_raw.setdefault(kind, []).append(raw)
            per_kind.setdefault(kind, []).append(raw - ov_ms * spans_per_step[j])
        result["timed_slice"]["ms_per_step_kind_events_removed"] = {k: float(np.median(v)) for k, v in per_kind.items()}
        result["timed_slice"]["ms_per_step_kind_with_events"] = {k: float(np.median(v)) for k, v in per_kind_raw.items()}
        # the dominant kernel: every launch of the weight-streaming GEMM kernel (the library
        # counts those launches a second time under their kernel's name)
        ks = stats.pop("k_gemm_stream")
        stats.pop("head_gemm", None)   # closed-loop classes: empty in this pass
        stats.pop("gen_other", None)
        gemm = [stats[k] for k in ("gemm_v", "gemm_qk", "gemm_o", "gemm_gate_up", "gemm_down")]
        total_ms = sum(v["ms"] for v in stats.values())
        k_ms, k_n = ks["ms"], max(ks["launches"], 1)
        achieved = ks["alg_bytes"] / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
        traffic = TRAFFIC_BYTES_PER_LAUNCH.get(cfg.name)
        result["roofline"] = {
            "kernel": "k_gemm_stream (every launch: fused gate/up, Q|K, output and down projections "
                      "of the recomputed rows)",
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "traffic_source": TRAFFIC_SOURCE.format(name=cfg.name) if traffic else None,
            "launches": ks["launches"], "avg_launch_us": 1e3 * k_ms / k_n,
            "avg_launch_us_with_event": 1e3 * ks["ms_raw"] / k_n,
            "event_overhead_us": 1e3 * ov_ms,
            "empty_span_us": 1e3 * empty["ms"] / max(empty["launches"], 1),
            "alg_bytes_per_launch": ks["alg_bytes"] / k_n,
            "mfma_tflops": ks["flops"] / (k_ms * 1e-3) / 1e12 if k_ms > 0 else 0.0,
            "share_of_kernel_time": k_ms / total_ms if total_ms > 0 else 0.0,
        }
        g_ms = sum(g["ms"] for g in gemm)
        if k_ms < 0.5 * g_ms:
            # many rows per launch (batched sequences): the LDS-direct tile kernels carry the
            # GEMM time and the matrix cores, not HBM, bound them
            t_ms = g_ms - k_ms
            t_fl = sum(g["flops"] for g in gemm) - ks["flops"]
            t_n = sum(g["launches"] for g in gemm) - ks["launches"]
            tf = t_fl / (t_ms * 1e-3) / 1e12 if t_ms > 0 else 0.0
            f32 = cfg.dtype == "f32"   # float32 models run the plain vector-ALU GEMM
            peak = FP32_VECTOR_PEAK_TFLOPS if f32 else MFMA_BF16_PEAK_TFLOPS
            result["roofline"] = {
                "kernel": ("k_gemm_simple (float32, vector ALU)" if f32 else
                           "k_gemm_fat / k_gemm_mid (every launch of the LDS-direct tile kernels)"),
                "bound": "alu" if f32 else "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s",
                "frac": tf / peak, "traffic": None, "launches": t_n,
                "avg_launch_us": 1e3 * t_ms / max(t_n, 1), "event_overhead_us": 1e3 * ov_ms,
                "flops_per_launch": t_fl / max(t_n, 1),
                "share_of_kernel_time": t_ms / total_ms if total_ms > 0 else 0.0,
            }
        result["all_gemms"] = {
            "launches": sum(g["launches"] for g in gemm), "ms_total": g_ms,
            "GBps": sum(g["alg_bytes"] for g in gemm) / (g_ms * 1e-3) / 1e9 if g_ms > 0 else 0.0,
            "TFLOPs": sum(g["flops"] for g in gemm) / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0,
            "share_of_kernel_time": g_ms / total_ms if total_ms > 0 else 0.0,
        }
        result["kernels"] = {
            k: {"launches": v["launches"], "ms_total": v["ms"],
                "avg_us": 1e3 * v["ms"] / max(v["launches"], 1),
                "GBps": (v["alg_bytes"] / (v["ms"] * 1e-3) / 1e9) if v["ms"] > 0 else 0.0,
                "TFLOPs": (v["flops"] / (v["ms"] * 1e-3) / 1e12) if v["ms"] > 0 else 0.0}
            for k, v in stats.items()}
        result["kernel_time_ms_per_step"] = total_ms / K
        # the same per kernel class for every step kind on its own (average us per launch, the
        # event's share removed)
        by_kind = {}
        den.step(hidden[0], 0, out)
        cursor[0] = 0
        for kind in ms_kind:
            run_indices(indices_of(kind, 1))
            den.profile_enable(True)
            run_indices(indices_of(kind, max(group[kind] // 2, 1)))
            st_k = den.profile_read(reset=True)
            den.profile_enable(False)
            by_kind[kind] = {k: {"launches": v["launches"],
                                 "avg_us": 1e3 * max(v["ms"] - ov_ms * v["launches"], 0.0) / v["launches"]}
                             for k, v in st_k.items() if v["launches"] and k != "event_overhead"}
        result["kernels_by_kind"] = by_kind

    # what this GPU delivers for the plainest kernels (1 GiB copy, 1 GiB read, MFMA loop from
    # registers): the measured ceilings beside the published peaks
    if not args.no_probes:
        n_probe = 1 << 30
        src = torch.empty(n_probe, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        sink = torch.zeros(256, dtype=torch.float32, device="cuda")

        def timed(fn, reps=10):
            for _ in range(2):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ts = []
            for _ in range(reps):
                a.record()
                fn()
                b.record()
                b.synchronize()
                ts.append(a.elapsed_time(b) * 1e-3)
            return float(np.median(ts))

        t_copy = timed(lambda: binding.probe_copy(src, dst))
        t_read = timed(lambda: binding.probe_read(src, sink))
        fl = [0.0]

        def mfma():
            fl[0] = binding.probe_mfma(4096, sink)
        t_mfma = timed(mfma)
        fl32 = [0.0]

        def mfma32():
            fl32[0] = binding.probe_mfma(4096, sink, shape=1)
        t_mfma32 = timed(mfma32)
        copy_gbs, read_gbs, mfma_tf = 2 * n_probe / t_copy / 1e9, n_probe / t_read / 1e9, fl[0] / t_mfma / 1e12
        result["achievable"] = {
            "copy_GBps": copy_gbs, "read_GBps": read_gbs, "mfma_bf16_TFLOPs": mfma_tf,
            "mfma_bf16_32x32x16_TFLOPs": fl32[0] / t_mfma32 / 1e12,
            "note": "1 GiB plain copy (bytes in + bytes out), 1 GiB plain read, back-to-back "
                    "16x16x32 / 32x32x16 bf16 MFMAs from registers; median of 10 launches",
        }
        rf = result.get("roofline")
        if rf:
            ceil = read_gbs if rf["bound"] == "hbm" else max(mfma_tf, fl32[0] / t_mfma32 / 1e12)
            rf["frac_of_measured_ceiling"] = rf["achieved"] / ceil if ceil > 0 else None
            rf["measured_ceiling"] = ceil
        del src, dst

    # the uncached forward on the same GPU: rho = 1, K_p = K_r = 1
    if not args.no_uncached:
        from oracle.dllm_cache_oracle import flops_uncached_step
        unc = make_denoiser(binding, cfg, weights, rho=1.0, K_p=1, K_r=1)
        for i in range(2):
            unc.step(hidden[i], i, out)
        torch.cuda.synchronize()
        reps = 6
        t0 = time.perf_counter()
        for i in range(reps):
            unc.step(hidden[i % cfg.steps], 2 + i, out)
        torch.cuda.synchronize()
        t_unc = (time.perf_counter() - t0) / reps
        unc.close()
        fl = cfg.B * flops_uncached_step(cfg.T, cfg.n, cfg.d, cfg.m)
        result["uncached_gpu"] = {
            "ms_per_step": 1e3 * t_unc, "steps_per_s": 1.0 / t_unc,
            "tflops": fl / t_unc / 1e12, "mfma_frac": fl / t_unc / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "speedup_schedule": 1e3 * t_unc / result["ms_per_step"],
        }
        if "adaptive" in ms_kind:
            result["uncached_gpu"]["speedup_adaptive_step"] = 1e3 * t_unc / ms_kind["adaptive"]

    # the closed loop: the same schedule driven by the model's own predictions (embedding
    # gather, cached step, mask-predictor head over the full vocabulary, remasking transition),
    # tokens never leave the device
    if not args.no_closed_loop:
        from paper_2506_06295_amd.inputs import device_head_weights, initial_tokens
        hw = device_head_weights(cfg)
        gen = binding.Generator(den, hw["embed"], hw["final_norm_g"], hw["lm_head"], cfg.steps,
                                cfg.block_len)
        tok0 = torch.from_numpy(initial_tokens(cfg).astype(np.int32)).cuda()

        def generation():
            tok = tok0.clone()
            for i in range(cfg.steps):
                gen.step(tok, i)
            return tok

        generation()
        torch.cuda.synchronize()
        reps = max(1, min(3, (K + cfg.steps - 1) // cfg.steps))
        t0 = time.perf_counter()
        for _ in range(reps):
            tok = generation()
        torch.cuda.synchronize()
        t_gen = (time.perf_counter() - t0) / reps
        head_bytes = cfg.vocab * cfg.d * (4 if cfg.dtype == "f32" else 2)
        result["closed_loop"] = {
            "ms_per_generation": 1e3 * t_gen, "steps_per_s": cfg.steps / t_gen,
            "response_tokens_per_s": cfg.B * cfg.L_r / t_gen,
            "ms_per_step_beyond_core_path": 1e3 * t_gen / cfg.steps - result["ms_per_step"],
            "vocab": cfg.vocab, "block_len": cfg.block_len or cfg.L_r,
            "lm_head_bytes_per_step": head_bytes,
            "all_revealed": bool((tok[:, cfg.L_p:] != cfg.vocab).all().item()),
        }
        if not args.no_profile:
            # one generation with events: the vocabulary projection on its own
            den.profile_enable(True)
            generation()
            gst = den.profile_read(reset=True)
            den.profile_enable(False)
            hg, go = gst["head_gemm"], gst["gen_other"]
            h_ms = max(hg["ms"] - result["roofline"]["event_overhead_us"] * 1e-3 * hg["launches"], 1e-9)
            result["closed_loop"]["head_gemm"] = {
                "launches": hg["launches"], "avg_us": 1e3 * h_ms / max(hg["launches"], 1),
                "GBps": hg["alg_bytes"] / (h_ms * 1e-3) / 1e9,
                "hbm_frac": hg["alg_bytes"] / (h_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "TFLOPs": hg["flops"] / (h_ms * 1e-3) / 1e12}
            result["closed_loop"]["other_kernels_ms_per_step"] = go["ms"] / cfg.steps
        gen.close()
        del hw, gen

    den.close()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, weights, hidden_host)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
