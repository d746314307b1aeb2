#!/usr/bin/env python3
"""Throughput of entropy-adaptive decoding on one MI355X.

A "step" is one iteration of Algorithm 1's loop for every sequence of the batch: the
active model's forward pass over the KV cache (plus any catch-up it owes), the fused
LM-head entropy / arg-max epilogue, the rolling window and the switch rule.  Prompt
prefill is outside the timed region; all inputs are resident in HBM when timing starts.

Prints ONE JSON line: tokens/s (whole job), the decode path's algorithmic HBM rate,
the large-model token share, a roofline entry for the dominant kernel (HIP-event
timing of its launches on the library's stream) and the CPU oracle's rate on a bounded
sample of the same workload.
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

import synth_inputs as si  # noqa: E402

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E peak

WORKLOADS = {
    # name: (pair, batch, prompt_lo, prompt_hi, default_steps, target_large_share, d_min)
    "llama_1b_8b_b1": ("llama", 1, 512, 512, 1024, 0.40, 10),
    "qwen_05b_14b_b32": ("qwen", 32, 256, 256, 256, 0.25, 10),
    "qwen_05b_14b_b64": ("qwen", 64, 128, 1024, 128, 0.25, 10),
    "tiny_fp32_b1": ("tiny", 1, 16, 16, 64, 0.40, 10),
    # the paper's other pair shapes, batch 1
    "llama_1b_3b_b1": ("llama_1b_3b", 1, 512, 512, 1024, 0.40, 10),
    "qwen_15b_14b_b1": ("qwen_15b_14b", 1, 512, 512, 1024, 0.25, 10),
    # stand-alone entropy / arg-max / window / switch epilogue on materialised logits
    "entropy_gate_b64": (None, 64, 0, 0, 4096, None, 10),
    # prompt prefill of both models (the step before the decode path): steps = repetitions
    "prefill_qwen_b64": ("qwen", 64, 128, 1024, 4, None, 10),
    "prefill_llama_b8": ("llama", 8, 512, 512, 8, None, 10),
}

MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def make_prompts(seed, batch, lo, hi, vocab):
    lens = si.prompt_lengths(seed, batch, lo, hi) if hi > lo else np.full(batch, lo, np.int32)
    return [si.prompt_np(seed, f"row{b}", int(lens[b]), vocab) for b in range(batch)]


def calibrate_tau(e, prompts, n_tokens, w, d_min, target):
    """Bisection on free-running calibration runs: tau such that about `target` of the
    tokens come from the large model (the percentile of the small model's windowed
    entropy is only the starting bracket, because the window is shared across switches)."""
    e.set_gate(w, 1e30, d_min)
    probe = e.generate(prompts, n_tokens)
    hb = probe["Hbar"].ravel()
    lo, hi = float(hb.min()) - 1.0, float(hb.max()) + 1e-3
    best = (2.0, hi)
    for _ in range(12):
        tau = 0.5 * (lo + hi)
        e.set_gate(w, tau, d_min)
        share = float(e.generate(prompts, n_tokens)["model_id"].mean())
        if abs(share - target) < abs(best[0] - target):
            best = (share, tau)
        if share > target:
            lo = tau            # too many large tokens: raise the threshold
        else:
            hi = tau
        if abs(share - target) < 0.02:
            break
    return best[1], best[0]


def cpu_baseline(pair_shapes, Ws, Wl, prompts, w, tau, d_min):
    """The oracle as it stands, timed on this host: Algorithm 1 on a bounded sample (first
    row, prompt cut to 16 tokens, 24 generated tokens); prompt handling is subtracted by
    timing a 1-token run."""
    import oracle
    ss, sl = pair_shapes
    t0 = time.time()
    os_ = oracle.Model(ss, {k: v.float().cpu().numpy() for k, v in Ws.items()})
    ol = oracle.Model(sl, {k: v.float().cpu().numpy() for k, v in Wl.items()})
    log(f"[cpu_baseline] weights on host in {time.time() - t0:.1f}s")
    prompt = prompts[0][:16]
    n = 24
    t0 = time.time(); oracle.generate(os_, ol, prompt, 1, w, tau, d_min); t1 = time.time()
    out = oracle.generate(os_, ol, prompt, n + 1, w, tau, d_min); t2 = time.time()
    dt = max((t2 - t1) - (t1 - t0), 1e-9)
    return {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"row 0, prompt cut to 16 tokens, {n} generated tokens after the first, batch 1, "
                      f"same w/tau/d_min; large share in sample {float(out['model_id'][1:].mean()):.2f}"}


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter runs, or None when
    there is none for this workload/kernel or the kernel sources changed since it was taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    h = hashlib.sha256()
    for f in ("common.hpp", "linear.hpp"):
        h.update(open(os.path.join(ROOT, "paper_2502_06833_amd", "csrc", f), "rb").read())
    if rec.get("kernel") != kernel or rec.get("kernel_source_sha256_16") != h.hexdigest()[:16]:
        return None
    return rec["traffic_bytes_per_launch"]


def linear_params(shape):
    """Parameters of the per-layer matrices (what a prompt position multiplies; no embedding, no LM head)."""
    hd = shape.d_model // shape.n_heads
    per_layer = shape.d_model * (shape.n_heads + 2 * shape.n_kv_heads) * hd + shape.n_heads * hd * shape.d_model \
        + 3 * shape.d_model * shape.d_ffn
    return per_layer * shape.n_layers


def bench_prefill(args):
    """Prompt prefill of both models (ead_begin): every prompt position but the last through all layers of
    the small and of the large model, in passes of up to 1024 rows; no LM head.  Reported against the dense
    bf16 matrix-core peak with the algorithmic flops 2 * parameters * positions (the second product per
    weight tile, for the low parts of the activations, is not counted) plus the causal attention flops."""
    import torch
    import paper_2502_06833_amd as ead
    pair, batch, plo, phi, dsteps, _, d_min = WORKLOADS[args.workload]
    reps = args.steps or dsteps
    ss, sl = si.PAIRS[pair]
    Ws = si.model_weights_torch(ss, args.seed, "cuda")
    Wl = si.model_weights_torch(sl, args.seed, "cuda")
    prompts = make_prompts(args.seed, batch, plo, phi, ss.vocab)
    e = ead.EAD(ss, Ws, sl, Wl, window=5, tau=0.0, d_min=d_min, max_batch=batch, max_seq=max(len(p) for p in prompts) + 16)
    del Ws, Wl
    torch.cuda.empty_cache()
    for _ in range(max(1, min(args.warmup, 2))):
        e.begin(prompts, 8)
    torch.cuda.synchronize()
    a = time.perf_counter()
    for _ in range(reps):
        e.begin(prompts, 8)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - a) / reps
    n_pos = sum(len(p) - 1 for p in prompts)
    flops = 0.0
    for sh in (ss, sl):
        hd = sh.d_model // sh.n_heads
        flops += 2.0 * linear_params(sh) * n_pos
        flops += sum(4.0 * sh.n_layers * sh.n_heads * hd * (len(p) - 1) * len(p) / 2.0 for p in prompts)
    tfl = flops / dt / 1e12
    log(f"[bench] prefill: {n_pos} prompt positions through both models in {dt * 1e3:.1f} ms = {n_pos / dt:.0f} positions/s, "
        f"{tfl:.0f} Tflop/s algorithmic ({tfl / MFMA_PEAK_TFLOPS:.1%} of the dense bf16 peak)")
    out = {"metric": "prompt positions/s at 1 GPU (prefill of both models)", "value": n_pos / dt, "unit": "positions/s",
           "n_gpus": 1, "steps": reps, "warmup": min(args.warmup, 2), "ms_per_step": dt * 1e3, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": args.workload, "small": ss.name, "large": sl.name, "batch": batch,
                      "prompt_len": [plo, phi], "positions": n_pos},
           "roofline": {"bound": "mfma", "achieved": tfl, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": tfl / MFMA_PEAK_TFLOPS, "traffic": None},
           "cpu_baseline": None}
    e.close()
    print(json.dumps(out), flush=True)


def bench_entropy_gate(args):
    """bf16 logits [64, 151936], row scales U[0.5, 8] (entropies from near 0 to near ln V), a pool
    of 32 distinct tensors (622 MB, larger than the 256 MB Infinity Cache) cycled for `steps`
    steps; every step = entropy + arg max of 64 rows, window w=5, tau=2.0 nats, d_min=10."""
    import torch
    import paper_2502_06833_amd as ead
    rows, V, w, tau, d_min, pool_n = 64, 151936, 5, 2.0, 10, 32
    steps, warmup = args.steps or 4096, max(args.warmup, 64)
    pool = [si.logits_torch(args.seed + i, "cfg2", rows, V, torch.bfloat16, "cuda") for i in range(pool_n)]
    g = ead.Gate(rows, w, tau, d_min)
    g.run_logits(pool, warmup, want_outputs=False)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a = time.perf_counter()
    e0.record()
    _, _, mid, _ = g.run_logits(pool, steps)
    e1.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - a
    ev_ms = e0.elapsed_time(e1)
    share = mid.float().mean()
    per_step_us = 1e3 * ev_ms / steps
    bytes_step = rows * V * 2
    out = {
        "metric": "generated tokens/s at 1 GPU", "value": rows * steps / dt, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * dt / steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "entropy_gate_b64", "rows": rows, "vocab": V, "window": w, "tau_nats": tau,
                   "d_min": d_min, "pool_tensors": pool_n},
        "large_token_share": float(share.item()), "event_ms_total": ev_ms,
        "roofline": {"bound": "hbm", "kernel": "entropy_partial (+ gate_step), 16 steps per launch pair",
                     "achieved": bytes_step / per_step_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": bytes_step / per_step_us / 1e3 / HBM_PEAK_GBS, "traffic": None,
                     "avg_launch_us": per_step_us, "bytes_per_launch": bytes_step, "launches": steps},
    }
    if not args.no_cpu_baseline:
        import oracle
        ref = si.logits_np(args.seed, "cfg2", rows, V)
        t0 = time.time()
        n = 0
        while time.time() - t0 < 10.0:
            oracle.entropy_rows(ref)
            n += rows
        out["cpu_baseline"] = {"value": n / (time.time() - t0), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "sample": "entropy + arg max of the 64 rows of one tensor, repeated for 10 s (single thread)"}
    g.close()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="llama_1b_8b_b1", choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-single-model", action="store_true", help="skip the small-only / large-only runs")
    ap.add_argument("--profile-steps", type=int, default=64)
    ap.add_argument("--fused", type=int, default=None, help="1/0: force the fused single-row decode kernel on/off")
    ap.add_argument("--tau", type=float, default=None, help="skip the calibration runs and use this threshold (nats)")
    ap.add_argument("--schedule", choices=["lockstep", "grouped"], default="lockstep",
                    help="grouped: small-model rows run ahead, large-model rows are served together")
    ap.add_argument("--sched-start", type=float, default=0.5, help="grouped: large model starts at this share of waiting rows")
    ap.add_argument("--sched-stop", type=float, default=0.25, help="grouped: ... and stops below this share")
    ap.add_argument("--temperature", type=float, default=0.0, help="sample at this temperature (0 = greedy, the default)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (sequences are independent, so more GPUs "
                 "would each run this same program on their share of the batch); use --gpus 1")

    import torch
    import paper_2502_06833_amd as ead
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.workload == "entropy_gate_b64":
        return bench_entropy_gate(args)
    if args.workload.startswith("prefill_"):
        return bench_prefill(args)
    pair, batch, plo, phi, dsteps, target, d_min = WORKLOADS[args.workload]
    steps = args.steps or dsteps
    warmup = args.warmup
    w = 5
    ss, sl = si.PAIRS[pair]
    t0 = time.time()
    Ws = si.model_weights_torch(ss, args.seed, "cuda")
    Wl = si.model_weights_torch(sl, args.seed, "cuda")
    torch.cuda.synchronize()
    log(f"[bench] weights generated in {time.time() - t0:.1f}s")
    prompts = make_prompts(args.seed, batch, plo, phi, ss.vocab)
    max_seq = max(len(p) for p in prompts) + warmup + steps + 8
    e = ead.EAD(ss, Ws, sl, Wl, window=w, tau=0.0, d_min=d_min, max_batch=batch, max_seq=max_seq)
    if args.no_cpu_baseline:
        del Ws, Wl
        torch.cuda.empty_cache()
    log(f"[bench] handle created at {time.time() - t0:.1f}s")
    if args.fused is not None:
        e.set_fused(bool(args.fused))
    if args.temperature > 0:
        e.set_sampling(args.temperature, args.seed)

    if args.copy_probe:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.tau is not None:
        tau = args.tau
        log(f"[bench] tau={tau:.6f} nats (given)")
    else:
        n_cal = min(256, warmup + steps)
        tau, share_cal = calibrate_tau(e, prompts, n_cal, w, d_min, target)
        log(f"[bench] tau={tau:.6f} nats -> large share {share_cal:.3f} over {n_cal} calibration tokens "
            f"at {time.time() - t0:.1f}s")

    def timed(force, grouped=False):
        e.force_model(force)
        e.set_schedule(grouped, args.sched_start, args.sched_stop)
        e.set_gate(w, tau, d_min)
        e.begin(prompts, warmup + steps)
        e.decode(warmup)
        e.reset_stats()
        torch.cuda.synchronize()
        a = time.perf_counter()
        e.decode(steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - a
        st = e.stats()
        e.force_model(-1)
        e.set_schedule(False)
        return dt, st

    grouped = args.schedule == "grouped"
    dt, st = timed(-1, grouped)
    n_tok = st["tokens_small"] + st["tokens_large"]
    tok_s = n_tok / dt
    algo_gbs = st["algorithmic_bytes"] / dt / 1e9
    log(f"[bench] EAD: {tok_s:.1f} tok/s, {algo_gbs:.0f} GB/s algorithmic ({algo_gbs / HBM_PEAK_GBS:.1%} of peak), "
        f"large share {st['large_share']:.3f}, switches {st['switches']}, host syncs {st['host_syncs']}")
    extra = {}
    if grouped:
        d1, s1 = timed(-1, False)
        n1 = s1["tokens_small"] + s1["tokens_large"]
        extra["lockstep"] = {"tokens_per_s": n1 / d1, "large_passes": s1["steps_large"], "small_passes": s1["steps_small"]}
        extra["grouped"] = {"start": args.sched_start, "stop": args.sched_stop, "large_passes": st["steps_large"],
                            "small_passes": st["steps_small"]}
        log(f"[bench] lock step: {n1 / d1:.1f} tok/s with {s1['steps_large']} large / {s1['steps_small']} small passes; "
            f"grouped: {st['steps_large']} / {st['steps_small']}")
    if not args.no_single_model:
        for name, which in (("small_only", 0), ("large_only", 1)):
            d2, s2 = timed(which)
            n2 = s2["tokens_small"] + s2["tokens_large"]
            extra[name] = {"tokens_per_s": n2 / d2, "hbm_frac": s2["algorithmic_bytes"] / d2 / 1e9 / HBM_PEAK_GBS}
            log(f"[bench] {name}: {n2 / d2:.1f} tok/s, {extra[name]['hbm_frac']:.1%} of HBM peak")

    # ---- per-kernel HIP-event timing on a separate, untimed run ----
    e.set_gate(w, tau, d_min)
    e.begin(prompts, warmup + args.profile_steps)
    e.decode(warmup)
    e.profile(True)
    e.decode(args.profile_steps)
    prof = e.profile_read()
    e.profile(False)
    by_kind = {}
    for r in prof:
        k = r["name"].split("/")[0]
        a = by_kind.setdefault(k, {"launches": 0, "total_ms": 0.0, "bytes": 0.0})
        a["launches"] += r["launches"]; a["total_ms"] += r["total_ms"]; a["bytes"] += r["bytes"]
    for r in sorted(prof, key=lambda r: -r["total_ms"]):
        gbs = r["bytes"] / max(r["total_ms"], 1e-9) / 1e6
        log(f"[prof] {r['name']:<28s} n={r['launches']:<6d} avg {1e3 * r['total_ms'] / r['launches']:8.2f} us  "
            f"{gbs:8.0f} GB/s")
    # the dominant kernel is reported per model (one kernel, one shape): the one that moves the most
    # bytes over the pass, which does not flip with timing noise the way a ranking by time can
    dom = max(prof, key=lambda r: r["bytes"])["name"]
    d = next(r for r in prof if r["name"] == dom)
    achieved = d["bytes"] / d["total_ms"] / 1e6
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(args.workload, dom),
                "avg_launch_us": 1e3 * d["total_ms"] / d["launches"],
                "bytes_per_launch": d["bytes"] / d["launches"], "launches": d["launches"]}

    out = {
        "metric": "generated tokens/s at 1 GPU", "value": tok_s, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * dt / steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if ss.bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "small": ss.name, "large": sl.name, "batch": batch,
                   "prompt_len": [int(plo), int(phi)], "window": w, "d_min": d_min, "tau_nats": tau,
                   "vocab": ss.vocab, "schedule": args.schedule, "temperature": args.temperature},
        "decode_hbm_gbs": algo_gbs, "decode_hbm_frac_of_peak": algo_gbs / HBM_PEAK_GBS,
        "large_token_share": st["large_share"], "param_ratio": st["param_ratio"], "switches": st["switches"],
        "host_syncs": st["host_syncs"], **extra, "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline((ss, sl), Ws, Wl, prompts, w, tau, d_min)
    e.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
