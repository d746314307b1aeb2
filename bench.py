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
    # name: (pair, batch, prompt_lo, prompt_hi, default_steps, tau rule, d_min)
    # tau rule ("share", x): bisection on calibration runs until about x of the tokens come from the
    # large model; ("percentile", q): the q-th percentile of the small model's windowed entropy.
    "llama_1b_8b_b1": ("llama", 1, 512, 512, 1024, ("share", 0.40), 10),
    "qwen_05b_14b_b32": ("qwen", 32, 256, 256, 256, ("share", 0.25), 10),
    "qwen_05b_14b_b64": ("qwen", 64, 128, 1024, 128, ("percentile", 75.0), 10),
    "tiny_fp32_b1": ("tiny", 1, 16, 16, 64, ("share", 0.40), 10),
    # the paper's other pair shapes, batch 1
    "llama_1b_3b_b1": ("llama_1b_3b", 1, 512, 512, 1024, ("share", 0.40), 10),
    "qwen_15b_14b_b1": ("qwen_15b_14b", 1, 512, 512, 1024, ("share", 0.25), 10),
    # stand-alone entropy / arg-max / window / switch epilogue on materialised logits
    "entropy_gate_b64": (None, 64, 0, 0, 4096, None, 10),
    # prompt prefill of both models (the step before the decode path): steps = repetitions
    "prefill_qwen_b64": ("qwen", 64, 128, 1024, 4, None, 10),
    "prefill_llama_b8": ("llama", 8, 512, 512, 8, None, 10),
}
# The headline workload: the largest configuration that fits one GPU (Qwen-0.5B / Qwen-14B shapes, batch 64,
# ragged prompts, every row its own instance of Algorithm 1), grouped two-lane schedule.
DEFAULT_WORKLOAD = "qwen_05b_14b_b64"
SECONDARY_WORKLOAD = "llama_1b_8b_b1"     # the batch-1 pair, reported beside the default workload

MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def make_prompts(seed, batch, lo, hi, vocab):
    lens = si.prompt_lengths(seed, batch, lo, hi) if hi > lo else np.full(batch, lo, np.int32)
    return [si.prompt_np(seed, f"row{b}", int(lens[b]), vocab) for b in range(batch)]


def run_lengths(max_prompt, settle, warmup, steps, profile_steps, n_cal, lead=0):
    """Tokens every leg of a run may generate per row, and the max_seq a handle needs to hold the longest
    of them.  The profiling leg never runs longer than the timed one.  lead: how far a row of a free-running
    batch may get ahead of the slowest one (0: rows move in steps); such a row must still not reach the end
    of its run inside the timed region, so its bound lies a lead (and a few passes' overshoot) further."""
    profile_steps = max(1, min(profile_steps, steps))
    margin = lead + 8 if lead else 0
    timed_new = settle + warmup + steps + margin
    profile_new = settle + warmup + profile_steps + margin
    return {"timed_new": timed_new, "profile_new": profile_new, "profile_steps": profile_steps, "cal_new": n_cal,
            "max_seq": max_prompt + max(timed_new, profile_new, n_cal) + 8}


def calibrate_tau(e, rule, n_tokens, w, d_min):
    """Threshold for the workload from free-running calibration runs on the prompts already in the caches.
    ("percentile", q): q-th percentile of the small model's windowed entropy (one small-only run).
    ("share", x): bisection until about x of the tokens come from the large model (the percentile is
    only the starting bracket, because the window is shared across switches)."""
    def run(tau):
        e.set_gate(w, tau, d_min)
        e.rewind(n_tokens)
        e.decode(n_tokens)
        return e.fetch()
    probe = run(1e30)
    hb = probe["Hbar"].ravel()
    if rule[0] == "percentile":
        return float(np.percentile(hb, rule[1])), None
    target = rule[1]
    lo, hi = float(hb.min()) - 1.0, float(hb.max()) + 1e-3
    best = (2.0, hi)
    for _ in range(10):
        tau = 0.5 * (lo + hi)
        share = float(run(tau)["model_id"].mean())
        if abs(share - target) < abs(best[0] - target):
            best = (share, tau)
        if share > target:
            lo = tau            # too many large tokens: raise the threshold
        else:
            hi = tau
        if abs(share - target) < 0.02:
            break
    return best[1], best[0]


def host_cpu():
    """(model name, physical cores) of this host from /proc/cpuinfo; (None, None) where that is not readable."""
    try:
        txt = open("/proc/cpuinfo").read()
    except OSError:
        return None, None
    name, cores, phys, core = None, set(), None, None
    for line in txt.splitlines() + [""]:
        k, _, v = line.partition(":")
        k, v = k.strip(), v.strip()
        if k == "model name" and name is None:
            name = v
        elif k == "physical id":
            phys = v
        elif k == "core id":
            core = v
        elif not line.strip():
            if core is not None:
                cores.add((phys, core))
            phys = core = None
    return name, (len(cores) or None)


def host_mem_available():
    """Bytes of host memory that can still be taken (MemAvailable), or None where that cannot be read."""
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable:"):
                return 1024.0 * float(line.split()[1])
    except OSError:
        pass
    return None


def cpu_baseline(pair_shapes, Ws, Wl, prompts, w, tau, d_min, n_prompt, n_new, budget_s=20.0, max_rows=8):
    """The oracle as it stands, timed on this host: Algorithm 1 on a bounded sample of the workload -- the
    first rows of the batch one after the other (the oracle has no batching), each with its prompt cut to
    n_prompt tokens and n_new generated tokens after the first, same w / tau / d_min, until budget_s
    seconds of oracle time are spent or max_rows rows are done.  A row's prompt handling is subtracted by
    timing a 1-token run of it first.  Rows that switch make the large model consume every earlier token,
    so the sample's rate depends on how many of its rows switch: the share is reported with it."""
    import oracle
    ss, sl = pair_shapes
    # the oracle keeps both models in float32 on the host: refuse (the leg is then reported as failed, the
    # JSON line is still printed) rather than be killed for memory half way through
    need = 4.0 * (ss.n_params() + sl.n_params()) * 1.25 + 4e9
    avail = host_mem_available()
    if avail is not None and avail < need:
        raise MemoryError(f"the oracle needs about {need / 1e9:.0f} GB of host memory for this pair, {avail / 1e9:.0f} GB are available")
    t0 = time.time()
    os_ = oracle.Model(ss, {k: v.float().cpu().numpy() for k, v in Ws.items()})
    ol = oracle.Model(sl, {k: v.float().cpu().numpy() for k, v in Wl.items()})
    log(f"[cpu_baseline] fp32 weights on the host in {time.time() - t0:.1f}s")
    spent, n_tok, n_large, rows = 0.0, 0, 0, 0
    for prompt in prompts[:max_rows]:
        prompt = prompt[:n_prompt]
        ta = time.time(); oracle.generate(os_, ol, prompt, 1, w, tau, d_min); tb = time.time()
        out = oracle.generate(os_, ol, prompt, n_new + 1, w, tau, d_min); tc = time.time()
        spent += max((tc - tb) - (tb - ta), 1e-9)
        n_tok += n_new; n_large += int(out["model_id"][1:].sum()); rows += 1
        if spent >= budget_s:
            break
    name, phys = host_cpu()
    return {"value": n_tok / spent, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "cpu_model": name, "physical_cores_on_host": phys, "oracle_seconds": spent,
            "sample": f"rows 0-{rows - 1} one after the other, prompts cut to {n_prompt} tokens, {n_new} generated tokens "
                      f"after the first per row, same w/tau/d_min; large-model share of the sample's tokens "
                      f"{n_large / max(n_tok, 1):.2f}"}


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter runs, or None when
    there is none for this workload/kernel or the kernel sources changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    if rec.get("kernel") != kernel or rec.get("kernel_source_sha256_16") != kernel_source_hash():
        return None
    return rec["traffic_bytes_per_launch"]


def kernel_source_hash():
    """Hash of every source file the library's kernels are compiled from."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2502_06833_amd", "csrc")
    h = hashlib.sha256()
    for f in sorted(os.listdir(csrc)):
        if f.endswith((".hpp", ".hip")):
            h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


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
        "roofline": {"bound": "hbm", "kernel": "entropy_rows (entropy, arg max, window and switch rule; 16 steps per launch)",
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
        name, phys = host_cpu()
        out["cpu_baseline"] = {"value": n / (time.time() - t0), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                               "cpu_model": name, "physical_cores_on_host": phys,
                               "sample": "entropy + arg max of the 64 rows of one tensor, repeated for 10 s (the oracle's "
                                         "entropy routine is single-threaded: one thread used)"}
    g.close()
    print(json.dumps(out), flush=True)


def run_secondary(workload, args):
    """Another workload through this same script in a child process (its own handle and weights); returns the
    fields of its JSON line that describe the decode path."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--workload", workload, "--secondary", "none", "--no-cpu-baseline",
           "--warmup", str(args.warmup), "--seed", str(args.seed)]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    for line in r.stderr.splitlines():
        if line.startswith("[bench]"):
            log("  (secondary) " + line)
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    if not lines:
        raise RuntimeError(f"secondary workload {workload} printed no result (exit {r.returncode}): {r.stderr[-400:]}")
    d = json.loads(lines[-1])
    keep = ("metric", "value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config", "decode_hbm_gbs", "decode_hbm_frac_of_peak",
            "large_token_share", "param_ratio", "switches", "small_only", "large_only", "ead_over_large_only", "roofline", "errors")
    return {k: d[k] for k in keep if k in d}


def build_probe():
    """Compile roofline_probe.hip (beside this file): a torch-free driver of the library's C ABI for
    hardware-counter runs (`rocprofv3 --pmc ... -- ./roofline_probe ...`)."""
    import subprocess
    from paper_2502_06833_amd import build as lib_build
    lib_build.build(force=False)
    libdir = os.path.join(ROOT, "paper_2502_06833_amd")
    exe = os.path.join(ROOT, "roofline_probe")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O2", "-std=c++17", "-o", exe, os.path.join(ROOT, "roofline_probe.hip"),
           "-L" + libdir, "-lead", "-Wl,-rpath," + libdir]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stderr)
    return exe


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--settle", type=int, default=32,
                    help="untimed decode steps before the warm-up steps, so that the timed steps see rows on both models, "
                         "pending catch-ups and contexts past the prompts (as prompt prefill, outside the timed region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-single-model", action="store_true", help="skip the small-only / large-only runs")
    ap.add_argument("--profile-steps", type=int, default=64, help="steps of the per-kernel timing leg (never more than --steps)")
    ap.add_argument("--fused", type=int, default=None, help="1/0: the fused single-row decode kernel on/off (2: its register-buffered variant)")
    ap.add_argument("--tau", type=float, default=None, help="skip the calibration runs and use this threshold (nats)")
    ap.add_argument("--schedule", choices=["lockstep", "grouped"], default=None,
                    help="grouped (default for batches): small-model rows run ahead, large-model rows are served together")
    ap.add_argument("--sched-start", type=float, default=0.5, help="grouped: large model starts at this share of waiting rows")
    ap.add_argument("--sched-stop", type=float, default=0.25, help="grouped: ... and stops below this share")
    ap.add_argument("--lead", type=int, default=32,
                    help="grouped: rows run freely, none more than this many tokens ahead of the slowest (a step is then "
                         "one token per row of batch progress: batch tokens in total); 0: every row exactly one token per step")
    ap.add_argument("--temperature", type=float, default=0.0, help="sample at this temperature (0 = greedy, the default)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for hardware byte counters)")
    ap.add_argument("--build-probe", action="store_true", help="compile roofline_probe.hip and exit")
    ap.add_argument("--secondary", default=None,
                    help="a second workload measured by a child process after this one and reported under 'secondary' in the same "
                         "JSON line ('none' to skip; default: the batch-1 workload when the default workload runs)")
    args = ap.parse_args()
    if args.build_probe:
        print(build_probe())
        return 0
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
    pair, batch, plo, phi, dsteps, rule, d_min = WORKLOADS[args.workload]
    steps = args.steps or dsteps
    warmup, settle = args.warmup, max(args.settle, 0)
    schedule = args.schedule or ("grouped" if batch > 1 else "lockstep")
    grouped = schedule == "grouped"
    w = 5
    ss, sl = si.PAIRS[pair]
    t0 = time.time()
    Ws = si.model_weights_torch(ss, args.seed, "cuda")
    Wl = si.model_weights_torch(sl, args.seed, "cuda")
    torch.cuda.synchronize()
    log(f"[bench] weights generated in {time.time() - t0:.1f}s")
    prompts = make_prompts(args.seed, batch, plo, phi, ss.vocab)
    n_cal = 64 if batch > 1 else 96
    lead = args.lead if grouped else 0
    ln = run_lengths(max(len(p) for p in prompts), settle, warmup, steps, args.profile_steps, n_cal, lead)
    e = ead.EAD(ss, Ws, sl, Wl, window=w, tau=0.0, d_min=d_min, max_batch=batch, max_seq=ln["max_seq"])
    if args.no_cpu_baseline:
        del Ws, Wl
        torch.cuda.empty_cache()
    log(f"[bench] handle created at {time.time() - t0:.1f}s")
    if args.fused is not None:
        e.set_fused(int(args.fused))
    if args.temperature > 0:
        e.set_sampling(args.temperature, args.seed)

    if args.copy_probe:
        src = torch.empty(1 << 29, dtype=torch.bfloat16, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # prompt prefill of both models, once; every leg below starts over from this state (ead_rewind)
    ta = time.perf_counter()
    e.begin(prompts, ln["timed_new"])
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - ta
    log(f"[bench] prompts prefilled ({sum(len(p) - 1 for p in prompts)} positions, both models) in {prefill_s:.2f}s")

    out = {
        "metric": "generated tokens/s at 1 GPU", "value": None, "unit": "tokens/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": None, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if ss.bf16 else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "small": ss.name, "large": sl.name, "batch": batch,
                   "prompt_len": [int(plo), int(phi)], "window": w, "d_min": d_min, "tau_nats": None, "tau_rule": list(rule),
                   "vocab": ss.vocab, "schedule": schedule, "temperature": args.temperature, "settle_steps": settle,
                   "step": ("free-running rows: a step is one token per row of batch progress (batch tokens), no row more than "
                            f"{lead} tokens ahead of the slowest") if lead else "one token for every row"},
        "prefill_s": prefill_s, "roofline": None, "cpu_baseline": None,
    }
    errors = {}

    def leg(name, fn):
        """Run one leg; a failure is recorded and the other legs still run."""
        try:
            return fn()
        except Exception as ex:  # noqa: BLE001
            errors[name] = f"{type(ex).__name__}: {ex}"
            log(f"[bench] leg '{name}' failed: {errors[name]}")
            return None

    def advance(n_steps, free):
        """n_steps steps of the batch: one token per row and step, or (free-running rows) batch tokens per step."""
        if free:
            e.decode_tokens(n_steps * batch, lead)
        else:
            e.decode(n_steps)

    def timed(force, grp):
        free = grp and lead > 0
        e.force_model(force)
        e.set_schedule(grp, args.sched_start, args.sched_stop)
        e.set_gate(w, tau, d_min)
        e.rewind(ln["timed_new"])
        if settle:
            advance(settle, free)
        advance(warmup, free)
        e.reset_stats()
        torch.cuda.synchronize()
        a = time.perf_counter()
        advance(steps, free)
        torch.cuda.synchronize()
        dt = time.perf_counter() - a
        st = e.stats()
        e.force_model(-1)
        e.set_schedule(False)
        return dt, st

    tau = args.tau

    def do_calibrate():
        nonlocal tau
        tau, share_cal = calibrate_tau(e, rule, n_cal, w, d_min)
        log(f"[bench] tau={tau:.6f} nats ({rule[0]} {rule[1]}"
            + (f" -> large share {share_cal:.3f}" if share_cal is not None else "")
            + f", {n_cal} calibration tokens per row) at {time.time() - t0:.1f}s")
    if tau is None:
        leg("calibration", do_calibrate)
    else:
        log(f"[bench] tau={tau:.6f} nats (given)")
    out["config"]["tau_nats"] = tau

    def do_headline():
        dt, st = timed(-1, grouped)
        n_tok = st["tokens_small"] + st["tokens_large"]
        algo_gbs = st["algorithmic_bytes"] / dt / 1e9
        out.update({"value": n_tok / dt, "ms_per_step": 1e3 * dt / (n_tok / batch), "tokens_timed": n_tok,
                    "decode_hbm_gbs": algo_gbs, "decode_hbm_frac_of_peak": algo_gbs / HBM_PEAK_GBS,
                    "large_token_share": st["large_share"], "param_ratio": st["param_ratio"], "switches": st["switches"],
                    "host_syncs": st["host_syncs"]})
        if grouped:
            out["grouped"] = {"start": args.sched_start, "stop": args.sched_stop, "max_lead": lead, "large_passes": st["steps_large"],
                              "small_passes": st["steps_small"], "catchup_rows_large": st["catchup_rows_large"]}
        log(f"[bench] EAD ({schedule}): {n_tok / dt:.1f} tok/s, {algo_gbs:.0f} GB/s algorithmic ({algo_gbs / HBM_PEAK_GBS:.1%} of peak), "
            f"large share {st['large_share']:.3f}, switches {st['switches']}, host syncs {st['host_syncs']}, "
            f"passes large/small {st['steps_large']}/{st['steps_small']}")

    def do_exact():
        # the grouped schedule with every row held to exactly `steps` tokens (rows that are ahead wait at the end)
        nonlocal lead
        keep, lead = lead, 0
        try:
            d1, s1 = timed(-1, True)
        finally:
            lead = keep
        n1 = s1["tokens_small"] + s1["tokens_large"]
        out["grouped_exact_steps"] = {"tokens_per_s": n1 / d1, "large_passes": s1["steps_large"], "small_passes": s1["steps_small"],
                                      "large_token_share": s1["large_share"]}
        log(f"[bench] grouped, exactly {steps} tokens per row: {n1 / d1:.1f} tok/s, large share {s1['large_share']:.3f}, "
            f"passes large/small {s1['steps_large']}/{s1['steps_small']}")

    def do_lockstep():
        d1, s1 = timed(-1, False)
        n1 = s1["tokens_small"] + s1["tokens_large"]
        out["lockstep"] = {"tokens_per_s": n1 / d1, "large_passes": s1["steps_large"], "small_passes": s1["steps_small"],
                           "large_token_share": s1["large_share"]}
        log(f"[bench] lock step: {n1 / d1:.1f} tok/s with {s1['steps_large']} large / {s1['steps_small']} small passes")

    def do_single(name, which):
        d2, s2 = timed(which, False)
        n2 = s2["tokens_small"] + s2["tokens_large"]
        out[name] = {"tokens_per_s": n2 / d2, "hbm_frac": s2["algorithmic_bytes"] / d2 / 1e9 / HBM_PEAK_GBS}
        log(f"[bench] {name}: {n2 / d2:.1f} tok/s, {out[name]['hbm_frac']:.1%} of HBM peak")

    def profiled_run(select, force=-1, grp=None):
        # per-kernel HIP-event timing on a separate, untimed run (events on the lanes' own streams)
        grp = grouped if grp is None else grp
        e.force_model(force)
        e.set_schedule(grp, args.sched_start, args.sched_stop)
        e.set_gate(w, tau, d_min)
        e.rewind(ln["profile_new"])
        free = grp and lead > 0
        if settle:
            advance(settle, free)
        advance(warmup, free)
        e.profile_select(select)
        e.profile(True)
        advance(ln["profile_steps"], free)
        prof = e.profile_read()
        e.profile(False)
        e.profile_select(None)
        e.set_schedule(False)
        e.force_model(-1)
        return prof

    def do_profile():
        prof = profiled_run(None)
        for r in sorted(prof, key=lambda r: -r["total_ms"]):
            gbs = r["bytes"] / max(r["total_ms"], 1e-9) / 1e6
            log(f"[prof] {r['name']:<28s} n={r['launches']:<6d} avg {1e3 * r['total_ms'] / r['launches']:8.2f} us  "
                f"{gbs:8.0f} GB/s")
        # The dominant kernel is reported per model (one kernel, one shape): the weight-streaming kernel that
        # moves the most bytes over the run, which does not flip with timing noise the way a ranking by time can.
        # (The attention kernel's bytes follow the contexts and catch-up rows the passes happen to carry: with
        # long prompts its total can pass that of the largest matrix, at two thirds of its time per launch; it
        # stays in the breakdown above.)  The roofline
        # entry is timed on the kernel's own model's passes (the other model idle, only this kernel's launches bracketed):
        # while both lanes' queues are busy, event brackets read about 25 us more than the kernel's begin and
        # end stamps in a rocprofv3 trace of the same launches, with one lane they agree to a few microseconds.
        linear = [r for r in prof if r["name"].startswith("linear_")]
        dom = max(linear or prof, key=lambda r: r["bytes"])["name"]
        which = 1 if dom.endswith("/large") else 0
        d = next(r for r in profiled_run(dom, force=which, grp=False) if r["name"] == dom)
        achieved = d["bytes"] / d["total_ms"] / 1e6
        both = next(r for r in prof if r["name"] == dom)
        log(f"[prof] {dom} on its model's own passes ({batch} rows): n={d['launches']} avg {1e3 * d['total_ms'] / d['launches']:.2f} us "
            f"= {achieved:.0f} GB/s")
        out["roofline"] = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(args.workload, dom),
                           "avg_launch_us": 1e3 * d["total_ms"] / d["launches"],
                           "bytes_per_launch": d["bytes"] / d["launches"], "launches": d["launches"],
                           "profiled_steps": ln["profile_steps"], "rows_per_pass": batch,
                           "timed_on": ("large" if which else "small") + "-model-only passes, one lane, this kernel's launches bracketed",
                           "avg_launch_us_both_lanes_bracketed": 1e3 * both["total_ms"] / both["launches"]}

    def do_cpu():
        big = sl.n_params() > 2e9
        out["cpu_baseline"] = cpu_baseline((ss, sl), Ws, Wl, prompts, w, tau, d_min,
                                           n_prompt=8 if big else 16, n_new=14 if big else 24)

    if tau is not None:
        leg("headline", do_headline)
        if grouped:
            if lead > 0:
                leg("grouped_exact_steps", do_exact)
            leg("lockstep", do_lockstep)
        if not args.no_single_model:
            leg("small_only", lambda: do_single("small_only", 0))
            leg("large_only", lambda: do_single("large_only", 1))
        if out.get("large_only") and out["value"]:
            out["ead_over_large_only"] = out["value"] / out["large_only"]["tokens_per_s"]
        leg("profile", do_profile)
        if not args.no_cpu_baseline:
            leg("cpu_baseline", do_cpu)
    leg("close", e.close)
    secondary = args.secondary or (SECONDARY_WORKLOAD if args.workload == DEFAULT_WORKLOAD else "none")
    if secondary != "none" and tau is not None:
        del e
        Ws = Wl = None
        torch.cuda.empty_cache()
        try:        # an extra: its failure is reported in place and does not fail the run
            out["secondary"] = run_secondary(secondary, args)
        except Exception as ex:  # noqa: BLE001
            out["secondary"] = {"workload": secondary, "error": f"{type(ex).__name__}: {ex}"}
            log(f"[bench] secondary workload failed: {out['secondary']['error']}")
    if errors:
        out["errors"] = errors
    print(json.dumps(out), flush=True)
    return 1 if errors or out["value"] is None else 0


if __name__ == "__main__":
    sys.exit(main() or 0)
