#!/usr/bin/env python3
"""Threshold sweep of Entropy Adaptive Decoding on a synthetic workload (needs a GPU).

The paper sweeps the threshold tau over a fixed grid and plots benchmark score against the share
of tokens the large model generated and the parameter ratio of Table 1 (Section 4, Fig. 1,
Table 1).  The score needs the paper's benchmark and trained weights; what can be reproduced on
synthetic, randomly initialised models of the same shapes is the cost side of that curve:
for every threshold, the large-token share, the parameter ratio and the measured tokens/s.
Randomly initialised models have entropies close to ln V, so the paper's absolute grid is
re-expressed as percentiles of the small model's windowed entropy on the same prompts.

  python tau_sweep.py --workload llama_1b_8b_b1 --steps 256 [--unit bits] [--schedule grouped]

One JSON line per threshold on stdout, then a table on stderr."""
import argparse
import json
import sys
import time

import numpy as np

import bench
import synth_inputs as si


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="llama_1b_8b_b1",
                    choices=sorted(k for k, v in bench.WORKLOADS.items() if v[0] is not None and not k.startswith("prefill_")))
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--unit", choices=["nats", "bits"], default="nats")
    ap.add_argument("--percentiles", default="0,10,25,40,50,60,75,90,100")
    ap.add_argument("--schedule", choices=["lockstep", "grouped"], default="lockstep")
    ap.add_argument("--temperature", type=float, default=0.0)
    args = ap.parse_args()
    import torch
    import paper_2502_06833_amd as ead
    if not torch.cuda.is_available():
        sys.exit("tau_sweep.py needs a GPU")
    pair, batch, plo, phi, _, _, d_min = bench.WORKLOADS[args.workload]
    w = 5
    ss, sl = si.PAIRS[pair]
    Ws = si.model_weights_torch(ss, args.seed, "cuda")
    Wl = si.model_weights_torch(sl, args.seed, "cuda")
    prompts = bench.make_prompts(args.seed, batch, plo, phi, ss.vocab)
    max_seq = max(len(p) for p in prompts) + args.warmup + args.steps + 8
    unit = ead.BITS if args.unit == "bits" else ead.NATS
    e = ead.EAD(ss, Ws, sl, Wl, window=w, tau=0.0, d_min=d_min, unit=unit, max_batch=batch, max_seq=max_seq)
    del Ws, Wl
    torch.cuda.empty_cache()
    if args.temperature > 0:
        e.set_sampling(args.temperature, args.seed)
    # the small model's windowed entropies on these prompts (threshold at +inf: never switches)
    e.set_gate(w, 1e30, d_min, unit)
    hb = e.generate(prompts, args.warmup + args.steps)["Hbar"].ravel()
    rows = []
    for pct in [float(x) for x in args.percentiles.split(",")]:
        tau = -1e30 if pct <= 0 else (1e30 if pct >= 100 else float(np.percentile(hb, pct)))
        e.set_schedule(args.schedule == "grouped")
        e.set_gate(w, tau, d_min, unit)
        e.begin(prompts, args.warmup + args.steps)
        e.decode(args.warmup)
        e.reset_stats()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e.decode(args.steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        st = e.stats()
        n_tok = st["tokens_small"] + st["tokens_large"]
        row = {"workload": args.workload, "unit": args.unit, "percentile": pct, "tau": tau,
               "large_token_share": st["large_share"], "param_ratio": st["param_ratio"],
               "tokens_per_s": n_tok / dt, "switches": st["switches"],
               "decode_hbm_frac_of_peak": st["algorithmic_bytes"] / dt / 1e9 / bench.HBM_PEAK_GBS,
               "schedule": args.schedule, "temperature": args.temperature}
        rows.append(row)
        print(json.dumps(row), flush=True)
    e.close()
    bench.log(f"{'pct':>5s} {'tau':>12s} {'large %':>8s} {'param ratio':>12s} {'tok/s':>10s} {'switches':>9s} {'HBM %':>6s}")
    for r in rows:
        bench.log(f"{r['percentile']:5.0f} {r['tau']:12.5g} {100 * r['large_token_share']:8.1f} {r['param_ratio']:12.3f} "
                  f"{r['tokens_per_s']:10.1f} {r['switches']:9d} {100 * r['decode_hbm_frac_of_peak']:6.1f}")


if __name__ == "__main__":
    main()
