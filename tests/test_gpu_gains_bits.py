"""RMSNorm gains that are not 1, and entropies in bits, through every kernel path against the oracle.

The definition x / sqrt(mean(x^2) + eps) * g has a factor g that a test with all gains at 1 cannot see:
here the gains are 1 + N(0, 0.3^2), different for the attention norm, the feed-forward norm and the final
norm of every layer, so a kernel that skipped, swapped or mis-indexed one of them fails by far more than any
tolerance.  Paths: 1-2 rows (FMA kernels, norm in the prologue), 5 and 24 rows (activation packing + matrix-core
kernels), 77 and 150 rows (wide sweeps, K split over workgroups), the fused single-row kernel, fp32 and bf16.
Eq. 2 is written in log2: the same runs are repeated with the handle in bits (tau in bits).
"""
import math

import numpy as np
import pytest

import oracle
import synth_inputs as si
from gpu_helpers import BAND, TOL_H, TOL_LOGIT, check_logits, check_replay_row, make_pair, trajectory_logit_stats

pytestmark = pytest.mark.gpu


def _ead():
    import paper_2502_06833_amd as ead
    return ead


def test_tiny_fp32_pair_with_random_gains():
    ead = _ead()
    Ws, Wl, os_, ol = make_pair(si.TINY_S, si.TINY_L, seed=3, gain_std=0.3)
    e = ead.EAD(si.TINY_S, Ws, si.TINY_L, Wl, window=5, tau=0.0, d_min=4, max_batch=4, max_seq=128)
    toks = si.prompt_np(3, "gains", 70, 512)
    for which, om in ((0, os_), (1, ol)):
        ref = om.forward_dense(toks)
        for n in (1, 2, 5, 70):
            out = e.score(which, toks[:n])
            check_logits(out["logits"], ref[:n], 1e-4)
            Hr, ar = oracle.entropy_rows(ref[:n])
            assert np.abs(out["H"] - Hr).max() < 1e-4 and (out["argmax"] == ar).all()
    prompt = toks[:12]
    probe = oracle.generate(os_, ol, prompt, 40, 5, 1e30, d_min=4)
    tau = float(np.percentile(probe["Hbar"], 50))
    ref = oracle.generate(os_, ol, prompt, 40, 5, tau, d_min=4)
    assert 0 < ref["model_id"].mean() < 1
    e.set_gate(5, tau, 4)
    for fused in (False, True):
        e.set_fused(fused)
        rp = e.replay([prompt], ref["tokens"], ref["model_id"])
        assert np.abs(rp["H"][0] - ref["H"]).max() < 1e-4, fused
        assert np.abs(rp["Hbar"][0] - ref["Hbar"]).max() < 1e-4
        assert (rp["argmax"][0] == ref["tokens"]).all()
    e.set_fused(False)
    e.close()


@pytest.mark.parametrize("pair,rows", [("llama", (1, 2, 5, 24, 150)), ("qwen", (1, 2, 5, 40, 77))])
def test_bf16_truncated_pair_with_random_gains(pair, rows):
    ead = _ead()
    ss, sl = (s.truncated(2) for s in si.PAIRS[pair])
    Ws, Wl, os_, ol = make_pair(ss, sl, seed=2, gain_std=0.3, lm_sigma=1.5)
    T = max(rows)
    e = ead.EAD(ss, Ws, sl, Wl, window=5, tau=0.0, d_min=4, max_batch=2, max_seq=T + 40)
    toks = si.prompt_np(2, pair + "/gains", T, ss.vocab)
    for which, om in ((0, os_), (1, ol)):
        print(f"{pair} gains: oracle model {which} on {T} positions", flush=True)
        ref = om.forward_dense(toks)
        Hr, ar = oracle.entropy_rows(ref)
        top2 = np.sort(ref, axis=1)
        clear = (top2[:, -1] - top2[:, -2]) > 2 * TOL_LOGIT * np.abs(ref).max(axis=1)
        for n in rows:
            out = e.score(which, toks[:n])
            err = check_logits(out["logits"], ref[:n], TOL_LOGIT)
            print(f"  rows={n}: logits rel err {err:.2e}, H err {np.abs(out['H'] - Hr[:n]).max():.2e}", flush=True)
            assert np.abs(out["H"] - Hr[:n]).max() < TOL_H
            assert (out["argmax"][clear[:n]] == ar[:n][clear[:n]]).all()
    # Algorithm 1 along the oracle's trajectory: single-row steps (FMA kernels) and catch-up chunks,
    # with the per-layer kernels and with the fused single-row kernel
    prompt = toks[:8]
    probe = oracle.generate(os_, ol, prompt, 24, 5, 1e30, d_min=4)
    tau = float(np.percentile(probe["Hbar"], 50))
    ref = oracle.generate(os_, ol, prompt, 24, 5, tau, d_min=4)
    stats = trajectory_logit_stats(os_, ol, prompt, ref["tokens"], ref["model_id"])
    assert 0 < ref["model_id"].mean() < 1
    e.set_gate(5, tau, 4)
    for fused in (False, True):
        e.set_fused(fused)
        rp = e.replay([prompt], ref["tokens"], ref["model_id"])
        n_dec, n_arg = check_replay_row(rp, 0, ref, tau, 24, stats)
        print(f"  fused={fused}: decisions checked outside the band {n_dec}/24, clear arg maxes {n_arg}/24", flush=True)
        assert n_dec >= 8
    e.set_fused(False)
    e.close()


def test_bits_through_a_handle_tiny_fp32():
    """Eq. 2 in log2: handle created in bits, tau in bits, against oracle.generate(unit = BITS)."""
    ead = _ead()
    Ws, Wl, os_, ol = make_pair(si.TINY_S, si.TINY_L, seed=0)
    prompt = si.prompt_np(0, "bits", 16, 512)
    probe = oracle.generate(os_, ol, prompt, 48, 5, 1e30, d_min=5, unit=oracle.BITS)
    tau_bits = float(np.percentile(probe["Hbar"], 55))
    assert abs(probe["H"].mean() - math.log2(512)) < 0.5          # about 9 bits
    ref = oracle.generate(os_, ol, prompt, 48, 5, tau_bits, d_min=5, unit=oracle.BITS)
    ref_nats = oracle.generate(os_, ol, prompt, 48, 5, tau_bits * math.log(2.0), d_min=5)
    assert np.abs(ref["H"] * math.log(2.0) - ref_nats["H"]).max() < 1e-5
    assert 0 < ref["model_id"].mean() < 1
    e = ead.EAD(si.TINY_S, Ws, si.TINY_L, Wl, window=5, tau=tau_bits, d_min=5, unit=ead.BITS, max_batch=2, max_seq=96)
    rp = e.replay([prompt], ref["tokens"], ref["model_id"])
    assert np.abs(rp["H"][0] - ref["H"]).max() < 1e-4 and np.abs(rp["Hbar"][0] - ref["Hbar"]).max() < 1e-4
    assert (rp["argmax"][0] == ref["tokens"]).all()
    safe = np.abs(ref["Hbar"] - tau_bits) > 1e-4
    want_next = np.concatenate([ref["model_id"][1:], rp["next_model"][0][-1:]])
    assert (rp["next_model"][0][safe] == want_next[safe]).all() and safe.sum() >= 16
    out = e.generate([prompt], 48)
    if safe.all():
        assert (out["tokens"][0] == ref["tokens"]).all() and (out["model_id"][0] == ref["model_id"]).all()
    assert np.abs(out["H"][0, :8] - ref["H"][:8]).max() < 1e-4       # the first tokens precede any possible divergence
    # switching the same handle to nats with the threshold converted gives the same run
    e.set_gate(5, tau_bits * math.log(2.0), 5, unit=ead.NATS)
    rn = e.replay([prompt], ref["tokens"], ref["model_id"])
    assert np.abs(rn["H"][0] - ref["H"] * math.log(2.0)).max() < 1e-4
    e.close()


def test_bits_through_a_handle_bf16_truncated():
    ead = _ead()
    ss, sl = (s.truncated(2) for s in si.PAIRS["qwen"])
    Ws, Wl, os_, ol = make_pair(ss, sl, seed=5, gain_std=0.5, lm_sigma=1.5)
    prompts = [si.prompt_np(5, f"bits{b}", n, ss.vocab) for b, n in enumerate((9, 30, 17))]
    hb = np.concatenate([oracle.generate(os_, ol, p, 20, 5, 1e30, d_min=3, unit=oracle.BITS)["Hbar"] for p in prompts])
    tau_bits = float(np.percentile(hb, 50))
    refs = [oracle.generate(os_, ol, p, 20, 5, tau_bits, d_min=3, unit=oracle.BITS) for p in prompts]
    assert 0 < np.mean([r["model_id"].mean() for r in refs]) < 1
    e = ead.EAD(ss, Ws, sl, Wl, window=5, tau=0.0, d_min=3, max_batch=3, max_seq=64)
    e.set_gate(5, tau_bits, 3, unit=ead.BITS)
    rp = e.replay(prompts, np.stack([r["tokens"] for r in refs]), np.stack([r["model_id"] for r in refs]))
    n_dec = 0
    for b, r in enumerate(refs):
        # tolerances are stated in nats: 1e-2 nats = 1.44e-2 bits
        d, _ = check_replay_row(rp, b, r, tau_bits, 20, None, tol_h=TOL_H / math.log(2.0), band=BAND / math.log(2.0))
        n_dec += d
    print(f"bits: decisions checked outside the band {n_dec}/60", flush=True)
    assert n_dec >= 20
    free = e.generate(prompts, 20)
    assert abs(free["H"].mean() / math.log2(ss.vocab) - 1) < 0.2    # entropies of the order of log2 V bits, not ln V nats
    e.close()


def test_half_precision_activations_saturate_instead_of_overflowing():
    """The matrix-core kernels round their activations to IEEE half, which ends at 65504.  A final-norm gain of
    1e5 pushes the LM head's input past that: passes of three or more rows must saturate (finite logits and
    entropies, arg max still defined), not produce infinities; passes of one or two rows keep float32 activations
    and follow the oracle as always."""
    ead = _ead()
    ss, sl = (s.truncated(1) for s in si.PAIRS["llama"])
    Ws = si.model_weights_torch(ss, 5, "cuda")
    Wl = si.model_weights_torch(sl, 5, "cuda")
    Ws["norm_final"] = Ws["norm_final"] * 1e5
    e = ead.EAD(ss, Ws, sl, Wl, window=5, tau=0.0, d_min=4, max_batch=1, max_seq=64)
    toks = si.prompt_np(5, "sat", 6, ss.vocab)
    wide = e.score(0, toks)                      # 6 rows: activation tiles in half precision
    assert np.isfinite(wide["logits"]).all() and np.isfinite(wide["H"]).all()
    assert np.abs(wide["logits"]).max() > 1e3    # the gain did reach the logits
    om = oracle.Model(ss, {k: v.float().cpu().numpy() for k, v in Ws.items()})
    ref = om.forward_dense(toks[:2])
    narrow = e.score(0, toks[:2])                # 2 rows: float32 activations, no saturation
    check_logits(narrow["logits"], ref, TOL_LOGIT)
    e.close()
