"""GPU parity of the decode path (through the C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

TOL_LOGIT = 2e-2     # max |diff| <= TOL * max |ref| per row  (bf16 kernels vs fp32 oracle)
TOL_H = 1e-2         # nats
BAND = 1e-2          # switch decisions are exempt when |window mean - tau| < BAND


def _ead():
    import paper_2502_06833_amd as ead
    return ead


def _pair(shape_s, shape_l, seed=0, std=0.02):
    Ws = si.model_weights_torch(shape_s, seed, "cuda", std)
    Wl = si.model_weights_torch(shape_l, seed, "cuda", std)
    os_ = oracle.Model(shape_s, {k: v.float().cpu().numpy() for k, v in Ws.items()})
    ol = oracle.Model(shape_l, {k: v.float().cpu().numpy() for k, v in Wl.items()})
    return Ws, Wl, os_, ol


def _check_logits(got, ref, tol):
    err = np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)
    assert err.max() < tol, err.max()
    return err.max()


MINI_S = si.ModelShape("gmini-s", 2, 64, 2, 2, 96, 512, 1e-5, 1e4, bf16=False)
MINI_L = si.ModelShape("gmini-l", 3, 128, 4, 2, 160, 512, 1e-5, 1e4, bf16=False)


@pytest.fixture(scope="module")
def tiny():
    ead = _ead()
    Ws, Wl, os_, ol = _pair(si.TINY_S, si.TINY_L)
    e = ead.EAD(si.TINY_S, Ws, si.TINY_L, Wl, window=5, tau=0.0, d_min=10, max_batch=4, max_seq=128)
    yield e, os_, ol
    e.close()


def test_tiny_fp32_score_matches_oracle(tiny):
    e, os_, ol = tiny
    toks = si.prompt_np(0, "score", 40, 512)
    for which, om in ((0, os_), (1, ol)):
        print(f"score tiny model {which}", flush=True)
        out = e.score(which, toks)
        ref = om.forward_dense(toks)
        _check_logits(out["logits"], ref, 1e-4)
        Hr, ar = oracle.entropy_rows(ref)
        assert np.abs(out["H"] - Hr).max() < 1e-4
        assert (out["argmax"] == ar).all()


def _calibrate_tau(os_, ol, prompt, n, w, q):
    probe = oracle.generate(os_, ol, prompt, n, w, 1e30)
    return float(np.percentile(probe["Hbar"], q))


def test_tiny_config1_free_running_and_replay(tiny):
    """Tiny fp32 pair, 16-token prompt, 64 greedy tokens, w=5, tau = 60th percentile of the
    small model's windowed entropy in a seed-0 calibration run."""
    e, os_, ol = tiny
    prompt = si.prompt_np(0, "cfg1", 16, 512)
    tau = _calibrate_tau(os_, ol, prompt, 64, 5, 60)
    for d_min in (10, 3, 1):
        print(f"config1 d_min={d_min} tau={tau}", flush=True)
        ref = oracle.generate(os_, ol, prompt, 64, 5, tau, d_min=d_min)
        assert 0 < ref["model_id"].mean() < 1
        e.set_gate(5, tau, d_min)
        rp = e.replay([prompt], ref["tokens"], ref["model_id"])
        assert np.abs(rp["H"][0] - ref["H"]).max() < 1e-4
        assert np.abs(rp["Hbar"][0] - ref["Hbar"]).max() < 1e-4
        assert (rp["argmax"][0] == ref["tokens"]).all()
        safe = np.abs(ref["Hbar"] - tau) > 1e-4
        want_next = np.concatenate([ref["model_id"][1:], rp["next_model"][0][-1:]])
        assert (rp["next_model"][0][safe] == want_next[safe]).all()
        out = e.generate([prompt], 64)
        n_same = int(np.argmax(np.concatenate([out["tokens"][0] != ref["tokens"], [True]])))
        print(f"  free-running: identical for {n_same}/64 tokens", flush=True)
        if safe.all():
            assert (out["tokens"][0] == ref["tokens"]).all()
            assert (out["model_id"][0] == ref["model_id"]).all()
        st = e.stats()
        assert st["tokens_small"] + st["tokens_large"] == 64
        assert abs(st["large_share"] - out["model_id"].mean()) < 1e-9


def test_extreme_thresholds(tiny):
    e, os_, ol = tiny
    prompt = si.prompt_np(1, "cfg1", 16, 512)
    e.set_gate(5, 1e30, 10)
    out = e.generate([prompt], 24)
    assert (out["model_id"] == 0).all()
    e.set_gate(5, 0.0, 10)
    out = e.generate([prompt], 24)
    assert list(out["model_id"][0]) == [0] * 10 + [1] * 14
    e.force_model(1)
    big = e.generate([prompt], 8)
    assert (big["model_id"] == 1).all()
    ref = ol.forward_dense(prompt)[-1]
    assert big["tokens"][0, 0] == oracle.entropy(ref)[1]
    e.force_model(-1)


def test_degenerate_shapes_of_a_run(tiny):
    """Prompts of a single token, a single new token, a window longer than the run, a window of
    one with d_min = 1 (a catch-up in one direction or the other at almost every step), a run
    that ends exactly at max_seq, and rows of one batch that end at different times (eos)."""
    e, os_, ol = tiny
    one = si.prompt_np(9, "one", 1, 512)
    # single-token prompt: nothing to prefill, the first decode step feeds the only token
    for w, d_min, n in ((5, 10, 12), (64, 2, 20), (1, 1, 30)):
        tau = _calibrate_tau(os_, ol, one, n, w, 50)
        ref = oracle.generate(os_, ol, one, n, w, tau, d_min=d_min)
        e.set_gate(w, tau, d_min)
        rp = e.replay([one], ref["tokens"], ref["model_id"])
        assert np.abs(rp["H"][0] - ref["H"]).max() < 1e-4, (w, d_min)
        assert np.abs(rp["Hbar"][0] - ref["Hbar"]).max() < 1e-4
        assert (rp["argmax"][0] == ref["tokens"]).all()
        if w == 1:
            assert (np.diff(ref["model_id"].astype(int)) != 0).sum() >= 5      # the gate really flips
            safe = np.abs(ref["Hbar"] - tau) > 1e-4
            if safe.all():
                out = e.generate([one], n)
                assert (out["tokens"][0] == ref["tokens"]).all() and (out["model_id"][0] == ref["model_id"]).all()
    # one new token
    e.set_gate(5, 0.0, 10)
    out = e.generate([si.prompt_np(9, "p", 7, 512)], 1)
    ref = oracle.generate(os_, ol, si.prompt_np(9, "p", 7, 512), 1, 5, 0.0)
    assert out["tokens"][0, 0] == ref["tokens"][0] and abs(out["H"][0, 0] - ref["H"][0]) < 1e-4
    # exactly max_seq positions (the fixture's handle has max_seq = 128)
    p100 = si.prompt_np(9, "long", 100, 512)
    out = e.generate([p100], 28)
    ref = oracle.generate(os_, ol, p100, 28, 5, 0.0)
    assert (out["lens"] == 28).all() and np.abs(out["H"][0] - ref["H"]).max() < 1e-4
    # rows that end at different times: eos = row 0's 4th token
    prompts = [si.prompt_np(s, "eos", 10, 512) for s in (20, 21, 22)]
    e.set_gate(5, 1e30, 10)
    free = e.generate(prompts, 16)
    eos = int(free["tokens"][0, 3])
    e.set_gate(5, 1e30, 10, eos_id=eos)
    cut = e.generate(prompts, 16)
    for b in range(3):
        hits = np.nonzero(free["tokens"][b] == eos)[0]
        want = int(hits[0]) + 1 if len(hits) else 16
        assert cut["lens"][b] == want, (b, cut["lens"], want)
        assert (cut["tokens"][b, :want] == free["tokens"][b, :want]).all()
    e.set_gate(5, 0.0, 10)


def test_batch_rows_are_independent(tiny):
    e, os_, ol = tiny
    prompts = [si.prompt_np(s, "b", n, 512) for s, n in ((0, 16), (1, 9), (2, 23), (3, 16))]
    tau = _calibrate_tau(os_, ol, prompts[0], 40, 5, 50)
    e.set_gate(5, tau, 4)
    both = e.generate(prompts, 40)
    for b, p in enumerate(prompts):
        one = e.generate([p], 40)
        assert (one["tokens"][0] == both["tokens"][b]).all()
        assert (one["model_id"][0] == both["model_id"][b]).all()
        assert np.abs(one["H"][0] - both["H"][b]).max() < 1e-5


def test_grouped_schedule_gives_the_same_rows(tiny):
    """Rows are independent instances of the algorithm: letting small-model rows run ahead and
    serving large-model rows in groups must reproduce the lock-step run row by row, whatever
    the grouping thresholds, also when the run is cut into several decode calls."""
    e, os_, ol = tiny
    prompts = [si.prompt_np(s, "g", n, 512) for s, n in ((0, 16), (1, 9), (2, 23), (3, 12))]
    tau = _calibrate_tau(os_, ol, prompts[0], 48, 5, 50)
    e.set_gate(5, tau, 4)
    e.set_schedule(False)
    lock = e.generate(prompts, 48)
    assert 0 < lock["model_id"].mean() < 1
    ref0 = oracle.generate(os_, ol, prompts[0], 48, 5, tau, d_min=4)
    assert (lock["tokens"][0] == ref0["tokens"]).all() and (lock["model_id"][0] == ref0["model_id"]).all()
    try:
        for hi, lo in ((0.5, 0.25), (1.0, 0.0), (0.26, 0.26)):
            e.set_schedule(True, hi, lo)
            got = e.generate(prompts, 48)
            assert (got["tokens"] == lock["tokens"]).all(), (hi, lo)
            assert (got["model_id"] == lock["model_id"]).all(), (hi, lo)
            assert np.abs(got["H"] - lock["H"]).max() < 1e-5
            assert np.abs(got["Hbar"] - lock["Hbar"]).max() < 1e-5
            st = e.stats()
            assert st["tokens_small"] + st["tokens_large"] == 4 * 48
        # the same run in pieces: every row gets up to n tokens per call
        e.set_schedule(True, 0.5, 0.25)
        e.begin(prompts, 48)
        for n in (1, 7, 13, 100):
            e.decode(n)
        got = e.fetch()
        assert (got["tokens"] == lock["tokens"]).all() and (got["model_id"] == lock["model_id"]).all()
        assert (got["lens"] == 48).all()
        # free-running rows (ead_decode_tokens): token budgets for the batch as a whole, no row more than
        # `lead` tokens ahead of the slowest; the rows still come out the same
        for lead, budget in ((5, 23), (64, 50), (1, 4)):
            e.begin(prompts, 48)
            total = 0
            for _ in range(400):
                e.decode_tokens(budget, lead)
                part = e.fetch()
                assert part["lens"].sum() >= min(total + budget, 4 * 48), (lead, budget)
                total = int(part["lens"].sum())
                unfinished = part["lens"][part["lens"] < 48]
                if len(unfinished):
                    assert part["lens"].max() - unfinished.min() <= lead + 1, (lead, part["lens"])   # + 1: a pass in flight
                if (part["lens"] == 48).all():
                    break
            assert (part["lens"] == 48).all(), (lead, budget)
            assert (part["tokens"] == lock["tokens"]).all() and (part["model_id"] == lock["model_id"]).all(), (lead, budget)
            st = e.stats()
            assert st["tokens_small"] + st["tokens_large"] == 4 * 48
    finally:
        e.set_schedule(False)


def test_catchup_invariance(tiny):
    """Logits after a catch-up equal that model's logits scored from scratch on the same tokens."""
    e, os_, ol = tiny
    prompt = si.prompt_np(4, "cfg1", 16, 512)
    e.set_gate(5, 0.0, 10)                       # 10 small tokens, then the large model catches up
    out = e.generate([prompt], 12)
    seq = np.concatenate([prompt, out["tokens"][0]])
    sc = e.score(1, seq[:-1], want_logits=False)
    assert abs(sc["H"][len(prompt) + 10 - 1] - out["H"][0, 10]) < 1e-5
    assert sc["argmax"][len(prompt) + 10 - 1] == out["tokens"][0, 10]


def test_eos_and_errors(tiny):
    ead = _ead()
    e, os_, ol = tiny
    prompt = si.prompt_np(0, "cfg1", 16, 512)
    e.set_gate(5, 1e30, 10)
    full = e.generate([prompt], 12)
    eos = int(full["tokens"][0, 4])
    k = int(np.argmax(full["tokens"][0] == eos))
    e.set_gate(5, 1e30, 10, eos_id=eos)
    out = e.generate([prompt], 12)
    assert out["lens"][0] == k + 1
    e.set_gate(5, 1e30, 10)
    with pytest.raises(ead.EadError):
        e.generate([np.arange(120, dtype=np.int32)], 64)         # exceeds max_seq
    with pytest.raises(ead.EadError):
        e.generate([np.array([600], np.int32)], 4)               # token out of range
    with pytest.raises(ead.EadError):
        e.generate([prompt] * 5, 4)                               # exceeds max_batch


@pytest.mark.parametrize("pair,layers,T", [("llama", 2, 24), ("qwen", 2, 24), ("llama_1b_3b", 2, 24), ("qwen_15b_14b", 2, 24),
                                           ("llama", 2, 150), ("qwen", 2, 77), ("llama", 2, 120)])   # > 64 rows: 128-row sweeps, K split over workgroups up to 128
def test_bf16_truncated_pair_score_and_replay(pair, layers, T):
    """Full-width, depth-truncated bf16 pairs: teacher-forced logits / entropy / arg max for
    single rows (FMA path) and chunks of 24 to 150 rows (MFMA paths), then Algorithm 1 along
    the oracle's trajectory including catch-ups."""
    ead = _ead()
    ss, sl = (s.truncated(layers) for s in si.PAIRS[pair])
    Ws, Wl, os_, ol = _pair(ss, sl)
    e = ead.EAD(ss, Ws, sl, Wl, window=5, tau=0.0, d_min=4, max_batch=2, max_seq=max(96, T + 8))
    toks = si.prompt_np(0, pair, T, ss.vocab)
    refs = {}
    for which, om in ((0, os_), (1, ol)):
        print(f"{pair} score model {which}", flush=True)
        ref = refs[which] = om.forward_dense(toks)
        out = e.score(which, toks)                       # 24-row chunk -> MFMA kernels
        err = _check_logits(out["logits"], ref, TOL_LOGIT)
        Hr, ar = oracle.entropy_rows(ref)
        print(f"  logits rel err {err:.2e}  H err {np.abs(out['H'] - Hr).max():.2e}", flush=True)
        assert np.abs(out["H"] - Hr).max() < TOL_H
        gap = np.sort(ref, axis=1)
        clear = (gap[:, -1] - gap[:, -2]) > 2 * TOL_LOGIT * np.abs(ref).max(axis=1)
        assert (out["argmax"][clear] == ar[clear]).all()
    # Algorithm 1 teacher-forced along the oracle's own trajectory
    prompt = toks[:8]
    probe = oracle.generate(os_, ol, prompt, 24, 5, 1e30, d_min=4)
    tau = float(np.percentile(probe["Hbar"], 50))
    ref = oracle.generate(os_, ol, prompt, 24, 5, tau, d_min=4)
    e.set_gate(5, tau, 4)
    rp = e.replay([prompt], ref["tokens"], ref["model_id"])
    print(f"  replay: large share {ref['model_id'].mean():.2f} H err {np.abs(rp['H'][0] - ref['H']).max():.2e}", flush=True)
    assert np.abs(rp["H"][0] - ref["H"]).max() < TOL_H
    assert np.abs(rp["Hbar"][0] - ref["Hbar"]).max() < TOL_H
    safe = np.abs(ref["Hbar"] - tau) > BAND
    want_next = np.concatenate([ref["model_id"][1:], rp["next_model"][0][-1:]])
    assert (rp["next_model"][0][safe] == want_next[safe]).all()
    print(f"  decisions checked outside the band: {int(safe.sum())}/24", flush=True)
    e.close()


def test_fused_single_row_kernel_matches_per_layer_kernels(tiny):
    """The persistent one-kernel-per-step decode path against the per-layer kernels and the oracle."""
    e, os_, ol = tiny
    prompt = si.prompt_np(5, "cfg1", 16, 512)
    tau = _calibrate_tau(os_, ol, prompt, 48, 5, 55)
    e.set_gate(5, tau, 5)
    ref = oracle.generate(os_, ol, prompt, 48, 5, tau, d_min=5)
    outs = []
    for fused in (False, True):
        e.set_fused(fused)
        outs.append(e.generate([prompt], 48))
        rp = e.replay([prompt], ref["tokens"], ref["model_id"])
        assert np.abs(rp["H"][0] - ref["H"]).max() < 1e-4
        assert (rp["argmax"][0] == ref["tokens"]).all()
    e.set_fused(False)
    assert np.abs(outs[0]["H"] - outs[1]["H"]).max() < 1e-4
    if (np.abs(ref["Hbar"] - tau) > 1e-4).all():
        assert (outs[0]["tokens"] == outs[1]["tokens"]).all() and (outs[1]["tokens"][0] == ref["tokens"]).all()


@pytest.mark.parametrize("pair", ["llama", "qwen"])
def test_fused_kernel_bf16_truncated(pair):
    ead = _ead()
    ss, sl = (s.truncated(2) for s in si.PAIRS[pair])
    Ws, Wl, os_, ol = _pair(ss, sl)
    e = ead.EAD(ss, Ws, sl, Wl, window=5, tau=0.0, d_min=4, max_batch=1, max_seq=64)
    prompt = si.prompt_np(1, pair, 8, ss.vocab)
    probe = oracle.generate(os_, ol, prompt, 20, 5, 1e30, d_min=4)
    tau = float(np.percentile(probe["Hbar"], 50))
    ref = oracle.generate(os_, ol, prompt, 20, 5, tau, d_min=4)
    e.set_gate(5, tau, 4)
    # 1: the streamed persistent kernel (weights through an LDS ring); 2: the register-buffered one
    for fused in (1, 2):
        e.set_fused(fused)
        rp = e.replay([prompt], ref["tokens"], ref["model_id"])
        print(f"{pair} fused={fused} replay H err {np.abs(rp['H'][0] - ref['H']).max():.2e}", flush=True)
        assert np.abs(rp["H"][0] - ref["H"]).max() < TOL_H
        assert np.abs(rp["Hbar"][0] - ref["Hbar"]).max() < TOL_H
        safe = np.abs(ref["Hbar"] - tau) > BAND
        assert safe.sum() >= len(safe) // 3
        want_next = np.concatenate([ref["model_id"][1:], rp["next_model"][0][-1:]])
        assert (rp["next_model"][0][safe] == want_next[safe]).all()
    e.set_fused(False)
    e.close()
