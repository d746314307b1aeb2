"""Helpers shared by the GPU parity tests (test infrastructure; calls only the oracle and the C-ABI binding)."""
import ctypes as C

import numpy as np

import oracle
import synth_inputs as si

TOL_LOGIT = 2e-2     # max |diff| <= TOL * max |ref| per row  (bf16 kernels vs fp32 oracle)
TOL_H = 1e-2         # nats
BAND = 1e-2          # switch decisions are exempt when |window mean - tau| < BAND


def lm_std_for(shape, sigma=1.5):
    """LM-head standard deviation that makes the logits about N(0, sigma^2) behind a unit-rms final norm."""
    return sigma / float(np.sqrt(shape.d_model))


def make_pair(shape_s, shape_l, seed=0, std=0.02, gain_std=0.0, lm_sigma=None):
    """Weights of a pair on the GPU and the same values (up-cast) in two oracle models.
    gain_std > 0: RMSNorm gains 1 + N(0, gain_std^2) instead of 1; lm_sigma: LM heads drawn so that the
    logits have about that standard deviation (a wider entropy spread from position to position)."""
    out = []
    for sh in (shape_s, shape_l):
        lm = lm_std_for(sh, lm_sigma) if lm_sigma else None
        W = si.model_weights_torch(sh, seed, "cuda", std, gain_std, lm)
        out.append((W, oracle.Model(sh, {k: v.float().cpu().numpy() for k, v in W.items()})))
    (Ws, os_), (Wl, ol) = out
    return Ws, Wl, os_, ol


def check_logits(got, ref, tol):
    err = np.abs(got - ref).max(axis=1) / np.abs(ref).max(axis=1)
    assert err.max() < tol, err.max()
    return err.max()


def trajectory_logit_stats(os_, ol, prompt, tokens, model_id):
    """Along a given trajectory (prompt, then tokens[i] produced by model_id[i]): for every generated
    position the producing model's logits through the oracle's cached forward pass, reduced to
    (H, arg max, gap between the two largest logits, largest |logit|).  A model consumes the positions it
    has not seen only when it is asked for logits, as in Algorithm 1."""
    L = oracle.lib()
    seq = np.concatenate([np.asarray(prompt, np.int32), np.asarray(tokens, np.int32)])
    n, P = len(tokens), len(prompt)
    models = (os_, ol)
    caches = [L.oracle_cache_new(C.byref(m.c), int(len(seq))) for m in models]
    V = os_.shape.vocab
    logits = np.empty(V, np.float32)
    H = np.zeros(n); am = np.zeros(n, np.int64); gap = np.zeros(n); top = np.zeros(n)
    try:
        for i in range(n):
            m = int(model_id[i])
            have = L.oracle_cache_len(caches[m])
            for pos in range(have, P + i):
                last = pos == P + i - 1
                rc = L.oracle_forward_cached(C.byref(models[m].c), caches[m], int(seq[pos]),
                                             logits.ctypes.data_as(C.POINTER(C.c_float)) if last else None)
                assert rc == 0
            H[i], am[i] = oracle.entropy(logits)
            two = np.partition(logits, V - 2)[V - 2:]
            gap[i] = float(two[1] - two[0]); top[i] = float(np.abs(logits).max())
    finally:
        for c in caches:
            L.oracle_cache_free(c)
    return {"H": H, "argmax": am, "gap": gap, "top": top}


def check_replay_row(rp, b, ref, tau, n_new, stats=None, tol_h=TOL_H, band=BAND, tol_logit=TOL_LOGIT):
    """One row of an ead_replay result against the oracle's run of that row: entropies, window means,
    the library's own arg max where the oracle's two best logits are further apart than twice the logit
    tolerance, and Eq. 4's decision wherever the window mean is outside the exemption band.
    Returns (decisions checked, arg maxes checked)."""
    assert np.abs(rp["H"][b] - ref["H"]).max() < tol_h, (b, np.abs(rp["H"][b] - ref["H"]).max())
    assert np.abs(rp["Hbar"][b] - ref["Hbar"]).max() < tol_h, b
    safe = np.abs(ref["Hbar"] - tau) > band
    want_next = np.concatenate([ref["model_id"][1:], rp["next_model"][b][-1:]])
    assert (rp["next_model"][b][safe] == want_next[safe]).all(), b
    n_arg = 0
    if stats is not None:
        assert np.abs(stats["H"] - ref["H"]).max() < 1e-4          # the oracle agrees with itself
        clear = stats["gap"] > 2 * tol_logit * stats["top"]
        assert (rp["argmax"][b][clear] == ref["tokens"][clear]).all(), b
        n_arg = int(clear.sum())
    return int(safe.sum()), n_arg
