"""Pins for the oracle's transformer forward pass and its Algorithm 1 loop."""
import math

import numpy as np
import pytest

import oracle
import synth_inputs as si
from np_forward import forward as np_forward

MINI = si.ModelShape("mini", 2, 64, 4, 2, 96, 97, 1e-5, 1e4, bf16=False)      # GQA, odd vocab
MINI_L = si.ModelShape("mini-l", 3, 96, 6, 3, 160, 97, 1e-5, 1e4, bf16=False)


def _weights(shape, seed=0, std=0.2):
    W = si.model_weights_np(shape, seed, std=std)
    rng = np.random.default_rng(seed + 100)
    for k in W:                                    # non-trivial gains so a dropped gain shows
        if "norm" in k:
            W[k] = (1 + 0.3 * rng.standard_normal(W[k].shape)).astype(np.float32)
    return W


@pytest.mark.parametrize("shape", [MINI, MINI_L, si.TINY_S], ids=lambda s: s.name)
def test_dense_cached_and_numpy64_agree(shape):
    W = _weights(shape, std=0.2 if shape.d_model < 128 else 0.05)
    toks = si.tokens_np(1, "t", 23, shape.vocab)
    mdl = oracle.Model(shape, W)
    dense, cached, ref = mdl.forward_dense(toks), mdl.forward_cached(toks), np_forward(shape, W, toks)
    scale = np.abs(ref).max()
    assert np.abs(dense - ref).max() < 1e-5 * scale
    assert np.abs(cached - ref).max() < 1e-5 * scale
    assert np.abs(cached - dense).max() < 1e-5 * scale


def test_single_token_one_layer_closed_form():
    # one key: softmax is 1, attention returns v, rotary plays no role (position 0)
    shape = si.ModelShape("one", 1, 64, 4, 2, 96, 97, 1e-5, 1e4, bf16=False)
    W = _weights(shape)
    f8 = lambda k: W[k].astype(np.float64)
    norm = lambda v, g: v / math.sqrt((v * v).mean() + shape.rms_eps) * g
    for tok in (0, 5, 96):
        x0 = f8("embed")[tok]
        v = f8("layers.0.wv") @ norm(x0, f8("layers.0.norm_attn"))              # [KV*hd]
        v = np.repeat(v.reshape(shape.n_kv_heads, shape.head_dim), 2, axis=0).ravel()
        x1 = x0 + f8("layers.0.wo") @ v
        b = norm(x1, f8("layers.0.norm_ffn"))
        g = f8("layers.0.w_gate") @ b
        x2 = x1 + f8("layers.0.w_down") @ (g / (1 + np.exp(-g)) * (f8("layers.0.w_up") @ b))
        want = f8("lm_head") @ norm(x2, f8("norm_final"))
        got = oracle.Model(shape, W).forward_dense([tok])[0]
        assert np.abs(got - want).max() < 1e-5 * np.abs(want).max()


def test_rope_invariants():
    L = oracle.lib()
    rng = np.random.default_rng(0)
    hd, nh = 32, 3
    v = rng.standard_normal(nh * hd).astype(np.float32)
    a = v.copy(); L.oracle_rope(oracle._fp(a), nh, hd, 0, 1e4)
    assert (a == v).all()                                        # position 0: identity
    a = v.copy(); L.oracle_rope(oracle._fp(a), nh, hd, 37, 1e4)
    assert np.allclose(np.linalg.norm(a.reshape(nh, hd), axis=1),
                       np.linalg.norm(v.reshape(nh, hd), axis=1), rtol=1e-6)
    # pair (i, i+hd/2) turns by pos * theta^(-2i/hd); element 0 pairs with element 16
    e = np.zeros(hd, np.float32); e[0] = 1
    L.oracle_rope(oracle._fp(e), 1, hd, 1, 1e4)
    assert abs(e[0] - math.cos(1.0)) < 1e-7 and abs(e[16] - math.sin(1.0)) < 1e-7
    e = np.zeros(hd, np.float32); e[3] = 1
    L.oracle_rope(oracle._fp(e), 1, hd, 5, 1e4)
    ang = 5 * 1e4 ** (-6 / 32)
    assert abs(e[3] - math.cos(ang)) < 1e-7 and abs(e[19] - math.sin(ang)) < 1e-7
    # q.k after rotation depends only on the position difference
    q = rng.standard_normal(hd).astype(np.float32); k = rng.standard_normal(hd).astype(np.float32)
    dots = []
    for pq, pk in ((9, 4), (105, 100), (5, 0)):
        a, b = q.copy(), k.copy()
        L.oracle_rope(oracle._fp(a), 1, hd, pq, 1e4); L.oracle_rope(oracle._fp(b), 1, hd, pk, 1e4)
        dots.append(float(a.astype(np.float64) @ b.astype(np.float64)))
    assert max(dots) - min(dots) < 1e-5


def test_gqa_equals_mha_with_replicated_kv_heads():
    W = _weights(MINI)
    mha = si.ModelShape("mha", MINI.n_layers, MINI.d_model, MINI.n_heads, MINI.n_heads, MINI.d_ffn,
                        MINI.vocab, MINI.rms_eps, MINI.rope_theta, bf16=False)
    W2 = dict(W)
    g, hd = MINI.n_heads // MINI.n_kv_heads, MINI.head_dim
    for l in range(MINI.n_layers):
        for n in ("wk", "wv"):
            w = W[f"layers.{l}.{n}"].reshape(MINI.n_kv_heads, hd, MINI.d_model)
            W2[f"layers.{l}.{n}"] = np.repeat(w, g, axis=0).reshape(-1, MINI.d_model)
    toks = si.tokens_np(2, "t", 11, MINI.vocab)
    a = oracle.Model(MINI, W).forward_dense(toks)
    b = oracle.Model(mha, W2).forward_dense(toks)
    assert np.abs(a - b).max() < 1e-6 * np.abs(a).max()


def test_zero_output_projections_give_lookup_table_model():
    W = _weights(MINI)
    for l in range(MINI.n_layers):
        W[f"layers.{l}.wo"][:] = 0
        W[f"layers.{l}.w_down"][:] = 0
    toks = si.tokens_np(3, "t", 9, MINI.vocab)
    got = oracle.Model(MINI, W).forward_dense(toks)
    E = W["embed"].astype(np.float64)[toks]
    n = E / np.sqrt((E * E).mean(-1, keepdims=True) + MINI.rms_eps) * W["norm_final"]
    want = n @ W["lm_head"].astype(np.float64).T
    assert np.abs(got - want).max() < 1e-5 * np.abs(want).max()


def test_causality():
    W = _weights(MINI)
    mdl = oracle.Model(MINI, W)
    toks = si.tokens_np(4, "t", 12, MINI.vocab)
    a = mdl.forward_dense(toks)
    t2 = toks.copy(); t2[8:] = (t2[8:] + 1) % MINI.vocab
    b = mdl.forward_dense(t2)
    assert (a[:8] == b[:8]).all() and not np.allclose(a[8:], b[8:])


# ----------------------------------------------------------------- Algorithm 1 loop
def _greedy(mdl, prompt, n):
    seq = list(prompt)
    Hs = []
    for _ in range(n):
        lg = mdl.forward_dense(seq)[-1]
        h, tok = oracle.entropy(lg)
        Hs.append(h); seq.append(tok)
    return np.array(seq[len(prompt):]), np.array(Hs)


@pytest.fixture(scope="module")
def pair():
    return (oracle.Model(MINI, _weights(MINI, 0)), oracle.Model(MINI_L, _weights(MINI_L, 1)))


def test_tau_infinite_is_small_only_greedy(pair):
    S, L = pair
    prompt = si.prompt_np(0, "p", 6, MINI.vocab)
    out = oracle.generate(S, L, prompt, 20, 5, 1e30, d_min=3)
    toks, Hs = _greedy(S, prompt, 20)
    assert (out["tokens"] == toks).all() and (out["model_id"] == 0).all()
    assert np.allclose(out["H"], Hs, atol=1e-5)


def test_tau_minus_infinite_dmin1_hands_over_after_first_token(pair):
    S, L = pair
    prompt = si.prompt_np(1, "p", 6, MINI.vocab)
    out = oracle.generate(S, L, prompt, 12, 5, -1e30, d_min=1)
    first, _ = _greedy(S, prompt, 1)
    rest, _ = _greedy(L, list(prompt) + [int(first[0])], 11)
    assert list(out["model_id"]) == [0] + [1] * 11
    assert out["tokens"][0] == first[0] and (out["tokens"][1:] == rest).all()


def test_generate_follows_gate_on_its_own_entropies(pair):
    # whatever the models say, ids must be what the gate yields on the recorded entropies,
    # and every recorded entropy/token must be the forced model's dense-forward value
    S, L = pair
    prompt = si.prompt_np(2, "p", 5, MINI.vocab)
    probe = oracle.generate(S, L, prompt, 30, 3, 1e30, d_min=2)
    tau = float(np.median(probe["Hbar"]))
    out = oracle.generate(S, L, prompt, 30, 3, tau, d_min=2)
    hb, ids = oracle.gate_trace(out["H"], 3, 2, tau)
    assert (ids == out["model_id"]).all() and (hb == out["Hbar"]).all()
    assert 0 < out["model_id"].sum() < 30                        # both models were used
    seq = np.concatenate([prompt, out["tokens"]])
    rp = oracle.replay(S, L, seq, out["model_id"], len(prompt), 3, tau, d_min=2)
    assert (rp["argmax"] == out["tokens"]).all()
    assert np.allclose(rp["H"], out["H"], atol=1e-5)
    assert (rp["next_model"][:-1] == out["model_id"][1:]).all()


def test_w1_dmin1_is_per_token_thresholding(pair):
    S, L = pair
    prompt = si.prompt_np(3, "p", 5, MINI.vocab)
    probe = oracle.generate(S, L, prompt, 20, 1, 1e30, d_min=1)
    tau = float(np.median(probe["H"]))
    out = oracle.generate(S, L, prompt, 20, 1, tau, d_min=1)
    assert (out["Hbar"] == out["H"]).all()
    want = np.concatenate([[0], (out["H"][:-1] > np.float32(tau)).astype(np.uint8)])
    assert (out["model_id"] == want).all()


def test_eos_stops_generation(pair):
    S, L = pair
    prompt = si.prompt_np(0, "p", 6, MINI.vocab)
    full = oracle.generate(S, L, prompt, 10, 5, 1e30)
    out = oracle.generate(S, L, prompt, 10, 5, 1e30, eos_id=int(full["tokens"][3]))
    k = int(np.argmax(full["tokens"] == full["tokens"][3]))
    assert len(out["tokens"]) == k + 1 and (out["tokens"] == full["tokens"][:k + 1]).all()
