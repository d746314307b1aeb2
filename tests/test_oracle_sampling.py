"""Pins for the oracle's sampling step (Algorithm 1: y ~ softmax(l / T)), CPU only.

The sampler is the Gumbel-max identity over a counter-based generator; nothing here calls the
GPU library.  Each test fails for a plausible mistake: a wrong round constant or word order
(known answers, integer re-implementation), a wrong uniform mapping (range / moments), a
missing temperature or a sign error in the noise (chi-square against softmax(l/T)), noise
applied to the entropy (entropy must stay that of the raw logits)."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle
import synth_inputs as si

HERE = os.path.dirname(os.path.abspath(__file__))


def _kat():
    rows = []
    for line in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_generator_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle.philox4x32_10(ctr, key) == want


def _philox_py(ctr, key):
    """Independent transcription of the round function with Python integers."""
    c = list(ctr); k = list(key)
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]; p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_generator_against_integer_reimplementation():
    rng = np.random.default_rng(5)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert oracle.philox4x32_10(ctr, key) == _philox_py(ctr, key)


def test_uniform_mapping_and_counter_layout():
    seed, b, n = 0x1234_5678_9ABC_DEF0, 3, 17
    for i in (0, 1, 2, 3, 4, 7, 1001, 151935):
        word = _philox_py([i >> 2, n, b, 0], [seed & 0xFFFFFFFF, seed >> 32])[i & 3]
        want = np.float32((2 * (word >> 9) + 1) / 2.0**24)
        assert oracle.uniform(seed, b, n, i) == want
    u = np.array([oracle.uniform(7, 0, 0, i) for i in range(20000)])
    assert u.min() > 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1.0 / 12.0) < 0.005
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    # distinct sequences, token positions and seeds give distinct streams
    base = [oracle.uniform(7, 0, 0, i) for i in range(64)]
    for other in ([oracle.uniform(7, 1, 0, i) for i in range(64)], [oracle.uniform(7, 0, 1, i) for i in range(64)],
                  [oracle.uniform(8, 0, 0, i) for i in range(64)]):
        assert sum(a == o for a, o in zip(base, other)) < 4


def test_gumbel_noise_moments():
    g = np.concatenate([oracle.gumbel(11, 0, n, 4096) for n in range(8)]).astype(np.float64)
    assert abs(g.mean() - 0.5772156649) < 0.02            # Euler-Mascheroni
    assert abs(g.var() - np.pi**2 / 6.0) < 0.06
    u = oracle.uniform(11, 0, 0, 5)
    assert abs(oracle.gumbel(11, 0, 0, 8)[5] - (-np.log(-np.log(np.float64(u))))) < 1e-6


@pytest.mark.parametrize("T", [0.5, 1.0, 2.0])
def test_sampled_frequencies_follow_softmax_of_scaled_logits(T):
    l = np.array([2.0, 1.0, 0.0, -1.0, 0.5, 1.5, -3.0, 0.25], dtype=np.float32)
    N = 20000
    counts = np.bincount([oracle.sample(l, T, 42, 0, n) for n in range(N)], minlength=l.size)
    p = np.exp(l.astype(np.float64) / T); p /= p.sum()
    chi = stats.chisquare(counts, p * N)
    assert chi.pvalue > 1e-3, (counts, p * N)
    # the same draws against softmax at another temperature must be rejected
    q = np.exp(l.astype(np.float64) / (3.0 * T)); q /= q.sum()
    assert stats.chisquare(counts, q * N).pvalue < 1e-6


def test_temperature_limits_and_determinism():
    l = si.logits_np(3, "samp", 1, 512)[0]
    am = int(np.argmax(l))
    assert oracle.sample(l, 0.0, 1, 0, 0) == am
    assert all(oracle.sample(l, 1e-4, 1, 0, n) == am for n in range(20))
    tie = np.zeros(16, np.float32); tie[[4, 9]] = 1.0
    assert oracle.sample(tie, 0.0, 1, 0, 0) == 4                      # lowest index on ties
    flat = np.zeros(8, np.float32)
    counts = np.bincount([oracle.sample(flat, 1.0, 9, 0, n) for n in range(8000)], minlength=8)
    assert stats.chisquare(counts).pvalue > 1e-3                       # uniform when all logits are equal
    assert oracle.sample(l, 0.8, 5, 2, 7) == oracle.sample(l, 0.8, 5, 2, 7)
    # the definition written out with the exposed noise
    g = oracle.gumbel(5, 2, 7, l.size)
    score = (l.astype(np.float64) * np.float64(np.float32(1.0) / np.float32(0.8)) + g.astype(np.float64)).astype(np.float32)
    assert oracle.sample(l, 0.8, 5, 2, 7) == int(np.argmax(score))


def test_algorithm1_with_sampling_keeps_raw_logit_entropy():
    ss, sl = si.TINY_S, si.TINY_L
    ms = oracle.Model(ss, si.model_weights_np(ss, 0)); ml = oracle.Model(sl, si.model_weights_np(sl, 0))
    prompt = si.prompt_np(0, "samp", 8, ss.vocab)
    greedy = oracle.generate(ms, ml, prompt, 12, 5, 1e30)
    a = oracle.generate(ms, ml, prompt, 12, 5, 1e30, temperature=1.0, seed=3)
    b = oracle.generate(ms, ml, prompt, 12, 5, 1e30, temperature=1.0, seed=3)
    c = oracle.generate(ms, ml, prompt, 12, 5, 1e30, temperature=1.0, seed=4)
    assert (a["tokens"] == b["tokens"]).all() and (a["H"] == b["H"]).all()
    assert (a["tokens"] != c["tokens"]).any()
    assert (a["tokens"] != greedy["tokens"]).any()          # near-uniform distributions: sampling differs from arg max
    assert a["H"][0] == greedy["H"][0]                      # the first entropy does not depend on T (same context, raw logits)
    # teacher-forced replay reproduces the sampled choices
    seq = np.concatenate([prompt, a["tokens"]])
    rp = oracle.replay(ms, ml, seq, a["model_id"], len(prompt), 5, 1e30, temperature=1.0, seed=3)
    assert (rp["choice"] == a["tokens"]).all()
    assert np.abs(rp["H"] - a["H"]).max() < 1e-5
