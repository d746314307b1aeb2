"""Pins for the oracle's entropy, window and gate (Eq. 1-4, Algorithm 1).

None of these re-types the oracle's formula: they are closed forms, invariants,
an independent float64 numpy evaluation, hand-derived traces and the values the
paper prints in Table 1.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- entropy
@pytest.mark.parametrize("V", [2, 512, 128256, 151936])
def test_uniform_logits_give_ln_V(V):
    for const in (0.0, -3.5, 17.0):
        H, am = oracle.entropy(np.full(V, const, np.float32))
        assert abs(H - math.log(V)) < 1e-9
        assert am == 0                      # lowest index on ties
    Hb, _ = oracle.entropy(np.zeros(V, np.float32), oracle.BITS)
    assert abs(Hb - math.log2(V)) < 1e-9


def test_bits_is_nats_over_ln2():
    rng = np.random.default_rng(0)
    l = rng.normal(0, 3, 1000).astype(np.float32)
    assert abs(oracle.entropy(l, oracle.BITS)[0] - oracle.entropy(l)[0] / math.log(2)) < 1e-12
    assert abs(oracle.entropy(np.zeros(512, np.float32), oracle.BITS)[0] - 9.0) < 1e-12


@pytest.mark.parametrize("V,k", [(512, 0), (512, 511), (151936, 77777)])
def test_one_hot_gives_zero(V, k):
    for low in (-np.inf, -1e4):
        l = np.full(V, low, np.float32)
        l[k] = 0.0
        H, am = oracle.entropy(l)
        assert H == 0.0 and am == k


def test_shift_invariance():
    rng = np.random.default_rng(1)
    l = rng.normal(0, 2, 4096).astype(np.float64)
    l = np.round(l * 64) / 64                      # exactly representable after a shift
    h0 = oracle.entropy(l.astype(np.float32))[0]
    for c in (8.0, -32.0, 100.0):
        assert abs(oracle.entropy((l + c).astype(np.float32))[0] - h0) < 1e-9


@pytest.mark.parametrize("V,a", [(512, 1.0), (512, 9.0), (151936, 12.5), (1000, -4.0)])
def test_one_raised_logit_closed_form(V, a):
    # l_0 = a, the rest 0: p = e^a / (e^a + V - 1); the rest share 1 - p equally
    l = np.zeros(V, np.float32)
    l[0] = a
    p = math.exp(a) / (math.exp(a) + V - 1)
    q = (1 - p) / (V - 1)
    want = -p * math.log(p) - (V - 1) * q * math.log(q)
    H, am = oracle.entropy(l)
    assert abs(H - want) < 1e-9 * max(1.0, want)
    assert am == (0 if a > 0 else 1)


@pytest.mark.parametrize("k", [1, 2, 7, 300])
def test_k_equal_logits_rest_minus_inf(k):
    l = np.full(1000, -np.inf, np.float32)
    idx = np.random.default_rng(k).choice(1000, k, replace=False)
    l[idx] = 2.5
    H, am = oracle.entropy(l)
    assert abs(H - math.log(k)) < 1e-12
    assert am == idx.min()


@pytest.mark.parametrize("seed", range(5))
def test_against_float64_numpy_definition(seed):
    rng = np.random.default_rng(seed)
    V = int(rng.integers(2, 1000))
    l = (rng.normal(0, rng.uniform(0.1, 10), V)).astype(np.float32)
    x = l.astype(np.float64)
    p = np.exp(x - x.max())
    p /= p.sum()
    want = -(p[p > 0] * np.log(p[p > 0])).sum()
    H, am = oracle.entropy(l)
    assert abs(H - want) < 1e-10
    assert abs(oracle.entropy_direct(l) - want) < 1e-10
    assert am == int(np.argmax(l))


def test_gaussian_logits_sanity():
    # N(0, s^2) logits, large V: H ~ ln V - s^2/2
    rng = np.random.default_rng(3)
    V, s = 151936, 0.5
    H, _ = oracle.entropy(rng.normal(0, s, V).astype(np.float32))
    assert abs(H - (math.log(V) - s * s / 2)) < 2e-2


@pytest.mark.parametrize("V", [512, 128256, 151936])
def test_argmax_planted_and_ties(V):
    rng = np.random.default_rng(V)
    base = rng.normal(0, 1, V).astype(np.float32)
    for k in (0, 1, V // 2 + 3, V - 1):
        l = base.copy()
        l[k] = 50.0
        assert oracle.entropy(l)[1] == k
    l = base.copy()
    l[[V - 1, 17, V // 3]] = 60.0               # exact three-way tie: lowest index wins
    assert oracle.entropy(l)[1] == 17


def test_chunk_merge_identity():
    # splitting the vocabulary and merging (m, Z, S) triples reproduces the one-shot
    # value: the identity any tiled implementation relies on, checked against the oracle
    rng = np.random.default_rng(7)
    l = rng.normal(0, 4, 5000).astype(np.float32)
    want = oracle.entropy(l)[0]
    x = l.astype(np.float64)
    for cuts in ([2500], [1, 4999], [100, 101, 3000], list(range(500, 5000, 500))):
        parts = np.split(x, cuts)
        M = max(p.max() for p in parts)
        Z = S = 0.0
        for p in parts:
            m = p.max(); e = np.exp(p - m); z = e.sum(); s = (e * (p - m)).sum()
            f = math.exp(m - M)
            Z += z * f
            S += f * (s + (m - M) * z)
        assert abs((math.log(Z) - S / Z) - want) < 1e-10


# ----------------------------------------------------------------- window
def test_window_mean_brute_force():
    rng = np.random.default_rng(0)
    H = rng.uniform(0, 12, 200).astype(np.float32)
    for w in (1, 2, 5, 17, 500):
        for t in range(1, len(H) + 1):
            n = min(t, w)
            want = np.float64(H[t - n:t].astype(np.float64).sum() / n)
            assert abs(oracle.window_mean(H[:t], w) - want) < 1e-5
    for t in range(1, 50):                                  # w = 1: the mean is H_t itself
        assert oracle.window_mean(H[:t], 1) == H[t - 1]
    c = np.full(40, 3.25, np.float32)                       # constant trace
    for t in range(1, 41):
        assert oracle.window_mean(c[:t], 5) == 3.25


def test_window_mean_float_order():
    # summed oldest to newest in float: 1e8 + 1 + 1 + 1 + 1 differs from the reverse order
    H = np.array([1e8, 1, 1, 1, 1], np.float32)
    s = np.float32(0)
    for v in H:
        s = np.float32(s + v)
    assert oracle.window_mean(H, 5) == np.float32(s / np.float32(5))


# ----------------------------------------------------------------- gate traces
def _traces():
    out = []
    for line in open(os.path.join(GOLD, "gate_traces.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, w, d, tau, H, Hb, ids = [f.strip() for f in line.split("|")]
        out.append(pytest.param(int(w), int(d), float(tau), [float(v) for v in H.split()],
                                [float(v) for v in Hb.split()],
                                [0 if c == "S" else 1 for c in ids.split()], id=name))
    return out


@pytest.mark.parametrize("w,d_min,tau,H,Hbar,ids", _traces())
def test_hand_derived_gate_traces(w, d_min, tau, H, Hbar, ids):
    hb, got = oracle.gate_trace(H, w, d_min, tau)
    assert list(got) == ids
    assert np.allclose(hb, Hbar, atol=1e-6)


def test_divide_by_w_reading_would_fail_T3():
    # the literal Eq. 3 (divide by w during warm-up) is NOT what the oracle does
    H = [10, 0, 0, 0, 0, 0]
    _, ids = oracle.gate_trace(H, 5, 1, 2.1)
    literal = [sum(H[max(0, t - 4):t + 1]) / 5 for t in range(6)]
    assert all(abs(v - 2.0) < 1e-12 for v in literal[:5])   # would never exceed tau = 2.1
    assert list(ids) == [0, 1, 1, 1, 1, 0]


def test_gate_brute_force_random():
    # an independent python transcription of Algorithm 1's control flow, random traces
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 80)); w = int(rng.integers(1, 8)); d = int(rng.integers(1, 13))
        H = rng.uniform(0, 4, n).astype(np.float32); tau = float(np.float32(rng.uniform(0, 4)))
        model, c, W, want = "S", 0, [], []
        for t in range(n):
            W.append(H[t])
            acc = np.float32(0)
            for v in W[-w:]:
                acc = np.float32(acc + v)
            hb = np.float32(acc / np.float32(len(W[-w:])))
            want.append(0 if model == "S" else 1)
            c += 1
            if c >= d:
                if model == "S" and hb > np.float32(tau):
                    model, c = "L", 0
                elif model == "L" and hb <= np.float32(tau):
                    model, c = "S", 0
        assert list(oracle.gate_trace(H, w, d, tau)[1]) == want


def test_gate_step_counter_semantics():
    # c is incremented before the test and reset only on an actual switch
    assert oracle.gate_step(oracle.SMALL, 0, 5.0, 1.0, 3) == (oracle.SMALL, 1)
    assert oracle.gate_step(oracle.SMALL, 1, 5.0, 1.0, 3) == (oracle.SMALL, 2)
    assert oracle.gate_step(oracle.SMALL, 2, 5.0, 1.0, 3) == (oracle.LARGE, 0)
    assert oracle.gate_step(oracle.SMALL, 7, 0.5, 1.0, 3) == (oracle.SMALL, 8)   # no reset
    assert oracle.gate_step(oracle.LARGE, 2, 1.0, 1.0, 3) == (oracle.SMALL, 0)   # tie goes small
    assert oracle.gate_step(oracle.LARGE, 2, 1.5, 1.0, 3) == (oracle.LARGE, 3)


# ----------------------------------------------------------------- Table 1 statistic
def test_param_ratio_reproduces_table1():
    rows = [l.split() for l in open(os.path.join(GOLD, "table1_param_ratio.txt"))
            if l.strip() and not l.startswith("#")]
    base = {r[0]: float(r[3]) / 100 for r in rows if r[1] == "99"}
    assert len(rows) == 32 and len(base) == 4
    # Rows the paper prints that do not follow from its own footnote and its own
    # tau=99 row (the table is at odds with itself there): the whole 11B/3B block
    # drifts by up to 0.8 points, and one 3B/1B row by 0.19.  Every other row must
    # reproduce to the printed decimal (inputs are rounded to 0.1 %, so <= 0.1).
    exact = 0
    for pair, tau, usage, ratio in rows:
        got = 100 * oracle.param_ratio(float(usage) / 100, base[pair], 1.0)
        loose = pair == "llama-11b-3b" or (pair, tau) == ("llama-3b-1b", "0.0625")
        assert abs(got - float(ratio)) <= (0.8 if loose else 0.1), (pair, tau, got, ratio)
        exact += not loose
    assert exact == 23
    assert oracle.param_ratio(0.0, 3.0, 12.0) == 0.25
    assert oracle.param_ratio(1.0, 3.0, 12.0) == 1.0
