"""GPU parity: entropy / arg max / window / switch rule kernels against the CPU oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

TOL_H = 1e-2        # nats


def _ead():
    import paper_2502_06833_amd as ead
    return ead


@pytest.mark.parametrize("V,rows,dtype", [(512, 3, torch.float32), (4096, 7, torch.bfloat16),
                                          (128256, 5, torch.bfloat16), (151936, 64, torch.bfloat16),
                                          (151936, 2, torch.float32), (1000, 4, torch.float32)])
def test_entropy_argmax_matches_oracle(V, rows, dtype):
    ead = _ead()
    print(f"entropy_argmax V={V} rows={rows} {dtype}", flush=True)
    lg = si.logits_torch(0, f"lg{V}", rows, V, dtype, "cuda")
    ref = si.logits_np(0, f"lg{V}", rows, V, bf16=(dtype == torch.bfloat16))
    assert (lg.float().cpu().numpy() == ref).all()          # same inputs on both sides
    for unit in (ead.NATS, ead.BITS):
        H, am = ead.entropy_argmax(lg, unit)
        Hr, ar = oracle.entropy_rows(ref, unit)
        tol = TOL_H / (math.log(2) if unit == ead.BITS else 1.0)
        assert np.abs(H.cpu().numpy() - Hr).max() < tol
        assert (am.cpu().numpy() == ar).all()
    assert Hr.min() < 0.6 * math.log2(V) and Hr.max() > 0.8 * math.log2(V) or rows < 8


def test_entropy_fixed_cases_on_gpu():
    ead = _ead()
    V = 151936
    x = torch.zeros(4, V, dtype=torch.bfloat16, device="cuda")
    x[1] = -1e4; x[1, 77777] = 0.0                      # one-hot
    x[2] = float("-inf"); x[2, 5] = 1.0; x[2, V - 1] = 1.0   # two equal, rest -inf
    x[3, V - 1] = 3.0; x[3, 17] = 3.0                   # tie: lowest index
    H, am = ead.entropy_argmax(x)
    H, am = H.cpu().numpy(), am.cpu().numpy()
    assert abs(H[0] - math.log(V)) < 1e-4 and am[0] == 0
    assert abs(H[1]) < 1e-6 and am[1] == 77777
    assert abs(H[2] - math.log(2)) < 1e-5 and am[2] == 5
    assert am[3] == 17
    ref = oracle.entropy(x[3].float().cpu().numpy())[0]
    assert abs(H[3] - ref) < 1e-4


@pytest.mark.parametrize("w,d_min,tau", [(5, 10, 2.0), (5, 1, 2.0), (2, 3, 1.0), (1, 1, 6.0), (7, 4, 9.5)])
def test_gate_step_bit_exact(w, d_min, tau):
    ead = _ead()
    rows, steps = 64, 200
    rng = np.random.default_rng(w * 100 + d_min)
    Hs = rng.uniform(0, 12, (steps, rows)).astype(np.float32)
    Hs[:, 0] = tau                                       # a row sitting exactly on the threshold
    g = ead.Gate(rows, w, tau, d_min)
    ids = np.zeros((steps, rows), np.uint8); hb = np.zeros((steps, rows), np.float32)
    nxt = np.zeros((steps, rows), np.uint8)
    Hd = torch.from_numpy(Hs).cuda()
    for t in range(steps):
        a, b, c = g.step(Hd[t])
        ids[t], hb[t], nxt[t] = a.cpu().numpy(), b.cpu().numpy(), c.cpu().numpy()
    for r in range(rows):
        hbr, idr = oracle.gate_trace(Hs[:, r], w, d_min, tau)
        assert (ids[:, r] == idr).all(), r
        assert (hb[:, r] == hbr).all(), r                # same fp32 sum order: bit-exact
        assert (nxt[:-1, r] == idr[1:]).all()
    g.close()


def test_hand_traces_on_gpu():
    ead = _ead()
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "gate_traces.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, w, d, tau, H, Hb, ids = [f.strip() for f in line.split("|")]
        H = np.array([float(v) for v in H.split()], np.float32)
        want = [0 if c == "S" else 1 for c in ids.split()]
        g = ead.Gate(1, int(w), float(tau), int(d))
        got = []
        for v in H:
            m, _, _ = g.step(torch.tensor([v], dtype=torch.float32, device="cuda"))
            got.append(int(m.cpu()[0]))
        assert got == want, name
        g.close()


def test_entropy_gate_stream_config2():
    """bf16 logits [64, 151936], row scales U[0.5, 8], window 5, tau 2.0 nats: the fused
    entropy + gate call tracks the oracle step by step (decisions exempt within 1e-2 of tau)."""
    ead = _ead()
    rows, V, steps, w, tau = 64, 151936, 12, 5, 2.0
    for d_min in (10, 1):
        g = ead.Gate(rows, w, tau, d_min)
        Hs = np.zeros((steps, rows), np.float32); ids = np.zeros((steps, rows), np.uint8)
        hbs = np.zeros((steps, rows), np.float32); Hr = np.zeros((steps, rows), np.float64)
        for t in range(steps):
            lg = si.logits_torch(t, "cfg2", rows, V, torch.bfloat16, "cuda")
            H, am, mid, hb, _ = g.step_logits(lg)
            Hs[t], ids[t], hbs[t] = H.cpu().numpy(), mid.cpu().numpy(), hb.cpu().numpy()
            if t < 3:
                ref = si.logits_np(t, "cfg2", rows, V)
                Hr[t], ar = oracle.entropy_rows(ref)
                assert (am.cpu().numpy() == ar).all()
                assert np.abs(Hs[t] - Hr[t]).max() < TOL_H
        for r in range(rows):
            hbr, idr = oracle.gate_trace(Hs[:, r], w, d_min, tau)     # gate on the GPU's own entropies
            assert (hbs[:, r] == hbr).all() and (ids[:, r] == idr).all()
        assert 0 < ids.mean() < 1
        g.close()


def test_multi_step_run_matches_single_steps():
    """ead_gate_run_logits (several steps per launch) against step-by-step calls and the oracle."""
    ead = _ead()
    rows, V, steps, w, tau, d_min = 64, 151936, 37, 5, 2.0, 3
    pool = [si.logits_torch(100 + i, "cfg2", rows, V, torch.bfloat16, "cuda") for i in range(5)]
    g1 = ead.Gate(rows, w, tau, d_min)
    H, am, mid, hb = g1.run_logits(pool, steps)
    g2 = ead.Gate(rows, w, tau, d_min)
    for t in range(steps):
        H2, am2, mid2, hb2, _ = g2.step_logits(pool[t % 5])
        assert (H[t] == H2).all() and (am[t] == am2).all() and (mid[t] == mid2).all() and (hb[t] == hb2).all()
    Hn, midn, hbn = H.cpu().numpy(), mid.cpu().numpy(), hb.cpu().numpy()
    for r in range(0, rows, 7):
        hbr, idr = oracle.gate_trace(Hn[:, r], w, d_min, tau)
        assert (hbn[:, r] == hbr).all() and (midn[:, r] == idr).all()
    ref = si.logits_np(102, "cfg2", rows, V)
    Hr, ar = oracle.entropy_rows(ref)
    assert np.abs(Hn[2] - Hr).max() < TOL_H and (am[2].cpu().numpy() == ar).all()
    assert 0 < midn.mean() < 1
    g1.close(); g2.close()
