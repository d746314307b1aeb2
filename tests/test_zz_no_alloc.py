"""The entry point that allocates nothing (ead_entropy_argmax_static) against ead_entropy_argmax."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu


def _call(fn, lg, H, am, unit=0):
    rc = fn(lg.data_ptr(), 1 if lg.dtype == torch.bfloat16 else 0, lg.shape[0], lg.shape[1], unit, H.data_ptr(),
            am.data_ptr(), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    return rc


def test_static_entry_point_matches_the_allocating_one():
    import paper_2502_06833_amd as ead
    L = ead.lib()
    # two calls in a row on one stream, the second with a smaller input: the array keeps the first
    # call's contents, and nothing of them may leak into the second result
    cases = [(64, 151936, torch.bfloat16), (5, 4096, torch.bfloat16), (3, 1000, torch.float32), (1, 8, torch.float32)]
    for i, (rows, V, dt) in enumerate(cases):
        print(f"static entropy case rows={rows} V={V} {dt}", flush=True)
        lg = si.logits_torch(7 + i, "static", rows, V, dt, "cuda")
        H0 = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda"); a0 = torch.full((rows,), -1, dtype=torch.int32, device="cuda")
        H1 = torch.full((rows,), -2.0, dtype=torch.float32, device="cuda"); a1 = torch.full((rows,), -2, dtype=torch.int32, device="cuda")
        assert _call(L.ead_entropy_argmax, lg, H0, a0) == 0
        assert _call(L.ead_entropy_argmax_static, lg, H1, a1) == 0
        torch.cuda.synchronize()
        # same kernels, same split of a row into chunks: bit-identical
        assert torch.equal(H0, H1) and torch.equal(a0, a1)
        Hr, ar = oracle.entropy_rows(si.logits_np(7 + i, "static", rows, V, bf16=(dt == torch.bfloat16)))
        assert np.abs(H1.cpu().numpy() - Hr).max() < 1e-2 and (a1.cpu().numpy() == ar).all()
    # bits
    lg = si.logits_torch(3, "static", 4, 2048, torch.bfloat16, "cuda")
    H0 = torch.empty(4, dtype=torch.float32, device="cuda"); a0 = torch.empty(4, dtype=torch.int32, device="cuda")
    H1 = torch.empty_like(H0); a1 = torch.empty_like(a0)
    assert _call(L.ead_entropy_argmax, lg, H0, a0, unit=1) == 0 and _call(L.ead_entropy_argmax_static, lg, H1, a1, unit=1) == 0
    torch.cuda.synchronize()
    assert torch.equal(H0, H1) and torch.equal(a0, a1)


def test_static_entry_point_rejects_what_does_not_fit():
    import paper_2502_06833_amd as ead
    L = ead.lib()
    rows, V = 4096, 32768            # 4096 rows x 2 chunks: fits; 4096 x 16 chunks (V = 262144) does not
    lg = torch.zeros((rows, V), dtype=torch.bfloat16, device="cuda")
    H = torch.empty(rows, dtype=torch.float32, device="cuda"); am = torch.empty(rows, dtype=torch.int32, device="cuda")
    assert _call(L.ead_entropy_argmax_static, lg, H, am) == 0
    torch.cuda.synchronize()
    assert abs(float(H[0]) - np.log(V)) < 1e-3 and int(am[0]) == 0
    del lg
    big = torch.zeros((2048, 262144), dtype=torch.bfloat16, device="cuda")   # 2048 rows x 16 chunks = 32768 partials
    Hb = torch.empty(2048, dtype=torch.float32, device="cuda"); ab = torch.empty(2048, dtype=torch.int32, device="cuda")
    rc = _call(L.ead_entropy_argmax_static, big, Hb, ab)
    assert rc == 1                                    # EAD_ERR_INVALID_ARG
    assert b"static scratch" in L.ead_last_error(None)
    assert _call(L.ead_entropy_argmax, big, Hb, ab) == 0          # the allocating entry point takes it
    torch.cuda.synchronize()
    assert abs(float(Hb[5]) - np.log(262144)) < 1e-3
