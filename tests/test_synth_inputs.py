"""The seeded input generators: numpy and torch versions are bit-identical."""
import numpy as np
import torch

import synth_inputs as si


def test_numpy_and_torch_generators_agree():
    for bf16, dt in ((False, torch.float32), (True, torch.bfloat16)):
        a = si.normal_np(3, "x", (300, 257), 0.02, bf16=bf16)
        b = si.normal_torch(3, "x", (300, 257), 0.02, dt, "cpu", chunk=10000).float().numpy()
        assert (a == b).all()
    a = si.logits_np(0, "lg", 5, 1000)
    b = si.logits_torch(0, "lg", 5, 1000, torch.bfloat16, "cpu").float().numpy()
    assert (a == b).all()


def test_distribution_and_streams():
    z = si.normal_np(1, "z", (400000,), 1.0)
    assert abs(z.mean()) < 5e-3 and abs(z.std() - 1) < 5e-3
    assert not (si.normal_np(1, "z", (100,), 1.0) == si.normal_np(2, "z", (100,), 1.0)).all()
    assert not (si.normal_np(1, "z", (100,), 1.0) == si.normal_np(1, "y", (100,), 1.0)).all()
    t = si.tokens_np(0, "p", 20000, 512)
    assert t.min() >= 0 and t.max() < 512 and len(np.unique(t)) == 512
    s = si.row_scales(0, "lg", 1000)
    assert s.min() >= 0.5 and s.max() <= 8.0 and abs(s.mean() - 4.25) < 0.3
    L = si.prompt_lengths(0, 64, 128, 1024)
    assert L.min() >= 128 and L.max() <= 1024


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -3.3, 1e-30], np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert (si._round_bf16_np(x) == want).all()


def test_shape_byte_counts():
    # parameters streamed per decode step and KV bytes per cached position
    assert si.LLAMA_1B.n_params() == 1235814400 and si.LLAMA_8B.n_params() == 7504924672
    assert si.QWEN_05B.n_params() == 494005120 and si.QWEN_14B.n_params() == 13990466560
    assert si.TINY_S.n_params() == 590464 and si.TINY_L.n_params() == 4327680
    assert [s.kv_bytes_per_pos() for s in (si.LLAMA_1B, si.LLAMA_8B, si.QWEN_05B, si.QWEN_14B)] == \
        [32768, 131072, 12288, 196608]
