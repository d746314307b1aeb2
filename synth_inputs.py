"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle's callers.

This module holds no arithmetic of the decoding method: it only manufactures
weights, prompts and logits tensors from integer counters, so that the CPU oracle
and the HIP library can be fed bit-identical data without sharing any code.

Every value is a pure function of (seed, tensor name, element index):

* a 64-bit key is mixed with the SplitMix64 finaliser (Steele, Lea & Flood,
  "Fast splittable pseudorandom number generators", OOPSLA 2014);
* an approximately standard-normal value is the centred sum of eight 16-bit
  fields of two such hashes (Irwin-Hall, n=8), which is an exact integer, so
  the float32 result is identical under numpy, torch-CPU and torch-ROCm;
* bf16 tensors are the float32 values rounded to nearest-even.

The same generator runs under numpy (uint64) and under torch (int64 with
wrap-around and masked logical shifts), so large tensors can be produced
directly in device memory.
"""
from __future__ import annotations

import math
import zlib
from dataclasses import dataclass, field

import numpy as np

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1

# sum of eight uniform 16-bit integers: mean and standard deviation
_IH_N = 8
_IH_MEAN = _IH_N * 65535 // 2            # 262140, exact
_IH_STD = math.sqrt(_IH_N * (65536.0 ** 2 - 1.0) / 12.0)


def _to_i64(u: int) -> int:
    """Reinterpret an unsigned 64-bit constant as a signed one (for torch.int64)."""
    u &= _MASK64
    return u - (1 << 64) if u >= (1 << 63) else u


def _mix_int(x: int) -> int:
    """SplitMix64 finaliser on a python int."""
    x = (x + _GOLDEN) & _MASK64
    x = ((x ^ (x >> 30)) * _M1) & _MASK64
    x = ((x ^ (x >> 27)) * _M2) & _MASK64
    return x ^ (x >> 31)


def stream_key(seed: int, name: str) -> int:
    """64-bit base key of the tensor called `name` under `seed`."""
    tag = zlib.crc32(name.encode("utf-8")) & 0xFFFFFFFF
    return _mix_int(_mix_int(seed & _MASK64) ^ (tag * 0x100000001B3 & _MASK64))


# --------------------------------------------------------------------------- numpy
def _mix_np(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = x + np.uint64(_GOLDEN)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(_M1)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(_M2)
        return x ^ (x >> np.uint64(31))


def _hash_np(key: int, idx: np.ndarray, lane: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        k = np.uint64(key) + idx.astype(np.uint64) * np.uint64(2) + np.uint64(lane)
    return _mix_np(k)


def _ih_sum_np(key: int, idx: np.ndarray) -> np.ndarray:
    s = np.zeros(idx.shape, dtype=np.int64)
    for lane in (0, 1):
        h = _hash_np(key, idx, lane)
        for sh in (0, 16, 32, 48):
            s += ((h >> np.uint64(sh)) & np.uint64(0xFFFF)).astype(np.int64)
    return s - _IH_MEAN


def _round_bf16_np(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest-even bf16, returned as float32 (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def normal_np(seed: int, name: str, shape, std: float, bf16: bool = False,
              chunk: int = 1 << 22) -> np.ndarray:
    """float32 array ~ N(0, std^2) (bf16-rounded values if `bf16`)."""
    n = int(np.prod(shape))
    key = stream_key(seed, name)
    scale = np.float32(std / _IH_STD)
    out = np.empty(n, dtype=np.float32)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        out[a:b] = _ih_sum_np(key, np.arange(a, b, dtype=np.int64)).astype(np.float32) * scale
    if bf16:
        out = _round_bf16_np(out)
    return out.reshape(shape)


def tokens_np(seed: int, name: str, n: int, vocab: int) -> np.ndarray:
    """int32 tokens drawn uniformly from [0, vocab)."""
    h = _hash_np(stream_key(seed, name), np.arange(n, dtype=np.int64), 0)
    return ((h >> np.uint64(11)) % np.uint64(vocab)).astype(np.int32)


def uniform_np(seed: int, name: str, n: int) -> np.ndarray:
    """float64 uniforms in [0, 1)."""
    h = _hash_np(stream_key(seed, name), np.arange(n, dtype=np.int64), 0)
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def row_scales(seed: int, name: str, rows: int, lo: float = 0.5, hi: float = 8.0) -> np.ndarray:
    """Per-row standard deviations s_r ~ Uniform[lo, hi] as float32."""
    return (lo + (hi - lo) * uniform_np(seed, name + "/scale", rows)).astype(np.float32)


def logits_np(seed: int, name: str, rows: int, vocab: int, bf16: bool = True,
              lo: float = 0.5, hi: float = 8.0) -> np.ndarray:
    """[rows, vocab] logits, row r ~ N(0, s_r^2), s_r ~ U[lo, hi] (float32 values)."""
    z = normal_np(seed, name, (rows, vocab), 1.0)
    out = z * row_scales(seed, name, rows, lo, hi)[:, None]
    return _round_bf16_np(out) if bf16 else out


# --------------------------------------------------------------------------- torch
def _lsr_t(x, k: int):
    """Logical shift right of an int64 torch tensor."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def _mix_t(x):
    x = x + _to_i64(_GOLDEN)
    x = (x ^ _lsr_t(x, 30)) * _to_i64(_M1)
    x = (x ^ _lsr_t(x, 27)) * _to_i64(_M2)
    return x ^ _lsr_t(x, 31)


def _ih_sum_t(key: int, idx):
    import torch
    s = torch.zeros_like(idx)
    for lane in (0, 1):
        h = _mix_t(idx * 2 + _to_i64(key + lane))
        for sh in (0, 16, 32, 48):
            s += _lsr_t(h, sh) & 0xFFFF if sh else h & 0xFFFF
    return s - _IH_MEAN


def normal_torch(seed: int, name: str, shape, std: float, dtype, device,
                 chunk: int = 1 << 25):
    """Tensor ~ N(0, std^2) of `dtype` (float32 or bfloat16) generated on `device`.

    Bit-identical to `normal_np(seed, name, shape, std, bf16=(dtype is bfloat16))`.
    """
    import torch
    n = int(np.prod(shape))
    key = stream_key(seed, name)
    scale = float(np.float32(std / _IH_STD))
    out = torch.empty(n, dtype=dtype, device=device)
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        idx = torch.arange(a, b, dtype=torch.int64, device=device)
        z = _ih_sum_t(key, idx).to(torch.float32) * scale
        out[a:b] = z.to(dtype)
    return out.reshape(shape)


def logits_torch(seed: int, name: str, rows: int, vocab: int, dtype, device,
                 lo: float = 0.5, hi: float = 8.0):
    """Device version of `logits_np` (same values)."""
    import torch
    z = normal_torch(seed, name, (rows, vocab), 1.0, torch.float32, device)
    s = torch.from_numpy(row_scales(seed, name, rows, lo, hi)).to(device)
    return (z * s[:, None]).to(dtype)


# --------------------------------------------------------------------------- models
@dataclass(frozen=True)
class ModelShape:
    """Shape of one pre-norm decoder (RMSNorm + rotary + GQA + SwiGLU)."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    bf16: bool = True

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    def truncated(self, n_layers: int) -> "ModelShape":
        """Same widths, fewer layers (used for parity at full width)."""
        return ModelShape(f"{self.name}-L{n_layers}", n_layers, self.d_model, self.n_heads,
                          self.n_kv_heads, self.d_ffn, self.vocab, self.rms_eps,
                          self.rope_theta, self.bf16)

    def n_params(self) -> int:
        """Parameters streamed by one decode step (all layers, final norm, LM head)."""
        hd = self.head_dim
        attn = self.d_model * (self.n_heads + 2 * self.n_kv_heads) * hd + self.n_heads * hd * self.d_model
        ffn = 3 * self.d_model * self.d_ffn
        return self.n_layers * (attn + ffn + 2 * self.d_model) + self.d_model + self.vocab * self.d_model

    def kv_bytes_per_pos(self) -> int:
        return self.n_layers * 2 * self.n_kv_heads * self.head_dim * (2 if self.bf16 else 4)


TINY_S = ModelShape("tiny-s", 2, 128, 4, 4, 512, 512, 1e-5, 1e4, bf16=False)
TINY_L = ModelShape("tiny-l", 4, 256, 8, 8, 1024, 512, 1e-5, 1e4, bf16=False)
LLAMA_1B = ModelShape("llama-1b", 16, 2048, 32, 8, 8192, 128256, 1e-5, 5e5)
LLAMA_8B = ModelShape("llama-8b", 32, 4096, 32, 8, 14336, 128256, 1e-5, 5e5)
LLAMA_3B = ModelShape("llama-3b", 28, 3072, 24, 8, 8192, 128256, 1e-5, 5e5)
QWEN_05B = ModelShape("qwen-0.5b", 24, 896, 14, 2, 4864, 151936, 1e-6, 1e6)
QWEN_15B = ModelShape("qwen-1.5b", 28, 1536, 12, 2, 8960, 151936, 1e-6, 1e6)
QWEN_14B = ModelShape("qwen-14b", 48, 5120, 40, 8, 13824, 151936, 1e-6, 1e6)

PAIRS = {
    "tiny": (TINY_S, TINY_L),
    "llama": (LLAMA_1B, LLAMA_8B),
    "qwen": (QWEN_05B, QWEN_14B),
    # the paper's other pairs (size ratios 3x and about 9x)
    "llama_1b_3b": (LLAMA_1B, LLAMA_3B),
    "qwen_15b_14b": (QWEN_15B, QWEN_14B),
}


def weight_names(shape: ModelShape):
    """(tensor name, shape, kind) for every tensor of a model; kind is 'normal' or 'ones'."""
    d, hd = shape.d_model, shape.head_dim
    yield "embed", (shape.vocab, d), "normal"
    for l in range(shape.n_layers):
        p = f"layers.{l}."
        yield p + "wq", (shape.n_heads * hd, d), "normal"
        yield p + "wk", (shape.n_kv_heads * hd, d), "normal"
        yield p + "wv", (shape.n_kv_heads * hd, d), "normal"
        yield p + "wo", (d, shape.n_heads * hd), "normal"
        yield p + "w_gate", (shape.d_ffn, d), "normal"
        yield p + "w_up", (shape.d_ffn, d), "normal"
        yield p + "w_down", (d, shape.d_ffn), "normal"
        yield p + "norm_attn", (d,), "ones"
        yield p + "norm_ffn", (d,), "ones"
    yield "norm_final", (d,), "ones"
    yield "lm_head", (shape.vocab, d), "normal"


def model_weights_np(shape: ModelShape, seed: int, std: float = 0.02, gain_std: float = 0.0,
                     lm_std: float | None = None) -> dict:
    """All weights as float32 numpy arrays (bf16-rounded values for bf16 models).

    Matrices are N(0, std^2) (the LM head N(0, lm_std^2) if given); norm gains are 1, or
    1 + N(0, gain_std^2) when gain_std > 0 (float32, never rounded).
    """
    out = {}
    for name, shp, kind in weight_names(shape):
        if kind == "ones":
            out[name] = np.ones(shp, dtype=np.float32)
            if gain_std > 0:
                out[name] = out[name] + normal_np(seed, f"{shape.name}/{name}", shp, gain_std)
        elif name == "lm_head" and lm_std is not None:
            out[name] = normal_np(seed, f"{shape.name}/{name}", shp, lm_std, bf16=shape.bf16)
        else:
            out[name] = normal_np(seed, f"{shape.name}/{name}", shp, std, bf16=shape.bf16)
    return out


def model_weights_torch(shape: ModelShape, seed: int, device, std: float = 0.02, gain_std: float = 0.0,
                        lm_std: float | None = None) -> dict:
    """All weights on `device`: matrices in the model dtype, gains in float32 (same values as model_weights_np)."""
    import torch
    dt = torch.bfloat16 if shape.bf16 else torch.float32
    out = {}
    for name, shp, kind in weight_names(shape):
        if kind == "ones":
            out[name] = torch.ones(shp, dtype=torch.float32, device=device)
            if gain_std > 0:
                out[name] = out[name] + normal_torch(seed, f"{shape.name}/{name}", shp, gain_std, torch.float32, device)
        elif name == "lm_head" and lm_std is not None:
            out[name] = normal_torch(seed, f"{shape.name}/{name}", shp, lm_std, dt, device)
        else:
            out[name] = normal_torch(seed, f"{shape.name}/{name}", shp, std, dt, device)
    return out


def prompt_np(seed: int, name: str, n: int, vocab: int) -> np.ndarray:
    return tokens_np(seed, "prompt/" + name, n, vocab)


def prompt_lengths(seed: int, batch: int, lo: int, hi: int) -> np.ndarray:
    """Per-row prompt lengths drawn uniformly from {lo..hi}."""
    u = uniform_np(seed, "prompt_len", batch)
    return (lo + np.floor(u * (hi - lo + 1))).astype(np.int32).clip(lo, hi)
