"""ctypes front end of the CPU oracle (oracle/ead_oracle.c) -- test infrastructure only.

Nothing in the GPU package imports this, and this imports nothing from it.
Arrays are numpy; weights are float32 dictionaries with the tensor names used by
`synth_inputs.weight_names` ("embed", "layers.<l>.wq", ..., "norm_final", "lm_head").
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build as _build

NATS, BITS = 0, 1
SMALL, LARGE = 0, 1

_FP = C.POINTER(C.c_float)
_FPP = C.POINTER(_FP)


class _CModel(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("embed", _FP),
                ("wq", _FPP), ("wk", _FPP), ("wv", _FPP), ("wo", _FPP),
                ("w_gate", _FPP), ("w_up", _FPP), ("w_down", _FPP),
                ("norm_attn", _FPP), ("norm_ffn", _FPP),
                ("norm_final", _FP), ("lm_head", _FP)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build())
        L.oracle_entropy.restype = C.c_double
        L.oracle_entropy.argtypes = [_FP, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
        L.oracle_entropy_direct.restype = C.c_double
        L.oracle_entropy_direct.argtypes = [_FP, C.c_int32, C.c_int32]
        L.oracle_window_mean.restype = C.c_float
        L.oracle_window_mean.argtypes = [_FP, C.c_int32, C.c_int32]
        L.oracle_gate_step.restype = None
        L.oracle_gate_step.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_float,
                                       C.c_float, C.c_int32]
        L.oracle_gate_trace.restype = None
        L.oracle_gate_trace.argtypes = [_FP, C.c_int32, C.c_int32, C.c_int32, C.c_float, _FP,
                                        C.POINTER(C.c_uint8)]
        L.oracle_param_ratio.restype = C.c_double
        L.oracle_param_ratio.argtypes = [C.c_double, C.c_double, C.c_double]
        L.oracle_rmsnorm.restype = None
        L.oracle_rmsnorm.argtypes = [_FP, _FP, C.c_int32, C.c_float, _FP]
        L.oracle_matvec.restype = None
        L.oracle_matvec.argtypes = [_FP, _FP, C.c_int32, C.c_int32, _FP, C.c_int32]
        L.oracle_rope.restype = None
        L.oracle_rope.argtypes = [_FP, C.c_int32, C.c_int32, C.c_int32, C.c_float]
        L.oracle_cache_new.restype = C.c_void_p
        L.oracle_cache_new.argtypes = [C.POINTER(_CModel), C.c_int32]
        L.oracle_cache_free.restype = None
        L.oracle_cache_free.argtypes = [C.c_void_p]
        L.oracle_cache_reset.restype = None
        L.oracle_cache_reset.argtypes = [C.c_void_p]
        L.oracle_cache_len.restype = C.c_int32
        L.oracle_cache_len.argtypes = [C.c_void_p]
        L.oracle_forward_cached.restype = C.c_int32
        L.oracle_forward_cached.argtypes = [C.POINTER(_CModel), C.c_void_p, C.c_int32, _FP]
        L.oracle_forward_dense.restype = C.c_int32
        L.oracle_forward_dense.argtypes = [C.POINTER(_CModel), C.POINTER(C.c_int32), C.c_int32, _FP]
        L.oracle_generate.restype = C.c_int32
        L.oracle_generate.argtypes = [C.POINTER(_CModel), C.POINTER(_CModel), C.POINTER(C.c_int32),
                                      C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_int32,
                                      C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                      C.POINTER(C.c_uint8), _FP, _FP]
        L.oracle_generate_sampled.restype = C.c_int32
        L.oracle_generate_sampled.argtypes = [C.POINTER(_CModel), C.POINTER(_CModel), C.POINTER(C.c_int32),
                                              C.c_int32, C.c_int32, C.c_int32, C.c_float, C.c_int32,
                                              C.c_int32, C.c_int32, C.c_float, C.c_uint64, C.c_int32,
                                              C.POINTER(C.c_int32), C.POINTER(C.c_uint8), _FP, _FP]
        L.oracle_philox4x32_10.restype = None
        L.oracle_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.oracle_uniform.restype = C.c_float
        L.oracle_uniform.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        L.oracle_gumbel.restype = C.c_float
        L.oracle_gumbel.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        L.oracle_sample.restype = C.c_int32
        L.oracle_sample.argtypes = [_FP, C.c_int32, C.c_float, C.c_uint64, C.c_int32, C.c_int32]
        L.oracle_num_threads.restype = C.c_int32
        L.oracle_num_threads.argtypes = []
        _lib = L
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _fp(a: np.ndarray):
    return a.ctypes.data_as(_FP)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


# ------------------------------------------------------------------ entropy / gate
def entropy(logits, unit: int = NATS):
    """(H, argmax) of one logits row: Eq. 1-2 of the paper."""
    l = _f32(logits).ravel()
    am = C.c_int32(-1)
    h = lib().oracle_entropy(_fp(l), l.size, unit, C.byref(am))
    return float(h), int(am.value)


def entropy_direct(logits, unit: int = NATS) -> float:
    l = _f32(logits).ravel()
    return float(lib().oracle_entropy_direct(_fp(l), l.size, unit))


def entropy_rows(logits, unit: int = NATS):
    """Row-wise (H[rows] float64, argmax[rows] int32)."""
    l = _f32(logits)
    H = np.empty(l.shape[0], dtype=np.float64)
    A = np.empty(l.shape[0], dtype=np.int32)
    for r in range(l.shape[0]):
        H[r], A[r] = entropy(l[r], unit)
    return H, A


def window_mean(W, w: int) -> float:
    """Mean of the last min(len(W), w) entries (Algorithm 1's rolling average)."""
    a = _f32(W).ravel()
    return float(lib().oracle_window_mean(_fp(a), a.size, w))


def gate_step(model: int, c: int, Hbar: float, tau: float, d_min: int):
    """One pass through Algorithm 1's switching block; returns (model, c)."""
    m, cc = C.c_int32(model), C.c_int32(c)
    lib().oracle_gate_step(C.byref(m), C.byref(cc), C.c_float(Hbar), C.c_float(tau), d_min)
    return int(m.value), int(cc.value)


def gate_trace(H, w: int, d_min: int, tau: float):
    """Run the gate on an entropy trace: (Hbar[n] float32, ids[n] uint8)."""
    a = _f32(H).ravel()
    hb = np.empty(a.size, dtype=np.float32)
    ids = np.empty(a.size, dtype=np.uint8)
    lib().oracle_gate_trace(_fp(a), a.size, w, d_min, C.c_float(tau), _fp(hb),
                            ids.ctypes.data_as(C.POINTER(C.c_uint8)))
    return hb, ids


def param_ratio(large_share: float, P_S: float, P_L: float) -> float:
    return float(lib().oracle_param_ratio(large_share, P_S, P_L))


# ------------------------------------------------------------------ model
class Model:
    """A decoder described by a shape object (n_layers, d_model, ...) and a weight dict."""

    def __init__(self, shape, weights: dict):
        self.shape = shape
        self._keep = []
        L = shape.n_layers

        def one(name):
            a = _f32(weights[name])
            self._keep.append(a)
            return _fp(a)

        def per_layer(name):
            arr = (_FP * L)(*[one(f"layers.{l}.{name}") for l in range(L)])
            self._keep.append(arr)
            return C.cast(arr, _FPP)

        self.c = _CModel(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads,
                         shape.head_dim, shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_theta,
                         one("embed"), per_layer("wq"), per_layer("wk"), per_layer("wv"),
                         per_layer("wo"), per_layer("w_gate"), per_layer("w_up"),
                         per_layer("w_down"), per_layer("norm_attn"), per_layer("norm_ffn"),
                         one("norm_final"), one("lm_head"))

    def forward_dense(self, tokens) -> np.ndarray:
        """Logits [T, vocab] of the whole sequence, explicit causal attention."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        out = np.empty((t.size, self.shape.vocab), dtype=np.float32)
        rc = lib().oracle_forward_dense(C.byref(self.c), t.ctypes.data_as(C.POINTER(C.c_int32)),
                                        t.size, _fp(out))
        if rc:
            raise ValueError("oracle_forward_dense: bad token")
        return out

    def forward_cached(self, tokens, max_seq=None) -> np.ndarray:
        """Same logits through the incremental KV-cached path."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        cache = lib().oracle_cache_new(C.byref(self.c), int(max_seq or t.size))
        out = np.empty((t.size, self.shape.vocab), dtype=np.float32)
        try:
            for i, tok in enumerate(t):
                if lib().oracle_forward_cached(C.byref(self.c), cache, int(tok), _fp(out[i])):
                    raise ValueError("oracle_forward_cached: bad token or cache full")
        finally:
            lib().oracle_cache_free(cache)
        return out


def philox4x32_10(counter, key):
    """One block of the counter-based generator behind the sampler (four 32-bit words)."""
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in counter])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = (C.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def uniform(seed: int, seq_index: int, token_index: int, i: int) -> float:
    return float(lib().oracle_uniform(seed, seq_index, token_index, i))


def gumbel(seed: int, seq_index: int, token_index: int, V: int) -> np.ndarray:
    """The noise g_i = -ln(-ln u_i) the sampler adds to l_i / T, for i < V (float32)."""
    L = lib()
    return np.array([L.oracle_gumbel(seed, seq_index, token_index, i) for i in range(V)], dtype=np.float32)


def sample(logits, temperature: float, seed: int, seq_index: int, token_index: int) -> int:
    """y ~ softmax(logits / temperature) by the Gumbel-max identity; temperature <= 0: arg max."""
    l = _f32(logits)
    return int(lib().oracle_sample(_fp(l), l.size, C.c_float(temperature), seed, seq_index, token_index))


def generate(small: Model, large: Model, prompt, max_new: int, w: int, tau: float,
             d_min: int = 10, unit: int = NATS, eos_id: int = -1, temperature: float = 0.0,
             seed: int = 0, seq_index: int = 0):
    """Algorithm 1 (greedy, or sampled at a temperature).  Returns dict(tokens, model_id, H, Hbar)."""
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    tok = np.zeros(max_new, dtype=np.int32)
    mid = np.zeros(max_new, dtype=np.uint8)
    H = np.zeros(max_new, dtype=np.float32)
    Hb = np.zeros(max_new, dtype=np.float32)
    n = lib().oracle_generate_sampled(C.byref(small.c), C.byref(large.c),
                                      p.ctypes.data_as(C.POINTER(C.c_int32)), p.size, max_new, w,
                                      C.c_float(tau), d_min, unit, eos_id,
                                      C.c_float(temperature), seed, seq_index,
                                      tok.ctypes.data_as(C.POINTER(C.c_int32)),
                                      mid.ctypes.data_as(C.POINTER(C.c_uint8)), _fp(H), _fp(Hb))
    if n < 0:
        raise ValueError(f"oracle_generate failed ({n})")
    return {"tokens": tok[:n], "model_id": mid[:n], "H": H[:n], "Hbar": Hb[:n]}


def replay(small: Model, large: Model, tokens, model_id, prompt_len: int, w: int, tau: float,
           d_min: int = 10, unit: int = NATS, temperature: float = 0.0, seed: int = 0, seq_index: int = 0):
    """Teacher-forced pass along a given trajectory.

    tokens: prompt followed by the generated tokens; model_id[i]: the model that
    produced generated token i.  Returns, for each generated position, the
    entropy and argmax of the forced model's logits, the window mean, and the
    model the gate would choose next when its current model is model_id[i] and
    its dwell counter follows the forced ids.
    """
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    model_id = np.asarray(model_id, dtype=np.uint8)
    n = tokens.size - prompt_len
    logits = [None, None]
    for m, mdl in ((SMALL, small), (LARGE, large)):
        if (model_id == m).any():
            logits[m] = mdl.forward_dense(tokens[:-1])
    H = np.zeros(n, dtype=np.float32)
    am = np.zeros(n, dtype=np.int32)
    choice = np.zeros(n, dtype=np.int32)
    Hbar = np.zeros(n, dtype=np.float32)
    nxt = np.zeros(n, dtype=np.uint8)
    c = 0
    for i in range(n):
        m = int(model_id[i])
        if i > 0 and model_id[i] != model_id[i - 1]:
            c = 0
        h, a = entropy(logits[m][prompt_len + i - 1], unit)
        H[i], am[i] = h, a
        choice[i] = sample(logits[m][prompt_len + i - 1], temperature, seed, seq_index, i) if temperature > 0 else a
        Hbar[i] = window_mean(H[: i + 1], w)
        nm, c = gate_step(m, c, float(Hbar[i]), tau, d_min)
        nxt[i] = nm
        if nm != m:
            c = 0
    return {"H": H, "argmax": am, "choice": choice, "Hbar": Hbar, "next_model": nxt, "logits": logits}
