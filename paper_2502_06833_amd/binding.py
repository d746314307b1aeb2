"""ctypes binding of include/ead.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("EAD_LIBRARY") or os.path.join(HERE, "libead.so")

NATS, BITS = 0, 1
SMALL, LARGE = 0, 1
F32, BF16 = 0, 1

_STATUS = {0: "OK", 1: "INVALID_ARG", 2: "SHAPE", 3: "VOCAB_MISMATCH", 4: "OOM", 5: "SEQ_OVERFLOW",
           6: "NONFINITE", 7: "DEVICE", 8: "NO_DEVICE", 9: "STATE"}


class EadError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"EAD_ERR_{_STATUS.get(status, status)}: {msg}")
        self.status = status


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("dtype", C.c_int32), ("embed", C.c_void_p),
                ("wq", C.POINTER(C.c_void_p)), ("wk", C.POINTER(C.c_void_p)),
                ("wv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("w_gate", C.POINTER(C.c_void_p)), ("w_up", C.POINTER(C.c_void_p)),
                ("w_down", C.POINTER(C.c_void_p)), ("norm_attn", C.POINTER(C.c_void_p)),
                ("norm_ffn", C.POINTER(C.c_void_p)), ("norm_final", C.c_void_p),
                ("lm_head", C.c_void_p)]


class Params(C.Structure):
    _fields_ = [("window", C.c_int32), ("tau", C.c_float), ("d_min", C.c_int32), ("unit", C.c_int32),
                ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("eos_id", C.c_int32),
                ("hip_stream", C.c_void_p)]


class Stats(C.Structure):
    _fields_ = [("tokens_small", C.c_int64), ("tokens_large", C.c_int64), ("switches", C.c_int64),
                ("steps_small", C.c_int64), ("steps_large", C.c_int64),
                ("catchup_rows_small", C.c_int64), ("catchup_rows_large", C.c_int64),
                ("host_syncs", C.c_int64), ("algorithmic_bytes", C.c_double),
                ("large_share", C.c_double), ("param_ratio", C.c_double)]


class KernelProfile(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double), ("bytes", C.c_double)]


_I32P, _U8P, _F32P = C.POINTER(C.c_int32), C.POINTER(C.c_uint8), C.POINTER(C.c_float)

# name -> (restype, argtypes); also the list of symbols include/ead.h declares
_SIGNATURES = {
    "ead_version": (C.c_int32, []),
    "ead_create": (C.c_int, [C.POINTER(ModelDesc), C.POINTER(ModelDesc), C.POINTER(Params), C.POINTER(C.c_void_p)]),
    "ead_destroy": (None, [C.c_void_p]),
    "ead_last_error": (C.c_char_p, [C.c_void_p]),
    "ead_set_gate": (C.c_int, [C.c_void_p, C.c_int32, C.c_float, C.c_int32, C.c_int32, C.c_int32]),
    "ead_generate": (C.c_int, [C.c_void_p, _I32P, _I32P, C.c_int32, C.c_int32, _I32P, _U8P, _F32P, _F32P, _I32P]),
    "ead_begin": (C.c_int, [C.c_void_p, _I32P, _I32P, C.c_int32, C.c_int32]),
    "ead_rewind": (C.c_int, [C.c_void_p, C.c_int32]),
    "ead_decode": (C.c_int, [C.c_void_p, C.c_int32]),
    "ead_decode_tokens": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32]),
    "ead_fetch": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _U8P, _F32P, _F32P, _I32P]),
    "ead_score": (C.c_int, [C.c_void_p, C.c_int32, _I32P, C.c_int32, _F32P, _F32P, _I32P]),
    "ead_replay": (C.c_int, [C.c_void_p, _I32P, _I32P, C.c_int32, C.c_int32, _I32P, _U8P, _I32P, _F32P, _F32P, _U8P]),
    "ead_entropy_argmax": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ead_entropy_argmax_static": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ead_gate_create": (C.c_int, [C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]),
    "ead_gate_step": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ead_gate_step_logits": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ead_gate_run_logits": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "ead_gate_reset": (C.c_int, [C.c_void_p]),
    "ead_gate_destroy": (None, [C.c_void_p]),
    "ead_get_stats": (C.c_int, [C.c_void_p, C.POINTER(Stats)]),
    "ead_reset_stats": (C.c_int, [C.c_void_p]),
    "ead_force_model": (C.c_int, [C.c_void_p, C.c_int32]),
    "ead_set_fused": (C.c_int, [C.c_void_p, C.c_int32]),
    "ead_set_schedule": (C.c_int, [C.c_void_p, C.c_int32, C.c_float, C.c_float]),
    "ead_set_sampling": (C.c_int, [C.c_void_p, C.c_float, C.c_uint64]),
    "ead_profile_enable": (C.c_int, [C.c_void_p, C.c_int32]),
    "ead_profile_select": (C.c_int, [C.c_void_p, C.c_char_p]),
    "ead_profile_read": (C.c_int, [C.c_void_p, C.POINTER(KernelProfile), C.c_int32, _I32P]),
}


def exported_symbols():
    return sorted(_SIGNATURES)


_lib = None


def lib():
    """Load libead.so (built by paper_2502_06833_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2502_06833_amd.build` "
                              "(there is no fallback path)")
        # PyTorch ships its own HIP runtime; load it first so that the library binds to the
        # same runtime (and the same device context) as the tensors it is handed
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _ptr(a: np.ndarray, ty):
    return a.ctypes.data_as(ty)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _desc(shape, weights) -> tuple:
    """ModelDesc from a shape object and a dict of CUDA tensors (names as in synth_inputs)."""
    L = shape.n_layers
    keep = []

    def dev(name):
        t = weights[name]
        assert t.is_cuda and t.is_contiguous(), name
        keep.append(t)
        return t.data_ptr()

    def per_layer(name):
        arr = (C.c_void_p * L)(*[dev(f"layers.{l}.{name}") for l in range(L)])
        keep.append(arr)
        return C.cast(arr, C.POINTER(C.c_void_p))

    d = ModelDesc(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                  shape.d_ffn, shape.vocab, shape.rms_eps, shape.rope_theta,
                  _dtype_code(weights["lm_head"]), dev("embed"),
                  per_layer("wq"), per_layer("wk"), per_layer("wv"), per_layer("wo"),
                  per_layer("w_gate"), per_layer("w_up"), per_layer("w_down"),
                  per_layer("norm_attn"), per_layer("norm_ffn"), dev("norm_final"), dev("lm_head"))
    return d, keep


class EAD:
    """A model pair plus Algorithm 1's parameters (wraps an ead_handle)."""

    def __init__(self, small_shape, small_weights, large_shape, large_weights, window=5, tau=0.0,
                 d_min=10, unit=NATS, max_batch=1, max_seq=256, eos_id=-1):
        import torch
        L = lib()
        ds, keep_s = _desc(small_shape, small_weights)
        dl, keep_l = _desc(large_shape, large_weights)
        p = Params(window, tau, d_min, unit, max_batch, max_seq, eos_id, _stream_ptr())
        h = C.c_void_p()
        rc = L.ead_create(C.byref(ds), C.byref(dl), C.byref(p), C.byref(h))
        if rc:
            raise EadError(rc, (L.ead_last_error(None) or b"").decode())
        torch.cuda.synchronize()
        del keep_s, keep_l                     # weights were copied; the caller may free them
        self._h = h
        self.vocab = small_shape.vocab
        self.max_seq, self.max_batch = max_seq, max_batch

    def _check(self, rc):
        if rc:
            raise EadError(rc, (lib().ead_last_error(self._h) or b"").decode())

    def close(self):
        if getattr(self, "_h", None):
            lib().ead_destroy(self._h)
            self._h = None

    __del__ = close

    def set_gate(self, window, tau, d_min=10, unit=NATS, eos_id=-1):
        self._check(lib().ead_set_gate(self._h, window, tau, d_min, unit, eos_id))

    def force_model(self, which: int):
        self._check(lib().ead_force_model(self._h, which))

    @staticmethod
    def _prompts(prompts):
        if isinstance(prompts, np.ndarray) and prompts.ndim == 1:
            prompts = [prompts]
        lens = np.array([len(p) for p in prompts], dtype=np.int32)
        flat = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]))
        return flat, lens

    def generate(self, prompts, max_new: int):
        flat, lens = self._prompts(prompts)
        B = len(lens)
        tok = np.zeros((B, max_new), np.int32); mid = np.zeros((B, max_new), np.uint8)
        H = np.zeros((B, max_new), np.float32); Hb = np.zeros((B, max_new), np.float32)
        n = np.zeros(B, np.int32)
        self._check(lib().ead_generate(self._h, _ptr(flat, _I32P), _ptr(lens, _I32P), B, max_new,
                                       _ptr(tok, _I32P), _ptr(mid, _U8P), _ptr(H, _F32P), _ptr(Hb, _F32P),
                                       _ptr(n, _I32P)))
        return {"tokens": tok, "model_id": mid, "H": H, "Hbar": Hb, "lens": n}

    def begin(self, prompts, max_new: int):
        flat, lens = self._prompts(prompts)
        self._B, self._max_new = len(lens), max_new
        self._check(lib().ead_begin(self._h, _ptr(flat, _I32P), _ptr(lens, _I32P), len(lens), max_new))

    def rewind(self, max_new: int):
        self._max_new = max_new
        self._check(lib().ead_rewind(self._h, max_new))

    def decode(self, n_steps: int):
        self._check(lib().ead_decode(self._h, n_steps))

    def decode_tokens(self, n_tokens: int, max_lead: int = 64):
        self._check(lib().ead_decode_tokens(self._h, n_tokens, max_lead))

    def fetch(self):
        B, max_new = self._B, self._max_new
        tok = np.zeros((B, max_new), np.int32); mid = np.zeros((B, max_new), np.uint8)
        H = np.zeros((B, max_new), np.float32); Hb = np.zeros((B, max_new), np.float32)
        n = np.zeros(B, np.int32)
        self._check(lib().ead_fetch(self._h, max_new, _ptr(tok, _I32P), _ptr(mid, _U8P), _ptr(H, _F32P),
                                    _ptr(Hb, _F32P), _ptr(n, _I32P)))
        return {"tokens": tok, "model_id": mid, "H": H, "Hbar": Hb, "lens": n}

    def score(self, which: int, tokens, want_logits=True):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        lg = np.zeros((t.size, self.vocab), np.float32) if want_logits else None
        H = np.zeros(t.size, np.float32); am = np.zeros(t.size, np.int32)
        self._check(lib().ead_score(self._h, which, _ptr(t, _I32P), t.size,
                                    _ptr(lg, _F32P) if want_logits else None, _ptr(H, _F32P), _ptr(am, _I32P)))
        return {"logits": lg, "H": H, "argmax": am}

    def replay(self, prompts, forced_tokens, forced_model_id):
        flat, lens = self._prompts(prompts)
        ft = np.ascontiguousarray(forced_tokens, dtype=np.int32).reshape(len(lens), -1)
        fm = np.ascontiguousarray(forced_model_id, dtype=np.uint8).reshape(len(lens), -1)
        B, n = ft.shape
        am = np.zeros((B, n), np.int32); H = np.zeros((B, n), np.float32); Hb = np.zeros((B, n), np.float32)
        dec = np.zeros((B, n), np.uint8)
        self._check(lib().ead_replay(self._h, _ptr(flat, _I32P), _ptr(lens, _I32P), B, n, _ptr(ft, _I32P),
                                     _ptr(fm, _U8P), _ptr(am, _I32P), _ptr(H, _F32P), _ptr(Hb, _F32P),
                                     _ptr(dec, _U8P)))
        # "choice": the token the library itself would have emitted (arg max, or the sampled one)
        return {"argmax": am, "choice": am, "H": H, "Hbar": Hb, "next_model": dec}

    def stats(self) -> dict:
        s = Stats()
        self._check(lib().ead_get_stats(self._h, C.byref(s)))
        return {k: getattr(s, k) for k, _ in Stats._fields_}

    def set_schedule(self, grouped: bool, start_fraction: float = 0.5, stop_fraction: float = 0.25):
        self._check(lib().ead_set_schedule(self._h, 1 if grouped else 0, start_fraction, stop_fraction))

    def set_sampling(self, temperature: float, seed: int = 0):
        self._check(lib().ead_set_sampling(self._h, temperature, seed))

    def set_fused(self, on):
        """False/0: per-layer kernels; True/1: one persistent kernel per single-row step (the streamed
        variant where the model has one); 2: the register-buffered persistent kernel even then."""
        self._check(lib().ead_set_fused(self._h, 2 if on == 2 and on is not True else (1 if on else 0)))

    def profile(self, on: bool):
        self._check(lib().ead_profile_enable(self._h, 1 if on else 0))

    def profile_select(self, name=None):
        self._check(lib().ead_profile_select(self._h, name.encode() if name else None))

    def profile_read(self) -> list:
        arr = (KernelProfile * 64)()
        n = C.c_int32(0)
        self._check(lib().ead_profile_read(self._h, arr, 64, C.byref(n)))
        return [{"name": arr[i].name.decode(), "launches": arr[i].launches, "total_ms": arr[i].total_ms,
                 "bytes": arr[i].bytes} for i in range(n.value)]

    def reset_stats(self):
        self._check(lib().ead_reset_stats(self._h))


def entropy_argmax(logits, unit=NATS, out=None, static=False):
    """Row-wise (H, argmax) of a CUDA logits tensor [rows, vocab] (bf16 or fp32).
    out: (H, argmax) tensors to write into; static: the entry point that allocates nothing."""
    import torch
    assert logits.is_cuda and logits.is_contiguous() and logits.dim() == 2
    rows, V = logits.shape
    if out is None:
        out = (torch.empty(rows, dtype=torch.float32, device=logits.device),
               torch.empty(rows, dtype=torch.int32, device=logits.device))
    H, am = out
    fn = lib().ead_entropy_argmax_static if static else lib().ead_entropy_argmax
    rc = fn(logits.data_ptr(), _dtype_code(logits), rows, V, unit, H.data_ptr(), am.data_ptr(), _stream_ptr())
    if rc:
        raise EadError(rc, (lib().ead_last_error(None) or b"").decode())
    return H, am


class Gate:
    """Rolling window + switch rule for `rows` sequences, state on the GPU (wraps ead_gate)."""

    def __init__(self, rows, window, tau, d_min):
        import torch
        g = C.c_void_p()
        rc = lib().ead_gate_create(rows, window, tau, d_min, _stream_ptr(), C.byref(g))
        if rc:
            raise EadError(rc, (lib().ead_last_error(None) or b"").decode())
        self._g, self.rows = g, rows
        dev = "cuda"
        self.model_id = torch.empty(rows, dtype=torch.uint8, device=dev)
        self.window_mean = torch.empty(rows, dtype=torch.float32, device=dev)
        self.next_model = torch.empty(rows, dtype=torch.uint8, device=dev)
        self.H = torch.empty(rows, dtype=torch.float32, device=dev)
        self.argmax = torch.empty(rows, dtype=torch.int32, device=dev)

    def step(self, H):
        rc = lib().ead_gate_step(self._g, H.data_ptr(), self.model_id.data_ptr(), self.window_mean.data_ptr(),
                                 self.next_model.data_ptr())
        if rc:
            raise EadError(rc, "ead_gate_step")
        return self.model_id, self.window_mean, self.next_model

    def step_logits(self, logits, unit=NATS):
        rc = lib().ead_gate_step_logits(self._g, logits.data_ptr(), _dtype_code(logits), logits.shape[1], unit,
                                        self.H.data_ptr(), self.argmax.data_ptr(), self.model_id.data_ptr(),
                                        self.window_mean.data_ptr(), self.next_model.data_ptr())
        if rc:
            raise EadError(rc, (lib().ead_last_error(None) or b"").decode())
        return self.H, self.argmax, self.model_id, self.window_mean, self.next_model

    def run_logits(self, tensors, n_steps, unit=NATS, want_outputs=True):
        """n_steps steps; step s reads tensors[s % len(tensors)].  Returns (H, argmax, model_id, window_mean),
        each [n_steps, rows] on the GPU (None when want_outputs is False)."""
        import torch
        arr = (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
        outs = (None, None, None, None)
        if want_outputs:
            outs = (torch.empty((n_steps, self.rows), dtype=torch.float32, device="cuda"),
                    torch.empty((n_steps, self.rows), dtype=torch.int32, device="cuda"),
                    torch.empty((n_steps, self.rows), dtype=torch.uint8, device="cuda"),
                    torch.empty((n_steps, self.rows), dtype=torch.float32, device="cuda"))
        ptr = [o.data_ptr() if o is not None else None for o in outs]
        rc = lib().ead_gate_run_logits(self._g, arr, len(tensors), n_steps, _dtype_code(tensors[0]), tensors[0].shape[1],
                                       unit, *ptr)
        if rc:
            raise EadError(rc, (lib().ead_last_error(None) or b"").decode())
        return outs

    def reset(self):
        lib().ead_gate_reset(self._g)

    def close(self):
        if getattr(self, "_g", None):
            lib().ead_gate_destroy(self._g)
            self._g = None

    __del__ = close
