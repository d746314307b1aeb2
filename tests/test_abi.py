"""The C-ABI library loads and exports every symbol include/ead.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "ead.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ead_[a-z_]+)\s*\(", src)))


def test_header_symbols_are_exported_and_bound():
    import paper_2502_06833_amd as ead
    L = ead.lib()
    names = _declared()
    assert len(names) >= 18
    for n in names:
        assert hasattr(L, n), f"{n} declared in ead.h but not exported"
    assert set(names) == set(ead.exported_symbols())
    assert L.ead_version() >= 100


def test_argument_errors_without_touching_the_gpu():
    import paper_2502_06833_amd as ead
    from paper_2502_06833_amd.binding import ModelDesc, Params
    L = ead.lib()
    h = ctypes.c_void_p()
    p = Params(5, 1.0, 10, 0, 1, 64, -1, None)
    assert L.ead_create(None, None, ctypes.byref(p), ctypes.byref(h)) == 1          # INVALID_ARG
    assert b"null" in L.ead_last_error(None)
    d = ModelDesc()
    assert L.ead_create(ctypes.byref(d), ctypes.byref(d), ctypes.byref(p), ctypes.byref(h)) == 1
    assert L.ead_create(ctypes.byref(d), ctypes.byref(d), None, ctypes.byref(h)) == 1
    assert L.ead_decode(None, 1) == 1 and L.ead_begin(None, None, None, 1, 1) == 1
    assert L.ead_gate_create(0, 5, 1.0, 10, None, ctypes.byref(h)) == 1
    assert L.ead_gate_create(4, 0, 1.0, 10, None, ctypes.byref(h)) == 1
    assert L.ead_gate_create(4, 5, float("nan"), 10, None, ctypes.byref(h)) == 1
    assert L.ead_entropy_argmax(None, 1, 4, 512, 0, None, None, None) == 1


def test_shape_and_vocab_checks():
    import paper_2502_06833_amd as ead
    from paper_2502_06833_amd.binding import ModelDesc, Params
    L = ead.lib()
    h = ctypes.c_void_p()
    p = Params(5, 1.0, 10, 0, 1, 64, -1, None)
    fake = ctypes.c_void_p(0x1000)
    arr = (ctypes.c_void_p * 1)(0x1000)
    pp = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))

    def desc(**kw):
        base = dict(n_layers=1, d_model=64, n_heads=2, n_kv_heads=2, head_dim=32, d_ffn=64, vocab=512)
        base.update(kw)
        return ModelDesc(base["n_layers"], base["d_model"], base["n_heads"], base["n_kv_heads"], base["head_dim"],
                         base["d_ffn"], base["vocab"], 1e-5, 1e4, 0, fake, pp, pp, pp, pp, pp, pp, pp, pp, pp, fake, fake)

    bad = desc(d_model=48)
    assert L.ead_create(ctypes.byref(bad), ctypes.byref(bad), ctypes.byref(p), ctypes.byref(h)) == 2   # SHAPE
    bad = desc(head_dim=48)
    assert L.ead_create(ctypes.byref(bad), ctypes.byref(bad), ctypes.byref(p), ctypes.byref(h)) == 2
    bad = desc(n_heads=3, n_kv_heads=2)
    assert L.ead_create(ctypes.byref(bad), ctypes.byref(bad), ctypes.byref(p), ctypes.byref(h)) == 2
    a, b = desc(), desc(vocab=1024)
    assert L.ead_create(ctypes.byref(a), ctypes.byref(b), ctypes.byref(p), ctypes.byref(h)) == 3       # VOCAB_MISMATCH
    bad_p = Params(0, 1.0, 10, 0, 1, 64, -1, None)
    assert L.ead_create(ctypes.byref(a), ctypes.byref(a), ctypes.byref(bad_p), ctypes.byref(h)) == 1
    assert not h.value
