"""The C ABI without a GPU: the library loads, exports every symbol the header declares,
and refuses bad shapes before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2503_00540_amd import rekv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rekv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rekv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = rekv.lib()
    names = _declared()
    assert sorted(rekv.SYMBOLS) == names
    for n in names:
        assert getattr(L, n) is not None


def test_create_refuses_bad_shapes_before_any_device_work():
    L = rekv.lib()
    h = ctypes.c_void_p()
    bad = [
        (rekv.RekvShape(28, 5, 128, 196, 1, 0.0), 1, "multiple"),      # Hq % Hkv != 0
        (rekv.RekvShape(28, 4, 96, 196, 1, 0.0), 2, "head_dim"),       # bf16 D unsupported
        (rekv.RekvShape(4, 1, 66, 16, 0, 0.0), 2, "head_dim"),         # fp32 D % 4 != 0
        (rekv.RekvShape(4, 1, 64, 0, 0, 0.0), 1, "tokens_per_frame"),
        (rekv.RekvShape(4, 1, 64, 16, 7, 0.0), 1, "dtype"),
        (rekv.RekvShape(4, 1, 64, 16, 0, -1.0), 1, "softmax_scale"),
    ]
    for shape, code, word in bad:
        st = L.rekv_create(ctypes.byref(shape), ctypes.byref(h))
        assert st == code and h.value is None
        assert word in L.rekv_last_error(None).decode()
    assert L.rekv_create(None, ctypes.byref(h)) == 1
    L.rekv_destroy(None)            # accepted


def test_entry_points_refuse_a_null_context():
    L = rekv.lib()
    assert L.rekv_encode_chunk(None, None, None, None, 0, 1, 1, 0, None, None) == 1
    assert L.rekv_frame_keys(None, None, 1, None, None) == 1
    assert L.rekv_retrieve_topk(None, None, 0, 1, None, 1, 1, 1, None, None, None, None) == 1
    assert L.rekv_gather_kv(None, None, None, 0, 1, None, 1, 1, None, None, None) == 1
    assert L.rekv_qa_attention(None, None, None, None, 0, None, None, 1, 1, None, None) == 1
    assert L.rekv_offload_kv(None, None, None, None, None, 0, 1, None) == 1
    assert L.rekv_offload_wait(None) == 1


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(rekv, "_lib", None)
    monkeypatch.setattr(rekv, "LIB_PATH", "/nonexistent/librekv.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        rekv.lib()
