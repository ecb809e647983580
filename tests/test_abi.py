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
    assert L.rekv_qa_attention(None, None, None, None, 0, None, None, None, 1, 1, None, None) == 1
    assert L.rekv_decode_attention(None, None, None, None, 0, None, None, None, 1, 1, 1, 1, None, None) == 1
    assert L.rekv_decode_attention_noalloc(None, None, None, None, 0, None, None, None, 1, 1, 1, 1, None, None) == 1
    assert L.rekv_attention_indexed(None, None, None, None, 1, None, 1, 1, None, None, None, 1, 1, 1, 1, None, None) == 1
    assert L.rekv_gather_kv_layers(None, None, None, 1, 1, None, 1, 1, None, None, None) == 1
    assert L.rekv_gather_kv_rope(None, None, None, 0, 1, None, 1, 1, None, None, 10000.0, 0, 0, 0, 0, 0, None) == 1
    assert L.rekv_offload_kv(None, None, None, None, None, 0, 1, None) == 1
    assert L.rekv_offload_wait(None) == 1
    assert L.rekv_offload_join(None, None) == 1


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(rekv, "_lib", None)
    monkeypatch.setattr(rekv, "LIB_PATH", "/nonexistent/librekv.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        rekv.lib()


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/rekv.h compiles as C99 with every warning on, and a C program that names every
    declared entry point links against librekv.so (nothing is called: no GPU here)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    names = _declared()
    assert set(names) == set(rekv.SYMBOLS)
    src = tmp_path / "use_abi.c"
    body = "\n".join(f"    table[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text(f"""#include "rekv.h"
#include <stdio.h>
int main(void) {{
    void (*table[{len(names)}])(void);
{body}
    rekv_shape shape = {{28, 4, 128, 196, REKV_BF16, 0.0f}};
    printf("%d %d\\n", (int)sizeof(shape), table[0] != 0);
    return 0;
}}
""")
    lib_dir = os.path.dirname(rekv.LIB_PATH)
    exe = tmp_path / "use_abi"
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
           "-L", lib_dir, "-l:librekv.so", "-Wl,--unresolved-symbols=ignore-in-shared-libs", "-o", str(exe)]
    p = subprocess.run(cmd, capture_output=True, text=True)
    assert p.returncode == 0, p.stderr
