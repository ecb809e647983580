"""The whole path driven through the C ABI by a plain C99 program (tests/abi_chain.c: no Python, no
PyTorch, HIP runtime C API for memory, default stream), checked against the CPU oracle.  The
program's inputs come from a linear congruential generator that is repeated here.  Needs a real
MI355X."""
import os
import subprocess

import numpy as np
import pytest

from oracle import rekv_oracle as O
from paper_2503_00540_amd import build as B

pytestmark = pytest.mark.gpu

HQ, HKV, D, NF, FRAMES, WINDOW_FRAMES, NQ_TOKENS, TOPK = 4, 2, 64, 5, 12, 3, 6, 3      # as in abi_chain.c


def _lcg(n, state):
    """n draws of the program's generator, uniform in [-0.5, 0.5) with 24 bits, times 2."""
    out = np.empty(n, dtype=np.float32)
    for i in range(n):
        state = (state * 1664525 + 1013904223) & 0xFFFFFFFF
        out[i] = np.float32(state >> 8) * np.float32(1.0 / 16777216.0) - np.float32(0.5)
    return out * np.float32(2.0), state


def test_c_program_runs_the_path_and_matches_the_oracle(tmp_path):
    if not os.path.exists(B.C_PROGRAM):
        B.build_c_program(verbose=False)
    dump = tmp_path / "abi_chain.bin"
    p = subprocess.run([B.C_PROGRAM, str(dump)], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0, p.stdout + p.stderr
    tokens = FRAMES * NF
    state = 12345
    shapes = [(tokens, HQ, D), (tokens, HKV, D), (tokens, HKV, D), (NQ_TOKENS, HQ, D), (NQ_TOKENS, HKV, D), (NQ_TOKENS, HKV, D)]
    arrays = []
    for shp in shapes:                                   # the program draws in this order
        flat, state = _lcg(int(np.prod(shp)), state)
        arrays.append(flat.reshape(shp).astype(np.float64))
    q, k, v, qq, qk, qv = arrays
    raw = np.fromfile(dump, dtype=np.float32)
    d_prime = HKV * D
    sizes = [tokens * HQ * D, FRAMES * d_prime, FRAMES, TOPK, 1, NQ_TOKENS * HQ * D]
    assert raw.size == sum(sizes)
    parts = np.split(raw, np.cumsum(sizes)[:-1])
    out = parts[0].reshape(tokens, HQ, D).astype(np.float64)
    fk = parts[1].reshape(FRAMES, d_prime).astype(np.float64)
    scores = parts[2].astype(np.float64)
    idx, n_sel = parts[3].view(np.int32), parts[4].view(np.int32)
    qa = parts[5].reshape(NQ_TOKENS, HQ, D).astype(np.float64)

    assert np.abs(out - O.encode_chunks(q, k, v, 0, NF, FRAMES, WINDOW_FRAMES * NF)).max() < 1e-4
    fk_ref = O.frame_keys(k, FRAMES, NF)
    assert np.abs(fk - fk_ref).max() < 1e-5
    ref_idx, ref_scores = O.retrieve(fk_ref, qq, HKV, TOPK)
    assert np.abs(scores - ref_scores).max() < 1e-5
    srt = np.sort(ref_scores)[::-1]
    assert srt[TOPK - 1] - srt[TOPK] > 1e-3              # a clear cut for these inputs: the selection is unique
    np.testing.assert_array_equal(idx, ref_idx)
    assert int(n_sel[0]) == TOPK
    rk, rv = O.gather_kv(k, v, ref_idx, NF)
    assert np.abs(qa - O.qa_attention(qq, rk, rv, qk, qv)).max() < 1e-4
    assert p.stdout.startswith("selected frames")
