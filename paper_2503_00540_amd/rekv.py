"""Thin ctypes binding over librekv.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (`include/rekv.h`).  PyTorch
appears here only as the owner of device / pinned memory and of the current stream.  If the
library has not been built the binding raises; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int32, c_int64, c_void_p

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "librekv.so")

REKV_F32, REKV_BF16 = 0, 1
_STATUS = {0: "REKV_OK", 1: "REKV_ERR_INVALID_ARG", 2: "REKV_ERR_UNSUPPORTED",
           3: "REKV_ERR_NOMEM", 4: "REKV_ERR_HIP"}
_DTYPES = {"f32": (REKV_F32, torch.float32), "bf16": (REKV_BF16, torch.bfloat16)}

# Every entry point include/rekv.h declares.
SYMBOLS = ("rekv_create", "rekv_destroy", "rekv_last_error", "rekv_encode_chunk",
           "rekv_frame_keys", "rekv_retrieve_topk", "rekv_gather_kv", "rekv_qa_attention",
           "rekv_decode_attention", "rekv_decode_attention_noalloc", "rekv_block_keys", "rekv_expand_blocks", "rekv_retrieve_external", "rekv_attention_indexed", "rekv_gather_kv_rope", "rekv_gather_kv_layers", "rekv_attention_indexed_rope",
           "rekv_offload_kv", "rekv_offload_wait", "rekv_offload_join", "rekv_probe_copy", "rekv_probe_mfma")


class RekvShape(ctypes.Structure):
    _fields_ = [("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32),
                ("tokens_per_frame", c_int32), ("dtype", c_int32), ("softmax_scale", c_float)]


class RekvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Loads librekv.so; raises if it has not been built (python -m paper_2503_00540_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_00540_amd.build`; "
                           "there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    L.rekv_create.argtypes = [POINTER(RekvShape), POINTER(c_void_p)]
    L.rekv_create.restype = c_int32
    L.rekv_destroy.argtypes = [c_void_p]
    L.rekv_destroy.restype = None
    L.rekv_last_error.argtypes = [c_void_p]
    L.rekv_last_error.restype = c_char_p
    L.rekv_encode_chunk.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32,
                                    c_int32, c_void_p, c_void_p]
    L.rekv_frame_keys.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
    L.rekv_retrieve_topk.argtypes = [c_void_p, c_void_p, c_int64, c_int32, c_void_p, c_int32, c_int32,
                                     c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    L.rekv_gather_kv.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_int32,
                                 c_int32, c_void_p, c_void_p, c_void_p]
    L.rekv_qa_attention.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p,
                                    c_int32, c_int32, c_void_p, c_void_p]
    L.rekv_retrieve_external.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_int32, c_float,
                                         c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    L.rekv_block_keys.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p]
    L.rekv_expand_blocks.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_int32, c_int32, c_void_p,
                                     c_void_p, c_void_p]
    L.rekv_decode_attention.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p,
                                        c_int64, c_int32, c_int32, c_int32, c_void_p, c_void_p]
    L.rekv_decode_attention_noalloc.argtypes = L.rekv_decode_attention.argtypes
    L.rekv_attention_indexed.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_int64,
                                         c_int32, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_int32, c_int32,
                                         c_void_p, c_void_p]
    L.rekv_gather_kv_layers.argtypes = [c_void_p, POINTER(c_void_p), POINTER(c_void_p), c_int32, c_int32, c_void_p,
                                        c_int32, c_int32, c_void_p, c_void_p, c_void_p]
    L.rekv_gather_kv_rope.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_int32, c_int32, c_void_p,
                                      c_void_p, ctypes.c_double, c_int32, c_int32, c_int64, c_int32, c_int64, c_void_p]
    L.rekv_attention_indexed_rope.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_void_p, c_int64, c_int32,
                                              c_void_p, c_void_p, ctypes.c_double, c_int32, c_int32, c_int64, c_int32, c_int64,
                                              c_void_p, c_void_p, c_int64, c_int32, c_int32, c_int32, c_void_p, c_void_p]
    L.rekv_offload_kv.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_int32,
                                  c_void_p]
    L.rekv_offload_wait.argtypes = [c_void_p]
    L.rekv_offload_join.argtypes = [c_void_p, c_void_p]
    L.rekv_probe_copy.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_void_p]
    L.rekv_probe_mfma.argtypes = [c_void_p, c_void_p, c_int32, c_int32, POINTER(ctypes.c_double), c_void_p]
    for name in SYMBOLS[3:]:
        getattr(L, name).restype = c_int32
    _lib = L
    return L


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Rekv:
    """One layer shape's context.  Methods mirror the C entry points one to one."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, tokens_per_frame: int,
                 dtype: str = "bf16", softmax_scale: float = 0.0):
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.tokens_per_frame = tokens_per_frame
        self.dtype_name = dtype
        code, self.torch_dtype = _DTYPES[dtype]
        self._lib = lib()
        shape = RekvShape(n_q_heads, n_kv_heads, head_dim, tokens_per_frame, code, softmax_scale)
        h = c_void_p()
        st = self._lib.rekv_create(byref(shape), byref(h))
        if st != 0:
            raise RekvError(st, self._lib.rekv_last_error(None).decode())
        self._h = h

    @classmethod
    def for_workload(cls, w, softmax_scale: float = 0.0) -> "Rekv":
        return cls(w.n_q_heads, w.n_kv_heads, w.head_dim, w.tokens_per_frame, w.dtype, softmax_scale)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.rekv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- marshalling helpers ------------------------------------------------------------
    def _check(self, st: int):
        if st != 0:
            raise RekvError(st, self._lib.rekv_last_error(self._h).decode())

    def _dev(self, t: torch.Tensor, dtype=None, last=None, name="tensor") -> int:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous CUDA tensor")
        if t.dtype != (dtype or self.torch_dtype):
            raise ValueError(f"{name} has dtype {t.dtype}, expected {dtype or self.torch_dtype}")
        if last is not None and tuple(t.shape[-len(last):]) != tuple(last):
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected trailing {tuple(last)}")
        return t.data_ptr()

    def _pinned(self, t: torch.Tensor, last, name) -> int:
        if t.is_cuda or not t.is_pinned() or not t.is_contiguous() or t.dtype != self.torch_dtype:
            raise ValueError(f"{name} must be a contiguous pinned host tensor of dtype {self.torch_dtype}")
        if tuple(t.shape[-len(last):]) != tuple(last):
            raise ValueError(f"{name} has shape {tuple(t.shape)}, expected trailing {tuple(last)}")
        return t.data_ptr()

    def _n_sel(self, n_sel, nq: int):
        if n_sel is None:
            return None
        if not n_sel.is_cuda or n_sel.dtype != torch.int32 or not n_sel.is_contiguous() or n_sel.numel() != nq:
            raise ValueError("n_sel must be a contiguous device int32 tensor with one entry per question")
        return n_sel.data_ptr()

    # -- the entry points -----------------------------------------------------------------
    def encode_chunk(self, q, k_cache, v_cache, first_token: int, l_x: int, n_chunks: int, l_l: int,
                     out=None):
        qh, kh = (self.n_q_heads, self.head_dim), (self.n_kv_heads, self.head_dim)
        if q.shape[0] != n_chunks * l_x:
            raise ValueError("q must hold n_chunks * l_x tokens")
        if k_cache.shape[0] < first_token + n_chunks * l_x or v_cache.shape[0] != k_cache.shape[0]:
            raise ValueError("k_cache / v_cache are shorter than first_token + n_chunks * l_x")
        out = torch.empty_like(q) if out is None else out
        if out.shape != q.shape:
            raise ValueError("out must have the shape of q")
        self._check(self._lib.rekv_encode_chunk(
            self._h, self._dev(q, last=qh, name="q"), self._dev(k_cache, last=kh, name="k_cache"),
            self._dev(v_cache, last=kh, name="v_cache"), first_token, l_x, n_chunks, l_l,
            self._dev(out, last=qh, name="out"), _stream()))
        return out

    def frame_keys(self, k, n_frames: int, out=None):
        kh = (self.n_kv_heads, self.head_dim)
        if k.shape[0] < n_frames * self.tokens_per_frame:
            raise ValueError("k is shorter than n_frames * tokens_per_frame")
        d_prime = self.n_kv_heads * self.head_dim
        out = torch.empty((n_frames, d_prime), dtype=torch.float32, device=k.device) if out is None else out
        if out.shape[0] < n_frames:
            raise ValueError("frame_keys output is shorter than n_frames")
        self._check(self._lib.rekv_frame_keys(
            self._h, self._dev(k, last=kh, name="k"), n_frames,
            self._dev(out, torch.float32, (d_prime,), "frame_keys"), _stream()))
        return out

    def retrieve_topk(self, frame_keys, n_frames: int, q_question, k: int, frame_keys_stride: int = 0,
                      want_scores: bool = False):
        """q_question [n_questions, N_q, Hq, D].  Returns (idx [n_questions, k] int32, n_sel, scores|None)."""
        if q_question.dim() != 4:
            raise ValueError("q_question must be [n_questions, N_q, Hq, D]")
        nq, n_q_tokens = q_question.shape[0], q_question.shape[1]
        d_prime = self.n_kv_heads * self.head_dim
        tables = nq if frame_keys_stride else 1
        need = (tables - 1) * frame_keys_stride + n_frames * d_prime
        if frame_keys.numel() < need:
            raise ValueError("frame_keys holds fewer elements than the tables addressed")
        dev = q_question.device
        idx = torch.empty((nq, k), dtype=torch.int32, device=dev)
        n_sel = torch.empty((nq,), dtype=torch.int32, device=dev)
        scores = torch.empty((nq, n_frames), dtype=torch.float32, device=dev) if want_scores else None
        self._check(self._lib.rekv_retrieve_topk(
            self._h, self._dev(frame_keys, torch.float32, name="frame_keys"), frame_keys_stride, n_frames,
            self._dev(q_question, last=(self.n_q_heads, self.head_dim), name="q_question"), nq, n_q_tokens, k,
            idx.data_ptr(), n_sel.data_ptr(), scores.data_ptr() if want_scores else None, _stream()))
        return idx, n_sel, scores

    def retrieve_external(self, frame_emb, q_emb, k: int, tau: float = 1.0, want_scores: bool = False):
        """frame_emb [n_frames, dim] fp32, q_emb [n_questions, dim] fp32 -> (idx, n_sel, scores|None)."""
        if frame_emb.dim() != 2 or q_emb.dim() != 2 or frame_emb.shape[1] != q_emb.shape[1]:
            raise ValueError("frame_emb [n_frames, dim] and q_emb [n_questions, dim] must share dim")
        n_frames, dim = frame_emb.shape
        nq = q_emb.shape[0]
        dev = q_emb.device
        idx = torch.empty((nq, max(k, 0)), dtype=torch.int32, device=dev)
        n_sel = torch.empty((nq,), dtype=torch.int32, device=dev)
        scores = torch.empty((nq, n_frames), dtype=torch.float32, device=dev) if want_scores else None
        self._check(self._lib.rekv_retrieve_external(
            self._h, self._dev(frame_emb, torch.float32, name="frame_emb"), n_frames, dim,
            self._dev(q_emb, torch.float32, name="q_emb"), nq, tau, k, idx.data_ptr(), n_sel.data_ptr(),
            scores.data_ptr() if want_scores else None, _stream()))
        return idx, n_sel, scores

    def block_keys(self, frame_keys, n_frames: int, b: int, out=None):
        """frame_keys [>= n_frames, D'] fp32 -> block vectors [ceil(n_frames / b), D'] fp32."""
        d_prime = self.n_kv_heads * self.head_dim
        n_blocks = -(-n_frames // b) if b > 0 else 0
        if frame_keys.numel() < n_frames * d_prime:
            raise ValueError("frame_keys holds fewer than n_frames rows")
        out = torch.empty((max(n_blocks, 1), d_prime), dtype=torch.float32, device=frame_keys.device) \
            if out is None else out
        if out.numel() < n_blocks * d_prime:
            raise ValueError("out holds fewer than ceil(n_frames / b) rows")
        self._check(self._lib.rekv_block_keys(self._h, self._dev(frame_keys, torch.float32, name="frame_keys"),
                                              n_frames, b, self._dev(out, torch.float32, name="block_keys"),
                                              _stream()))
        return out

    def expand_blocks(self, block_idx, b: int, n_frames: int):
        """block_idx [n_questions, k_blocks] int32 -> (frame_idx [n_questions, k_blocks * b], n_sel)."""
        if block_idx.dim() != 2 or block_idx.dtype != torch.int32 or not block_idx.is_cuda:
            raise ValueError("block_idx must be a device tensor [n_questions, k_blocks] int32")
        nq, kb = block_idx.shape
        frame_idx = torch.empty((nq, kb * max(b, 0)), dtype=torch.int32, device=block_idx.device)
        n_sel = torch.empty((nq,), dtype=torch.int32, device=block_idx.device)
        self._check(self._lib.rekv_expand_blocks(self._h, block_idx.contiguous().data_ptr(), nq, kb, b, n_frames,
                                                 frame_idx.data_ptr(), n_sel.data_ptr(), _stream()))
        return frame_idx, n_sel

    def gather_kv(self, src_k, src_v, idx, n_src_frames: int | None = None, dst_k=None, dst_v=None,
                  host_mode: int = 2):
        """idx [n_questions, k] int32 on the device.  src on the device, or pinned on the host
        (host_mode 1: copy-engine copies per frame run, 2: the kernel reads host memory itself)."""
        kh = (self.n_kv_heads, self.head_dim)
        on_host = not src_k.is_cuda
        nf = src_k.shape[0] // self.tokens_per_frame if n_src_frames is None else n_src_frames
        if src_k.shape[0] < nf * self.tokens_per_frame or src_v.shape != src_k.shape:
            raise ValueError("src_k / src_v are shorter than n_src_frames frames")
        if idx.dim() != 2 or idx.dtype != torch.int32:
            raise ValueError("idx must be [n_questions, k] int32")
        nq, k = idx.shape
        shape = (nq, k * self.tokens_per_frame, *kh)
        dst_k = torch.empty(shape, dtype=self.torch_dtype, device=idx.device) if dst_k is None else dst_k
        dst_v = torch.empty(shape, dtype=self.torch_dtype, device=idx.device) if dst_v is None else dst_v
        if tuple(dst_k.shape) != shape or tuple(dst_v.shape) != shape:
            raise ValueError(f"dst_k / dst_v must have shape {shape}")
        ps = (self._pinned(src_k, kh, "src_k"), self._pinned(src_v, kh, "src_v")) if on_host else \
             (self._dev(src_k, last=kh, name="src_k"), self._dev(src_v, last=kh, name="src_v"))
        self._check(self._lib.rekv_gather_kv(
            self._h, ps[0], ps[1], host_mode if on_host else 0, nf, self._dev(idx, torch.int32, name="idx"), nq, k,
            self._dev(dst_k, name="dst_k"), self._dev(dst_v, name="dst_v"), _stream()))
        return dst_k, dst_v

    def gather_kv_layers(self, src_k: list, src_v: list, idx, n_src_frames: int | None = None, dst_k=None, dst_v=None):
        """rekv_gather_kv_layers: src_k / src_v are lists of one device arena per layer; idx
        [n_layers, n_questions, k] int32 on the device."""
        kh = (self.n_kv_heads, self.head_dim)
        n_layers = len(src_k)
        if len(src_v) != n_layers or idx.dim() != 3 or idx.shape[0] != n_layers or idx.dtype != torch.int32:
            raise ValueError("idx must be [n_layers, n_questions, k] int32 with one arena pair per layer")
        nf = src_k[0].shape[0] // self.tokens_per_frame if n_src_frames is None else n_src_frames
        for t in list(src_k) + list(src_v):
            if t.shape[0] < nf * self.tokens_per_frame:
                raise ValueError("an arena is shorter than n_src_frames frames")
        _, nq, k = idx.shape
        shape = (n_layers, nq, k * self.tokens_per_frame, *kh)
        dst_k = torch.empty(shape, dtype=self.torch_dtype, device=idx.device) if dst_k is None else dst_k
        dst_v = torch.empty(shape, dtype=self.torch_dtype, device=idx.device) if dst_v is None else dst_v
        if dst_k.numel() != dst_v.numel() or dst_k.numel() != n_layers * nq * k * self.tokens_per_frame * kh[0] * kh[1]:
            raise ValueError(f"dst_k / dst_v must hold {shape}")
        pk = (c_void_p * n_layers)(*[self._dev(t, last=kh, name="src_k") for t in src_k])
        pv = (c_void_p * n_layers)(*[self._dev(t, last=kh, name="src_v") for t in src_v])
        self._check(self._lib.rekv_gather_kv_layers(
            self._h, pk, pv, n_layers, nf, self._dev(idx, torch.int32, name="idx"), nq, k,
            self._dev(dst_k, name="dst_k"), self._dev(dst_v, name="dst_v"), _stream()))
        return dst_k, dst_v

    def gather_kv_rope(self, src_k, src_v, idx, n_src_frames: int | None = None, mode: str = "consecutive",
                       pos_offset: int = 0, src_rotated: bool = False, src_pos_offset: int = 0,
                       base: float = 10000.0, layout: str = "half"):
        """rekv_gather_kv_rope: idx [n_questions, k] int32 on the device; source in HBM or pinned on the host."""
        kh = (self.n_kv_heads, self.head_dim)
        on_host = not src_k.is_cuda
        nf = src_k.shape[0] // self.tokens_per_frame if n_src_frames is None else n_src_frames
        if src_k.shape[0] < nf * self.tokens_per_frame or src_v.shape != src_k.shape:
            raise ValueError("src_k / src_v are shorter than n_src_frames frames")
        if idx.dim() != 2 or idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous():
            raise ValueError("idx must be a contiguous device tensor [n_questions, k] int32")
        nq, k = idx.shape
        shape = (nq, k * self.tokens_per_frame, *kh)
        dst_k = torch.empty(shape, dtype=self.torch_dtype, device=idx.device)
        dst_v = torch.empty(shape, dtype=self.torch_dtype, device=idx.device)
        ps = (self._pinned(src_k, kh, "src_k"), self._pinned(src_v, kh, "src_v")) if on_host else \
             (self._dev(src_k, last=kh, name="src_k"), self._dev(src_v, last=kh, name="src_v"))
        self._check(self._lib.rekv_gather_kv_rope(
            self._h, ps[0], ps[1], int(on_host), nf,
            idx.data_ptr(), nq, k, dst_k.data_ptr(), dst_v.data_ptr(), base,
            {"half": 0, "interleaved": 1}[layout], {"consecutive": 0, "static": 1}[mode], pos_offset,
            int(src_rotated), src_pos_offset, _stream()))
        return dst_k, dst_v

    def attention_indexed_rope(self, q, k_src, v_src, idx, k_text, v_text, n_text_tokens: int,
                               n_src_frames: int | None = None, n_sel=None, mode: str = "consecutive",
                               pos_offset: int = 0, src_rotated: bool = False, src_pos_offset: int = 0,
                               base: float = 10000.0, layout: str = "half", k_pos=None, out=None):
        """rekv_attention_indexed_rope: idx [n_questions, n_ret_frames] int32 (contiguous, device).
        Returns (out, k_pos)."""
        qh, kh = (self.n_q_heads, self.head_dim), (self.n_kv_heads, self.head_dim)
        if q.dim() != 4 or k_text.dim() != 4 or idx.dim() != 2 or idx.dtype != torch.int32 or not idx.is_cuda \
                or not idx.is_contiguous():
            raise ValueError("q, k_text must be 4-d; idx a contiguous device tensor [n_questions, n_ret_frames] int32")
        nq, n_new = q.shape[0], q.shape[1]
        n_ret = idx.shape[1]
        if idx.shape[0] != nq or k_text.shape[0] != nq or v_text.shape != k_text.shape:
            raise ValueError("idx, k_text, v_text must have one row per question")
        nf = k_src.shape[0] // self.tokens_per_frame if n_src_frames is None else n_src_frames
        if k_src.shape[0] < nf * self.tokens_per_frame or v_src.shape != k_src.shape:
            raise ValueError("k_src / v_src are shorter than n_src_frames frames")
        shape = (nq, n_ret * self.tokens_per_frame, *kh)
        k_pos = torch.empty(shape, dtype=self.torch_dtype, device=q.device) if k_pos is None else k_pos
        if tuple(k_pos.shape) != shape:
            raise ValueError(f"k_pos must have shape {shape}")
        out = torch.empty_like(q) if out is None else out
        if out.shape != q.shape:
            raise ValueError("out must have the shape of q")
        self._check(self._lib.rekv_attention_indexed_rope(
            self._h, self._dev(q, last=qh, name="q"), self._dev(k_src, last=kh, name="k_src"),
            self._dev(v_src, last=kh, name="v_src"), nf, idx.data_ptr(), n_ret, n_ret, self._n_sel(n_sel, nq),
            self._dev(k_pos, last=kh, name="k_pos"), base, {"half": 0, "interleaved": 1}[layout],
            {"consecutive": 0, "static": 1}[mode], pos_offset, int(src_rotated), src_pos_offset,
            self._dev(k_text, last=kh, name="k_text"), self._dev(v_text, last=kh, name="v_text"),
            k_text.shape[1], n_text_tokens, nq, n_new, self._dev(out, last=qh, name="out"), _stream()))
        return out, k_pos

    def qa_attention(self, q, k_ret, v_ret, k_self, v_self, out=None, n_sel=None):
        """q [n_questions, N_q, Hq, D]; k_ret/v_ret [n_questions, n_ret, Hkv, D]; k_self/v_self
        [n_questions, N_q, Hkv, D]."""
        qh, kh = (self.n_q_heads, self.head_dim), (self.n_kv_heads, self.head_dim)
        if q.dim() != 4 or k_ret.dim() != 4 or k_self.dim() != 4:
            raise ValueError("q, k_ret, k_self must be 4-d with a leading question dimension")
        nq, n_q_tokens = q.shape[0], q.shape[1]
        n_ret = k_ret.shape[1]
        if k_ret.shape[0] != nq or v_ret.shape != k_ret.shape:
            raise ValueError("k_ret / v_ret must be [n_questions, n_ret, Hkv, D]")
        if tuple(k_self.shape[:2]) != (nq, n_q_tokens) or v_self.shape != k_self.shape:
            raise ValueError("k_self / v_self must be [n_questions, N_q, Hkv, D]")
        out = torch.empty_like(q) if out is None else out
        if out.shape != q.shape:
            raise ValueError("out must have the shape of q")
        self._check(self._lib.rekv_qa_attention(
            self._h, self._dev(q, last=qh, name="q"),
            self._dev(k_ret, last=kh, name="k_ret") if n_ret else None,
            self._dev(v_ret, last=kh, name="v_ret") if n_ret else None, n_ret, self._n_sel(n_sel, nq),
            self._dev(k_self, last=kh, name="k_self"), self._dev(v_self, last=kh, name="v_self"),
            nq, n_q_tokens, self._dev(out, last=qh, name="out"), _stream()))
        return out

    def decode_attention(self, q, k_ret, v_ret, k_text, v_text, n_text_tokens: int, out=None, n_sel=None,
                         no_alloc: bool = False):
        """q [n_questions, n_new, Hq, D]; k_ret/v_ret [n_questions, n_ret, Hkv, D]; k_text/v_text
        [n_questions, text_stride, Hkv, D] whose first n_text_tokens rows are valid and end with
        the new tokens' own K/V."""
        qh, kh = (self.n_q_heads, self.head_dim), (self.n_kv_heads, self.head_dim)
        if q.dim() != 4 or k_ret.dim() != 4 or k_text.dim() != 4:
            raise ValueError("q, k_ret, k_text must be 4-d with a leading question dimension")
        nq, n_new = q.shape[0], q.shape[1]
        n_ret, stride = k_ret.shape[1], k_text.shape[1]
        if k_ret.shape[0] != nq or v_ret.shape != k_ret.shape:
            raise ValueError("k_ret / v_ret must be [n_questions, n_ret, Hkv, D]")
        if k_text.shape[0] != nq or v_text.shape != k_text.shape:
            raise ValueError("k_text / v_text must be [n_questions, text_stride, Hkv, D]")
        out = torch.empty_like(q) if out is None else out
        if out.shape != q.shape:
            raise ValueError("out must have the shape of q")
        fn = self._lib.rekv_decode_attention_noalloc if no_alloc else self._lib.rekv_decode_attention
        self._check(fn(
            self._h, self._dev(q, last=qh, name="q"),
            self._dev(k_ret, last=kh, name="k_ret") if n_ret else None,
            self._dev(v_ret, last=kh, name="v_ret") if n_ret else None, n_ret, self._n_sel(n_sel, nq),
            self._dev(k_text, last=kh, name="k_text"), self._dev(v_text, last=kh, name="v_text"),
            stride, n_text_tokens, nq, n_new, self._dev(out, last=qh, name="out"), _stream()))
        return out

    def attention_indexed(self, q, k_src, v_src, idx, n_ret_frames: int, k_text, v_text, n_text_tokens: int,
                          n_src_frames: int | None = None, out=None, n_sel=None):
        """Eq. 3 with the retrieved KV read in place: q [n_questions, n_new, Hq, D]; k_src/v_src the
        arena [tokens, Hkv, D]; idx [n_questions, >= n_ret_frames] int32; k_text/v_text
        [n_questions, text_stride, Hkv, D]."""
        qh, kh = (self.n_q_heads, self.head_dim), (self.n_kv_heads, self.head_dim)
        if q.dim() != 4 or k_text.dim() != 4 or idx.dim() != 2 or idx.dtype != torch.int32:
            raise ValueError("q, k_text must be 4-d; idx [n_questions, slots] int32")
        nq, n_new = q.shape[0], q.shape[1]
        if idx.shape[0] != nq or k_text.shape[0] != nq or v_text.shape != k_text.shape:
            raise ValueError("idx, k_text, v_text must have one row per question")
        nf = k_src.shape[0] // self.tokens_per_frame if n_src_frames is None else n_src_frames
        if k_src.shape[0] < nf * self.tokens_per_frame or v_src.shape != k_src.shape:
            raise ValueError("k_src / v_src are shorter than n_src_frames frames")
        out = torch.empty_like(q) if out is None else out
        if out.shape != q.shape:
            raise ValueError("out must have the shape of q")
        if not idx.is_cuda or not idx.is_contiguous():
            raise ValueError("idx must be a contiguous device tensor")
        self._check(self._lib.rekv_attention_indexed(
            self._h, self._dev(q, last=qh, name="q"), self._dev(k_src, last=kh, name="k_src"),
            self._dev(v_src, last=kh, name="v_src"), nf, idx.data_ptr(), idx.shape[1], n_ret_frames,
            self._n_sel(n_sel, nq), self._dev(k_text, last=kh, name="k_text"), self._dev(v_text, last=kh, name="v_text"),
            k_text.shape[1], n_text_tokens, nq, n_new, self._dev(out, last=qh, name="out"), _stream()))
        return out

    def offload_kv(self, dev_k, dev_v, host_k, host_v, first_frame: int, n_frames: int):
        kh = (self.n_kv_heads, self.head_dim)
        need = (first_frame + n_frames) * self.tokens_per_frame
        if min(dev_k.shape[0], dev_v.shape[0], host_k.shape[0], host_v.shape[0]) < need:
            raise ValueError("a K/V array is shorter than first_frame + n_frames frames")
        self._check(self._lib.rekv_offload_kv(
            self._h, self._dev(dev_k, last=kh, name="dev_k"), self._dev(dev_v, last=kh, name="dev_v"),
            self._pinned(host_k, kh, "host_k"), self._pinned(host_v, kh, "host_v"), first_frame, n_frames,
            _stream()))

    def offload_wait(self):
        self._check(self._lib.rekv_offload_wait(self._h))

    def offload_join(self):
        """rekv_offload_join: the current stream waits (on the device) for the offloads issued so far."""
        self._check(self._lib.rekv_offload_join(self._h, _stream()))

    def probe_copy(self, dst: torch.Tensor, src: torch.Tensor) -> int:
        """rekv_probe_copy: streaming copy of src into dst; returns the bytes copied."""
        n_bytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() != n_bytes or not (dst.is_cuda and src.is_cuda):
            raise ValueError("probe_copy: dst and src must be device tensors of the same byte size")
        if not (dst.is_contiguous() and src.is_contiguous()):
            raise ValueError("probe_copy: tensors must be contiguous")
        self._check(self._lib.rekv_probe_copy(self._h, dst.data_ptr(), src.data_ptr(), n_bytes, _stream()))
        return n_bytes

    def probe_mfma(self, sink: torch.Tensor, n_workgroups: int, n_iters: int) -> float:
        """rekv_probe_mfma: register-resident MFMA loop; returns the launch's flop count."""
        if sink.dtype != torch.float32 or not sink.is_cuda or sink.numel() < n_workgroups * 256:
            raise ValueError("probe_mfma: sink must be a device fp32 tensor of >= n_workgroups * 256 elements")
        flop = ctypes.c_double(0.0)
        self._check(self._lib.rekv_probe_mfma(self._h, sink.data_ptr(), n_workgroups, n_iters,
                                              ctypes.byref(flop), _stream()))
        return flop.value
