"""ctypes binding of include/flashprefill.h: argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are torch CUDA tensors
(PyTorch-ROCm owns device memory and streams); all arithmetic happens in the HIP kernels.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflashprefill.so")

FP_OK, FP_ERR_INVALID_ARG, FP_ERR_UNSUPPORTED, FP_ERR_DEVICE, FP_ERR_NOMEM, FP_ERR_WORKSPACE, FP_ERR_STATIC_LIMIT = range(7)

EXPORTS = ("fp_status_string", "fp_layout", "fp_workspace_bytes", "fp_plan_create", "fp_plan_create_in",
           "fp_plan_destroy", "fp_block_search", "fp_block_search_static",
           "fp_threshold", "fp_search_select", "fp_sparse_prefill", "fp_dense_prefill")


class fp_shape(ctypes.Structure):
    _fields_ = [("nseq", ctypes.c_int32), ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)),
                ("hq", ctypes.c_int32), ("hkv", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block", ctypes.c_int32), ("scale", ctypes.c_float),
                ("cu_seqlens_k", ctypes.POINTER(ctypes.c_int32))]


class fp_params(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_float), ("sink_tokens", ctypes.c_int32), ("window_tokens", ctypes.c_int32)]


class FlashPrefillError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (fp_status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the built library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2603_06199_amd.build` (needs hipcc)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        L.fp_status_string.restype = ctypes.c_char_p
        L.fp_status_string.argtypes = [ctypes.c_int]
        L.fp_layout.argtypes = [ctypes.POINTER(fp_shape), ctypes.POINTER(i32), ctypes.POINTER(i32), vp]
        L.fp_workspace_bytes.argtypes = [ctypes.POINTER(fp_shape)]
        L.fp_workspace_bytes.restype = ctypes.c_size_t
        L.fp_plan_create.argtypes = [ctypes.POINTER(fp_shape), ctypes.c_int, ctypes.POINTER(vp)]
        L.fp_plan_create_in.argtypes = [ctypes.POINTER(fp_shape), ctypes.c_int, vp, ctypes.c_size_t, ctypes.POINTER(vp)]
        L.fp_plan_destroy.argtypes = [vp]
        L.fp_plan_destroy.restype = None
        L.fp_block_search.argtypes = [vp, vp, vp, f32, vp, vp]
        L.fp_block_search_static.argtypes = [vp, vp, vp, f32, vp, vp]
        L.fp_threshold.argtypes = [vp, vp, ctypes.POINTER(fp_params), vp, vp, vp]
        L.fp_search_select.argtypes = [vp, vp, vp, f32, ctypes.POINTER(fp_params), vp, vp, vp]
        L.fp_sparse_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fp_dense_prefill.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().fp_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != FP_OK:
        raise FlashPrefillError(status, where)


def make_shape(cu_seqlens: Sequence[int], hq: int, hkv: int, head_dim: int = 128, block: int = 128,
               scale: float = 0.0, cu_seqlens_k: Optional[Sequence[int]] = None):
    """Builds an fp_shape; returns (shape, keepalive) where keepalive owns the host arrays."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    ck = None if cu_seqlens_k is None else np.ascontiguousarray(cu_seqlens_k, dtype=np.int32)
    if ck is not None and ck.size != cu.size:
        raise ValueError("cu_seqlens_k must have as many entries as cu_seqlens")
    s = fp_shape(int(cu.size - 1), cu.ctypes.data_as(i32p), hq, hkv, head_dim, block, float(scale),
                 None if ck is None else ck.ctypes.data_as(i32p))
    return s, (cu, ck)


def fp_layout(cu_seqlens: Sequence[int], hq: int, hkv: int, head_dim: int = 128, block: int = 128,
              scale: float = 0.0, cu_seqlens_k: Optional[Sequence[int]] = None):
    """Host-only shape check; returns (m_total, n_max, row_offset)."""
    s, keep = make_shape(cu_seqlens, hq, hkv, head_dim, block, scale, cu_seqlens_k)
    m, n = ctypes.c_int32(), ctypes.c_int32()
    ro = np.zeros(max(int(s.nseq) + 1, 1), np.int32)
    _check(lib().fp_layout(ctypes.byref(s), ctypes.byref(m), ctypes.byref(n), ro.ctypes.data_as(ctypes.c_void_p)),
           "fp_layout")
    return int(m.value), int(n.value), ro


def fp_workspace_bytes(cu_seqlens: Sequence[int], hq: int, hkv: int, head_dim: int = 128, block: int = 128,
                       scale: float = 0.0, cu_seqlens_k: Optional[Sequence[int]] = None) -> int:
    """Host-only: bytes of device memory a plan for this shape needs (0 for a shape the library rejects)."""
    s, keep = make_shape(cu_seqlens, hq, hkv, head_dim, block, scale, cu_seqlens_k)
    return int(lib().fp_workspace_bytes(ctypes.byref(s)))


def _stream_ptr(stream) -> Optional[int]:
    import torch
    st = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(st.cuda_stream)


def _dev_ptr(t, dtype, shape, name: str):
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA tensor")
    if t.dtype != dtype or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise TypeError(f"{name}: expected contiguous {dtype} of shape {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


class Plan:
    """Owns an fp_plan (device tables + pooled-key workspace) for one packed-batch shape."""

    def __init__(self, cu_seqlens: Sequence[int], hq: int, hkv: int, head_dim: int = 128, block: int = 128,
                 scale: float = 0.0, device: int = 0, cu_seqlens_k: Optional[Sequence[int]] = None, workspace=None):
        self.cu_seqlens = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        self.cu_seqlens_k = None if cu_seqlens_k is None else np.ascontiguousarray(cu_seqlens_k, dtype=np.int32)
        self.hq, self.hkv, self.head_dim, self.block = hq, hkv, head_dim, block
        self.device = device
        self.m_total, self.n_max, self.row_offset = fp_layout(self.cu_seqlens, hq, hkv, head_dim, block, scale,
                                                              self.cu_seqlens_k)
        self.T = int(self.cu_seqlens[-1])                                                   # query tokens
        self.Tk = self.T if self.cu_seqlens_k is None else int(self.cu_seqlens_k[-1])      # key tokens
        s, keep = make_shape(self.cu_seqlens, hq, hkv, head_dim, block, scale, self.cu_seqlens_k)
        h = ctypes.c_void_p()
        self._workspace = workspace          # a caller-owned torch.uint8 CUDA tensor, kept alive with the plan
        if workspace is None:
            _check(lib().fp_plan_create(ctypes.byref(s), device, ctypes.byref(h)), "fp_plan_create")
        else:
            _check(lib().fp_plan_create_in(ctypes.byref(s), device, ctypes.c_void_p(workspace.data_ptr()),
                                           workspace.numel() * workspace.element_size(), ctypes.byref(h)),
                   "fp_plan_create_in")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().fp_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # --- the compute calls --------------------------------------------------------------------
    def fp_block_search(self, Q, K, scores=None, eps: float = 1e-10, stream=None):
        import torch
        q = _dev_ptr(Q, torch.bfloat16, (self.T, self.hq, self.head_dim), "Q")
        k = _dev_ptr(K, torch.bfloat16, (self.Tk, self.hkv, self.head_dim), "K")
        if scores is None:
            # zero-filled: the library leaves the columns past a sequence's own last key block alone
            scores = torch.zeros((self.hq, self.m_total, self.n_max), dtype=torch.float32, device=Q.device)
        s = _dev_ptr(scores, torch.float32, (self.hq, self.m_total, self.n_max), "scores")
        _check(lib().fp_block_search(self._h, q, k, float(eps), s, _stream_ptr(stream)), "fp_block_search")
        return scores

    def fp_block_search_static(self, Q, K, scores, eps: float = 1e-10, stream=None):
        """fp_block_search with the pooled keys in the library's built-in scratch; `scores` is the caller's."""
        import torch
        q = _dev_ptr(Q, torch.bfloat16, (self.T, self.hq, self.head_dim), "Q")
        k = _dev_ptr(K, torch.bfloat16, (self.Tk, self.hkv, self.head_dim), "K")
        s = _dev_ptr(scores, torch.float32, (self.hq, self.m_total, self.n_max), "scores")
        _check(lib().fp_block_search_static(self._h, q, k, float(eps), s, _stream_ptr(stream)), "fp_block_search_static")
        return scores

    def fp_threshold(self, scores, alpha: float, sink_tokens: int = 256, window_tokens: int = 512, idx=None,
                     cnt=None, stream=None):
        import torch
        s = _dev_ptr(scores, torch.float32, (self.hq, self.m_total, self.n_max), "scores")
        if idx is None:
            idx = torch.empty((self.hq, self.m_total, self.n_max), dtype=torch.int32, device=scores.device)
        if cnt is None:
            cnt = torch.empty((self.hq, self.m_total), dtype=torch.int32, device=scores.device)
        i = _dev_ptr(idx, torch.int32, (self.hq, self.m_total, self.n_max), "idx")
        c = _dev_ptr(cnt, torch.int32, (self.hq, self.m_total), "cnt")
        prm = fp_params(float(alpha), int(sink_tokens), int(window_tokens))
        _check(lib().fp_threshold(self._h, s, ctypes.byref(prm), i, c, _stream_ptr(stream)), "fp_threshold")
        return idx, cnt

    def fp_search_select(self, Q, K, alpha: float, sink_tokens: int = 256, window_tokens: int = 512, idx=None,
                         cnt=None, eps: float = 1e-10, stream=None):
        import torch
        q = _dev_ptr(Q, torch.bfloat16, (self.T, self.hq, self.head_dim), "Q")
        k = _dev_ptr(K, torch.bfloat16, (self.Tk, self.hkv, self.head_dim), "K")
        if idx is None:
            idx = torch.empty((self.hq, self.m_total, self.n_max), dtype=torch.int32, device=Q.device)
        if cnt is None:
            cnt = torch.empty((self.hq, self.m_total), dtype=torch.int32, device=Q.device)
        i = _dev_ptr(idx, torch.int32, (self.hq, self.m_total, self.n_max), "idx")
        c = _dev_ptr(cnt, torch.int32, (self.hq, self.m_total), "cnt")
        prm = fp_params(float(alpha), int(sink_tokens), int(window_tokens))
        _check(lib().fp_search_select(self._h, q, k, float(eps), ctypes.byref(prm), i, c, _stream_ptr(stream)),
               "fp_search_select")
        return idx, cnt

    def _qkv(self, Q, K, V):
        import torch
        return (_dev_ptr(Q, torch.bfloat16, (self.T, self.hq, self.head_dim), "Q"),
                _dev_ptr(K, torch.bfloat16, (self.Tk, self.hkv, self.head_dim), "K"),
                _dev_ptr(V, torch.bfloat16, (self.Tk, self.hkv, self.head_dim), "V"))

    def fp_sparse_prefill(self, Q, K, V, idx, cnt, O=None, lse=None, want_lse: bool = True, stream=None):
        import torch
        q, k, v = self._qkv(Q, K, V)
        i = _dev_ptr(idx, torch.int32, (self.hq, self.m_total, self.n_max), "idx")
        c = _dev_ptr(cnt, torch.int32, (self.hq, self.m_total), "cnt")
        if O is None:
            O = torch.empty_like(Q)
        if lse is None and want_lse:
            lse = torch.empty((self.hq, self.T), dtype=torch.float32, device=Q.device)
        o = _dev_ptr(O, torch.bfloat16, (self.T, self.hq, self.head_dim), "O")
        ls = _dev_ptr(lse, torch.float32, (self.hq, self.T), "lse")
        _check(lib().fp_sparse_prefill(self._h, q, k, v, i, c, o, ls, _stream_ptr(stream)), "fp_sparse_prefill")
        return O, lse

    def fp_dense_prefill(self, Q, K, V, O=None, lse=None, want_lse: bool = True, stream=None):
        import torch
        q, k, v = self._qkv(Q, K, V)
        if O is None:
            O = torch.empty_like(Q)
        if lse is None and want_lse:
            lse = torch.empty((self.hq, self.T), dtype=torch.float32, device=Q.device)
        o = _dev_ptr(O, torch.bfloat16, (self.T, self.hq, self.head_dim), "O")
        ls = _dev_ptr(lse, torch.float32, (self.hq, self.T), "lse")
        _check(lib().fp_dense_prefill(self._h, q, k, v, o, ls, _stream_ptr(stream)), "fp_dense_prefill")
        return O, lse


def to_device_bf16(bits: np.ndarray, device: str = "cuda:0"):
    """uint16 bf16 bit patterns on the host -> torch.bfloat16 tensor on the device (a copy, no arithmetic)."""
    import torch
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)
