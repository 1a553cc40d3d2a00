"""ctypes loader for the CPU oracle (``fp_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may import
this package.  It imports nothing from the GPU package and the GPU package never imports it.

All tensors are numpy arrays on the host: Q/K/V as uint16 bf16 bit patterns
([T, Hq, d] / [Tk, Hkv, d]), scores float32 [Hq, m_total, n_max], idx int32 like scores,
cnt int32 [Hq, m_total], O float32 [T, Hq, d], lse float32 [Hq, T].  ``cu_seqlens_k`` (optional)
gives the key-side lengths for chunked prefill: the queries are then the last tokens of each
sequence and the prefix kv_len - q_len must be a multiple of the block size.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fp_oracle.c")
_SO = os.path.join(_HERE, "libfp_oracle.so")
_lib = None

BLOCK = 128
SINK_TOKENS = 256      # Appendix A: attention-sink size in tokens
WINDOW_TOKENS = 512    # Appendix A: local-window size in tokens
EPS = 1e-10


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 arithmetic, no fused contraction, OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=gnu11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        vp, i32, f64, f32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_float
        L.fpo_num_threads.restype = i32
        L.fpo_layout.argtypes = [i32, vp, vp, i32, vp, vp, vp]
        L.fpo_block_search.argtypes = [vp, vp, i32, vp, vp, i32, i32, i32, i32, f64, f64, vp, i32, vp]
        L.fpo_threshold.argtypes = [vp, i32, vp, vp, i32, i32, f32, i32, i32, vp, vp]
        L.fpo_sparse_prefill.argtypes = [vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, f64, vp, vp, vp, i32, vp, vp]
        L.fpo_dense_prefill.argtypes = [vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, f64, vp, i32, vp, vp]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().fpo_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a: np.ndarray, dtype, name: str) -> np.ndarray:
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: expected C-contiguous {np.dtype(dtype).name}, got {a.dtype}")
    return a


def _cu(cu_seqlens: Sequence[int]) -> np.ndarray:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    if cu.ndim != 1 or cu.size < 2 or cu[0] != 0 or np.any(np.diff(cu) <= 0):
        raise ValueError("cu_seqlens must start at 0 and increase strictly")
    return cu


def _cuk(cu: np.ndarray, cu_seqlens_k) -> Optional[np.ndarray]:
    """Key-side cumulative lengths for chunked prefill (None: keys = queries)."""
    if cu_seqlens_k is None:
        return None
    ck = _cu(cu_seqlens_k)
    if ck.size != cu.size:
        raise ValueError("cu_seqlens_k must have as many entries as cu_seqlens")
    return ck


def layout(cu_seqlens: Sequence[int], block: int = BLOCK, cu_seqlens_k=None):
    cu = _cu(cu_seqlens)
    ck = _cuk(cu, cu_seqlens_k)
    m, n = ctypes.c_int32(), ctypes.c_int32()
    ro = np.zeros(cu.size, np.int32)
    rc = lib().fpo_layout(cu.size - 1, _p(cu), _p(ck), block, ctypes.byref(m), ctypes.byref(n), _p(ro))
    if rc != 0:
        raise ValueError("lengths not supported: every sequence needs kv_len >= q_len >= 1 and a prefix "
                         "(kv_len - q_len) that is a multiple of the block size")
    return int(m.value), int(n.value), ro


def _rows(rows):
    if rows is None:
        return None, 0
    r = np.ascontiguousarray(rows, dtype=np.int32)
    return r, int(r.size)


def block_search(Q, K, cu_seqlens, tau: Optional[float] = None, block: int = BLOCK, eps: float = EPS,
                 rows=None, out: Optional[np.ndarray] = None, cu_seqlens_k=None) -> np.ndarray:
    """Block importance map P (Alg. 1).  Returns float32 [Hq, m_total, n_max]."""
    cu = _cu(cu_seqlens)
    ck = _cuk(cu, cu_seqlens_k)
    _chk(Q, np.uint16, "Q"); _chk(K, np.uint16, "K")
    T, hq, d = Q.shape
    hkv = K.shape[1]
    assert K.shape == ((T if ck is None else ck[-1]), hkv, d) and T == cu[-1] and hq % hkv == 0
    m_total, n_max, _ = layout(cu, block, ck)
    if out is None:
        out = np.zeros((hq, m_total, n_max), np.float32)
    _chk(out, np.float32, "out")
    assert out.shape == (hq, m_total, n_max)
    tau = 1.0 / np.sqrt(d) if tau is None else float(tau)
    r, nr = _rows(rows)
    rc = lib().fpo_block_search(_p(Q), _p(K), cu.size - 1, _p(cu), _p(ck), hq, hkv, d, block, tau, eps, _p(r), nr,
                                _p(out))
    assert rc == 0
    return out


def threshold(scores, cu_seqlens, alpha: float, block: int = BLOCK, sink_tokens: int = SINK_TOKENS,
              window_tokens: int = WINDOW_TOKENS, cu_seqlens_k=None):
    """Active block lists (Alg. 2).  Returns (idx int32 [Hq, m_total, n_max], cnt int32 [Hq, m_total])."""
    cu = _cu(cu_seqlens)
    ck = _cuk(cu, cu_seqlens_k)
    _chk(scores, np.float32, "scores")
    hq, m_total, n_max = scores.shape
    assert (m_total, n_max) == layout(cu, block, ck)[:2]
    idx = np.empty((hq, m_total, n_max), np.int32)
    cnt = np.empty((hq, m_total), np.int32)
    rc = lib().fpo_threshold(_p(scores), cu.size - 1, _p(cu), _p(ck), hq, block, float(alpha), sink_tokens,
                             window_tokens, _p(idx), _p(cnt))
    assert rc == 0
    return idx, cnt


def sparse_prefill(Q, K, V, cu_seqlens, idx, cnt, tau: Optional[float] = None, block: int = BLOCK, rows=None,
                   O: Optional[np.ndarray] = None, lse: Optional[np.ndarray] = None, cu_seqlens_k=None):
    """Attention over the listed blocks only (Alg. 3).  Returns (O float32 [T,Hq,d], lse float32 [Hq,T])."""
    cu = _cu(cu_seqlens)
    ck = _cuk(cu, cu_seqlens_k)
    for a, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _chk(a, np.uint16, n)
    _chk(idx, np.int32, "idx"); _chk(cnt, np.int32, "cnt")
    T, hq, d = Q.shape
    hkv = K.shape[1]
    assert K.shape == V.shape == ((T if ck is None else ck[-1]), hkv, d) and T == cu[-1] and hq % hkv == 0
    m_total, n_max, _ = layout(cu, block, ck)
    assert idx.shape == (hq, m_total, n_max) and cnt.shape == (hq, m_total)
    O = np.zeros((T, hq, d), np.float32) if O is None else _chk(O, np.float32, "O")
    lse = np.zeros((hq, T), np.float32) if lse is None else _chk(lse, np.float32, "lse")
    tau = 1.0 / np.sqrt(d) if tau is None else float(tau)
    r, nr = _rows(rows)
    rc = lib().fpo_sparse_prefill(_p(Q), _p(K), _p(V), cu.size - 1, _p(cu), _p(ck), hq, hkv, d, block, tau, _p(idx),
                                  _p(cnt), _p(r), nr, _p(O), _p(lse))
    assert rc == 0
    return O, lse


def dense_prefill(Q, K, V, cu_seqlens, tau: Optional[float] = None, block: int = BLOCK, rows=None,
                  O: Optional[np.ndarray] = None, lse: Optional[np.ndarray] = None, cu_seqlens_k=None):
    """Full causal attention.  Returns (O float32 [T,Hq,d], lse float32 [Hq,T])."""
    cu = _cu(cu_seqlens)
    ck = _cuk(cu, cu_seqlens_k)
    for a, n in ((Q, "Q"), (K, "K"), (V, "V")):
        _chk(a, np.uint16, n)
    T, hq, d = Q.shape
    hkv = K.shape[1]
    assert K.shape == V.shape == ((T if ck is None else ck[-1]), hkv, d) and T == cu[-1] and hq % hkv == 0
    if ck is not None:
        layout(cu, block, ck)   # raises on lengths the path does not take
    O = np.zeros((T, hq, d), np.float32) if O is None else _chk(O, np.float32, "O")
    lse = np.zeros((hq, T), np.float32) if lse is None else _chk(lse, np.float32, "lse")
    tau = 1.0 / np.sqrt(d) if tau is None else float(tau)
    r, nr = _rows(rows)
    rc = lib().fpo_dense_prefill(_p(Q), _p(K), _p(V), cu.size - 1, _p(cu), _p(ck), hq, hkv, d, block, tau, _p(r), nr,
                                 _p(O), _p(lse))
    assert rc == 0
    return O, lse
