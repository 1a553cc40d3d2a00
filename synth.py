"""Seeded synthetic Q/K/V and block-list generators.

This module only *draws inputs*: random numbers, rotary position embedding,
planted structure, rounding to bf16.  It holds none of the method's arithmetic
(no pooling, scoring, thresholding or attention) and is the one module that
both the GPU path's tests/bench and the CPU oracle's tests may use.

Tensors are returned as numpy ``uint16`` arrays holding bf16 bit patterns:
``Q`` is ``[T, Hq, d]``, ``K`` and ``V`` are ``[T, Hkv, d]`` (token-major,
packed: sequence ``s`` owns tokens ``cu_seqlens[s]:cu_seqlens[s+1]``).

The workloads stand in, by shape only, for the attention layers the paper
measures (Qwen3-30B-A3B: 32 query heads / 4 KV heads / head_dim 128;
Llama-3-8B: 32 / 8 / 128; 4K-256K tokens, Experiments section).  No dataset
item or model weight is reproduced.

Two planting modes:

``literal``
    N(0,1) draws, RoPE (theta 1e6, rotate-half pairing, positions restart at
    each sequence), then: ``K[p] += k_gain*u`` at ``n_vert`` seeded positions
    (always including position 0) and ``Q[t] += q_gain*u`` for every token,
    ``u`` one shared unit vector (``n_vert = -1`` picks ``round(16 (L/4096)^0.32)``
    positions from the sequence length); and for every KV head ``n_slash`` lags
    ``l``: ``K[t] += slash_gain * unit(Q_rope[t+l, first q-head of group])``.

``coherent``
    same draws, but structure is planted per 128-token block so it survives
    mean pooling of a key block: the vertical gain is added to *all* keys of
    each planted block, and slash structure uses one random unit vector
    ``w[b]`` per block ``b`` (``Q[t] += slash_q_gain*w[t//B]``,
    ``K[t] += slash_gain*w[t//B + lag_blocks]``).  This is the supplementary
    input that reaches the sparse regime the paper reports densities for.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Sequence, Tuple

import numpy as np

BLOCK = 128

_TENSOR_Q, _TENSOR_K, _TENSOR_V, _TENSOR_AUX = 0, 1, 2, 3


@dataclasses.dataclass(frozen=True)
class Workload:
    """A named synthetic attention-layer input recipe."""

    name: str
    seqlens: Tuple[int, ...]
    hq: int
    hkv: int
    head_dim: int = 128
    seed: int = 0
    n_vert: int = 16
    n_slash: int = 0
    mode: str = "literal"
    k_gain: float = 4.0
    q_gain: float = 0.5
    slash_gain: float = 4.0
    slash_q_gain: float = 0.0
    rope_theta: float = 1.0e6
    alpha: float = 0.12

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seqlens)]).astype(np.int32)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seqlens))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to the float32 values they denote."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, seq: int, tensor: int, head: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 20) ^ (seq << 8) ^ tensor, head]))


def _rope_tables(length: int, d: int, theta: float) -> Tuple[np.ndarray, np.ndarray]:
    half = d // 2
    inv_freq = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / d)
    ang = np.arange(length, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def _apply_rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    half = x.shape[-1] // 2
    a, b = x[:, :half], x[:, half:]
    out = np.empty_like(x)
    out[:, :half] = a * cos - b * sin
    out[:, half:] = b * cos + a * sin
    return out


def _unit(v: np.ndarray) -> np.ndarray:
    return v / np.linalg.norm(v, axis=-1, keepdims=True)


def _seq_plan(w: Workload, s: int, length: int):
    """Seeded structure for one sequence: shared direction, vertical positions, lags."""
    g = _rng(w.seed, s, _TENSOR_AUX, 0)
    u = _unit(g.standard_normal(w.head_dim)).astype(np.float32)
    nv = w.n_vert if w.n_vert >= 0 else int(round(16.0 * (length / 4096.0) ** 0.32))
    nv = min(nv, length)
    if nv > 0:
        rest = g.choice(np.arange(1, length), size=nv - 1, replace=False) if nv > 1 else np.empty(0, np.int64)
        vert = np.sort(np.concatenate([[0], rest])).astype(np.int64)
    else:
        vert = np.empty(0, np.int64)
    lags = []
    nblk = (length + BLOCK - 1) // BLOCK
    for hk in range(w.hkv):
        gh = _rng(w.seed, s, _TENSOR_AUX, 1 + hk)
        if w.n_slash == 0 or length <= 2 * BLOCK:
            lags.append(np.empty(0, np.int64))
        elif w.mode == "literal":
            lags.append(np.sort(gh.integers(BLOCK, max(BLOCK + 1, length // 2), size=w.n_slash)).astype(np.int64))
        else:
            hi = max(5, nblk // 2)
            lags.append(np.sort(gh.integers(4, hi, size=w.n_slash)).astype(np.int64))  # in blocks
    return u, vert, lags


def _block_dirs(w: Workload, s: int, nblk: int) -> np.ndarray:
    g = _rng(w.seed, s, _TENSOR_AUX, 1000)
    return _unit(g.standard_normal((nblk, w.head_dim))).astype(np.float32)


def _make_sequence(w: Workload, s: int, length: int, Q: np.ndarray, K: np.ndarray, V: np.ndarray, pool: ThreadPoolExecutor):
    d, g = w.head_dim, w.hq // w.hkv
    cos, sin = _rope_tables(length, d, w.rope_theta)
    u, vert, lags = _seq_plan(w, s, length)
    nblk = (length + BLOCK - 1) // BLOCK
    coherent = w.mode == "coherent"
    wdir = _block_dirs(w, s, nblk) if coherent and w.n_slash > 0 else None
    tok_blk = np.arange(length) // BLOCK

    def q_rope(h: int) -> np.ndarray:
        x = _rng(w.seed, s, _TENSOR_Q, h).standard_normal((length, d), dtype=np.float32)
        return _apply_rope(x, cos, sin)

    def do_q(h: int):
        x = q_rope(h)
        x += np.float32(w.q_gain) * u
        if wdir is not None and w.slash_q_gain != 0.0:
            x += np.float32(w.slash_q_gain) * wdir[tok_blk]
        Q[:, h, :] = f32_to_bf16_bits(x)

    def do_k(hk: int):
        x = _rng(w.seed, s, _TENSOR_K, hk).standard_normal((length, d), dtype=np.float32)
        x = _apply_rope(x, cos, sin)
        if coherent:
            planted = np.unique(vert // BLOCK)
            sel = np.isin(tok_blk, planted)
            x[sel] += np.float32(w.k_gain) * u
        else:
            x[vert] += np.float32(w.k_gain) * u
        if lags[hk].size:
            if coherent:
                for lb in lags[hk]:
                    src = tok_blk + int(lb)
                    ok = src < nblk
                    x[ok] += np.float32(w.slash_gain) * wdir[src[ok]]
            else:
                qhat = _unit(q_rope(hk * g))
                for lag in lags[hk]:
                    lag = int(lag)
                    if lag < length:
                        x[: length - lag] += np.float32(w.slash_gain) * qhat[lag:]
        K[:, hk, :] = f32_to_bf16_bits(x)

    def do_v(hk: int):
        x = _rng(w.seed, s, _TENSOR_V, hk).standard_normal((length, d), dtype=np.float32)
        V[:, hk, :] = f32_to_bf16_bits(x)

    futs = [pool.submit(do_q, h) for h in range(w.hq)]
    futs += [pool.submit(do_k, hk) for hk in range(w.hkv)]
    futs += [pool.submit(do_v, hk) for hk in range(w.hkv)]
    for f in futs:
        f.result()


def make_qkv(w: Workload, threads: int = 8) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Draw (Q, K, V) bf16-bit arrays for a workload.  Deterministic in ``w`` alone."""
    T, d = w.total_tokens, w.head_dim
    Q = np.empty((T, w.hq, d), np.uint16)
    K = np.empty((T, w.hkv, d), np.uint16)
    V = np.empty((T, w.hkv, d), np.uint16)
    cu = w.cu_seqlens
    with ThreadPoolExecutor(max_workers=threads) as pool:
        for s, length in enumerate(w.seqlens):
            a, b = int(cu[s]), int(cu[s + 1])
            _make_sequence(w, s, length, Q[a:b], K[a:b], V[a:b], pool)
    return Q, K, V


def random_qkv(seqlens: Sequence[int], hq: int, hkv: int, d: int, seed: int, scale: float = 1.0):
    """Plain N(0, scale^2) bf16 Q/K/V with no structure (unit-test inputs)."""
    T = int(sum(seqlens))
    g = np.random.default_rng(seed)
    mk = lambda h: f32_to_bf16_bits((g.standard_normal((T, h, d), dtype=np.float32) * np.float32(scale)))
    return mk(hq), mk(hkv), mk(hkv)


# --- the five benchmark configurations --------------------------------------------------------

def config(i: int, mode: str = "literal") -> Workload:
    """Configurations 0..4 of the benchmark (4K toy GQA, Qwen3 shape at 32K/128K/256K, Llama varlen).

    ``mode="coherent"`` gives the block-coherent planting with gains calibrated so the kept
    fraction of causal blocks falls with length roughly as the paper's density table does.
    """
    base = [
        dict(name="c0_4k_gqa4x1", seqlens=(4096,), hq=4, hkv=1, n_vert=16, n_slash=0, alpha=0.12),
        dict(name="c1_qwen3_32k", seqlens=(32768,), hq=32, hkv=4, n_vert=64, n_slash=8, alpha=0.12),
        dict(name="c2_qwen3_128k", seqlens=(131072,), hq=32, hkv=4, n_vert=128, n_slash=8, alpha=0.12),
        dict(name="c3_qwen3_256k", seqlens=(262144,), hq=32, hkv=4, n_vert=128, n_slash=8, alpha=0.12),
        dict(name="c4_llama_varlen", seqlens=(4096, 16384, 65536, 131072), hq=32, hkv=8, n_vert=64, n_slash=8, alpha=0.18),
    ][i]
    if mode == "coherent":
        base = dict(base)
        base.update(mode="coherent", name=base["name"] + "_coherent", k_gain=4.0, q_gain=8.0,
                    slash_gain=4.0, slash_q_gain=8.0)
        # the vertical floor on density is (planted blocks) / N: n_vert = -1 picks, per sequence,
        # round(16 (L/4096)^0.32) planted positions, which with the always-kept sink and window
        # blocks tracks the paper's density-vs-length table (about 70 % at 4K down to 3.5 % at 256K)
        base["n_vert"] = -1
        base["n_slash"] = min(base["n_slash"], 2) if base["n_slash"] else 0
    return Workload(**base)


def small(name: str, seqlens: Sequence[int], hq: int, hkv: int, seed: int = 0, mode: str = "coherent", **kw) -> Workload:
    """A small test workload with the same recipe (several tiles, optionally ragged tails)."""
    args = dict(name=name, seqlens=tuple(int(x) for x in seqlens), hq=hq, hkv=hkv, seed=seed, mode=mode,
                n_vert=4, n_slash=2 if max(seqlens) > 4 * BLOCK else 0)
    if mode == "coherent":
        args.update(k_gain=4.0, q_gain=8.0, slash_gain=4.0, slash_q_gain=8.0)
    args.update(kw)
    return Workload(**args)


# --- forced-density block lists (inputs for the sparse kernel alone) ----------------------------

def layout(cu_seqlens: Sequence[int], block: int = BLOCK):
    """Row bookkeeping of a packed batch: (m_total, n_max, row_offset[nseq+1])."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    nblk = (np.diff(cu) + block - 1) // block
    row_offset = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int32)
    return int(row_offset[-1]), int(nblk.max()) if nblk.size else 0, row_offset


def forced_density_lists(cu_seqlens: Sequence[int], hq: int, density: float, seed: int,
                         sink_blocks: int = 2, window_blocks: int = 4, block: int = BLOCK):
    """Random causal block lists with a target kept fraction; sink and window blocks always kept.

    Returns (idx[hq, m_total, n_max] int32, cnt[hq, m_total] int32); ``idx`` rows are ascending
    and entries past ``cnt`` are left at -1.
    """
    m_total, n_max, row_offset = layout(cu_seqlens, block)
    idx = np.full((hq, m_total, n_max), -1, np.int32)
    cnt = np.zeros((hq, m_total), np.int32)
    g = np.random.default_rng(seed)
    for s in range(len(row_offset) - 1):
        n = int(row_offset[s + 1] - row_offset[s])
        for h in range(hq):
            keep = g.random((n, n)) < density
            I = np.arange(n)[:, None]
            J = np.arange(n)[None, :]
            keep |= (J < sink_blocks) | ((I - J >= 0) & (I - J < window_blocks))
            keep &= J <= I
            for i in range(n):
                js = np.nonzero(keep[i])[0].astype(np.int32)
                r = int(row_offset[s]) + i
                idx[h, r, : js.size] = js
                cnt[h, r] = js.size
    return idx, cnt
