"""Comparison variants of the pattern search and of the block selection, on the CPU.  TEST
INFRASTRUCTURE ONLY (same import rule as the rest of this package); plain numpy in fp64.

The paper compares its block scoring (Sec. 3.2, "Method 3", the one ``block_search`` computes)
with two others (Sec. 3.3, Tab. 1) and its max-based threshold (Sec. 3.4) with Top-k / Top-p
selection (Sec. 1, Sec. 3.4, Tab. 8).  The accuracy columns of those tables need a benchmark suite
and trained weights; what can be reported on synthetic inputs is what each variant *selects*:
density and agreement with the hot-path method.  This module provides

* ``method1_scores``  mean-pooled queries against mean-pooled keys, softmax over the causal blocks
                      (Sec. 3.3, method 1);
* ``method2_scores``  every query against the mean-pooled keys, softmax over the causal blocks per
                      query, then the mean over the queries of the block (Sec. 3.1, the form
                      without the block approximation of Sec. 3.2; this is the L x L/B intermediate);
* ``select_topk`` / ``select_topp``  the two selection rules the paper argues against, with the
                      same always-kept sink and window blocks and the same list format as Alg. 2;
* ``density`` / ``overlap``  what is reported.

Conventions follow the package: Q, K are uint16 bf16 bit patterns [T, H, d]; scores are float32
[Hq, m_total, n_max] with zeros past the diagonal; lists are int32 [Hq, m_total, n_max] + counts.
Readings: the softmax of methods 1 and 2 runs over block columns J <= I only (the pair-level
causal restriction of the hot path, so that the three maps are comparable); a partial last block
pools the keys and queries it has; ties in Top-k / Top-p go to the lower block index.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np

BLOCK = 128


def _bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _layout(cu: Sequence[int], block: int):
    cu = np.asarray(cu, dtype=np.int64)
    nblk = (np.diff(cu) + block - 1) // block
    ro = np.concatenate([[0], np.cumsum(nblk)]).astype(np.int64)
    return cu, ro, int(ro[-1]), int(nblk.max())


def _pool(x: np.ndarray, a: int, b: int, block: int) -> np.ndarray:
    """Mean of each block of rows a..b-1 of x [T, H, d] -> [n, H, d]; the last block may be partial."""
    n = (b - a + block - 1) // block
    out = np.empty((n,) + x.shape[1:], np.float64)
    for j in range(n):
        out[j] = x[a + j * block:min(a + (j + 1) * block, b)].mean(axis=0)
    return out


def _softmax_causal(logits: np.ndarray, I: int) -> np.ndarray:
    """Softmax over columns 0..I of the last axis; zeros elsewhere."""
    z = logits[..., :I + 1]
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    out = np.zeros_like(logits)
    out[..., :I + 1] = e / e.sum(axis=-1, keepdims=True)
    return out


def method1_scores(Q, K, cu_seqlens, tau: Optional[float] = None, block: int = BLOCK) -> np.ndarray:
    """Sec. 3.3 method 1: score[h, I, J] = softmax_{J <= I}(tau * mean(Q_I) . mean(K_J))."""
    q, k = _bf16_to_f64(Q), _bf16_to_f64(K)
    hq, hkv, d = q.shape[1], k.shape[1], q.shape[2]
    g = hq // hkv
    tau = 1.0 / np.sqrt(d) if tau is None else tau
    cu, ro, m_total, n_max = _layout(cu_seqlens, block)
    P = np.zeros((hq, m_total, n_max), np.float32)
    for s in range(len(cu) - 1):
        qb = _pool(q, int(cu[s]), int(cu[s + 1]), block)          # [n, hq, d]
        kb = _pool(k, int(cu[s]), int(cu[s + 1]), block)          # [n, hkv, d]
        n = qb.shape[0]
        for h in range(hq):
            logits = tau * qb[:, h, :] @ kb[:, h // g, :].T       # [n, n]
            for I in range(n):
                P[h, ro[s] + I, :n] = _softmax_causal(logits[I], I)
    return P


def method2_scores(Q, K, cu_seqlens, tau: Optional[float] = None, block: int = BLOCK) -> np.ndarray:
    """Sec. 3.1: a[i, J] = softmax_{J <= I(i)}(tau * q_i . mean(K_J)) for every query i, then
    score[h, I, J] = mean over the queries of block I of a[i, J]."""
    q, k = _bf16_to_f64(Q), _bf16_to_f64(K)
    hq, hkv, d = q.shape[1], k.shape[1], q.shape[2]
    g = hq // hkv
    tau = 1.0 / np.sqrt(d) if tau is None else tau
    cu, ro, m_total, n_max = _layout(cu_seqlens, block)
    P = np.zeros((hq, m_total, n_max), np.float32)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        kb = _pool(k, a, b, block)
        n = kb.shape[0]
        for h in range(hq):
            kbh = kb[:, h // g, :]
            for I in range(n):
                qi = q[a + I * block:min(a + (I + 1) * block, b), h, :]      # [nq, d]
                att = _softmax_causal(tau * qi @ kbh.T, I)                    # [nq, n]
                P[h, ro[s] + I, :n] = att.mean(axis=0)
    return P


def _always_kept(I: int, n: int, sink_blocks: int, window_blocks: int) -> np.ndarray:
    J = np.arange(n)
    return (J <= I) & ((J < sink_blocks) | (I - J < window_blocks))


def _emit(keep_rows, hq, m_total, n_max):
    idx = np.full((hq, m_total, n_max), n_max, np.int32)
    cnt = np.zeros((hq, m_total), np.int32)
    for (h, r), keep in keep_rows.items():
        js = np.nonzero(keep)[0]
        idx[h, r, :js.size] = js
        cnt[h, r] = js.size
    return idx, cnt


def _select(scores, cu_seqlens, block, sink_tokens, window_tokens, rule):
    cu, ro, m_total, n_max = _layout(cu_seqlens, block)
    hq = scores.shape[0]
    sb, wb = -(-sink_tokens // block), -(-window_tokens // block)
    rows = {}
    for s in range(len(cu) - 1):
        n = int(ro[s + 1] - ro[s])
        for I in range(n):
            base = _always_kept(I, n_max, sb, wb)
            for h in range(hq):
                p = scores[h, ro[s] + I, :I + 1].astype(np.float64)
                keep = base.copy()
                keep[:I + 1] |= rule(p)
                rows[(h, int(ro[s] + I))] = keep
    return _emit(rows, hq, m_total, n_max)


def select_topk(scores, cu_seqlens, k: int, block: int = BLOCK, sink_tokens: int = 0, window_tokens: int = 0):
    """The k highest-scoring causal blocks of every row (all of them if the row has fewer), united
    with the sink and window blocks; ascending lists padded with n_max."""
    def rule(p):
        order = np.argsort(-p, kind="stable")          # ties: lower block index first
        keep = np.zeros(p.size, bool)
        keep[order[:k]] = True
        return keep
    return _select(scores, cu_seqlens, block, sink_tokens, window_tokens, rule)


def select_topp(scores, cu_seqlens, p_mass: float, block: int = BLOCK, sink_tokens: int = 0, window_tokens: int = 0):
    """The shortest prefix of the row's blocks in descending score order whose scores add up to at
    least p_mass of the row's total, united with the sink and window blocks."""
    def rule(p):
        order = np.argsort(-p, kind="stable")
        c = np.cumsum(p[order])
        need = int(np.searchsorted(c, p_mass * c[-1] * (1.0 - 1e-12), side="left")) + 1
        keep = np.zeros(p.size, bool)
        keep[order[:min(need, p.size)]] = True
        return keep
    return _select(scores, cu_seqlens, block, sink_tokens, window_tokens, rule)


def density(cnt, cu_seqlens, block: int = BLOCK) -> float:
    """Kept block pairs / causal block pairs, over all heads."""
    cu, ro, m_total, n_max = _layout(cu_seqlens, block)
    n = np.diff(ro)
    return float(cnt.sum()) / float(cnt.shape[0] * (n * (n + 1) // 2).sum())


def _mask(idx, cnt):
    hq, m, n = idx.shape
    out = np.zeros((hq, m, n + 1), bool)
    valid = np.arange(n)[None, None, :] < cnt[:, :, None]
    h, r, j = np.nonzero(valid)
    out[h, r, idx[h, r, j]] = True
    return out[:, :, :n]


def overlap(idx_a, cnt_a, idx_b, cnt_b):
    """(Jaccard index, fraction of b's pairs that a also keeps) of two sets of lists."""
    a, b = _mask(idx_a, cnt_a), _mask(idx_b, cnt_b)
    inter = float((a & b).sum())
    return inter / float((a | b).sum()), inter / float(b.sum())


def attention_mass(Q, K, cu_seqlens, idx, cnt, tau: Optional[float] = None, block: int = BLOCK, rows=None):
    """Mean over (head, query) of the share of the exact causal softmax mass that falls on the
    listed blocks: the quantity every selection rule tries to keep high with few blocks.
    rows: q-block rows to evaluate (default: all)."""
    q, k = _bf16_to_f64(Q), _bf16_to_f64(K)
    hq, hkv, d = q.shape[1], k.shape[1], q.shape[2]
    g = hq // hkv
    tau = 1.0 / np.sqrt(d) if tau is None else tau
    cu, ro, m_total, n_max = _layout(cu_seqlens, block)
    keep = _mask(idx, cnt)
    tot, num = 0.0, 0
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        n = int(ro[s + 1] - ro[s])
        for I in range(n):
            r = int(ro[s] + I)
            if rows is not None and r not in rows:
                continue
            q0, q1 = a + I * block, min(a + (I + 1) * block, b)
            for h in range(hq):
                logits = tau * q[q0:q1, h, :] @ k[a:q1, h // g, :].T           # [nq, keys up to the block's end]
                pos_q = np.arange(q0, q1)[:, None]
                pos_k = np.arange(a, q1)[None, :]
                logits = np.where(pos_k <= pos_q, logits, -np.inf)
                w = np.exp(logits - logits.max(axis=1, keepdims=True))
                w /= w.sum(axis=1, keepdims=True)
                kept_tok = np.repeat(keep[h, r, :I + 1], block)[:q1 - a]
                tot += float(w[:, kept_tok].sum())
                num += q1 - q0
    return tot / max(num, 1)
