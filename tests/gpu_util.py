"""Helpers shared by the GPU parity tests: run the HIP path, run the oracle, compare."""
import numpy as np

import oracle
from paper_2603_06199_amd import binding as B
import synth

# Tolerances.  Attention outputs: bf16 inputs, fp32 accumulation, P rounded to bf16 before the
# PV product and O rounded to bf16 on store -> max-abs 2e-2, mean-abs 2e-3.  Block scores: the
# pooled key is carried as bf16 hi+lo (relative 2^-17 per component) and logits accumulate in
# fp32, so a score's relative error stays a few 1e-5; 5e-4 leaves margin, with an absolute floor
# for scores that flush to zero (the GPU's exp2 has no denormal results).
O_MAX_ABS, O_MEAN_ABS = 2e-2, 2e-3
SCORE_RTOL, SCORE_ATOL = 5e-4, 1e-30
# lse = c*m + log2(sum p): the row sum is taken over the fp32 exponentials (before they are rounded
# to bf16 for the PV product), so what is left is the fp32 accumulation of the logits (128 exact
# bf16 x bf16 products each: a few 1e-6 relative of |q||k|), the hardware exp2 / log2 (1 ulp) and
# the fp32 sum of up to 2^18 terms; logits here reach a few tens, so 5e-4 absolute leaves an
# order of magnitude of margin over the largest error the randomised sweeps met.
LSE_ATOL = 5e-4
BAND = 1e-3           # near-threshold band: |score - alpha*max| <= BAND * alpha*max


def dev(bits):
    return B.to_device_bf16(bits)


def f32(t):
    return t.float().cpu().numpy()


def causal_mask(cu, block=128):
    m_total, n_max, ro = synth.layout(cu, block)
    mask = np.zeros((m_total, n_max), bool)
    for s in range(len(ro) - 1):
        n = ro[s + 1] - ro[s]
        mask[ro[s]:ro[s + 1], :n] = np.tril(np.ones((n, n), bool))
    return mask


def own_columns_mask(cu, block=128):
    """[m_total, n_max] bool: column J belongs to the row's own sequence (J < its number of key blocks)."""
    m_total, n_max, ro = synth.layout(cu, block)
    mask = np.zeros((m_total, n_max), bool)
    for s in range(len(ro) - 1):
        mask[ro[s]:ro[s + 1], :ro[s + 1] - ro[s]] = True
    return mask


def compare_scores(P_gpu, P_ref, cu, rows=None, block=128):
    mask = causal_mask(cu, block)
    own = own_columns_mask(cu, block)
    if rows is not None:
        sel = np.zeros(mask.shape[0], bool); sel[list(rows)] = True
        mask &= sel[:, None]
        own &= sel[:, None]
    a, b = P_gpu[:, mask], P_ref[:, mask]
    np.testing.assert_allclose(a, b, rtol=SCORE_RTOL, atol=SCORE_ATOL)
    assert np.all(P_gpu[:, own & ~mask] == 0.0), "entries above the diagonal, up to the sequence's last block, must be written as 0"


def compare_lists_exact(idx_g, cnt_g, idx_r, cnt_r):
    assert np.array_equal(cnt_g, cnt_r)
    n = idx_r.shape[2]
    valid = np.arange(n)[None, None, :] < cnt_r[:, :, None]
    assert np.array_equal(idx_g[valid], idx_r[valid])


def lists_to_mask(idx, cnt):
    hq, m, n = idx.shape
    out = np.zeros((hq, m, n + 1), bool)
    valid = np.arange(n)[None, None, :] < cnt[:, :, None]
    h, r, j = np.nonzero(valid)
    out[h, r, idx[h, r, j]] = True
    return out[:, :, :n]


def compare_lists_banded(idx_g, cnt_g, P_ref, cu, alpha, sink_tokens=256, window_tokens=512, rows=None, block=128):
    """Lists from GPU scores vs lists from oracle scores: equal except for pairs whose oracle
    score lies within BAND (relative) of the threshold.  Returns (#mismatching pairs, #pairs in band)."""
    idx_r, cnt_r = oracle.threshold(P_ref, cu, alpha, block=block, sink_tokens=sink_tokens, window_tokens=window_tokens)
    mg, mr = lists_to_mask(idx_g, cnt_g), lists_to_mask(idx_r, cnt_r)
    cm = causal_mask(cu, block)
    if rows is not None:
        sel = np.zeros(cm.shape[0], bool); sel[list(rows)] = True
        cm &= sel[:, None]
    assert not np.any(mg & ~cm[None]) or rows is not None, "GPU list has a non-causal or out-of-range block"
    mx = np.where(cm[None], P_ref, -np.inf).max(axis=2, keepdims=True)
    thr = np.float32(alpha) * mx
    band = (np.abs(P_ref - thr) <= BAND * np.abs(thr)) & cm[None]
    diff = (mg != mr) & cm[None]
    assert not np.any(diff & ~band), f"{int((diff & ~band).sum())} list mismatches outside the near-threshold band"
    return int(diff.sum()), int(band.sum())


def compare_lists_same_outside_band(idx_a, cnt_a, idx_b, cnt_b, P, cm, alpha):
    """Two lists from the library's own paths (numpy): equal, except that pairs whose score P lies
    within BAND (relative) of alpha * row max may differ.  cm: causal mask [m, n].  Returns #differences."""
    ma, mb = lists_to_mask(idx_a, cnt_a), lists_to_mask(idx_b, cnt_b)
    thr = np.float32(alpha) * np.where(cm[None], P, -np.inf).max(axis=2, keepdims=True)
    band = (np.abs(P - thr) <= BAND * np.abs(thr)) & cm[None]
    diff = (ma != mb)
    assert not np.any(diff & ~band), f"{int((diff & ~band).sum())} differences outside the near-threshold band"
    return int(diff.sum())


def compare_O(O_gpu, O_ref, tok_sel=None):
    a = f32(O_gpu) if not isinstance(O_gpu, np.ndarray) else O_gpu
    if tok_sel is not None:
        a, O_ref = a[tok_sel], O_ref[tok_sel]
    err = np.abs(a - O_ref)
    assert np.isfinite(a).all()
    assert err.max() <= O_MAX_ABS, f"max-abs {err.max()}"
    assert err.mean() <= O_MEAN_ABS, f"mean-abs {err.mean()}"
    return float(err.max()), float(err.mean())


def row_tokens(cu, rows, block=128):
    m_total, n_max, ro = synth.layout(cu, block)
    toks = []
    for r in rows:
        s = int(np.searchsorted(ro, r, side="right") - 1)
        t0 = cu[s] + (r - ro[s]) * block
        toks.extend(range(t0, min(t0 + block, cu[s + 1])))
    return np.array(toks, np.int64)
