"""Pins for the oracle's block-sparse (Sec. 3.5, Alg. 3) and full causal attention."""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import oracle
import synth

LOG2E = 1.4426950408889634


def _f64(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def _masked_attention(Q, K, V, tau, allow):
    """softmax over an explicit token-level boolean mask allow[h, t, u], library routines only."""
    Qf, Kf, Vf = _f64(Q), _f64(K), _f64(V)
    T, hq, d = Qf.shape
    g = hq // Kf.shape[1]
    O = np.zeros((T, hq, d))
    lse = np.zeros((hq, T))
    for h in range(hq):
        logits = tau * (Qf[:, h] @ Kf[:, h // g].T)
        logits[~allow[h]] = -np.inf
        O[:, h] = softmax(logits, axis=1) @ Vf[:, h // g]
        lse[h] = logsumexp(logits, axis=1) * LOG2E
    return O, lse


def _token_mask(cu, idx, cnt, hq, block):
    T = cu[-1]
    _, _, ro = synth.layout(cu, block)
    allow = np.zeros((hq, T, T), bool)
    for s in range(len(cu) - 1):
        for I in range(ro[s + 1] - ro[s]):
            t0, t1 = cu[s] + I * block, min(cu[s] + (I + 1) * block, cu[s + 1])
            for h in range(hq):
                for J in idx[h, ro[s] + I, :cnt[h, ro[s] + I]]:
                    u0, u1 = cu[s] + J * block, min(cu[s] + (J + 1) * block, cu[s + 1])
                    allow[h, t0:t1, u0:u1] = True
    allow &= np.tril(np.ones((T, T), bool))[None]
    return allow


@pytest.mark.parametrize("seqlens,hq,hkv,d,block", [
    ([256], 2, 1, 32, 64),
    ([200], 4, 2, 16, 64),             # ragged tail
    ([128, 70, 192], 4, 2, 16, 64),    # packed batch
])
def test_dense_matches_library_sdpa(seqlens, hq, hkv, d, block):
    Q, K, V = synth.random_qkv(seqlens, hq, hkv, d, seed=21, scale=1.3)
    cu = np.concatenate([[0], np.cumsum(seqlens)])
    tau = 0.3
    O, lse = oracle.dense_prefill(Q, K, V, cu, tau=tau, block=block)
    g = hq // hkv
    for s in range(len(seqlens)):
        sl = slice(cu[s], cu[s + 1])
        q = torch.from_numpy(_f64(Q)[sl]).permute(1, 0, 2)[None]
        k = torch.from_numpy(_f64(K)[sl]).permute(1, 0, 2).repeat_interleave(g, 0)[None]
        v = torch.from_numpy(_f64(V)[sl]).permute(1, 0, 2).repeat_interleave(g, 0)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=tau)[0].permute(1, 0, 2).numpy()
        np.testing.assert_allclose(O[sl], ref, rtol=1e-5, atol=2e-6)
    allow = np.zeros((hq, cu[-1], cu[-1]), bool)
    for s in range(len(seqlens)):
        allow[:, cu[s]:cu[s + 1], cu[s]:cu[s + 1]] = np.tril(np.ones((seqlens[s], seqlens[s]), bool))
    O2, lse2 = _masked_attention(Q, K, V, tau, allow)
    np.testing.assert_allclose(O, O2, rtol=1e-5, atol=2e-6)
    np.testing.assert_allclose(lse, lse2, rtol=1e-6, atol=1e-5)


@pytest.mark.parametrize("seqlens,density", [([512], 0.3), ([300, 200], 0.5), ([448], 0.05)])
def test_sparse_matches_explicit_token_mask(seqlens, density):
    hq, hkv, d, block = 4, 2, 16, 64
    Q, K, V = synth.random_qkv(seqlens, hq, hkv, d, seed=22, scale=1.3)
    cu = np.concatenate([[0], np.cumsum(seqlens)])
    m_total, n_max, ro = synth.layout(cu, block)
    g = np.random.default_rng(5)
    idx = np.full((hq, m_total, n_max), -7, np.int32)
    cnt = np.zeros((hq, m_total), np.int32)
    for s in range(len(seqlens)):
        for I in range(ro[s + 1] - ro[s]):
            for h in range(hq):
                keep = np.nonzero((g.random(I + 1) < density) | (np.arange(I + 1) == I))[0]   # diagonal always there
                idx[h, ro[s] + I, :keep.size] = keep
                cnt[h, ro[s] + I] = keep.size
    O, lse = oracle.sparse_prefill(Q, K, V, cu, idx, cnt, tau=0.3, block=block)
    O2, lse2 = _masked_attention(Q, K, V, 0.3, _token_mask(cu, idx, cnt, hq, block))
    np.testing.assert_allclose(O, O2, rtol=1e-5, atol=2e-6)
    np.testing.assert_allclose(lse, lse2, rtol=1e-6, atol=1e-5)


def test_all_causal_blocks_listed_equals_dense():
    # alpha <= 0 keeps every causal block (threshold disabled), so sparse == dense.
    w = synth.small("eq", [640, 200], hq=4, hkv=2, seed=3, head_dim=32)
    Q, K, V = synth.make_qkv(w)
    cu = w.cu_seqlens
    P = oracle.block_search(Q, K, cu)
    idx, cnt = oracle.threshold(P, cu, 0.0)
    Os, ls = oracle.sparse_prefill(Q, K, V, cu, idx, cnt)
    Od, ld = oracle.dense_prefill(Q, K, V, cu)
    np.testing.assert_allclose(Os, Od, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(ls, ld, rtol=1e-6, atol=1e-6)


def test_single_block_list_is_plain_softmax_over_that_block():
    hq, d, block = 1, 16, 64
    Q, K, V = synth.random_qkv([256], hq, 1, d, seed=23)
    idx = np.zeros((1, 4, 4), np.int32)
    cnt = np.ones((1, 4), np.int32)
    idx[0, :, 0] = [0, 0, 1, 2]                    # rows 1..3 attend to one strictly-past block
    O, _ = oracle.sparse_prefill(Q, K, V, [0, 256], idx, cnt, tau=0.25, block=block)
    Qf, Kf, Vf = _f64(Q)[:, 0], _f64(K)[:, 0], _f64(V)[:, 0]
    for I, J in ((1, 0), (2, 1), (3, 2)):
        p = softmax(0.25 * Qf[I * 64:(I + 1) * 64] @ Kf[J * 64:(J + 1) * 64].T, axis=1)
        np.testing.assert_allclose(O[I * 64:(I + 1) * 64, 0], p @ Vf[J * 64:(J + 1) * 64], rtol=1e-5, atol=2e-6)


def test_log_sum_exp_merge_identity():
    # Online softmax (Alg. 3): attention over a disjoint union of block lists is the
    # log-sum-exp-weighted mix of the attentions over the parts.
    hq, d, block, n = 2, 16, 64, 6
    Q, K, V = synth.random_qkv([n * block], hq, 1, d, seed=24)
    cu = [0, n * block]
    full_idx = np.tile(np.arange(n, dtype=np.int32), (hq, n, 1))
    A = np.zeros_like(full_idx); B = np.zeros_like(full_idx)
    ca = np.zeros((hq, n), np.int32); cb = np.zeros((hq, n), np.int32); cf = np.zeros((hq, n), np.int32)
    for I in range(n):
        js = np.arange(I + 1)
        a, b = js[js % 2 == I % 2], js[js % 2 != I % 2]        # a holds the diagonal
        A[:, I, :a.size] = a; ca[:, I] = a.size
        B[:, I, :b.size] = b; cb[:, I] = b.size
        cf[:, I] = I + 1
    Of, lf = oracle.sparse_prefill(Q, K, V, cu, full_idx, cf, block=block)
    Oa, la = oracle.sparse_prefill(Q, K, V, cu, A, ca, block=block)
    Ob, lb = oracle.sparse_prefill(Q, K, V, cu, B, cb, block=block)
    rows = slice(block, None)                                   # row 0 has an empty b part
    wa = 1.0 / (1.0 + np.exp2(lb.T[rows] - la.T[rows]))
    mix = wa[..., None] * Oa[rows] + (1 - wa)[..., None] * Ob[rows]
    np.testing.assert_allclose(mix, Of[rows], rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(np.logaddexp2(la, lb)[:, block:], lf[:, block:], rtol=1e-6, atol=1e-5)


def test_heads_of_a_kv_group_permute_together():
    w = synth.small("perm", [512], hq=4, hkv=2, seed=4, head_dim=32)
    Q, K, V = synth.make_qkv(w)
    cu = w.cu_seqlens
    idx, cnt = oracle.threshold(oracle.block_search(Q, K, cu), cu, 0.12)
    O, _ = oracle.sparse_prefill(Q, K, V, cu, idx, cnt)
    perm = [1, 0, 3, 2]
    Qp = np.ascontiguousarray(Q[:, perm])
    idxp, cntp = oracle.threshold(oracle.block_search(Qp, K, cu), cu, 0.12)
    assert np.array_equal(idxp, idx[perm]) and np.array_equal(cntp, cnt[perm])
    Op, _ = oracle.sparse_prefill(Qp, K, V, cu, idxp, cntp)
    np.testing.assert_array_equal(Op, O[:, perm])


def test_row_subset_equals_full():
    Q, K, V = synth.random_qkv([640], 2, 1, 16, seed=25)
    O, l = oracle.dense_prefill(Q, K, V, [0, 640])
    Op, lp = oracle.dense_prefill(Q, K, V, [0, 640], rows=[4, 1])
    for r in (4, 1):
        np.testing.assert_array_equal(Op[r * 128:(r + 1) * 128], O[r * 128:(r + 1) * 128])
        np.testing.assert_array_equal(lp[:, r * 128:(r + 1) * 128], l[:, r * 128:(r + 1) * 128])
    assert np.all(Op[:128] == 0) and np.all(Op[256:512] == 0)


def test_empty_list_gives_zero_output_and_minus_infinite_lse():
    """Not a paper case: a query whose list holds no visible key.  The reading taken is O = 0 and
    lse = -inf (the log of an empty sum); every other row is unaffected."""
    Q, K, V = synth.random_qkv([300], 2, 1, 128, seed=5)
    cu = [0, 300]
    idx, cnt = oracle.threshold(oracle.block_search(Q, K, cu), cu, 0.0)
    O_all, lse_all = oracle.sparse_prefill(Q, K, V, cu, idx, cnt)
    cnt2 = cnt.copy()
    cnt2[:, 1] = 0
    O, lse = oracle.sparse_prefill(Q, K, V, cu, idx, cnt2)
    assert not O[128:256].any() and np.all(np.isneginf(lse[:, 128:256]))
    keep = np.r_[0:128, 256:300]
    np.testing.assert_array_equal(O[keep], O_all[keep])
    np.testing.assert_array_equal(lse[:, keep], lse_all[:, keep])
