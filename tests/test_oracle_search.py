"""Pins for the oracle's block search (pattern discovery, Sec. 3.1-3.2, Eq. 1-4, Alg. 1).

Every expected value here comes from a closed form, a library routine (numpy mean / matmul,
scipy softmax / logsumexp) or an invariant, never from the oracle itself.
"""
import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
import synth


def _f64(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def _expected_map(Q, K, cu, block, tau):
    """P_I. = softmax_J( logsumexp_i tau q_i.kbar_J ): Eq. 1-4 with the max shifts cancelled
    algebraically (S'_IJ = sum_i exp(x_i - M_I)), built from library routines only."""
    Qf, Kf = _f64(Q), _f64(K)
    T, hq, d = Qf.shape
    hkv = Kf.shape[1]
    g = hq // hkv
    m_total, n_max, ro = synth.layout(cu, block)
    out = np.zeros((hq, m_total, n_max))
    for s in range(len(cu) - 1):
        a, b = cu[s], cu[s + 1]
        nb = ro[s + 1] - ro[s]
        for h in range(hq):
            kbar = np.stack([Kf[a + J * block:min(a + (J + 1) * block, b), h // g].mean(axis=0) for J in range(nb)])
            for I in range(nb):
                q = Qf[a + I * block:min(a + (I + 1) * block, b), h]
                x = tau * (q @ kbar[:I + 1].T)            # [queries, J]
                out[h, ro[s] + I, :I + 1] = softmax(logsumexp(x, axis=0))
    return out


def test_block_one_is_textbook_causal_softmax():
    # block = 1: the pooled key is the key, S = 1, so P is the causal row softmax of tau q.k.
    Q, K, _ = synth.random_qkv([24], hq=2, hkv=2, d=16, seed=1)
    P = oracle.block_search(Q, K, [0, 24], block=1, eps=0.0)
    for h in range(2):
        logits = (_f64(Q)[:, h] @ _f64(K)[:, h].T) / 4.0
        logits[np.triu_indices(24, 1)] = -np.inf
        np.testing.assert_allclose(P[h], softmax(logits, axis=1), rtol=2e-6, atol=1e-12)


def test_zero_queries_give_uniform_rows():
    Q, K, _ = synth.random_qkv([1024], hq=2, hkv=1, d=32, seed=2)
    Q[:] = 0
    P = oracle.block_search(Q, K, [0, 1024], eps=0.0)
    for I in range(8):
        np.testing.assert_allclose(P[:, I, :I + 1], 1.0 / (I + 1), rtol=1e-6)
        assert np.all(P[:, I, I + 1:] == 0.0)


def test_equal_keys_give_uniform_rows():
    Q, K, _ = synth.random_qkv([640], hq=2, hkv=2, d=32, seed=3)
    K[:] = K[0:1, 0:1, :]
    P = oracle.block_search(Q, K, [0, 640], eps=0.0)
    for I in range(5):
        np.testing.assert_allclose(P[:, I, :I + 1], 1.0 / (I + 1), rtol=1e-6)


@pytest.mark.parametrize("seqlens,hq,hkv,d,block", [
    ([512], 2, 1, 32, 128),
    ([300], 4, 2, 16, 128),          # ragged tail: last block holds 44 tokens
    ([256, 130, 64], 4, 2, 16, 64),  # packed batch, ragged middle sequence
    ([1024], 8, 2, 128, 128),
])
def test_matches_library_formulation(seqlens, hq, hkv, d, block):
    Q, K, _ = synth.random_qkv(seqlens, hq, hkv, d, seed=7, scale=1.5)
    cu = np.concatenate([[0], np.cumsum(seqlens)])
    tau = 0.37
    P = oracle.block_search(Q, K, cu, tau=tau, block=block, eps=0.0)
    np.testing.assert_allclose(P, _expected_map(Q, K, cu, block, tau), rtol=3e-6, atol=1e-30)


def test_default_scale_is_inverse_sqrt_head_dim():
    Q, K, _ = synth.random_qkv([384], 2, 1, 64, seed=8)
    np.testing.assert_array_equal(oracle.block_search(Q, K, [0, 384]),
                                  oracle.block_search(Q, K, [0, 384], tau=0.125))


def test_invariants_on_structured_input():
    w = synth.small("inv", [1536], hq=4, hkv=2, seed=5)
    Q, K, _ = synth.make_qkv(w)
    P = oracle.block_search(Q, K, w.cu_seqlens)
    n = 12
    assert P.shape == (4, n, n)
    assert np.all(P >= 0) and np.all(P <= 1)
    np.testing.assert_allclose(P.sum(axis=2), 1.0, atol=1e-5)
    assert np.all(P[:, np.triu_indices(n, 1)[0], np.triu_indices(n, 1)[1]] == 0)
    np.testing.assert_allclose(P[:, 0, 0], 1.0, atol=1e-6)


def test_dominant_block_gives_one_hot_row():
    # Scaling one block's keys along the query direction makes its pooled key dominate the row.
    Q, K, _ = synth.random_qkv([1024], 1, 1, 32, seed=9)
    Qf, Kf = _f64(Q), _f64(K)
    Qf[:] = np.abs(Qf)                     # every query has a positive overlap with the all-ones direction
    Kf[3 * 128:4 * 128] += 40.0
    P = oracle.block_search(synth.f32_to_bf16_bits(Qf.astype(np.float32)), synth.f32_to_bf16_bits(Kf.astype(np.float32)), [0, 1024])
    for I in range(3, 8):
        assert P[0, I, 3] > 1 - 1e-6


def test_heads_of_a_kv_group_permute_together():
    Q, K, _ = synth.random_qkv([768], 4, 2, 32, seed=10)
    P = oracle.block_search(Q, K, [0, 768])
    perm = [1, 0, 3, 2]                     # swaps inside each KV group
    P2 = oracle.block_search(np.ascontiguousarray(Q[:, perm]), K, [0, 768])
    np.testing.assert_array_equal(P2, P[perm])


def test_packed_sequences_are_independent():
    lens = [384, 200, 128]
    Q, K, _ = synth.random_qkv(lens, 2, 1, 32, seed=11)
    cu = np.concatenate([[0], np.cumsum(lens)])
    P = oracle.block_search(Q, K, cu)
    _, _, ro = synth.layout(cu)
    for s in range(3):
        Ps = oracle.block_search(np.ascontiguousarray(Q[cu[s]:cu[s + 1]]), np.ascontiguousarray(K[cu[s]:cu[s + 1]]), [0, lens[s]])
        nb = ro[s + 1] - ro[s]
        np.testing.assert_array_equal(P[:, ro[s]:ro[s + 1], :nb], Ps)
        assert np.all(P[:, ro[s]:ro[s + 1], nb:] == 0)


def test_row_subset_equals_full():
    Q, K, _ = synth.random_qkv([1280], 2, 1, 32, seed=12)
    P = oracle.block_search(Q, K, [0, 1280])
    part = oracle.block_search(Q, K, [0, 1280], rows=[9, 0, 4])
    for r in (9, 0, 4):
        np.testing.assert_array_equal(part[:, r], P[:, r])
    assert np.all(part[:, [1, 2, 3, 5, 6, 7, 8]] == 0)


def test_pooled_probe_lower_bounds_block_mass():
    # AM-GM (Sec. 3.1): exp(q.kbar) <= mean_t exp(q.k_t).  With identical queries in a tile the
    # un-normalised row is B*exp(tau q.kbar_J), so P_IJ / P_IK ratios are bounded through it;
    # here the inequality is checked directly on the oracle's map against per-key masses.
    Q, K, _ = synth.random_qkv([512], 1, 1, 16, seed=13)
    Q[:] = Q[0:1]                                        # one query vector everywhere
    tau = 0.25
    P = oracle.block_search(Q, K, [0, 512], tau=tau, eps=0.0)
    q = _f64(Q)[0, 0]
    mass = np.exp(tau * (_f64(K)[:, 0] @ q)).reshape(4, 128).mean(axis=1)   # AM per block
    probe = P[0, 3] / P[0, 3].sum()                      # proportional to exp(tau q.kbar_J) (GM per block)
    gm = np.exp(tau * (_f64(K)[:, 0].reshape(4, 128, 16).mean(axis=1) @ q))
    np.testing.assert_allclose(probe, gm / gm.sum(), rtol=1e-5)
    assert np.all(gm <= mass * (1 + 1e-12))


@pytest.mark.parametrize("seqlens,hq,hkv,d,block,eps", [
    ([24], 2, 2, 16, 1, 5.0),            # block = 1: P_IJ = exp(x_J - M) / (sum_K exp(x_K - M) + eps)
    ([512], 2, 1, 32, 128, 5.0),
    ([300, 130], 4, 2, 16, 64, 0.75),    # packed, ragged tails
])
def test_visible_eps_enters_the_denominator_after_the_rescale_to_the_row_max(seqlens, hq, hkv, d, block, eps):
    # Eq. 3-4 with an eps that is not a rounding no-op.  After the rescale to M_I = max_{i,J} x_iJ
    # the row's un-normalised entries are S'_IJ = sum_i exp(x_iJ - M_I) and their total is
    # T_I = sum_{i,J} exp(x_iJ - M_I) >= 1, so P_IJ = S'_IJ / (T_I + eps): the row sums to
    # T_I / (T_I + eps) and equals the eps-free softmax scaled by that factor.  An eps applied
    # before the rescale, to each pair's own sum, or to a differently referenced total fails this.
    Q, K, _ = synth.random_qkv(seqlens, hq, hkv, d, seed=21, scale=1.5)
    cu = np.concatenate([[0], np.cumsum(seqlens)])
    tau = 0.41
    P = oracle.block_search(Q, K, cu, tau=tau, block=block, eps=eps)
    Qf, Kf = _f64(Q), _f64(K)
    g = hq // hkv
    _, _, ro = synth.layout(cu, block)
    saw_visible = False
    for s in range(len(seqlens)):
        a, b = cu[s], cu[s + 1]
        nb = ro[s + 1] - ro[s]
        for h in range(hq):
            kbar = np.stack([Kf[a + J * block:min(a + (J + 1) * block, b), h // g].mean(axis=0) for J in range(nb)])
            for I in range(nb):
                q = Qf[a + I * block:min(a + (I + 1) * block, b), h]
                x = tau * (q @ kbar[:I + 1].T)
                T_I = np.exp(logsumexp(x) - x.max())            # library log-sum-exp over every (i, J) of the row
                assert T_I >= 1.0
                f = T_I / (T_I + eps)
                saw_visible |= f < 0.9
                row = P[h, ro[s] + I, :I + 1].astype(np.float64)
                np.testing.assert_allclose(row.sum(), f, rtol=2e-6)
                np.testing.assert_allclose(row, softmax(logsumexp(x, axis=0)) * f, rtol=3e-6, atol=1e-30)
    assert saw_visible
