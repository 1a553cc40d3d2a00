"""Pins for the oracle-side comparison variants (other block scorings, Top-k / Top-p selection).

Each check is against something other than the function itself: a closed form, a brute-force
restatement on tiny inputs, or the independently written C oracle where the definitions coincide."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle
from oracle import variants as V
import synth


def _bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, np.float32))


def _rand_qk(T, hq, hkv, seed, d=128):
    rng = np.random.default_rng(seed)
    return _bits(rng.standard_normal((T, hq, d))), _bits(rng.standard_normal((T, hkv, d)))


def test_method2_rows_are_distributions_over_the_causal_blocks():
    Q, K = _rand_qk(700, 4, 2, 0)
    cu = [0, 300, 700]
    P = V.method2_scores(Q, K, cu)
    m, n, ro = oracle.layout(cu)
    for s in range(2):
        for I in range(ro[s + 1] - ro[s]):
            row = P[:, ro[s] + I]
            np.testing.assert_allclose(row[:, :I + 1].sum(-1), 1.0, rtol=1e-6)
            assert not row[:, I + 1:].any()
    P1 = V.method1_scores(Q, K, cu)
    np.testing.assert_allclose(P1.sum(-1), 1.0, rtol=1e-6)


def test_identical_queries_in_a_block_make_the_three_methods_agree():
    """If every query of a block is the same vector, per-query softmax, pooled-query softmax and the
    max / sum-of-exponentials reduction of Eq. 1-4 all reduce to softmax_J(tau q . kbar_J)."""
    rng = np.random.default_rng(1)
    T, hq, hkv, d = 512, 4, 2, 128
    qrow = rng.standard_normal((4, hq, d)).astype(np.float32)
    Q = _bits(np.repeat(qrow, 128, axis=0))
    K = _bits(rng.standard_normal((T, hkv, d)))
    cu = [0, T]
    P1, P2 = V.method1_scores(Q, K, cu), V.method2_scores(Q, K, cu)
    P3 = oracle.block_search(Q, K, cu)
    np.testing.assert_allclose(P1, P2, rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(P3, P2, rtol=1e-5, atol=1e-9)
    # and the common value is the plain softmax over pooled-key logits
    kf = synth.bf16_bits_to_f32(K).astype(np.float64).reshape(4, 128, hkv, d).mean(1)
    qf = synth.bf16_bits_to_f32(Q).astype(np.float64)[::128]
    for h in range(hq):
        for I in range(4):
            ref = softmax(qf[I, h] @ kf[:I + 1, h // 2].T / np.sqrt(d))
            np.testing.assert_allclose(P2[h, I, :I + 1], ref, rtol=1e-6)


def test_block_size_one_is_token_level_attention():
    Q, K = _rand_qk(37, 2, 1, 2, d=16)
    P2 = V.method2_scores(Q, K, [0, 37], block=1)
    P1 = V.method1_scores(Q, K, [0, 37], block=1)
    q = synth.bf16_bits_to_f32(Q).astype(np.float64)
    k = synth.bf16_bits_to_f32(K).astype(np.float64)
    for h in range(2):
        logits = q[:, h] @ k[:, 0].T / 4.0
        for i in range(37):
            ref = softmax(logits[i, :i + 1])
            np.testing.assert_allclose(P2[h, i, :i + 1], ref, rtol=1e-6)
    np.testing.assert_allclose(P1, P2, rtol=1e-6, atol=1e-12)


def test_pooled_logit_never_exceeds_the_blocks_log_mean_exp():
    """Sec. 3.1: exp(q . kbar) is the geometric mean of the block's exp(q . k_i), hence at most their
    arithmetic mean.  Checked on the unnormalised quantities the scores are built from."""
    rng = np.random.default_rng(3)
    q = rng.standard_normal(64)
    k = rng.standard_normal((128, 64))
    x = k @ q
    assert np.exp(q @ k.mean(0)) <= np.exp(x).mean() * (1 + 1e-12)


def _random_scores(hq, cu, seed):
    m, n, ro = oracle.layout(cu)
    rng = np.random.default_rng(seed)
    P = rng.random((hq, m, n)).astype(np.float32) + 1e-3
    for s in range(len(cu) - 1):
        for I in range(ro[s + 1] - ro[s]):
            P[:, ro[s] + I, I + 1:] = 0
        P[:, ro[s]:ro[s + 1], ro[s + 1] - ro[s]:] = 0
    return P, m, n, ro


def test_topk_brute_force():
    cu = [0, 128 * 9, 128 * 9 + 128 * 5 - 17]
    P, m, n, ro = _random_scores(3, cu, 4)
    for k in (1, 3, 100):
        idx, cnt = V.select_topk(P, cu, k)
        for h in range(3):
            for s in range(2):
                for I in range(ro[s + 1] - ro[s]):
                    r = ro[s] + I
                    js = idx[h, r, :cnt[h, r]]
                    assert cnt[h, r] == min(k, I + 1)
                    assert np.all(np.diff(js) > 0) and js.max() <= I
                    assert np.all(idx[h, r, cnt[h, r]:] == n)
                    dropped = np.setdiff1d(np.arange(I + 1), js)
                    if dropped.size:
                        assert P[h, r, js].min() >= P[h, r, dropped].max()


def test_topp_brute_force_minimal_prefix():
    cu = [0, 128 * 12]
    P, m, n, ro = _random_scores(2, cu, 5)
    for p in (0.3, 0.9, 1.0):
        idx, cnt = V.select_topp(P, cu, p)
        for h in range(2):
            for I in range(12):
                js = idx[h, I, :cnt[h, I]]
                row = P[h, I, :I + 1].astype(np.float64)
                kept = row[js]
                assert kept.sum() >= p * row.sum() * (1 - 1e-9)
                assert kept.sum() - kept.min() < p * row.sum()          # nothing to spare
                dropped = np.setdiff1d(np.arange(I + 1), js)
                if dropped.size:
                    assert kept.min() >= row[dropped].max()
        if p == 1.0:
            assert np.array_equal(cnt[0], np.arange(1, 13))


def test_structural_blocks_match_the_c_oracle():
    """With nothing selected by score (k = 0) only sink and window blocks remain: the same lists the
    C oracle's Alg. 2 gives when the threshold is above every score."""
    cu = [0, 128 * 11 + 5, 128 * 11 + 5 + 300]
    P, m, n, ro = _random_scores(2, cu, 6)
    for sink, win in ((256, 512), (100, 129), (0, 128)):
        idx, cnt = V.select_topk(P, cu, 0, sink_tokens=sink, window_tokens=win)
        idx_r, cnt_r = oracle.threshold(P, cu, 2.0, sink_tokens=sink, window_tokens=win)
        assert np.array_equal(cnt, cnt_r)
        assert np.array_equal(idx, idx_r)


def test_density_and_overlap_closed_forms():
    cu = [0, 128 * 4]
    idx = np.full((1, 4, 4), 4, np.int32)
    cnt = np.zeros((1, 4), np.int32)
    for I in range(4):
        idx[0, I, :I + 1] = np.arange(I + 1)
        cnt[0, I] = I + 1
    assert V.density(cnt, cu) == 1.0
    diag_idx = np.full((1, 4, 4), 4, np.int32)
    diag_idx[0, :, 0] = np.arange(4)
    diag_cnt = np.ones((1, 4), np.int32)
    assert V.density(diag_cnt, cu) == pytest.approx(4 / 10)
    jac, rec = V.overlap(diag_idx, diag_cnt, idx, cnt)
    assert jac == pytest.approx(0.4) and rec == pytest.approx(0.4)
    jac, rec = V.overlap(idx, cnt, diag_idx, diag_cnt)
    assert jac == pytest.approx(0.4) and rec == 1.0


def test_attention_mass_against_explicit_softmax():
    Q, K = _rand_qk(300, 2, 1, 7, d=32)
    cu = [0, 300]
    m, n, ro = oracle.layout(cu)
    full_idx, full_cnt = V.select_topk(np.ones((2, m, n), np.float32), cu, n)
    assert V.attention_mass(Q, K, cu, full_idx, full_cnt) == pytest.approx(1.0, abs=1e-12)
    # window of one block: mass = share of the softmax on keys of the query's own block
    idx, cnt = V.select_topk(np.ones((2, m, n), np.float32), cu, 0, window_tokens=128)
    q = synth.bf16_bits_to_f32(Q).astype(np.float64)
    k = synth.bf16_bits_to_f32(K).astype(np.float64)
    tot = 0.0
    for h in range(2):
        for i in range(300):
            w = softmax(q[i, h] @ k[:i + 1, 0].T / np.sqrt(32))
            tot += w[(i // 128) * 128:].sum()
    assert V.attention_mass(Q, K, cu, idx, cnt) == pytest.approx(tot / 600, rel=1e-9)
