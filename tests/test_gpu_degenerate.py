"""GPU parity on the method's degenerate inputs: all-equal scores (ties at the threshold), sequences
of one token, a threshold factor at and above 1, sink / window settings that keep everything, and
logits large enough to saturate the softmax.  Every stage against the oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_2603_06199_amd import binding as B
import synth

from gpu_util import LSE_ATOL, compare_lists_banded, compare_lists_exact, compare_O, compare_scores, dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _bits(x):
    return synth.f32_to_bf16_bits(np.ascontiguousarray(x, dtype=np.float32))


def _all_stages(Q, K, V, cu, hq, hkv, alpha, sink=256, window=512, lists_exact=False):
    plan = B.Plan(cu, hq, hkv)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    P_ref = oracle.block_search(Q, K, cu)
    P = plan.fp_block_search(dQ, dK)
    torch.cuda.synchronize()
    compare_scores(P.cpu().numpy(), P_ref, cu)
    idx_r, cnt_r = oracle.threshold(P_ref, cu, alpha, sink_tokens=sink, window_tokens=window)
    idx, cnt = plan.fp_threshold(torch.from_numpy(P_ref).cuda(), alpha, sink_tokens=sink, window_tokens=window)
    idx_g, cnt_g = plan.fp_threshold(P, alpha, sink_tokens=sink, window_tokens=window)
    idx_f, cnt_f = plan.fp_search_select(dQ, dK, alpha, sink_tokens=sink, window_tokens=window)
    torch.cuda.synchronize()
    compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)
    compare_lists_exact(idx_f.cpu().numpy(), cnt_f.cpu().numpy(), idx_g.cpu().numpy(), cnt_g.cpu().numpy())
    if lists_exact:
        compare_lists_exact(idx_g.cpu().numpy(), cnt_g.cpu().numpy(), idx_r, cnt_r)
    else:
        compare_lists_banded(idx_g.cpu().numpy(), cnt_g.cpu().numpy(), P_ref, cu, alpha, sink_tokens=sink, window_tokens=window)
    O_ref, lse_ref = oracle.sparse_prefill(Q, K, V, cu, idx_r, cnt_r)
    O, lse = plan.fp_sparse_prefill(dQ, dK, dV, torch.from_numpy(idx_r).cuda(), torch.from_numpy(cnt_r).cuda())
    Od_ref, lsed_ref = oracle.dense_prefill(Q, K, V, cu)
    Od, lsed = plan.fp_dense_prefill(dQ, dK, dV)
    torch.cuda.synchronize()
    compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    compare_O(Od, Od_ref)
    np.testing.assert_allclose(lsed.cpu().numpy(), lsed_ref, atol=LSE_ATOL, rtol=0)
    out = dict(P_ref=P_ref, idx_r=idx_r, cnt_r=cnt_r, O=O, Od=Od, lse=lse, lsed=lsed)
    plan.close()
    return out


def test_all_zero_queries_and_keys_give_uniform_scores_and_keep_everything():
    """Every logit is 0: a row's scores are all 1 / (I + 1), every block ties with the row maximum, so
    every causal block is kept for any alpha <= 1, and attention is the running mean of V."""
    rng = np.random.default_rng(0)
    cu = np.array([0, 1300, 1300 + 700], np.int32)
    hq, hkv, T = 4, 2, int(cu[-1])
    Q, K = _bits(np.zeros((T, hq, 128))), _bits(np.zeros((T, hkv, 128)))
    V = _bits(rng.standard_normal((T, hkv, 128)))
    print("\n[degenerate] zero Q and K", flush=True)
    for alpha in (0.12, 1.0):
        r = _all_stages(Q, K, V, cu, hq, hkv, alpha, lists_exact=True)
        m, n, ro = oracle.layout(cu)
        for s in range(2):
            for I in range(ro[s + 1] - ro[s]):
                assert np.all(r["cnt_r"][:, ro[s] + I] == I + 1)
                np.testing.assert_allclose(r["P_ref"][:, ro[s] + I, :I + 1], 1.0 / (I + 1), rtol=1e-6)   # the oracle stores fp32
        assert torch.equal(r["O"].view(torch.int16), r["Od"].view(torch.int16))
    Vf = synth.bf16_bits_to_f32(V)     # the running mean of V within each sequence, per KV head
    for s in range(2):
        a, b = int(cu[s]), int(cu[s + 1])
        mean = np.cumsum(Vf[a:b].astype(np.float64), axis=0) / np.arange(1, b - a + 1)[:, None, None]
        got = r["Od"][a:b].float().cpu().numpy()
        np.testing.assert_allclose(got, np.repeat(mean, hq // hkv, axis=1), atol=2e-2)


@pytest.mark.parametrize("seqlens", [[1], [1, 1, 1], [1, 129, 1, 128]])
def test_sequences_of_one_token(seqlens):
    rng = np.random.default_rng(1)
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    hq, hkv, T = 4, 1, int(cu[-1])
    Q, K, V = (_bits(rng.standard_normal((T, h, 128))) for h in (hq, hkv, hkv))
    print(f"\n[degenerate] seqlens {seqlens}", flush=True)
    r = _all_stages(Q, K, V, cu, hq, hkv, 0.12)
    # a one-token sequence attends to itself only: O = V (already bf16), lse = its own logit
    Vb = synth.bf16_bits_to_f32(V)
    for s, L in enumerate(seqlens):
        if L == 1:
            t = int(cu[s])
            np.testing.assert_array_equal(r["Od"][t].float().cpu().numpy(), np.repeat(Vb[t], hq // hkv, axis=0))


@pytest.mark.parametrize("alpha", [1.0, 1.5])
def test_threshold_factor_at_and_above_one(alpha):
    """alpha = 1 keeps the row's best block (and what is always kept); above 1 nothing but the sink and window blocks."""
    w = synth.small("alpha_high", [2100, 900], 8, 2, seed=31)
    Q, K, V = synth.make_qkv(w)
    print(f"\n[degenerate] alpha {alpha}", flush=True)
    r = _all_stages(Q, K, V, w.cu_seqlens, w.hq, w.hkv, alpha)
    m, n, ro = oracle.layout(w.cu_seqlens)
    for s in range(2):
        for I in range(ro[s + 1] - ro[s]):
            structural = len({0, 1} & set(range(I + 1)) | set(range(max(0, I - 3), I + 1)))
            c = r["cnt_r"][:, ro[s] + I]
            assert np.all(c >= structural) and np.all(c <= structural + (1 if alpha == 1.0 else 0))


def test_sink_and_window_that_cover_the_sequence_keep_everything():
    w = synth.small("keep_all", [1900, 333], 4, 2, seed=32)
    Q, K, V = synth.make_qkv(w)
    print("\n[degenerate] window covers everything", flush=True)
    for sink, window in ((0, 4096), (4096, 0)):
        r = _all_stages(Q, K, V, w.cu_seqlens, w.hq, w.hkv, 2.0, sink=sink, window=window, lists_exact=True)
        m, n, ro = oracle.layout(w.cu_seqlens)
        for s in range(2):
            for I in range(ro[s + 1] - ro[s]):
                assert np.all(r["cnt_r"][:, ro[s] + I] == I + 1)
        assert torch.equal(r["O"].view(torch.int16), r["Od"].view(torch.int16)) and torch.equal(r["lse"], r["lsed"])


@pytest.mark.parametrize("gain", [6.0, 16.0])
def test_logits_that_saturate_the_softmax(gain):
    """Queries scaled up until a row's attention sits on one or two keys and the block scores span
    hundreds of binary orders of magnitude: the running reference point of the attention kernel moves
    by large steps, most exponentials flush to zero, the search leaves its reference-free path."""
    rng = np.random.default_rng(2)
    cu = np.array([0, 2500], np.int32)
    hq, hkv, T = 4, 2, int(cu[-1])
    Q = _bits(gain * rng.standard_normal((T, hq, 128)))
    K = _bits(rng.standard_normal((T, hkv, 128)))
    V = _bits(rng.standard_normal((T, hkv, 128)))
    print(f"\n[degenerate] logits x{gain}", flush=True)
    _all_stages(Q, K, V, cu, hq, hkv, 0.12)
