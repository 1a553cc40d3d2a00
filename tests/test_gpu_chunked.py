"""GPU parity for chunked prefill (queries = the last tokens of a longer key sequence): every
stage against the oracle's chunked form on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_2603_06199_amd import binding as B
import synth

from gpu_util import LSE_ATOL, compare_lists_exact, compare_O, dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CASES = {
    "aligned": dict(kv=[1024], q=[384], hq=4, hkv=2),
    "ragged_end": dict(kv=[1000], q=[360], hq=4, hkv=1),
    "one_query_block_long_prefix": dict(kv=[128 * 41], q=[128], hq=8, hkv=2),
    "short_chunk": dict(kv=[128 * 9 + 5], q=[5], hq=4, hkv=4),
    "varlen_mixed": dict(kv=[640, 900, 256, 128 * 70 + 77], q=[128, 900, 128, 128 * 6 + 77], hq=8, hkv=2),
}


@pytest.fixture(scope="module", params=list(CASES), ids=list(CASES))
def case(request):
    c = CASES[request.param]
    rng = np.random.default_rng(11)
    Tk, Tq = sum(c["kv"]), sum(c["q"])
    cuk = np.concatenate([[0], np.cumsum(c["kv"])]).astype(np.int32)
    cuq = np.concatenate([[0], np.cumsum(c["q"])]).astype(np.int32)
    hq, hkv = c["hq"], c["hkv"]
    # a shared direction on a few key tokens so that some blocks stand out and the lists are not trivial
    u = rng.standard_normal(128).astype(np.float32); u /= np.linalg.norm(u)
    Kf = rng.standard_normal((Tk, hkv, 128)).astype(np.float32)
    hot = rng.choice(Tk, size=max(2, Tk // 300), replace=False)
    for t in hot:
        lo = (t // 128) * 128
        Kf[lo:lo + 128] += 3.0 * u
    Qf = rng.standard_normal((Tq, hq, 128)).astype(np.float32) + 1.5 * u
    Q, K = synth.f32_to_bf16_bits(Qf), synth.f32_to_bf16_bits(Kf)
    V = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hkv, 128)).astype(np.float32))
    print(f"\n[case] chunked {request.param} kv={c['kv']} q={c['q']} hq={hq} hkv={hkv}", flush=True)
    plan = B.Plan(cuq, hq, hkv, cu_seqlens_k=cuk)
    P_ref = oracle.block_search(Q, K, cuq, cu_seqlens_k=cuk)
    yield dict(cuq=cuq, cuk=cuk, Q=Q, K=K, V=V, dQ=dev(Q), dK=dev(K), dV=dev(V), plan=plan, P_ref=P_ref, hq=hq)
    plan.close()


def _causal(case):
    m, n, ro = oracle.layout(case["cuq"], cu_seqlens_k=case["cuk"])
    mask = np.zeros((m, n), bool)
    for s in range(len(ro) - 1):
        pb = ((case["cuk"][s + 1] - case["cuk"][s]) - (case["cuq"][s + 1] - case["cuq"][s])) // 128
        for I in range(ro[s + 1] - ro[s]):
            mask[ro[s] + I, :I + pb + 1] = True
    return mask


def _own(case):
    """Columns of each row that belong to its own sequence (J < the sequence's key blocks)."""
    m, n, ro = oracle.layout(case["cuq"], cu_seqlens_k=case["cuk"])
    own = np.zeros((m, n), bool)
    for s in range(len(ro) - 1):
        own[ro[s]:ro[s + 1], :-(-(case["cuk"][s + 1] - case["cuk"][s]) // 128)] = True
    return own


def test_scores(case):
    plan = case["plan"]
    P = torch.full((case["hq"], plan.m_total, plan.n_max), float("nan"), dtype=torch.float32, device="cuda")
    plan.fp_block_search(case["dQ"], case["dK"], P)
    torch.cuda.synchronize()
    P = P.cpu().numpy()
    cm, own = _causal(case), _own(case)
    assert not P[:, own & ~cm].any()             # zeros above the diagonal, up to the sequence's last block
    assert np.isnan(P[:, ~own]).all()            # columns of longer sequences are not written
    np.testing.assert_allclose(P[:, cm], case["P_ref"][:, cm], rtol=5e-4, atol=1e-30)


def test_threshold_on_oracle_scores_is_exact(case):
    for alpha, sink, win in ((0.2, 256, 512), (0.5, 0, 128)):
        idx_r, cnt_r = oracle.threshold(case["P_ref"], case["cuq"], alpha, sink_tokens=sink, window_tokens=win,
                                        cu_seqlens_k=case["cuk"])
        idx, cnt = case["plan"].fp_threshold(torch.from_numpy(case["P_ref"]).cuda(), alpha, sink_tokens=sink,
                                             window_tokens=win)
        torch.cuda.synchronize()
        compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)


def test_lists_from_gpu_scores_and_the_one_pass_entry_point(case):
    alpha = 0.2
    plan = case["plan"]
    idx, cnt = plan.fp_threshold(plan.fp_block_search(case["dQ"], case["dK"]), alpha)
    idx_f, cnt_f = plan.fp_search_select(case["dQ"], case["dK"], alpha)
    torch.cuda.synchronize()
    compare_lists_exact(idx_f.cpu().numpy(), cnt_f.cpu().numpy(), idx.cpu().numpy(), cnt.cpu().numpy())
    # against the oracle: equal except pairs whose score is within 1e-3 (relative) of the threshold
    idx_r, cnt_r = oracle.threshold(case["P_ref"], case["cuq"], alpha, cu_seqlens_k=case["cuk"])
    from gpu_util import BAND, lists_to_mask
    mg, mr = lists_to_mask(idx.cpu().numpy(), cnt.cpu().numpy()), lists_to_mask(idx_r, cnt_r)
    cm = _causal(case)
    assert not np.any(mg & ~cm[None])
    thr = np.float32(alpha) * np.where(cm[None], case["P_ref"], -np.inf).max(axis=2, keepdims=True)
    band = (np.abs(case["P_ref"] - thr) <= BAND * np.abs(thr)) & cm[None]
    assert not np.any((mg != mr) & ~band)


def test_sparse_and_dense_attention(case):
    cuq, cuk = case["cuq"], case["cuk"]
    idx_r, cnt_r = oracle.threshold(case["P_ref"], cuq, 0.2, cu_seqlens_k=cuk)
    O_ref, lse_ref = oracle.sparse_prefill(case["Q"], case["K"], case["V"], cuq, idx_r, cnt_r, cu_seqlens_k=cuk)
    O, lse = case["plan"].fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], torch.from_numpy(idx_r).cuda(),
                                            torch.from_numpy(cnt_r).cuda())
    torch.cuda.synchronize()
    compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    Od_ref, lsed_ref = oracle.dense_prefill(case["Q"], case["K"], case["V"], cuq, cu_seqlens_k=cuk)
    Od, lsed = case["plan"].fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    torch.cuda.synchronize()
    compare_O(Od, Od_ref)
    np.testing.assert_allclose(lsed.cpu().numpy(), lsed_ref, atol=LSE_ATOL, rtol=0)


def test_chunk_equals_the_tail_of_a_plain_prefill_bitwise(case):
    """Property that needs no oracle: running the whole sequences as a plain prefill and keeping the
    chunk's tokens gives the same dense output bit for bit (same kernel, same tiles, same order)."""
    cuq, cuk = case["cuq"], case["cuk"]
    hq = case["hq"]
    rng = np.random.default_rng(5)
    Tk = int(cuk[-1])
    Qfull = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hq, 128)).astype(np.float32))
    sel = np.concatenate([np.arange(cuk[s + 1] - (cuq[s + 1] - cuq[s]), cuk[s + 1]) for s in range(len(cuq) - 1)])
    Qfull[sel] = case["Q"]
    full = B.Plan(cuk, hq, case["K"].shape[1])
    Of, lf = full.fp_dense_prefill(dev(Qfull), case["dK"], case["dV"])
    Oc, lc = case["plan"].fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    torch.cuda.synchronize()
    st = torch.from_numpy(sel).cuda()
    assert torch.equal(Of[st], Oc) and torch.equal(lf[:, st], lc)
    full.close()


def test_largest_row_next_to_a_small_plan():
    """One query block against 4096 key blocks (the most a sequence may have), with a small plan
    created afterwards: kernel limits are per library, not per plan, so the large plan still runs."""
    rng = np.random.default_rng(3)
    Tk, hq, hkv = 4096 * 128, 2, 1
    u = rng.standard_normal(128).astype(np.float32); u /= np.linalg.norm(u)
    Kf = rng.standard_normal((Tk, hkv, 128)).astype(np.float32)
    for j in rng.choice(4096, size=12, replace=False):      # a dozen key blocks that stand out
        Kf[j * 128:(j + 1) * 128] += 4.0 * u
    K = synth.f32_to_bf16_bits(Kf)
    V = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hkv, 128)).astype(np.float32))
    Q = synth.f32_to_bf16_bits(rng.standard_normal((128, hq, 128)).astype(np.float32) + 6.0 * u)
    cuq, cuk = [0, 128], [0, Tk]
    big = B.Plan(cuq, hq, hkv, cu_seqlens_k=cuk)
    small = B.Plan([0, 256], hq, hkv)
    assert (big.m_total, big.n_max) == (1, 4096)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    P = big.fp_block_search(dQ, dK)
    idx, cnt = big.fp_threshold(P, 0.5)
    idx_f, cnt_f = big.fp_search_select(dQ, dK, 0.5)
    torch.cuda.synchronize()
    P_ref = oracle.block_search(Q, K, cuq, cu_seqlens_k=cuk)
    np.testing.assert_allclose(P.cpu().numpy(), P_ref, rtol=5e-4, atol=1e-30)
    idx_r, cnt_r = oracle.threshold(P.cpu().numpy(), cuq, 0.5, cu_seqlens_k=cuk)
    compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)
    # a row of 128 tiles: the one-pass entry point scores it on the hi plane and re-scores what matters,
    # so its list may differ from the two-call one only on pairs within the near-threshold band
    from gpu_util import compare_lists_same_outside_band
    nd = compare_lists_same_outside_band(idx_f.cpu().numpy(), cnt_f.cpu().numpy(), idx_r, cnt_r, P_ref,
                                         np.ones((1, 4096), bool), 0.5)
    print(f"one-pass vs two-call lists on the 4096-block row: {nd} differing pairs")
    O, lse = big.fp_sparse_prefill(dQ, dK, dV, idx, cnt)
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.sparse_prefill(Q, K, V, cuq, idx_r, cnt_r, cu_seqlens_k=cuk)
    compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    print(f"4096-block row: kept {int(cnt_r.sum())} of {hq * 4096} pairs")
    big.close(); small.close()
