"""GPU parity at block sizes 64 and 256 (head dimension 128): the paper fixes the block at 128, a
serving integration may not.  Every entry point against the oracle at the same block size, through
the C ABI: a 64-query block gets a two-wave attention workgroup over 32-key tiles, a 256-query block
takes two workgroups per row in the attention kernel and one head per workgroup in the search."""
import numpy as np
import pytest

import oracle
from paper_2603_06199_amd import binding as B
import synth

from gpu_util import LSE_ATOL, compare_lists_banded, compare_lists_exact, compare_O, compare_scores, dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CASES = [
    # name, seqlens, hq, hkv
    ("tiny_ragged", [5], 2, 2),
    ("one_block_and_a_bit", [300], 4, 1),
    ("several_tiles", [1536], 8, 2),
    ("packed_ragged", [640, 77, 1300, 128, 64, 257], 8, 4),
    ("g8_long_row", [9000], 8, 1),         # more than 32 key blocks at either block size
    ("g3_odd_group", [1100, 300], 6, 2),
]


@pytest.fixture(scope="module", params=[(b, c) for b in (64, 256) for c in CASES],
                ids=[f"b{b}-{c[0]}" for b in (64, 256) for c in CASES])
def case(request):
    blk, (name, seqlens, hq, hkv) = request.param
    w = synth.small(name, seqlens, hq, hkv, seed=23)
    Q, K, V = synth.make_qkv(w)
    cu = w.cu_seqlens
    print(f"\n[case] block {blk} {name} seqlens={seqlens} hq={hq} hkv={hkv}", flush=True)
    plan = B.Plan(cu, hq, hkv, block=blk)
    assert (plan.m_total, plan.n_max) == oracle.layout(cu, block=blk)[:2]
    out = dict(w=w, blk=blk, cu=cu, Q=Q, K=K, V=V, plan=plan, dQ=dev(Q), dK=dev(K), dV=dev(V))
    out["P_ref"] = oracle.block_search(Q, K, cu, block=blk)
    yield out
    plan.close()


def test_scores_and_lists(case):
    plan, w, cu, blk = case["plan"], case["w"], case["cu"], case["blk"]
    P = plan.fp_block_search(case["dQ"], case["dK"])
    torch.cuda.synchronize()
    compare_scores(P.cpu().numpy(), case["P_ref"], cu, block=blk)
    for alpha, sink, win in ((w.alpha, 256, 512), (0.3, 100, 200), (0.0, 0, 0)):
        idx_r, cnt_r = oracle.threshold(case["P_ref"], cu, alpha, block=blk, sink_tokens=sink, window_tokens=win)
        idx, cnt = plan.fp_threshold(torch.from_numpy(case["P_ref"]).cuda(), alpha, sink_tokens=sink, window_tokens=win)
        idx2, cnt2 = plan.fp_threshold(P, alpha, sink_tokens=sink, window_tokens=win)
        idx_f, cnt_f = plan.fp_search_select(case["dQ"], case["dK"], alpha, sink_tokens=sink, window_tokens=win)
        torch.cuda.synchronize()
        compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)
        compare_lists_banded(idx2.cpu().numpy(), cnt2.cpu().numpy(), case["P_ref"], cu, alpha, sink_tokens=sink,
                             window_tokens=win, block=blk)
        compare_lists_exact(idx_f.cpu().numpy(), cnt_f.cpu().numpy(), idx2.cpu().numpy(), cnt2.cpu().numpy())


def test_attention(case):
    w, cu, blk = case["w"], case["cu"], case["blk"]
    idx_r, cnt_r = oracle.threshold(case["P_ref"], cu, w.alpha, block=blk)
    O_ref, lse_ref = oracle.sparse_prefill(case["Q"], case["K"], case["V"], cu, idx_r, cnt_r, block=blk)
    O, lse = case["plan"].fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], torch.from_numpy(idx_r).cuda(),
                                            torch.from_numpy(cnt_r).cuda())
    torch.cuda.synchronize()
    compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    Od_ref, lsed_ref = oracle.dense_prefill(case["Q"], case["K"], case["V"], cu, block=blk)
    Od, lsed = case["plan"].fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    torch.cuda.synchronize()
    compare_O(Od, Od_ref)
    np.testing.assert_allclose(lsed.cpu().numpy(), lsed_ref, atol=LSE_ATOL, rtol=0)
    idx_a, cnt_a = oracle.threshold(case["P_ref"], cu, 0.0, block=blk)
    Oa, lsea = case["plan"].fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], torch.from_numpy(idx_a).cuda(),
                                              torch.from_numpy(cnt_a).cuda())
    torch.cuda.synchronize()
    assert torch.equal(Oa.view(torch.int16), Od.view(torch.int16)) and torch.equal(lsea, lsed)


def test_random_lists_and_empty_rows(case):
    cu, hq, blk = case["cu"], case["w"].hq, case["blk"]
    idx, cnt = synth.forced_density_lists(cu, hq, 0.4, seed=3, sink_blocks=0, window_blocks=0, block=blk)
    cnt[:, ::5] = 0
    O_ref, lse_ref = oracle.sparse_prefill(case["Q"], case["K"], case["V"], cu, idx, cnt, block=blk)
    O, lse = case["plan"].fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], torch.from_numpy(idx).cuda(),
                                            torch.from_numpy(cnt).cuda())
    torch.cuda.synchronize()
    compare_O(O, O_ref)
    got, fin = lse.cpu().numpy(), np.isfinite(lse_ref)
    np.testing.assert_allclose(got[fin], lse_ref[fin], atol=LSE_ATOL, rtol=0)
    assert np.all(np.isneginf(got[~fin]))


@pytest.mark.parametrize("blk", [64, 256])
def test_chunked_prefill(blk):
    rng = np.random.default_rng(40 + blk)
    kv, q, hq, hkv = [blk * 9 + 60, 5 * blk], [blk * 2 + 60, blk], 4, 2
    cuk = np.concatenate([[0], np.cumsum(kv)]).astype(np.int32)
    cuq = np.concatenate([[0], np.cumsum(q)]).astype(np.int32)
    u = rng.standard_normal(128).astype(np.float32); u /= np.linalg.norm(u)
    Kf = rng.standard_normal((cuk[-1], hkv, 128)).astype(np.float32)
    Kf[2 * blk:3 * blk] += 3.0 * u
    Q = synth.f32_to_bf16_bits(rng.standard_normal((cuq[-1], hq, 128)).astype(np.float32) + 1.5 * u)
    K = synth.f32_to_bf16_bits(Kf)
    V = synth.f32_to_bf16_bits(rng.standard_normal((cuk[-1], hkv, 128)).astype(np.float32))
    plan = B.Plan(cuq, hq, hkv, block=blk, cu_seqlens_k=cuk)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    P_ref = oracle.block_search(Q, K, cuq, block=blk, cu_seqlens_k=cuk)
    P = plan.fp_block_search(dQ, dK)
    torch.cuda.synchronize()
    m, n, ro = oracle.layout(cuq, block=blk, cu_seqlens_k=cuk)
    cm = np.zeros((m, n), bool)
    for s in range(2):
        pb = (kv[s] - q[s]) // blk
        for I in range(ro[s + 1] - ro[s]):
            cm[ro[s] + I, :I + pb + 1] = True
    np.testing.assert_allclose(P.cpu().numpy()[:, cm], P_ref[:, cm], rtol=5e-4, atol=1e-30)
    idx_r, cnt_r = oracle.threshold(P_ref, cuq, 0.2, block=blk, cu_seqlens_k=cuk)
    idx, cnt = plan.fp_threshold(torch.from_numpy(P_ref).cuda(), 0.2)
    torch.cuda.synchronize()
    compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)
    O_ref, lse_ref = oracle.sparse_prefill(Q, K, V, cuq, idx_r, cnt_r, block=blk, cu_seqlens_k=cuk)
    O, lse = plan.fp_sparse_prefill(dQ, dK, dV, torch.from_numpy(idx_r).cuda(), torch.from_numpy(cnt_r).cuda())
    Od_ref, _ = oracle.dense_prefill(Q, K, V, cuq, block=blk, cu_seqlens_k=cuk)
    Od, _ = plan.fp_dense_prefill(dQ, dK, dV)
    torch.cuda.synchronize()
    compare_O(O, O_ref); compare_O(Od, Od_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    plan.close()
    with pytest.raises(B.FlashPrefillError) as e:      # block sizes other than 128 come with head dimension 128 only
        B.Plan([0, 512], 4, 2, head_dim=64, block=64)
    assert e.value.status == B.FP_ERR_UNSUPPORTED
