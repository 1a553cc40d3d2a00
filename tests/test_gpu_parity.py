"""GPU parity: every stage of the HIP path against the CPU oracle, element by element, through
the C ABI.  Sizes span several tiles, ragged tails, packed batches and every GQA grouping the
kernels special-case (g = 1, 2, 4, 8)."""
import numpy as np
import pytest

import oracle
from paper_2603_06199_amd import binding as B
import synth

from gpu_util import (LSE_ATOL, compare_lists_banded, compare_lists_exact, compare_O, compare_scores, dev, f32)

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CASES = [
    # name, seqlens, hq, hkv
    ("one_block", [128], 4, 1),
    ("tiny_ragged", [5], 2, 2),
    ("several_tiles", [1536], 8, 2),
    ("ragged_tail", [1000], 4, 1),
    ("packed_ragged", [640, 77, 1300, 128], 8, 4),
    ("mha_g1", [700], 2, 2),
    ("g2", [900], 4, 2),
    ("g8_long_row", [5000], 8, 1),        # > 32 key blocks: more than one pooled-key tile per row
    ("g3_odd_group", [1100, 300], 6, 2),  # odd group size: the search kernel's second head slot is idle in one chunk
    ("many_short", [int(x) for x in np.random.default_rng(7).integers(1, 1500, size=40)], 4, 2),
]


@pytest.fixture(scope="module", params=CASES, ids=[c[0] for c in CASES])
def case(request):
    name, seqlens, hq, hkv = request.param
    w = synth.small(name, seqlens, hq, hkv, seed=11)
    Q, K, V = synth.make_qkv(w)
    cu = w.cu_seqlens
    print(f"\n[case] {name} seqlens={seqlens} hq={hq} hkv={hkv}", flush=True)
    plan = B.Plan(cu, hq, hkv)
    d = dict(w=w, cu=cu, Q=Q, K=K, V=V, plan=plan, dQ=dev(Q), dK=dev(K), dV=dev(V))
    d["P_ref"] = oracle.block_search(Q, K, cu)
    yield d
    plan.close()


def test_block_search_matches_oracle(case):
    P = case["plan"].fp_block_search(case["dQ"], case["dK"])
    torch.cuda.synchronize()
    compare_scores(P.cpu().numpy(), case["P_ref"], case["cu"])


@pytest.mark.parametrize("alpha", [0.12, 0.0, 1.0, 0.5])
def test_threshold_bit_exact_on_same_scores(case, alpha):
    P_ref = case["P_ref"]
    idx_r, cnt_r = oracle.threshold(P_ref, case["cu"], alpha)
    idx, cnt = case["plan"].fp_threshold(torch.from_numpy(P_ref).cuda(), alpha)
    torch.cuda.synchronize()
    compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)


def test_threshold_other_sink_and_window(case):
    P_ref = case["P_ref"]
    for sink, win in ((0, 0), (100, 200), (1024, 128)):
        idx_r, cnt_r = oracle.threshold(P_ref, case["cu"], 0.3, sink_tokens=sink, window_tokens=win)
        idx, cnt = case["plan"].fp_threshold(torch.from_numpy(P_ref).cuda(), 0.3, sink_tokens=sink, window_tokens=win)
        torch.cuda.synchronize()
        compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)


def test_threshold_ignores_entries_past_the_diagonal(case):
    """Scores with J > I are documented not to matter: poison them and expect the oracle's lists."""
    from gpu_util import causal_mask
    P_ref = case["P_ref"]
    idx_r, cnt_r = oracle.threshold(P_ref, case["cu"], 0.25)
    poisoned = np.where(causal_mask(case["cu"])[None], P_ref, np.float32(np.nan)).astype(np.float32)
    poisoned[:, :, 1::2] = np.where(causal_mask(case["cu"])[None, :, 1::2], P_ref[:, :, 1::2], np.float32(3e38))
    idx, cnt = case["plan"].fp_threshold(torch.from_numpy(poisoned).cuda(), 0.25)
    torch.cuda.synchronize()
    compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)


def test_search_plus_threshold_lists(case):
    plan = case["plan"]
    P = plan.fp_block_search(case["dQ"], case["dK"])
    idx, cnt = plan.fp_threshold(P, case["w"].alpha)
    torch.cuda.synchronize()
    nd, nb = compare_lists_banded(idx.cpu().numpy(), cnt.cpu().numpy(), case["P_ref"], case["cu"], case["w"].alpha)
    print(f"list mismatches {nd} (all inside the near-threshold band of {nb} pairs)")


def test_fused_search_select_lists(case):
    """The one-pass entry point against the oracle's Alg. 1 + Alg. 2 (same band rule as above), for the
    default and a second sink/window setting; it must also agree entry by entry with the library's
    own two-call path, whose decisions it is documented to reproduce."""
    plan, w = case["plan"], case["w"]
    for alpha, sink, win in ((w.alpha, 256, 512), (0.3, 100, 200), (0.0, 0, 0)):
        idx, cnt = plan.fp_search_select(case["dQ"], case["dK"], alpha, sink_tokens=sink, window_tokens=win)
        torch.cuda.synchronize()
        nd, nb = compare_lists_banded(idx.cpu().numpy(), cnt.cpu().numpy(), case["P_ref"], case["cu"], alpha,
                                      sink_tokens=sink, window_tokens=win)
        idx2, cnt2 = plan.fp_threshold(plan.fp_block_search(case["dQ"], case["dK"]), alpha, sink_tokens=sink,
                                       window_tokens=win)
        torch.cuda.synchronize()
        compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx2.cpu().numpy(), cnt2.cpu().numpy())


def test_sparse_prefill_matches_oracle_on_oracle_lists(case):
    cu = case["cu"]
    idx_r, cnt_r = oracle.threshold(case["P_ref"], cu, case["w"].alpha)
    O_ref, lse_ref = oracle.sparse_prefill(case["Q"], case["K"], case["V"], cu, idx_r, cnt_r)
    O, lse = case["plan"].fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], torch.from_numpy(idx_r).cuda(),
                                            torch.from_numpy(cnt_r).cuda())
    torch.cuda.synchronize()
    mx, mean = compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    print(f"sparse O max-abs {mx:.2e} mean-abs {mean:.2e}")


def test_dense_prefill_matches_oracle(case):
    O_ref, lse_ref = oracle.dense_prefill(case["Q"], case["K"], case["V"], case["cu"])
    O, lse = case["plan"].fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    torch.cuda.synchronize()
    mx, mean = compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    print(f"dense O max-abs {mx:.2e} mean-abs {mean:.2e}")


def test_threshold_disabled_equals_dense_bitwise(case):
    plan = case["plan"]
    P = plan.fp_block_search(case["dQ"], case["dK"])
    idx, cnt = plan.fp_threshold(P, 0.0)
    Os, ls = plan.fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], idx, cnt)
    Od, ld = plan.fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    torch.cuda.synchronize()
    assert torch.equal(Os.view(torch.int16), Od.view(torch.int16))
    assert torch.equal(ls, ld)


def test_random_lists_without_diagonal_and_empty_rows(case):
    # lists need not contain the diagonal; a row with cnt == 0 yields O = 0 (library contract)
    cu, hq = case["cu"], case["w"].hq
    idx, cnt = synth.forced_density_lists(cu, hq, 0.4, seed=3, sink_blocks=0, window_blocks=0)
    cnt[:, ::5] = 0
    O_ref, lse_ref = oracle.sparse_prefill(case["Q"], case["K"], case["V"], cu, idx, cnt)
    O, lse = case["plan"].fp_sparse_prefill(case["dQ"], case["dK"], case["dV"], torch.from_numpy(idx).cuda(),
                                            torch.from_numpy(cnt).cuda())
    torch.cuda.synchronize()
    compare_O(O, O_ref)                         # empty rows: O = 0 on both sides
    got = lse.cpu().numpy()
    fin = np.isfinite(lse_ref)
    assert not fin.all() and np.all(np.isneginf(lse_ref[~fin]))
    np.testing.assert_allclose(got[fin], lse_ref[fin], atol=LSE_ATOL, rtol=0)
    assert np.all(np.isneginf(got[~fin]))


def test_outputs_are_deterministic(case):
    plan = case["plan"]
    a = plan.fp_block_search(case["dQ"], case["dK"]).clone()
    b = plan.fp_block_search(case["dQ"], case["dK"])
    Oa, _ = plan.fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    Ob, _ = plan.fp_dense_prefill(case["dQ"], case["dK"], case["dV"])
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(Oa.view(torch.int16), Ob.view(torch.int16))


def test_two_plans_on_two_streams():
    """Plans own their workspaces, so two layers may run concurrently on two streams."""
    ws = [synth.small("stream_a", [1400, 300], 8, 2, seed=21), synth.small("stream_b", [2100], 4, 4, seed=22)]
    data = []
    for w in ws:
        Q, K, V = synth.make_qkv(w)
        plan = B.Plan(w.cu_seqlens, w.hq, w.hkv)
        data.append(dict(w=w, plan=plan, dQ=dev(Q), dK=dev(K), dV=dev(V)))
    ref = []
    for d in data:                                  # one after the other on the current stream
        idx, cnt = d["plan"].fp_search_select(d["dQ"], d["dK"], 0.2)
        O, lse = d["plan"].fp_sparse_prefill(d["dQ"], d["dK"], d["dV"], idx, cnt)
        ref.append((cnt.clone(), O.clone(), lse.clone()))
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    out = [None, None]
    for rep in range(3):
        for i, d in enumerate(data):
            with torch.cuda.stream(streams[i]):
                idx, cnt = d["plan"].fp_search_select(d["dQ"], d["dK"], 0.2, stream=streams[i])
                O, lse = d["plan"].fp_sparse_prefill(d["dQ"], d["dK"], d["dV"], idx, cnt, stream=streams[i])
                out[i] = (cnt, O, lse)
        torch.cuda.synchronize()
        for got, want in zip(out, ref):
            for a, b in zip(got, want):
                assert torch.equal(a, b)
    for d in data:
        d["plan"].close()


def test_custom_softmax_scale_and_eps():
    """A softmax scale other than 1/sqrt(d) and an eps large enough to matter, against the oracle."""
    w = synth.small("custom_scale", [1700, 260], 8, 2, seed=31)
    Q, K, V = synth.make_qkv(w)
    cu, tau, eps = w.cu_seqlens, 0.05, 5.0
    plan = B.Plan(cu, w.hq, w.hkv, scale=tau)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    P_ref = oracle.block_search(Q, K, cu, tau=tau, eps=eps)
    P = plan.fp_block_search(dQ, dK, eps=eps)
    torch.cuda.synchronize()
    compare_scores(P.cpu().numpy(), P_ref, cu)
    assert abs(float(P_ref[0, 5].sum()) - 1.0) > 1e-2          # eps is visible in the normalisation
    idx_r, cnt_r = oracle.threshold(P_ref, cu, 0.3)
    idx_f, cnt_f = plan.fp_search_select(dQ, dK, 0.3, eps=eps)
    torch.cuda.synchronize()
    compare_lists_banded(idx_f.cpu().numpy(), cnt_f.cpu().numpy(), P_ref, cu, 0.3)
    O_ref, lse_ref = oracle.sparse_prefill(Q, K, V, cu, idx_r, cnt_r, tau=tau)
    O, lse = plan.fp_sparse_prefill(dQ, dK, dV, torch.from_numpy(idx_r).cuda(), torch.from_numpy(cnt_r).cuda())
    torch.cuda.synchronize()
    compare_O(O, O_ref)
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, atol=LSE_ATOL, rtol=0)
    plan.close()


@pytest.mark.parametrize("seqlens,hq,hkv,mode,qscale,eps", [
    ([40000], 4, 2, "coherent", 1, 1e-10),
    ([128 * 300 + 5, 128 * 290], 8, 1, "coherent", 1, 1e-10),   # ragged last q-block of a long row; 4 head pairs per KV head
    ([36000], 6, 2, "literal", 1, 1e-10),                        # flat score map: many pairs close to the row max
    ([40000], 4, 2, "coherent", 16, 1e-10),                      # logits beyond the norm bound: Eq. 1-2 with the pair max
    ([36000], 4, 2, "literal", 1, 0.5),                          # a visible eps: the pair max is tracked for Eq. 4
])
def test_one_pass_selection_on_long_rows(seqlens, hq, hkv, mode, qscale, eps):
    """Rows of more than 128 key blocks: fp_search_select scores them on the pooled key's hi plane and
    re-scores exactly the pairs that may hold the row max or straddle the threshold.  Its lists are
    held to the same rule as the two-call path (equal to the oracle's outside the near-threshold
    band) and may differ from the two-call lists only inside that band."""
    from gpu_util import causal_mask, compare_lists_same_outside_band
    w = synth.small("long_rows", seqlens, hq, hkv, seed=17, mode=mode)
    Q, K, _ = synth.make_qkv(w)
    if qscale != 1:      # a power of two: exact in bf16
        Q = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(Q) * np.float32(qscale))
    cu = w.cu_seqlens
    dQ, dK = dev(Q), dev(K)
    plan = B.Plan(cu, hq, hkv)
    P_ref = oracle.block_search(Q, K, cu, eps=eps)
    P = plan.fp_block_search(dQ, dK, eps=eps)
    torch.cuda.synchronize()
    compare_scores(P.cpu().numpy(), P_ref, cu)
    cm = causal_mask(cu)
    for alpha, sink, win in ((0.12, 256, 512), (0.5, 0, 128), (1.0, 256, 512), (0.97, 0, 0), (3e-3, 0, 0)):
        idx2, cnt2 = plan.fp_threshold(P, alpha, sink_tokens=sink, window_tokens=win)
        idx, cnt = plan.fp_search_select(dQ, dK, alpha, sink_tokens=sink, window_tokens=win, eps=eps)
        torch.cuda.synchronize()
        nd, nb = compare_lists_banded(idx.cpu().numpy(), cnt.cpu().numpy(), P_ref, cu, alpha, sink_tokens=sink,
                                      window_tokens=win)
        nd2 = compare_lists_same_outside_band(idx.cpu().numpy(), cnt.cpu().numpy(), idx2.cpu().numpy(),
                                              cnt2.cpu().numpy(), P_ref, cm, alpha)
        kept = int(cnt.sum())
        print(f"alpha {alpha} sink {sink} window {win}: kept {kept}, vs oracle {nd} mismatches (band {nb}), vs two calls {nd2}")
    plan.close()


def test_plan_in_a_caller_owned_workspace():
    """fp_workspace_bytes + fp_plan_create_in: the plan's tables and pooled keys live in a buffer the
    caller allocated; results are those of a library-allocated plan, nothing is written past the
    stated size, and a buffer one byte short is refused."""
    w = synth.small("caller_ws", [1300, 77, 640], 8, 4, seed=5)
    Q, K, V = synth.make_qkv(w)
    cu = w.cu_seqlens
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    need = B.fp_workspace_bytes(cu, w.hq, w.hkv)
    assert need > 0
    guard = 4096
    buf = torch.full((need + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    assert buf.data_ptr() % 256 == 0
    own = B.Plan(cu, w.hq, w.hkv)
    mine = B.Plan(cu, w.hq, w.hkv, workspace=buf[:need])
    for plan in (own, mine):
        plan.res = (plan.fp_block_search(dQ, dK),) + plan.fp_search_select(dQ, dK, 0.12) + plan.fp_dense_prefill(dQ, dK, dV)
    torch.cuda.synchronize()
    P0, idx0, cnt0, O0, lse0 = own.res
    P1, idx1, cnt1, O1, lse1 = mine.res
    cm = torch.from_numpy(np.broadcast_to(causal_mask_np(cu), P0.shape).copy()).cuda()
    assert torch.equal(P0[cm], P1[cm]) and torch.equal(cnt0, cnt1) and torch.equal(O0, O1) and torch.equal(lse0, lse1)
    valid = torch.arange(idx0.shape[2], device="cuda")[None, None, :] < cnt0[:, :, None]
    assert torch.equal(idx0[valid], idx1[valid])
    assert bool((buf[need:] == 0xA5).all())
    with pytest.raises(B.FlashPrefillError) as e:
        B.Plan(cu, w.hq, w.hkv, workspace=buf[:need - 1])
    assert e.value.status == B.FP_ERR_WORKSPACE
    own.close(); mine.close()


def causal_mask_np(cu):
    from gpu_util import causal_mask
    return causal_mask(cu)[None]
