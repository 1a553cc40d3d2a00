"""The compute calls only enqueue kernels (no allocation, no synchronisation, no host reads), so a
whole layer can be captured into a HIP graph and replayed.  Every replay is checked against the
eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2603_06199_amd import binding as B
import synth

from gpu_util import dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_layer_captured_in_a_graph_replays_bit_exactly():
    w = synth.small("graph_case", seqlens=(128 * 9 + 40, 700), hq=8, hkv=2, seed=3)
    Q, K, V = synth.make_qkv(w)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    plan = B.Plan(w.cu_seqlens, w.hq, w.hkv)
    hq, m, n = w.hq, plan.m_total, plan.n_max
    scores = torch.empty((hq, m, n), dtype=torch.float32, device="cuda")
    idx = torch.zeros((hq, m, n), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((hq, m), dtype=torch.int32, device="cuda")
    idx2, cnt2 = torch.zeros_like(idx), torch.zeros_like(cnt)
    O, O2, Od = torch.empty_like(dQ), torch.empty_like(dQ), torch.empty_like(dQ)
    lse = torch.empty((hq, plan.T), dtype=torch.float32, device="cuda")

    def layer():
        plan.fp_block_search(dQ, dK, scores)
        plan.fp_threshold(scores, 0.3, idx=idx, cnt=cnt)
        plan.fp_sparse_prefill(dQ, dK, dV, idx, cnt, O, lse)
        plan.fp_search_select(dQ, dK, 0.3, idx=idx2, cnt=cnt2)
        plan.fp_sparse_prefill(dQ, dK, dV, idx2, cnt2, O2, want_lse=False)
        plan.fp_dense_prefill(dQ, dK, dV, Od, want_lse=False)

    layer()
    torch.cuda.synchronize()
    want = [t.clone() for t in (scores, cnt, O, lse, cnt2, O2, Od)]
    # columns past a sequence's own last key block are not written by the search: compare the rest
    ro = plan.row_offset
    own = torch.zeros((m, n), dtype=torch.bool, device="cuda")
    for s in range(len(ro) - 1):
        own[ro[s]:ro[s + 1], :ro[s + 1] - ro[s]] = True
    valid = torch.arange(n, device="cuda")[None, None, :] < cnt[:, :, None]
    want_idx = torch.where(valid, idx, torch.zeros_like(idx))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer()
    for rep in range(3):
        for t in (scores, O, lse, O2, Od):
            t.fill_(float("nan"))                 # eager work between replays; fill kernels, no memset nodes in the graph
        cnt.zero_(); cnt2.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = (scores, cnt, O, lse, cnt2, O2, Od)
        for k, (a, b) in enumerate(zip(got, want)):
            if k == 0:
                a, b = a[:, own], b[:, own]
            assert torch.equal(a, b), f"replay {rep} differs from the eager run"
        assert torch.equal(torch.where(valid, idx, torch.zeros_like(idx)), want_idx)
        assert torch.equal(torch.where(valid, idx2, torch.zeros_like(idx)), want_idx)
    plan.close()
