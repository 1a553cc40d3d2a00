"""GPU parity on randomly drawn valid shapes: sequence counts and lengths, KV prefixes, GQA groupings,
head dimensions, block sizes, threshold / sink / window / softmax-scale settings, with a few rows emptied.  Every stage is checked
against the oracle as in the fixed cases; the seeds are fixed, so the cases are the same every run."""
import numpy as np
import pytest

import oracle
from paper_2603_06199_amd import binding as B
import synth

from gpu_util import BAND, LSE_ATOL, compare_lists_exact, compare_O, dev, lists_to_mask

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.mark.parametrize("seed", range(16))
def test_random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    it = seed
    nseq = int(rng.integers(1, 5))
    hkv = int(rng.choice([1, 2, 4])); g = int(rng.choice([1, 2, 3, 4, 8])); hq = hkv * g
    q_lens, pbs = [], []
    chunked = rng.random() < 0.5
    for s in range(nseq):
        ql = int(rng.integers(1, 1400))
        pb = int(rng.integers(0, 12)) if chunked and rng.random() < 0.7 else 0
        q_lens.append(ql); pbs.append(pb)
    d = int(rng.choice([64, 128, 128, 256]))
    blk = (128, 64, 256, 128)[seed % 4] if d == 128 else 128     # other block sizes exist at head dimension 128
    kv_lens = [ql + blk * pb for ql, pb in zip(q_lens, pbs)]
    cuq = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32); cuk = np.concatenate([[0], np.cumsum(kv_lens)]).astype(np.int32)
    alpha = float(rng.choice([0.0, 0.05, 0.12, 0.3, 0.9])); sink = int(rng.choice([0, 100, 256, 700])); win = int(rng.choice([0, 128, 512, 1000]))
    tau = float(rng.choice([0.0, 0.05, 0.15]))
    Tk, Tq = int(cuk[-1]), int(cuq[-1])
    u = rng.standard_normal(d).astype(np.float32); u /= np.linalg.norm(u)
    Kf = rng.standard_normal((Tk, hkv, d)).astype(np.float32)
    for t in rng.choice(Tk, size=max(1, Tk // 400), replace=False):
        lo = (t // blk) * blk; Kf[lo:lo + blk] += 3.0 * u
    Qf = rng.standard_normal((Tq, hq, d)).astype(np.float32) + float(rng.choice([0.0, 1.5])) * u
    Q, K = synth.f32_to_bf16_bits(Qf), synth.f32_to_bf16_bits(Kf)
    V = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hkv, d)).astype(np.float32))
    print(f"\n[random shape {it}] q={q_lens} kv={kv_lens} hq={hq} hkv={hkv} d={d} block={blk} alpha={alpha} sink={sink} win={win} tau={tau}", flush=True)
    ck = cuk if chunked else None
    if not chunked: assert list(cuq) == list(cuk)
    plan = B.Plan(cuq, hq, hkv, head_dim=d, block=blk, scale=tau, cu_seqlens_k=ck)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    tau_o = None if tau == 0.0 else tau
    P_ref = oracle.block_search(Q, K, cuq, block=blk, tau=tau_o, cu_seqlens_k=ck)
    m, n, ro = oracle.layout(cuq, block=blk, cu_seqlens_k=ck)
    P = torch.full((hq, m, n), float("nan"), dtype=torch.float32, device="cuda")
    plan.fp_block_search(dQ, dK, P); torch.cuda.synchronize(); Pg = P.cpu().numpy()
    cm, own = np.zeros((m, n), bool), np.zeros((m, n), bool)
    for s in range(nseq):
        pb = pbs[s]
        own[ro[s]:ro[s + 1], :-(-kv_lens[s] // blk)] = True
        for I in range(ro[s + 1] - ro[s]): cm[ro[s] + I, :I + pb + 1] = True
    assert not Pg[:, own & ~cm].any() and np.isnan(Pg[:, ~own]).all()   # zeros up to the sequence's last block, nothing beyond
    P = torch.nan_to_num(P, nan=0.0)
    np.testing.assert_allclose(Pg[:, cm], P_ref[:, cm], rtol=5e-4, atol=1e-30)
    idx_r, cnt_r = oracle.threshold(P_ref, cuq, alpha, block=blk, sink_tokens=sink, window_tokens=win, cu_seqlens_k=ck)
    idx, cnt = plan.fp_threshold(torch.from_numpy(P_ref).cuda(), alpha, sink_tokens=sink, window_tokens=win); torch.cuda.synchronize()
    compare_lists_exact(idx.cpu().numpy(), cnt.cpu().numpy(), idx_r, cnt_r)
    idx_f, cnt_f = plan.fp_search_select(dQ, dK, alpha, sink_tokens=sink, window_tokens=win)
    idx_2, cnt_2 = plan.fp_threshold(P, alpha, sink_tokens=sink, window_tokens=win); torch.cuda.synchronize()
    compare_lists_exact(idx_f.cpu().numpy(), cnt_f.cpu().numpy(), idx_2.cpu().numpy(), cnt_2.cpu().numpy())
    mg, mr = lists_to_mask(idx_f.cpu().numpy(), cnt_f.cpu().numpy()), lists_to_mask(idx_r, cnt_r)
    thr = np.float32(alpha) * np.where(cm[None], P_ref, -np.inf).max(axis=2, keepdims=True)
    band = (np.abs(P_ref - thr) <= BAND * np.abs(thr)) & cm[None]
    assert not np.any((mg != mr) & ~band)
    if cnt_r.size and rng.random() < 0.3:      # sometimes empty a few rows
        cnt_r = cnt_r.copy(); cnt_r[:, rng.integers(0, m)] = 0
    O_ref, lse_ref = oracle.sparse_prefill(Q, K, V, cuq, idx_r, cnt_r, block=blk, tau=tau_o, cu_seqlens_k=ck)
    O, lse = plan.fp_sparse_prefill(dQ, dK, dV, torch.from_numpy(idx_r).cuda(), torch.from_numpy(cnt_r).cuda()); torch.cuda.synchronize()
    compare_O(O, O_ref)
    lg, lr = lse.cpu().numpy(), lse_ref
    fin = np.isfinite(lr)
    assert np.array_equal(np.isfinite(lg), fin)
    np.testing.assert_allclose(lg[fin], lr[fin], atol=LSE_ATOL, rtol=0)
    Od_ref, lsed_ref = oracle.dense_prefill(Q, K, V, cuq, block=blk, tau=tau_o, cu_seqlens_k=ck)
    Od, lsed = plan.fp_dense_prefill(dQ, dK, dV); torch.cuda.synchronize()
    compare_O(Od, Od_ref)
    np.testing.assert_allclose(lsed.cpu().numpy(), lsed_ref, atol=LSE_ATOL, rtol=0)
    plan.close()
