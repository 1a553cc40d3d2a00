"""Pins for the oracle's chunked-prefill form (queries = the last tokens of a longer key sequence).

The plain form is pinned elsewhere against closed forms and library routines; here the chunked form
must reproduce the plain form's rows for the same tokens, and a library attention with an explicit
bottom-right-aligned causal mask."""
import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")


def _case(seed, kv_lens, q_lens, hq=4, hkv=2, d=128):
    rng = np.random.default_rng(seed)
    Tk = sum(kv_lens)
    Qf = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hq, d)).astype(np.float32))
    K = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hkv, d)).astype(np.float32))
    V = synth.f32_to_bf16_bits(rng.standard_normal((Tk, hkv, d)).astype(np.float32))
    cuk = np.concatenate([[0], np.cumsum(kv_lens)]).astype(np.int32)
    cuq = np.concatenate([[0], np.cumsum(q_lens)]).astype(np.int32)
    sel = np.concatenate([np.arange(cuk[s + 1] - q_lens[s], cuk[s + 1]) for s in range(len(kv_lens))])
    return Qf, np.ascontiguousarray(Qf[sel]), K, V, cuq, cuk, sel


def _row_map(cuq, cuk):
    """Row of the full layout for each row of the chunked layout, and the chunk's prefix in blocks."""
    m_f, n_f, ro_f = oracle.layout(cuk)
    m_c, n_c, ro_c = oracle.layout(cuq, cu_seqlens_k=cuk)
    assert n_c == n_f
    rows, pbs = [], []
    for s in range(len(cuq) - 1):
        pb = ((cuk[s + 1] - cuk[s]) - (cuq[s + 1] - cuq[s])) // 128
        for I in range(ro_c[s + 1] - ro_c[s]):
            rows.append(ro_f[s] + pb + I)
            pbs.append(pb)
    return np.array(rows), np.array(pbs)


@pytest.mark.parametrize("kv_lens,q_lens", [
    ([1024], [384]),                      # block-aligned chunk
    ([1000], [360]),                      # ragged end: prefix 640 = 5 blocks
    ([640, 900, 256], [128, 900, 100 + 28]),   # prefixes 512, 0, 128; one sequence is a plain prefill
])
def test_chunked_equals_the_rows_of_the_full_prefill(kv_lens, q_lens):
    Qf, Qc, K, V, cuq, cuk, sel = _case(0, kv_lens, q_lens)
    rows, _ = _row_map(cuq, cuk)
    P_full = oracle.block_search(Qf, K, cuk)
    P_ch = oracle.block_search(Qc, K, cuq, cu_seqlens_k=cuk)
    np.testing.assert_array_equal(P_ch, P_full[:, rows])
    for alpha, sink, win in ((0.3, 256, 512), (0.05, 0, 128)):
        idx_f, cnt_f = oracle.threshold(P_full, cuk, alpha, sink_tokens=sink, window_tokens=win)
        idx_c, cnt_c = oracle.threshold(P_ch, cuq, alpha, sink_tokens=sink, window_tokens=win, cu_seqlens_k=cuk)
        np.testing.assert_array_equal(cnt_c, cnt_f[:, rows])
        np.testing.assert_array_equal(idx_c, idx_f[:, rows])
        O_f, l_f = oracle.sparse_prefill(Qf, K, V, cuk, idx_f, cnt_f)
        O_c, l_c = oracle.sparse_prefill(Qc, K, V, cuq, idx_c, cnt_c, cu_seqlens_k=cuk)
        np.testing.assert_array_equal(O_c, O_f[sel])
        np.testing.assert_array_equal(l_c, l_f[:, sel])
    Od_f, ld_f = oracle.dense_prefill(Qf, K, V, cuk)
    Od_c, ld_c = oracle.dense_prefill(Qc, K, V, cuq, cu_seqlens_k=cuk)
    np.testing.assert_array_equal(Od_c, Od_f[sel])
    np.testing.assert_array_equal(ld_c, ld_f[:, sel])


def test_chunked_dense_against_library_attention_with_explicit_mask():
    kv_lens, q_lens = [428], [428 - 256]               # prefix 256
    Qf, Qc, K, V, cuq, cuk, sel = _case(1, kv_lens, q_lens, hq=2, hkv=1, d=64)
    O, lse = oracle.dense_prefill(Qc, K, V, cuq, cu_seqlens_k=cuk)
    q = torch.from_numpy(synth.bf16_bits_to_f32(Qc)).double().permute(1, 0, 2)          # [h, Tq, d]
    k = torch.from_numpy(synth.bf16_bits_to_f32(K)).double().permute(1, 0, 2).expand(2, -1, -1)
    v = torch.from_numpy(synth.bf16_bits_to_f32(V)).double().permute(1, 0, 2).expand(2, -1, -1)
    Tq, Tk = q.shape[1], k.shape[1]
    mask = (torch.arange(Tk)[None, :] <= (torch.arange(Tq)[:, None] + (Tk - Tq)))          # bottom-right aligned
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask)
    np.testing.assert_allclose(O, ref.permute(1, 0, 2).numpy(), rtol=0, atol=2e-6)
    logits = (q @ k.transpose(1, 2)) / 8.0
    ref_lse = torch.logsumexp(logits.masked_fill(~mask, -float("inf")), dim=-1) * 1.4426950408889634
    np.testing.assert_allclose(lse, ref_lse.numpy(), rtol=0, atol=1e-5)


def test_chunked_layout_and_rejected_lengths():
    m, n, ro = oracle.layout([0, 200, 328], cu_seqlens_k=[0, 200 + 384, 200 + 384 + 128 + 512])
    assert (m, n) == (3, 5) and list(ro) == [0, 2, 3]
    with pytest.raises(ValueError):
        oracle.layout([0, 200], cu_seqlens_k=[0, 300])        # prefix 100 is not a block multiple
    with pytest.raises(ValueError):
        oracle.layout([0, 200], cu_seqlens_k=[0, 100])        # fewer keys than queries
    with pytest.raises(ValueError):
        oracle.layout([0, 200, 400], cu_seqlens_k=[0, 200])   # lengths of different size
