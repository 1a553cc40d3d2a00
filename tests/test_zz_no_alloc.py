"""The entry point that allocates nothing (fp_block_search_static): its scores against those of
fp_block_search, on two calls in a row, the second with a smaller input that leaves most of the
built-in scratch holding the first call's pooled keys."""
import ctypes

import numpy as np
import pytest

from paper_2603_06199_amd import binding as B
import synth

from gpu_util import causal_mask, dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _case(name, seqlens, hq, hkv, seed):
    w = synth.small(name, seqlens, hq, hkv, seed=seed)
    Q, K, _ = synth.make_qkv(w)
    return w, dev(Q), dev(K)


def test_static_scratch_entry_point_matches_fp_block_search_twice_in_a_row():
    cases = [_case("static_big", [128 * 37 + 50, 700, 128 * 12], 8, 2, 3),
             _case("static_small", [900, 128], 4, 1, 4)]            # second call: smaller input
    for w, dQ, dK in cases:
        cu = w.cu_seqlens
        plan = B.Plan(cu, w.hq, w.hkv)
        shape = (w.hq, plan.m_total, plan.n_max)
        want = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
        plan.fp_block_search(dQ, dK, want)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        plan.fp_block_search_static(dQ, dK, got)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before          # no device memory taken or given back
        # integer-and-index bar: the same kernels ran on the same inputs, so every written entry
        # (finite in `want`) is bit-identical and every unwritten entry is still the sentinel
        assert torch.equal(torch.isnan(got), torch.isnan(want))
        assert torch.equal(torch.nan_to_num(got), torch.nan_to_num(want))
        cm = torch.from_numpy(np.broadcast_to(causal_mask(cu)[None], shape).copy()).cuda()
        assert bool(torch.isfinite(got[cm]).all()) and bool((got[cm] >= 0).all())
        plan.close()


def test_static_scratch_limit_is_an_error_not_a_launch():
    # 16385 key blocks x Hkv = 1 exceed the built-in array: rejected on the host, nothing launched
    lens = [4096 * 128] * 4 + [128]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    plan = B.Plan(cu, 1, 1)
    one = torch.zeros(1, dtype=torch.bfloat16, device="cuda")      # never dereferenced
    st = B.lib().fp_block_search_static(plan._h, ctypes.c_void_p(one.data_ptr()), ctypes.c_void_p(one.data_ptr()),
                                        ctypes.c_float(1e-10), ctypes.c_void_p(one.data_ptr()), None)
    assert st == B.FP_ERR_STATIC_LIMIT
    assert "built-in" in B.status_string(st)
    torch.cuda.synchronize()
    plan.close()
