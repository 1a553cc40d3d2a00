"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and rejects
bad shapes with the documented codes before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2603_06199_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2603_06199_amd import build
        build.build()
    return B.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "flashprefill.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    for s in range(6):
        assert len(B.status_string(s)) > 0
    assert B.status_string(0) == "ok"


def test_layout_matches_block_arithmetic(lib):
    m, n, ro = B.fp_layout([0, 300, 1000, 1128], 8, 2)
    assert (m, n) == (3 + 6 + 1, 6)
    assert ro.tolist() == [0, 3, 9, 10]


@pytest.mark.parametrize("cu,hq,hkv,d,blk,scale,code", [
    ([0, 128], 8, 3, 128, 128, 0.0, B.FP_ERR_INVALID_ARG),     # hq % hkv
    ([0, 128, 128], 8, 2, 128, 128, 0.0, B.FP_ERR_INVALID_ARG),  # empty sequence
    ([0, 256, 128], 8, 2, 128, 128, 0.0, B.FP_ERR_INVALID_ARG),  # decreasing
    ([1, 128], 8, 2, 128, 128, 0.0, B.FP_ERR_INVALID_ARG),     # does not start at 0
    ([0, 128], 0, 1, 128, 128, 0.0, B.FP_ERR_INVALID_ARG),
    ([0, 128], 8, 2, 128, 128, float("nan"), B.FP_ERR_INVALID_ARG),
    ([0, 128], 8, 2, 96, 128, 0.0, B.FP_ERR_UNSUPPORTED),      # head_dim other than 64, 128, 256
    ([0, 128], 8, 2, 128, 32, 0.0, B.FP_ERR_UNSUPPORTED),      # block other than 64, 128, 256
    ([0, 128], 8, 2, 64, 256, 0.0, B.FP_ERR_UNSUPPORTED),      # blocks other than 128 need head_dim 128
    ([0, 4097 * 128], 8, 2, 128, 128, 0.0, B.FP_ERR_UNSUPPORTED),  # more than 4096 blocks in a sequence
])
def test_bad_shapes_are_rejected_on_the_host(lib, cu, hq, hkv, d, blk, scale, code):
    with pytest.raises(B.FlashPrefillError) as e:
        B.fp_layout(cu, hq, hkv, d, blk, scale)
    assert e.value.status == code


def test_null_arguments(lib):
    assert lib.fp_layout(None, None, None, None) == B.FP_ERR_INVALID_ARG
    s, keep = B.make_shape([0, 128], 4, 1)
    assert lib.fp_plan_create(ctypes.byref(s), 0, None) == B.FP_ERR_INVALID_ARG
    assert lib.fp_plan_create_in(ctypes.byref(s), 0, None, 0, None) == B.FP_ERR_INVALID_ARG
    assert lib.fp_workspace_bytes(None) == 0
    for call, nargs in ((lib.fp_block_search, 6), (lib.fp_threshold, 6), (lib.fp_search_select, 8),
                        (lib.fp_sparse_prefill, 9), (lib.fp_dense_prefill, 7)):
        args = [None] * nargs
        if call in (lib.fp_block_search, lib.fp_search_select):
            args[3] = 0.0
        assert call(*args) == B.FP_ERR_INVALID_ARG
    lib.fp_plan_destroy(None)   # documented no-op


def test_plan_create_without_a_gpu_reports_device_error(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(B.FlashPrefillError) as e:
        B.Plan([0, 256], 4, 1)
    assert e.value.status == B.FP_ERR_DEVICE


def test_workspace_bytes_cover_tables_and_pooled_keys(lib):
    # three sequences of 3 + 6 + 1 q-blocks = key blocks, Hkv = 2: two 32-byte row records, one rank
    # entry and one 8-byte key-block record per block, two bf16 planes of pooled keys, two fp32 norms per pooled key; each part
    # rounded up to 256 bytes
    up = lambda b: (b + 255) // 256 * 256
    want = 2 * up(10 * 32) + up(10 * 4) + up(10 * 8) + 2 * up(10 * 2 * 128 * 2) + up(10 * 2 * 8)
    assert B.fp_workspace_bytes([0, 300, 1000, 1128], 8, 2) == want
    # chunked prefill: 3 q-block rows, 5 + 5 key blocks
    want = 2 * up(3 * 32) + up(3 * 4) + up(10 * 8) + 2 * up(10 * 2 * 128 * 2) + up(10 * 2 * 8)
    assert B.fp_workspace_bytes([0, 200, 328], 8, 2, cu_seqlens_k=[0, 584, 1224]) == want
    assert B.fp_workspace_bytes([0, 128], 8, 3) == 0            # invalid shape
    assert B.fp_workspace_bytes([0, 128], 8, 2, head_dim=80) == 0   # unsupported shape


def test_caller_workspace_is_checked_before_the_gpu_is_touched(lib):
    s, keep = B.make_shape([0, 1024], 4, 1)
    need = lib.fp_workspace_bytes(ctypes.byref(s))
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x10000)      # aligned, never dereferenced: the size check comes first
    assert lib.fp_plan_create_in(ctypes.byref(s), 0, fake, need - 1, ctypes.byref(h)) == B.FP_ERR_WORKSPACE
    assert lib.fp_plan_create_in(ctypes.byref(s), 0, ctypes.c_void_p(0x10010), need, ctypes.byref(h)) == B.FP_ERR_WORKSPACE
    assert not h.value


def test_largest_supported_sequence_is_accepted(lib):
    m, n, _ = B.fp_layout([0, 4096 * 128], 32, 4)
    assert (m, n) == (4096, 4096)


def test_layout_with_a_kv_prefix(lib):
    """Chunked prefill: rows count q-blocks, n_max counts key blocks; the prefix must be a block multiple."""
    m, n, ro = B.fp_layout([0, 200, 328], 8, 2, cu_seqlens_k=[0, 200 + 384, 200 + 384 + 128 + 512])
    assert (m, n) == (3, 5) and list(ro) == [0, 2, 3]
    assert (m, n, list(ro)) == (lambda r: (r[0], r[1], list(r[2])))(oracle_layout([0, 200, 328], [0, 584, 1224]))
    with pytest.raises(B.FlashPrefillError) as e:
        B.fp_layout([0, 200], 8, 2, cu_seqlens_k=[0, 300])
    assert e.value.status == B.FP_ERR_UNSUPPORTED
    with pytest.raises(B.FlashPrefillError) as e:
        B.fp_layout([0, 200], 8, 2, cu_seqlens_k=[0, 100])
    assert e.value.status == B.FP_ERR_INVALID_ARG
    with pytest.raises(B.FlashPrefillError) as e:
        B.fp_layout([0, 128], 8, 2, cu_seqlens_k=[0, 4097 * 128])
    assert e.value.status == B.FP_ERR_UNSUPPORTED


def oracle_layout(cu, cuk):
    import oracle
    return oracle.layout(cu, cu_seqlens_k=cuk)
