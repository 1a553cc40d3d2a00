"""Host-side checks of the seeded input generators and of the three independent row-layout
implementations (generator module, oracle, C ABI)."""
import numpy as np
import pytest

import oracle
from paper_2603_06199_amd import binding as B
import synth


def test_bf16_rounding_is_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40, 0.0], np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1 + 2^-7 and 1 + 2^-6: goes to 1 + 2^-6 (even)
    back = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625) and back[3] == -2.5
    # every bf16 value survives a round trip
    bits = np.arange(0, 0x7F80, 97, dtype=np.uint16)
    assert np.array_equal(synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(bits)), bits)


def test_generation_is_deterministic_and_seed_dependent():
    w = synth.small("det", [640, 300], hq=4, hkv=2, seed=3)
    a = synth.make_qkv(w, threads=1)
    b = synth.make_qkv(w, threads=4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    c = synth.make_qkv(synth.small("det", [640, 300], hq=4, hkv=2, seed=4))
    assert not np.array_equal(a[0], c[0])


def test_sequences_of_a_packed_batch_are_generated_independently():
    w = synth.small("pack", [512, 384], hq=2, hkv=1, seed=5)
    Q, K, V = synth.make_qkv(w)
    assert Q.shape == (896, 2, 128) and K.shape == V.shape == (896, 1, 128)
    # streams are keyed by the sequence index and positions restart at each sequence, so the
    # second sequence does not depend on the length of the first
    w2 = synth.small("pack", [256, 384], hq=2, hkv=1, seed=5)
    Q2, K2, V2 = synth.make_qkv(w2)
    assert np.array_equal(Q[512:], Q2[256:]) and np.array_equal(K[512:], K2[256:]) and np.array_equal(V[512:], V2[256:])
    assert not np.array_equal(Q[:256], Q[512:768])


@pytest.mark.parametrize("cu", [[0, 128], [0, 5], [0, 300, 1000, 1128], [0, 4096, 20480, 86016, 217088]])
def test_three_layout_implementations_agree(cu):
    a = synth.layout(cu)
    b = oracle.layout(cu)
    c = B.fp_layout(cu, 8, 2)
    assert a[0] == b[0] == c[0] and a[1] == b[1] == c[1]
    assert np.array_equal(a[2], b[2]) and np.array_equal(a[2], c[2])


def test_forced_density_lists_are_valid_and_near_target():
    cu = [0, 8192, 8192 + 6000]
    idx, cnt = synth.forced_density_lists(cu, hq=2, density=0.3, seed=1)
    m_total, n_max, ro = synth.layout(cu)
    kept = 0
    for s in range(2):
        for I in range(ro[s + 1] - ro[s]):
            for h in range(2):
                l = idx[h, ro[s] + I, :cnt[h, ro[s] + I]]
                assert np.all(np.diff(l) > 0) and l[0] >= 0 and l[-1] <= I
                assert set(range(min(2, I + 1))) <= set(l.tolist()) and set(range(max(0, I - 3), I + 1)) <= set(l.tolist())
                kept += l.size
    total = sum((ro[s + 1] - ro[s]) * (ro[s + 1] - ro[s] + 1) // 2 for s in range(2)) * 2
    assert 0.3 < kept / total < 0.6      # 0.3 plus the always-kept sink and window blocks


def test_benchmark_configurations_have_the_stated_shapes():
    shapes = [(4096, 4, 1), (32768, 32, 4), (131072, 32, 4), (262144, 32, 4), (217088, 32, 8)]
    for i, (T, hq, hkv) in enumerate(shapes):
        for mode in ("literal", "coherent"):
            w = synth.config(i, mode)
            assert (w.total_tokens, w.hq, w.hkv, w.head_dim) == (T, hq, hkv, 128)
    assert synth.config(4).seqlens == (4096, 16384, 65536, 131072) and synth.config(4).alpha == 0.18
    assert synth.config(3).alpha == 0.12
