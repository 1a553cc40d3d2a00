"""Pins for the oracle's max-based dynamic threshold and index compression (Sec. 3.4, Alg. 2)."""
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "threshold_worked_example.txt")


def _load_golden():
    rows, cases, cur = {}, [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.replace(":", " ").split()
        if tok[0] == "row":
            rows[int(tok[1])] = [float(x) for x in tok[2:]]
        elif tok[0] == "case":
            cur = dict(alpha=float(tok[1]), sink=int(tok[2]), window=int(tok[3]), expect={})
            cases.append(cur)
        elif tok[0] == "expect":
            cur["expect"][int(tok[1])] = [int(x) for x in tok[2:]]
    return rows, cases


def test_hand_worked_example():
    rows, cases = _load_golden()
    n = 10
    scores = np.zeros((1, n, n), np.float32)
    for I in range(n):
        scores[0, I, :I + 1] = rows.get(I, [1.0 / (I + 1)] * (I + 1))
    for c in cases:
        idx, cnt = oracle.threshold(scores, [0, 1280], c["alpha"], sink_tokens=c["sink"], window_tokens=c["window"])
        for I, want in c["expect"].items():
            assert cnt[0, I] == len(want), (c, I)
            assert idx[0, I, :cnt[0, I]].tolist() == want, (c, I)
            assert np.all(idx[0, I, cnt[0, I]:] == n)            # Alg. 2 fills inactive slots with N


def _random_scores(hq, n, seed):
    g = np.random.default_rng(seed)
    s = g.pareto(1.2, size=(hq, n, n)).astype(np.float32)         # long-tailed rows, as in Fig. 7's premise
    s *= np.tril(np.ones((n, n), np.float32))
    return s / s.sum(axis=2, keepdims=True)


def _lists(idx, cnt, h, r):
    return idx[h, r, :cnt[h, r]]


def test_structural_invariants_and_always_kept_blocks():
    n, hq = 48, 3
    scores = _random_scores(hq, n, 0)
    idx, cnt = oracle.threshold(scores, [0, n * 128], 0.12)
    for h in range(hq):
        for I in range(n):
            l = _lists(idx, cnt, h, I)
            assert l.size >= 1 and np.all(np.diff(l) > 0)              # ascending, duplicate-free
            assert l[0] >= 0 and l[-1] <= I                            # in range, causal
            must = set(range(min(2, I + 1))) | set(range(max(0, I - 3), I + 1)) | {int(np.argmax(scores[h, I, :I + 1]))}
            assert must <= set(l.tolist())
            assert cnt[h, I] >= min(I + 1, 6)
    # something is actually pruned on long-tailed rows
    assert cnt.sum() < 0.8 * hq * n * (n + 1) / 2


def test_alpha_nesting_and_extremes():
    n = 40
    scores = _random_scores(2, n, 1)
    cu = [0, n * 128]
    prev = None
    for alpha in (0.0, 0.05, 0.12, 0.5, 1.0):
        idx, cnt = oracle.threshold(scores, cu, alpha)
        cur = [[set(_lists(idx, cnt, h, I).tolist()) for I in range(n)] for h in range(2)]
        if prev is not None:
            assert all(cur[h][I] <= prev[h][I] for h in range(2) for I in range(n))
        prev = cur
    idx0, cnt0 = oracle.threshold(scores, cu, 0.0)
    assert np.array_equal(cnt0, np.tile(np.arange(1, n + 1, dtype=np.int32), (2, 1)))
    idxn, cntn = oracle.threshold(scores, cu, -1.0)
    assert np.array_equal(cntn, cnt0) and np.array_equal(idxn, idx0)
    idx1, cnt1 = oracle.threshold(scores, cu, 1.0, sink_tokens=0, window_tokens=0)
    for h in range(2):
        for I in range(n):
            assert _lists(idx1, cnt1, h, I).tolist() == [int(np.argmax(scores[h, I, :I + 1]))]


def test_lists_do_not_depend_on_row_normalisation():
    # The rule compares each score with alpha times the row max, so scaling a row by a power of
    # two (exact in fp32) must not change its list: lists from S' and from P agree.
    n = 32
    scores = _random_scores(2, n, 2)
    a = oracle.threshold(scores, [0, n * 128], 0.12)
    b = oracle.threshold((scores * np.float32(64.0)), [0, n * 128], 0.12)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_upper_triangle_is_never_listed_even_if_nonzero():
    n = 16
    g = np.random.default_rng(3)
    scores = g.random((1, n, n)).astype(np.float32)                  # garbage above the diagonal
    idx, cnt = oracle.threshold(scores, [0, n * 128], 0.12)
    for I in range(n):
        assert _lists(idx, cnt, 0, I).max() <= I


def test_varlen_rows_use_their_own_sequence():
    lens = [1024, 300, 2048]
    cu = np.concatenate([[0], np.cumsum(lens)])
    m_total, n_max, ro = synth.layout(cu)
    g = np.random.default_rng(4)
    scores = g.pareto(1.0, size=(2, m_total, n_max)).astype(np.float32)
    idx, cnt = oracle.threshold(scores, cu, 0.2)
    for s in range(3):
        sub = np.ascontiguousarray(scores[:, ro[s]:ro[s + 1], :ro[s + 1] - ro[s]])
        i2, c2 = oracle.threshold(sub, [0, lens[s]], 0.2)
        assert np.array_equal(cnt[:, ro[s]:ro[s + 1]], c2)
        for h in range(2):
            for I in range(ro[s + 1] - ro[s]):
                assert np.array_equal(_lists(idx, cnt, h, ro[s] + I), _lists(i2, c2, h, I))
