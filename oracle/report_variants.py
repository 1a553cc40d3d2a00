"""Prints, for seeded synthetic inputs, what the paper's alternative block scorings (Sec. 3.3,
Tab. 1) and selection rules (Top-k, Top-p; Sec. 3.4, Tab. 8) would select compared with the
hot-path method (Eq. 1-4 scores + Alg. 2 threshold): density, agreement of the lists, and the share
of the exact attention mass the lists retain.  CPU only (oracle code); run as
    python -m oracle.report_variants [tokens ...]
The paper's accuracy columns need its benchmark suites and trained weights and are not reproduced.
"""
from __future__ import annotations

import dataclasses
import sys
import time

import numpy as np

import oracle
from oracle import variants as V
import synth


def report(tokens: int, mode: str) -> None:
    w = dataclasses.replace(synth.config(0, mode), seqlens=(tokens,), name=f"hq4_{tokens // 1024}k_{mode}")
    Q, K, _ = synth.make_qkv(w, threads=8)
    cu = w.cu_seqlens
    t0 = time.time()
    P3 = oracle.block_search(Q, K, cu)
    P2 = V.method2_scores(Q, K, cu)
    P1 = V.method1_scores(Q, K, cu)
    hot = oracle.threshold(P3, cu, w.alpha)
    m, n, _ = oracle.layout(cu)
    rows = set(range(0, m, max(1, m // 16))) | {m - 1}          # sampled rows for the mass column
    sel = {
        f"Eq.1-4 + threshold a={w.alpha} (hot path)": hot,
        f"method 2 + threshold a={w.alpha}": oracle.threshold(P2, cu, w.alpha),
        f"method 1 + threshold a={w.alpha}": oracle.threshold(P1, cu, w.alpha),
        "Eq.1-4 + top-8": V.select_topk(P3, cu, 8, sink_tokens=256, window_tokens=512),
        "method 2 + top-8": V.select_topk(P2, cu, 8, sink_tokens=256, window_tokens=512),
        "method 1 + top-8": V.select_topk(P1, cu, 8, sink_tokens=256, window_tokens=512),
        "Eq.1-4 + top-p 0.9": V.select_topp(P3, cu, 0.9, sink_tokens=256, window_tokens=512),
        "Eq.1-4 + top-p 0.99": V.select_topp(P3, cu, 0.99, sink_tokens=256, window_tokens=512),
    }
    print(f"\n### {w.name}: Hq={w.hq} Hkv={w.hkv} d=128, {tokens} tokens, {mode} planting")
    print("| scoring + selection | density | Jaccard vs hot path | hot-path pairs also kept | attention mass kept (sampled rows) |")
    print("|---|---|---|---|---|")
    for name, (idx, cnt) in sel.items():
        jac, rec = V.overlap(idx, cnt, *hot)
        mass = V.attention_mass(Q, K, cu, idx, cnt, rows=rows)
        print(f"| {name} | {100 * V.density(cnt, cu):.1f} % | {jac:.3f} | {100 * rec:.1f} % | {100 * mass:.2f} % |")
    print(f"(computed in {time.time() - t0:.1f} s on {oracle.num_threads()} threads)")


if __name__ == "__main__":
    sizes = [int(a) for a in sys.argv[1:]] or [4096, 16384]
    for t in sizes:
        report(t, "coherent")
    report(sizes[0], "literal")
