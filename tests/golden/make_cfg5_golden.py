#!/usr/bin/env python3
"""Writes tests/golden/cfg5_chunk_selection.txt: the oracle's chunked-prefill selection (Sec. 5.2 with per-query
Eq. 5 votes summed over heads and over the chunk's queries) on configuration 5 at full size -- 512 queries x 262144
cached tokens, 32 query heads over 8 KV heads, head_dim 128, k = 4096.

Calls only the CPU oracle and the seeded input generator (about 5e11 fp64 multiply-adds: minutes on 8-16 cores).
Stored: the index set and count; the votes of the 512 tokens ranked k-256 .. k+255 (the band rule of the parity
tests needs the votes around the k-th one); the natural log-sum-exp of all 512 x 32 softmax rows; the vote total.

Usage: python tests/golden/make_cfg5_golden.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle            # noqa: E402
import workloads as W    # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg5_chunk_selection.txt")


def main():
    w = W.config5()
    N = int(w.extra["n_cached"])
    C, H = w.C, w.H
    votes = np.zeros(N, dtype=np.float64)
    lse = np.zeros((C, H), dtype=np.float64)
    t0 = time.time()
    for c in range(C):
        S = oracle.paged_qk_scores(np.ascontiguousarray(w.q[0, c]), w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N)
        v, m, z = oracle.soft_vote(S, 1.0, with_stats=True)
        votes += v
        lse[c] = m + np.log(z)
        if c % 32 == 31:
            print("query %d of %d, %.0f s" % (c + 1, C, time.time() - t0), flush=True)
    idx, cnt = oracle.topk(oracle.decision_votes(votes), w.k)
    order = np.argsort(-votes, kind="stable")
    band = order[max(0, cnt - 256):cnt + 256]
    with open(OUT, "w") as f:
        f.write("# oracle selection of configuration 5 (seed %d): Sec. 5.2 with per-query Eq. 5 votes, k = %d\n" % (w.seed, w.k))
        f.write("# written by tests/golden/make_cfg5_golden.py (CPU oracle only)\n")
        f.write("cached_tokens %d\nchunk %d\nheads %d\ncount %d\nvote_total %.17g\n" % (N, C, H, cnt, float(votes.sum())))
        f.write("idx %d\n" % cnt)
        f.write(" ".join(str(int(t)) for t in idx[:cnt]) + "\n")
        f.write("band %d\n" % len(band))
        for t in band:
            f.write("%d %.17g\n" % (int(t), float(votes[t])))
        f.write("lse %d %d\n" % (C, H))
        for c in range(C):
            f.write(" ".join("%.17g" % x for x in lse[c]) + "\n")
    print("wrote", OUT, "in %.0f s" % (time.time() - t0))


if __name__ == "__main__":
    main()
