"""A sequence beyond 16 Mi tokens: the score pass runs with every workgroup walking hundreds of tile runs, the radix
select leaves its short form (whose finishing workgroup indexes at most 8192 chunks) for the five-pass form at its real
size, and the compact form must refuse the problem.  To keep the inputs small the page table draws its 1 Mi entries
from 16384 distinct pages, so every cached token has about 64 exact copies: the votes tie in large classes, and the
selection must cut the tie class of the k-th vote at the lowest token indices, as the oracle does."""
import dataclasses

import numpy as np
import pytest

import workloads as W
from parity_util import check_decode_against_oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    yield ts
    torch.cuda.empty_cache()


def test_decode_step_beyond_16_mi_tokens(gpu):
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device
    P, U, k = 16, 16384, 2048
    N = (1 << 24) + 5000 + 7                      # ragged last page and last tile
    print("long sequence", N, flush=True)
    base = W.make_workload("long_seq_pages", dtype=W.BF16, H=2, H_kv=1, D=64, P=P, seq_lens=[U * P], k=k, beta=2.0,
                           planted_per_head=4, seed=2024)
    rng = np.random.default_rng(7)
    npages = (N + P - 1) // P
    table = rng.integers(0, U, size=npages).astype(np.int32)
    w = dataclasses.replace(base, seq_lens=np.array([N], dtype=np.int32), page_indptr=np.array([0, npages], dtype=np.int32),
                            page_indices=table, planted=[])
    layer = DecodeLayer.from_workload(w)
    q = to_device(w.q)
    exc = check_decode_against_oracle(w, layer, q, score_scale=0.125, label="beyond 16 Mi tokens")
    assert exc == []                              # ties are exact copies: nothing for the band rule to tolerate
    # the compact form's finish cannot index that many chunks: refused before any launch (the votes stand in for bounds)
    with pytest.raises(gpu.TokenSelectError) as err:
        gpu.ts_topk_exact(layer.problem, q, layer.votes, layer.row_stats, 0.125, layer.k, layer.idx, layer.count, None, layer.ws)
    assert err.value.status == -2
    del layer
    torch.cuda.empty_cache()
