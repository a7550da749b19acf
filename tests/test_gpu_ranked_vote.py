"""The five-call selection with the vote launch that also builds the first histogram of
the TopK (ts_soft_vote_ranked + ts_topk with TS_TOPK_VOTE_HIST): the parity cases of test_gpu_decode_parity run again
that way (every stage against the oracle, the radix select bit-exact on the GPU's own votes), plus what is specific
to the pair: it agrees with ts_soft_vote + ts_topk, and it leaves the workspace as it found it."""
import numpy as np
import pytest

import parity_util
import workloads as W
from parity_util import compare_index_sets, oracle_decode
from test_gpu_decode_parity import (  # noqa: F401  (gpu is a fixture; the tests are collected here again)
    gpu, make_layer, test_config1_tiny_fp32, test_config2_shape_bf16_reduced_length, test_shapes,
    test_staged_runs_of_several_tiles, test_forced_initial_and_recent_tokens,
    test_ragged_batch_with_empty_and_short_sequences, test_large_batch_of_short_sequences,
    test_max_seq_len_larger_than_every_sequence, test_ties_go_to_lower_index_and_zero_query,
    test_topk_with_more_tied_candidates_than_one_batch, test_five_pass_topk_path_gives_the_same_result,
    test_k_larger_than_n_equals_full_attention, test_config2_full_size, test_config4_full_size)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def ranked_vote():
    parity_util.RANKED_VOTE = True
    yield
    parity_util.RANKED_VOTE = False


@pytest.mark.parametrize("shape", [(W.BF16, 32, 8, 128, [9000, 3333, 0, 17]), (W.BF16, 28, 4, 128, [70000]),
                                   (W.F32, 8, 2, 64, [5000, 1025, 1024, 1023]), (W.BF16, 128, 16, 128, [2500]),
                                   (W.F32, 6, 2, 64, [4100])], ids=lambda s: "dt%d_H%d_%d_D%d_%s" % s)
@pytest.mark.parametrize("forced", [(0, 0), (128, 512)], ids=["plain", "forced128+512"])
def test_ranked_pair_agrees_with_the_plain_pair_and_restores_the_workspace(gpu, shape, forced):
    from paper_2411_02886_amd.runtime import to_host
    dtype, H, H_kv, D, lens = shape
    ni, nl = forced
    w = W.make_workload("rv", dtype=dtype, B=len(lens), H=H, H_kv=H_kv, D=D, P=16, seq_lens=lens, k=200, beta=2.5,
                        planted_per_head=2, seed=sum(lens) + H)
    layer, q = make_layer(w, num_initial=ni, num_local=nl)
    print("ranked pair", shape, forced, flush=True)
    layer.select_compact(q, 1.0, None); torch.cuda.synchronize()
    idx_c = to_host(layer.idx).copy()
    layer.select(q, 1.0, None); torch.cuda.synchronize()
    v_p, st_p, idx_p, cnt_p = (to_host(x).copy() for x in (layer.votes, layer.row_stats, layer.idx, layer.count))
    for rep in range(2):                                 # twice: the second call starts from what the first one left
        layer.votes.fill_(-1.0); layer.idx.fill_(-9); layer.count.fill_(-9); layer.row_stats.fill_(0)
        layer.select(q, 1.0, None, ranked_vote=True); torch.cuda.synchronize()
        v_r, st_r, idx_r, cnt_r = (to_host(x).copy() for x in (layer.votes, layer.row_stats, layer.idx, layer.count))
        for b, N in enumerate(lens):
            if N == 0:
                continue
            # the same statistics merge and the same vote arithmetic: the same bits
            assert np.array_equal(st_r[b], st_p[b]) and np.array_equal(v_r[b, :N], v_p[b, :N]), (rep, b)
            assert np.all(v_r[b, N:] == -1.0)            # untouched past the sequence
            assert np.array_equal(idx_r[b], idx_p[b])
            compare_index_sets(idx_r[b], int(cnt_r[b]), oracle_decode(w, b, score_scale=1.0, n_init=ni, n_local=nl), "ranked b=%d" % b)
        # the radix select that started from the vote launch's histogram against the plain one on the same votes
        layer.idx.fill_(-9); layer.count.fill_(-9)
        gpu.ts_topk(layer.problem, layer.votes, layer.k, layer.idx, layer.count, None, layer.ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(layer.idx), idx_r) and np.array_equal(to_host(layer.count), cnt_r), rep
        assert np.array_equal(cnt_r, cnt_p)
    # the section the histogram lived in is shared with the compact form: it still gives what it gave before
    layer.idx.fill_(-9)
    layer.select_compact(q, 1.0, None); torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.idx), idx_c)
