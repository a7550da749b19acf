"""Pins for the CPU oracle: each checks it against something other than itself -- a textbook
library routine on un-paged data, a closed form, an invariant, brute force on tiny inputs, a
hand-worked example (tests/golden/), or a trace of Algorithm 1 written out by hand."""
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle
import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny(dtype=W.F32, N=200, H=4, H_kv=2, D=16, P=4, seed=3, **kw):
    return W.make_workload("tiny", dtype=dtype, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[N], k=8, seed=seed, **kw)


def unpaged(w, b=0):
    """Logical [N][H_kv][D] float64 K and V gathered with numpy fancy indexing."""
    slots = w.slots_of(b)
    K = W.as_f32(w.k_pool, w.dtype).reshape(-1, w.H_kv, w.D)[slots].astype(np.float64)
    V = W.as_f32(w.v_pool, w.dtype).reshape(-1, w.H_kv, w.D)[slots].astype(np.float64)
    Q = W.as_f32(w.q, w.dtype)[b, 0].astype(np.float64)
    return Q, K, V


# ---------------------------------------------------------------- Algorithm 2: paged scores

@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
@pytest.mark.parametrize("N,P", [(200, 4), (37, 16), (1, 16), (64, 1)])
def test_scores_match_einsum_on_unpaged(dtype, N, P):
    w = tiny(dtype=dtype, N=N, P=P)
    Q, K, _ = unpaged(w)
    Kh = np.repeat(K, w.G, axis=1)                       # kv(h) = h // G: contiguous groups
    ref = np.einsum("hd,nhd->hn", Q, Kh)
    S = oracle.paged_qk_scores(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N)
    np.testing.assert_allclose(S, ref, rtol=0, atol=1e-12)


def test_scores_gqa_mapping_is_contiguous_groups():
    # K of KV head 1 is zero: exactly the query heads of the second group must score 0.
    w = tiny(H=6, H_kv=2)
    w.k_pool[:, :, 1, :] = 0
    S = oracle.paged_qk_scores(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 200)
    assert np.all(S[3:] == 0) and np.all(np.abs(S[:3]).max(axis=1) > 0)


def test_scores_paging_invariance():
    a = tiny(seed=11, identity_pages=True)
    b = tiny(seed=11, identity_pages=False, extra_pool_pages=5)
    # same seed draws different streams once the permutation is drawn, so rebuild b's pool from a's logical data
    la = W.as_f32(a.k_pool, a.dtype).reshape(-1, a.H_kv, a.D)[a.slots_of(0)]
    b.k_pool.reshape(-1, b.H_kv, b.D)[b.slots_of(0)] = la
    b.q[:] = a.q
    Sa = oracle.paged_qk_scores(a.q[0, 0], a.k_pool, a.dtype, a.H_kv, a.P, a.pages_of(0), 200)
    Sb = oracle.paged_qk_scores(b.q[0, 0], b.k_pool, b.dtype, b.H_kv, b.P, b.pages_of(0), 200)
    assert not np.array_equal(a.pages_of(0), b.pages_of(0))
    assert np.array_equal(Sa, Sb)


def test_bf16_widening_is_exact():
    w = tiny(dtype=W.BF16, N=16, H=2, H_kv=1, D=4)
    w.q[:] = 0
    w.q[0, 0, 0, 2] = 0x3F80            # 1.0 in bf16
    S = oracle.paged_qk_scores(w.q[0, 0], w.k_pool, w.dtype, 1, w.P, w.pages_of(0), 16)
    _, K, _ = unpaged(w)
    assert np.array_equal(S[0], K[:, 0, 2]) and np.all(S[1] == 0)


# ---------------------------------------------------------------- Eq. 5: head soft vote

def test_soft_vote_matches_scipy_softmax_and_invariants():
    rng = np.random.default_rng(5)
    S = rng.normal(size=(6, 333)) * 7
    for c in (1.0, 0.125):
        v, m, z = oracle.soft_vote(S, c, with_stats=True)
        np.testing.assert_allclose(v, sp_softmax(c * S, axis=1).sum(axis=0), rtol=1e-13, atol=0)
        assert abs(v.sum() - 6.0) < 1e-12                 # every per-head softmax sums to one
        assert np.all(v > 0) and np.all(v <= 6.0)
        np.testing.assert_allclose(m, (c * S).max(axis=1), rtol=0, atol=0)
        np.testing.assert_allclose(z, np.exp(c * S - m[:, None]).sum(axis=1), rtol=1e-13)
    one = oracle.soft_vote(S[:1], 1.0)
    assert abs(one.sum() - 1.0) < 1e-13
    # adding a constant to one head's scores changes nothing
    S2 = S.copy(); S2[2] += 11.5
    np.testing.assert_allclose(oracle.soft_vote(S2, 1.0), oracle.soft_vote(S, 1.0), rtol=1e-12)
    # closed form: scale 0 -> every head votes 1/N for every token
    np.testing.assert_allclose(oracle.soft_vote(S, 0.0), np.full(333, 6.0 / 333), rtol=1e-14)


def test_soft_vote_is_a_sum_over_heads_not_over_tokens():
    # a transposed reduction would give 1 for every head instead
    S = np.array([[0.0, math.log(3.0)], [0.0, 0.0], [math.log(7.0), 0.0]])
    v = oracle.soft_vote(S, 1.0)
    np.testing.assert_allclose(v, [0.25 + 0.5 + 0.875, 0.75 + 0.5 + 0.125], rtol=1e-14)


# ---------------------------------------------------------------- TopK

def brute_topk(v, k):
    v = list(v); chosen = []
    for _ in range(min(k, len(v))):
        best = None
        for i, x in enumerate(v):
            if i in chosen:
                continue
            if best is None or x > v[best]:
                best = i                                   # strict '>' keeps the lowest index among equals
        chosen.append(best)
    return sorted(chosen)


@pytest.mark.parametrize("seed", range(6))
def test_topk_vs_brute_force(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(1, 64)); k = int(rng.integers(1, 70))
    v = rng.integers(0, 6, size=N).astype(np.float64)      # many ties
    idx, cnt = oracle.topk(v, k)
    assert cnt == min(k, N)
    assert list(idx[:cnt]) == brute_topk(v, k)
    assert np.all(idx[cnt:] == -1)


def test_topk_ties_lower_index_and_k_ge_n():
    v = np.array([1.0, 5.0, 5.0, 2.0, 5.0, 5.0])
    idx, cnt = oracle.topk(v, 3)
    assert list(idx) == [1, 2, 4] and cnt == 3
    idx, cnt = oracle.topk(v, 9)
    assert list(idx[:6]) == [0, 1, 2, 3, 4, 5] and cnt == 6 and np.all(idx[6:] == -1)
    idx, cnt = oracle.topk(np.zeros(5), 2)
    assert list(idx) == [0, 1]


def test_single_head_soft_vote_topk_equals_argsort_of_raw_logits():
    # H = 1: Eq. 5 reduces to Eq. 3 because softmax is monotone
    w = tiny(H=1, H_kv=1, N=500, seed=9)
    idx, cnt, votes, S = oracle.select(w.q[0, 0], w.k_pool, w.dtype, 1, w.P, w.pages_of(0), 500, 25, details=True)
    Q, K, _ = unpaged(w)
    raw = K[:, 0, :] @ Q[0]
    assert sorted(np.argsort(-raw, kind="stable")[:25].tolist()) == idx.tolist()


# ---------------------------------------------------------------- Algorithm 1: Selection Cache

def test_selection_cache_trace():
    D = 8
    e = np.eye(D, dtype=np.float32)
    cq = np.zeros((1, D), dtype=np.float32)
    first = np.ones(1, dtype=np.uint8)
    cidx = np.full(2, -7, dtype=np.int32); ccnt = np.zeros(1, dtype=np.int32)
    calls = []

    def sel(q):
        calls.append(q.copy())
        return np.array([len(calls), 10 * len(calls)], dtype=np.int32), 2

    th = 0.9
    # step 0: first flag set -> always select, state updated
    i, c, r = oracle.selcache_step(e[0:1].copy(), cq, cidx, ccnt, first, th, sel)
    assert (not r) and list(i) == [1, 10] and first[0] == 0 and np.array_equal(cq, e[0:1])
    # step 1: positive multiple of cached query -> cos = 1 -> reuse, cached state untouched
    i, c, r = oracle.selcache_step(3 * e[0:1], cq, cidx, ccnt, first, th, sel)
    assert r and list(i) == [1, 10] and np.array_equal(cq, e[0:1]) and len(calls) == 1
    # step 2: cos = 0.9055 (>= 0.9) -> reuse
    q = (e[0:1] + 0.4685 * e[1:2]).astype(np.float32)
    assert 0.9 < oracle.cosine(q, cq, W.F32) < 0.91
    i, c, r = oracle.selcache_step(q, cq, cidx, ccnt, first, th, sel)
    assert r and len(calls) == 1
    # step 3: cos = 0.894 (< 0.9) -> reselect; C_Q becomes this query (anchor = last miss)
    q3 = (e[0:1] + 0.5 * e[1:2]).astype(np.float32)
    i, c, r = oracle.selcache_step(q3, cq, cidx, ccnt, first, th, sel)
    assert (not r) and list(i) == [2, 20] and np.array_equal(cq, q3)
    # step 4: orthogonal -> miss; opposite -> miss (cos = -1)
    i, c, r = oracle.selcache_step(e[2:3].copy(), cq, cidx, ccnt, first, th, sel)
    assert not r
    i, c, r = oracle.selcache_step(-e[2:3], cq, cidx, ccnt, first, th, sel)
    assert (not r) and len(calls) == 4
    # threshold exactly met counts as reuse (reselect only when cos < theta)
    i, c, r = oracle.selcache_step(-e[2:3], cq, cidx, ccnt, first, 1.0, sel)
    assert r
    # zero query: cosine defined as 0 -> miss for theta > 0
    i, c, r = oracle.selcache_step(np.zeros((1, D), np.float32), cq, cidx, ccnt, first, th, sel)
    assert not r


def test_selection_cache_threshold_extremes():
    rng = np.random.default_rng(2)
    qs = rng.normal(size=(10, 4, 8)).astype(np.float32)
    for theta, expect in ((1.0 + 1e-9, [False] * 10), (-1.0, [False] + [True] * 9)):
        cq = np.zeros((4, 8), np.float32); first = np.ones(1, np.uint8)
        cidx = np.zeros(1, np.int32); ccnt = np.zeros(1, np.int32); n = [0]

        def sel(q):
            n[0] += 1
            return np.array([n[0]], np.int32), 1
        got = [oracle.selcache_step(qs[t].copy(), cq, cidx, ccnt, first, theta, sel)[2] for t in range(10)]
        assert got == expect


def test_cosine_matches_numpy():
    rng = np.random.default_rng(4)
    a = rng.normal(size=(32, 128)).astype(np.float32); b = (0.9 * a + 0.3 * rng.normal(size=a.shape)).astype(np.float32)
    ref = float((a.astype(np.float64) * b).sum() / np.linalg.norm(a.astype(np.float64)) / np.linalg.norm(b.astype(np.float64)))
    assert abs(oracle.cosine(a, b, W.F32) - ref) < 1e-14


# ---------------------------------------------------------------- Eq. 1 / Eq. 2: attention

def numpy_attention(Q, K, V, G, tokens, scale):
    out = np.zeros_like(Q)
    for h in range(Q.shape[0]):
        logits = K[tokens, h // G, :] @ Q[h] * scale
        out[h] = sp_softmax(logits) @ V[tokens, h // G, :]
    return out


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_full_attention_matches_numpy(dtype):
    w = tiny(dtype=dtype, N=150)
    Q, K, V = unpaged(w)
    ref = numpy_attention(Q, K, V, w.G, np.arange(150), 0.25)
    got = oracle.full_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 150, 0.25)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_sparse_attention_matches_numpy_on_subset_and_extra_tokens():
    w = tiny(N=150)
    Q, K, V = unpaged(w)
    idx = np.array([3, 17, 18, 99, 140], dtype=np.int32)
    got, lse = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), idx, 5, 0.25,
                                  with_lse=True)
    np.testing.assert_allclose(got, numpy_attention(Q, K, V, w.G, idx, 0.25), rtol=1e-12, atol=1e-13)
    for h in range(w.H):
        ref = np.log(np.exp(K[idx, h // w.G, :] @ Q[h] * 0.25).sum())
        assert abs(lse[h] - ref) < 1e-12
    # Eq. 2's [K_select, K_current]: the appended tokens join the same softmax
    got2 = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), idx, 5, 0.25,
                              extra_first=145, n_extra=3)
    ref2 = numpy_attention(Q, K, V, w.G, np.array([3, 17, 18, 99, 140, 145, 146, 147]), 0.25)
    np.testing.assert_allclose(got2, ref2, rtol=1e-12, atol=1e-13)


def test_selecting_everything_is_full_attention_bitwise():
    w = tiny(N=123)
    idx, cnt = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 123, 500)
    assert cnt == 123 and list(idx[:123]) == list(range(123))
    a = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), idx, cnt, 0.25)
    b = oracle.full_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 123, 0.25)
    assert np.array_equal(a, b)


def test_attention_special_cases():
    w = tiny(N=40)
    _, _, V = unpaged(w)
    one = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), np.array([7], np.int32), 1, 0.3)
    np.testing.assert_allclose(one, np.repeat(V[7], w.G, axis=0), rtol=1e-15)
    w.k_pool[:] = 1.0                                       # all keys equal -> uniform weights
    idx = np.array([1, 5, 9, 30], np.int32)
    mean = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), idx, 4, 0.3)
    np.testing.assert_allclose(mean, np.repeat(V[idx].mean(axis=0), w.G, axis=0), rtol=1e-13)


# ---------------------------------------------------------------- worked example, planted tokens, Def. 1 objective, Lemma 1

def test_hand_worked_example():
    gold = {}
    for line in open(os.path.join(GOLD, "hand_example_eq5_eq2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        gold[key] = [float(x) for x in vals]
    q = np.array([[1, 0], [0, 1]], np.float32)
    kp = np.array([[math.log(2), 0], [0, math.log(3)], [0, 0]], np.float32).reshape(3, 1, 1, 2)
    vp = np.array([[3, 0], [0, 3], [7, 7]], np.float32).reshape(3, 1, 1, 2)
    pages = np.arange(3, dtype=np.int32)
    idx, cnt, votes, S = oracle.select(q, kp, W.F32, 1, 1, pages, 3, 2, details=True)
    np.testing.assert_allclose(votes, gold["votes"], atol=2e-7)
    assert idx.tolist() == [int(x) for x in gold["topk2"]]
    out = oracle.sparse_attn(q, kp, vp, W.F32, 1, 1, pages, idx, cnt, 1.0)
    np.testing.assert_allclose(out[0], gold["out_head0"], atol=1e-6)
    np.testing.assert_allclose(out[1], gold["out_head1"], atol=1e-6)


def test_planted_tokens_are_selected_when_strongly_boosted():
    # boost 8, H * n_planted == k: the selected set is exactly the planted set
    w = W.config1(seed=21, N=1024, beta=8.0, planted_per_head=8, k=64)
    idx, cnt = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 1024, 64)
    assert sorted(np.concatenate(list(w.planted[0])).tolist()) == idx.tolist()


def test_error_vanishes_as_k_reaches_n():
    w = tiny(N=256, seed=13)
    full = oracle.full_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 256, 0.25)
    errs = []
    for k in (8, 64, 192, 256):
        idx, cnt = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 256, k, score_scale=0.25)
        o = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), idx, cnt, 0.25)
        errs.append(float(((o - full) ** 2).sum()))
    assert errs[0] > errs[1] > errs[2] > errs[3] == 0.0


def test_lemma1_positive_multiple_and_sufficient_bound():
    # Lemma 1 with one head: q2 = c*q1 (cos = 1) selects the same set; and any q2 whose cosine
    # with q1 satisfies the lemma's sufficient bound selects the same set.
    rng = np.random.default_rng(17)
    N, D, k = 60, 8, 5
    w = W.make_workload("l1", dtype=W.F32, H=1, H_kv=1, D=D, P=4, seq_lens=[N], k=k, seed=17)
    q1 = w.q[0, 0].copy()
    base, _ = oracle.select(q1, w.k_pool, w.dtype, 1, w.P, w.pages_of(0), N, k)
    again, _ = oracle.select((2.5 * q1).astype(np.float32), w.k_pool, w.dtype, 1, w.P, w.pages_of(0), N, k)
    assert base.tolist() == again.tolist()
    Q, K, _ = unpaged(w)
    s = np.sort(K[:, 0, :] @ Q[0])[::-1]
    eta_hat = (s[k - 1] - s[k]) / np.linalg.norm(Q[0])
    kmax = np.linalg.norm(K[:, 0, :], axis=1).max()
    bound = 1.0 / math.sqrt(1.0 + (eta_hat / (2 * kmax)) ** 2)
    for _ in range(50):
        p = rng.normal(size=D); p -= p @ Q[0] / (Q[0] @ Q[0]) * Q[0]; p /= np.linalg.norm(p)
        ang = math.acos(bound) * rng.uniform(0, 0.999)
        q2 = (math.cos(ang) * Q[0] / np.linalg.norm(Q[0]) + math.sin(ang) * p).astype(np.float32)
        got, _ = oracle.select(q2.reshape(1, D), w.k_pool, w.dtype, 1, w.P, w.pages_of(0), N, k)
        assert got.tolist() == base.tolist()


def test_chunk_selection_sums_votes_over_queries():
    w = W.make_workload("c", dtype=W.F32, C=3, H=4, H_kv=2, D=16, P=4, seq_lens=[90], k=10, seed=8)
    idx, cnt, votes = oracle.select_chunk(w.q[0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 80, 10, details=True)
    assert abs(votes.sum() - 3 * 4) < 1e-12
    ref = sum(oracle.soft_vote(oracle.paged_qk_scores(np.ascontiguousarray(w.q[0, c]), w.k_pool, w.dtype, w.H_kv, w.P,
                                                      w.pages_of(0), 80)) for c in range(3))
    assert brute_topk(ref.astype(np.float32), 10) == idx.tolist()


# ---------------------------------------------------------------- forced tokens (Sec. 6.1: 128 initial + n_local recent)

def test_ranked_range_cases():
    assert oracle.ranked_range(1000, 0, 0) == (0, 1000)
    assert oracle.ranked_range(1000, 128, 512) == (128, 488)
    assert oracle.ranked_range(600, 128, 512) == (128, 128)      # blocks overlap: nothing left to rank
    assert oracle.ranked_range(100, 128, 512) == (100, 100)      # the initial block alone covers the sequence
    assert oracle.ranked_range(0, 128, 512) == (0, 0)


@pytest.mark.parametrize("n_init,n_local", [(5, 0), (0, 9), (7, 11)])
def test_forced_tokens_selection_is_plain_selection_on_the_middle(n_init, n_local):
    """Ranking [lo, hi) of a sequence must be the plain selection applied to a sequence that holds only
    those tokens (built here from un-paged copies), shifted by lo -- an independent route to the result."""
    N, k = 97, 12
    w = tiny(N=N, P=1, seed=21)                       # one token per page: any sub-range is a page list
    idx, cnt, votes, S = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, k, details=True,
                                       n_init=n_init, n_local=n_local)
    lo, hi = n_init, N - n_local
    sub_pages = w.pages_of(0)[lo:hi]
    idx2, cnt2, votes2, _ = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, sub_pages, hi - lo, k, details=True)
    assert cnt == cnt2 == k
    assert (idx[:cnt] - lo).tolist() == idx2[:cnt2].tolist()
    np.testing.assert_array_equal(votes[lo:hi], votes2)
    assert not votes[:lo].any() and not votes[hi:].any()
    assert abs(votes.sum() - w.H) < 1e-12             # each head's softmax runs over the ranked range only
    # and against numpy directly
    ref = sp_softmax(S[:, lo:hi], axis=1).sum(axis=0)
    assert brute_topk(ref.astype(np.float32), k) == (idx[:cnt] - lo).tolist()


def test_forced_tokens_attended_list_and_degenerate_cases():
    N = 60
    w = tiny(N=N, seed=22)
    idx, cnt = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 6, n_init=4, n_local=10)
    att = oracle.attended_tokens(idx, cnt, N, 4, 10)
    assert att.tolist() == list(range(4)) + idx[:cnt].tolist() + list(range(50, 60))
    assert len(set(att.tolist())) == len(att) and np.all(np.diff(att) > 0)       # disjoint blocks, ascending
    # a selection cached at N = 60 used at N = 63: the recent block follows the current length, the rest stays
    att2 = oracle.attended_tokens(idx, cnt, 63, 4, 10)
    assert att2.tolist() == list(range(4)) + idx[:cnt].tolist() + list(range(53, 63))
    # forced blocks that cover the sequence: nothing is ranked and Eq. 2 becomes Eq. 1 (bitwise: same order)
    idx0, cnt0 = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 6, n_init=30, n_local=40)
    assert cnt0 == 0
    att0 = oracle.attended_tokens(idx0, cnt0, N, 30, 40)
    assert att0.tolist() == list(range(N))
    a = oracle.sparse_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), att0, N, 0.25)
    b = oracle.full_attn(w.q[0, 0], w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 0.25)
    assert np.array_equal(a, b)
    # no forced tokens: unchanged behaviour
    i1, c1 = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 6)
    i2, c2 = oracle.select(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 6, n_init=0, n_local=0)
    assert c1 == c2 and i1.tolist() == i2.tolist()
    assert oracle.attended_tokens(i1, c1, N).tolist() == i1[:c1].tolist()


# ---------------------------------------------------------------- Sec. 5.2: chunk selection with the mean query

def test_mean_query_matches_numpy_and_rounds_to_nearest_even():
    rng = np.random.Generator(np.random.PCG64(5))
    q32 = rng.standard_normal((7, 3, 16), dtype=np.float32)
    np.testing.assert_array_equal(oracle.mean_query(q32, W.F32), q32.astype(np.float64).mean(axis=0).astype(np.float32))
    qb = W.store(q32, W.BF16)
    m = oracle.mean_query(qb, W.BF16)
    exact = W.as_f32(qb, W.BF16).astype(np.float64).mean(axis=0)
    got = W.as_f32(m, W.BF16).astype(np.float64)
    assert m.dtype == np.uint16
    # nearest: within half a bf16 ulp (8 significant bits: ulp = 2^(floor(log2|x|) - 7)) of the exact mean
    half_ulp = 0.5 * 2.0 ** (np.floor(np.log2(np.abs(exact))) - 7)
    assert np.all(np.abs(got - exact) <= half_ulp * (1 + 1e-6))
    # constructed halfway cases: mean of {1, 1 + 2^-7} = 1 + 2^-8 is halfway between bf16 neighbours -> even (1.0);
    # mean of {1 + 2^-7, 1 + 2^-6} = 1 + 3 * 2^-8 -> halfway again -> even mantissa (1 + 2^-6)
    vals = np.array([[1.0, 1.0 + 2.0 ** -7], [1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6]], dtype=np.float32)   # [case][c]
    qh = W.store(np.ascontiguousarray(vals.T).reshape(2, 1, 2), W.BF16)            # C = 2, H = 1, D = 2
    mh = W.as_f32(oracle.mean_query(qh, W.BF16), W.BF16).reshape(2)
    assert mh[0] == np.float32(1.0) and mh[1] == np.float32(1.0 + 2.0 ** -6)


def test_mean_query_selection_special_cases():
    w = W.make_workload("c", dtype=W.BF16, C=4, H=4, H_kv=2, D=16, P=4, seq_lens=[90], k=10, seed=9)
    N = 86
    # a chunk of one query, or of identical queries, is the decode selection with that query
    q1 = np.ascontiguousarray(w.q[0, :1])
    a = oracle.select_chunk_mean_query(q1, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 10)
    b = oracle.select(np.ascontiguousarray(w.q[0, 0]), w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 10)
    assert a[1] == b[1] and a[0].tolist() == b[0].tolist()
    qrep = np.ascontiguousarray(np.repeat(w.q[0, :1], 4, axis=0))
    c = oracle.select_chunk_mean_query(qrep, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, 10)
    assert c[0].tolist() == b[0].tolist()
    # linearity (fp32 storage, no second rounding to speak of): scores of the mean query = mean of the scores
    w32 = W.make_workload("c32", dtype=W.F32, C=5, H=4, H_kv=2, D=16, P=4, seq_lens=[70], k=10, seed=10)
    _, _, _, S = oracle.select_chunk_mean_query(w32.q[0], w32.k_pool, w32.dtype, w32.H_kv, w32.P, w32.pages_of(0), 65, 10,
                                                details=True)
    Sm = np.mean([oracle.paged_qk_scores(np.ascontiguousarray(w32.q[0, c]), w32.k_pool, w32.dtype, w32.H_kv, w32.P,
                                         w32.pages_of(0), 65) for c in range(5)], axis=0)
    np.testing.assert_allclose(S, Sm, rtol=0, atol=2e-6)


# ---------------------------------------------------------------- Eq. 3 / Eq. 4: the ablation selection functions

def brute_head_vote(S, k):
    H, N = S.shape
    votes = np.zeros(N)
    for h in range(H):
        order = sorted(range(N), key=lambda t: (-np.float32(S[h, t]), t))      # descending value, ascending index
        for t in order[:k]:
            votes[t] += 1
    return votes


def test_sum_and_head_vote_against_brute_force():
    w = tiny(N=70, seed=41)
    S = oracle.paged_qk_scores(w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 70)
    np.testing.assert_allclose(oracle.sum_vote(S), S.sum(axis=0), rtol=1e-14)
    for k in (1, 5, 69, 70, 100):
        hv = oracle.head_vote(S, k)
        assert np.array_equal(hv, brute_head_vote(S, k))
        assert hv.sum() == w.H * min(k, 70) and hv.max() <= w.H
        for kind, votes in (("sum", S.sum(axis=0)), ("head", hv)):
            idx, cnt = oracle.select_with(kind, w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 70, k)
            assert idx[:cnt].tolist() == brute_topk(votes.astype(np.float32), k)
    # k >= N: every head takes every token, all votes equal H, ties resolve to the first tokens
    idx, cnt = oracle.select_with("head", w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 70, 70)
    assert cnt == 70 and idx.tolist() == list(range(70))


def test_single_head_makes_the_three_selection_functions_agree():
    # H = 1: Eq. 3, Eq. 4 and Eq. 5 are all the top-k of that head's raw logits
    w = W.make_workload("h1", dtype=W.F32, H=1, H_kv=1, D=16, P=4, seq_lens=[120], k=9, seed=42)
    ref = None
    for kind in ("soft", "sum", "head"):
        idx, cnt = oracle.select_with(kind, w.q[0, 0], w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 120, 9)
        ref = idx.tolist() if ref is None else ref
        assert cnt == 9 and idx.tolist() == ref, kind


def test_head_vote_ties_go_to_lower_index():
    S = np.array([[1.0, 3.0, 3.0, 0.0, 3.0], [2.0, 2.0, 2.0, 2.0, 2.0]])
    assert oracle.head_vote(S, 2).tolist() == [1.0, 2.0, 1.0, 0.0, 0.0]   # head 0 takes tokens 1, 2; head 1 takes 0, 1


def test_sum_vote_is_dominated_by_a_head_with_large_logits_while_votes_are_not():
    # the weakness the paper names for Eq. 3: scale one head's query by 50 and its preferences decide Eq. 3,
    # while Eq. 4 still gives that head one vote per token like every other head
    w = W.make_workload("dom", dtype=W.F32, H=4, H_kv=4, D=16, P=4, seq_lens=[200], k=10, seed=43)
    q = w.q[0, 0].copy(); q[0] *= 50.0
    S = oracle.paged_qk_scores(q, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 200)
    top_h0 = set(brute_topk(S[0].astype(np.float32), 10))
    i_sum, _ = oracle.select_with("sum", q, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 200, 10)
    assert len(top_h0 & set(i_sum.tolist())) >= 9
    hv = oracle.head_vote(S, 10)
    assert hv.max() <= 4 and hv.sum() == 40


def test_chunk_selection_with_forced_tokens_is_plain_chunk_selection_on_the_middle():
    C, N, k, ni, nl = 3, 90, 10, 6, 13
    w = W.make_workload("cf", dtype=W.F32, C=C, H=4, H_kv=2, D=16, P=1, seq_lens=[N + C], k=k, seed=23)
    qc = w.q[0]
    idx, cnt, votes = oracle.select_chunk(qc, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, k, details=True,
                                          n_init=ni, n_local=nl)
    lo, hi = ni, N - nl
    idx2, cnt2, votes2 = oracle.select_chunk(qc, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0)[lo:hi], hi - lo, k, details=True)
    assert cnt == cnt2 == k and (idx[:cnt] - lo).tolist() == idx2[:cnt2].tolist()
    np.testing.assert_array_equal(votes[lo:hi], votes2)
    assert not votes[:lo].any() and not votes[hi:].any() and abs(votes.sum() - C * w.H) < 1e-12
    # the attended list of query c: initial block, selection, the cached tokens just before the chunk, chunk tokens 0..c
    att = oracle.attended_tokens(idx, cnt, N, ni, nl)
    assert att.tolist() == list(range(ni)) + idx[:cnt].tolist() + list(range(N - nl, N))
    # forced blocks covering the cache: every query sees the whole cache plus its causal part of the chunk = full
    # causal attention over the sequence up to itself (bitwise: same order of terms)
    idx0, cnt0 = oracle.select_chunk(qc, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, k, n_init=50, n_local=60)
    assert cnt0 == 0
    att0 = oracle.attended_tokens(idx0, cnt0, N, 50, 60)
    for c in range(C):
        a = oracle.sparse_attn(np.ascontiguousarray(qc[c]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), att0, N, 0.25,
                               extra_first=N, n_extra=c + 1)
        b = oracle.full_attn(np.ascontiguousarray(qc[c]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N + c + 1, 0.25)
        assert np.array_equal(a, b), c
