"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, run the oracle on
the same seeded inputs, and compare stage by stage."""
import math

import numpy as np

import oracle
import workloads as W


def ulp32(x: float) -> float:
    return float(np.spacing(np.float32(abs(x))))


def oracle_decode(w, b, q=None, score_scale=1.0, sm_scale=None, k=None, n_init=0, n_local=0):
    """Oracle results for sequence b: dict(S, votes, idx, count, out)."""
    N = int(w.seq_lens[b])
    k = w.k if k is None else k
    qb = np.ascontiguousarray((w.q if q is None else q)[b, 0])
    sm = 1.0 / math.sqrt(w.D) if sm_scale is None else sm_scale
    if N == 0:
        return dict(S=np.zeros((w.H, 0)), votes=np.zeros(0), idx=np.full(k, -1, np.int32), count=0,
                    out=np.zeros((w.H, w.D)))
    idx, cnt, votes, S = oracle.select(qb, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), N, k,
                                       score_scale=float(np.float32(score_scale)), details=True,
                                       n_init=n_init, n_local=n_local)
    att = oracle.attended_tokens(idx, cnt, N, n_init, n_local)
    out = oracle.sparse_attn(qb, w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), att, len(att),
                             float(np.float32(sm)))
    return dict(S=S, votes=votes, idx=idx, count=cnt, out=out)


def compare_index_sets(gpu_idx, gpu_cnt, ora, label=""):
    """Bit-exact, except tokens whose oracle vote lies within 1e-6 relative of the k-th vote.
    Returns the list of tolerated exceptions (token, relative distance)."""
    cnt = ora["count"]
    assert gpu_cnt == cnt, (label, gpu_cnt, cnt)
    g = gpu_idx[:cnt]
    assert np.all(np.diff(g) > 0), label + ": indices must be strictly ascending"
    assert np.all(gpu_idx[cnt:] == -1), label
    o = ora["idx"][:cnt]
    if np.array_equal(g, o):
        return []
    votes = ora["votes"]
    kth = np.sort(votes)[::-1][cnt - 1]
    diff = np.setxor1d(g, o)
    exc = [(int(t), float(abs(votes[t] - kth) / kth)) for t in diff]
    for t, d in exc:
        print("%s: token %d differs, |vote-kth|/kth = %.3e" % (label, t, d))
    assert all(d <= 1e-6 for _, d in exc), (label, exc)
    return exc


# True: the five-call selection of check_decode_against_oracle runs ts_soft_vote_ranked + ts_topk(TS_TOPK_VOTE_HIST)
# instead of ts_soft_vote + ts_topk (tests/test_gpu_ranked_vote.py runs the parity cases again that way)
RANKED_VOTE = False


def check_decode_against_oracle(w, layer, q_dev, *, score_scale=1.0, attn_tol=None, label="", skip_rows=(),
                                expect_tol_S=None):
    """Runs select + attend on the GPU for the workload's query and checks every stage.  Forced tokens
    (layer.num_initial / num_local) restrict statistics, votes and top-k to the ranked range."""
    import torch
    from paper_2411_02886_amd.runtime import to_host
    sm = 1.0 / math.sqrt(w.D)
    layer.select(q_dev, score_scale, None, ranked_vote=RANKED_VOTE)
    layer.attend(q_dev, sm)
    torch.cuda.synchronize()
    S_g = to_host(layer.scores); st_g = to_host(layer.row_stats); v_g = to_host(layer.votes)
    idx_g = to_host(layer.idx); cnt_g = to_host(layer.count)
    out_g = to_host(layer.out, bits16=(w.dtype == W.BF16))
    tol = attn_tol if attn_tol is not None else (2e-2 if w.dtype == W.BF16 else 1e-4)
    c = float(np.float32(score_scale))
    exceptions = []
    for b in range(w.B):
        if b in skip_rows:
            continue
        N = int(w.seq_lens[b])
        ni, nl = layer.num_initial, layer.num_local
        lo, hi = oracle.ranked_range(N, ni, nl)
        ora = oracle_decode(w, b, score_scale=score_scale, n_init=ni, n_local=nl)
        lab = "%s b=%d N=%d" % (label, b, N)
        if N == 0:
            assert cnt_g[b] == 0 and np.all(idx_g[b] == -1), lab
            assert np.all(W.as_f32(out_g[b, 0], w.dtype) == 0), lab
            continue
        # 1. scores (Alg. 2): float accumulation of D exact products; a few ulp of the largest score
        Sg = np.ascontiguousarray(S_g[b, :N, :].T).astype(np.float64)      # stored [token][head]
        tolS = expect_tol_S if expect_tol_S is not None else 6 * ulp32(np.abs(ora["S"]).max())
        errS = np.abs(Sg - ora["S"]).max()
        assert errS <= tolS, (lab, "scores", errS, tolS)
        # 2. statistics over the ranked range: max is exactly the max of the stored scores; sum-exp matches a
        #    double recomputation
        if hi > lo:
            Sr = Sg[:, lo:hi]
            assert np.array_equal(st_g[b, :, 0], S_g[b, lo:hi, :].max(axis=0)), lab
            z = np.exp(c * (Sr - Sr.max(axis=1, keepdims=True))).sum(axis=1)
            np.testing.assert_allclose(st_g[b, :, 1], z, rtol=5e-6, err_msg=lab)
            # 3. votes (Eq. 5): against the oracle formula applied to the GPU's own scores, and the invariant
            v_from_gpuS = oracle.soft_vote(np.ascontiguousarray(Sr), c)
            np.testing.assert_allclose(v_g[b, lo:hi], v_from_gpuS, rtol=5e-6, atol=1e-44, err_msg=lab)
            assert abs(float(v_g[b, lo:hi].astype(np.float64).sum()) - w.H) < 1e-4 * w.H, lab
        assert not v_g[b, :lo].any() and not v_g[b, hi:N].any(), (lab, "votes outside the ranked range must be 0")
        # 4. top-k (radix select) in isolation: bit-exact on the GPU's own votes
        i_iso, c_iso = oracle.topk(v_g[b, lo:hi].astype(np.float64), layer.k)
        i_iso = i_iso.copy(); i_iso[:c_iso] += lo
        assert cnt_g[b] == c_iso and np.array_equal(idx_g[b], i_iso), (lab, "radix select")
        # 5. end to end: index set against the oracle's selection (1e-6 band rule)
        exceptions += compare_index_sets(idx_g[b], int(cnt_g[b]), ora, lab)
        # 6. attention (Eq. 2) on the GPU-selected set against the oracle on the same set
        qb = np.ascontiguousarray(w.q[b, 0])
        att = oracle.attended_tokens(idx_g[b], int(cnt_g[b]), N, ni, nl)
        o_ref = oracle.sparse_attn(qb, w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), att, len(att),
                                   float(np.float32(sm)))
        o_g = W.as_f32(out_g[b, 0], w.dtype).astype(np.float64)
        err = np.abs(o_g - o_ref).max()
        assert err <= tol, (lab, "attention", err, tol)
        if not exceptions:
            assert np.abs(o_g - ora["out"]).max() <= tol, (lab, "attention end-to-end")
    return exceptions
