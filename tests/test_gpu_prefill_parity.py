"""GPU parity of the chunked-prefill selection (MFMA score sweeps, per-query votes summed over the
chunk, shared top-k) against the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest

import oracle
import workloads as W
from parity_util import compare_index_sets, ulp32

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    return ts


def run_chunk_selection(ts, w, k, scale, n_init=0, n_local=0):
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device, to_host
    sel = ChunkSelector.from_workload(w, k=k, num_initial=n_init, num_local=n_local)
    q = to_device(w.q)
    sel.select(q, scale)
    sel.attend(q)
    torch.cuda.synchronize()
    return (to_host(sel.row_stats), to_host(sel.votes), to_host(sel.idx), to_host(sel.count),
            to_host(sel.out, bits16=True), to_host(sel.lse))


def check_chunk(ts, w, k, scale, label, n_init=0, n_local=0, gpu_w=None):
    """gpu_w: the workload as the GPU sees it when that is not w itself (same tokens, other pools and page ids)."""
    st_g, v_g, idx_g, cnt_g, out_g, lse_g_attn = run_chunk_selection(ts, gpu_w if gpu_w is not None else w, k, scale, n_init, n_local)
    sm = float(np.float32(1.0 / math.sqrt(w.D)))
    c = float(np.float32(scale))
    for b in range(w.B):
        Nc = max(int(w.seq_lens[b]) - w.C, 0)
        lo, hi = oracle.ranked_range(Nc, n_init, n_local)          # forced blocks are taken from the cached tokens
        lab = "%s b=%d Nc=%d" % (label, b, Nc)
        if int(w.seq_lens[b]) < w.C:
            # shorter than the chunk (an idle slot of the batch): nothing selected, nothing attended, rows zero
            assert cnt_g[b] == 0 and np.all(idx_g[b] == -1), lab
            assert not out_g[b].any() and np.all(np.isneginf(lse_g_attn[b])), (lab, "idle sequence")
            continue
        if hi <= lo:
            assert cnt_g[b] == 0 and np.all(idx_g[b] == -1), lab
        # Eq. 2, chunk form: query c over the forced and selected tokens plus the chunk's tokens 0..c (one softmax)
        att = oracle.attended_tokens(idx_g[b], int(cnt_g[b]), Nc, n_init, n_local)
        for ci in sorted(set([0, 1, w.C // 2, w.C - 1]) if w.C > 8 else range(w.C)):
            o_ref, l_ref = oracle.sparse_attn(np.ascontiguousarray(w.q[b, ci]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P,
                                              w.pages_of(b), att, len(att), sm, extra_first=Nc,
                                              n_extra=ci + 1, with_lse=True)
            err = np.abs(W.as_f32(out_g[b, ci], w.dtype).astype(np.float64) - o_ref).max()
            assert err <= 2e-2, (lab, "chunk attention", ci, err)
            assert np.abs(lse_g_attn[b, ci] - l_ref).max() <= 2e-2, (lab, "chunk attention lse", ci)
        assert not v_g[b, :lo].any() and not v_g[b, hi:Nc].any(), (lab, "votes outside the ranked range must be 0")
        if hi <= lo:
            continue
        votes = np.zeros(Nc)
        smax = 0.0
        for ci in range(w.C):
            S = oracle.paged_qk_scores(np.ascontiguousarray(w.q[b, ci]), w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), Nc)
            v, m, z = oracle.soft_vote(np.ascontiguousarray(S[:, lo:hi]), c, with_stats=True)
            votes[lo:hi] += v
            smax = max(smax, float(np.abs(S).max()))
            # sweep 1: the row's log-sum-exp (stored base 2 as a high/low pair): score rounding + fast exp2
            lse_g = (st_g[b, ci, :, 0].astype(np.float64) + st_g[b, ci, :, 1]) * math.log(2.0)
            assert np.abs(lse_g - (m + np.log(z))).max() <= 8 * ulp32(smax) * c + 2e-5, (lab, ci, "row log-sum-exp")
        # sweep 2: votes; float arithmetic with the fast exponential: 3e-5 relative
        np.testing.assert_allclose(v_g[b, lo:hi], votes[lo:hi], rtol=3e-5, atol=1e-30, err_msg=lab + " votes")
        assert abs(float(v_g[b, lo:hi].astype(np.float64).sum()) - w.C * w.H) < 1e-4 * w.C * w.H, lab
        # radix select in isolation on the GPU's own votes: bit-exact
        i_iso, c_iso = oracle.topk(v_g[b, lo:hi].astype(np.float64), k)
        i_iso = i_iso.copy(); i_iso[:c_iso] += lo
        assert cnt_g[b] == c_iso and np.array_equal(idx_g[b], i_iso), (lab, "radix select")
        # end to end against the oracle's chunk selection (1e-6 band rule)
        i_o, c_o = oracle.topk(oracle.decision_votes(votes[lo:hi]), k)
        i_o = i_o.copy(); i_o[:c_o] += lo
        compare_index_sets(idx_g[b], int(cnt_g[b]), dict(idx=i_o, count=c_o, votes=votes), lab)


CASES = [
    # C, H, H_kv, D, P, seq_len (cached = seq_len - C), k, scale
    (48, 8, 2, 128, 16, 3048, 64, 0.0884),      # fewer rows than one 256-row block, ragged token tiles
    (128, 32, 8, 128, 16, 5128, 256, 1.0),      # config 5's head shapes, two row blocks per KV head
    (100, 28, 4, 128, 16, 2100, 100, 0.0884),   # group of seven: row blocks that straddle queries
    (64, 16, 4, 64, 16, 1500, 50, 0.125),       # head_dim 64
    (16, 8, 8, 128, 4, 400, 400, 0.0884),       # G = 1, k larger than the cached length
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "C%d_H%d_%d_D%d_P%d_L%d_k%d" % c[:7])
def test_chunk_selection_shapes(gpu, case):
    C, H, H_kv, D, P, L, k, scale = case
    print("chunk case", case, flush=True)
    w = W.make_workload("chunk", dtype=W.BF16, C=C, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[L], k=k, beta=2.5,
                        planted_per_head=max(1, (L - C) // 200), plant_limit=L - C, seed=L + C)
    check_chunk(gpu, w, k, scale, str(case))


@pytest.mark.parametrize("forced", [(128, 512), (3, 0), (0, 70), (64, 64)])
def test_chunk_selection_with_forced_tokens(gpu, forced):
    # forced blocks are taken from the cached tokens before the chunk; sequences shorter than the blocks included
    ni, nl = forced
    C = 40
    lens = [C + 3000, C + 640, C + 700, C + 100, C, C + 641, C + 63]
    w = W.make_workload("chunkf", dtype=W.BF16, B=len(lens), C=C, H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=50, seed=41 + ni)
    print("chunk forced", forced, lens, flush=True)
    check_chunk(gpu, w, 50, 0.0884, "chunk forced %d+%d" % forced, n_init=ni, n_local=nl)
    w = W.make_workload("chunkf2", dtype=W.BF16, C=130, H=32, H_kv=8, D=128, P=16, seq_lens=[130 + 4000], k=256, seed=43)
    check_chunk(gpu, w, 256, 1.0, "chunk forced cfg5 heads %d+%d" % forced, n_init=ni, n_local=nl)


def test_chunk_batch_with_idle_sequences(gpu):
    # sequences shorter than the chunk, the last one with no page at all: they hold no chunk; their rows come back
    # zero and nothing is read through their page table entries
    C = 48
    lens = [C + 1500, 0, 7, C - 1, C + 300, 0]
    w = W.make_workload("chunk_idle", dtype=W.BF16, B=len(lens), C=C, H=16, H_kv=4, D=128, P=16, seq_lens=lens, k=64, seed=88)
    print("chunk idle", lens, flush=True)
    for forced in ((0, 0), (16, 32)):
        check_chunk(gpu, w, 64, 1.0, "idle %d+%d" % forced, n_init=forced[0], n_local=forced[1])
    # a key list long enough to be split over workgroups: the idle rows go through the merge of the splits
    check_chunk(gpu, w, 1024, 1.0, "idle, split key list")


def test_chunk_selection_ragged_batch(gpu):
    C = 32
    lens = [C, C + 1, C + 63, C + 64, C + 65, 900]
    w = W.make_workload("chunkb", dtype=W.BF16, B=len(lens), C=C, H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=40, seed=3)
    print("chunk ragged batch", lens, flush=True)
    check_chunk(gpu, w, 40, 0.0884, "ragged")


@pytest.mark.timeout(900)
def test_config5_full_size_sampled(gpu):
    """Configuration 5 at full size (512 queries x 262144 cached tokens).  The oracle needs minutes for all
    16384 softmax rows, so the check is on samples: (a) the log-sum-exp of every head of 6 sampled queries
    against the oracle; (b) the votes of 768 sampled tokens (the GPU's top 256, the first 256 below its
    threshold, 256 random) recomputed in double from oracle-style scores and the row log-sum-exps;
    (c) the radix select on the GPU's votes, exact; (d) chunk attention of 3 sampled queries."""
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device, to_host
    w = W.config5()
    N = int(w.extra["n_cached"]); C, H, G, D = w.C, w.H, w.G, w.D
    print("cfg5 full size: generating done", flush=True)
    sel = ChunkSelector.from_workload(w)
    q = to_device(w.q)
    sel.select(q, 1.0); sel.attend(q)
    torch.cuda.synchronize()
    st = to_host(sel.row_stats)[0]; v_g = to_host(sel.votes)[0, :N]; idx_g = to_host(sel.idx)[0]; cnt_g = int(to_host(sel.count)[0])
    out_g = to_host(sel.out, bits16=True)[0]
    lse2 = st[..., 0].astype(np.float64) + st[..., 1]                     # [C][H] base-2 log-sum-exp
    rng = np.random.default_rng(55)
    # (a) sampled rows
    for ci in sorted(rng.choice(C, size=6, replace=False).tolist()):
        S = oracle.paged_qk_scores(np.ascontiguousarray(w.q[0, ci]), w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N)
        _, m, z = oracle.soft_vote(S, 1.0, with_stats=True)
        assert np.abs(lse2[ci] * math.log(2.0) - (m + np.log(z))).max() <= 8 * ulp32(float(np.abs(S).max())) + 2e-5, ci
    print("cfg5 rows ok", flush=True)
    # (c) radix select alone
    i_iso, c_iso = oracle.topk(v_g.astype(np.float64), w.k)
    assert cnt_g == c_iso and np.array_equal(idx_g, i_iso)
    # (b) sampled tokens
    order = np.argsort(-v_g, kind="stable")
    sample = np.unique(np.concatenate([order[:256], order[w.k:w.k + 256], rng.choice(N, size=256, replace=False)]))
    slots = w.slots_of(0)[sample]
    Ks = W.as_f32(w.k_pool, w.dtype).reshape(-1, w.H_kv, D)[slots].astype(np.float64)      # [T][H_kv][D]
    Q = W.as_f32(w.q, w.dtype)[0].astype(np.float64)                                       # [C][H][D]
    S = np.einsum("chd,thd->cht", Q, np.repeat(Ks, G, axis=1))                             # [C][H][T]
    votes_ref = np.exp(S - (lse2 * math.log(2.0))[:, :, None]).sum(axis=(0, 1))
    np.testing.assert_allclose(v_g[sample], votes_ref, rtol=3e-5, atol=1e-30)
    assert abs(float(v_g.astype(np.float64).sum()) - C * H) < 1e-4 * C * H
    print("cfg5 votes ok", flush=True)
    # (d) chunk attention
    sm = float(np.float32(1.0 / math.sqrt(D)))
    for ci in (0, 257, C - 1):
        o_ref = oracle.sparse_attn(np.ascontiguousarray(w.q[0, ci]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0),
                                   idx_g, cnt_g, sm, extra_first=N, n_extra=ci + 1)
        assert np.abs(W.as_f32(out_g[ci], w.dtype).astype(np.float64) - o_ref).max() <= 2e-2, ci


# ---------------------------------------------------------------- Sec. 5.2 as printed: mean-query selection

def check_mean_query(ts, w, k, scale, label, n_init=0, n_local=0):
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device, to_host
    sel = ChunkSelector.from_workload(w, k=k, num_initial=n_init, num_local=n_local)
    q = to_device(w.q)
    sel.select_mean_query(q, scale)
    sel.attend(q)
    torch.cuda.synchronize()
    m = sel._mean_query_state()
    qm_g = to_host(m["q_mean"], bits16=True); S_g = to_host(m["scores"]); v_g = to_host(sel.votes)
    idx_g = to_host(sel.idx); cnt_g = to_host(sel.count); out_g = to_host(sel.out, bits16=True)
    c = float(np.float32(scale)); sm = float(np.float32(1.0 / math.sqrt(w.D)))
    for b in range(w.B):
        Nc = max(int(w.seq_lens[b]) - w.C, 0)
        lab = "%s b=%d Nc=%d" % (label, b, Nc)
        qm_o = oracle.mean_query(np.ascontiguousarray(w.q[b]), w.dtype)
        assert np.array_equal(qm_g[b, 0], qm_o), (lab, "mean query must match bit for bit")
        if Nc == 0:
            assert cnt_g[b] == 0 and np.all(idx_g[b] == -1), lab
            continue
        lo, hi = oracle.ranked_range(Nc, n_init, n_local)
        i_o, c_o, votes, S = oracle.select_chunk_mean_query(np.ascontiguousarray(w.q[b]), w.k_pool, w.dtype, w.H_kv, w.P,
                                                            w.pages_of(b), Nc, k, score_scale=c, details=True,
                                                            n_init=n_init, n_local=n_local)
        Sg = np.ascontiguousarray(S_g[b, :Nc, :].T).astype(np.float64)
        assert np.abs(Sg - S).max() <= 6 * ulp32(np.abs(S).max()), (lab, "scores")
        if hi > lo:
            np.testing.assert_allclose(v_g[b, lo:hi], oracle.soft_vote(np.ascontiguousarray(Sg[:, lo:hi]), c), rtol=5e-6,
                                       atol=1e-44, err_msg=lab)
        assert not v_g[b, :lo].any() and not v_g[b, hi:Nc].any(), lab
        i_iso, c_iso = oracle.topk(v_g[b, lo:hi].astype(np.float64), k)
        i_iso = i_iso.copy(); i_iso[:c_iso] += lo
        assert cnt_g[b] == c_iso and np.array_equal(idx_g[b], i_iso), (lab, "radix select")
        compare_index_sets(idx_g[b], int(cnt_g[b]), dict(idx=i_o, count=c_o, votes=votes), lab)
        att = oracle.attended_tokens(idx_g[b], int(cnt_g[b]), Nc, n_init, n_local)
        for ci in sorted(set([0, w.C // 2, w.C - 1])):
            o_ref = oracle.sparse_attn(np.ascontiguousarray(w.q[b, ci]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P,
                                       w.pages_of(b), att, len(att), sm, extra_first=Nc, n_extra=ci + 1)
            assert np.abs(W.as_f32(out_g[b, ci], w.dtype).astype(np.float64) - o_ref).max() <= 2e-2, (lab, "attention", ci)


@pytest.mark.parametrize("case", [(48, 8, 2, 128, 16, 3048, 64, 0.0884), (128, 32, 8, 128, 16, 5128, 256, 1.0),
                                  (7, 28, 4, 128, 16, 1200, 100, 0.0884), (64, 16, 4, 64, 1, 900, 50, 0.125)],
                         ids=lambda c: "C%d_H%d_%d_D%d_P%d_L%d_k%d" % c[:7])
def test_mean_query_selection_shapes(gpu, case):
    C, H, H_kv, D, P, L, k, scale = case
    print("mean-query case", case, flush=True)
    w = W.make_workload("chunkmq", dtype=W.BF16, C=C, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[L], k=k, beta=2.5,
                        planted_per_head=max(1, (L - C) // 200), plant_limit=L - C, seed=L + C + 1)
    check_mean_query(gpu, w, k, scale, "mq " + str(case))


def test_mean_query_selection_with_forced_tokens(gpu):
    C = 24
    lens = [C + 2000, C + 100, C + 641, C]
    w = W.make_workload("chunkmqf", dtype=W.BF16, B=len(lens), C=C, H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=40, seed=45)
    check_mean_query(gpu, w, 40, 0.0884, "mq forced", n_init=128, n_local=512)
    check_mean_query(gpu, w, 40, 1.0, "mq forced small", n_init=5, n_local=9)


def test_mean_query_selection_ragged_batch(gpu):
    C = 32
    lens = [C, C + 1, C + 63, 900, C + 300]
    w = W.make_workload("chunkmqb", dtype=W.BF16, B=len(lens), C=C, H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=40, seed=4)
    print("mean-query ragged batch", lens, flush=True)
    check_mean_query(gpu, w, 40, 0.0884, "mq ragged")


@pytest.mark.parametrize("direction", ["rising", "falling", "spikes"])
def test_chunk_selection_with_scores_that_keep_outgrowing_the_reference(gpu, direction):
    # Sweep 1 keeps lazy per-lane reference exponents; here every row's scores drift by hundreds of units along
    # the sequence (or jump in isolated spikes), so references are raised again and again and far apart.
    C, H, H_kv, D, P, L, k = 40, 8, 2, 128, 16, 2600, 64
    w = W.make_workload("drift", dtype=W.BF16, C=C, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[L], k=k, seed=61)
    Nc = L - C
    rng = np.random.Generator(np.random.PCG64(62))
    kf = W.as_f32(w.k_pool, w.dtype).reshape(-1, H_kv, D).copy()
    qf = W.as_f32(w.q, w.dtype)[0]                          # [C][H][D]
    slots = w.slots_of(0)
    dirs = qf.mean(axis=0).reshape(H_kv, H // H_kv, D).mean(axis=1)      # one direction per KV head
    dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    t = np.arange(Nc, dtype=np.float32)
    if direction == "rising":
        amp = -12.0 + 24.0 * t / Nc
    elif direction == "falling":
        amp = 12.0 - 24.0 * t / Nc
    else:
        amp = np.zeros(Nc, np.float32); amp[rng.choice(Nc, size=12, replace=False)] = rng.uniform(8.0, 20.0, size=12)
    kf[slots[:Nc]] += amp[:, None, None] * dirs[None, :, :] * 3.0
    w.k_pool[:] = W.store(kf.reshape(w.k_pool.shape), w.dtype)
    check_chunk(gpu, w, k, 1.0, "drift " + direction)
    check_chunk(gpu, w, k, 0.0884, "drift " + direction + " scaled")


def load_cfg5_golden():
    """tests/golden/cfg5_chunk_selection.txt, written by tests/golden/make_cfg5_golden.py from the CPU oracle alone."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "cfg5_chunk_selection.txt")
    lines = [l for l in open(path).read().split("\n") if l and not l.startswith("#")]
    g = {}
    i = 0
    while i < len(lines):
        key, *rest = lines[i].split()
        if key == "idx":
            g["idx"] = np.array(lines[i + 1].split(), dtype=np.int64); i += 2
        elif key == "band":
            n = int(rest[0])
            rows = [l.split() for l in lines[i + 1:i + 1 + n]]
            g["band_tok"] = np.array([int(r[0]) for r in rows]); g["band_vote"] = np.array([float(r[1]) for r in rows]); i += 1 + n
        elif key == "lse":
            C, H = int(rest[0]), int(rest[1])
            g["lse"] = np.array([[float(x) for x in l.split()] for l in lines[i + 1:i + 1 + C]]); i += 1 + C
            assert g["lse"].shape == (C, H)
        else:
            g[key] = float(rest[0]) if "." in rest[0] or "e" in rest[0] else int(rest[0]); i += 1
    return g


@pytest.mark.timeout(900)
def test_config5_full_size_against_the_oracles_selection(gpu):
    """Configuration 5 at full size against the oracle's own run of it (Sec. 5.2 with per-query Eq. 5 votes): the
    whole index set under the 1e-6 band rule, every one of the 16384 softmax rows' log-sum-exp, the vote total, and
    the GPU's votes of the 512 tokens around the k-th one."""
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device, to_host
    g = load_cfg5_golden()
    w = W.config5()
    N = int(w.extra["n_cached"])
    assert g["cached_tokens"] == N and g["chunk"] == w.C and g["heads"] == w.H and g["count"] == w.k
    sel = ChunkSelector.from_workload(w)
    q = to_device(w.q)
    print("cfg5 against the stored oracle selection", flush=True)
    sel.select(q, 1.0)
    torch.cuda.synchronize()
    st = to_host(sel.row_stats)[0]; v_g = to_host(sel.votes)[0, :N]; idx_g = to_host(sel.idx)[0]; cnt_g = int(to_host(sel.count)[0])
    # every row's log-sum-exp (the GPU stores base-2 values as a high/low pair)
    lse_g = (st[..., 0].astype(np.float64) + st[..., 1]) * math.log(2.0)
    err = np.abs(lse_g - g["lse"]).max()
    print("cfg5: worst log-sum-exp error over %d rows %.3e" % (lse_g.size, err), flush=True)
    assert err <= 1e-4
    assert abs(float(v_g.astype(np.float64).sum()) - g["vote_total"]) <= 1e-5 * g["vote_total"]
    # votes around the k-th one
    rel = np.abs(v_g[g["band_tok"]].astype(np.float64) - g["band_vote"]) / g["band_vote"]
    kth = g["band_vote"][min(255, g["count"] - 1)]
    gap = (g["band_vote"][255] - g["band_vote"][256]) / g["band_vote"][255]
    print("cfg5: k/(k+1) relative vote gap %.3e; worst relative error of the GPU's votes among the 512 tokens around the k-th %.3e"
          % (gap, rel.max()), flush=True)
    assert rel.max() <= 3e-5
    # the index set: bit-exact except tokens whose oracle vote lies within 1e-6 relative of the k-th vote
    assert cnt_g == g["count"] and np.all(np.diff(idx_g[:cnt_g]) > 0)
    diff = np.setxor1d(idx_g[:cnt_g], g["idx"])
    band = dict(zip(g["band_tok"].tolist(), g["band_vote"].tolist()))
    for t in diff.tolist():
        assert t in band, ("token differs far from the k-th vote", t)
        assert abs(band[t] - kth) / kth <= 1e-6, ("token differs outside the 1e-6 band", t, abs(band[t] - kth) / kth)
    print("cfg5: index set identical to the oracle's except %d tokens inside the 1e-6 band" % len(diff), flush=True)


@pytest.mark.parametrize("name,C,H,H_kv,D,P,lens,k,ni,nl,scale", [
    ("512 queries x 1M cached", 512, 32, 8, 128, 16, [1_048_576 + 512], 4096, 0, 0, 1.0),
    ("100 queries, G 7", 100, 28, 4, 128, 16, [300_100], 2048, 0, 0, 1.0),
    ("33 queries, G 1, D 64", 33, 16, 16, 64, 16, [50_033], 512, 0, 0, 1.0),
    ("1024 queries, forced tokens", 1024, 32, 8, 128, 16, [200_000], 4096, 128, 512, 1.0),
    ("batch of 3, ragged", 256, 32, 8, 128, 16, [70_000, 300, 12_345], 1024, 0, 0, 1.0),
    ("page size 1", 128, 32, 8, 64, 1, [40_128], 512, 0, 0, 1.0),
    ("G 3, 2 queries, scale 1/sqrt(D)", 2, 24, 8, 128, 16, [10_002], 100, 0, 0, 1.0 / math.sqrt(128)),
])
def test_chunk_selection_invariants_at_sizes_no_oracle_run_covers(gpu, name, C, H, H_kv, D, P, lens, k, ni, nl, scale):
    """Properties that hold at any size (inputs generated on the GPU): every softmax row sums to one, so the votes of the
    ranked range sum to C * H -- which also ties the two sweeps together, the second normalises with the first's
    log-sum-exps; count = min(k, ranked tokens); indices ascending, inside the ranked range, none below the k-th vote."""
    from paper_2411_02886_amd.runtime import ChunkSelector, to_host
    dev = "cuda:0"
    g = torch.Generator(device=dev); g.manual_seed(9)
    B = len(lens)
    pages = [(n + P - 1) // P for n in lens]
    npages = sum(pages) + 3
    kp = torch.randn((npages, P, H_kv, D), device=dev, dtype=torch.bfloat16, generator=g).view(torch.int16)
    vp = torch.randn((npages, P, H_kv, D), device=dev, dtype=torch.bfloat16, generator=g).view(torch.int16)
    q = torch.randn((B, C, H, D), device=dev, dtype=torch.bfloat16, generator=g).view(torch.int16)
    perm = np.random.default_rng(1).permutation(npages).astype(np.int32)[: sum(pages)]
    indptr = np.concatenate([[0], np.cumsum(pages)]).astype(np.int32)
    print("chunk invariants:", name, flush=True)
    sel = ChunkSelector(C=C, H=H, H_kv=H_kv, D=D, P=P, k=k, k_pool=kp, v_pool=vp, page_indptr=indptr, page_indices=perm,
                        seq_lens=lens, device=dev, num_initial=ni, num_local=nl)
    sel.select(q, scale)
    torch.cuda.synchronize()
    v = to_host(sel.votes); idx = to_host(sel.idx); cnt = to_host(sel.count)
    for b in range(B):
        Nc = max(lens[b] - C, 0)
        lo = min(ni, Nc); hi = max(lo, Nc - nl)
        c = int(cnt[b])
        assert c == min(k, hi - lo), (name, b, c)
        want = float(C * H) if hi > lo else 0.0
        tot = float(v[b, lo:hi].astype(np.float64).sum())
        assert abs(tot - want) <= 2e-5 * max(want, 1.0), (name, b, tot, want)
        assert np.all(np.diff(idx[b, :c]) > 0) and np.all(idx[b, c:] == -1), (name, b)
        if c > 0:
            assert idx[b, 0] >= lo and idx[b, c - 1] < hi, (name, b)
        if 0 < c < hi - lo:
            kth = np.sort(v[b, lo:hi])[::-1][c - 1]
            assert v[b, idx[b, :c]].min() >= kth, (name, b, "a selected token lies below the k-th vote")
    sel.attend(q)
    torch.cuda.synchronize()
    o = (to_host(sel.out).view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    assert np.isfinite(o).all(), (name, "attention")
    del sel, kp, vp
    torch.cuda.empty_cache()
