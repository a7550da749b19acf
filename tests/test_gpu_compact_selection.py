"""GPU parity of the compact selection (ts_paged_qk_codes / ts_soft_vote_bounds / ts_topk_exact): the bytes are
re-derived from the definition in the header, the vote bounds must contain the oracle's votes, and the index set
must be the oracle's (1e-6 band rule) and the dense path's."""
import math

import numpy as np
import pytest

import oracle
import workloads as W
from parity_util import compare_index_sets, oracle_decode

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    return ts


def make_layer(w, **kw):
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device
    layer = DecodeLayer.from_workload(w, **kw)
    return layer, to_device(w.q)


def codes_from_definition(S, lo, hi, bt, c2):
    """codes[t][h] = clamp(255 + ceil(4 * c2 * (s - M)), 0, 255) in float arithmetic, M = the head's maximum over
    the ranked tokens [lo, hi) of the token's block of bt tokens.  S: float32 [N][H]."""
    N, H = S.shape
    out = np.zeros((N, H), dtype=np.uint8)
    f4c2 = np.float32(4.0) * np.float32(c2)
    for b0 in range(0, N, bt):
        b1 = min(N, b0 + bt)
        r0, r1 = max(b0, lo), min(b1, hi)
        if r1 > r0:
            M = S[r0:r1].max(axis=0)
        else:
            M = np.full(H, -np.inf, dtype=np.float32)
        with np.errstate(invalid="ignore", over="ignore"):
            y = (f4c2 * (S[b0:b1] - M[None, :]).astype(np.float32)).astype(np.float32)
            v = np.float32(255.0) + np.ceil(y)
            v = np.where(np.isnan(v), np.float32(0.0), v)
        out[b0:b1] = np.clip(v, 0.0, 255.0).astype(np.uint8)
    return out


def check_compact(w, layer, q_dev, *, score_scale=1.0, label="", score_variant=2, codes_run_tiles=0):
    """Both forms of the compact score pass against the five-call form.  With the matrix-core kernels switched off
    both passes run the vector kernel, with them on (and the score variant at its default, 2) both run the
    matrix-core kernel: the bytes then follow from the five-call form's scores bit for bit.  A caller that has set
    score variant 0 or 1 (the vector kernel for the score matrix) says so: the matrix-core bytes may then differ
    from that matrix by a few ulp per score."""
    import paper_2411_02886_amd as ts
    for mfma in (0, 1):
        ts.ts_debug_set_codes_path(mfma, codes_run_tiles if mfma else 0)
        try:
            _check_compact(w, layer, q_dev, score_scale=score_scale, label=label + (" mfma" if mfma else " valu"),
                           exact_bytes=(mfma == 0 or score_variant == 2))
        finally:
            ts.ts_debug_set_codes_path(1, 0)


def _check_compact(w, layer, q_dev, *, score_scale=1.0, label="", exact_bytes=True):
    from paper_2411_02886_amd.runtime import to_host
    c = float(np.float32(score_scale))
    c2 = np.float32(np.float32(score_scale) * np.float32(1.44269504088896340736))
    layer.select(q_dev, score_scale, None)
    torch.cuda.synchronize()
    S_g = to_host(layer.scores).copy(); st_d = to_host(layer.row_stats).copy(); v_d = to_host(layer.votes).copy()
    idx_d = to_host(layer.idx).copy(); cnt_d = to_host(layer.count).copy()
    layer.idx.fill_(-7); layer.count.fill_(-7)
    layer.select_compact(q_dev, score_scale, None)
    torch.cuda.synchronize()
    codes = to_host(layer.codes); st_c = to_host(layer.row_stats); hi_g = to_host(layer.vote_hi); lo_g = to_host(layer.vote_lo)
    idx_c = to_host(layer.idx); cnt_c = to_host(layer.count)
    ncand = []
    for b in range(w.B):
        N = int(w.seq_lens[b])
        lab = "%s b=%d N=%d" % (label, b, N)
        ni, nl = layer.num_initial, layer.num_local
        lo, hi = oracle.ranked_range(N, ni, nl)
        if N == 0:
            assert cnt_c[b] == 0 and np.all(idx_c[b] == -1), lab
            continue
        # 1. the bytes: one of the three block lengths reproduces them exactly from the dense path's scores
        best = None
        for bt in (32, 64, 128, 256):
            d = np.abs(codes_from_definition(S_g[b, :N], lo, hi, bt, c2)[lo:hi].astype(np.int32) - codes[b, lo:hi].astype(np.int32))
            if best is None or d.sum() < best.sum():
                best = d
        if best.size == 0:
            pass
        elif exact_bytes:
            assert best.max() == 0, (lab, "codes do not follow their definition for any block length")
        else:
            # a score a few ulp away may fall on the other side of a quarter-octave boundary, never further
            assert best.max() <= 1 and (best != 0).mean() <= 0.01, (lab, "codes", int(best.max()), float((best != 0).mean()))
        # 2. statistics: same maximum as the dense path, same sum within rounding
        if hi > lo:
            if exact_bytes:
                assert np.array_equal(st_c[b, :, 0], st_d[b, :, 0]), lab
            else:
                assert np.abs(st_c[b, :, 0] - st_d[b, :, 0]).max() <= 6 * np.spacing(np.float32(np.abs(S_g[b, :N]).max())), lab
            np.testing.assert_allclose(st_c[b, :, 1], st_d[b, :, 1], rtol=3e-5 if not exact_bytes else 5e-6, err_msg=lab)
        # 3. bounds contain the dense path's votes and the oracle's, and are tight
        ora = oracle_decode(w, b, score_scale=score_scale, n_init=ni, n_local=nl)
        vd = v_d[b, lo:hi].astype(np.float64); vh = hi_g[b, lo:hi].astype(np.float64); vl = lo_g[b, lo:hi].astype(np.float64)
        assert np.all(vl <= vd) and np.all(vd <= vh), (lab, "bounds vs dense votes")
        vo = ora["votes"][lo:hi]
        assert np.all(vl * (1 - 1e-5) <= vo) and np.all(vo <= vh * (1 + 1e-5)), (lab, "bounds vs oracle votes")
        # a quarter octave plus twice the guard (1e-3 octaves + c2 * |largest head maximum| * 2^-18 for the float
        # scores' own rounding).  Heads whose byte is 0 are open towards minus infinity: the kernel takes the most they
        # can have put into the upper sum, 2^(-63.75 + guard) * H, off every token's lower bound once.  That widens
        # tokens whose whole vote is within 2^14 of this floor by more than the 1.0005 allows for (with one to three
        # heads the median token can lie there: votes below 2^-49 * H), so the width is checked on the tokens above
        # it; single tokens with a byte-0 head are wider, hence the median.
        guard = 1e-3 + float(c2) * float(np.abs(st_c[b, :, 0]).max()) / 262144.0 if hi > lo else 0.0
        pos = vl > w.H * 2.0 ** (-63.75 + guard + 14)
        if pos.any():
            width = 2 ** (0.25 + 2 * guard) * 1.0005
            assert np.median(vh[pos] / vl[pos]) <= width, (lab, "bounds too wide", np.median(vh[pos] / vl[pos]), width)
        assert not hi_g[b, :lo].any() and not hi_g[b, hi:N].any() and not lo_g[b, :lo].any() and not lo_g[b, hi:N].any(), lab
        # 4. index set: the oracle's (band rule) and the dense path's
        compare_index_sets(idx_c[b], int(cnt_c[b]), ora, lab)
        if not np.array_equal(idx_c[b], idx_d[b]):
            kth = np.sort(ora["votes"])[::-1][int(cnt_c[b]) - 1]
            for t in np.setxor1d(idx_c[b][:cnt_c[b]], idx_d[b][:cnt_d[b]]):
                assert abs(ora["votes"][t] - kth) / kth <= 1e-6, (lab, "differs from the dense path", int(t))
        # candidates the exact pass looked at (for the record)
        kk = int(cnt_c[b])
        if kk > 0:
            lk = np.sort(vl)[::-1][kk - 1]
            ncand.append((int((vh >= lk).sum()), kk))
    print(label, "candidates/k:", ncand, flush=True)


def test_config1_tiny_fp32(gpu):
    w = W.config1()
    layer, q = make_layer(w)
    for scale in (1.0, 1.0 / math.sqrt(w.D)):
        print("compact cfg1 scale", scale, flush=True)
        check_compact(w, layer, q, score_scale=scale, label="cfg1 c=%.3f" % scale)


@pytest.mark.parametrize("variant", [0, 1, 2], ids=["fma", "dot2", "matrix-cores"])
def test_config2_shape_reduced(gpu, variant):
    gpu.ts_debug_set_score_variant(variant, 0)
    try:
        w = W.config2(N=5000, k=300, seed=77)
        layer, q = make_layer(w)
        for scale in (1.0, 1.0 / math.sqrt(w.D)):
            print("compact cfg2-small variant", variant, "scale", scale, flush=True)
            check_compact(w, layer, q, score_scale=scale, label="cfg2s v%d c=%.3f" % (variant, scale), score_variant=variant)
    finally:
        gpu.ts_debug_set_score_variant(2, 0)


SHAPES = [
    (W.F32, 4, 1, 64, 16, 777, 50),
    (W.F32, 8, 8, 128, 16, 300, 64),
    (W.BF16, 28, 4, 128, 16, 2500, 128),
    (W.BF16, 16, 2, 64, 16, 1000, 100),
    (W.BF16, 32, 16, 128, 16, 600, 64),
    (W.BF16, 32, 8, 128, 1, 333, 40),
    (W.F32, 8, 2, 64, 4, 515, 33),
    (W.BF16, 8, 4, 128, 2, 130, 130),
    (W.F32, 6, 2, 64, 16, 450, 30),
    (W.BF16, 2, 2, 128, 16, 200, 16),
    (W.BF16, 64, 32, 64, 16, 260, 20),
    (W.BF16, 128, 16, 128, 16, 180, 20),
    # shapes of the matrix-core score pass: every group size it takes, both head dims, both wave-tile widths,
    # pages shorter than a wave step, two KV-head units per token
    (W.BF16, 24, 8, 128, 16, 1500, 100),
    (W.BF16, 24, 4, 64, 16, 900, 64),
    (W.BF16, 32, 4, 128, 4, 700, 50),
    (W.BF16, 64, 16, 64, 2, 400, 40),
    (W.BF16, 20, 4, 128, 1, 350, 30),
    (W.BF16, 32, 8, 64, 16, 1234, 77),
    # one and two heads, D = 128: most tokens' votes lie near the byte-0 floor of the bounds
    (W.BF16, 1, 1, 128, 16, 3000, 100),
    (W.F32, 2, 1, 128, 1, 2600, 16),
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "dt%d_H%d_%d_D%d_P%d_N%d_k%d" % s)
def test_shapes(gpu, shape):
    dtype, H, H_kv, D, P, N, k = shape
    print("compact shape", shape, flush=True)
    w = W.make_workload("shape", dtype=dtype, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[N], k=k, beta=3.0,
                        planted_per_head=2, seed=N + H)
    layer, q = make_layer(w)
    for scale in (1.0, 1.0 / math.sqrt(D)):
        check_compact(w, layer, q, score_scale=scale, label=str(shape) + " c=%.3f" % scale)


@pytest.mark.parametrize("run_tiles", [2, 4])
def test_longer_blocks(gpu, run_tiles):
    gpu.ts_debug_set_score_variant(1, 0, run_tiles)
    try:
        w = W.config2(N=9000, k=500, seed=5)
        layer, q = make_layer(w)
        print("compact run_tiles", run_tiles, flush=True)
        check_compact(w, layer, q, score_scale=1.0, label="rr%d" % run_tiles, score_variant=1)
    finally:
        gpu.ts_debug_set_score_variant(2, 0, 0)


@pytest.mark.parametrize("rr,wg", [(1, 0), (3, 5), (8, 2), (5, 0), (2, 1)])
@pytest.mark.parametrize("heads", [(32, 8), (28, 4)])
def test_matrix_core_score_pass_run_lengths_and_grids(gpu, rr, wg, heads):
    """The matrix-core score pass with other run lengths and with grids so small that a wave takes several runs."""
    gpu.ts_debug_set_score_variant(2, wg, 0)              # both forms on the matrix cores, same grid and run length
    try:
        w = W.make_workload("mfma_runs", dtype=W.BF16, H=heads[0], H_kv=heads[1], D=128, P=16, B=2, seq_lens=[9000, 3333],
                            k=300, beta=2.5, planted_per_head=2, seed=77 + rr)
        layer, q = make_layer(w)
        print("compact matrix-core run_tiles", rr, "workgroups", wg, heads, flush=True)
        check_compact(w, layer, q, score_scale=1.0, label="mfma rr%d wg%d" % (rr, wg), codes_run_tiles=rr)
    finally:
        gpu.ts_debug_set_codes_path(1, 0); gpu.ts_debug_set_score_variant(2, 0, 0)


@pytest.mark.parametrize("lens,parts", [([70000, 66000, 41000], 2), ([150000, 9000], 1), ([30000], 4), ([70000, 70000, 70000, 3000], 1)],
                         ids=["2-per-chunk", "1-per-chunk", "4-per-chunk", "1-per-chunk-batch4"])
def test_refine_with_several_workgroups_per_chunk(gpu, lens, parts):
    """The exact re-evaluation runs 256 / (chunks x batch) workgroups per 2048-token chunk, four at most: every split
    gives the oracle's selection."""
    w = W.make_workload("parts", dtype=W.BF16, H=8, H_kv=2, D=64, P=16, B=len(lens), seq_lens=lens, k=700, beta=2.5,
                        planted_per_head=2, seed=sum(lens) % 977)
    layer, q = make_layer(w)
    nblk = (max(lens) + 2047) // 2048
    assert max(1, min(4, 256 // (nblk * len(lens)))) == parts
    print("compact refine parts", parts, lens, flush=True)
    check_compact(w, layer, q, score_scale=1.0, label="parts%d" % parts)


def test_batch_ragged_and_forced(gpu):
    w = W.make_workload("ragged", dtype=W.BF16, H=32, H_kv=8, D=128, P=16, B=6, seq_lens=[4100, 0, 37, 2048, 9999, 1],
                        k=256, beta=2.5, planted_per_head=0, seed=11)
    layer, q = make_layer(w)
    print("compact ragged", flush=True)
    check_compact(w, layer, q, score_scale=1.0, label="ragged")
    layer2, q2 = make_layer(w, num_initial=128, num_local=512)
    print("compact ragged forced", flush=True)
    check_compact(w, layer2, q2, score_scale=1.0, label="ragged forced")


def test_flat_votes_zero_scale(gpu):
    # score_scale 0: every vote is H / N, every token is a candidate; ties go to the lower index
    w = W.config2(N=3000, k=100, seed=3)
    layer, q = make_layer(w)
    print("compact zero scale", flush=True)
    check_compact(w, layer, q, score_scale=0.0, label="c=0")


def margin_report(ora, v_gpu, lo, hi, label):
    """k/(k+1) relative gap of the oracle's votes and the worst relative vote error of the GPU near the k-th vote."""
    votes = ora["votes"]; cnt = ora["count"]
    s = np.sort(votes)[::-1]
    gap = float((s[cnt - 1] - s[cnt]) / s[cnt - 1]) if cnt < len(s) and s[cnt - 1] > 0 else float("inf")
    near = np.where(np.abs(votes[lo:hi] - s[cnt - 1]) <= 0.05 * s[cnt - 1])[0] + lo
    err = float(np.max(np.abs(v_gpu[near].astype(np.float64) - votes[near]) / votes[near])) if len(near) else 0.0
    print("%s: k/(k+1) relative vote gap %.3e; worst relative error of the five-call path's votes within 5%% of the k-th vote %.3e (%d tokens)"
          % (label, gap, err, len(near)), flush=True)
    return gap, err


@pytest.mark.parametrize("cfg", [2, 4])
def test_full_size_compact_selection(gpu, cfg):
    """Configurations 2 and 4 at full size in the launch configuration bench.py times (compact form, matrix-core
    score pass): index set against the oracle (1e-6 band rule) and against the five-call form, with the margins
    on record."""
    from paper_2411_02886_amd.runtime import to_host
    w = W.CONFIGS[cfg]()
    layer, q = make_layer(w)
    print("compact full size cfg", cfg, flush=True)
    layer.select(q, 1.0, None); torch.cuda.synchronize()
    idx_d = to_host(layer.idx).copy(); v_d = to_host(layer.votes).copy()
    layer.idx.fill_(-7)
    layer.select_compact(q, 1.0, None); torch.cuda.synchronize()
    idx_c = to_host(layer.idx).copy(); cnt_c = to_host(layer.count).copy()
    N = int(w.seq_lens[0])
    ora = oracle_decode(w, 0, score_scale=1.0)
    margin_report(ora, v_d[0], 0, N, "cfg%d" % cfg)
    exc = compare_index_sets(idx_c[0], int(cnt_c[0]), ora, "cfg%d compact" % cfg)
    print("cfg%d compact: tolerated near-tie exceptions %d; identical to the five-call form: %s"
          % (cfg, len(exc), bool(np.array_equal(idx_c, idx_d))), flush=True)
    # the votes the compact form decided on (exact scores): error against the oracle over the whole selection
    sv = to_host(layer.sel_votes)[0, :int(cnt_c[0])].astype(np.float64)
    vo_sel = ora["votes"][idx_c[0, :int(cnt_c[0])]]
    rel = np.abs(sv - vo_sel) / vo_sel
    print("cfg%d compact: relative error of the selected tokens' votes against the oracle: max %.3e, rms %.3e"
          % (cfg, rel.max(), np.sqrt((rel ** 2).mean())), flush=True)
    # what is left is the float statistics of the score pass: the maximum of a head is a rounded score, and that
    # rounding (a few ulp of a score of about 60) is a common factor on every vote share of the head
    assert rel.max() <= 3e-5
    vh = to_host(layer.vote_hi)[0, :N].astype(np.float64); vl = to_host(layer.vote_lo)[0, :N].astype(np.float64)
    assert np.all(vl * (1 - 1e-5) <= ora["votes"]) and np.all(ora["votes"] <= vh * (1 + 1e-5)), "bounds vs oracle votes"
    lk = np.sort(vl)[::-1][w.k - 1]
    print("cfg%d compact: candidates %d for k = %d" % (cfg, int((vh >= lk).sum()), w.k), flush=True)
    # attention over the compact selection
    layer.attend(q, 1.0 / math.sqrt(w.D)); torch.cuda.synchronize()
    att = oracle.attended_tokens(idx_c[0], int(cnt_c[0]), N, 0, 0)
    o_ref = oracle.sparse_attn(np.ascontiguousarray(w.q[0, 0]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), att, len(att),
                               float(np.float32(1.0 / math.sqrt(w.D))))
    o_g = W.as_f32(to_host(layer.out, bits16=True)[0, 0], w.dtype).astype(np.float64)
    assert np.abs(o_g - o_ref).max() <= 2e-2


@pytest.mark.parametrize("H,H_kv", [(28, 4), (12, 4), (20, 4), (32, 8)])
def test_head_maxima_hundreds_apart(gpu, H, H_kv):
    """Raw logits (score_scale 1) whose per-head maxima differ by several hundred: every vote stays finite and the
    votes sum to H, in the five-call form (whose padded lanes once compared a shadow head with the wrong maximum) and
    in the compact form."""
    from paper_2411_02886_amd.runtime import to_host
    w = W.make_workload("spread", dtype=W.BF16, H=H, H_kv=H_kv, D=128, P=16, seq_lens=[3000], k=64, seed=H)
    qf = W.as_f32(w.q, w.dtype).copy()
    for h in range(H):
        qf[0, 0, h] *= 0.2 + 6.0 * (h % 5)         # head norms from 0.2x to 24x: maxima from a few to several hundred
    w.q = W.store(qf, w.dtype)
    layer, q = make_layer(w)
    layer.select(q, 1.0, None); torch.cuda.synchronize()
    st = to_host(layer.row_stats)[0]; v = to_host(layer.votes)[0]
    print("H=%d head maxima from %.1f to %.1f" % (H, st[:, 0].min(), st[:, 0].max()), flush=True)
    assert st[:, 0].max() - st[:, 0].min() > 300
    assert np.isfinite(v).all() and abs(float(v.astype(np.float64).sum()) - H) < 1e-3 * H
    check_compact(w, layer, q, score_scale=1.0, label="spread H=%d" % H)


def test_tuning_knob_changed_between_the_calls_of_a_step(gpu):
    """The statistics partial count travels through the workspace: a grid knob flipped between the score pass and
    the vote does not change the votes."""
    from paper_2411_02886_amd.runtime import to_host
    w = W.config2(N=9000, k=500, seed=8)
    layer, q = make_layer(w)
    ora = oracle_decode(w, 0, score_scale=1.0)
    try:
        gpu.ts_paged_qk_scores(layer.problem, q, layer.scores, 1.0, None, layer.ws)
        gpu.ts_debug_set_score_variant(1, 7, 4)            # another grid, another run length
        gpu.ts_soft_vote(layer.problem, layer.scores, 1.0, layer.row_stats, layer.votes, None, layer.ws)
        gpu.ts_topk(layer.problem, layer.votes, layer.k, layer.idx, layer.count, None, layer.ws)
        torch.cuda.synchronize()
        v = to_host(layer.votes)[0].astype(np.float64)
        np.testing.assert_allclose(v, ora["votes"], rtol=3e-5, atol=1e-44)
        compare_index_sets(to_host(layer.idx)[0], int(to_host(layer.count)[0]), ora, "knob flip, five calls")
        gpu.ts_debug_set_score_variant(2, 0, 0)
        gpu.ts_paged_qk_codes(layer.problem, q, layer_codes(layer), 1.0, None, layer.ws)
        gpu.ts_debug_set_score_variant(0, 3, 1); gpu.ts_debug_set_codes_path(0, 1)
        gpu.ts_soft_vote_bounds(layer.problem, layer.codes, 1.0, layer.row_stats, layer.vote_hi, layer.vote_lo, None, layer.ws)
        gpu.ts_topk_exact(layer.problem, q, layer.vote_hi, layer.row_stats, 1.0, layer.k, layer.idx, layer.count, None, layer.ws)
        torch.cuda.synchronize()
        compare_index_sets(to_host(layer.idx)[0], int(to_host(layer.count)[0]), ora, "knob flip, compact")
    finally:
        gpu.ts_debug_set_score_variant(2, 0, 0); gpu.ts_debug_set_codes_path(1, 0)


def layer_codes(layer):
    if getattr(layer, "codes", None) is None:
        B, M = layer.B, layer.max_seq_len
        layer.codes = torch.empty((B, M, layer.H), dtype=torch.uint8, device=layer.device)
        layer.vote_hi = torch.empty((B, M), dtype=torch.float32, device=layer.device)
        layer.vote_lo = torch.empty((B, M), dtype=torch.float32, device=layer.device)
        layer.sel_votes = torch.zeros((B, layer.k), dtype=torch.float32, device=layer.device)
    return layer.codes


def test_workspace_init_restores_a_dirtied_workspace(gpu):
    """A workspace whose histograms and state were left dirty (what an abandoned selection leaves) selects wrongly;
    ts_workspace_init makes it usable again, for both forms."""
    from paper_2411_02886_amd.runtime import to_host
    w = W.config2(N=6000, k=300, seed=9)
    layer, q = make_layer(w)
    ora = oracle_decode(w, 0, score_scale=1.0)
    layer.ws.fill_(3)                                        # every histogram bin, state word and count dirty
    gpu.ts_workspace_init(layer.ws)
    layer.select(q, 1.0, None); torch.cuda.synchronize()
    compare_index_sets(to_host(layer.idx)[0], int(to_host(layer.count)[0]), ora, "after init, five calls")
    layer.ws.fill_(5)
    gpu.ts_workspace_init(layer.ws)
    layer.select_compact(q, 1.0, None); torch.cuda.synchronize()
    compare_index_sets(to_host(layer.idx)[0], int(to_host(layer.count)[0]), ora, "after init, compact")
    # and the two forms may alternate on one workspace
    layer.select(q, 1.0, None); layer.select_compact(q, 1.0, None); layer.select(q, 1.0, None); torch.cuda.synchronize()
    compare_index_sets(to_host(layer.idx)[0], int(to_host(layer.count)[0]), ora, "alternating forms")


def test_compact_selection_cache_run_and_graph_replay(gpu):
    """Algorithm 1 with the compact selection: 12 steps with AR(1) queries and appended tokens against the oracle's
    run, then the same run captured as a HIP graph and replayed with eager work in between."""
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device, to_host
    steps = 12
    w = W.config3(B=3, lo=3000, hi=9000, steps=steps, seed=21)
    qs_h = W.ar1_queries(w, steps, rho=0.95)
    ks, vs = W.appended_kv(w, steps)
    layer = DecodeLayer.from_workload(w, max_seq_len=int(w.seq_lens.max()) + steps)
    qs = [to_device(x) for x in qs_h]
    ksd, vsd = to_device(ks), to_device(vs)
    slots = np.empty((steps, w.B), dtype=np.int64)
    for b in range(w.B):
        pos = int(w.seq_lens[b]) + np.arange(steps)
        slots[:, b] = w.pages_of(b).astype(np.int64)[pos // w.P] * w.P + pos % w.P
    slots_d = torch.from_numpy(slots).to("cuda:0")
    kflat = layer.k_pool.view(-1, w.H_kv, w.D); vflat = layer.v_pool.view(-1, w.H_kv, w.D)
    len0 = layer.seq_lens.clone()
    idx_log = torch.zeros((steps,) + tuple(layer.idx.shape), dtype=torch.int32, device="cuda:0")
    reuse_log = torch.zeros((steps, w.B), dtype=torch.uint8, device="cuda:0")
    layer_codes(layer)

    def run():
        layer.seq_lens.copy_(len0); layer.first.fill_(1)
        for t in range(steps):
            kflat.index_copy_(0, slots_d[t], ksd[t]); vflat.index_copy_(0, slots_d[t], vsd[t])
            layer.seq_lens.add_(1)
            layer.step(qs[t], theta=0.9, score_scale=1.0, compact=True)
            idx_log[t].copy_(layer.idx); reuse_log[t].copy_(layer.reuse)

    run(); torch.cuda.synchronize()
    idx_e = to_host(idx_log).copy(); reuse_e = to_host(reuse_log).copy()
    # the oracle's run of Algorithm 1 on the same inputs
    kpf = w.k_pool.reshape(-1, w.H_kv, w.D); vpf = w.v_pool.reshape(-1, w.H_kv, w.D)
    cq = [np.zeros((w.H, w.D), np.uint16) for _ in range(w.B)]
    first = [np.ones(1, np.uint8) for _ in range(w.B)]
    cidx = [np.full(w.k, -1, np.int32) for _ in range(w.B)]
    ccnt = [np.zeros(1, np.int32) for _ in range(w.B)]
    hits = 0
    for t in range(steps):
        for b in range(w.B):
            kpf[slots[t, b]] = ks[t, b]; vpf[slots[t, b]] = vs[t, b]
            N = int(w.seq_lens[b]) + t + 1
            qb = np.ascontiguousarray(qs_h[t][b, 0])
            holder = {}

            def sel(qq, b=b, N=N, holder=holder):
                i, c, votes, _ = oracle.select(qq, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), N, w.k, details=True)
                holder["votes"] = votes
                return i, c
            i_o, c_o, r_o = oracle.selcache_step(qb, cq[b], cidx[b], ccnt[b], first[b], float(np.float32(0.9)), sel)
            assert bool(reuse_e[t, b]) == r_o, ("reuse flag", t, b)
            hits += int(r_o)
            if not r_o:
                compare_index_sets(idx_e[t, b], c_o, dict(idx=i_o, count=c_o, votes=holder["votes"]), "compact run t=%d b=%d" % (t, b))
                cidx[b][:] = idx_e[t, b]                    # follow the GPU's (band-equivalent) choice from here on
            else:
                assert np.array_equal(idx_e[t, b], i_o), ("cached index set must stay", t, b)
    print("compact Selection Cache run: %d hits of %d" % (hits, steps * w.B), flush=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side); torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run()
    for rep in range(3):
        idx_log.fill_(-3); reuse_log.fill_(9); layer.idx.fill_(-3); torch.cuda.synchronize()
        g.replay(); torch.cuda.synchronize()
        assert np.array_equal(to_host(idx_log), idx_e) and np.array_equal(to_host(reuse_log), reuse_e), ("graph replay", rep)
        _ = (layer.votes * 2).sum().item()                   # eager work between the replays


@pytest.mark.parametrize("N,H,H_kv,D,k", [(3_900_000, 128, 16, 64, 1024), (16_000_000, 8, 2, 64, 4096)])
def test_long_sequences_both_forms_agree(gpu, N, H, H_kv, D, k):
    """Sizes no oracle run covers (K generated on the GPU): 3.9M tokens with 128 heads, where the vote-bounds kernel has to
    shorten its workgroups' token range to keep its table in LDS, and 16M tokens, the longest the finishing workgroup
    indexes.  Properties: the compact form selects the five-call form's tokens, its bounds contain the five-call votes."""
    from paper_2411_02886_amd.runtime import DecodeLayer, to_host
    dev = "cuda:0"
    g = torch.Generator(device=dev); g.manual_seed(5)
    P = 16
    npages = (N + P - 1) // P
    kp = torch.randn((npages, P, H_kv, D), device=dev, dtype=torch.bfloat16, generator=g).view(torch.int16)
    vp = torch.randn((npages, P, H_kv, D), device=dev, dtype=torch.bfloat16, generator=g).view(torch.int16)
    perm = np.random.default_rng(1).permutation(npages).astype(np.int32)
    layer = DecodeLayer(dtype=gpu.TS_BF16, H=H, H_kv=H_kv, D=D, P=P, k=k, k_pool=kp, v_pool=vp, page_indptr=[0, npages],
                        page_indices=perm, seq_lens=[N], device=dev)
    q = torch.randn((1, 1, H, D), device=dev, dtype=torch.bfloat16, generator=g).view(torch.int16)
    print("long sequence", N, H, H_kv, D, "five-call form", flush=True)
    layer.select(q, 1.0, None); torch.cuda.synchronize()
    idx_d = to_host(layer.idx).copy(); v = to_host(layer.votes)[0, :N]
    print("long sequence", N, "compact form", flush=True)
    layer.idx.fill_(-5); layer.select_compact(q, 1.0, None); torch.cuda.synchronize()
    idx_c = to_host(layer.idx)
    assert int(to_host(layer.count)[0]) == k
    kth = np.sort(v)[::-1][k - 1]
    for t in np.setxor1d(idx_d[0], idx_c[0]):
        assert abs(v[t] - kth) / kth <= 1e-5, ("forms differ away from the k-th vote", int(t))
    vh = to_host(layer.vote_hi)[0, :N]; vl = to_host(layer.vote_lo)[0, :N]
    assert np.all(vl <= v) and np.all(v <= vh)
    del layer, kp, vp
    torch.cuda.empty_cache()
