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


def check_compact(w, layer, q_dev, *, score_scale=1.0, label=""):
    """Both forms of the compact score pass: the vector form shares the dense path's score arithmetic (its bytes
    follow from the dense scores bit for bit), the matrix-core form may differ by a few ulp per score."""
    import paper_2411_02886_amd as ts
    for mfma in (0, 1):
        ts.ts_debug_set_codes_path(mfma, 0)
        try:
            _check_compact(w, layer, q_dev, score_scale=score_scale, label=label + (" mfma" if mfma else " valu"), exact_bytes=(mfma == 0))
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
        pos = vl > 0
        if pos.any():
            # a quarter octave plus guards; heads whose byte is 0 (open towards minus infinity) widen single tokens
            assert np.median(vh[pos] / vl[pos]) <= 2 ** 0.26, (lab, "bounds too wide", np.median(vh[pos] / vl[pos]))
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


@pytest.mark.parametrize("variant", [0, 1])
def test_config2_shape_reduced(gpu, variant):
    gpu.ts_debug_set_score_variant(variant, 0)
    try:
        w = W.config2(N=5000, k=300, seed=77)
        layer, q = make_layer(w)
        for scale in (1.0, 1.0 / math.sqrt(w.D)):
            print("compact cfg2-small variant", variant, "scale", scale, flush=True)
            check_compact(w, layer, q, score_scale=scale, label="cfg2s v%d c=%.3f" % (variant, scale))
    finally:
        gpu.ts_debug_set_score_variant(1, 0)


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
        check_compact(w, layer, q, score_scale=1.0, label="rr%d" % run_tiles)
    finally:
        gpu.ts_debug_set_score_variant(1, 0, 0)


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
