"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs -- element by element at sizes that span several tiles and ragged tails, plus edge cases."""
import math

import numpy as np
import pytest

import oracle
import workloads as W
from parity_util import check_decode_against_oracle, compare_index_sets, oracle_decode

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


def test_config1_tiny_fp32(gpu):
    w = W.config1()
    layer, q = make_layer(w)
    for scale in (1.0, 1.0 / math.sqrt(w.D)):
        print("cfg1 scale", scale, flush=True)
        check_decode_against_oracle(w, layer, q, score_scale=scale, label="cfg1 c=%.3f" % scale)


@pytest.mark.parametrize("variant", [0, 1, 2], ids=["fma", "dot2", "matrix-cores"])
def test_config2_shape_bf16_reduced_length(gpu, variant):
    # config 2's head shapes at 5000 tokens (not a multiple of the 32-token tile nor of the page)
    gpu.ts_debug_set_score_variant(variant, 0)
    try:
        w = W.config2(N=5000, k=300, seed=77)
        layer, q = make_layer(w)
        for scale in (1.0, 1.0 / math.sqrt(w.D)):
            print("cfg2-small variant", variant, "scale", scale, flush=True)
            check_decode_against_oracle(w, layer, q, score_scale=scale, label="cfg2s v%d c=%.3f" % (variant, scale))
    finally:
        gpu.ts_debug_set_score_variant(2, 0)          # back to the library default


SHAPES = [
    # dtype, H, H_kv, D, P, N, k
    (W.F32, 4, 1, 64, 16, 777, 50),        # one KV head: four tokens per wave step
    (W.F32, 8, 8, 128, 16, 300, 64),       # G = 1, fp32 D = 128 (four loads per row)
    (W.BF16, 28, 4, 128, 16, 2500, 128),   # config 4's group of seven
    (W.BF16, 16, 2, 64, 16, 1000, 100),    # G = 8, D = 64 bf16 (one load per row)
    (W.BF16, 32, 16, 128, 16, 600, 64),    # 16 KV heads: two head blocks per token tile
    (W.BF16, 32, 8, 128, 1, 333, 40),      # page size 1 (the paper's own setting)
    (W.F32, 8, 2, 64, 4, 515, 33),         # small pages, H_kv = 2
    (W.BF16, 8, 4, 128, 2, 130, 130),      # page size 2, k == N
    (W.F32, 6, 2, 64, 16, 450, 30),        # G = 3: head rows that are no multiple of 16 bytes
    (W.BF16, 2, 2, 128, 16, 200, 16),      # two heads in all
    (W.BF16, 64, 32, 64, 16, 260, 20),     # 32 KV heads: four head blocks
    (W.BF16, 128, 16, 128, 16, 180, 20),   # 128 query heads, G = 8
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "dt%d_H%d_%d_D%d_P%d_N%d_k%d" % s)
def test_shapes(gpu, shape):
    dtype, H, H_kv, D, P, N, k = shape
    print("shape", shape, flush=True)
    w = W.make_workload("shape", dtype=dtype, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[N], k=k, beta=3.0,
                        planted_per_head=2, seed=N + H)
    layer, q = make_layer(w)
    check_decode_against_oracle(w, layer, q, score_scale=1.0 / math.sqrt(D), label=str(shape))


@pytest.mark.parametrize("run_tiles", [2, 4])
def test_staged_runs_of_several_tiles(gpu, run_tiles):
    # the score pass may stage 2 or 4 consecutive 32-token tiles per wave before writing them out (chosen
    # automatically for long sequences); forced here on short ones, with ragged last runs and a ragged batch
    gpu.ts_debug_set_score_variant(1, 0, run_tiles)
    try:
        for shape in [(W.BF16, 32, 8, 128, 16, 5000, 300), (W.BF16, 28, 4, 128, 16, 2500, 128),
                      (W.F32, 6, 2, 64, 16, 450, 30), (W.BF16, 64, 32, 64, 16, 260, 20), (W.BF16, 32, 8, 128, 1, 333, 40)]:
            dtype, H, H_kv, D, P, N, k = shape
            print("run_tiles", run_tiles, "shape", shape, flush=True)
            w = W.make_workload("shape", dtype=dtype, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[N], k=k, beta=3.0,
                                planted_per_head=2, seed=N + H + run_tiles)
            layer, q = make_layer(w)
            check_decode_against_oracle(w, layer, q, score_scale=1.0 / math.sqrt(D), label="run%d %s" % (run_tiles, shape))
        lens = [0, 1, 31, 32, 33, 2049, 700, 15, 129, 64]
        w = W.make_workload("ragged", dtype=W.BF16, B=len(lens), H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=40,
                            beta=3.0, planted_per_head=0, seed=6)
        layer, q = make_layer(w)
        print("run_tiles", run_tiles, "ragged batch", lens, flush=True)
        check_decode_against_oracle(w, layer, q, score_scale=0.1, label="ragged run%d" % run_tiles)
    finally:
        gpu.ts_debug_set_score_variant(2, 0, 0)


@pytest.mark.parametrize("n_init,n_local", [(128, 512), (5, 0), (0, 33), (16, 100)])
def test_forced_initial_and_recent_tokens(gpu, n_init, n_local):
    # Sec. 6.1: initial and most recent tokens are attended in addition to the k selected ones; the
    # selection ranks only the tokens between them.  Sequences shorter than the forced blocks included.
    lens = [5000, 640, 700, 130, 100, 0, 1, 641, 2048]
    w = W.make_workload("forced", dtype=W.BF16, B=len(lens), H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=64,
                        beta=3.0, planted_per_head=0, seed=31 + n_init)
    layer, q = make_layer(w, num_initial=n_init, num_local=n_local)
    print("forced tokens", n_init, n_local, lens, flush=True)
    check_decode_against_oracle(w, layer, q, score_scale=0.2, label="forced %d+%d" % (n_init, n_local))
    w = W.make_workload("forced32", dtype=W.F32, H=8, H_kv=2, D=64, P=16, seq_lens=[3000], k=256, beta=3.0,
                        planted_per_head=4, seed=32)
    layer, q = make_layer(w, num_initial=n_init, num_local=n_local)
    check_decode_against_oracle(w, layer, q, score_scale=1.0, label="forced fp32 %d+%d" % (n_init, n_local))


def test_ragged_batch_with_empty_and_short_sequences(gpu):
    lens = [0, 1, 31, 32, 33, 2049, 700, 15]
    w = W.make_workload("ragged", dtype=W.BF16, B=len(lens), H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=40,
                        beta=3.0, planted_per_head=0, seed=5)
    layer, q = make_layer(w)
    print("ragged batch", lens, flush=True)
    check_decode_against_oracle(w, layer, q, score_scale=0.1, label="ragged")


def test_large_batch_of_short_sequences(gpu):
    rng = np.random.Generator(np.random.PCG64(71))
    lens = [int(x) for x in rng.integers(0, 1500, size=40)]
    w = W.make_workload("batch40", dtype=W.BF16, B=40, H=28, H_kv=4, D=128, P=16, seq_lens=lens, k=48, seed=72)
    layer, q = make_layer(w, num_initial=4, num_local=16)
    print("batch of 40", flush=True)
    check_decode_against_oracle(w, layer, q, score_scale=0.2, label="batch40")


def test_serving_sized_batch(gpu):
    # 600 sequences in one call (grid extents in the hundreds along the batch axis), both forms, every sequence checked
    from test_gpu_compact_selection import check_compact
    rng = np.random.Generator(np.random.PCG64(73))
    lens = [int(x) for x in rng.integers(0, 260, size=600)]
    w = W.make_workload("batch600", dtype=W.BF16, B=600, H=8, H_kv=2, D=64, P=16, seq_lens=lens, k=24, seed=74)
    layer, q = make_layer(w, num_initial=2, num_local=8)
    print("batch of 600", flush=True)
    check_decode_against_oracle(w, layer, q, score_scale=0.25, label="batch600")
    check_compact(w, layer, q, score_scale=0.25, label="batch600")


def test_two_layers_on_two_streams_give_their_single_stream_results(gpu):
    """Calls on different workspaces may overlap in time: two layers of different shapes run whole steps on two
    streams, launches interleaved on the host, and each must end with the results of its own single-stream run."""
    from paper_2411_02886_amd.runtime import to_host
    wa = W.config2(N=30000, k=512, seed=301)
    wb = W.make_workload("other_stream", dtype=W.BF16, B=3, H=28, H_kv=4, D=128, P=16, seq_lens=[9000, 0, 14001], k=300,
                         beta=2.5, planted_per_head=2, seed=302)
    sm = 1.0 / math.sqrt(128)
    runs = []
    for w in (wa, wb):
        layer, q = make_layer(w, num_initial=4, num_local=32)
        want = {}
        for compact in (False, True):
            layer.idx.fill_(-5); layer.out.zero_()
            layer.first.fill_(1)
            layer.step(q, theta=0.9, score_scale=1.0, sm_scale=sm, compact=compact)
            torch.cuda.synchronize()
            want[compact] = (to_host(layer.idx).copy(), to_host(layer.count).copy(), to_host(layer.out).copy())
        runs.append((w, layer, q, want))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for compact in (False, True):
        for _, layer, _, _ in runs:
            layer.idx.fill_(-5); layer.out.zero_()
        torch.cuda.synchronize()
        for it in range(6):
            for (w, layer, q, _), st in zip(runs, streams):
                with torch.cuda.stream(st):
                    layer.first.fill_(1)                      # every step a miss: the whole chain runs each time
                    layer.step(q, theta=0.9, score_scale=1.0, sm_scale=sm, compact=compact)
        torch.cuda.synchronize()
        for w, layer, q, want in runs:
            idx, cnt, out = want[compact]
            assert np.array_equal(to_host(layer.idx), idx) and np.array_equal(to_host(layer.count), cnt), (w.name, compact)
            assert np.array_equal(to_host(layer.out), out), (w.name, compact, "attention output")


def test_attention_bounds_stale_and_corrupt_selection_state(gpu):
    """idx and count live in device memory between steps (the cached selection of Algorithm 1); the attention kernels
    bound what they read from them: token ids are clamped into the sequence, counts into [0, k], and an empty
    sequence attends nothing whatever its count says (it may own no page at all)."""
    from paper_2411_02886_amd.runtime import to_device, to_host
    lens = [900, 300, 0]
    w = W.make_workload("stale", dtype=W.BF16, B=3, H=8, H_kv=2, D=128, P=16, seq_lens=lens, k=32, seed=17)
    layer, q = make_layer(w)
    layer.select(q, 1.0, None)
    torch.cuda.synchronize()
    idx = to_host(layer.idx).copy(); cnt = to_host(layer.count).copy()
    idx[0, 3] = -12; idx[0, 5] = 10 ** 9; idx[1, 0] = 300
    cnt[1] = 1000
    cnt[2] = 17; idx[2, :17] = 5
    layer.idx.copy_(to_device(idx)); layer.count.copy_(to_device(cnt))
    sm = 1.0 / math.sqrt(w.D)
    layer.attend(q, sm)
    torch.cuda.synchronize()
    out = W.as_f32(to_host(layer.out, bits16=True), w.dtype).astype(np.float64)
    for b, N in enumerate(lens):
        if N == 0:
            assert not out[b].any()
            continue
        att = np.clip(idx[b, :min(max(int(cnt[b]), 0), w.k)], 0, N - 1).astype(np.int32)
        ref = oracle.sparse_attn(np.ascontiguousarray(w.q[b, 0]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(b),
                                 att, len(att), float(np.float32(sm)))
        assert np.abs(out[b, 0] - ref).max() <= 2e-2, b


def test_attention_with_several_chunks_per_workgroup(gpu):
    # 8192 and more chunk workgroups: a workgroup folds four chunks of 64 tokens into its partial with a running
    # maximum and sum; ragged ends (a last workgroup with one, two or three chunks, a last chunk of a few tokens),
    # empty sequences and forced tokens included
    rng = np.random.Generator(np.random.PCG64(75))
    lens = [int(x) for x in rng.integers(1100, 1500, size=70)]
    lens[3] = 0; lens[10] = 5; lens[20] = 129; lens[30] = 64 * 4 + 1; lens[40] = 64 * 7; lens[69] = 0
    w = W.make_workload("multichunk", dtype=W.BF16, B=70, H=16, H_kv=8, D=128, P=16, seq_lens=lens, k=900, seed=76)
    for forced in ((0, 0), (10, 50)):
        layer, q = make_layer(w, num_initial=forced[0], num_local=forced[1])
        nsplit = (w.k + sum(forced) + 63) // 64
        assert nsplit * w.H_kv * w.B >= 8192
        print("multi-chunk attention", forced, nsplit, flush=True)
        check_decode_against_oracle(w, layer, q, score_scale=0.2, label="multichunk %d+%d" % forced)
    w = W.make_workload("multichunk32", dtype=W.F32, B=40, H=8, H_kv=8, D=64, P=4, seq_lens=[700] * 39 + [3], k=1700, seed=77)
    layer, q = make_layer(w)
    assert ((1700 + 63) // 64) * 8 * 40 >= 8192
    check_decode_against_oracle(w, layer, q, score_scale=0.125, label="multichunk fp32")


def test_max_seq_len_larger_than_every_sequence(gpu):
    w = W.make_workload("odd", dtype=W.F32, H=4, H_kv=2, D=64, P=16, seq_lens=[203], k=20, seed=12)
    layer, q = make_layer(w, max_seq_len=205)
    check_decode_against_oracle(w, layer, q, score_scale=0.125, label="odd extent")


def test_ties_go_to_lower_index_and_zero_query(gpu):
    # duplicated K rows give bitwise identical votes; a zero query makes every vote equal
    w = W.make_workload("ties", dtype=W.F32, H=4, H_kv=2, D=64, P=16, seq_lens=[400], k=10, seed=31)
    kl = w.k_pool.reshape(-1, w.H_kv, w.D)
    slots = w.slots_of(0)
    ora0 = oracle_decode(w, 0, score_scale=0.125, k=400)
    order = np.argsort(-ora0["votes"], kind="stable")
    top = order[9]                      # the 10th best token: copy it onto three other tokens
    for t in (5, 17, 333):
        kl[slots[t]] = kl[slots[top]]
    layer, q = make_layer(w)
    check_decode_against_oracle(w, layer, q, score_scale=0.125, label="ties")
    w.q[:] = 0
    layer, q = make_layer(w)
    check_decode_against_oracle(w, layer, q, score_scale=1.0, label="zero query")
    from paper_2411_02886_amd.runtime import to_host
    assert to_host(layer.idx)[0].tolist() == list(range(10))


def test_topk_with_more_tied_candidates_than_one_batch(gpu):
    # a zero query over 20000 tokens: every vote is equal, all tokens share the k-th key's bin, so the finishing
    # workgroup of the short top-k path walks its list in several batches; the first k tokens must win
    from paper_2411_02886_amd.runtime import to_host
    w = W.make_workload("ties20k", dtype=W.BF16, B=2, H=8, H_kv=2, D=128, P=16, seq_lens=[20000, 9000], k=300, seed=33)
    w.q[:] = 0
    layer, q = make_layer(w)
    check_decode_against_oracle(w, layer, q, score_scale=1.0, label="zero query 20k")
    assert to_host(layer.idx)[0].tolist() == list(range(300)) and to_host(layer.idx)[1].tolist() == list(range(300))
    # half of the tokens get one duplicated K row: thousands of exact ties around the threshold
    w = W.make_workload("ties20k2", dtype=W.BF16, H=8, H_kv=2, D=128, P=16, seq_lens=[20000], k=6000, seed=34)
    kl = w.k_pool.reshape(-1, w.H_kv, w.D); slots = w.slots_of(0)
    kl[slots[1::2]] = kl[slots[1]]
    layer, q = make_layer(w)
    check_decode_against_oracle(w, layer, q, score_scale=0.05, label="many ties 20k")


@pytest.mark.parametrize("forced", [(0, 0), (128, 640)])
def test_largest_selection_the_attention_takes(gpu, forced):
    # k + forced tokens = 32768, the most the decode attention merges (512 splits of 64 tokens); both forms
    from test_gpu_compact_selection import check_compact
    ni, nl = forced
    k = 32768 - ni - nl
    print("largest k", k, forced, flush=True)
    w = W.make_workload("kmax", dtype=W.BF16, B=2, H=8, H_kv=2, D=64, P=16, seq_lens=[40000, 33000], k=k, beta=2.0,
                        planted_per_head=4, seed=91 + ni)
    layer, q = make_layer(w, num_initial=ni, num_local=nl)
    check_decode_against_oracle(w, layer, q, score_scale=0.125, label="largest k %d" % k)
    check_compact(w, layer, q, score_scale=0.125, label="largest k %d" % k)


def test_five_pass_topk_path_gives_the_same_result(gpu):
    # the five-pass radix select (kept for sequences beyond 16 Mi tokens) forced on small inputs
    from paper_2411_02886_amd.runtime import to_host
    gpu.ts_debug_set_topk_path(1)
    try:
        for shape in [(W.BF16, 32, 8, 128, 16, [5000], 300), (W.F32, 8, 2, 64, 4, [0, 1, 31, 2049, 700, 4100], 33)]:
            dtype, H, H_kv, D, P, lens, k = shape
            print("five-pass", shape, flush=True)
            w = W.make_workload("fp", dtype=dtype, B=len(lens), H=H, H_kv=H_kv, D=D, P=P, seq_lens=lens, k=k, seed=sum(lens))
            layer, q = make_layer(w)
            check_decode_against_oracle(w, layer, q, score_scale=1.0 / math.sqrt(D), label="five-pass %s" % (shape,))
        w = W.make_workload("fp0", dtype=W.F32, H=4, H_kv=2, D=64, P=16, seq_lens=[5000], k=10, seed=35)
        w.q[:] = 0
        layer, q = make_layer(w)
        check_decode_against_oracle(w, layer, q, score_scale=1.0, label="five-pass zero query")
        assert to_host(layer.idx)[0].tolist() == list(range(10))
    finally:
        gpu.ts_debug_set_topk_path(0)
    # the same form chosen per call
    w = W.make_workload("flat", dtype=W.BF16, B=2, H=8, H_kv=2, D=128, P=16, seq_lens=[5000, 2100], k=100, seed=37)
    layer, q = make_layer(w)
    layer.select(q, 0.01, None)                      # a small scale: nearly uniform votes
    torch.cuda.synchronize()
    idx_a, cnt_a = to_host(layer.idx).copy(), to_host(layer.count).copy()
    layer.idx.fill_(-7); layer.count.fill_(-7)
    gpu.ts_topk(layer.problem, layer.votes, layer.k, layer.idx, layer.count, None, layer.ws, flags=gpu.TS_TOPK_FLAT_VOTES)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(layer.idx), idx_a) and np.array_equal(to_host(layer.count), cnt_a)


def test_k_larger_than_n_equals_full_attention(gpu):
    w = W.make_workload("full", dtype=W.F32, H=8, H_kv=2, D=64, P=16, seq_lens=[150], k=256, seed=41)
    layer, q = make_layer(w)
    check_decode_against_oracle(w, layer, q, score_scale=0.125, label="k>N")
    from paper_2411_02886_amd.runtime import to_host
    full = oracle.full_attn(np.ascontiguousarray(w.q[0, 0]), w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), 150,
                            float(np.float32(1 / math.sqrt(64))))
    assert np.abs(to_host(layer.out)[0, 0] - full).max() < 1e-4


@pytest.mark.parametrize("fused,compact,ranked", [(False, False, False), (True, False, False), (True, True, False), (True, False, True)],
                         ids=["check-call", "check-in-score-launch", "check-in-codes-launch", "check-in-score-launch+ranked-vote"])
def test_selection_cache_loop_matches_algorithm_1(gpu, fused, compact, ranked):
    # fused: ts_paged_qk_scores_checked / ts_paged_qk_codes_checked take the decision in the score launch
    from paper_2411_02886_amd.runtime import to_device, to_host
    steps, theta = 12, 0.9
    w = W.make_workload("sc", dtype=W.BF16, B=3, H=8, H_kv=2, D=128, P=16, seq_lens=[300, 1000, 64], k=32, seed=19,
                        beta=3.0, planted_per_head=1)
    qs = W.ar1_queries(w, steps, rho=0.95)
    layer, _ = make_layer(w)
    # oracle state per sequence
    cq = [np.zeros((w.H, w.D), np.uint16) for _ in range(w.B)]
    first = [np.ones(1, np.uint8) for _ in range(w.B)]
    cidx = [np.full(w.k, -1, np.int32) for _ in range(w.B)]
    ccnt = [np.zeros(1, np.int32) for _ in range(w.B)]
    hits = 0
    for t in range(steps):
        print("selcache step", t, flush=True)
        qd = to_device(qs[t])
        layer.step(qd, theta=theta, score_scale=0.1, fused_check=fused, compact=compact, ranked_vote=ranked)
        torch.cuda.synchronize()
        reuse_g = to_host(layer.reuse); idx_g = to_host(layer.idx); cnt_g = to_host(layer.count)
        out_g = to_host(layer.out, bits16=True)
        assert not to_host(layer.first).any(), t
        for b in range(w.B):
            qb = np.ascontiguousarray(qs[t][b, 0])
            sel = lambda qq, b=b: oracle.select(qq, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), int(w.seq_lens[b]), w.k,
                                                score_scale=float(np.float32(0.1)))
            i_o, c_o, r_o = oracle.selcache_step(qb, cq[b], cidx[b], ccnt[b], first[b], float(np.float32(theta)), sel)
            assert bool(reuse_g[b]) == r_o, (t, b)
            hits += r_o
            assert cnt_g[b] == c_o and np.array_equal(idx_g[b], i_o), (t, b)
            o_ref = oracle.sparse_attn(qb, w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), i_o, c_o,
                                       float(np.float32(1 / math.sqrt(w.D))))
            assert np.abs(W.as_f32(out_g[b, 0], w.dtype) - o_ref).max() <= 2e-2, (t, b)
        assert np.array_equal(to_host(layer.cached_q, bits16=True), np.stack(cq)), t
    assert 0 < hits < steps * w.B          # the run exercises both branches


def planted_stats(w, idx, cnt):
    pl = set(np.concatenate(list(w.planted[0])).tolist())
    sel = set(idx[:cnt].tolist())
    return len(pl & sel) / max(1, len(pl)), len(pl & sel) / max(1, cnt)


@pytest.mark.timeout(600)
def test_config2_full_size(gpu):
    # configuration 2 as bench.py times it: 131072 tokens, k = 2048, library-default launch shape
    w = W.config2()
    layer, q = make_layer(w)
    print("cfg2 full size", flush=True)
    exc = check_decode_against_oracle(w, layer, q, score_scale=1.0, label="cfg2 full")
    from paper_2411_02886_amd.runtime import to_host
    ora = oracle_decode(w, 0)
    rg, pg = planted_stats(w, to_host(layer.idx)[0], int(to_host(layer.count)[0]))
    ro, po = planted_stats(w, ora["idx"], ora["count"])
    print("cfg2 planted recall/precision gpu %.4f/%.4f oracle %.4f/%.4f, tolerated exceptions %d" % (rg, pg, ro, po, len(exc)))
    if not exc:
        assert (rg, pg) == (ro, po)


@pytest.mark.timeout(600)
def test_config2_full_size_with_the_papers_forced_tokens(gpu):
    # configuration 2 with the 128 initial + 512 most recent tokens that the paper's runs always attend
    w = W.config2()
    layer, q = make_layer(w, num_initial=128, num_local=512)
    print("cfg2 full size, forced 128 + 512", flush=True)
    check_decode_against_oracle(w, layer, q, score_scale=1.0, label="cfg2 full forced")


@pytest.mark.timeout(900)
def test_config4_full_size(gpu):
    # configuration 4: 1048576 tokens, 28 query heads over 4 KV heads, k = 4096
    w = W.config4()
    layer, q = make_layer(w)
    print("cfg4 full size", flush=True)
    exc = check_decode_against_oracle(w, layer, q, score_scale=1.0, label="cfg4 full")
    from paper_2411_02886_amd.runtime import to_host
    ora = oracle_decode(w, 0)
    rg, pg = planted_stats(w, to_host(layer.idx)[0], int(to_host(layer.count)[0]))
    ro, po = planted_stats(w, ora["idx"], ora["count"])
    print("cfg4 planted recall/precision gpu %.4f/%.4f oracle %.4f/%.4f, tolerated exceptions %d" % (rg, pg, ro, po, len(exc)))
    if not exc:
        assert (rg, pg) == (ro, po)


@pytest.mark.parametrize("forced", [(0, 0), (16, 64)], ids=["plain", "forced16+64"])
def test_config3_shape_decode_run_with_appended_tokens(gpu, forced):
    # configuration 3 at reduced lengths: ragged batch, AR(1) queries, one K/V row appended per
    # sequence per step, theta = 0.9; Algorithm 1 (anchor = query of the last reselect) on both sides.
    # With forced tokens a reused selection stays as cached while the recent block follows the growing length.
    from paper_2411_02886_amd.runtime import to_device, to_host
    ni, nl = forced
    steps, theta, scale = 24, 0.9, 1.0
    w = W.config3(seed=1003, B=4, lo=700, hi=3000, steps=steps, k=128)
    qs = W.ar1_queries(w, steps, rho=0.95)
    ks, vs = W.appended_kv(w, steps)
    layer, _ = make_layer(w, max_seq_len=int(w.seq_lens.max()) + steps, num_initial=ni, num_local=nl)
    lens = w.seq_lens.copy()
    cq = [np.zeros((w.H, w.D), np.uint16) for _ in range(w.B)]
    first = [np.ones(1, np.uint8) for _ in range(w.B)]
    cidx = [np.full(w.k, -1, np.int32) for _ in range(w.B)]
    ccnt = [np.zeros(1, np.int32) for _ in range(w.B)]
    kflat = w.k_pool.reshape(-1, w.H_kv, w.D); vflat = w.v_pool.reshape(-1, w.H_kv, w.D)
    kdev = layer.k_pool.view(-1, w.H_kv, w.D); vdev = layer.v_pool.view(-1, w.H_kv, w.D)
    reuse_total = 0
    for t in range(steps):
        print("cfg3 step", t, flush=True)
        # append the current token's K/V row (it is part of the cached tokens the query looks at)
        for b in range(w.B):
            pos = int(lens[b])
            slot = int(w.pages_of(b)[pos // w.P]) * w.P + pos % w.P
            kflat[slot] = ks[t, b]; vflat[slot] = vs[t, b]
            kdev[slot] = to_device(ks[t, b]); vdev[slot] = to_device(vs[t, b])
            lens[b] += 1
        layer.seq_lens.copy_(to_device(lens))
        qd = to_device(qs[t])
        layer.step(qd, theta=theta, score_scale=scale)
        torch.cuda.synchronize()
        reuse_g = to_host(layer.reuse); idx_g = to_host(layer.idx); cnt_g = to_host(layer.count)
        out_g = to_host(layer.out, bits16=True)
        for b in range(w.B):
            qb = np.ascontiguousarray(qs[t][b, 0])
            sel = lambda qq, b=b: oracle.select(qq, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), int(lens[b]), w.k,
                                                score_scale=float(np.float32(scale)), n_init=ni, n_local=nl)
            i_o, c_o, r_o = oracle.selcache_step(qb, cq[b], cidx[b], ccnt[b], first[b], float(np.float32(theta)), sel)
            assert bool(reuse_g[b]) == r_o, (t, b)
            reuse_total += r_o
            assert cnt_g[b] == c_o and np.array_equal(idx_g[b], i_o), (t, b)
            att = oracle.attended_tokens(i_o, c_o, int(lens[b]), ni, nl)
            o_ref = oracle.sparse_attn(qb, w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), att, len(att),
                                       float(np.float32(1 / math.sqrt(w.D))))
            assert np.abs(W.as_f32(out_g[b, 0], w.dtype) - o_ref).max() <= 2e-2, (t, b)
    rate = reuse_total / (steps * w.B)
    print("cfg3 reuse rate %.3f" % rate)
    assert 0.2 < rate < 0.9


@pytest.mark.timeout(1500)
def test_config3_full_size_selection_cache_run(gpu):
    # configuration 3 as bench.py runs it: 8 sequences of 16384..65536 cached tokens, 64 steps, AR(1) queries, one
    # K/V row appended per sequence per step, theta = 0.9.  Reuse flags and index sets of every step and sequence
    # against Algorithm 1 on the oracle (band rule for the sets); attention on a sample of (step, sequence) pairs.
    from paper_2411_02886_amd.runtime import to_device, to_host
    theta, scale = 0.9, 1.0
    w = W.config3()
    steps = int(w.extra["steps"])
    qs = W.ar1_queries(w, steps, rho=0.95)
    ks, vs = W.appended_kv(w, steps)
    layer, _ = make_layer(w, max_seq_len=int(w.seq_lens.max()) + steps)
    lens = w.seq_lens.copy()
    cq = [np.zeros((w.H, w.D), np.uint16) for _ in range(w.B)]
    first = [np.ones(1, np.uint8) for _ in range(w.B)]
    cidx = [np.full(w.k, -1, np.int32) for _ in range(w.B)]
    ccnt = [np.zeros(1, np.int32) for _ in range(w.B)]
    kflat = w.k_pool.reshape(-1, w.H_kv, w.D); vflat = w.v_pool.reshape(-1, w.H_kv, w.D)
    kdev = layer.k_pool.view(-1, w.H_kv, w.D); vdev = layer.v_pool.view(-1, w.H_kv, w.D)
    reuse_total, exceptions = 0, 0
    sm = float(np.float32(1 / math.sqrt(w.D)))
    for t in range(steps):
        slots = np.array([int(w.pages_of(b)[int(lens[b]) // w.P]) * w.P + int(lens[b]) % w.P for b in range(w.B)])
        kflat[slots] = ks[t]; vflat[slots] = vs[t]
        sd = torch.from_numpy(slots).to(layer.device)
        kdev.index_copy_(0, sd, to_device(ks[t])); vdev.index_copy_(0, sd, to_device(vs[t]))
        lens += 1
        layer.seq_lens.copy_(to_device(lens))
        layer.step(to_device(qs[t]), theta=theta, score_scale=scale)
        torch.cuda.synchronize()
        reuse_g = to_host(layer.reuse); idx_g = to_host(layer.idx); cnt_g = to_host(layer.count)
        out_g = to_host(layer.out, bits16=True)
        for b in range(w.B):
            qb = np.ascontiguousarray(qs[t][b, 0])
            holder = {}

            def sel(qq, b=b):
                i, c, v, _ = oracle.select(qq, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), int(lens[b]), w.k,
                                           score_scale=float(np.float32(scale)), details=True)
                holder["votes"] = v
                return i, c
            i_o, c_o, r_o = oracle.selcache_step(qb, cq[b], cidx[b], ccnt[b], first[b], float(np.float32(theta)), sel)
            assert bool(reuse_g[b]) == r_o, (t, b)
            reuse_total += r_o
            if not r_o:     # a fresh selection: compare with the band rule, then adopt the GPU's set as the cached one
                exc = compare_index_sets(idx_g[b], int(cnt_g[b]), dict(idx=i_o, count=c_o, votes=holder["votes"]),
                                         "cfg3 t=%d b=%d" % (t, b))
                exceptions += len(exc)
                cidx[b][:] = idx_g[b]
            else:
                assert cnt_g[b] == c_o and np.array_equal(idx_g[b], cidx[b]), (t, b)
            if (t * w.B + b) % 37 == 0:
                o_ref = oracle.sparse_attn(qb, w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(b), idx_g[b], int(cnt_g[b]), sm)
                assert np.abs(W.as_f32(out_g[b, 0], w.dtype) - o_ref).max() <= 2e-2, (t, b)
        if t % 16 == 0:
            print("cfg3 full step", t, "reuse so far", reuse_total, flush=True)
    rate = reuse_total / (steps * w.B)
    print("cfg3 full size: reuse rate %.4f, tolerated near-tie exceptions %d" % (rate, exceptions))
    assert 0.5 < rate < 0.75


@pytest.mark.parametrize("dtype,H,H_kv,D,compact", [(W.F32, 8, 2, 64, False), (W.F32, 8, 2, 64, True), (W.BF16, 32, 8, 128, False),
                                                   (W.BF16, 32, 8, 128, True), (W.BF16, 28, 4, 128, True), (W.BF16, 6, 2, 64, True)],
                         ids=["f32-scores", "f32-codes", "bf16-scores", "bf16-codes-mfma", "bf16-28/4-codes-mfma", "bf16-6/2-codes"])
def test_check_inside_the_score_launch_equals_the_separate_check(gpu, dtype, H, H_kv, D, compact):
    """Algorithm 1 with the test taken in the prologue of the score kernels against the run that calls
    ts_selcache_check first: same reuse flags, C_Q, first flags, index sets and attention outputs, bit for bit, at
    every step of a run with hits and misses (the thresholds sit where the AR(1) queries cross them)."""
    from paper_2411_02886_amd.runtime import to_device, to_host
    steps = 16
    w = W.make_workload("scf", dtype=dtype, B=5, H=H, H_kv=H_kv, D=D, P=16, seq_lens=[900, 2500, 0, 70, 4100], k=64, seed=77,
                        beta=3.0, planted_per_head=1)
    qs = W.ar1_queries(w, steps, rho=0.95)
    bits16 = dtype == W.BF16
    hits = 0
    for theta in (0.9, 0.8):
        la, _ = make_layer(w); lb, _ = make_layer(w)
        for t in range(steps):
            print("fused check", theta, t, flush=True)
            qd = to_device(qs[t])
            la.step(qd, theta=theta, score_scale=0.2, compact=compact)
            lb.step(qd, theta=theta, score_scale=0.2, compact=compact, fused_check=True)
            torch.cuda.synchronize()
            ra, rb = to_host(la.reuse), to_host(lb.reuse)
            assert np.array_equal(ra, rb), (theta, t)
            hits += int(ra.sum())
            assert np.array_equal(to_host(la.cached_q, bits16=bits16), to_host(lb.cached_q, bits16=bits16)), (theta, t)
            assert np.array_equal(to_host(la.first), to_host(lb.first)), (theta, t)
            assert np.array_equal(to_host(la.idx), to_host(lb.idx)) and np.array_equal(to_host(la.count), to_host(lb.count)), (theta, t)
            assert np.array_equal(to_host(la.out, bits16=bits16), to_host(lb.out, bits16=bits16)), (theta, t)
    assert 0 < hits < 2 * steps * w.B


def test_step_picks_a_form_by_size_and_both_give_the_oracles_selection(gpu):
    from paper_2411_02886_amd.runtime import to_host
    w = W.config2(N=5000, k=300, seed=91)
    layer, q = make_layer(w)
    assert not layer.compact_form_pays()
    ora = oracle_decode(w, 0, score_scale=1.0)
    for form in (None, True, False):
        layer.idx.fill_(-3)
        layer.step(q, score_scale=1.0, compact=form, ranked_vote=True)
        torch.cuda.synchronize()
        compare_index_sets(to_host(layer.idx)[0], int(to_host(layer.count)[0]), ora, "form %s" % form)
    big = W.make_workload("big", dtype=W.BF16, H=32, H_kv=8, D=128, P=16, seq_lens=[300], k=16, seed=92)
    lb, _ = make_layer(big, max_seq_len=262144)
    assert lb.compact_form_pays()


def test_kernels_are_deterministic(gpu):
    from paper_2411_02886_amd.runtime import to_host
    w = W.config2(N=3000, k=200, seed=3)
    layer, q = make_layer(w)
    outs = []
    for _ in range(2):
        layer.step(q, score_scale=1.0)
        torch.cuda.synchronize()
        outs.append([to_host(x).copy() for x in (layer.scores, layer.row_stats, layer.votes, layer.idx, layer.out)])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("fused", [False, True], ids=["plain-calls", "check-in-score-launch+ranked-vote"])
def test_decode_steps_captured_in_a_hip_graph_replay_identically(gpu, fused):
    # Every hit/miss decision is taken on the device and the library neither allocates nor synchronises, so a
    # run of decode steps can be captured once and replayed.  Several replays, with eager work and
    # synchronisations in between, must each reproduce the eager run (indices, reuse flags, outputs).
    # fused: the run alternates the two (C_Q, first) buffers; an even number of steps leaves them where they began.
    from paper_2411_02886_amd.runtime import to_device, to_host
    steps, theta = 6, 0.9
    w = W.make_workload("graph", dtype=W.BF16, B=3, H=8, H_kv=2, D=128, P=16, seq_lens=[900, 2500, 70], k=48, seed=51,
                        beta=3.0, planted_per_head=1)
    qs = [to_device(q) for q in W.ar1_queries(w, steps, rho=0.95)]
    layer, _ = make_layer(w, num_initial=4, num_local=16)
    reuse_log = torch.zeros((steps, w.B), dtype=torch.uint8, device=layer.device)
    idx_log = torch.zeros((steps, w.B, w.k), dtype=torch.int32, device=layer.device)
    out_log = torch.zeros((steps,) + tuple(layer.out.shape), dtype=layer.out.dtype, device=layer.device)

    def run():
        layer.first.fill_(1)
        for t in range(steps):
            layer.step(qs[t], theta=theta, score_scale=0.1, fused_check=fused, ranked_vote=fused)
            reuse_log[t].copy_(layer.reuse); idx_log[t].copy_(layer.idx); out_log[t].copy_(layer.out)

    run(); torch.cuda.synchronize()
    ref = (to_host(reuse_log).copy(), to_host(idx_log).copy(), to_host(out_log).copy())
    assert 0 < ref[0].sum() < ref[0].size                      # hits and misses both occur
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side); torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run()
    for rep in range(4):
        reuse_log.zero_(); idx_log.fill_(-9); out_log.zero_()
        layer.idx.fill_(-9); layer.cached_q.zero_(); layer.cached_q_next.zero_()   # eager work between the replays
        torch.cuda.synchronize()
        g.replay(); torch.cuda.synchronize()
        got = (to_host(reuse_log), to_host(idx_log), to_host(out_log))
        for a, b in zip(got, ref):
            assert np.array_equal(a, b), rep
