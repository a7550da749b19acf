"""HIP-graph capture of the entry points that the decode graph test does not reach: the chunk step (both MFMA sweeps,
the flat-vote radix select, chunk attention with its slot and merge kernels), the mean-query chunk selection, the
Eq. 3 / Eq. 4 selection functions and the compact form.  The library neither allocates nor synchronises and clears
its scratch with fill kernels, so each of them can be recorded once and replayed; several replays, with eager work
and synchronisations in between, must each reproduce the eager results bit for bit."""
import math

import numpy as np
import pytest

import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    return ts


def capture_and_replay(run, outputs, scribble):
    """run(): launches on the current stream.  outputs: tensors it writes.  scribble(): eager work between replays."""
    from paper_2411_02886_amd.runtime import to_host
    run(); torch.cuda.synchronize()
    ref = [to_host(t).copy() for t in outputs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side); torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run()
    for rep in range(4):
        scribble()
        torch.cuda.synchronize()
        g.replay(); torch.cuda.synchronize()
        for i, (t, r) in enumerate(zip(outputs, ref)):
            assert np.array_equal(to_host(t), r), (rep, i)
    return ref


@pytest.mark.parametrize("mean_query", [False, True], ids=["per-query-votes", "mean-query"])
def test_chunk_step_replays_identically(gpu, mean_query):
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device
    C, L, k = 80, 3700, 160
    w = W.make_workload("graph_chunk", dtype=W.BF16, C=C, H=32, H_kv=8, D=128, P=16, seq_lens=[L], k=k, beta=2.5,
                        planted_per_head=6, plant_limit=L - C, seed=61)
    sel = ChunkSelector.from_workload(w, k=k, num_initial=8, num_local=24)
    q = to_device(w.q)
    if mean_query:
        sel.select_mean_query(q, 1.0); torch.cuda.synchronize()     # allocates its decode-shaped buffers on first use

    def run():
        if mean_query:
            sel.select_mean_query(q, 1.0)
        else:
            sel.select(q, 1.0)
        sel.attend(q)

    def scribble():
        sel.votes.fill_(7.0); sel.idx.fill_(-9); sel.count.fill_(-9); sel.out.zero_(); sel.lse.fill_(3.0)
        if not mean_query:
            sel.row_stats.fill_(1.0)

    # votes are defined for the cached tokens before the chunk; the entries behind them are not written
    ref = capture_and_replay(run, [sel.votes[:, :L - C], sel.idx, sel.count, sel.out, sel.lse], scribble)
    assert ref[2][0] == k and (ref[1][0] >= 0).all()


@pytest.mark.parametrize("kind", ["sum", "head", "compact"])
def test_other_selection_forms_replay_identically(gpu, kind):
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device
    w = W.make_workload("graph_forms", dtype=W.BF16, B=2, H=32, H_kv=8, D=128, P=16, seq_lens=[5200, 1300], k=96,
                        beta=3.0, planted_per_head=2, seed=62)
    layer = DecodeLayer.from_workload(w, num_initial=4, num_local=16)
    q = to_device(w.q)
    sm = 1.0 / math.sqrt(w.D)
    if kind == "compact":
        layer.select_compact(q, 1.0, None)
    else:
        layer.select(q, 1.0, None, kind=kind)                    # first use allocates the form's buffers
    torch.cuda.synchronize()

    def run():
        if kind == "compact":
            layer.select_compact(q, 1.0, None)
        else:
            layer.select(q, 1.0, None, kind=kind)
        layer.attend(q, sm)

    def scribble():
        layer.idx.fill_(-9); layer.count.fill_(-9); layer.out.zero_(); layer.votes.fill_(5.0)
        if kind == "compact":
            layer.codes.fill_(3); layer.vote_hi.fill_(2.0)

    n0, n1 = int(w.seq_lens[0]), int(w.seq_lens[1])            # entries behind a sequence's length are not written
    per_token = layer.vote_hi if kind == "compact" else layer.votes
    outs = [layer.idx, layer.count, layer.out, per_token[0, :n0], per_token[1, :n1]]
    ref = capture_and_replay(run, outs, scribble)
    assert (ref[1] == w.k).all()
