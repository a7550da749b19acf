"""NaN / Inf in the inputs: the results are unspecified, but every index a kernel forms from data is an integer key
digit, a clamped token id or a count bounded by its buffer, so the calls must complete and leave indices inside the
sequence; after ts_workspace_init the same layer must give the oracle's results again."""
import math

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
    return ts


def poison(t, dtype, where, what):
    """Overwrites the elements `where` (flat indices) of a device tensor with NaN / +Inf / -Inf bit patterns."""
    flat = t.view(-1)
    if dtype == W.BF16:
        bits = {"nan": 0x7fc0, "inf": 0x7f80, "-inf": 0xff80}[what]
        val = np.array([bits], dtype=np.uint16).view(np.int16)[0]
        flat[where] = int(val)
    else:
        flat[where] = {"nan": float("nan"), "inf": float("inf"), "-inf": float("-inf")}[what]


@pytest.mark.parametrize("dtype", [W.BF16, W.F32], ids=["bf16", "f32"])
@pytest.mark.parametrize("what", ["nan", "inf", "-inf"])
def test_decode_calls_survive_nonfinite_inputs(gpu, dtype, what):
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device, to_host
    lens = [3000, 700]
    w = W.make_workload("nonfinite", dtype=dtype, B=2, H=32, H_kv=8, D=128, P=16, seq_lens=lens, k=64, beta=2.0,
                        planted_per_head=1, seed=5)
    layer = DecodeLayer.from_workload(w, num_initial=4, num_local=16)
    sm = 1.0 / math.sqrt(w.D)
    rng = np.random.default_rng(3)
    for target in ("q", "k", "both"):
        print("nonfinite", what, target, flush=True)
        q = to_device(w.q)
        kp = layer.k_pool.clone()
        if target in ("q", "both"):
            poison(q, dtype, torch.from_numpy(rng.choice(q.numel(), 5, replace=False)).to(q.device), what)
        if target in ("k", "both"):
            poison(kp, dtype, torch.from_numpy(rng.choice(kp.numel(), 200, replace=False)).to(q.device), what)
        saved = layer.k_pool
        layer.swap_pool(kp, layer.v_pool)
        for compact in (False, True):
            layer.idx.fill_(-7); layer.count.fill_(-7); layer.first.fill_(1)
            layer.step(q, theta=0.9, score_scale=1.0, sm_scale=sm, compact=compact)
            torch.cuda.synchronize()
            idx, cnt = to_host(layer.idx), to_host(layer.count)
            for b, N in enumerate(lens):
                assert 0 <= cnt[b] <= min(w.k, N), (what, target, compact, b, cnt[b])
                assert ((idx[b] >= -1) & (idx[b] < N)).all(), (what, target, compact, b)
        layer.swap_pool(saved, layer.v_pool)
        gpu.ts_workspace_init(layer.ws)
    # the layer is healthy afterwards
    check_decode_against_oracle(w, layer, to_device(w.q), score_scale=1.0, label="after nonfinite inputs")


def test_chunk_calls_survive_nonfinite_inputs(gpu):
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device, to_host
    from test_gpu_prefill_parity import check_chunk
    C, L, k = 64, 2600, 100
    w = W.make_workload("nonfinite_chunk", dtype=W.BF16, C=C, H=16, H_kv=4, D=128, P=16, seq_lens=[L], k=k, beta=2.0,
                        planted_per_head=4, plant_limit=L - C, seed=6)
    rng = np.random.default_rng(4)
    for what in ("nan", "inf", "-inf"):
        print("nonfinite chunk", what, flush=True)
        sel = ChunkSelector.from_workload(w, k=k)
        q = to_device(w.q)
        poison(q, W.BF16, torch.from_numpy(rng.choice(q.numel(), 9, replace=False)).to(q.device), what)
        poison(sel.k_pool, W.BF16, torch.from_numpy(rng.choice(sel.k_pool.numel(), 300, replace=False)).to(q.device), what)
        sel.select(q, 1.0)
        sel.attend(q)
        torch.cuda.synchronize()
        idx, cnt = to_host(sel.idx), to_host(sel.count)
        assert 0 <= cnt[0] <= k and ((idx[0] >= -1) & (idx[0] < L - C)).all(), what
    check_chunk(gpu, w, k, 1.0, "after nonfinite inputs")
