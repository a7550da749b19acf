"""Pools beyond 4 GiB.  The pages of the sequences lie scattered over a K pool and a V pool of 5 GiB each, three quarters
of them above the 4 GiB line and one at the very end, so byte offsets into the pools need more than 32 bits in every
kernel that reads K or V: both score kernels, the exact re-evaluation of the compact form, both attention forms and the
chunk sweeps.  The oracle sees the same tokens in the small pool they were generated in."""
import dataclasses
import math

import numpy as np
import pytest

import workloads as W
from parity_util import check_decode_against_oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

POOL_BYTES = 5 << 30


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    yield ts
    torch.cuda.empty_cache()


def spread_over_large_pools(w, seed):
    """The workload with its pages moved into two zero-filled device pools of POOL_BYTES each."""
    from paper_2411_02886_amd.runtime import to_device
    page_bytes = w.P * w.H_kv * w.D * (2 if w.dtype == W.BF16 else 4)
    big_pages, line = POOL_BYTES // page_bytes, (4 << 30) // page_bytes
    n = w.num_pages
    assert n >= 8 and big_pages - line > n
    rng = np.random.default_rng(seed)
    below = rng.choice(line, size=n // 4, replace=False)
    above = line + rng.choice(big_pages - 1 - line, size=n - n // 4 - 1, replace=False)
    new_ids = np.concatenate([below, above, [big_pages - 1]]).astype(np.int64)
    rng.shuffle(new_ids)
    dt = torch.int16 if w.dtype == W.BF16 else torch.float32
    big_k = torch.zeros((big_pages, w.P, w.H_kv, w.D), dtype=dt, device="cuda:0")
    big_v = torch.zeros((big_pages, w.P, w.H_kv, w.D), dtype=dt, device="cuda:0")
    ids = torch.from_numpy(new_ids).to("cuda:0")
    big_k[ids] = to_device(w.k_pool)
    big_v[ids] = to_device(w.v_pool)
    assert big_k.numel() * big_k.element_size() > (4 << 30)
    return dataclasses.replace(w, k_pool=big_k, v_pool=big_v, page_indices=new_ids[w.page_indices].astype(np.int32))


@pytest.mark.parametrize("shape", [(W.BF16, 32, 8, 128, 16, [6000, 3333], 256),      # matrix-core score kernels
                                   (W.BF16, 28, 4, 128, 16, [4500], 128),
                                   (W.F32, 8, 2, 64, 1, [2500, 700], 64),              # vector score kernel, one token per page
                                   (W.F32, 16, 16, 128, 4, [1800], 100)],
                         ids=lambda s: "dt%d_H%d_%d_D%d_P%d" % s[:5])
def test_decode_step_on_pools_beyond_4_gib(gpu, shape):
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device
    from test_gpu_compact_selection import check_compact
    dtype, H, H_kv, D, P, lens, k = shape
    print("large pool decode", shape, flush=True)
    w = W.make_workload("large_pool", dtype=dtype, B=len(lens), H=H, H_kv=H_kv, D=D, P=P, seq_lens=lens, k=k, beta=3.0,
                        planted_per_head=2, seed=H * 131 + D)
    wl = spread_over_large_pools(w, seed=H)
    layer = DecodeLayer.from_workload(wl, num_initial=4, num_local=16)
    q = to_device(w.q)
    check_decode_against_oracle(w, layer, q, score_scale=1.0, label="large pool " + str(shape))
    check_compact(w, layer, q, score_scale=1.0 / math.sqrt(D), label="large pool " + str(shape))
    del layer, wl
    torch.cuda.empty_cache()


def test_chunk_step_on_pools_beyond_4_gib(gpu):
    from test_gpu_prefill_parity import check_chunk
    C, H, H_kv, D, P, L, k = 96, 32, 8, 128, 16, 4200, 200
    print("large pool chunk", (C, H, H_kv, D, P, L, k), flush=True)
    w = W.make_workload("large_pool_chunk", dtype=W.BF16, C=C, H=H, H_kv=H_kv, D=D, P=P, seq_lens=[L], k=k, beta=2.5,
                        planted_per_head=8, plant_limit=L - C, seed=77)
    wl = spread_over_large_pools(w, seed=5)
    check_chunk(gpu, w, k, 1.0, "large pool chunk", n_init=8, n_local=32, gpu_w=wl)
    del wl
    torch.cuda.empty_cache()
