"""The entry point that allocates nothing (ts_topk_noalloc: workspace in a device array of the library image)
against ts_topk on the same votes: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _problem(ts, B, N, dev):
    # ts_topk reads only the shape fields and seq_lens; the pool pointers may stay empty tensors of the right type
    seq = torch.full((B,), N, dtype=torch.int32, device=dev)
    indptr = torch.zeros((B + 1,), dtype=torch.int32, device=dev)
    pages = torch.zeros((1,), dtype=torch.int32, device=dev)
    pool = torch.zeros((1, 16, 2, 64), dtype=torch.float32, device=dev)
    return ts.Problem(batch=B, chunk=1, num_q_heads=8, num_kv_heads=2, head_dim=64, page_size=16, max_seq_len=N,
                      dtype=ts.TS_F32, k_pool=pool, v_pool=pool, page_indptr=indptr, page_indices=pages, seq_lens=seq), seq


def test_noalloc_topk_matches_workspace_topk_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    dev = "cuda:0"
    rng = np.random.Generator(np.random.PCG64(2024))
    for B, N, k, flags in ((3, 50000, 700, 0), (2, 4100, 300, 0), (1, 9000, 64, ts.TS_TOPK_FLAT_VOTES), (2, 777, 1000, 0)):
        print("no-alloc top-k: B=%d N=%d k=%d flags=%d" % (B, N, k, flags), flush=True)
        p, seq = _problem(ts, B, N, dev)
        seq[B - 1] = max(1, N - 333)                      # ragged last sequence
        v = rng.standard_normal((B, N)).astype(np.float32)
        v[:, ::7] = v[:, 3:4]                              # heavy ties
        votes = torch.from_numpy(np.exp(v)).to(dev)
        nbytes = ts.ts_workspace_bytes(p, k)
        ws = torch.empty((nbytes + 255) // 256 * 64, dtype=torch.int32, device=dev)
        ts.ts_workspace_init(ws)
        idx_a = torch.full((B, k), -9, dtype=torch.int32, device=dev); cnt_a = torch.full((B,), -9, dtype=torch.int32, device=dev)
        idx_b = torch.full((B, k), -8, dtype=torch.int32, device=dev); cnt_b = torch.full((B,), -8, dtype=torch.int32, device=dev)
        ts.ts_topk(p, votes, k, idx_a, cnt_a, None, ws, flags=flags)
        ts.ts_topk_noalloc(p, votes, k, idx_b, cnt_b, None, flags=flags)
        torch.cuda.synchronize()
        assert torch.equal(cnt_a, cnt_b), (B, N, k)
        assert torch.equal(idx_a, idx_b), (B, N, k)


def test_noalloc_topk_rejects_sizes_beyond_its_array():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2411_02886_amd as ts
    ts.load()
    dev = "cuda:0"
    for B, N in ((17, 100), (1, 524288 + 2048), (16, 40000)):
        p, _ = _problem(ts, B, N, dev)
        votes = torch.zeros((1,), dtype=torch.float32, device=dev)
        idx = torch.zeros((B, 4), dtype=torch.int32, device=dev); cnt = torch.zeros((B,), dtype=torch.int32, device=dev)
        with pytest.raises(ts.TokenSelectError) as e:
            ts.ts_topk_noalloc(p, votes, 4, idx, cnt, None)
        assert e.value.status == -2
