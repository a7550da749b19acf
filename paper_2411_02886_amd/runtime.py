"""Device-side buffers for one attention layer's decode loop and the five-call step.

Orchestration only: uploads a paged workload given as numpy arrays, allocates the intermediate
buffers with torch (device memory) and issues the C-ABI calls in the order of Fig. 4 / Algorithm 1.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as ts


def to_device(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """numpy -> device tensor; uint16 (bf16 bit patterns) travel as int16 raw bits."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(device)


def to_host(t: torch.Tensor, bits16: bool = False) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if bits16 else a


class DecodeLayer:
    """Paged KV pool of B sequences on the GPU plus every buffer the decode step needs."""

    def __init__(self, *, dtype, H, H_kv, D, P, k, k_pool, v_pool, page_indptr, page_indices, seq_lens,
                 max_seq_len=None, device="cuda:0", num_initial=0, num_local=0):
        self.device = device
        self.dtype, self.H, self.H_kv, self.D, self.P, self.k = dtype, H, H_kv, D, P, k
        self.num_initial, self.num_local = int(num_initial), int(num_local)   # forced tokens (Sec. 6.1)
        self.B = int(len(seq_lens))
        self.k_pool = k_pool if torch.is_tensor(k_pool) else to_device(k_pool, device)
        self.v_pool = v_pool if torch.is_tensor(v_pool) else to_device(v_pool, device)
        self.page_indptr = to_device(np.asarray(page_indptr, dtype=np.int32), device)
        self.page_indices = to_device(np.asarray(page_indices, dtype=np.int32), device)
        self.seq_lens = to_device(np.asarray(seq_lens, dtype=np.int32), device)
        self.max_seq_len = int(max_seq_len if max_seq_len is not None else max(1, int(np.max(seq_lens))))
        self._make_problem()
        B, Hq, M = self.B, H, self.max_seq_len
        self.scores = torch.empty((B, M, Hq), dtype=torch.float32, device=device)
        self.row_stats = torch.empty((B, Hq, 2), dtype=torch.float32, device=device)
        self.votes = torch.empty((B, M), dtype=torch.float32, device=device)
        self.idx = torch.full((B, k), -1, dtype=torch.int32, device=device)
        self.count = torch.zeros((B,), dtype=torch.int32, device=device)
        edt = torch.int16 if dtype == ts.TS_BF16 else torch.float32
        self.out = torch.zeros((B, 1, Hq, D), dtype=edt, device=device)
        self.lse = torch.empty((B, 1, Hq), dtype=torch.float32, device=device)
        self.cached_q = torch.zeros((B, Hq, D), dtype=edt, device=device)
        self.first = torch.ones((B,), dtype=torch.uint8, device=device)
        self.reuse = torch.zeros((B,), dtype=torch.uint8, device=device)
        # second (C_Q, first) pair of the steps that run Algorithm 1's test inside the score launch
        self.cached_q_next = torch.zeros((B, Hq, D), dtype=edt, device=device)
        self.first_next = torch.ones((B,), dtype=torch.uint8, device=device)
        nbytes = ts.ts_workspace_bytes(self.problem, k)
        self.ws = torch.empty((nbytes + 255) // 256 * 64, dtype=torch.int32, device=device)
        ts.ts_workspace_init(self.ws)

    def _make_problem(self):
        self.problem = ts.Problem(batch=self.B, chunk=1, num_q_heads=self.H, num_kv_heads=self.H_kv, head_dim=self.D,
                                  page_size=self.P, max_seq_len=self.max_seq_len, dtype=self.dtype,
                                  k_pool=self.k_pool, v_pool=self.v_pool, page_indptr=self.page_indptr,
                                  page_indices=self.page_indices, seq_lens=self.seq_lens,
                                  num_initial=self.num_initial, num_local=self.num_local)

    @classmethod
    def from_workload(cls, w, device="cuda:0", max_seq_len=None, num_initial=0, num_local=0):
        return cls(dtype=w.dtype, H=w.H, H_kv=w.H_kv, D=w.D, P=w.P, k=w.k, k_pool=w.k_pool, v_pool=w.v_pool,
                   page_indptr=w.page_indptr, page_indices=w.page_indices, seq_lens=w.seq_lens,
                   max_seq_len=max_seq_len, device=device, num_initial=num_initial, num_local=num_local)

    def swap_pool(self, k_pool: torch.Tensor, v_pool: torch.Tensor, page_indices: torch.Tensor = None):
        """Points the layer at another resident pool of the same shape (benchmark cache rotation)."""
        self.k_pool, self.v_pool = k_pool, v_pool
        if page_indices is not None:
            self.page_indices = page_indices
        self._make_problem()

    # ---- the five calls
    def selcache_check(self, q, theta):
        ts.ts_selcache_check(self.problem, q, self.cached_q, self.first, theta, self.reuse)

    def _swap_selcache_state(self):
        self.cached_q, self.cached_q_next = self.cached_q_next, self.cached_q
        self.first, self.first_next = self.first_next, self.first

    def select(self, q, score_scale=1.0, skip=None, kind="soft", check_theta=None, ranked_vote=False):
        """kind: "soft" = Eq. 5 (the method), "sum" = Eq. 3, "head" = Eq. 4 (the paper's ablation baselines).
        check_theta: run Algorithm 1's test inside the score launch (skip is then self.reuse).
        ranked_vote (Eq. 5 only): the vote launch also builds the first histogram of the TopK
        (ts_soft_vote_ranked + TS_TOPK_VOTE_HIST)."""
        if check_theta is not None:
            ts.ts_paged_qk_scores_checked(self.problem, q, self.cached_q, self.cached_q_next, self.first, self.first_next,
                                          self.reuse, check_theta, self.scores, score_scale, self.ws)
            self._swap_selcache_state()
            skip = self.reuse
        else:
            ts.ts_paged_qk_scores(self.problem, q, self.scores, score_scale, skip, self.ws)
        if kind == "soft" and ranked_vote:
            ts.ts_soft_vote_ranked(self.problem, self.scores, score_scale, self.row_stats, self.votes, skip, self.ws)
            ts.ts_topk(self.problem, self.votes, self.k, self.idx, self.count, skip, self.ws, flags=ts.TS_TOPK_VOTE_HIST)
            return
        if kind == "soft":
            ts.ts_soft_vote(self.problem, self.scores, score_scale, self.row_stats, self.votes, skip, self.ws)
        elif kind == "sum":
            ts.ts_sum_vote(self.problem, self.scores, self.votes, skip)
        elif kind == "head":
            if getattr(self, "_hv_scratch", None) is None:
                nb = ts.ts_head_vote_scratch_bytes(self.problem)
                self._hv_scratch = torch.empty((nb + 255) // 256 * 64, dtype=torch.int32, device=self.device)
            ts.ts_head_vote(self.problem, self.scores, self.k, self.votes, skip, self._hv_scratch)
        else:
            raise ValueError(kind)
        ts.ts_topk(self.problem, self.votes, self.k, self.idx, self.count, skip, self.ws)

    def select_compact(self, q, score_scale=1.0, skip=None, check_theta=None, lower_bounds=True):
        """Eq. 5 selection without the score matrix in memory: one byte per score, vote bounds, exact votes of
        the candidates.  Same idx / count as select(kind="soft")."""
        if getattr(self, "codes", None) is None:
            B, M = self.B, self.max_seq_len
            self.codes = torch.empty((B, M, self.H), dtype=torch.uint8, device=self.device)
            self.vote_hi = torch.empty((B, M), dtype=torch.float32, device=self.device)
            self.vote_lo = torch.empty((B, M), dtype=torch.float32, device=self.device)
            self.sel_votes = torch.zeros((B, self.k), dtype=torch.float32, device=self.device)
        if check_theta is not None:
            ts.ts_paged_qk_codes_checked(self.problem, q, self.cached_q, self.cached_q_next, self.first, self.first_next,
                                         self.reuse, check_theta, self.codes, score_scale, self.ws)
            self._swap_selcache_state()
            skip = self.reuse
        else:
            ts.ts_paged_qk_codes(self.problem, q, self.codes, score_scale, skip, self.ws)
        ts.ts_soft_vote_bounds(self.problem, self.codes, score_scale, self.row_stats, self.vote_hi,
                               self.vote_lo if lower_bounds else None, skip,
                               self.ws)
        ts.ts_topk_exact(self.problem, q, self.vote_hi, self.row_stats, score_scale, self.k, self.idx, self.count, skip,
                         self.ws, sel_votes=getattr(self, "sel_votes", None))

    def attend(self, q, sm_scale):
        ts.ts_sparse_paged_attn(self.problem, q, self.idx, self.k, self.count, sm_scale, self.out, self.lse, self.ws)

    def compact_form_pays(self) -> bool:
        """Which form of the Eq. 5 selection is the faster step here (measured on MI355X): while the fp32 score matrix
        fits the L2 with room to spare (131072 tokens of 32 heads: 16 MiB) the five-call form is, beyond that the
        compact form, which never writes it (crossover between 128K and 256K tokens of 32 heads)."""
        return self.B * self.max_seq_len * self.H * 4 > 24 * 2**20

    def step(self, q, *, theta=None, score_scale=1.0, sm_scale=None, compact=False, fused_check=False, ranked_vote=False):
        """One decode step: Selection Cache check (when theta is given), selection on a miss, sparse
        attention.  No host synchronisation.  compact: the form of the selection (None = whichever is the faster one
        at this size, see compact_form_pays).  fused_check: the check runs inside the score launch (one launch
        less; self.cached_q / self.first are swapped with their second copies after the step)."""
        sm = sm_scale if sm_scale is not None else 1.0 / float(np.sqrt(self.D))
        if compact is None:
            compact = self.compact_form_pays()
        skip, check_theta = None, None
        if theta is not None:
            if fused_check:
                check_theta = theta
            else:
                self.selcache_check(q, theta)
                skip = self.reuse
        if compact:
            self.select_compact(q, score_scale, skip, check_theta=check_theta, lower_bounds=False)
        else:
            self.select(q, score_scale, skip, check_theta=check_theta, ranked_vote=ranked_vote)
        self.attend(q, sm)


class ChunkSelector:
    """Chunked-prefill selection for one layer: the C queries of a chunk are the last C tokens of
    their sequences; two MFMA sweeps give the votes, ts_topk the shared index set."""

    def __init__(self, *, C, H, H_kv, D, P, k, k_pool, v_pool, page_indptr, page_indices, seq_lens, max_seq_len=None,
                 device="cuda:0", num_initial=0, num_local=0):
        self.C, self.H, self.H_kv, self.D, self.P, self.k = C, H, H_kv, D, P, k
        self.num_initial, self.num_local = int(num_initial), int(num_local)   # forced cached tokens (Sec. 6.1)
        self.B = int(len(seq_lens))
        self.k_pool = k_pool if torch.is_tensor(k_pool) else to_device(k_pool, device)
        self.v_pool = v_pool if torch.is_tensor(v_pool) else to_device(v_pool, device)
        self.page_indptr = to_device(np.asarray(page_indptr, dtype=np.int32), device)
        self.page_indices = to_device(np.asarray(page_indices, dtype=np.int32), device)
        self.seq_lens = to_device(np.asarray(seq_lens, dtype=np.int32), device)
        self.max_seq_len = int(max_seq_len if max_seq_len is not None else max(1, int(np.max(seq_lens))))
        self.problem = ts.Problem(batch=self.B, chunk=C, num_q_heads=H, num_kv_heads=H_kv, head_dim=D, page_size=P,
                                  max_seq_len=self.max_seq_len, dtype=ts.TS_BF16, k_pool=self.k_pool,
                                  v_pool=self.v_pool, page_indptr=self.page_indptr, page_indices=self.page_indices,
                                  seq_lens=self.seq_lens, num_initial=self.num_initial, num_local=self.num_local)
        B, M = self.B, self.max_seq_len
        self.row_stats = torch.empty((B, C, H, 2), dtype=torch.float32, device=device)
        self.votes = torch.zeros((B, M), dtype=torch.float32, device=device)
        self.idx = torch.full((B, k), -1, dtype=torch.int32, device=device)
        self.count = torch.zeros((B,), dtype=torch.int32, device=device)
        self.out = torch.zeros((B, C, H, D), dtype=torch.int16, device=device)
        self.lse = torch.empty((B, C, H), dtype=torch.float32, device=device)
        nbytes = ts.ts_workspace_bytes(self.problem, k)
        self.ws = torch.empty((nbytes + 255) // 256 * 64, dtype=torch.int32, device=device)
        ts.ts_workspace_init(self.ws)

    @classmethod
    def from_workload(cls, w, k=None, device="cuda:0", num_initial=0, num_local=0):
        return cls(C=w.C, H=w.H, H_kv=w.H_kv, D=w.D, P=w.P, k=w.k if k is None else k, k_pool=w.k_pool, v_pool=w.v_pool,
                   page_indptr=w.page_indptr, page_indices=w.page_indices, seq_lens=w.seq_lens, device=device,
                   num_initial=num_initial, num_local=num_local)

    def select(self, q, score_scale=1.0):
        ts.ts_chunk_row_stats(self.problem, q, score_scale, self.row_stats, self.ws)
        ts.ts_chunk_soft_vote(self.problem, q, self.row_stats, score_scale, self.votes, self.ws)
        ts.ts_topk(self.problem, self.votes, self.k, self.idx, self.count, None, self.ws)

    def attend(self, q, sm_scale=None):
        sm = sm_scale if sm_scale is not None else 1.0 / float(np.sqrt(self.D))
        ts.ts_sparse_paged_attn(self.problem, q, self.idx, self.k, self.count, sm, self.out, self.lse, self.ws)

    # ---- Sec. 5.2 as printed: one selection per chunk with the mean query, through the decode calls
    def _mean_query_state(self):
        if getattr(self, "_mq", None) is None:
            dev = self.k_pool.device
            B, M = self.B, self.max_seq_len
            cached = torch.clamp(self.seq_lens - self.C, min=0).to(torch.int32)
            prob = ts.Problem(batch=B, chunk=1, num_q_heads=self.H, num_kv_heads=self.H_kv, head_dim=self.D,
                              page_size=self.P, max_seq_len=M, dtype=ts.TS_BF16, k_pool=self.k_pool, v_pool=self.v_pool,
                              page_indptr=self.page_indptr, page_indices=self.page_indices, seq_lens=cached,
                              num_initial=self.num_initial, num_local=self.num_local)
            nbytes = ts.ts_workspace_bytes(prob, self.k)
            ws = torch.empty((nbytes + 255) // 256 * 64, dtype=torch.int32, device=dev)
            ts.ts_workspace_init(ws)
            self._mq = dict(problem=prob, cached=cached, ws=ws,
                            q_mean=torch.zeros((B, 1, self.H, self.D), dtype=torch.int16, device=dev),
                            scores=torch.empty((B, M, self.H), dtype=torch.float32, device=dev),
                            row_stats=torch.empty((B, self.H, 2), dtype=torch.float32, device=dev))
        return self._mq

    def select_mean_query(self, q, score_scale=1.0):
        """Mean of the chunk's queries -> decode score pass, soft vote and top-k over the cached tokens.
        Fills self.votes / self.idx / self.count like select()."""
        m = self._mean_query_state()
        ts.ts_chunk_mean_query(self.problem, q, m["q_mean"])
        ts.ts_paged_qk_scores(m["problem"], m["q_mean"], m["scores"], score_scale, None, m["ws"])
        ts.ts_soft_vote(m["problem"], m["scores"], score_scale, m["row_stats"], self.votes, None, m["ws"])
        # the mean of many queries can be short, its votes flat: take the distribution-independent select
        ts.ts_topk(m["problem"], self.votes, self.k, self.idx, self.count, None, m["ws"], flags=ts.TS_TOPK_FLAT_VOTES)
