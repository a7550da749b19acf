"""CPU oracle of the TokenSelect hot path -- TEST INFRASTRUCTURE ONLY.

A plain double-precision implementation (C, oracle/tokenselect_oracle.c, driven from numpy) of
what the GPU library computes: Algorithm 2 (paged dot product), Eq. 5 (head soft vote), the TopK
of Eq. 3-5, Algorithm 1 (Selection Cache), Eq. 2 (selective sparse attention) and Eq. 1 (full
attention, brute force); composed in numpy from these: Eq. 3 and Eq. 4 (the ablation selection
functions), forced initial / recent tokens (Sec. 6.1) and the mean-query chunk selection (Sec. 5.2).  It imports nothing from the HIP package and the HIP package imports
nothing from here; only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.

Readings of the paper taken here (each is an explicit argument or a named constant):
  * Eq. 5 carries no 1/sqrt(d): the vote softmax uses `score_scale` (default 1.0).
  * GQA: query head h reads KV head h // (H / H_kv).
  * Algorithm 1's cosine is one cosine over the flattened H*D query; reuse iff not first and
    cos >= theta; C_Q is the query of the last reselect.
  * TopK ties go to the lower token index; indices are returned ascending.
  * The top-k decision is an integer decided by floating point: it is taken on votes rounded to
    float32, the precision in which the library stores votes (`vote_dtype`).
  * Decode: the cached tokens already contain the current token; nothing is appended in Eq. 2.
  * Eq. 3 is read as the top-k of the dot products summed over the heads (the form whose weakness the
    paper describes: heads with large logits dominate); Eq. 4 lets every head vote for k tokens.
  * Forced tokens: the first n_init and last n_local cached tokens are attended in addition to the k
    selected ones; the selection function sees only the tokens between them (`ranked_range`).
  * Chunked prefill (`select_chunk`): votes are summed over heads and over the chunk's queries;
    `select_chunk_mean_query` is the paper's Sec. 5.2 form (mean query fed to the decode selection).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tokenselect_oracle.c")
_LIB = os.path.join(_HERE, "_build", "liboracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math) into oracle/_build/."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
                               "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_cosine.restype = ctypes.c_double
        _lib.oracle_selcache_check.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(a: np.ndarray, dtype: int) -> np.ndarray:
    want = np.uint16 if dtype == BF16 else np.float32
    assert a.dtype == want and a.flags.c_contiguous, (a.dtype, want)
    return a


def paged_qk_scores(q, k_pool, dtype, H_kv, P, page_indices, N) -> np.ndarray:
    """Algorithm 2.  q: [H][D] -> S [H][N] float64."""
    H, D = q.shape
    S = np.empty((H, N), dtype=np.float64)
    pi = np.ascontiguousarray(page_indices, dtype=np.int32)
    lib().oracle_paged_qk_scores(_p(_check(q, dtype)), _p(_check(k_pool, dtype)), ctypes.c_int(dtype),
                                 ctypes.c_int(H), ctypes.c_int(H_kv), ctypes.c_int(D), ctypes.c_int(P),
                                 _p(pi), ctypes.c_int64(N), _p(S))
    return S


def soft_vote(S: np.ndarray, score_scale: float = 1.0, with_stats: bool = False):
    """Eq. 5.  S: [H][N] float64 -> votes [N] float64 (and per-head (max, sum-exp))."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    H, N = S.shape
    votes = np.empty(N, dtype=np.float64)
    rmax = np.empty(H, dtype=np.float64)
    rsum = np.empty(H, dtype=np.float64)
    lib().oracle_soft_vote(_p(S), ctypes.c_int(H), ctypes.c_int64(N), ctypes.c_double(score_scale),
                           _p(votes), _p(rmax), _p(rsum))
    return (votes, rmax, rsum) if with_stats else votes


def topk(values: np.ndarray, k: int) -> Tuple[np.ndarray, int]:
    """TopK with ties to the lower index; returns (idx[k] ascending, -1 padded; count)."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    idx = np.empty(max(k, 0), dtype=np.int32)
    cnt = ctypes.c_int32(0)
    lib().oracle_topk(_p(v), ctypes.c_int64(v.size), ctypes.c_int(k), _p(idx), ctypes.byref(cnt))
    return idx, int(cnt.value)


def cosine(a: np.ndarray, b: np.ndarray, dtype: int) -> float:
    return float(lib().oracle_cosine(_p(_check(a, dtype)), _p(_check(b, dtype)), ctypes.c_int(dtype),
                                     ctypes.c_int64(a.size)))


def selcache_check(q: np.ndarray, cached_q: np.ndarray, dtype: int, first: np.ndarray, theta: float) -> int:
    """Condition + state update of Algorithm 1 (without calling S).  `first` is a uint8[1] cell and
    `cached_q` is updated in place on a miss.  Returns 1 for reuse."""
    assert first.dtype == np.uint8 and first.size == 1
    return int(lib().oracle_selcache_check(_p(_check(q, dtype)), _p(_check(cached_q, dtype)), ctypes.c_int(dtype),
                                           ctypes.c_int64(q.size), _p(first), ctypes.c_double(theta)))


def sparse_attn(q, k_pool, v_pool, dtype, H_kv, P, page_indices, idx, count, sm_scale,
                extra_first: int = 0, n_extra: int = 0, with_lse: bool = False):
    """Eq. 2 for one query position.  q: [H][D] -> out [H][D] float64."""
    H, D = q.shape
    out = np.empty((H, D), dtype=np.float64)
    lse = np.empty(H, dtype=np.float64)
    pi = np.ascontiguousarray(page_indices, dtype=np.int32)
    ix = np.ascontiguousarray(idx, dtype=np.int32)
    lib().oracle_sparse_attn(_p(_check(q, dtype)), _p(_check(k_pool, dtype)), _p(_check(v_pool, dtype)),
                             ctypes.c_int(dtype), ctypes.c_int(H), ctypes.c_int(H_kv), ctypes.c_int(D),
                             ctypes.c_int(P), _p(pi), _p(ix), ctypes.c_int(count), ctypes.c_int64(extra_first),
                             ctypes.c_int(n_extra), ctypes.c_double(sm_scale), _p(out), _p(lse))
    return (out, lse) if with_lse else out


def full_attn(q, k_pool, v_pool, dtype, H_kv, P, page_indices, N, sm_scale) -> np.ndarray:
    """Eq. 1, brute force over all N cached tokens."""
    H, D = q.shape
    out = np.empty((H, D), dtype=np.float64)
    pi = np.ascontiguousarray(page_indices, dtype=np.int32)
    lib().oracle_full_attn(_p(_check(q, dtype)), _p(_check(k_pool, dtype)), _p(_check(v_pool, dtype)),
                           ctypes.c_int(dtype), ctypes.c_int(H), ctypes.c_int(H_kv), ctypes.c_int(D),
                           ctypes.c_int(P), _p(pi), ctypes.c_int64(N), ctypes.c_double(sm_scale), _p(out))
    return out


# ------------------------------------------------------------------------------------------------
# The method's steps chained in the paper's order
# ------------------------------------------------------------------------------------------------

def decision_votes(votes64: np.ndarray) -> np.ndarray:
    """Votes in the precision the top-k decision is taken in (float32, widened back to float64)."""
    return votes64.astype(np.float32).astype(np.float64)


def ranked_range(N: int, n_init: int = 0, n_local: int = 0) -> Tuple[int, int]:
    """[lo, hi): the cached tokens that the selection ranks when the first n_init and the last n_local
    tokens are attended unconditionally (Sec. 6.1, implementation details: 128 initial and n_local most
    recent tokens are attended in addition to the k selected ones).  The initial block wins an overlap."""
    lo = min(max(int(n_init), 0), N)
    hi = max(lo, N - max(int(n_local), 0))
    return lo, hi


def select(q, k_pool, dtype, H_kv, P, page_indices, N, k, score_scale=1.0, details=False, n_init=0, n_local=0):
    """S(Q, k) of Eq. 5 for one decode query: scores -> soft vote -> top-k.  Returns (idx, count).
    With forced tokens (n_init, n_local) the selection function is applied to the K rows of the ranked
    range only: the softmax of Eq. 5 runs over that range and the k tokens come from it; the returned
    votes are 0 outside it."""
    S = paged_qk_scores(q, k_pool, dtype, H_kv, P, page_indices, N)
    lo, hi = ranked_range(N, n_init, n_local)
    votes = np.zeros(N, dtype=np.float64)
    if hi > lo:
        votes[lo:hi] = soft_vote(np.ascontiguousarray(S[:, lo:hi]), score_scale)
    idx, cnt = topk(decision_votes(votes[lo:hi]), k)
    idx = idx.copy()
    idx[:cnt] += lo
    return (idx, cnt, votes, S) if details else (idx, cnt)


def sum_vote(S: np.ndarray) -> np.ndarray:
    """Criticality of Eq. 3 (I_topk): the raw dot products summed over the heads.  S: [H][N] -> [N]."""
    votes = np.zeros(S.shape[1], dtype=np.float64)
    for h in range(S.shape[0]):          # head order 0..H-1, as the library sums
        votes += S[h]
    return votes


def head_vote(S: np.ndarray, k_head: int) -> np.ndarray:
    """Criticality of Eq. 4 (I_head-vote): every head takes its own top-k_head tokens of its raw dot products
    (float32 values as stored by the library, ties to the lower token index); a token's vote is the number of
    heads that took it.  S: [H][N] -> [N] integer-valued."""
    votes = np.zeros(S.shape[1], dtype=np.float64)
    for h in range(S.shape[0]):
        idx, cnt = topk(decision_votes(np.ascontiguousarray(S[h])), k_head)
        votes[idx[:cnt]] += 1.0
    return votes


def select_with(kind: str, q, k_pool, dtype, H_kv, P, page_indices, N, k, score_scale=1.0, details=False):
    """The three selection functions of Sec. 5.1 behind one call: kind = "soft" (Eq. 5), "sum" (Eq. 3) or
    "head" (Eq. 4, every head votes for k tokens).  Returns (idx, count[, votes, S])."""
    S = paged_qk_scores(q, k_pool, dtype, H_kv, P, page_indices, N)
    if kind == "soft":
        votes = soft_vote(S, score_scale)
    elif kind == "sum":
        votes = sum_vote(S)
    elif kind == "head":
        votes = head_vote(S, k)
    else:
        raise ValueError(kind)
    idx, cnt = topk(decision_votes(votes), k)
    return (idx, cnt, votes, S) if details else (idx, cnt)


def attended_tokens(idx, count, N, n_init=0, n_local=0) -> np.ndarray:
    """Token list of Eq. 2 with forced tokens: initial block, then the selected tokens, then the most
    recent block of the *current* length N (a cached selection made at a smaller N stays as it is)."""
    lo, hi = ranked_range(N, n_init, n_local)
    return np.concatenate([np.arange(lo, dtype=np.int32), np.asarray(idx[:count], dtype=np.int32),
                           np.arange(hi, N, dtype=np.int32)])


def select_chunk(qc, k_pool, dtype, H_kv, P, page_indices, N, k, score_scale=1.0, details=False, n_init=0, n_local=0):
    """Chunked-prefill selection with per-query votes: votes[t] = sum_c sum_h softmax_t(c*S[c][h][:])[t]
    over the N cached tokens; one top-k shared by the chunk.  qc: [C][H][D].  With forced tokens the first n_init
    and the last n_local *cached* tokens (the ones just before the chunk) are attended by every query of the chunk
    and only the tokens between them are ranked (the softmax of every query runs over that range)."""
    lo, hi = ranked_range(N, n_init, n_local)
    votes = np.zeros(N, dtype=np.float64)
    if hi > lo:
        for c in range(qc.shape[0]):
            S = paged_qk_scores(np.ascontiguousarray(qc[c]), k_pool, dtype, H_kv, P, page_indices, N)
            votes[lo:hi] += soft_vote(np.ascontiguousarray(S[:, lo:hi]), score_scale)
    idx, cnt = topk(decision_votes(votes[lo:hi]), k)
    idx = idx.copy()
    idx[:cnt] += lo
    return (idx, cnt, votes) if details else (idx, cnt)


def mean_query(qc: np.ndarray, dtype: int) -> np.ndarray:
    """Sec. 5.2: the mean of the chunk's queries, in the queries' element type.  qc: [C][H][D] -> [H][D]."""
    qc = _check(qc, dtype)
    out = np.empty(qc.shape[1:], dtype=qc.dtype)
    lib().oracle_mean_query(_p(qc), ctypes.c_int(dtype), ctypes.c_int(qc.shape[0]), ctypes.c_int64(out.size), _p(out))
    return out


def select_chunk_mean_query(qc, k_pool, dtype, H_kv, P, page_indices, N, k, score_scale=1.0, details=False,
                            n_init=0, n_local=0):
    """Sec. 5.2 as printed: one selection per chunk, S applied to the mean query over the N cached tokens."""
    return select(mean_query(qc, dtype), k_pool, dtype, H_kv, P, page_indices, N, k, score_scale, details,
                  n_init=n_init, n_local=n_local)


def selcache_step(q, cached_q, cached_idx, cached_cnt, first, theta, select_fn):
    """Algorithm 1 in full.  select_fn(q) -> (idx, count).  State (cached_q, cached_idx, cached_cnt[1],
    first[1]) is updated in place.  Returns (idx, count, reused)."""
    dtype = BF16 if q.dtype == np.uint16 else F32
    reuse = selcache_check(q, cached_q, dtype, first, theta)
    if not reuse:
        idx, cnt = select_fn(q)
        cached_idx[:] = idx
        cached_cnt[0] = cnt
    return cached_idx.copy(), int(cached_cnt[0]), bool(reuse)
