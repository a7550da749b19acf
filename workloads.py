"""Seeded synthetic inputs for the TokenSelect hot path (decode and chunked prefill).

This module only *draws and lays out data*: random normals, bf16 rounding of the
inputs, the page permutation and the planted "critical" tokens.  It holds none of
the method's arithmetic (no scores, softmax, top-k or attention), so both the CPU
oracle's tests and the HIP path's tests/bench may use it without sharing code.

Stand-in statement: the paper evaluates on InfiniteBench / RULER / LongBench with
Qwen2-7B, Llama-3-8B and Yi-1.5-6B (Experiments, "Datasets"/"Baselines").  Neither
the datasets nor the weights are available, so these generators reproduce only the
*shapes* (head counts, head_dim, KV lengths 128K-1M, chunk 512, k = 2K/4K,
theta = 0.9) and the structural observation of Sec. 4 that critical tokens are few,
non-contiguous and head-specific (modelled as planted tokens whose key is pushed
towards one query head's direction).

Layouts (all C-contiguous numpy arrays):
  q            [B][C][H][D]            float32, or uint16 bf16 bit patterns
  k_pool/v_pool[num_pages][P][H_kv][D] same element type (token-major inside a page)
  page_indptr  [B+1] int32, page_indices [sum pages] int32 (logical order -> physical page)
  seq_lens     [B] int32
GQA head mapping: query head h reads KV head h // (H / H_kv) (contiguous groups).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_CHUNK_PAGES = 256          # pages per independently seeded chunk of K/V rows
_WORKERS = max(1, min(16, (os.cpu_count() or 1)))

F32 = 0
BF16 = 1


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bit patterns.

    Works through the array in cache-sized pieces with in-place integer operations."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.reshape(-1).view(np.uint32)
    out = np.empty(u.shape, dtype=np.uint16)
    step = 1 << 18
    tmp = np.empty(step, dtype=np.uint32)
    for i in range(0, u.size, step):
        c = u[i:i + step]
        t = tmp[:c.size]
        np.right_shift(c, 16, out=t)
        np.bitwise_and(t, 1, out=t)
        np.add(t, 0x7FFF, out=t)
        np.add(t, c, out=t)
        np.right_shift(t, 16, out=t)
        out[i:i + step] = t
    return out.reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f32(a: np.ndarray, dtype: int) -> np.ndarray:
    """Exact float32 view of a stored tensor of the given element type."""
    return bf16_bits_to_f32(a) if dtype == BF16 else np.asarray(a, dtype=np.float32)


def store(a_f32: np.ndarray, dtype: int) -> np.ndarray:
    """Quantise float32 values once into the storage element type."""
    if dtype == BF16:
        return f32_to_bf16_bits(a_f32)
    return np.ascontiguousarray(a_f32, dtype=np.float32)


@dataclass
class Workload:
    name: str
    dtype: int                 # F32 | BF16
    B: int
    C: int                     # queries per sequence (1 = decode)
    H: int
    H_kv: int
    D: int
    P: int                     # tokens per page
    k: int                     # tokens to select
    seq_lens: np.ndarray       # [B] int32 cached tokens per sequence
    q: np.ndarray              # [B][C][H][D]
    k_pool: np.ndarray         # [num_pages][P][H_kv][D]
    v_pool: np.ndarray
    page_indptr: np.ndarray    # [B+1] int32
    page_indices: np.ndarray   # int32
    planted: List[np.ndarray] = field(default_factory=list)   # per sequence: [H][n_planted] logical token ids
    beta: float = 0.0
    seed: int = 0
    extra: Dict[str, object] = field(default_factory=dict)

    @property
    def G(self) -> int:
        return self.H // self.H_kv

    @property
    def num_pages(self) -> int:
        return int(self.k_pool.shape[0])

    @property
    def max_seq_len(self) -> int:
        return int(self.seq_lens.max()) if self.B else 0

    def pages_of(self, b: int) -> np.ndarray:
        return self.page_indices[self.page_indptr[b]:self.page_indptr[b + 1]]

    def slots_of(self, b: int) -> np.ndarray:
        """Physical token slot (page*P + offset) of each logical cached token of sequence b."""
        n = int(self.seq_lens[b])
        t = np.arange(n, dtype=np.int64)
        return self.pages_of(b).astype(np.int64)[t // self.P] * self.P + t % self.P

    def esize(self) -> int:
        return 2 if self.dtype == BF16 else 4


def _choose_planted(rng: np.random.Generator, N: int, H: int, n_per_head: int,
                    non_contiguous: bool) -> np.ndarray:
    """Planted logical positions per query head: [H][n_per_head], uniform without replacement.

    Heads get disjoint positions when H*n_per_head <= N.  With non_contiguous=True a position
    adjacent (|dt| = 1) to any already planted one is rejected (Sec. 4: critical tokens are
    non-contiguous)."""
    total = H * n_per_head
    if total == 0:
        return np.zeros((H, 0), dtype=np.int64)
    if not non_contiguous:
        if total <= N:
            pos = rng.choice(N, size=total, replace=False)
            return np.sort(pos.reshape(H, n_per_head), axis=1).astype(np.int64)
        return np.stack([np.sort(rng.choice(N, size=n_per_head, replace=False)) for _ in range(H)]).astype(np.int64)
    # rejection on a candidate stream: keep a candidate only if neither neighbour is taken
    assert 3 * total <= N, "too many planted tokens for the non-contiguous recipe"
    taken = np.zeros(N + 2, dtype=bool)          # index shifted by one; guards at both ends
    out = np.empty(total, dtype=np.int64)
    n = 0
    while n < total:
        cand = rng.integers(0, N, size=2 * (total - n) + 16)
        for c in cand:
            if not (taken[c] or taken[c + 1] or taken[c + 2]):
                taken[c + 1] = True
                out[n] = c
                n += 1
                if n == total:
                    break
    rng.shuffle(out)
    return np.sort(out.reshape(H, n_per_head), axis=1)


def make_workload(name: str, *, dtype: int, B: int = 1, C: int = 1, H: int, H_kv: int, D: int,
                  P: int = 16, seq_lens, k: int, beta: float = 0.0, planted_per_head=0,
                  non_contiguous: bool = False, seed: int = 0, spare_tokens: int = 0,
                  identity_pages: bool = False, extra_pool_pages: int = 0,
                  plant_limit: Optional[int] = None) -> Workload:
    """Draw one workload.

    Q, K, V ~ N(0,1) in float32; the j-th planted token of query head h gets
    K[t, kv(h), :] += beta * Q[c, h]/|Q[c, h]| with c = j mod C (decode: c = 0); planted positions
    lie in the first `plant_limit` tokens (default: the whole sequence); values are then rounded
    once to the storage type.  The pool holds exactly the pages the sequences need (+ extra_pool_pages),
    and the logical->physical page map is a random permutation (identity_pages=True keeps logical
    order).  spare_tokens reserves room (pages are allocated for seq_len + spare_tokens) so that a
    decode loop can append tokens; the spare slots hold N(0,1) rows as well."""
    rng = np.random.Generator(np.random.PCG64(seed))
    seq_lens = np.asarray(seq_lens, dtype=np.int32).reshape(B)
    G = H // H_kv
    assert H % H_kv == 0
    q32 = rng.standard_normal((B, C, H, D), dtype=np.float32)
    pages_per_seq = [(int(n) + spare_tokens + P - 1) // P for n in seq_lens]
    page_indptr = np.zeros(B + 1, dtype=np.int32)
    page_indptr[1:] = np.cumsum(pages_per_seq)
    need = int(page_indptr[-1])
    num_pages = need + extra_pool_pages
    perm = np.arange(num_pages, dtype=np.int32) if identity_pages else rng.permutation(num_pages).astype(np.int32)
    page_indices = np.ascontiguousarray(perm[:need])
    elt = np.uint16 if dtype == BF16 else np.float32
    k_pool = np.zeros((num_pages, P, H_kv, D), dtype=elt)
    v_pool = np.zeros((num_pages, P, H_kv, D), dtype=elt)
    # pages not owned by any sequence still hold random data (a shared pool is never "clean")
    for pg in perm[need:]:
        k_pool[pg] = store(rng.standard_normal((P, H_kv, D), dtype=np.float32), dtype)
        v_pool[pg] = store(rng.standard_normal((P, H_kv, D), dtype=np.float32), dtype)
    planted_all: List[np.ndarray] = []
    for b in range(B):
        n = int(seq_lens[b])
        npg = pages_per_seq[b]
        cap = npg * P
        npl = planted_per_head if isinstance(planted_per_head, int) else int(planted_per_head[b])
        nplant = n if plant_limit is None else min(n, int(plant_limit))
        pl = _choose_planted(rng, nplant, H, npl, non_contiguous) if nplant > 0 else np.zeros((H, 0), dtype=np.int64)
        planted_all.append(pl)
        # planted (token, kv head) -> direction added to K, grouped by page-chunk for the workers below
        bumps = []
        if beta != 0.0 and pl.size:
            for h in range(H):
                for c in range(min(C, pl.shape[1])):
                    qh = q32[b, c, h]
                    u = (np.float32(beta) * qh / np.float32(np.linalg.norm(qh.astype(np.float64)))).astype(np.float32)
                    bumps.append((pl[h, c::C], h // G, u))
        pg = page_indices[page_indptr[b]:page_indptr[b + 1]]
        # K and V rows are drawn in chunks of _CHUNK_PAGES pages, each chunk from its own child stream
        # (SeedSequence(seed, spawn_key=(b, chunk))) so that chunks can be filled by a thread pool
        nchunks = (npg + _CHUNK_PAGES - 1) // _CHUNK_PAGES
        # planted tokens of a chunk: (local token, kv head, vector)
        per_chunk = [[] for _ in range(nchunks)]
        ctoks = _CHUNK_PAGES * P
        for toks, hkv, u in bumps:
            ci = toks // ctoks
            for cidx in np.unique(ci):
                per_chunk[int(cidx)].append((toks[ci == cidx] - int(cidx) * ctoks, hkv, u))

        def fill(ci, b=b, pg=pg, per_chunk=per_chunk, npg=npg):
            p0, p1 = ci * _CHUNK_PAGES, min(npg, (ci + 1) * _CHUNK_PAGES)
            g = np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed, spawn_key=(b + 1, ci))))
            kl = g.standard_normal(((p1 - p0) * P, H_kv, D), dtype=np.float32)
            vl = g.standard_normal(((p1 - p0) * P, H_kv, D), dtype=np.float32)
            for toks, hkv, u in per_chunk[ci]:
                kl[toks, hkv, :] += u
            k_pool[pg[p0:p1]] = store(kl, dtype).reshape(p1 - p0, P, H_kv, D)
            v_pool[pg[p0:p1]] = store(vl, dtype).reshape(p1 - p0, P, H_kv, D)

        if nchunks > 1:
            with ThreadPoolExecutor(max_workers=_WORKERS) as ex:
                list(ex.map(fill, range(nchunks)))
        else:
            for ci in range(nchunks):
                fill(ci)
    return Workload(name=name, dtype=dtype, B=B, C=C, H=H, H_kv=H_kv, D=D, P=P, k=k,
                    seq_lens=seq_lens, q=store(q32, dtype), k_pool=k_pool, v_pool=v_pool,
                    page_indptr=page_indptr, page_indices=page_indices, planted=planted_all,
                    beta=beta, seed=seed)


# ---------------------------------------------------------------------------------------------
# The five named configurations (shapes and recipes; `scale` < 1 shrinks the token count only)
# ---------------------------------------------------------------------------------------------

def config1(seed: int = 1001, N: int = 4096, **kw) -> Workload:
    """Tiny decode, fp32: H 8 over 2 KV heads, D 64, 4096 tokens, 32 planted per head (beta 3), k 256."""
    args = dict(dtype=F32, H=8, H_kv=2, D=64, seq_lens=[N], k=256, beta=3.0,
                planted_per_head=min(32, N // 8), seed=seed)
    args.update(kw)
    return make_workload("cfg1_tiny_fp32", **args)


def config2(seed: int = 1002, N: int = 131072, **kw) -> Workload:
    """Llama-3-8B-shaped layer, bf16: H 32 / 8, D 128, 131072 tokens, 0.5% planted per head (beta 2.5), k 2048."""
    args = dict(dtype=BF16, H=32, H_kv=8, D=128, seq_lens=[N], k=2048, beta=2.5,
                planted_per_head=int(round(0.005 * N)), seed=seed)
    args.update(kw)
    return make_workload("cfg2_llama3_8b_bf16_128k", **args)


def config3_lengths(seed: int = 1003, B: int = 8, lo: int = 16384, hi: int = 65536) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    return rng.integers(lo, hi + 1, size=B).astype(np.int32)


def config3(seed: int = 1003, B: int = 8, lo: int = 16384, hi: int = 65536, steps: int = 64, **kw) -> Workload:
    """Selection-Cache decode run, bf16, Llama-3-8B head shapes: B sequences with lengths uniform in
    [lo, hi]; pages are reserved for `steps` appended tokens.  The query stream comes from
    ar1_queries()."""
    lens = config3_lengths(seed, B, lo, hi)
    args = dict(dtype=BF16, B=B, H=32, H_kv=8, D=128, seq_lens=lens, k=2048, beta=2.5,
                planted_per_head=[int(round(0.005 * int(n))) for n in lens], seed=seed, spare_tokens=steps)
    args.update(kw)
    w = make_workload("cfg3_selcache_bf16", **args)
    w.extra["steps"] = steps
    return w


def ar1_queries(w: Workload, steps: int, rho: float = 0.95, seed: Optional[int] = None) -> np.ndarray:
    """Query stream q_t = rho*q_{t-1} + sqrt(1-rho^2)*eps, eps ~ N(0,1) elementwise, q_0 = the
    workload's query.  Returned in the workload's storage type, shape [steps][B][1][H][D]; each
    step's value is rounded to the storage type *after* the float32 recursion."""
    rng = np.random.Generator(np.random.PCG64((w.seed if seed is None else seed) + 104729))
    cur = as_f32(w.q, w.dtype).astype(np.float32).copy()
    out = np.empty((steps,) + cur.shape, dtype=w.q.dtype)
    out[0] = store(cur, w.dtype)
    s = np.float32(np.sqrt(1.0 - rho * rho))
    for t in range(1, steps):
        cur = np.float32(rho) * cur + s * rng.standard_normal(cur.shape, dtype=np.float32)
        out[t] = store(cur, w.dtype)
    return out


def appended_kv(w: Workload, steps: int, seed: Optional[int] = None):
    """K/V rows appended per decode step: ([steps][B][H_kv][D], same) in the storage type."""
    rng = np.random.Generator(np.random.PCG64((w.seed if seed is None else seed) + 1299709))
    ks = store(rng.standard_normal((steps, w.B, w.H_kv, w.D), dtype=np.float32), w.dtype)
    vs = store(rng.standard_normal((steps, w.B, w.H_kv, w.D), dtype=np.float32), w.dtype)
    return ks, vs


def config4(seed: int = 1004, N: int = 1048576, **kw) -> Workload:
    """Qwen2-7B-shaped layer, bf16: H 28 / 4, D 128, 1048576 tokens, 0.1% planted per head at
    non-contiguous positions (beta 2.5, the value of the 128K configuration), k 4096."""
    args = dict(dtype=BF16, H=28, H_kv=4, D=128, seq_lens=[N], k=4096, beta=2.5,
                planted_per_head=int(round(0.001 * N)), non_contiguous=True, seed=seed)
    args.update(kw)
    return make_workload("cfg4_qwen2_7b_bf16_1m", **args)


def config5(seed: int = 1005, N: int = 262144, C: int = 512, **kw) -> Workload:
    """Chunked-prefill selection, bf16: C consecutive queries over N cached tokens, H 32 / 8, D 128,
    0.5% planted per head (beta 2.5), shared k 4096.  The chunk's own K/V rows are the last C tokens
    of the sequence (seq_len = N + C); selection looks at the first N only."""
    args = dict(dtype=BF16, C=C, H=32, H_kv=8, D=128, seq_lens=[N + C], k=4096, beta=2.5,
                planted_per_head=int(round(0.005 * N)), seed=seed, plant_limit=N)
    args.update(kw)
    w = make_workload("cfg5_prefill_bf16", **args)
    w.extra["n_cached"] = N
    return w


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
