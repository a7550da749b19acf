"""ctypes binding of include/tokenselect.h: argument marshalling only.

Every function takes torch tensors that already live on the GPU (PyTorch is used for device memory
and streams, nothing else) and forwards their data pointers; all arithmetic runs in the HIP kernels
of libtokenselect.so.  There is no CPU fallback: if the library is missing, load() raises.
"""
from __future__ import annotations

import ctypes
import os
import re
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtokenselect.so")
_HEADER = os.path.join(os.path.dirname(_HERE), "include", "tokenselect.h")

TS_F32, TS_BF16 = 0, 1
TS_TOPK_FLAT_VOTES = 1
TS_TOPK_VOTE_HIST = 2


class TokenSelectError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, ts_strerror(status), status))


class _CProblem(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("chunk", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("max_seq_len", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p), ("page_indptr", ctypes.c_void_p),
        ("page_indices", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("num_initial", ctypes.c_int32), ("num_local", ctypes.c_int32),
    ]


class _CSelcache(ctypes.Structure):
    _fields_ = [("cached_q", ctypes.c_void_p), ("cached_q_next", ctypes.c_void_p), ("first", ctypes.c_void_p),
                ("first_next", ctypes.c_void_p), ("reuse", ctypes.c_void_p), ("theta", ctypes.c_float)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def declared_symbols():
    """Names of the functions include/tokenselect.h declares."""
    text = open(_HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ts_[a-z_]+)\s*\(", text)))


def load():
    """Loads libtokenselect.so (built by paper_2411_02886_amd.build).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError("%s is missing: run `python -m paper_2411_02886_amd.build` (no CPU fallback exists)"
                                    % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        pp = ctypes.POINTER(_CProblem)
        L.ts_version.restype = i32
        L.ts_strerror.restype = ctypes.c_char_p
        L.ts_strerror.argtypes = [i32]
        L.ts_workspace_bytes.argtypes = [pp, i32, ctypes.POINTER(sz)]
        L.ts_workspace_init.argtypes = [vp, sz, vp]
        L.ts_paged_qk_scores.argtypes = [pp, vp, vp, f32, vp, vp, sz, vp]
        L.ts_soft_vote.argtypes = [pp, vp, f32, vp, vp, vp, vp, sz, vp]
        L.ts_soft_vote_ranked.argtypes = [pp, vp, f32, vp, vp, vp, vp, sz, vp]
        L.ts_topk.argtypes = [pp, vp, i32, vp, vp, vp, i32, vp, sz, vp]
        L.ts_topk_noalloc.argtypes = [pp, vp, i32, vp, vp, vp, i32, vp]
        L.ts_paged_qk_codes.argtypes = [pp, vp, vp, f32, vp, vp, sz, vp]
        L.ts_soft_vote_bounds.argtypes = [pp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
        L.ts_topk_exact.argtypes = [pp, vp, vp, vp, f32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.ts_selcache_check.argtypes = [pp, vp, vp, vp, f32, vp, vp]
        L.ts_paged_qk_scores_checked.argtypes = [pp, vp, ctypes.POINTER(_CSelcache), vp, f32, vp, sz, vp]
        L.ts_paged_qk_codes_checked.argtypes = [pp, vp, ctypes.POINTER(_CSelcache), vp, f32, vp, sz, vp]
        L.ts_sparse_paged_attn.argtypes = [pp, vp, vp, i32, vp, f32, vp, vp, vp, sz, vp]
        L.ts_chunk_row_stats.argtypes = [pp, vp, f32, vp, vp, sz, vp]
        L.ts_chunk_soft_vote.argtypes = [pp, vp, vp, f32, vp, vp, sz, vp]
        L.ts_chunk_mean_query.argtypes = [pp, vp, vp, vp]
        L.ts_sum_vote.argtypes = [pp, vp, vp, vp, vp]
        L.ts_head_vote_scratch_bytes.argtypes = [pp, ctypes.POINTER(sz)]
        L.ts_head_vote.argtypes = [pp, vp, i32, vp, vp, vp, sz, vp]
        L.ts_debug_set_score_variant.argtypes = [i32, i32, i32]
        L.ts_debug_set_topk_path.argtypes = [i32]
        L.ts_debug_set_codes_path.argtypes = [i32, i32]
        L.ts_debug_event_create.argtypes = [ctypes.POINTER(vp)]
        L.ts_debug_event_destroy.argtypes = [vp]
        L.ts_debug_event_elapsed_ms.argtypes = [vp, vp, ctypes.POINTER(f32)]
        L.ts_debug_set_score_timing_events.argtypes = [vp, vp]
        for name in ("ts_workspace_bytes", "ts_workspace_init", "ts_paged_qk_scores", "ts_soft_vote", "ts_topk",
                     "ts_selcache_check", "ts_sparse_paged_attn", "ts_debug_set_score_variant", "ts_chunk_row_stats",
                     "ts_chunk_soft_vote", "ts_chunk_mean_query", "ts_sum_vote", "ts_head_vote_scratch_bytes",
                     "ts_head_vote", "ts_debug_set_topk_path", "ts_debug_event_create", "ts_debug_event_destroy",
                     "ts_debug_event_elapsed_ms", "ts_debug_set_score_timing_events", "ts_paged_qk_codes",
                     "ts_soft_vote_bounds", "ts_topk_exact", "ts_debug_set_codes_path", "ts_topk_noalloc",
                     "ts_paged_qk_scores_checked", "ts_paged_qk_codes_checked", "ts_soft_vote_ranked"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def _ok(status: int, where: str) -> None:
    if status != 0:
        raise TokenSelectError(status, where)


class Problem:
    """ts_problem plus references that keep the tensors it points at alive."""

    def __init__(self, *, batch, chunk=1, num_q_heads, num_kv_heads, head_dim, page_size, max_seq_len, dtype,
                 k_pool, v_pool, page_indptr, page_indices, seq_lens, num_initial=0, num_local=0):
        self._keep = (k_pool, v_pool, page_indptr, page_indices, seq_lens)
        self.c = _CProblem(batch, chunk, num_q_heads, num_kv_heads, head_dim, page_size, max_seq_len, dtype,
                           _ptr(k_pool), _ptr(v_pool), _ptr(page_indptr), _ptr(page_indices), _ptr(seq_lens),
                           int(num_initial), int(num_local))

    def ref(self):
        return ctypes.byref(self.c)


def ts_version() -> int:
    return int(load().ts_version())


def ts_strerror(status: int) -> str:
    return load().ts_strerror(int(status)).decode()


def ts_workspace_bytes(p: Problem, k: int) -> int:
    out = ctypes.c_size_t(0)
    _ok(load().ts_workspace_bytes(p.ref(), int(k), ctypes.byref(out)), "ts_workspace_bytes")
    return int(out.value)


def ts_workspace_init(ws, stream=None) -> None:
    _ok(load().ts_workspace_init(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "ts_workspace_init")


def ts_debug_set_score_variant(variant: int, wg: int = 0, run_tiles: int = 0) -> None:
    _ok(load().ts_debug_set_score_variant(int(variant), int(wg), int(run_tiles)), "ts_debug_set_score_variant")


def ts_debug_set_codes_path(mfma: int, run_tiles: int = 0) -> None:
    _ok(load().ts_debug_set_codes_path(int(mfma), int(run_tiles)), "ts_debug_set_codes_path")


def ts_debug_set_topk_path(five_pass: int) -> None:
    _ok(load().ts_debug_set_topk_path(int(five_pass)), "ts_debug_set_topk_path")


def ts_debug_event_create() -> int:
    ev = ctypes.c_void_p(0)
    _ok(load().ts_debug_event_create(ctypes.byref(ev)), "ts_debug_event_create")
    return int(ev.value)


def ts_debug_event_destroy(ev: int) -> None:
    _ok(load().ts_debug_event_destroy(ctypes.c_void_p(ev)), "ts_debug_event_destroy")


def ts_debug_event_elapsed_ms(start: int, stop: int) -> float:
    ms = ctypes.c_float(0.0)
    _ok(load().ts_debug_event_elapsed_ms(ctypes.c_void_p(start), ctypes.c_void_p(stop), ctypes.byref(ms)),
        "ts_debug_event_elapsed_ms")
    return float(ms.value)


def ts_debug_set_score_timing_events(start, stop) -> None:
    _ok(load().ts_debug_set_score_timing_events(ctypes.c_void_p(start) if start else None,
                                                ctypes.c_void_p(stop) if stop else None),
        "ts_debug_set_score_timing_events")


def _nbytes(ws) -> int:
    return ws.numel() * ws.element_size() if ws is not None else 0


def ts_paged_qk_scores(p: Problem, q, scores, score_scale: float, skip, ws, stream=None) -> None:
    _ok(load().ts_paged_qk_scores(p.ref(), _ptr(q), _ptr(scores), float(score_scale), _ptr(skip), _ptr(ws), _nbytes(ws),
                                  _stream(stream)), "ts_paged_qk_scores")


def ts_soft_vote(p: Problem, scores, score_scale: float, row_stats, votes, skip, ws, stream=None) -> None:
    _ok(load().ts_soft_vote(p.ref(), _ptr(scores), float(score_scale), _ptr(row_stats), _ptr(votes), _ptr(skip),
                            _ptr(ws), _nbytes(ws), _stream(stream)), "ts_soft_vote")


def _selcache(cached_q, cached_q_next, first, first_next, reuse, theta) -> _CSelcache:
    return _CSelcache(_ptr(cached_q), _ptr(cached_q_next), _ptr(first), _ptr(first_next), _ptr(reuse), float(theta))


def ts_paged_qk_scores_checked(p: Problem, q, cached_q, cached_q_next, first, first_next, reuse, theta: float, scores,
                               score_scale: float, ws, stream=None) -> None:
    sc = _selcache(cached_q, cached_q_next, first, first_next, reuse, theta)
    _ok(load().ts_paged_qk_scores_checked(p.ref(), _ptr(q), ctypes.byref(sc), _ptr(scores), float(score_scale), _ptr(ws),
                                          _nbytes(ws), _stream(stream)), "ts_paged_qk_scores_checked")


def ts_paged_qk_codes_checked(p: Problem, q, cached_q, cached_q_next, first, first_next, reuse, theta: float, codes,
                              score_scale: float, ws, stream=None) -> None:
    sc = _selcache(cached_q, cached_q_next, first, first_next, reuse, theta)
    _ok(load().ts_paged_qk_codes_checked(p.ref(), _ptr(q), ctypes.byref(sc), _ptr(codes), float(score_scale), _ptr(ws),
                                         _nbytes(ws), _stream(stream)), "ts_paged_qk_codes_checked")


def ts_soft_vote_ranked(p: Problem, scores, score_scale: float, row_stats, votes, skip, ws, stream=None) -> None:
    _ok(load().ts_soft_vote_ranked(p.ref(), _ptr(scores), float(score_scale), _ptr(row_stats), _ptr(votes), _ptr(skip),
                                   _ptr(ws), _nbytes(ws), _stream(stream)), "ts_soft_vote_ranked")


def ts_paged_qk_codes(p: Problem, q, codes, score_scale: float, skip, ws, stream=None) -> None:
    _ok(load().ts_paged_qk_codes(p.ref(), _ptr(q), _ptr(codes), float(score_scale), _ptr(skip), _ptr(ws), _nbytes(ws),
                                 _stream(stream)), "ts_paged_qk_codes")


def ts_soft_vote_bounds(p: Problem, codes, score_scale: float, row_stats, vote_hi, vote_lo, skip, ws, stream=None) -> None:
    _ok(load().ts_soft_vote_bounds(p.ref(), _ptr(codes), float(score_scale), _ptr(row_stats), _ptr(vote_hi),
                                   _ptr(vote_lo), _ptr(skip), _ptr(ws), _nbytes(ws), _stream(stream)),
        "ts_soft_vote_bounds")


def ts_topk_exact(p: Problem, q, vote_hi, row_stats, score_scale: float, k: int, idx, count, skip, ws, stream=None,
                  sel_votes=None) -> None:
    _ok(load().ts_topk_exact(p.ref(), _ptr(q), _ptr(vote_hi), _ptr(row_stats), float(score_scale), int(k), _ptr(idx),
                             _ptr(count), _ptr(sel_votes), _ptr(skip), _ptr(ws), _nbytes(ws), _stream(stream)), "ts_topk_exact")


def ts_chunk_row_stats(p: Problem, q, score_scale: float, row_stats, ws, stream=None) -> None:
    _ok(load().ts_chunk_row_stats(p.ref(), _ptr(q), float(score_scale), _ptr(row_stats), _ptr(ws), _nbytes(ws),
                                  _stream(stream)), "ts_chunk_row_stats")


def ts_chunk_soft_vote(p: Problem, q, row_stats, score_scale: float, votes, ws, stream=None) -> None:
    _ok(load().ts_chunk_soft_vote(p.ref(), _ptr(q), _ptr(row_stats), float(score_scale), _ptr(votes), _ptr(ws),
                                  _nbytes(ws), _stream(stream)), "ts_chunk_soft_vote")


def ts_sum_vote(p: Problem, scores, votes, skip, stream=None) -> None:
    _ok(load().ts_sum_vote(p.ref(), _ptr(scores), _ptr(votes), _ptr(skip), _stream(stream)), "ts_sum_vote")


def ts_head_vote_scratch_bytes(p: Problem) -> int:
    out = ctypes.c_size_t(0)
    _ok(load().ts_head_vote_scratch_bytes(p.ref(), ctypes.byref(out)), "ts_head_vote_scratch_bytes")
    return int(out.value)


def ts_head_vote(p: Problem, scores, k_head: int, votes, skip, scratch, stream=None) -> None:
    _ok(load().ts_head_vote(p.ref(), _ptr(scores), int(k_head), _ptr(votes), _ptr(skip), _ptr(scratch), _nbytes(scratch),
                            _stream(stream)), "ts_head_vote")


def ts_chunk_mean_query(p: Problem, q, q_mean, stream=None) -> None:
    _ok(load().ts_chunk_mean_query(p.ref(), _ptr(q), _ptr(q_mean), _stream(stream)), "ts_chunk_mean_query")


def ts_topk(p: Problem, votes, k: int, idx, count, skip, ws, stream=None, flags: int = 0) -> None:
    _ok(load().ts_topk(p.ref(), _ptr(votes), int(k), _ptr(idx), _ptr(count), _ptr(skip), int(flags), _ptr(ws), _nbytes(ws),
                       _stream(stream)), "ts_topk")


def ts_topk_noalloc(p: Problem, votes, k: int, idx, count, skip, stream=None, flags: int = 0) -> None:
    _ok(load().ts_topk_noalloc(p.ref(), _ptr(votes), int(k), _ptr(idx), _ptr(count), _ptr(skip), int(flags),
                               _stream(stream)), "ts_topk_noalloc")


def ts_selcache_check(p: Problem, q, cached_q, first, theta: float, reuse, stream=None) -> None:
    _ok(load().ts_selcache_check(p.ref(), _ptr(q), _ptr(cached_q), _ptr(first), float(theta), _ptr(reuse),
                                 _stream(stream)), "ts_selcache_check")


def ts_sparse_paged_attn(p: Problem, q, idx, idx_stride: int, count, sm_scale: float, out, lse, ws,
                         stream=None) -> None:
    _ok(load().ts_sparse_paged_attn(p.ref(), _ptr(q), _ptr(idx), int(idx_stride), _ptr(count), float(sm_scale),
                                    _ptr(out), _ptr(lse), _ptr(ws),
                                    ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
        "ts_sparse_paged_attn")
