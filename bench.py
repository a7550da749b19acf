#!/usr/bin/env python3
"""Benchmark of the TokenSelect decode hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input already resident in HBM:
Selection Cache check (Alg. 1) -> paged q.k score pass (Alg. 2) -> head soft vote (Eq. 5) -> top-k
-> sparse paged attention (Eq. 2).  Default workload: configuration 4, the largest single-GPU one
(Qwen2-7B-shaped layer, bf16, 1048576 cached tokens in 16-token pages, k = 4096); configuration 2
(Llama-3-8B-shaped layer, 131072 tokens, k = 2048), the other end of the 128K-1M range, is run after it with
the same protocol and reported as `secondary`.  The selection runs in its compact form by default (no fp32
score matrix in memory; --path dense times the five-call form), with Algorithm 1's test taken inside the score
launch (--check call: as the ts_selcache_check call of its own; the default for configuration 3).  To keep neither the L2s nor the 256 MB
last-level cache warm, the steps rotate over R physical copies of the pool (same logical sequence,
different random page permutation each) and over R different queries, so that every step is a
Selection Cache miss (cosine of independent queries ~ 0 < theta = 0.9) and scans all cached tokens.

Prints ONE JSON line: metric, value (tokens scanned per second over whole steps), ms_per_step, the score
kernel's roofline (achieved GB/s from HIP events bound to its dispatch, on at least 32 steps run right after the
timed region), and the CPU oracle timed on the same workload.  Beside it, informational: the same steps replayed as a
HIP graph (`hip_graph_replay`) and with two independent steps in flight on two streams (`two_steps_in_flight`).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the score kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for plain copy kernels of known size in the same run (FETCH_SIZE x 1.966 / 1.982, WRITE_SIZE x 1.00:
# profiles/decode_step_cfg4_hbm_traffic.md, profiles/decode_step_cfg2_hbm_traffic.md)
MEASURED_TRAFFIC_BYTES = {(4, "compact"): int((512.30 * 1.966 + 31.73 * 1.00) * 2**20),
                          (2, "compact"): int((128.26 * 1.982 + 4.63 * 1.00) * 2**20),
                          (4, "dense"): int((512.26 * 1.966 + 112.38 * 1.00) * 2**20),
                          (2, "dense"): int((128.21 * 1.982 + 16.13 * 1.00) * 2**20)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 5],
                    help="4 (default) is the headline workload, the largest single-GPU configuration (1 Mi tokens), with "
                         "configuration 2 (131072 tokens) carried as `secondary`; 3 is the Selection Cache decode run; 5 is chunked prefill")
    ap.add_argument("--path", choices=["compact", "dense"], default=None,
                    help="compact (default for configurations 1, 2, 4): selection without the score matrix in memory "
                         "(ts_paged_qk_codes + ts_soft_vote_bounds + ts_topk_exact); dense (default for configuration 3, a batch "
                         "of short sequences, where it is the faster form): the five calls with the fp32 score matrix")
    ap.add_argument("--no-secondary", action="store_true", help="config 4: do not run configuration 2 as well")
    ap.add_argument("--pools", type=int, default=0, help="physical pool copies to rotate over (0 = enough for >= 2 GiB)")
    ap.add_argument("--variant", type=int, default=-1, help="score pass of the five-call form: 0 fma, 1 bf16 dot2, 2 matrix cores, -1 library default (2)")
    ap.add_argument("--score-wg", type=int, default=0)
    ap.add_argument("--run-tiles", type=int, default=0, help="tiles per run of the matrix-core score kernel (tuning; 0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tokens", type=int, default=0, help="override the number of cached tokens (profiling only)")
    ap.add_argument("--theta", type=float, default=0.9, help="Selection Cache threshold of the config-3 run")
    ap.add_argument("--theta-sweep", action="store_true",
                    help="config 3: also run the thresholds of the paper's theta study (0.5 ... 1.0) and report reuse rate and steps/s for each")
    ap.add_argument("--no-graph", action="store_true", help="time the host-driven single-stream loop only (no HIP-graph replay, no two-steps-in-flight run)")
    ap.add_argument("--page-size", type=int, default=16, help="tokens per page (16 in the configurations; 1 is the paper's own setting)")
    ap.add_argument("--selection", choices=["soft", "sum", "head"], default="soft",
                    help="selection function: soft = Eq. 5 (the method, default), sum = Eq. 3, head = Eq. 4 (ablation baselines)")
    ap.add_argument("--vote", choices=["ranked", "plain"], default="ranked",
                    help="five-call form: ts_soft_vote_ranked + ts_topk(TS_TOPK_VOTE_HIST) (one launch less) or ts_soft_vote + ts_topk")
    ap.add_argument("--check", choices=["fused", "call"], default=None,
                    help="Selection Cache test: inside the score launch (fused) or as the ts_selcache_check call before it "
                         "(default: fused, except for the batch of config 3, where the call is the faster form)")
    ap.add_argument("--n-init", type=int, default=0, help="forced initial tokens (the paper's runs use 128); default 0 as in the configurations")
    ap.add_argument("--n-local", type=int, default=0, help="forced most recent tokens (the paper's runs use 512); default 0")
    args = ap.parse_args()
    if args.check is None:
        args.check = "call" if args.config == 3 else "fused"
    return args


def cpu_baseline(w, budget_s=12.0, n_init=0, n_local=0):
    """The oracle as it stands, timed on this host for whole decode steps of the same workload."""
    import oracle
    N = int(w.seq_lens[0])
    qb = np.ascontiguousarray(w.q[0, 0])
    sm = float(np.float32(1.0 / math.sqrt(w.D)))
    times = []
    t_all = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        idx, cnt = oracle.select(qb, w.k_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), N, w.k, n_init=n_init, n_local=n_local)
        att = oracle.attended_tokens(idx, cnt, N, n_init, n_local)
        oracle.sparse_attn(qb, w.k_pool, w.v_pool, w.dtype, w.H_kv, w.P, w.pages_of(0), att, len(att), sm)
        times.append(time.perf_counter() - t0)
        if time.perf_counter() - t_all > budget_s or len(times) >= 150:
            break
    t = float(np.median(times))
    return {"value": N / t, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d full decode steps (selection + sparse attention) of the same workload, median %.3f s/step"
                      % (len(times), t),
            "steps_per_s": 1.0 / t}


def selection_cache_run(args):
    """Configuration 3: B = 8 sequences of 16384..65536 cached tokens, 64 consecutive decode steps with
    AR(1) queries, one K/V row appended per sequence per step, theta = 0.9.  Reports the reuse rate
    (Algorithm 1: C_Q is the query of the last reselect) and decode steps/s."""
    import torch
    import workloads as W
    import paper_2411_02886_amd as ts
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device, to_host
    dev = "cuda:0"
    w = W.config3()
    steps = int(w.extra["steps"])
    qs = [to_device(q, dev) for q in W.ar1_queries(w, steps, rho=0.95)]
    ks, vs = W.appended_kv(w, steps)
    ksd, vsd = to_device(ks, dev), to_device(vs, dev)
    layer = DecodeLayer.from_workload(w, device=dev, max_seq_len=int(w.seq_lens.max()) + steps,
                                      num_initial=args.n_init, num_local=args.n_local)
    slots = np.empty((steps, w.B), dtype=np.int64)
    for b in range(w.B):
        pos = int(w.seq_lens[b]) + np.arange(steps)
        slots[:, b] = w.pages_of(b).astype(np.int64)[pos // w.P] * w.P + pos % w.P
    slots_d = torch.from_numpy(slots).to(dev)
    # K and V pools as the two halves of one tensor, so that a step's new K/V rows go in with one launch
    kv = torch.stack([layer.k_pool, layer.v_pool])
    layer.swap_pool(kv[0], kv[1])
    kvflat = kv.view(2, -1, w.H_kv, w.D)
    kvsd = torch.stack([ksd, vsd], dim=1).contiguous()          # [steps][2][B][H_kv][D]
    del ksd, vsd
    # the lengths of every step are inputs of the run (a scheduler knows them): one ts_problem per step points at its row
    lens_all = (layer.seq_lens[None, :] + 1 + torch.arange(steps, device=dev, dtype=torch.int32)[:, None]).contiguous()
    problems = []
    for t in range(steps):
        layer.seq_lens = lens_all[t]; layer._make_problem(); problems.append(layer.problem)
    sm, theta, scale = 1.0 / math.sqrt(w.D), args.theta, 1.0
    compact = args.path == "compact"                           # default here: the five-call form
    reuse_log = torch.zeros((steps, w.B), dtype=torch.uint8, device=dev)

    def run(theta=theta):
        layer.first.fill_(1)
        for t in range(steps):
            kvflat.index_copy_(1, slots_d[t], kvsd[t])          # append this step's K/V rows
            layer.problem, layer.reuse = problems[t], reuse_log[t]   # the step's lengths; its reuse flags go straight to the log
            layer.step(qs[t], theta=theta, score_scale=scale, sm_scale=sm, compact=compact, fused_check=args.check == "fused", ranked_vote=args.vote == "ranked")

    run(); torch.cuda.synchronize()
    reps = max(1, args.steps // steps)
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    dt_eager = (time.perf_counter() - t0) / reps
    reuse_eager = to_host(reuse_log).copy(); idx_eager = to_host(layer.idx).copy(); out_eager = to_host(layer.out).copy()
    # The 64-step run is launch-bound on the host (11 launches per step), so it is also captured once as a HIP
    # graph (every hit/miss decision is taken on the device, nothing in it depends on the host) and replayed.
    dt, mode = dt_eager, "eager"
    if not args.no_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                run()                                            # warm-up on the capture stream
            torch.cuda.current_stream().wait_stream(side); torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                run()
            ok = True
            for _ in range(3):                                   # replays, eager work and synchronisations in between
                reuse_log.zero_(); layer.idx.fill_(-5); torch.cuda.synchronize()
                g.replay(); torch.cuda.synchronize()
                ok = ok and np.array_equal(to_host(reuse_log), reuse_eager) and np.array_equal(to_host(layer.idx), idx_eager) \
                    and np.array_equal(to_host(layer.out), out_eager)
            if ok:
                t0 = time.perf_counter()
                for _ in range(reps):
                    g.replay()
                torch.cuda.synchronize()
                dt, mode = (time.perf_counter() - t0) / reps, "graph"
            else:
                print("bench.py: graph replays did not reproduce the eager run; reporting the eager loop", file=sys.stderr)
        except Exception as e:                                   # capture not possible: the eager figure stands
            print("bench.py: graph capture failed (%s); reporting the eager loop" % e, file=sys.stderr)
    reuse = reuse_eager.astype(bool)
    lens = w.seq_lens.astype(np.int64)[None, :] + 1 + np.arange(steps)[:, None]
    scanned = int((lens * (~reuse)).sum())
    res = {"metric": "decode steps/s over the Selection Cache run (batch of 8 sequences per step)",
           "value": steps / dt, "unit": "batch-steps/s", "n_gpus": 1, "steps": steps * reps, "warmup": steps,
           "ms_per_step": dt * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": w.name, "batch": w.B, "cached_tokens": [int(x) for x in w.seq_lens], "k": w.k,
                      "theta": theta, "score_scale": scale, "query_process": "AR(1) rho=0.95", "steps_per_run": steps,
                      "anchor": "query of the last reselect (Algorithm 1)",
                      "forced_initial_tokens": args.n_init, "forced_recent_tokens": args.n_local},
           "reuse_rate": float(reuse.mean()), "sequence_steps_per_s": steps * w.B / dt,
           "tokens_scanned_per_s": scanned / dt,
           "execution": mode, "eager_batch_steps_per_s": steps / dt_eager,
           "selection_form": "compact (no score matrix in memory)" if compact else "five calls (fp32 score matrix)",
           "selection_cache_check": "inside the score launch" if args.check == "fused" else "ts_selcache_check before the score launch",
           "note": ("%d library launches + 1 torch launch (the append of the step's K/V rows) per step; " %
                    ((8 if compact else (8 if args.vote == "ranked" else 9)) - (1 if args.check == "fused" else 0))) +
                   "'graph' = the whole 64-step run captured once as a HIP graph "
                   "and replayed (replays checked against the eager run), 'eager' = host-driven loop"}
    if args.theta_sweep:
        sweep = []
        for th in (0.5, 0.6, 0.7, 0.8, 0.85, 0.9, 0.95, 1.0):       # the thresholds of the paper's theta study
            run(th); torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(th); torch.cuda.synchronize()
            d = time.perf_counter() - t0
            sweep.append({"theta": th, "reuse_rate": float(to_host(reuse_log).astype(bool).mean()),
                          "batch_steps_per_s": steps / d})
        res["theta_sweep"] = sweep
    print(json.dumps(res))


def chunked_prefill_run(args):
    """Configuration 5: one chunked-prefill step = two MFMA score sweeps (row log-sum-exps, votes summed over
    heads and over the chunk's 512 queries), shared top-k of 4096, chunk-form sparse attention."""
    import torch
    import workloads as W
    import paper_2411_02886_amd as ts
    from paper_2411_02886_amd.runtime import ChunkSelector, to_device
    w = W.config5()
    N = int(w.extra["n_cached"])
    sel = ChunkSelector.from_workload(w, num_initial=args.n_init, num_local=args.n_local)
    q = to_device(w.q)
    names = ["row_stats", "soft_vote", "topk", "attention"]
    calls = [lambda: ts.ts_chunk_row_stats(sel.problem, q, 1.0, sel.row_stats, sel.ws),
             lambda: ts.ts_chunk_soft_vote(sel.problem, q, sel.row_stats, 1.0, sel.votes, sel.ws),
             lambda: ts.ts_topk(sel.problem, sel.votes, sel.k, sel.idx, sel.count, None, sel.ws),
             lambda: sel.attend(q)]
    steps = max(1, min(args.steps, 50)); warm = max(1, min(args.warmup, 5))
    for _ in range(warm):
        for f in calls:
            f()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(steps)]
    t0 = time.perf_counter()
    for s in range(steps):
        ev[s][0].record()
        for i, f in enumerate(calls):
            f(); ev[s][i + 1].record()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    per = np.array([[ev[s][i].elapsed_time(ev[s][i + 1]) for i in range(len(calls))] for s in range(steps)]).mean(axis=0)
    flop = 2.0 * w.C * w.H * w.D * N                                     # one sweep of Q K^T
    peak = 2500.0
    tf = flop / (per[1] * 1e-3) / 1e12
    res = {"metric": "query-token pairs/s of one chunked-prefill step (2 score sweeps + top-k + chunk attention)",
           "value": w.C * N / dt, "unit": "pairs/s", "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": dt * 1e3,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": w.name, "chunk": w.C, "cached_tokens": N, "num_q_heads": w.H, "num_kv_heads": w.H_kv,
                      "head_dim": w.D, "k": w.k, "score_scale": 1.0,
                      "forced_initial_tokens": args.n_init, "forced_recent_tokens": args.n_local},
           "ms_per_call": dict(zip(names, [float(x) for x in per])),
           "roofline": {"bound": "mfma", "kernel": "ts::prefill_qk_kernel<128, 2> (vote sweep of ts_chunk_soft_vote)",
                        "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak, "traffic": None,
                        "flop_per_launch": flop, "exp_per_launch": float(w.C) * w.H * N,
                        "stats_sweep_tflops": flop / (per[0] * 1e-3) / 1e12}}
    # Sec. 5.2 as printed for comparison: one selection per chunk with the mean query (decode path, HBM-bound)
    idx_pq = set(sel.idx[0, : int(sel.count[0])].tolist())
    for _ in range(warm):
        sel.select_mean_query(q, 1.0)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        sel.select_mean_query(q, 1.0)
    b.record(); torch.cuda.synchronize()
    idx_mq = set(sel.idx[0, : int(sel.count[0])].tolist())
    planted = set(np.concatenate(list(w.planted[0])).tolist()) if len(w.planted) else set()
    res["mean_query_selection"] = {
        "ms": a.elapsed_time(b) / steps, "per_query_selection_ms": float(per[0] + per[1] + per[2]),
        "index_overlap_with_per_query_votes": len(idx_pq & idx_mq) / max(1, len(idx_pq)),
        "planted_among_selected": {"per_query_votes": len(idx_pq & planted) / max(1, len(idx_pq)),
                                   "mean_query": len(idx_mq & planted) / max(1, len(idx_mq))},
        "note": "mean of the chunk's 512 queries fed to the decode selection (ts_chunk_mean_query + score pass + vote + top-k)"}
    print(json.dumps(res))


def decode_bench(cfg, args, *, steps, warmup, with_cpu_baseline, with_graph, with_overlap=None):
    """One decode configuration (1, 2 or 4): whole steps in the timed region, then a separate sampled loop that
    times the score kernel alone with HIP events bound to its dispatch."""
    import torch
    import workloads as W
    import paper_2411_02886_amd as ts
    from paper_2411_02886_amd.runtime import DecodeLayer, to_device, to_host

    dev = "cuda:0"
    kw = {"N": args.tokens} if args.tokens else {}
    if args.page_size != 16:
        kw["P"] = args.page_size
    w = W.CONFIGS[cfg](**kw)
    N = int(w.seq_lens[0])
    if args.variant >= 0 or args.score_wg:
        ts.ts_debug_set_score_variant(args.variant if args.variant >= 0 else 2, args.score_wg)
    if args.run_tiles:
        ts.ts_debug_set_codes_path(1, args.run_tiles)
    compact = args.path != "dense" and args.selection == "soft"
    layer = DecodeLayer.from_workload(w, device=dev, num_initial=args.n_init, num_local=args.n_local)
    esize = w.esize()
    k_bytes = N * w.H_kv * w.D * esize                      # algorithmic bytes of the score pass
    gather_bytes = 2 * min(w.k + args.n_init + args.n_local, N) * w.H_kv * w.D * esize   # K and V rows of sparse attention
    pool_bytes = w.k_pool.nbytes + w.v_pool.nbytes
    R = args.pools if args.pools > 0 else max(2, int(math.ceil(2 * 2**30 / pool_bytes)))
    R = min(R, 8)

    # R physical copies of the same logical sequence, each under its own page permutation
    rng = np.random.Generator(np.random.PCG64(w.seed + 424242))
    pools = [(layer.k_pool, layer.v_pool, layer.page_indices)]
    pi0 = layer.page_indices.long()
    for r in range(1, R):
        perm = to_device(rng.permutation(w.num_pages)[: pi0.numel()].astype(np.int32), dev)
        kp = torch.empty_like(layer.k_pool); vp = torch.empty_like(layer.v_pool)
        kp.index_copy_(0, perm.long(), layer.k_pool.index_select(0, pi0))
        vp.index_copy_(0, perm.long(), layer.v_pool.index_select(0, pi0))
        pools.append((kp, vp, perm))
    qs = [to_device(w.q, dev)]
    for r in range(1, R):
        qs.append(to_device(W.store(rng.standard_normal(w.q.shape, dtype=np.float32), w.dtype), dev))
    torch.cuda.synchronize()

    sm = 1.0 / math.sqrt(w.D)
    theta, scale = 0.9, 1.0
    problems = []
    for kp, vp, pi in pools:
        layer.swap_pool(kp, vp, pi)
        problems.append(layer.problem)
    hv_scratch = None
    if args.selection == "head":
        nb = ts.ts_head_vote_scratch_bytes(layer.problem)
        hv_scratch = torch.empty((nb + 255) // 256 * 64, dtype=torch.int32, device=dev)
    if compact:
        layer.codes = torch.empty((w.B, layer.max_seq_len, w.H), dtype=torch.uint8, device=dev)
        layer.vote_hi = torch.empty((w.B, layer.max_seq_len), dtype=torch.float32, device=dev)
        layer.vote_lo = torch.empty((w.B, layer.max_seq_len), dtype=torch.float32, device=dev)

    fused_check = args.check == "fused"       # Algorithm 1's test inside the score launch (one launch less)
    ranked_vote = args.vote == "ranked"       # five-call form: the TopK's first histogram is built inside the vote launch

    def score_pass(p, q, stream, layer):
        if fused_check:
            st = (layer.cached_q, layer.cached_q_next, layer.first, layer.first_next, layer.reuse, theta)
            if compact:
                ts.ts_paged_qk_codes_checked(p, q, *st, layer.codes, scale, layer.ws, stream)
            else:
                ts.ts_paged_qk_scores_checked(p, q, *st, layer.scores, scale, layer.ws, stream)
            layer._swap_selcache_state()
        elif compact:
            ts.ts_paged_qk_codes(p, q, layer.codes, scale, layer.reuse, layer.ws, stream)
        else:
            ts.ts_paged_qk_scores(p, q, layer.scores, scale, layer.reuse, layer.ws, stream)

    def step(i, ev=None, kev=None, layer=layer, problems=problems, stream=None):
        p = problems[i % R]
        q = qs[i % R]
        if stream is None:
            stream = torch.cuda.current_stream()  # the capture stream while a graph is being recorded
        if not fused_check:
            ts.ts_selcache_check(p, q, layer.cached_q, layer.first, theta, layer.reuse, stream)
        if ev is not None:
            ev[0].record(stream)
        if kev is not None:          # HIP events bound to the score kernel's own start and end
            ts.ts_debug_set_score_timing_events(kev[0], kev[1])
        score_pass(p, q, stream, layer)
        if kev is not None:
            ts.ts_debug_set_score_timing_events(None, None)
        if compact:
            ts.ts_soft_vote_bounds(p, layer.codes, scale, layer.row_stats, layer.vote_hi, None, layer.reuse, layer.ws, stream)
            ts.ts_topk_exact(p, q, layer.vote_hi, layer.row_stats, scale, layer.k, layer.idx, layer.count, layer.reuse, layer.ws, stream)
        else:
            if args.selection == "soft" and ranked_vote:
                ts.ts_soft_vote_ranked(p, layer.scores, scale, layer.row_stats, layer.votes, layer.reuse, layer.ws, stream)
            elif args.selection == "soft":
                ts.ts_soft_vote(p, layer.scores, scale, layer.row_stats, layer.votes, layer.reuse, layer.ws, stream)
            elif args.selection == "sum":
                ts.ts_sum_vote(p, layer.scores, layer.votes, layer.reuse, stream)
            else:
                ts.ts_head_vote(p, layer.scores, layer.k, layer.votes, layer.reuse, hv_scratch, stream)
            ts.ts_topk(p, layer.votes, layer.k, layer.idx, layer.count, layer.reuse, layer.ws, stream,
                       flags=ts.TS_TOPK_VOTE_HIST if (args.selection == "soft" and ranked_vote) else 0)
        if ev is not None:
            ev[1].record(stream)
        ts.ts_sparse_paged_attn(p, q, layer.idx, layer.k, layer.count, sm, layer.out, layer.lse, layer.ws, stream)

    # sanity before timing: paging invariance across the pool copies (same query -> same selection), and the
    # compact form against the five-call form on the workload's own query
    ref_idx = None
    for r in range(min(R, 2)):
        kp, vp, pi = pools[r]
        layer.swap_pool(kp, vp, pi)
        layer.first.fill_(1)
        if compact:
            layer.select_compact(qs[0], scale, None)
        else:
            layer.select(qs[0], scale, None, kind=args.selection)
        torch.cuda.synchronize()
        got = to_host(layer.idx).copy()
        if ref_idx is None:
            ref_idx = got
        assert np.array_equal(got, ref_idx), "selection changed with the physical page layout"
    dense_agrees = None
    if compact:
        layer.select(qs[0], scale, None, kind="soft")
        torch.cuda.synchronize()
        dense_idx = to_host(layer.idx).copy()
        dense_agrees = float(np.intersect1d(dense_idx[0], ref_idx[0]).size) / max(1, int((ref_idx[0] >= 0).sum()))
    layer.first.fill_(1)
    planted = set(np.concatenate(list(w.planted[0])).tolist()) if len(w.planted) and w.planted[0].size else set()
    sel_set = set(ref_idx[0][ref_idx[0] >= 0].tolist())
    quality = {"planted_tokens": len(planted), "selected": len(sel_set),
               "precision": len(sel_set & planted) / max(1, len(sel_set)),
               "recall": len(sel_set & planted) / max(1, len(planted))}

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # ---- the timed region: `steps` whole steps, nothing else on the stream
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    misses = int((to_host(layer.reuse) == 0).sum())
    assert misses == w.B, "the benchmark step must be a Selection Cache miss"
    ms_step = (t1 - t0) * 1e3 / steps

    # ---- after it: the same steps again, every one carrying HIP events bound to the score kernel's dispatch (its own
    # start and end) and stream-ordered events around the selection; at least 32 launches whatever --steps is
    nsample = max(32, min(steps, 64))
    events = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(2)) for _ in range(nsample)]
    kevents = [(ts.ts_debug_event_create(), ts.ts_debug_event_create()) for _ in range(nsample)]
    for i in range(nsample):
        step(warmup + steps + i, events[i], kevents[i])
    torch.cuda.synchronize()
    select_ms = np.array([e[0].elapsed_time(e[1]) for e in events], dtype=np.float64)
    score_ms = np.array([ts.ts_debug_event_elapsed_ms(a, b) for a, b in kevents], dtype=np.float64)
    for a, b in kevents:
        ts.ts_debug_event_destroy(a); ts.ts_debug_event_destroy(b)
    score_avg_ms = float(score_ms.mean())
    achieved = k_bytes / (score_avg_ms * 1e-3) / 1e9

    # Two independent steps in flight: a second layer state (own workspace, score / code / vote buffers, Selection
    # Cache state; same pools) takes every other step on a second stream, as two micro-batches of a server would.
    # The small latency-bound launches of one step then run beside the other step's score pass.  Informational:
    # `value` stays the single-stream loop above, where a step's launches depend on each other.
    overlap_info = None
    if (with_graph if with_overlap is None else with_overlap) and args.selection == "soft":
        try:
            layer_b = DecodeLayer(dtype=w.dtype, H=w.H, H_kv=w.H_kv, D=w.D, P=w.P, k=w.k, k_pool=layer.k_pool,
                                  v_pool=layer.v_pool, page_indptr=w.page_indptr, page_indices=w.page_indices,
                                  seq_lens=w.seq_lens, device=dev, num_initial=args.n_init, num_local=args.n_local)
            if compact:
                layer_b.codes = torch.empty_like(layer.codes); layer_b.vote_hi = torch.empty_like(layer.vote_hi)
                layer_b.vote_lo = torch.empty_like(layer.vote_lo)
            problems_b = []
            for kp, vp, pi in pools:
                layer_b.swap_pool(kp, vp, pi)
                problems_b.append(layer_b.problem)
            # what each layer must hold after its last step, from the single-stream path
            n2 = max(8, steps // 2)
            want = []
            for j in (n2 - 1, n2):
                step(j); torch.cuda.synchronize(); want.append(to_host(layer.idx).copy())
            layer.first.fill_(1)
            sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
            for timed in (False, True):
                torch.cuda.synchronize()
                sa.wait_stream(torch.cuda.current_stream()); sb.wait_stream(torch.cuda.current_stream())
                tt = time.perf_counter()
                for i in range(n2):
                    step(i, layer=layer, problems=problems, stream=sa)
                    step(i + 1, layer=layer_b, problems=problems_b, stream=sb)      # one query on: every step a miss
                torch.cuda.synchronize()
                tt = time.perf_counter() - tt
            ok = (np.array_equal(to_host(layer.idx), want[0]) and np.array_equal(to_host(layer_b.idx), want[1])
                  and int((to_host(layer.reuse) == 0).sum()) == w.B and int((to_host(layer_b.reuse) == 0).sum()) == w.B)
            overlap_info = {"what": "two layer states on two streams, each running whole steps back to back",
                            "ms_per_step": tt * 1e3 / (2 * n2), "steps": 2 * n2, "selections_match_single_stream": bool(ok),
                            "whole_step_roofline_frac": (k_bytes + gather_bytes) / (tt / (2 * n2)) / 1e9 / HBM_PEAK_GBS}
            del layer_b, problems_b
        except Exception as e:
            overlap_info = {"error": str(e)[:200]}
        layer.first.fill_(1)

    # The same steps as one HIP graph (R consecutive steps, one per pool copy), replayed: what the step costs
    # without the host in the loop.  Informational; `value` is the host-driven loop above.
    graph_info = None
    RG = 2 * R if (fused_check and R % 2) else R      # an even number of steps: the fused check alternates two state buffers
    if with_graph:
        try:
            idx_ref = []
            for i in range(RG):
                step(i); torch.cuda.synchronize(); idx_ref.append(to_host(layer.idx).copy())
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            idx_log = torch.zeros((RG,) + tuple(layer.idx.shape), dtype=torch.int32, device=dev)

            def steps_r():
                for i in range(RG):
                    step(i); idx_log[i].copy_(layer.idx)
            with torch.cuda.stream(side):
                steps_r()
            torch.cuda.current_stream().wait_stream(side); torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                steps_r()
            ok = True
            for _ in range(3):
                idx_log.fill_(-3); layer.idx.fill_(-3); torch.cuda.synchronize()
                g.replay(); torch.cuda.synchronize()
                ok = ok and all(np.array_equal(to_host(idx_log[i]), idx_ref[i]) for i in range(RG))
            nrep = max(1, steps // RG)
            tg = time.perf_counter()
            for _ in range(nrep):
                g.replay()
            torch.cuda.synchronize()
            graph_info = {"ms_per_step": (time.perf_counter() - tg) * 1e3 / (nrep * RG), "steps": nrep * RG,
                          "replays_match_eager": bool(ok)}
        except Exception as e:
            graph_info = {"error": str(e)[:200]}

    kernel_name = ("ts::score_codes_mfma_kernel (the one launch of ts_paged_qk_codes%s)" if compact else
                   "the one launch of ts_paged_qk_scores%s (ts::score_codes_mfma_kernel<.., DENSE> for bf16 with 3..8 query heads per KV head, else ts::score_decode_kernel)") % ("_checked, Selection Cache test included" if fused_check else "")
    traffic = MEASURED_TRAFFIC_BYTES.get((cfg, "compact" if compact else "dense")) if not args.tokens and args.page_size == 16 else None
    res = {
        "ms_per_step": ms_step,
        "tokens_scanned_per_s": N / (ms_step * 1e-3),
        "decode_steps_per_s": 1e3 / ms_step,
        "dtype": "bf16" if w.dtype == W.BF16 else "f32",
        "config": {"workload": w.name, "batch": w.B, "cached_tokens": N, "num_q_heads": w.H, "num_kv_heads": w.H_kv,
                   "head_dim": w.D, "page_size": w.P, "k": w.k, "score_scale": scale, "theta": theta,
                   "pool_copies_rotated": R, "selection_cache": "every step is a miss",
                   "forced_initial_tokens": args.n_init, "forced_recent_tokens": args.n_local,
                   "selection_function": {"soft": "Eq. 5 head soft vote", "sum": "Eq. 3 summed dot products",
                                          "head": "Eq. 4 head vote"}[args.selection],
                   "selection_form": ("compact: ts_paged_qk_codes + ts_soft_vote_bounds + ts_topk_exact (no score matrix in memory)"
                                      if compact else ("five calls: ts_paged_qk_scores + ts_soft_vote_ranked + ts_topk (fp32 score matrix; the TopK's first histogram built inside the vote launch)"
                                            if (ranked_vote and args.selection == "soft") else "five calls: ts_paged_qk_scores + ts_soft_vote + ts_topk (fp32 score matrix)"))},
        "launches_per_step": None if args.selection != "soft" else
        (8 if compact else (8 if ranked_vote else 9)) - (1 if fused_check else 0),
        "selection_cache_check": ("inside the score launch (ts_paged_qk_%s_checked)" % ("codes" if compact else "scores")) if fused_check else "ts_selcache_check before the score launch",
        "planted_token_quality": quality,
        "compact_vs_five_call_index_overlap": dense_agrees,
        "hip_graph_replay": graph_info,
        "two_steps_in_flight": overlap_info,
        "selection_ms": {"what": "score pass + vote + top-k (the selection of Eq. 5), stream-ordered events, %d steps after the timed region" % nsample,
                         "avg": float(select_ms.mean()), "median": float(np.median(select_ms)), "min": float(select_ms.min())},
        "whole_step_roofline": {"what": "(K bytes of the score pass + K/V rows gathered by sparse attention) / ms_per_step / 8 TB/s",
                                "algorithmic_bytes_per_step": k_bytes + gather_bytes,
                                "frac": (k_bytes + gather_bytes) / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "kernel": kernel_name,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "algorithmic_bytes_per_launch": k_bytes,
                     "avg_launch_ms": score_avg_ms, "median_launch_ms": float(np.median(score_ms)),
                     "min_launch_ms": float(score_ms.min()), "launches_timed": nsample,
                     "timing": "HIP events bound to the kernel's dispatch (start and end of the launch itself) on %d whole steps "
                               "run right after the timed region (a launch that carries such events costs the step a few "
                               "microseconds, so the timed region carries none)" % nsample,
                     "score_pass_tokens_per_s": N / (score_avg_ms * 1e-3)},
    }
    if with_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, n_init=args.n_init, n_local=args.n_local)
    del pools, problems, layer
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.config == 3:
        return selection_cache_run(args)
    if args.config == 5:
        return chunked_prefill_run(args)
    import torch
    import paper_2411_02886_amd as ts
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    ts.load()
    head = decode_bench(args.config, args, steps=args.steps, warmup=args.warmup,
                        with_cpu_baseline=not args.no_cpu_baseline, with_graph=not args.no_graph)
    res = {
        "metric": "KV tokens scanned/s (whole decode step: Selection Cache check + score pass + soft vote + top-k + sparse attention)",
        "value": head["tokens_scanned_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
    }
    for k in ("config", "decode_steps_per_s", "launches_per_step", "selection_cache_check", "planted_token_quality", "compact_vs_five_call_index_overlap",
              "hip_graph_replay", "two_steps_in_flight", "selection_ms", "whole_step_roofline", "roofline", "cpu_baseline"):
        if k in head:
            res[k] = head[k]
    # the other end of the 128K-1M range rides along (its own timed region, same protocol)
    if args.config == 4 and not args.no_secondary and not args.tokens:
        sec = decode_bench(2, args, steps=args.steps, warmup=args.warmup, with_cpu_baseline=False, with_graph=False,
                           with_overlap=not args.no_graph)
        res["secondary"] = {k: sec[k] for k in ("config", "ms_per_step", "tokens_scanned_per_s", "decode_steps_per_s",
                                                 "launches_per_step", "selection_ms", "whole_step_roofline", "roofline",
                                                 "two_steps_in_flight")}
        if args.path != "dense" and args.selection == "soft":
            # at 128K tokens the five-call form (fp32 score matrix in memory) is the faster step although its score
            # pass is the slower kernel: both on record
            import copy
            a2 = copy.copy(args); a2.path = "dense"
            d2 = decode_bench(2, a2, steps=args.steps, warmup=args.warmup, with_cpu_baseline=False, with_graph=False)
            res["secondary"]["five_call_form"] = {"ms_per_step": d2["ms_per_step"], "score_pass_frac": d2["roofline"]["frac"],
                                                  "score_pass_ms": d2["roofline"]["avg_launch_ms"]}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
