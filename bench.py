#!/usr/bin/env python3
"""Benchmark of the k-LPM scheduling step on one MI355X.

A step is one pass of the whole path over the waiting queue: prefix-match every waiting query
against the GPU-resident radix tree, pick the k-LPM batch, commit it (insert + LRU-evict to the KV
budget), retire the batch from the queue and enqueue the next arrivals.  The workload is the large
configuration (about 100M cached tokens, 65,536 waiting queries of up to 8,192 tokens, k = 8,
batch 1,024); inputs are synthetic, seeded and already resident in HBM when timing starts.

Prints one JSON line: prefix-match tokens/s over the timed steps, plus the roofline figures of the
match kernel (algorithmic bytes / measured kernel time, against the 8 TB/s HBM peak) and the CPU
oracle timed on the host cores over a bounded sample of the same steps.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TIE_SEED = 2502046770


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(sum_match: int, n_queries: int) -> int:
    """Bytes the match kernel has to move for one launch: for every compared position (the matched
    tokens and the first mismatch) 4 B of query token and 4 B of edge token, plus per query its
    offset (8 B), length (4 B) and the 4 B result.  Child-table slots are left out (lower bound)."""
    return 8 * (sum_match + n_queries) + 16 * n_queries


def recorded_traffic():
    """HBM bytes per match launch from the committed rocprofv3 counter summary, or None when the
    kernel sources have changed since those counters were taken (or the summary is missing)."""
    import hashlib

    path = os.path.join(ROOT, "profiles", "k_match_cfg2-large_hbm_counters.txt")
    try:
        fields = dict(line.strip().split("=", 1) for line in open(path) if "=" in line and not line.startswith(" "))
        h = hashlib.sha256()
        for rel in ("paper_2502_04677_amd/csrc/match.hip", "paper_2502_04677_amd/csrc/klpm_device.hpp"):
            h.update(open(os.path.join(ROOT, rel), "rb").read())
        if fields.get("kernel_source_sha256") != h.hexdigest():
            return None
        return float(fields["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def build_workload(scale: float, steps_total: int, deep: bool = False):
    import workloads as W

    t0 = time.time()
    gen = W.config2_deep if deep else W.config2
    batch = max(4, int(round(1024 * scale)))
    w = gen(scale=scale, extra_queries=steps_total * batch)
    assert w.batch == batch
    log(f"generated {w.name} scale={scale}: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, "
        f"queue {w.queries.n}, later arrivals {w.extra.n} in {time.time() - t0:.1f}s")
    return w, W.concat_prompts(w.queries, w.extra)


def cpu_baseline(w, allq, steps: int, threads: int, rate_bits: int = 0, random_ties: bool = False,
                 dynamic: bool = False):
    """The oracle run over the first `steps` steps of the same workload (match on `threads` host
    threads, select and commit serial), timed without the tree build."""
    import oracle

    tree = oracle.OracleTree()
    tree.build(w.cache)
    n0, batch = w.queries.n, w.batch
    waiting = np.arange(n0, dtype=np.int64)
    enq = np.zeros(allq.n, dtype=np.uint64)
    enq[:n0] = w.queries.arrival
    clock, phase, matched = 0, 0, 0
    step_sums = []
    t_match = 0.0
    t0 = time.perf_counter()
    for s in range(steps):
        off, ln, arr = allq.off[waiting], allq.len[waiting], enq[waiting]
        ta = time.perf_counter()
        m = tree.match(allq.tokens, off, ln, threads=threads)
        t_match += time.perf_counter() - ta
        sc = oracle.score_hit_rate(m, ln, rate_bits) if rate_bits else m
        tk = oracle.tie_keys(TIE_SEED, s, waiting) if random_ties else None
        if dynamic:
            idx, phase, _ = oracle.select_dynamic(allq.tokens, off, ln, arr, m, w.k, batch, phase)
        else:
            idx, phase = oracle.select(arr, sc, w.k, batch, phase, tie_key=tk)
        tree.commit(allq.tokens, off, ln, idx, w.budget)
        clock += max(1, int((ln[idx].astype(np.int64) - m[idx]).sum()))
        keep = np.ones(waiting.shape[0], dtype=bool)
        keep[idx] = False
        new = np.arange(n0 + s * batch, n0 + (s + 1) * batch, dtype=np.int64)
        enq[new] = clock
        waiting = np.concatenate([waiting[keep], new])
        matched += int(m.sum())
        step_sums.append(int(m.sum()))
    dt = time.perf_counter() - t0
    return matched / dt, dt, t_match, step_sums


def bench_def3(args) -> int:
    """Second workload: a Regular Arrival Shuffled Queue (Def. 3) at the shape of the paper's table on
    varying the prefix-length ratio (n = 2000, 4 queries per shared prefix, prompt length 6000), served
    one query per step with one prompt of cache under Def. 2's timeline with an attention term.  A
    step is match -> select -> commit -> timed queue advance on a device-resident queue; the queue
    length never leaves the device."""
    import torch

    import paper_2502_04677_amd as K
    import workloads as W

    dev = torch.device("cuda:0")
    n, rep, c_num, c_den = 2000, 4, 1, 1 << 16
    u, d = args.def3_u, 6000 - args.def3_u
    if args.sweep:
        return bench_def3_sweep(args, n, rep, u, d, c_num, c_den)
    gap = ((u // rep + d) + (u + d)) // 2
    p, _ = W.shuffled_queue(n, u, rep, d, gap, seed=W.generators.SEED_BASE + 100)
    p.arrival[:] = p.arrival * np.uint64(c_den)
    k, cap, budget = rep, 2048, u + d
    q = K.DeviceQueries.from_host(p, dev)
    cfg = K.size_config(0, 0, budget, 1, u + d, extra_prompts=2)

    def one_run():
        sched = K.Scheduler(cfg, None, cap, dev)
        run = K.TimedRun(sched, q, cap, p.arrival, c_num=c_num, c_den=c_den)
        graphs = {}
        if args.graph:  # one captured step per queue buffer set, replayed in turn
            K.kLPM_reserve_clock(sched.tree, n + 8)
            for _ in range(2):
                parity = run.cur
                graphs[parity] = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graphs[parity]):
                    run.step(k, 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):  # one query per step: exactly n steps serve everybody
            if graphs:
                graphs[run.cur].replay()
                run.cur = 1 - run.cur
            else:
                run.step(k, 1)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert int(run.queue.n.item()) == 0 and int(run.queue.n_joined.item()) == n
        assert int(run.dev_error.item()) == 0 and sched.read_stats().device_error == 0
        return dt, run

    for _ in range(args.warmup):
        one_run()
    times = []
    for _ in range(max(1, args.steps // 4)):
        dt, run = one_run()
        times.append(dt)
    dt = float(np.mean(times))
    ttft = run.ttft[:n].cpu().numpy()
    matched = int(run.matched.item())
    out = {
        "metric": "scheduling steps/sec (match + select + commit + timed queue advance, one query per step)",
        "value": n / dt, "unit": "steps/s", "n_gpus": 1, "steps": n * len(times), "warmup": n * args.warmup,
        "ms_per_step": dt / n * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"def3-n{n}-rep{rep}-u{u}-d{d}", "k": k, "batch": 1, "kv_budget_tokens": budget,
                   "arrival_gap_tokens": gap, "c_attn": c_num / c_den, "queue_cap": cap,
                   "launch": "hip graph replay" if args.graph else "stream"},
        "matched_tokens_per_run": matched,
        "ttft_token_times": {f"p{int(x * 100)}": float(np.sort(ttft)[int(np.ceil(x * n)) - 1]) / c_den
                             for x in (0.5, 0.9, 0.95, 0.99)},
        "roofline": None,  # launch-latency bound at this size (a few KB per step); see the large configuration
    }
    if args.cpu_steps > 0:
        import oracle

        t0 = time.perf_counter()
        r = oracle.simulate_timed(p, k, 1, budget, c_num=c_num, c_den=c_den, queue_cap=cap)
        cdt = time.perf_counter() - t0
        assert r.ttft.tolist() == ttft.tolist(), "GPU and oracle disagree on the TTFT of the timed run"
        out["cpu_baseline"] = {"value": r.steps / cdt, "unit": "steps/s", "cores": 1, "kind": "oracle",
                               "sample": f"the whole run ({r.steps} steps), {cdt:.2f}s"}
    print(json.dumps(out), flush=True)
    return 0


def bench_def3_sweep(args, n, rep, u, d, c_num, c_den) -> int:
    """Thm. 2's setting over a sweep of the arrival gap s and of k: processing starts when everything
    has arrived (T = s n), equal match lengths are ordered by random keys, one query per step, one
    prompt of cache.  Every run's TTFTs are checked against the oracle's; the table lists TTFT
    percentiles in token times per (s, k)."""
    import torch

    import oracle
    import paper_2502_04677_amd as K
    import workloads as W

    dev = torch.device("cuda:0")
    cap, budget, seed = 2048, u + d, 99
    cfg = K.size_config(0, 0, budget, 1, u + d, extra_prompts=2)
    rows, gpu_s, cpu_s, steps = [], 0.0, 0.0, 0
    # late start (everything has arrived: Thm. 2), then service from time 0 at gaps between the cost of
    # a query with full reuse and with none (the request-rate axis of the paper's TTFT plots)
    full, none = u // rep + d, u + d
    cases = [(g, True) for g in (u // 6, u // 2, 5 * u // 6, 7 * u // 6, 5 * u // 3)]
    cases += [(g, False) for g in (full + (none - full) // 8, (full + none) // 2, none - (none - full) // 8, none + none // 8)]
    for s_gap, late in cases:
        p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=W.generators.SEED_BASE + 100)
        p.arrival[:] = p.arrival * np.uint64(c_den)
        q = K.DeviceQueries.from_host(p, dev)
        t_start = s_gap * n * c_den if late else 0
        arms = [1, 2, rep, 2 * rep, K.KLPM_K_INFINITY]
        # the fixed values of k, then k chosen per window of 20 steps by the device-side epsilon-greedy
        # rule over the same values (a quarter of the pulls exploring)
        for k in arms + ["adaptive"]:
            sched = K.Scheduler(cfg, None, cap, dev)
            run = K.TimedRun(sched, q, cap, p.arrival, c_num=c_num, c_den=c_den, t_start=t_start, tie_seed=seed)
            ad = K.AdaptiveK(arms, 20, 1 << 30, seed) if k == "adaptive" else None
            k_host = 0 if ad is not None else k
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                run.step(k_host, 1, adaptive=ad)
            torch.cuda.synchronize()
            gpu_s += time.perf_counter() - t0
            assert int(run.queue.n.item()) == 0 and int(run.dev_error.item()) == 0
            ttft = run.ttft[:n].cpu().numpy()
            ad_ref = oracle.AdaptiveK(arms, 20, 1 << 30, seed) if ad is not None else None
            t0 = time.perf_counter()
            r = oracle.simulate_timed(p, k_host, 1, budget, c_num=c_num, c_den=c_den, queue_cap=cap, t_start=t_start,
                                      tie_seed=seed, adaptive=ad_ref)
            cpu_s += time.perf_counter() - t0
            assert r.ttft.tolist() == ttft.tolist(), f"GPU and oracle disagree at s={s_gap} k={k}"
            steps += n
            t = np.sort(ttft) / c_den
            rows.append({"s": s_gap, "start": "after the last arrival" if late else "0",
                         "k": "inf" if k == K.KLPM_K_INFINITY else k,
                         **{name: round(float(t[int(np.ceil(x * n)) - 1])) for name, x in
                            (("p50", 0.5), ("p95", 0.95), ("p99", 0.99), ("max", 1.0))}})
            if ad is not None:
                st = ad.read()
                assert list(st.count)[:len(arms)] == ad_ref.count and list(st.cost)[:len(arms)] == ad_ref.cost
                rows[-1]["pulls_per_arm"] = ad_ref.count
            log(f"s={s_gap} k={rows[-1]['k']}: {rows[-1]}")
    out = {
        "metric": "scheduling steps/sec (match + tie keys + select + commit + timed queue advance, one query per step)",
        "value": steps / gpu_s, "unit": "steps/s", "n_gpus": 1, "steps": steps, "warmup": 0,
        "ms_per_step": gpu_s / steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"def3-n{n}-rep{rep}-u{u}-d{d}-gap-sweep", "batch": 1, "kv_budget_tokens": budget,
                   "c_attn": c_num / c_den, "queue_cap": cap, "ties": "random"},
        "sweep_ttft_token_times": rows,
        "roofline": None,  # launch-latency bound at this size; see the large configuration
        "cpu_baseline": {"value": steps / cpu_s, "unit": "steps/s", "cores": 1, "kind": "oracle",
                         "sample": f"every run of the sweep ({steps} steps), {cpu_s:.1f}s"},
    }
    print(json.dumps(out), flush=True)
    return 0


def bench_cfg4(args) -> int:
    """The online-stream configuration: 1,000 scheduling steps, Poisson(128) arrivals per step from
    the large configuration's group recipe, empty cache at the start, 4M-token KV budget with LRU
    eviction, k = 4, batch 256; prefill cost = uncached tokens.  Reports steps/s and the simulated
    TTFT distribution; the oracle runs the same stream on the host as the baseline."""
    import torch

    import paper_2502_04677_amd as K
    import workloads as W

    dev = torch.device("cuda:0")
    stream = W.config4_stream()
    hq = stream.queries
    cap = 8192
    q = K.DeviceQueries.from_host(hq, dev)
    cfg = K.size_config(0, 0, stream.budget, stream.batch, int(hq.len.max()), extra_prompts=hq.n)
    ids = [torch.arange(int(stream.step_start[s]), int(stream.step_start[s + 1]), dtype=torch.int32, device=dev)
           for s in range(stream.steps)]

    def one_run():
        sched = K.Scheduler(cfg, None, cap, dev)
        run = K.OnlineRun(sched, q, cap, np.arange(int(stream.step_start[0]), int(stream.step_start[1])))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(stream.steps):
            run.step(stream.k, stream.batch, ids[s + 1] if s + 1 < stream.steps else None)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        assert int(run.dev_error.item()) == 0 and K.kLPM_read_stats(sched.tree).device_error == 0
        return dt, run

    for _ in range(max(1, min(args.warmup, 1))):
        one_run()
    times = []
    for _ in range(max(1, args.steps // 10)):
        dt, run = one_run()
        times.append(dt)
    dt = float(np.mean(times))
    ttft = run.ttft[:hq.n].cpu().numpy()
    done = np.sort(ttft[ttft >= 0])
    out = {
        "metric": "scheduling steps/sec (online stream: match + select + commit + queue update per step)",
        "value": stream.steps / dt, "unit": "steps/s", "n_gpus": 1, "steps": stream.steps * len(times),
        "warmup": stream.steps, "ms_per_step": dt / stream.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": stream.name, "steps": stream.steps, "queries": hq.n, "stream_tokens": int(hq.tokens.shape[0]),
                   "k": stream.k, "batch": stream.batch, "kv_budget_tokens": stream.budget},
        "matched_tokens_per_run": int(run.matched.item()),
        "ttft_uncached_tokens": {"p50": int(done[int(np.ceil(0.5 * done.shape[0])) - 1]),
                                 "p99": int(done[int(np.ceil(0.99 * done.shape[0])) - 1]), "admitted": int(done.shape[0])},
        "roofline": None,  # a few hundred waiting queries per step: launch-latency bound, see the large configuration
    }
    if args.cpu_steps > 0:
        import oracle

        t0 = time.perf_counter()
        r = oracle.simulate_stream(stream)
        cdt = time.perf_counter() - t0
        assert r.ttft.tolist() == ttft.tolist(), "GPU and oracle disagree on the TTFT of the stream"
        out["cpu_baseline"] = {"value": stream.steps / cdt, "unit": "steps/s", "cores": 1, "kind": "oracle",
                               "sample": f"the whole stream ({stream.steps} steps), {cdt:.2f}s"}
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only)")
    ap.add_argument("--cpu-steps", type=int, default=32, help="oracle steps timed for the CPU baseline, at most all the steps run on the GPU (0 = skip)")
    ap.add_argument("--deep", action="store_true",
                    help="deep-tree variant of the workload (about 50-90 tokens per tree node)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain copy kernel over this many MiB (reference point for HBM byte counters)")
    ap.add_argument("--score", choices=("length", "rate"), default="length",
                    help="what longest-match picks maximise: match length (default) or hit rate m/|x|")
    ap.add_argument("--random-ties", action="store_true", help="break score ties uniformly at random (Philox keys)")
    ap.add_argument("--dynamic", action="store_true",
                    help="in-batch rescoring: scores follow the prompts picked earlier in the same batch")
    ap.add_argument("--sweep", action="store_true",
                    help="with --workload def3: sweep the arrival gap and k in the setting of Thm. 2 (late start, random ties)")
    ap.add_argument("--rematch", action="store_true",
                    help="let the commit match the admitted prompts again instead of taking the step's match results")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed steps, replay K more steps from one captured HIP graph and report them too")
    ap.add_argument("--extras", action="store_true",
                    help="also time the prefill-token cut and the cache-slot output on the last batch")
    ap.add_argument("--workload", choices=("cfg2-large", "def3", "cfg4"), default="cfg2-large",
                    help="def3: the timed Regular Arrival Shuffled Queue run; cfg4: the 1,000-step online stream")
    ap.add_argument("--def3-u", type=int, default=3000, help="shared-prefix length of the def3 workload (prompt = 6000)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; --gpus must be 1 (there is no multi-GPU path to time)",
              file=sys.stderr)
        return 2

    import torch

    import paper_2502_04677_amd as K

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "def3":
        return bench_def3(args)
    if args.workload == "cfg4":
        return bench_cfg4(args)
    dev = torch.device("cuda:0")
    # warm-up, the K timed steps, K further steps for the per-phase breakdown, then the graph passes
    steps_total = args.warmup + 2 * args.steps + (2 * args.steps if args.graph else 0)
    w, allq = build_workload(args.scale, steps_total, args.deep)
    batch, k, n0 = w.batch, w.k, w.queries.n
    max_len = int(max(w.cache.len.max(), allq.len.max()))

    t0 = time.time()
    cache_d = K.DeviceQueries.from_host(w.cache, dev)
    all_d = K.DeviceQueries.from_host(allq, dev)
    cfg = K.size_config(int(w.cache.tokens.shape[0]), w.cache.n, w.budget, batch, max_len,
                        extra_prompts=steps_total * batch)
    sched = K.Scheduler(cfg, cache_d, n0, dev)
    torch.cuda.synchronize()
    st = K.kLPM_read_stats(sched.tree)
    log(f"tree built on the GPU in {time.time() - t0:.1f}s: {st.total_tokens} tokens, {st.n_nodes} nodes, "
        f"device_error={st.device_error}")
    del cache_d
    run = K.OnlineRun(sched, all_d, n0, np.arange(n0), first_arrival=w.queries.arrival)
    new_ids = [torch.arange(n0 + s * batch, n0 + (s + 1) * batch, dtype=torch.int32, device=dev)
               for s in range(steps_total)]
    sums = torch.zeros(steps_total, dtype=torch.int64, device=dev)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps_total)]

    rate_bits = 26  # two histogram levels; exact as a ratio order for prompts up to 8,192 tokens
    score = torch.zeros(n0, dtype=torch.int32, device=dev) if args.score == "rate" else None
    tie = torch.zeros(n0, dtype=torch.int32, device=dev) if args.random_ties else None

    if args.dynamic:
        dyn_bytes = K.kLPM_select_dynamic_workspace_bytes(n0)
        dyn_ws = K.alloc_aligned(dyn_bytes, dev)
        dyn = torch.zeros(n0, dtype=torch.int32, device=dev)

    # Event records cost about 3.5 us each on the stream.  The timed steps carry only the two that
    # bracket the match launch (the roofline figure needs them); the other phases are timed on K
    # further steps that do not count towards the throughput.  None while a graph is being captured.
    timing = {"on": True, "phases": True}

    def mark(s: int, i: int) -> None:
        if timing["on"] and (timing["phases"] or i <= 1):
            ev[s][i].record()

    def one_step(s: int) -> None:
        q = run.view()
        mark(s, 0)
        sched.match(q)  # lengths and end nodes: the commit takes the admitted prompts' matches from here
        mark(s, 1)
        if args.dynamic:  # Algorithm 1 on scores that follow the picks made so far in the bin
            K.kLPM_select_dynamic(q, sched.match_len, sched.last_node, k, batch, sched.phase, dyn, sched.batch_idx,
                                  sched.n_selected, dyn_ws, dyn_bytes)
            mark(s, 2)
            sched.commit(q, batch, reuse_match=not args.rematch)
            mark(s, 3)
            run.advance(batch, new_ids[s], matched=sums[s:s + 1])
            mark(s, 4)
            return
        if score is not None:  # hit rate instead of match length (the wording of Algorithm 1)
            K.kLPM_score_hit_rate(sched.match_len, q.len, n0, rate_bits, score)
        if tie is not None:  # uniformly random tie-break, redrawn every step, keyed by query id
            K.kLPM_tie_keys(TIE_SEED, s, run.queue.id, n0, tie)
        # the queue is kept in arrival order
        sched.select(q, k, batch, fifo=True, score=score, score_max=1 << rate_bits, tie_key=tie)
        mark(s, 2)
        sched.commit(q, batch, reuse_match=not args.rematch)
        mark(s, 3)
        run.advance(batch, new_ids[s], matched=sums[s:s + 1])
        mark(s, 4)

    if args.calib_copy_mib > 0:
        # a plain elementwise copy of known size: reads and writes calib_copy_mib MiB each
        n_el = args.calib_copy_mib * (1 << 20) // 4
        src = torch.ones(n_el, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    timing["phases"] = False
    t_start = time.perf_counter()
    for s in range(args.warmup, args.warmup + args.steps):
        one_step(s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    timing["phases"] = True
    phase_steps = range(args.warmup + args.steps, args.warmup + 2 * args.steps)
    for s in phase_steps:
        one_step(s)
    torch.cuda.synchronize()

    graph_elapsed = None
    if args.graph:
        # the next K steps once more, captured into one HIP graph (every library call only enqueues
        # kernels) and replayed in one go: the same launches without the per-launch host cost
        # (two graphs of K steps each: the first replay is a warm-up of the graph machinery)
        K.kLPM_reserve_clock(sched.tree, (2 * args.steps + 1) * batch)
        g_warm, g = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        timing["on"] = False
        with torch.cuda.graph(g_warm):
            for s in range(args.warmup + 2 * args.steps, args.warmup + 3 * args.steps):
                one_step(s)
        with torch.cuda.graph(g):
            for s in range(args.warmup + 3 * args.steps, steps_total):
                one_step(s)
        timing["on"] = True
        g_warm.replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        graph_elapsed = time.perf_counter() - t_g

    st = sched.read_stats()
    assert st.device_error == 0 and int(run.dev_error.item()) == 0, f"device error {st.device_error}"
    sums_h = sums.cpu().numpy()
    timed = range(args.warmup, args.warmup + args.steps)
    match_ms = np.array([ev[s][0].elapsed_time(ev[s][1]) for s in timed])
    match_p_ms = np.array([ev[s][0].elapsed_time(ev[s][1]) for s in phase_steps])
    select_ms = np.array([ev[s][1].elapsed_time(ev[s][2]) for s in phase_steps])
    commit_ms = np.array([ev[s][2].elapsed_time(ev[s][3]) for s in phase_steps])
    adv_ms = np.array([ev[s][3].elapsed_time(ev[s][4]) for s in phase_steps])
    sum_timed = int(sums_h[args.warmup:args.warmup + args.steps].sum())
    value = sum_timed / elapsed
    alg_bytes = float(np.mean([algorithmic_bytes(int(sums_h[s]), n0) for s in timed]))
    match_s = float(match_ms.mean()) * 1e-3
    achieved = alg_bytes / match_s / 1e9

    out = {
        "metric": "prefix-match tokens/sec (whole scheduling step: match + select + commit + queue update)",
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": w.name if args.scale == 1.0 else f"{w.name}-scale{args.scale}",
                   "cache_tokens": int(st.total_tokens), "tree_nodes": int(st.n_nodes), "waiting_queries": n0,
                   "batch": batch, "k": k, "kv_budget_tokens": int(w.budget), "max_prompt_len": max_len,
                   "score": args.score, "ties": "random" if args.random_ties else "arrival",
                   "rescoring": "in-batch" if args.dynamic else "per step"},
        "schedule_latency_us": elapsed / args.steps * 1e6,
        "phase_ms": {"match": float(match_p_ms.mean()), "select": float(select_ms.mean()),
                     "commit": float(commit_ms.mean()), "queue_advance": float(adv_ms.mean())},
        "phase_ms_from": "the K steps after the timed ones, with an event record after every phase (about 3.5 us "
                         "each, which is why they stay out of the timed region; the timed steps only bracket the "
                         "match launch)",
        "match_tokens_per_s_kernel": float(np.mean(sums_h[args.warmup:args.warmup + args.steps])) / match_s,
        "matched_tokens_per_step": float(np.mean(sums_h[args.warmup:args.warmup + args.steps])),
        "roofline": {"kernel": "k_match", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (recorded_traffic()
                                 if args.scale == 1.0 and args.steps == 20 and args.warmup == 3 and not args.deep else None),
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": float(match_ms.mean())},
    }

    if graph_elapsed is not None:
        g_sum = int(sums_h[args.warmup + 3 * args.steps:].sum())
        out["graph_replay"] = {"steps": args.steps, "ms_per_step": graph_elapsed / args.steps * 1e3,
                               "value": g_sum / graph_elapsed, "unit": "tokens/s",
                               "note": "K later steps captured into one HIP graph and replayed once (after a warm-up replay of K steps)"}

    if args.extras:
        # serving-side steps on the last step's state (outside the timed loop): the prefill-token cut
        # of the batch and the cache slots of its matched prefixes
        q = run.view()
        sched.match(q)
        sched.select(q, k, batch, fifo=True)
        n_m = torch.zeros(batch, dtype=torch.int32, device=dev)
        slots = torch.empty(batch * max_len, dtype=torch.int64, device=dev)
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        reps = 20
        for _ in range(3):
            K.kLPM_kv_slots(sched.tree, q, sched.batch_idx, sched.n_selected, batch, max_len, n_m, slots)
        e0.record()
        for _ in range(reps):
            K.kLPM_batch_token_budget(q, sched.match_len, sched.batch_idx, sched.n_selected, batch, 1 << 50, k, sched.phase)
        e1.record()
        for _ in range(reps):
            K.kLPM_kv_slots(sched.tree, q, sched.batch_idx, sched.n_selected, batch, max_len, n_m, slots)
        e2.record()
        torch.cuda.synchronize()
        m_batch = int(n_m.sum().item())
        kv_ms = e1.elapsed_time(e2) / reps
        # what plain streaming reaches on this GPU (context for the match kernel's figure): a 1 GiB
        # device-to-device copy (read + write) and a 1 GiB read-only sweep
        big = torch.empty(1 << 28, dtype=torch.int32, device=dev).fill_(1)
        dst = torch.empty_like(big)
        sink = torch.zeros(1, dtype=torch.int64, device=dev)
        c0, c1, c2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        dst.copy_(big)
        K.kLPM_probe_read(big, sink)
        c0.record()
        for _ in range(5):
            dst.copy_(big)
        c1.record()
        for _ in range(5):
            K.kLPM_probe_read(big, sink)
        c2.record()
        torch.cuda.synchronize()
        copy_gbs = 2.0 * big.numel() * 4 / (c0.elapsed_time(c1) / 5 * 1e-3) / 1e9
        read_gbs = 1.0 * big.numel() * 4 / (c1.elapsed_time(c2) / 5 * 1e-3) / 1e9
        del big, dst
        out["extras"] = {"stream_copy_GBps": copy_gbs, "stream_read_GBps": read_gbs,
                         "token_budget_ms": e0.elapsed_time(e1) / reps, "kv_slots_ms": kv_ms,
                         "kv_slots_matched_tokens": m_batch,
                         # per matched token: 4 B query + 4 B edge token read, 8 B slot written
                         "kv_slots_GBps": 16.0 * m_batch / (kv_ms * 1e-3) / 1e9}

    if args.cpu_steps > 0:
        cores = len(os.sched_getaffinity(0))
        threads = max(1, min(cores, 16))
        cpu_steps = min(args.cpu_steps, steps_total)
        v, dt, t_match, step_sums = cpu_baseline(w, allq, cpu_steps, threads, rate_bits if score is not None else 0,
                                                 args.random_ties, args.dynamic)
        # matched tokens of every sampled step: they depend on all earlier selections and commits
        assert step_sums == [int(v) for v in sums_h[:cpu_steps]], f"GPU and oracle disagree: {sums_h[:cpu_steps]} vs {step_sums}"
        out["cpu_baseline"] = {"value": v, "unit": "tokens/s", "cores": threads, "kind": "oracle",
                               "sample": f"first {cpu_steps} steps of the same workload (match on {threads} threads, "
                                         f"select/commit serial), {dt:.1f}s; match alone {t_match:.2f}s"}
        log(f"cpu baseline: {v:.3e} tokens/s on {threads} threads ({dt:.1f}s for {cpu_steps} steps)")
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
