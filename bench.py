#!/usr/bin/env python3
"""Benchmark of the k-LPM scheduling step on one MI355X.

A step is one pass of the whole path over the waiting queue: prefix-match every waiting query
against the GPU-resident radix tree, pick the k-LPM batch, commit it (insert + LRU-evict to the KV
budget), retire the batch from the queue and enqueue the next arrivals.  The default workload is
the large configuration (about 100M cached tokens, 65,536 waiting queries of up to 8,192 tokens,
k = 8, batch 1,024); inputs are synthetic, seeded and already resident in HBM when timing starts.

Prints one JSON line: prefix-match tokens/s over the timed steps; the roofline record of the match
kernel (algorithmic bytes / kernel time against the 8 TB/s HBM peak, and beside it the counter
traffic, the compulsory bytes, the kernel time on cold caches and what a plain streaming read
reaches on the same GPU); per-phase times of the same steps; the distribution of the per-step
latency; and the CPU oracle timed on the host cores over a bounded sample of the same steps.
`--workload cfg0|cfg1|cfg3` time the single-step configurations (match once, then select; cfg3 with
its sweep of k); `--workload def3|cfg4` the timed Def. 3 queue and the 1,000-step online stream.
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
FLUSH_BYTES = 1 << 30  # swept between cold launches: four times the 256 MB Infinity Cache


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(sum_match: int, n_queries: int) -> int:
    """Bytes the match kernel has to move for one launch: for every compared position (the matched
    tokens and the first mismatch) 4 B of query token and 4 B of edge token, plus per query its
    offset (8 B), length (4 B) and the 4 B result.  Child-table slots (32 B per node visited) are
    left out, so the figure is a lower bound."""
    return 8 * (sum_match + n_queries) + 16 * n_queries


def query_side_bytes(sum_match: int, n_queries: int) -> int:
    """The part of the algorithmic bytes that no cache can serve: every query token is read once."""
    return 4 * (sum_match + n_queries) + 16 * n_queries


def recorded_traffic(workload: str):
    """HBM bytes per match launch from the committed rocprofv3 counter summary of this workload, or
    None when the kernel sources have changed since those counters were taken (or there is none)."""
    import hashlib

    path = os.path.join(ROOT, "profiles", f"k_match_{workload}_hbm_counters.txt")
    try:
        fields = dict(line.strip().split("=", 1) for line in open(path) if "=" in line and not line.startswith(" "))
        h = hashlib.sha256()
        for rel in ("paper_2502_04677_amd/csrc/match.hip", "paper_2502_04677_amd/csrc/klpm_device.hpp"):
            h.update(open(os.path.join(ROOT, rel), "rb").read())
        if fields.get("kernel_source_sha256") != h.hexdigest():
            return None
        return {"bytes_per_launch": float(fields["traffic_bytes_per_launch"]),
                "bytes_per_cold_launch": float(fields["traffic_bytes_per_cold_launch"])
                if "traffic_bytes_per_cold_launch" in fields else None}
    except (OSError, KeyError, ValueError):
        return None


def pct(values, p: float) -> float:
    """Nearest-rank percentile."""
    v = np.sort(np.asarray(values, dtype=np.float64))
    return float(v[max(1, int(np.ceil(p * v.shape[0]))) - 1])


class MatchProbe:
    """Measurements around one queue-wide match launch on a fixed state: the launch on cold caches
    (a 1 GiB read sweep before each launch pushes queries and tree out of L2 and the Infinity
    Cache), the launch repeated back to back, the plain streaming-read rate of the same GPU, and the
    tree-side bytes the launch must fetch at least once."""

    def __init__(self, K, torch, dev):
        self.K, self.torch, self.dev = K, torch, dev
        self.flush = torch.empty(FLUSH_BYTES // 4, dtype=torch.int32, device=dev).fill_(1)
        self.sink = torch.zeros(1, dtype=torch.int64, device=dev)

    def _events(self, n):
        return [(self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)) for _ in range(n)]

    def stream_read_gbs(self, reps: int = 5) -> float:
        K, torch = self.K, self.torch
        K.kLPM_probe_read(self.flush, self.sink)
        ev = self._events(reps)
        for a, b in ev:
            a.record()
            K.kLPM_probe_read(self.flush, self.sink)
            b.record()
        torch.cuda.synchronize()
        ms = float(np.median([a.elapsed_time(b) for a, b in ev]))
        return FLUSH_BYTES / (ms * 1e-3) / 1e9

    def match_ms(self, sched, q, reps: int, cold: bool) -> float:
        K, torch = self.K, self.torch
        ev = self._events(reps)
        sched.match(q)
        for a, b in ev:
            if cold:
                K.kLPM_probe_read(self.flush, self.sink)
            a.record()
            sched.match(q)
            b.record()
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in ev]))

    def unique_tree_tokens(self, sched, q, max_len: int) -> int:
        """Distinct cached tokens that the queue's matched prefixes cover: the cache slots of every
        query's matched prefix (kLPM_kv_slots, a chunk of queries at a time) marked in a bitmap over
        the token pool."""
        K, torch, dev = self.K, self.torch, self.dev
        chunk = 2048
        if getattr(self, "_slots", None) is None or self._slots.numel() != chunk * max_len:
            self._slots = torch.empty(chunk * max_len, dtype=torch.int64, device=dev)
            self._n_m = torch.zeros(chunk, dtype=torch.int32, device=dev)
            self._n_sel = torch.zeros(1, dtype=torch.int32, device=dev)
            self._col = torch.arange(max_len, dtype=torch.int32, device=dev)[None, :]
        pool = 2 * int(sched.cfg.pool_tokens)
        if getattr(self, "_touched", None) is None or self._touched.numel() != pool:
            self._touched = torch.zeros(pool, dtype=torch.bool, device=dev)
        touched, slots, n_m = self._touched.zero_(), self._slots, self._n_m
        for lo in range(0, q.n, chunk):
            idx = torch.arange(lo, lo + chunk, dtype=torch.int32, device=dev)
            self._n_sel.fill_(min(chunk, q.n - lo))
            K.kLPM_kv_slots(sched.tree, q, idx, self._n_sel, chunk, max_len, n_m, slots)
            valid = self._col < n_m[:, None]
            touched[slots.view(chunk, max_len)[valid]] = True
        return int(touched.sum().item())


def oracle_split(tree, tokens, off, ln, arrival, k, batch, threads, commit_budget=None):
    """The oracle's phases timed one by one on one queue: match on one thread and on `threads`
    threads, the literal Algorithm 1 loop, and (with a budget) the commit."""
    import oracle

    t0 = time.perf_counter()
    m1 = tree.match(tokens, off, ln, threads=1)
    t_m1 = time.perf_counter() - t0
    t0 = time.perf_counter()
    m = tree.match(tokens, off, ln, threads=threads)
    t_mt = time.perf_counter() - t0
    assert (m == m1).all()
    t0 = time.perf_counter()
    idx, phase = oracle.select(arrival, m, k, batch, 0)
    t_sel = time.perf_counter() - t0
    t_com = None
    if commit_budget is not None:
        t0 = time.perf_counter()
        tree.commit(tokens, off, ln, idx, commit_budget)
        t_com = time.perf_counter() - t0
    return m, idx, phase, t_m1, t_mt, t_sel, t_com


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


def bench_cfg4_overload(args) -> int:
    """The online stream served with a batch smaller than the arrival rate (Poisson(128) arrivals against a
    batch of `--overload-batch`, default 96), so that the queue backs up and k decides who waits: the same
    1,000 steps of arrivals, then steps without arrivals until the queue has drained, once per k of
    {1, 2, 4, 8, infinity}.  Reports steps/s and the simulated TTFT distribution (uncached-token times) per k;
    with --cpu-steps > 0 the oracle runs every stream too and every TTFT must agree."""
    import torch

    import paper_2502_04677_amd as K
    import workloads as W

    dev = torch.device("cuda:0")
    base = W.config4_stream()
    hq = base.queries
    batch = int(args.overload_batch)
    drain = (hq.n + batch - 1) // batch - base.steps
    step_start = np.concatenate([base.step_start, np.full(max(drain, 0), base.step_start[-1], dtype=np.int64)])
    steps = int(step_start.shape[0] - 1)
    cap = 1 << 16
    q = K.DeviceQueries.from_host(hq, dev)
    cfg = K.size_config(0, 0, base.budget, batch, int(hq.len.max()), extra_prompts=hq.n)
    ids = [torch.arange(int(step_start[s]), int(step_start[s + 1]), dtype=torch.int32, device=dev) if step_start[s + 1] > step_start[s]
           else None for s in range(steps)]
    rows = []
    total_dt = 0.0
    for k in (1, 2, 4, 8, 0xFFFFFFFF):
        def one_run():
            sched = K.Scheduler(cfg, None, cap, dev)
            run = K.OnlineRun(sched, q, cap, np.arange(int(step_start[0]), int(step_start[1])))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(steps):
                run.step(k, batch, ids[s + 1] if s + 1 < steps else None)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            assert int(run.dev_error.item()) == 0 and K.kLPM_read_stats(sched.tree).device_error == 0
            return dt, run
        one_run()
        dt, run = one_run()
        total_dt += dt
        ttft = run.ttft[:hq.n].cpu().numpy()
        assert (ttft >= 0).all(), "the drain steps must admit every query"
        done = np.sort(ttft)
        pct = lambda p: int(done[int(np.ceil(p * done.shape[0])) - 1])
        row = {"k": "inf" if k == 0xFFFFFFFF else k, "steps": steps, "steps_per_s": steps / dt, "ms_per_step": dt / steps * 1e3,
               "matched_tokens": int(run.matched.item()), "makespan": int(run.sim_clock.item()),
               "ttft_p50": pct(0.5), "ttft_p90": pct(0.9), "ttft_p99": pct(0.99), "ttft_max": int(done[-1])}
        if args.cpu_steps > 0:
            import oracle

            t0 = time.perf_counter()
            r = oracle.simulate_stream(W.generators.Stream(base.name + "-overload", hq, step_start, k, batch, base.budget))
            row["oracle_steps_per_s"] = steps / (time.perf_counter() - t0)
            assert r.ttft.tolist() == ttft.tolist() and r.clock == row["makespan"], f"GPU and oracle disagree on the stream (k = {k})"
        log(f"overloaded stream k={row['k']}: {row['steps_per_s']:.0f} steps/s, TTFT p50 {row['ttft_p50']} p99 {row['ttft_p99']} max {row['ttft_max']}")
        rows.append(row)
    out = {
        "metric": "scheduling steps/sec (overloaded online stream: match + select + commit + queue update per step)",
        "value": 5 * steps / total_dt, "unit": "steps/s", "n_gpus": 1, "steps": 5 * steps, "warmup": 5 * steps,
        "ms_per_step": total_dt / (5 * steps) * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": base.name + "-overload", "arrival_steps": base.steps, "drain_steps": steps - base.steps,
                   "queries": hq.n, "batch": batch, "kv_budget_tokens": base.budget, "k": [r["k"] for r in rows]},
        "per_k": rows, "roofline": None,
    }
    if args.cpu_steps > 0:
        out["cpu_baseline"] = {"value": float(np.mean([r["oracle_steps_per_s"] for r in rows])), "unit": "steps/s", "cores": 1,
                               "kind": "oracle", "sample": "every stream of the sweep; every TTFT equal to the GPU's"}
    print(json.dumps(out), flush=True)
    return 0


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
    threads, select and commit serial), timed without the tree build; before the first step the
    match of the initial queue is also timed on one thread."""
    import oracle

    tree = oracle.OracleTree()
    tree.build(w.cache)
    n0, batch = w.queries.n, w.batch
    waiting = np.arange(n0, dtype=np.int64)
    enq = np.zeros(allq.n, dtype=np.uint64)
    enq[:n0] = w.queries.arrival
    t0 = time.perf_counter()
    m_1t = tree.match(allq.tokens, allq.off[waiting], allq.len[waiting], threads=1)
    t_match_1t = time.perf_counter() - t0
    clock, phase, matched = 0, 0, 0
    step_sums = []
    t_match = t_select = t_commit = 0.0
    t0 = time.perf_counter()
    for s in range(steps):
        off, ln, arr = allq.off[waiting], allq.len[waiting], enq[waiting]
        ta = time.perf_counter()
        m = tree.match(allq.tokens, off, ln, threads=threads)
        tb = time.perf_counter()
        sc = oracle.score_hit_rate(m, ln, rate_bits) if rate_bits else m
        tk = oracle.tie_keys(TIE_SEED, s, waiting) if random_ties else None
        if dynamic:
            idx, phase, _ = oracle.select_dynamic(allq.tokens, off, ln, arr, m, w.k, batch, phase)
        else:
            idx, phase = oracle.select(arr, sc, w.k, batch, phase, tie_key=tk)
        tc = time.perf_counter()
        tree.commit(allq.tokens, off, ln, idx, w.budget)
        td = time.perf_counter()
        t_match, t_select, t_commit = t_match + tb - ta, t_select + tc - tb, t_commit + td - tc
        clock += max(1, int((ln[idx].astype(np.int64) - m[idx]).sum()))
        keep = np.ones(waiting.shape[0], dtype=bool)
        keep[idx] = False
        new = np.arange(n0 + s * batch, n0 + (s + 1) * batch, dtype=np.int64)
        enq[new] = clock
        waiting = np.concatenate([waiting[keep], new])
        matched += int(m.sum())
        step_sums.append(int(m.sum()))
    dt = time.perf_counter() - t0
    return {"tokens_per_s": matched / dt, "seconds": dt, "match_s": t_match, "select_s": t_select, "commit_s": t_commit,
            "match_1thread_s": t_match_1t, "match_1thread_tokens": int(m_1t.sum()), "matched": matched,
            "step_sums": step_sums}


def bench_cfg2(args) -> int:
    import torch

    import paper_2502_04677_amd as K

    dev = torch.device("cuda:0")
    W_, K_, L_ = args.warmup, args.steps, args.latency_steps
    graph_steps = 2 * K_ if args.graph else 0
    steps_total = W_ + max(K_ + graph_steps, L_)
    w, allq = build_workload(args.scale, steps_total, args.deep)
    batch, k, n0 = w.batch, w.k, w.queries.n
    max_len = int(max(w.cache.len.max(), allq.len.max()))
    name = w.name if args.scale == 1.0 else f"{w.name}-scale{args.scale}"

    cache_d = K.DeviceQueries.from_host(w.cache, dev)
    all_d = K.DeviceQueries.from_host(allq, dev)
    cfg = K.size_config(int(w.cache.tokens.shape[0]), w.cache.n, w.budget, batch, max_len,
                        extra_prompts=steps_total * batch)
    new_ids = [torch.arange(n0 + s * batch, n0 + (s + 1) * batch, dtype=torch.int32, device=dev)
               for s in range(steps_total)]
    rate_bits = 26  # two histogram levels; exact as a ratio order for prompts up to 8,192 tokens
    score = torch.zeros(n0, dtype=torch.int32, device=dev) if args.score == "rate" else None
    tie = torch.zeros(n0, dtype=torch.int32, device=dev) if args.random_ties else None
    if args.dynamic:
        dyn_bytes = K.kLPM_select_dynamic_workspace_bytes(n0)
        dyn_ws = K.alloc_aligned(dyn_bytes, dev)
        dyn = torch.zeros(n0, dtype=torch.int32, device=dev)

    class Pass:
        """The workload from its initial state: a fresh tree, queue and per-step records."""

        def __init__(self, n_steps: int, marks):
            t0 = time.time()
            self.sched = K.Scheduler(cfg, cache_d, n0, dev)
            self.run = K.OnlineRun(self.sched, all_d, n0, np.arange(n0), first_arrival=w.queries.arrival)
            self.sums = torch.zeros(n_steps, dtype=torch.int64, device=dev)
            self.marks = marks  # event slots recorded in each step: subset of (0..4)
            self.ev = [[torch.cuda.Event(enable_timing=True) if i in marks else None for i in range(5)]
                       for _ in range(n_steps)]
            self.on = True
            torch.cuda.synchronize()
            self.build_s = time.time() - t0

        def mark(self, s: int, i: int) -> None:
            if self.on and self.ev[s][i] is not None:
                self.ev[s][i].record()

        def step(self, s: int) -> None:
            sched, run = self.sched, self.run
            q = run.view()
            self.mark(s, 0)
            sched.match(q)  # lengths and end nodes: the commit takes the admitted prompts' matches from here
            self.mark(s, 1)
            if args.dynamic:  # Algorithm 1 on scores that follow the picks made so far in the bin
                K.kLPM_select_dynamic(q, sched.match_len, sched.last_node, k, batch, sched.phase, dyn, sched.batch_idx,
                                      sched.n_selected, dyn_ws, dyn_bytes, flags=K.KLPM_SELECT_FIFO, max_match=max_len)
            else:
                if score is not None:  # hit rate instead of match length (the wording of Algorithm 1)
                    K.kLPM_score_hit_rate(sched.match_len, q.len, n0, rate_bits, score)
                if tie is not None:  # uniformly random tie-break, redrawn every step, keyed by query id
                    K.kLPM_tie_keys(TIE_SEED, s, run.queue.id, n0, tie)
                # the queue is kept in arrival order
                sched.select(q, k, batch, fifo=True, score=score, score_max=1 << rate_bits, tie_key=tie)
            self.mark(s, 2)
            sched.commit(q, batch, reuse_match=not args.rematch)
            self.mark(s, 3)
            run.advance(batch, new_ids[s], matched=self.sums[s:s + 1])
            self.mark(s, 4)

        def ms(self, s: int, a: int, b: int) -> float:
            return self.ev[s][a].elapsed_time(self.ev[s][b])

        def check(self) -> None:
            st = self.sched.read_stats()
            assert st.device_error == 0 and int(self.run.dev_error.item()) == 0, f"device error {st.device_error}"

    # ---- pass A: the timed steps.  Event records cost about 3.5 us each on the stream, so the timed
    # steps carry only the two that bracket the match launch (the roofline figure needs them).
    A = Pass(W_ + K_ + graph_steps, (0, 1))
    st0 = K.kLPM_read_stats(A.sched.tree)
    log(f"tree built on the GPU in {A.build_s:.1f}s: {st0.total_tokens} tokens, {st0.n_nodes} nodes, "
        f"device_error={st0.device_error}")
    if args.calib_copy_mib > 0:
        # a plain elementwise copy of known size: reads and writes calib_copy_mib MiB each
        n_el = args.calib_copy_mib * (1 << 20) // 4
        src = torch.ones(n_el, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for s in range(W_):
        A.step(s)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(W_, W_ + K_):
        A.step(s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    A.check()
    timed = range(W_, W_ + K_)
    sums_h = A.sums.cpu().numpy()
    match_ms = np.array([A.ms(s, 0, 1) for s in timed])
    sum_timed = int(sums_h[W_:W_ + K_].sum())
    alg_bytes = float(np.mean([algorithmic_bytes(int(sums_h[s]), n0) for s in timed]))
    match_s = float(match_ms.mean()) * 1e-3
    achieved = alg_bytes / match_s / 1e9
    st = A.sched.read_stats()

    rec = recorded_traffic(name) if not (args.dynamic or args.random_ties or args.score != "length") else None
    traffic = rec["bytes_per_launch"] if rec else None
    traffic_cold = rec["bytes_per_cold_launch"] if rec else None

    graph_elapsed = None
    if args.graph:
        # the next K steps once more, captured into one HIP graph (every library call only enqueues
        # kernels) and replayed in one go: the same launches without the per-launch host cost
        # (two graphs of K steps each: the first replay is a warm-up of the graph machinery)
        K.kLPM_reserve_clock(A.sched.tree, (2 * K_ + 1) * batch)
        g_warm, g = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        A.on = False
        with torch.cuda.graph(g_warm):
            for s in range(W_ + K_, W_ + 2 * K_):
                A.step(s)
        with torch.cuda.graph(g):
            for s in range(W_ + 2 * K_, W_ + 3 * K_):
                A.step(s)
        A.on = True
        g_warm.replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        graph_elapsed = time.perf_counter() - t_g
        A.check()
        g_sum = int(A.sums.cpu().numpy()[W_ + 2 * K_:W_ + 3 * K_].sum())

    extras = None
    if args.extras:
        # serving-side steps on the last state (outside the timed loop): the prefill-token cut of the
        # batch and the cache slots of its matched prefixes
        sched = A.sched
        q_now = A.run.view()
        sched.match(q_now)
        sched.select(q_now, k, batch, fifo=True)
        n_m = torch.zeros(batch, dtype=torch.int32, device=dev)
        slots = torch.empty(batch * max_len, dtype=torch.int64, device=dev)
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        reps = 20
        for _ in range(3):
            K.kLPM_kv_slots(sched.tree, q_now, sched.batch_idx, sched.n_selected, batch, max_len, n_m, slots)
        e0.record()
        for _ in range(reps):
            K.kLPM_batch_token_budget(q_now, sched.match_len, sched.batch_idx, sched.n_selected, batch, 1 << 50, k, sched.phase)
        e1.record()
        for _ in range(reps):
            K.kLPM_kv_slots(sched.tree, q_now, sched.batch_idx, sched.n_selected, batch, max_len, n_m, slots)
        e2.record()
        torch.cuda.synchronize()
        m_batch = int(n_m.sum().item())
        kv_ms = e1.elapsed_time(e2) / reps
        big = torch.empty(FLUSH_BYTES // 4, dtype=torch.int32, device=dev).fill_(1)
        dst = torch.empty_like(big)
        c0, c1 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
        dst.copy_(big)
        c0.record()
        for _ in range(5):
            dst.copy_(big)
        c1.record()
        torch.cuda.synchronize()
        extras = {"stream_copy_GBps": 2.0 * big.numel() * 4 / (c0.elapsed_time(c1) / 5 * 1e-3) / 1e9,
                  "token_budget_ms": e0.elapsed_time(e1) / reps, "kv_slots_ms": kv_ms,
                  "kv_slots_matched_tokens": m_batch,
                  # per matched token: 4 B query + 4 B edge token read, 8 B slot written
                  "kv_slots_GBps": 16.0 * m_batch / (kv_ms * 1e-3) / 1e9}
        del dst, big
    del A
    torch.cuda.empty_cache()

    # ---- pass B: the same steps from the same initial state with an event record after every phase
    B = Pass(W_ + K_, (0, 1, 2, 3, 4))
    for s in range(W_ + K_):
        B.step(s)
    torch.cuda.synchronize()
    B.check()
    assert (B.sums.cpu().numpy() == sums_h[:W_ + K_]).all(), "the two passes did not do the same steps"
    phase = {"match": float(np.mean([B.ms(s, 0, 1) for s in timed])),
             "select": float(np.mean([B.ms(s, 1, 2) for s in timed])),
             "commit": float(np.mean([B.ms(s, 2, 3) for s in timed])),
             "queue_advance": float(np.mean([B.ms(s, 3, 4) for s in timed]))}
    phase["sum"] = float(sum(phase.values()))
    del B
    torch.cuda.empty_cache()

    # ---- pass C: per-step latency over more steps, one event record per step
    latency = None
    if L_ > 0:
        C = Pass(W_ + L_, (0,))
        end = torch.cuda.Event(enable_timing=True)
        for s in range(W_ + L_):
            C.step(s)
        end.record()
        torch.cuda.synchronize()
        C.check()
        marks = [C.ev[s][0] for s in range(W_, W_ + L_)] + [end]
        lat = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(L_)]) * 1e3
        latency = {"steps": L_, "mean": float(lat.mean()), "p50": pct(lat, 0.5), "p90": pct(lat, 0.9),
                   "p99": pct(lat, 0.99), "max": float(lat.max()),
                   "from": f"{L_} steps after {W_} warm-up steps from the same initial state, one event record "
                           "(about 3.5 us) per step"}
        del C
        torch.cuda.empty_cache()

    # ---- pass D: the timed steps' match launches on cold caches.  Before each of those steps the
    # launch is made once more after a 1 GiB read sweep has emptied L2 and the Infinity Cache (the
    # step then runs as usual), and the distinct cached tokens under the queue's matches are counted:
    # with every query token read once they are what the launch must fetch at least.
    probe = MatchProbe(K, torch, dev)
    read_gbs = probe.stream_read_gbs()
    D = Pass(W_ + K_, ())
    cold_ev, uniq = [], []
    for s in range(W_ + K_):
        if s >= W_:
            q_s = D.run.view()
            uniq.append(probe.unique_tree_tokens(D.sched, q_s, max_len))
            K.kLPM_probe_read(probe.flush, probe.sink)
            e = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            e[0].record()
            D.sched.match(q_s)
            e[1].record()
            cold_ev.append(e)
        D.step(s)
    torch.cuda.synchronize()
    D.check()
    assert (D.sums.cpu().numpy() == sums_h[:W_ + K_]).all(), "the cold pass did not do the same steps"
    cold_ms = float(np.mean([a.elapsed_time(b) for a, b in cold_ev]))
    compulsory = float(np.mean([query_side_bytes(int(sums_h[s]), n0) + 4 * uniq[s - W_] for s in timed]))
    del D, probe
    torch.cuda.empty_cache()

    out = {
        "metric": "prefix-match tokens/sec (whole scheduling step: match + select + commit + queue update)",
        "value": sum_timed / elapsed,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": K_,
        "warmup": W_,
        "ms_per_step": elapsed / K_ * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": name,
                   "cache_tokens": int(st.total_tokens), "tree_nodes": int(st.n_nodes), "waiting_queries": n0,
                   "batch": batch, "k": k, "kv_budget_tokens": int(w.budget), "max_prompt_len": max_len,
                   "score": args.score, "ties": "random" if args.random_ties else "arrival",
                   "rescoring": "in-batch" if args.dynamic else "per step"},
        "schedule_latency_us": latency if latency is not None else {"mean": elapsed / K_ * 1e6},
        "phase_ms": phase,
        "phase_ms_from": "the same steps as the timed ones (same initial state, same batches), run again with an event "
                         "record after every phase; the four extra records cost those steps about 14 us each, which is "
                         "why the timed steps only bracket the match launch",
        "match_tokens_per_s_kernel": float(np.mean(sums_h[W_:W_ + K_])) / match_s,
        "matched_tokens_per_step": float(np.mean(sums_h[W_:W_ + K_])),
        "roofline": {"kernel": "k_match", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "achieved_is": "algorithmic bytes per launch / kernel time; the tree side of those bytes is "
                                    "mostly served by L2 and the Infinity Cache, so this is not an HBM rate",
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": float(match_ms.mean()),
                     "traffic_GBps": traffic / match_s / 1e9 if traffic else None,
                     "frac_traffic": traffic / match_s / 1e9 / HBM_PEAK_GBS if traffic else None,
                     "compulsory_bytes_per_launch": compulsory,
                     "compulsory_GBps": compulsory / match_s / 1e9,
                     "frac_compulsory": compulsory / match_s / 1e9 / HBM_PEAK_GBS,
                     "overread": (traffic - compulsory) / compulsory if traffic else None,
                     "stream_read_GBps": read_gbs,
                     "cold": {"what": "the same launches (same initial state, same steps) each made once more after a 1 GiB "
                                      "read sweep that empties L2 and the Infinity Cache",
                              "kernel_ms": cold_ms,
                              "unique_tree_tokens_per_launch": float(np.mean(uniq)),
                              "achieved": alg_bytes / (cold_ms * 1e-3) / 1e9,
                              "compulsory_GBps": compulsory / (cold_ms * 1e-3) / 1e9,
                              "frac_compulsory": compulsory / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "traffic": traffic_cold,
                              "traffic_GBps": traffic_cold / (cold_ms * 1e-3) / 1e9 if traffic_cold else None,
                              "frac_traffic": traffic_cold / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if traffic_cold else None,
                              "overread": (traffic_cold - compulsory) / compulsory if traffic_cold else None}},
        # queue-wide match launches in dispatch order, for reading a profiler's per-dispatch records
        "match_launches": [["timed pass: warm-up", W_], ["timed pass: timed", K_], ["timed pass: graph capture", graph_steps],
                           ["phase pass", W_ + K_], ["latency pass", (W_ + L_) if L_ > 0 else 0],
                           ["cold pass: warm-up", W_], ["cold pass: (cold launch, the step's own launch) pairs", 2 * K_]],
    }
    if graph_elapsed is not None:
        out["graph_replay"] = {"steps": K_, "ms_per_step": graph_elapsed / K_ * 1e3,
                               "value": g_sum / graph_elapsed, "unit": "tokens/s",
                               "note": "K later steps captured into one HIP graph and replayed once (after a warm-up replay of K steps)"}
    if extras is not None:
        out["extras"] = extras

    if args.cpu_steps > 0:
        cores = len(os.sched_getaffinity(0))
        threads = max(1, min(cores, 16))
        cpu_steps = min(args.cpu_steps, W_ + K_)
        r = cpu_baseline(w, allq, cpu_steps, threads, rate_bits if score is not None else 0, args.random_ties, args.dynamic)
        # matched tokens of every sampled step: they depend on all earlier selections and commits
        assert r["step_sums"] == [int(v) for v in sums_h[:cpu_steps]], f"GPU and oracle disagree: {sums_h[:cpu_steps]} vs {r['step_sums']}"
        out["cpu_baseline"] = {
            "value": r["tokens_per_s"], "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {cpu_steps} steps of the same workload (match on {threads} threads, select/commit "
                      f"serial), {r['seconds']:.1f}s; every step's matched tokens equal the GPU's",
            "ms_per_step": r["seconds"] / cpu_steps * 1e3,
            "match_tokens_per_s_1thread": r["match_1thread_tokens"] / r["match_1thread_s"],
            "match_tokens_per_s_allcores": r["matched"] / r["match_s"], "allcores": threads,
            "match_ms": r["match_s"] / cpu_steps * 1e3, "select_ms": r["select_s"] / cpu_steps * 1e3,
            "commit_ms": r["commit_s"] / cpu_steps * 1e3}
        log(f"cpu baseline: {r['tokens_per_s']:.3e} tokens/s on {threads} threads ({r['seconds']:.1f}s for {cpu_steps} steps)")
    print(json.dumps(out), flush=True)
    return 0


def bench_single_step(args) -> int:
    """The single-step configurations: the tree is built from the cached prompts, the whole waiting
    queue is matched once and the k-LPM batch is selected (cfg3: once per k of its sweep).  A step
    here is match + select; nothing is committed, so the step repeats on the same state."""
    import torch

    import paper_2502_04677_amd as K
    import workloads as W

    dev = torch.device("cuda:0")
    t0 = time.time()
    w = {"cfg0": W.config0, "cfg1": W.config1, "cfg3": W.config3}[args.workload]()
    log(f"generated {w.name}: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, queue {w.queries.n} "
        f"({w.queries.tokens.shape[0]} tokens) in {time.time() - t0:.1f}s")
    hq = w.queries
    n0, batch = hq.n, w.batch
    ks = list(w.ks) if w.ks else [w.k]
    max_len = int(max(w.cache.len.max(), hq.len.max()))
    cache_d = K.DeviceQueries.from_host(w.cache, dev)
    q = K.DeviceQueries.from_host(hq, dev)
    cfg = K.size_config(int(w.cache.tokens.shape[0]), w.cache.n, w.budget, batch, max_len)
    t0 = time.time()
    sched = K.Scheduler(cfg, cache_d, n0, dev)
    torch.cuda.synchronize()
    st = K.kLPM_read_stats(sched.tree)
    log(f"tree built on the GPU in {time.time() - t0:.1f}s: {st.total_tokens} tokens, {st.n_nodes} nodes")
    fifo = bool((np.diff(hq.arrival.astype(np.int64)) >= 0).all())  # all of these queues are in arrival order
    R = max(args.steps, 20)
    if args.calib_copy_mib > 0:
        # a plain elementwise copy of known size: reads and writes calib_copy_mib MiB each
        n_el = args.calib_copy_mib * (1 << 20) // 4
        src = torch.ones(n_el, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def step(k_):
        sched.set_phase(0)
        e = (ev(), ev(), ev())
        e[0].record()
        sched.match(q, want_nodes=False)
        e[1].record()
        sched.select(q, k_, batch, fifo=fifo)
        e[2].record()
        return e

    for k_ in ks:
        step(k_)
    torch.cuda.synchronize()
    per_k = []
    batches = {}
    for k_ in ks:
        evs = [step(k_) for _ in range(R)]
        torch.cuda.synchronize()
        batches[k_] = (sched.batch().tolist(), sched.phase_value())
        per_k.append({"k": "inf" if k_ in (0, K.KLPM_K_INFINITY) else int(k_),
                      "match_us": float(np.median([a.elapsed_time(b) for a, b, _ in evs])) * 1e3,
                      "select_us": float(np.median([b.elapsed_time(c) for _, b, c in evs])) * 1e3,
                      "schedule_latency_us": {"p50": pct([a.elapsed_time(c) * 1e3 for a, _, c in evs], 0.5),
                                              "max": float(max(a.elapsed_time(c) for a, _, c in evs)) * 1e3}})
    main_k = w.k if w.k in ks else ks[0]
    main = per_k[ks.index(main_k)]
    m_gpu = sched.match_len[:n0].cpu().numpy()
    sum_m = int(np.maximum(m_gpu, 0).sum())
    probe = MatchProbe(K, torch, dev)
    read_gbs = probe.stream_read_gbs()
    cold_ms = probe.match_ms(sched, q, args.cold_reps, cold=True)
    hot_ms = probe.match_ms(sched, q, args.cold_reps, cold=False)
    uniq = probe.unique_tree_tokens(sched, q, max_len)
    alg = algorithmic_bytes(sum_m, n0)
    compulsory = query_side_bytes(sum_m, n0) + 4 * uniq
    rec = recorded_traffic(w.name)
    traffic = rec["bytes_per_launch"] if rec else None
    traffic_cold = rec["bytes_per_cold_launch"] if rec else None
    step_ms = main["schedule_latency_us"]["p50"] * 1e-3
    assert K.kLPM_read_stats(sched.tree).device_error == 0
    out = {
        "metric": "prefix-match tokens/sec (single scheduling step: match + select)",
        "value": sum_m / (step_ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": R, "warmup": len(ks),
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": w.name, "cache_tokens": int(st.total_tokens), "tree_nodes": int(st.n_nodes),
                   "waiting_queries": n0, "batch": batch, "k": "inf" if main_k in (0, K.KLPM_K_INFINITY) else int(main_k),
                   "max_prompt_len": max_len, "queue_in_arrival_order": fifo},
        "schedule_latency_us": main["schedule_latency_us"],
        "k_sweep": per_k,
        "match_tokens_per_s_kernel": sum_m / (hot_ms * 1e-3),
        "matched_tokens_per_step": sum_m,
        "roofline": {"kernel": "k_match", "bound": "hbm", "achieved": alg / (hot_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": alg / (hot_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": traffic,
                     "achieved_is": "algorithmic bytes / kernel time of the launch repeated back to back on the same "
                                    "queue (inputs warm in the Infinity Cache as far as they fit); `cold` is the HBM figure",
                     "algorithmic_bytes_per_launch": alg, "kernel_ms": hot_ms,
                     "compulsory_bytes_per_launch": compulsory, "unique_tree_tokens": uniq,
                     "stream_read_GBps": read_gbs,
                     "cold": {"kernel_ms_cold": cold_ms, "algorithmic_GBps_cold": alg / (cold_ms * 1e-3) / 1e9,
                              "compulsory_GBps_cold": compulsory / (cold_ms * 1e-3) / 1e9,
                              "frac_cold": compulsory / (cold_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "traffic": traffic_cold,
                              "traffic_GBps": traffic_cold / (cold_ms * 1e-3) / 1e9 if traffic_cold else None,
                              "overread": (traffic_cold - compulsory) / compulsory if traffic_cold else None}},
        # queue-wide match launches in dispatch order, for reading a profiler's per-dispatch records
        "match_launches": [["warm-up", len(ks)], ["timed steps", R * len(ks)], ["cold: one untimed, then timed after a sweep", 1 + args.cold_reps],
                           ["back to back: one untimed, then timed", 1 + args.cold_reps]],
    }
    if args.cpu_steps > 0:
        import oracle

        cores = len(os.sched_getaffinity(0))
        threads = max(1, min(cores, 16))
        tree = oracle.OracleTree()
        tree.build(w.cache)
        sel_ms = []
        for i, k_ in enumerate(ks):
            m, idx, ph, t_m1, t_mt, t_sel, _ = oracle_split(tree, hq.tokens, hq.off, hq.len, hq.arrival, k_, batch, threads)
            assert (m == m_gpu).all(), "GPU and oracle disagree on the match lengths"
            assert (idx.tolist(), ph) == batches[k_], f"GPU and oracle disagree on the batch for k={k_}"
            sel_ms.append(t_sel * 1e3)
            if i == 0:
                t_1, t_all = t_m1, t_mt
        sel_main = sel_ms[ks.index(main_k)]
        out["cpu_baseline"] = {
            "value": sum_m / (t_all + sel_main * 1e-3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"the whole step once per k (match on {threads} threads, select serial); match lengths and every "
                      "batch of the sweep equal the GPU's",
            "ms_per_step": t_all * 1e3 + sel_main,
            "match_tokens_per_s_1thread": sum_m / t_1, "match_tokens_per_s_allcores": sum_m / t_all, "allcores": threads,
            "match_ms": t_all * 1e3, "select_ms": sel_main, "select_ms_by_k": sel_ms}
    print(json.dumps(out), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the workload (testing only)")
    ap.add_argument("--cpu-steps", type=int, default=25, help="oracle steps timed for the CPU baseline, at most the warm-up and timed steps (0 = skip)")
    ap.add_argument("--latency-steps", type=int, default=200,
                    help="steps of the separate pass that records the per-step latency distribution (0 = skip)")
    ap.add_argument("--cold-reps", type=int, default=10, help="match launches timed on cold caches (and as many back to back)")
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
    ap.add_argument("--workload", choices=("cfg2-large", "cfg0", "cfg1", "cfg3", "def3", "cfg4"), default="cfg2-large",
                    help="cfg0/cfg1/cfg3: the single-step configurations; def3: the timed Regular Arrival Shuffled "
                         "Queue run; cfg4: the 1,000-step online stream")
    ap.add_argument("--overload", action="store_true",
                    help="with --workload cfg4: a batch below the arrival rate (the queue backs up), k swept over {1,2,4,8,inf}, drained at the end")
    ap.add_argument("--overload-batch", type=int, default=96, help="batch size of --overload (arrivals are Poisson(128) per step)")
    ap.add_argument("--def3-u", type=int, default=3000, help="shared-prefix length of the def3 workload (prompt = 6000)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; --gpus must be 1 (there is no multi-GPU path to time)",
              file=sys.stderr)
        return 2

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload == "def3":
        return bench_def3(args)
    if args.workload == "cfg4":
        return bench_cfg4_overload(args) if args.overload else bench_cfg4(args)
    if args.workload in ("cfg0", "cfg1", "cfg3"):
        return bench_single_step(args)
    return bench_cfg2(args)


if __name__ == "__main__":
    sys.exit(main())
