"""CPU-only pins for the oracle: each test checks it against something other than itself
(the paper's printed example, closed forms from the proof of Thm. 2, brute-force models in
plain Python, textbook special cases)."""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as W
from helpers import PathModel, lcp, parse_snapshot, select_literal, snapshot_paths

K_INF = W.K_LPM_ENDPOINT


# ----------------------------------------------------------------------------- match
@pytest.mark.parametrize("seed", range(12))
def test_match_equals_bruteforce_pairwise_overlap(seed):
    w = W.random_small(seed, n_cache=14, n_query=30, vocab=3, max_len=9)
    tree = oracle.OracleTree()
    tree.build(w.cache)
    got = tree.match(w.queries.tokens, w.queries.off, w.queries.len)
    cached = w.cache.as_lists()
    want = [max(lcp(x, y) for y in cached) for x in w.queries.as_lists()]
    assert got.tolist() == want


def test_match_special_cases():
    w = W.config0()
    empty = oracle.OracleTree()
    assert not empty.match(w.queries.tokens, w.queries.off, w.queries.len).any()
    tree = oracle.OracleTree()
    tree.build(w.cache)
    # a cached prompt matches in full; a full match is legal (an identical prompt costs nothing, Sec. 3.1 proof)
    m = tree.match(w.cache.tokens, w.cache.off, w.cache.len)
    assert (m == w.cache.len).all()
    # idempotence: after committing the queries with no eviction each matches in full
    tree.commit(w.queries.tokens, w.queries.off, w.queries.len, np.arange(w.queries.n), 1 << 60)
    m2 = tree.match(w.queries.tokens, w.queries.off, w.queries.len)
    assert (m2 == w.queries.len).all()


def test_match_threads_agree():
    w = W.config0()
    tree = oracle.OracleTree()
    tree.build(w.cache)
    a = tree.match(w.queries.tokens, w.queries.off, w.queries.len)
    b = tree.match(w.queries.tokens, w.queries.off, w.queries.len, threads=5)
    assert (a == b).all()
    # group-derived queries see at least the 128-token group prefix, fresh ones (almost) nothing
    assert (a >= 128).mean() > 0.6 and (a <= 2).mean() > 0.15


# ----------------------------------------------------------------------------- select
def _rand_scores(rng, n):
    arrival = rng.integers(0, max(2, n // 2), size=n).astype(np.uint64)  # many ties
    m = rng.integers(0, 5, size=n).astype(np.int32)
    return arrival, m


@pytest.mark.parametrize("seed", range(10))
def test_select_equals_literal_loop(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    arrival, m = _rand_scores(rng, n)
    for k in (1, 2, 3, 4, 7, 1000, 0, K_INF):
        for batch in (1, 3, n, n + 5):
            for phase in (0, 1, 5):
                got, ph = oracle.select(arrival, m, k, batch, phase)
                want, wph = select_literal(arrival, m, k, batch, phase)
                assert got.tolist() == want and ph == wph


def test_select_endpoints_are_fcfs_and_lpm():
    rng = np.random.default_rng(99)
    n = 200
    arrival, m = _rand_scores(rng, n)
    idx = np.arange(n)
    fcfs = sorted(idx, key=lambda i: (int(arrival[i]), i))
    lpm = sorted(idx, key=lambda i: (-int(m[i]), int(arrival[i]), i))
    for batch in (1, 17, n):
        got, _ = oracle.select(arrival, m, 1, batch)
        assert got.tolist() == fcfs[:batch]  # k = 1 reduces to FCFS (Sec. 4)
        for kinf in (0, K_INF):
            got, ph = oracle.select(arrival, m, kinf, batch)
            assert got.tolist() == lpm[:batch] and ph == 0  # k = infinity reduces to LPM (Sec. 4)
        # a finite k >= batch with phase 0: the oldest query, then LPM order of the rest
        got, _ = oracle.select(arrival, m, 1000, batch)
        rest = [i for i in lpm if i != fcfs[0]]
        assert got.tolist() == ([fcfs[0]] + rest)[:batch]
        # the LPM endpoint maximises the summed match length of the batch
        best = np.sort(m)[::-1][:batch].sum()
        assert m[oracle.select(arrival, m, K_INF, batch)[0]].sum() == best


def test_select_slot_property_and_no_duplicates():
    rng = np.random.default_rng(5)
    n = 300
    arrival, m = _rand_scores(rng, n)
    for k in (2, 3, 8):
        for phase in (0, 1, k - 1):
            got, ph = oracle.select(arrival, m, k, 64, phase)
            assert len(set(got.tolist())) == 64
            assert ph == (phase + 64) % k
            left = set(range(n))
            for j, p in enumerate(got.tolist()):
                if (phase + j) % k == 0:
                    assert (int(arrival[p]), p) == min((int(arrival[i]), i) for i in left)
                else:
                    assert (-int(m[p]), int(arrival[p]), p) == min((-int(m[i]), int(arrival[i]), i) for i in left)
                left.remove(p)


def test_select_degenerate():
    got, ph = oracle.select(np.zeros(0, np.uint64), np.zeros(0, np.int32), 4, 8, 3)
    assert got.shape[0] == 0 and ph == 3
    got, ph = oracle.select(np.array([5], np.uint64), np.array([0], np.int32), 4, 0, 2)
    assert got.shape[0] == 0 and ph == 2


# ----------------------------------------------------------------------------- worked example
def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "toy_example.txt")
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, vals = line.split(":")
        out[key.strip()] = [int(v) for v in vals.split()]
    return out


def test_toy_example_def2_values():
    g = _golden()
    # spaced arrivals (s = 10): FCFS gives every query a TTFT of 10
    p = W.toy_example(10)
    order, _ = oracle.select(p.arrival, np.zeros(4, np.int32), 1, 4)
    ttft = oracle.def2_completion(p, order) - p.arrival.astype(np.float64)
    assert ttft.tolist() == g["s10_fcfs_ttft"]
    # burst (s = 0)
    p = W.toy_example(0)
    order, _ = oracle.select(p.arrival, np.zeros(4, np.int32), 1, 4)
    assert (order + 1).tolist() == g["s0_fcfs_order"]
    ttft = oracle.def2_completion(p, order)
    assert ttft.tolist() == g["s0_fcfs_ttft"] and ttft.max() == g["s0_fcfs_max"][0]
    # LPM with a last-prompt cache, through the radix-tree pipeline (one prompt of budget, batch 1)
    order = oracle.schedule_with_tree(p, K_INF, budget=10)
    assert (order + 1).tolist() == g["s0_lpm_order"]
    ttft = oracle.def2_completion(p, order)
    assert ttft[order].tolist() == g["s0_lpm_ttft_in_processing_order"] and ttft.max() == g["s0_lpm_max"][0]
    # k-LPM with k = 2 gives the same order here
    assert (oracle.schedule_with_tree(p, 2, budget=10) + 1).tolist() == g["s0_lpm_order"]
    # FCFS through the same pipeline
    assert (oracle.schedule_with_tree(p, 1, budget=10) + 1).tolist() == g["s0_fcfs_order"]


def test_def2_is_prefill_recurrence_with_attention_term():
    # two prompts "ab" and "abc" with c_attn = 0.5: R1 = 0 + (1+0.5*2)*2 = 4, R2 = max(4, 7) + (1+0.5*3)*(3-2) = 9.5
    p = W.generators._from_lists([[7, 8], [7, 8, 9]], [0, 7])
    r = oracle.def2_completion(p, [0, 1], c_attn=0.5)
    assert r.tolist() == [4.0, 9.5]
    # reversed order: R(abc) = 7 + 2.5*3 = 14.5, R(ab) = 14.5 + 2*(2-2) = 14.5
    r = oracle.def2_completion(p, [1, 0], c_attn=0.5)
    assert r.tolist() == [14.5, 14.5]


# ----------------------------------------------------------------------------- closed forms (proof of Thm. 2)
@pytest.mark.parametrize("seed,n,u,k,d,s", [(1, 12, 6, 3, 4, 2), (2, 20, 9, 4, 3, 1), (3, 16, 5, 2, 7, 3)])
def test_shuffled_queue_closed_forms(seed, n, u, k, d, s):
    p, user_of = W.shuffled_queue(n, u, k, d, s, seed=seed)
    T = s * n + 3  # processing starts once everything has arrived
    # LPM: the j-th processed query completes at T + ceil(j/k) u + d j
    order = oracle.schedule_with_tree(p, K_INF, budget=u + d)
    comp = oracle.def2_completion(p, order, t_start=T)
    for j, q in enumerate(order.tolist(), start=1):
        assert comp[q] == T + -(-j // k) * u + d * j
    # FCFS: the whole queue takes T + n(u+d) - u * sum_i I_i, I_i = same user as the previous arrival
    order = oracle.schedule_with_tree(p, 1, budget=u + d)
    assert order.tolist() == np.argsort(p.arrival, kind="stable").tolist()
    comp = oracle.def2_completion(p, order, t_start=T)
    same = sum(1 for a, b in zip(order[:-1], order[1:]) if user_of[a] == user_of[b])
    assert comp[order[-1]] == T + n * (u + d) - u * same
    # k-LPM with k = replication: every cycle consumes one whole user group, total n(u/k + d),
    # and max TTFT <= T + n(u/k + d - s/k) for any arrival order
    order = oracle.schedule_with_tree(p, k, budget=u + d)
    for c in range(n // k):
        assert len({int(user_of[q]) for q in order[c * k : (c + 1) * k]}) == 1
    comp = oracle.def2_completion(p, order, t_start=T)
    assert comp.max() == T + n * u // k + n * d
    ttft = comp - p.arrival.astype(np.float64)
    assert ttft.max() <= T + n * (u / k + d - s / k) + 1e-9


# ----------------------------------------------------------------------------- commit / evict
@pytest.mark.parametrize("seed", range(10))
def test_commit_and_evict_equal_path_model(seed):
    rng = np.random.default_rng(seed)
    w = W.random_small(seed + 100, n_cache=10, n_query=24, vocab=3, max_len=8)
    tree, model = oracle.OracleTree(), PathModel()
    tree.build(w.cache)
    model.commit(w.cache.as_lists(), 1 << 60)
    assert tree.snapshot() == model.snapshot()
    q = w.queries
    qs = q.as_lists()
    for step in range(4):
        batch = rng.choice(q.n, size=6, replace=False).astype(np.int32)
        budget = int(rng.integers(0, max(1, model.total())))
        before = tree.total_tokens
        st = tree.commit(q.tokens, q.off, q.len, batch, budget)
        model.commit([qs[i] for i in batch], budget)
        assert tree.snapshot() == model.snapshot()
        assert tree.match(q.tokens, q.off, q.len).tolist() == [model.match(x) for x in qs]
        # conservation and budget
        assert before + st.inserted_tokens - st.evicted_tokens == st.total_tokens == model.total()
        assert st.total_tokens <= budget


@pytest.mark.parametrize("seed", range(6))
def test_commit_statistics_equal_path_model(seed):
    """Every counter a commit reports (inserted / evicted tokens, new / evicted nodes, nodes, total, clock)
    recomputed from the dictionary-of-paths model: insertion and eviction (Sec. 1) applied one after the other
    there, node and token counts taken before, between and after."""
    rng = np.random.default_rng(300 + seed)
    w = W.random_small(seed + 500, n_cache=8, n_query=30, vocab=3, max_len=9)
    tree, model = oracle.OracleTree(), PathModel()
    st = tree.build(w.cache)
    for x in w.cache.as_lists():
        model.insert(x)
    assert (st.n_nodes, st.total_tokens, st.clock) == (len(model.nodes), model.total(), w.cache.n)
    assert (st.inserted_tokens, st.new_nodes, st.evicted_tokens, st.evicted_nodes) == (model.total(), len(model.nodes), 0, 0)
    q = w.queries
    qs = q.as_lists()
    for step in range(5):
        batch = rng.choice(q.n, size=int(rng.integers(1, 8)), replace=False).astype(np.int32)
        budget = int(rng.integers(0, model.total() + 10))
        nodes0, total0, clock0 = len(model.nodes), model.total(), model.clock
        for i in batch:
            model.insert(qs[i])
        nodes1, total1 = len(model.nodes), model.total()
        gone = model.evict(budget)
        st = tree.commit(q.tokens, q.off, q.len, batch, budget)
        assert st.inserted_tokens == total1 - total0 and st.new_nodes == nodes1 - nodes0, step
        assert st.evicted_tokens == total1 - model.total() and st.evicted_nodes == gone, step
        assert (st.n_nodes, st.total_tokens, st.clock) == (len(model.nodes), model.total(), clock0 + len(batch)), step
        assert tree.snapshot() == model.snapshot()


def test_commit_invariants_on_config0():
    w = W.config0()
    tree = oracle.OracleTree()
    st0 = tree.build(w.cache)
    n_nodes, total, clock, rec, tok = parse_snapshot(tree.snapshot())
    assert total == st0.total_tokens == int(rec["edge_len"].sum()) and clock == w.cache.n
    # token conservation against brute-force overlaps: each prompt adds its length minus its best overlap
    cached = w.cache.as_lists()
    want = 0
    for i, x in enumerate(cached):
        want += len(x) - max((lcp(x, y) for y in cached[:i]), default=0)
    assert total == want
    # radix property: siblings start with distinct tokens, no empty edge; ticks never increase downwards
    paths = snapshot_paths(tree.snapshot())
    assert all(len(p) > 0 for p in paths)
    by_parent = {}
    for p in paths:
        par = max((len(o) for o in paths if len(o) < len(p) and p[: len(o)] == o), default=0)
        by_parent.setdefault(p[:par], []).append(p[par])
        if par:
            assert paths[p[:par]] >= paths[p]
    assert all(len(v) == len(set(v)) for v in by_parent.values())
    # leaf ticks pairwise distinct
    leaves = [p for p in paths if not any(len(o) > len(p) and o[: len(p)] == p for o in paths)]
    assert len({paths[p] for p in leaves}) == len(leaves)


def test_structure_independent_of_insertion_order():
    w = W.random_small(4242, n_cache=16, n_query=4, vocab=3, max_len=9)
    rng = np.random.default_rng(0)
    ref = None
    for _ in range(5):
        perm = rng.permutation(w.cache.n).astype(np.int32)
        t = oracle.OracleTree()
        t.commit(w.cache.tokens, w.cache.off, w.cache.len, perm, 1 << 60)
        n_nodes, total, clock, rec, tok = parse_snapshot(t.snapshot())
        shape = (rec["depth_start"].tolist(), rec["edge_len"].tolist(), rec["n_children"].tolist(), tok.tolist())
        ref = ref or shape
        assert shape == ref


def test_split_at_prompt_end_either_order():
    a = W.generators._from_lists([[1, 2], [1, 2, 3]])
    for order in ([0, 1], [1, 0]):
        t = oracle.OracleTree()
        t.commit(a.tokens, a.off, a.len, np.array(order, np.int32), 1 << 60)
        n_nodes, total, clock, rec, tok = parse_snapshot(t.snapshot())
        assert n_nodes == 2 and total == 3 and rec["edge_len"].tolist() == [2, 1]


@pytest.mark.parametrize("seed", range(6))
def test_lru_equals_sorted_prefix_rule(seed):
    """Repeatedly removing the min-tick leaf == removing the shortest prefix of the nodes
    ordered by (tick ascending, depth descending) that brings the total within budget."""
    w = W.random_small(seed + 500, n_cache=30, n_query=2, vocab=3, max_len=10)
    tree = oracle.OracleTree()
    tree.build(w.cache)
    paths = snapshot_paths(tree.snapshot())
    total = tree.total_tokens
    budget = total // 2

    def edge_len(p):
        return len(p) - max((len(o) for o in paths if len(o) < len(p) and p[: len(o)] == o), default=0)

    order = sorted(paths, key=lambda p: (paths[p], -len(p)))
    survivors = dict(paths)
    remaining = total
    for p in order:
        if remaining <= budget:
            break
        remaining -= edge_len(p)
        del survivors[p]
    st = tree.commit(w.cache.tokens, w.cache.off, w.cache.len, np.zeros(0, np.int32), budget)
    assert st.total_tokens == remaining <= budget
    assert snapshot_paths(tree.snapshot()) == survivors


# ----------------------------------------------------------------------------- stream glue
def test_stream_simulation_bookkeeping():
    s = W.config4_stream(steps=25, rate=12, groups=300, budget=60_000, batch=16)
    r = oracle.simulate_stream(s, snapshot_every=5)
    n = s.queries.n
    seen = np.concatenate(r.batches)
    assert len(set(seen.tolist())) == seen.shape[0]
    assert all(st.total_tokens <= s.budget for st in r.stats)
    assert all(len(b) <= s.batch for b in r.batches)
    admitted = r.ttft >= 0
    assert admitted.sum() == seen.shape[0] and (r.ttft[admitted] >= 1).all()
    # a query is never admitted before the step it arrives in
    step_of = np.searchsorted(s.step_start, np.arange(n), side="right") - 1
    assert (r.admitted_step[admitted] >= step_of[admitted]).all()
    # the simulated clock is the sum of per-step costs, each at least 1
    assert r.clock >= s.steps
    assert oracle.percentile_nearest_rank([5, 1, 3, 2, 4], 0.5) == 3
    assert oracle.percentile_nearest_rank(np.arange(1, 101), 0.99) == 99


def test_stream_fcfs_admits_in_arrival_order():
    s = W.config4_stream(steps=20, rate=20, groups=100, budget=50_000, batch=8)
    s.k = 1
    r = oracle.simulate_stream(s)
    flat = np.concatenate(r.batches)
    assert (np.diff(flat) > 0).all()  # global ids are in arrival order, FCFS must preserve it


def _toy_stream(k):
    """The four queries of the worked example of Sec. 4.2 as an online stream: all of them arrive in
    step 0 (the s = 0 case), one query per bin, a cache of one prompt (Def. 2's last-prompt cache)."""
    p = W.toy_example(0)
    return W.generators.Stream("toy", p, np.array([0, 4, 4, 4, 4], dtype=np.int64), k, 1, 10)


@pytest.mark.parametrize("k", (1, 2, K_INF))
def test_stream_clock_and_ttft_on_the_worked_example(k):
    """Sec. 4.2 prints the per-query TTFT of the burst case: FCFS 10, 20, 30, 40 in arrival order;
    LPM processes x1, x3, x2, x4 and they finish after 10, 15, 25, 30 (k-LPM with k = 2 takes the
    same order).  With every enqueue time 0 the TTFT is the clock at which the query's bin ends, so
    these values pin cost = sum(|x| - m), the running clock and TTFT = finish - enqueue."""
    g = _golden()
    r = oracle.simulate_stream(_toy_stream(k))
    order = [int(b[0]) + 1 for b in r.batches]
    if k == 1:
        assert order == g["s0_fcfs_order"]
        assert r.ttft.tolist() == g["s0_fcfs_ttft"] and r.clock == g["s0_fcfs_max"][0]
    else:
        assert order == g["s0_lpm_order"]
        assert [int(r.ttft[i - 1]) for i in order] == g["s0_lpm_ttft_in_processing_order"]
        assert r.clock == g["s0_lpm_max"][0]
    assert all(len(b) == 1 for b in r.batches)


@pytest.mark.parametrize("k,batch", ((4, 16), (1, 8), (K_INF, 5)))
def test_stream_clock_and_ttft_recomputed_step_by_step(k, batch):
    """Def. 2 with c_attn = 0 charges a query its uncached tokens; the queries of a bin finish
    together (Sec. 2.1); a bin that costs nothing still takes one unit of time.  Every step's cost,
    the clock and every TTFT are recomputed here from the recorded batches and match lengths with
    plain Python integers, and the enqueue times from the clock at the start of the arrival step."""
    s = W.config4_stream(steps=30, rate=14, groups=40, budget=40_000, batch=batch)
    s.k = k
    r = oracle.simulate_stream(s)
    lens = s.queries.len.tolist()
    clock, want, enq = 0, {}, {}
    zero_cost_steps = 0
    for step in range(s.steps):
        for gid in range(int(s.step_start[step]), int(s.step_start[step + 1])):
            enq[gid] = clock
        pos = {int(g): i for i, g in enumerate(r.waiting_ids[step].tolist())}
        m = r.match_lens[step].tolist()
        cost = 0
        for gid in r.batches[step].tolist():
            assert gid in enq and gid not in want  # waiting, not served before
            cost += lens[gid] - m[pos[gid]]
        zero_cost_steps += cost == 0
        clock += cost if cost > 0 else 1
        for gid in r.batches[step].tolist():
            want[gid] = clock - enq[gid]
    assert r.clock == clock
    got = {i: int(t) for i, t in enumerate(r.ttft.tolist()) if t >= 0}
    assert got == want
    # the stream reuses prefixes (some cost is saved) and some prompts cost their full length
    full = sum(lens[g] for b in r.batches for g in b.tolist())
    assert 0 < clock - zero_cost_steps < full


def test_stream_bin_that_costs_nothing_takes_one_time_unit():
    """An identical prompt costs nothing (Sec. 3.1); the simulated clock still moves by one."""
    p = W.generators._from_lists([[1, 2, 3], [1, 2, 3], [1, 2, 3, 4]], [0, 0, 0])
    s = W.generators.Stream("dup", p, np.array([0, 3, 3, 3], dtype=np.int64), 1, 1, 100)
    r = oracle.simulate_stream(s)
    assert r.ttft.tolist() == [3, 4, 5] and r.clock == 5


def test_stream_backlog_and_an_empty_stream():
    """Queries still waiting when the stream ends keep TTFT -1 and admission step -1; a stream that never
    steps ends at time 0."""
    p = W.generators._from_lists([[1, 2], [3, 4, 5], [6], [7, 8, 9, 10]], [0, 0, 0, 0])
    s = W.generators.Stream("backlog", p, np.array([0, 4, 4], dtype=np.int64), 1, 1, 100)  # two steps, one pick each
    r = oracle.simulate_stream(s)
    assert r.ttft.tolist() == [2, 5, -1, -1] and r.admitted_step.tolist() == [0, 1, -1, -1] and r.clock == 5
    empty = W.generators.Stream("none", p, np.array([0], dtype=np.int64), 1, 1, 100)
    r = oracle.simulate_stream(empty)
    assert r.clock == 0 and r.ttft.tolist() == [-1] * 4 and r.batches == []


def test_percentile_is_nearest_rank():
    """sorted[ceil(p n) - 1], ranks counted from one; the smallest element for every p <= 1/n."""
    v = [40, 10, 30, 20]
    assert [oracle.percentile_nearest_rank(v, p) for p in (0.0, 0.01, 0.25, 0.26, 0.5, 0.51, 0.75, 0.76, 0.99, 1.0)] == [
        10, 10, 10, 20, 20, 30, 30, 40, 40, 40]
    assert oracle.percentile_nearest_rank([7, 5], 0.5) == 5 and oracle.percentile_nearest_rank([7], 0.99) == 7
    assert oracle.percentile_nearest_rank([], 0.5) == 0
    rng = np.random.default_rng(3)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        x = rng.integers(0, 100, size=n)
        p_ = float(rng.random())
        # definition: the smallest value with at least a fraction p of the sample at or below it
        want = min(int(t) for t in x if (x <= t).sum() >= p_ * n)
        assert oracle.percentile_nearest_rank(x, p_) == want


# ----------------------------------------------------------------------------- timed arrivals (Def. 2 timeline)
def test_timed_toy_example_values():
    g = _golden()
    # arrivals every 10 (s = 10): each query is done before the next one arrives, whatever k is
    for k in (1, 2, K_INF):
        r = oracle.simulate_timed(W.toy_example(10), k, batch=1, budget=10)
        assert r.ttft.tolist() == g["s10_fcfs_ttft"]
    # burst (s = 0), processing starts at 0
    r = oracle.simulate_timed(W.toy_example(0), 1, batch=1, budget=10)
    assert (r.order + 1).tolist() == g["s0_fcfs_order"] and r.ttft.tolist() == g["s0_fcfs_ttft"]
    for k in (2, K_INF):
        r = oracle.simulate_timed(W.toy_example(0), k, batch=1, budget=10)
        assert (r.order + 1).tolist() == g["s0_lpm_order"]
        assert r.ttft[r.order].tolist() == g["s0_lpm_ttft_in_processing_order"]
        assert r.clock == g["s0_lpm_max"][0]


@pytest.mark.parametrize("seed,n,u,rep,d", [(1, 24, 6, 3, 4), (2, 40, 9, 4, 3), (3, 32, 5, 2, 7)])
@pytest.mark.parametrize("c_num,c_den", [(0, 1), (3, 64)])
def test_timed_run_equals_def2_recurrence(seed, n, u, rep, d, c_num, c_den):
    """Batch 1 with one prompt of cache: arrival + TTFT must be Def. 2's R(.) of the order taken,
    evaluated by the stand-alone recurrence (pairwise overlap with the previous prompt)."""
    for s in (0, 1, (u + d) // 2, 3 * (u + d)):
        p, _ = W.shuffled_queue(n, u, rep, d, s, seed=seed)
        p.arrival[:] = p.arrival * np.uint64(c_den)
        for k in (1, rep, K_INF):
            r = oracle.simulate_timed(p, k, batch=1, budget=u + d, c_num=c_num, c_den=c_den)
            assert sorted(r.order.tolist()) == list(range(n))
            # the recurrence works in token times: rescale arrivals, then scale its result back
            q = W.Prompts(p.tokens, p.off, p.len, p.arrival // np.uint64(c_den))
            comp = oracle.def2_completion(q, r.order, c_attn=c_num / c_den) * c_den
            assert (r.ttft + p.arrival.astype(np.int64)).tolist() == comp.tolist()
            # nothing is processed before it arrives, nor scheduled while it was not there
            start = r.ttft + p.arrival.astype(np.int64)
            assert (r.ttft >= 0).all() and r.clock == start.max()


def test_timed_slow_arrivals_are_served_on_arrival():
    n, u, rep, d, c_num, c_den = 20, 7, 4, 5, 1, 16
    x = u + d
    s = x * (c_den + c_num * x) // c_den + 1  # longer than any processing time
    p, user_of = W.shuffled_queue(n, u, rep, d, s, seed=5)
    p.arrival[:] = p.arrival * np.uint64(c_den)
    by_arrival = np.argsort(p.arrival, kind="stable")
    for k in (1, 2, K_INF):
        r = oracle.simulate_timed(p, k, batch=1, budget=x, c_num=c_num, c_den=c_den)
        assert r.order.tolist() == by_arrival.tolist() and r.steps == n
        prev_same = np.zeros(n, dtype=bool)
        prev_same[by_arrival[1:]] = user_of[by_arrival[1:]] == user_of[by_arrival[:-1]]
        want = (x - u * prev_same) * (c_den + c_num * x)
        assert r.ttft.tolist() == want.tolist()


@pytest.mark.parametrize("seed,n,u,rep,d,s", [(1, 12, 6, 3, 4, 2), (2, 20, 9, 4, 3, 1)])
def test_timed_run_after_all_arrived_meets_closed_forms(seed, n, u, rep, d, s):
    p, user_of = W.shuffled_queue(n, u, rep, d, s, seed=seed)
    T = s * n + 3
    r = oracle.simulate_timed(p, K_INF, batch=1, budget=u + d, t_start=T)
    done = r.ttft + p.arrival.astype(np.int64)
    for j, q in enumerate(r.order.tolist(), start=1):
        assert done[q] == T + -(-j // rep) * u + d * j  # j-th completion under LPM (proof of Thm. 2)
    r = oracle.simulate_timed(p, rep, batch=1, budget=u + d, t_start=T)
    assert r.clock == T + n * u // rep + n * d
    assert r.ttft.max() <= T + n * (u / rep + d - s / rep) + 1e-9


@pytest.mark.parametrize("s", [400, 1500, 2600])
def test_timed_run_meets_the_separation_theorem_at_the_paper_shape(s):
    """Thm. 2 with c_attn = 0 on a Def. 3 queue at the shape of the paper's table (n = 2000, k = 4,
    u = d = 3000), processing from T = s n on, LPM with random ties: the k-LPM bound holds exactly,
    the LPM and FCFS lower bounds hold up to their (1 - eps), and for 0 < s < u k-LPM has the lowest
    maximum TTFT (Corollary 1)."""
    n, rep, u, d = 2000, 4, 3000, 3000
    p, _ = W.shuffled_queue(n, u, rep, d, s, seed=21)
    T = s * n
    worst = {}
    for k in (1, rep, K_INF):
        r = oracle.simulate_timed(p, k, batch=1, budget=u + d, t_start=T, tie_seed=4)
        worst[k] = int(r.ttft.max())
    assert worst[rep] <= T + n * (u // rep + d) - n * s // rep
    assert worst[K_INF] >= 0.97 * (T + n * (u // rep + d))
    assert worst[1] >= 0.97 * (T + n * (u + d - s))
    assert worst[rep] < worst[K_INF] and worst[rep] < worst[1]


def test_timed_random_ties_follow_the_keys():
    """With a tie seed, a step's longest-match pick among equal match lengths is the query with the
    smallest key of that step, whatever its arrival; without one it is the earliest arrival."""
    n, u, rep, d = 12, 5, 3, 4
    p, _ = W.shuffled_queue(n, u, rep, d, 1, seed=3)
    r = oracle.simulate_timed(p, K_INF, batch=1, budget=u + d, t_start=n, tie_seed=9)  # everybody waits from the start
    r0 = oracle.simulate_timed(p, K_INF, batch=1, budget=u + d, t_start=n)
    assert sorted(r.order.tolist()) == list(range(n)) and r.clock == r0.clock  # same reuse, other order
    for step in range(n):
        w, m = r.waiting_ids[step], r.match_lens[step]
        best = np.flatnonzero(m == m.max())
        keys = oracle.tie_keys(9, step, w)[best]
        assert int(r.batches[step][0]) == int(w[best[np.argmin(keys)]])
        w0, m0 = r0.waiting_ids[step], r0.match_lens[step]
        best0 = np.flatnonzero(m0 == m0.max())
        assert int(r0.batches[step][0]) == int(w0[best0[np.argmin(p.arrival[w0[best0]])]])


def test_timed_bounded_queue_keeps_everyone_and_fcfs_order():
    p, _ = W.shuffled_queue(24, 6, 3, 4, 1, seed=9)
    full = oracle.simulate_timed(p, 1, batch=2, budget=40)
    small = oracle.simulate_timed(p, 1, batch=2, budget=40, queue_cap=3)
    assert full.order.tolist() == small.order.tolist() == np.argsort(p.arrival, kind="stable").tolist()
    r = oracle.simulate_timed(p, K_INF, batch=2, budget=40, queue_cap=3)
    assert sorted(r.order.tolist()) == list(range(24)) and all(len(w) <= 3 for w in r.waiting_ids)
    # a batch of B finishes together: both members of a step get the same completion time
    done = r.ttft + p.arrival.astype(np.int64)
    for b in r.batches:
        assert len(set(done[b].tolist())) == 1


# ----------------------------------------------------------------------------- score and tie variants
def test_philox_known_answers():
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [[int(v, 16) for v in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        assert list(oracle.philox4x32_10(r[0:4], r[4:6])) == r[6:10]
    # the array form used for tie keys runs the same rounds
    rng = np.random.default_rng(3)
    ids = rng.integers(0, 2**31, size=50)
    for seed, step in ((0, 0), (rows[2][4] | (rows[2][5] << 32), 12345678901234)):
        want = [oracle.philox4x32_10((int(i), 0, step & 0xFFFFFFFF, step >> 32), (seed & 0xFFFFFFFF, seed >> 32))[0]
                for i in ids]
        assert oracle.tie_keys(seed, step, ids).tolist() == want
    # a tie key is word 0 at counter (id, 0, step lo, step hi) under key (seed lo, seed hi)
    assert oracle.tie_keys(0, 0, [0])[0] == rows[0][6]
    seed, step = (0x299F31D0 << 32) | 0xA4093822, (0x03707344 << 32) | 0x13198A2E
    assert oracle.philox4x32_10((0x243F6A88, 0, step & 0xFFFFFFFF, step >> 32), (seed & 0xFFFFFFFF, seed >> 32))[0] == \
        oracle.tie_keys(seed, step, [0x243F6A88])[0]


@pytest.mark.parametrize("seed", range(12))
def test_select_with_tie_keys_equals_literal_loop(seed):
    rng = np.random.default_rng(500 + seed)
    n = int(rng.integers(1, 60))
    arrival, m = _rand_scores(rng, n)
    tie = rng.integers(0, 4, size=n).astype(np.uint32) if seed % 2 else oracle.tie_keys(seed, 3, np.arange(n))
    for k in (1, 2, 3, 5, K_INF):
        for batch in (1, n // 2 + 1, n + 3):
            got, ph = oracle.select(arrival, m, k, batch, phase=seed % 3, tie_key=tie)
            want, ph_want = select_literal(arrival, m, k, batch, seed % 3, tie_key=tie)
            assert got.tolist() == want and ph == ph_want
    # a constant tie key changes nothing; oldest picks never look at it
    base, _ = oracle.select(arrival, m, 3, n, 0)
    same, _ = oracle.select(arrival, m, 3, n, 0, tie_key=np.full(n, 77, np.uint32))
    assert base.tolist() == same.tolist()
    fcfs, _ = oracle.select(arrival, m, 1, n, 0, tie_key=tie)
    assert fcfs.tolist() == np.lexsort((np.arange(n), arrival)).tolist()


def test_random_tie_break_is_uniform_over_the_tied_queries():
    """Footnote of Sec. 4.2: ties are broken uniformly at random.  Eight queries share the top
    score; over 4,000 scheduling steps each must be picked first about 500 times, and the order of
    the first two picks must cover all 56 ordered pairs about evenly."""
    n, steps = 12, 4000
    m = np.array([9] * 8 + [1, 2, 3, 4], np.int32)
    arrival = np.arange(n, dtype=np.uint64)
    first = np.zeros(8, np.int64)
    pairs = np.zeros((8, 8), np.int64)
    for step in range(steps):
        got, _ = oracle.select(arrival, m, K_INF, 2, 0, tie_key=oracle.tie_keys(20250204677, step, np.arange(n)))
        assert got[0] < 8 and got[1] < 8
        first[got[0]] += 1
        pairs[got[0], got[1]] += 1
    chi2 = float(((first - steps / 8) ** 2 / (steps / 8)).sum())
    assert chi2 < 24.3  # 7 degrees of freedom, p = 0.001
    off = pairs[~np.eye(8, dtype=bool)]
    chi2 = float(((off - steps / 56) ** 2 / (steps / 56)).sum())
    assert chi2 < 93.2  # 55 degrees of freedom, p = 0.001
    # without tie keys the earliest of the tied queries always wins
    got, _ = oracle.select(arrival, m, K_INF, 2, 0)
    assert got.tolist() == [0, 1]


def test_hit_rate_score_orders_like_the_exact_ratio():
    from fractions import Fraction

    rng = np.random.default_rng(77)
    ln = rng.integers(1, 1 << 15, size=400)
    m = (rng.random(400) * (ln + 1)).astype(np.int64).clip(0, ln)
    m[:20], m[20:40] = 0, ln[20:40]
    sc = oracle.score_hit_rate(m, ln, 30)
    assert (sc[:20] == 0).all() and (sc[20:40] == 1 << 30).all()
    fr = [Fraction(int(a), int(b)) for a, b in zip(m, ln)]
    for i in range(400):
        for j in range(i + 1, 400, 7):
            assert (sc[i] < sc[j]) == (fr[i] < fr[j]) and (sc[i] == sc[j]) == (fr[i] == fr[j])
    # equal prompt lengths (the setting of the paper's theory): the rate orders like the match length
    ln_eq = np.full(50, 1000)
    m_eq = rng.integers(0, 1001, size=50)
    arrival = rng.integers(0, 5, size=50).astype(np.uint64)
    a, _ = oracle.select(arrival, m_eq.astype(np.int32), 3, 50, 0)
    b, _ = oracle.select(arrival, oracle.score_hit_rate(m_eq, ln_eq, 20), 3, 50, 0)
    assert a.tolist() == b.tolist()
    # and where lengths differ the two keys disagree: a short prompt cached in full beats a long half-cached one
    a, _ = oracle.select(np.zeros(2, np.uint64), np.array([500, 40], np.int32), K_INF, 1, 0)
    b, _ = oracle.select(np.zeros(2, np.uint64), oracle.score_hit_rate([500, 40], [1000, 40]), K_INF, 1, 0)
    assert a.tolist() == [0] and b.tolist() == [1]


# ----------------------------------------------------------------------------- in-batch rescoring
def _dynamic_literal(p, arrival, m, k, batch, phase):
    """Literal form on Python lists: pick by the current scores, then raise the others' scores to
    their common prefix with the picked prompt."""
    inf = k in (0, K_INF)
    toks = [p.tokens[int(o): int(o) + int(l)].tolist() for o, l in zip(p.off, p.len)]
    score = [int(v) for v in m]
    remaining = list(range(p.n))
    out = []
    ph = 0 if inf else phase % k
    for j in range(min(batch, p.n)):
        if not inf and (ph + j) % k == 0:
            pick = min(remaining, key=lambda i: (int(arrival[i]), i))
        else:
            pick = min(remaining, key=lambda i: (-score[i], int(arrival[i]), i))
        out.append(pick)
        remaining.remove(pick)
        for i in remaining:
            score[i] = max(score[i], lcp(toks[i], toks[pick]))
    return out, (0 if inf else (ph + len(out)) % k), score


@pytest.mark.parametrize("seed", range(10))
def test_dynamic_select_equals_literal_and_sequential_steps(seed):
    w = W.random_small(seed + 300, n_cache=8, n_query=30, vocab=3, max_len=9)
    q = w.queries
    tree = oracle.OracleTree()
    tree.build(w.cache)
    m = tree.match(q.tokens, q.off, q.len)
    for k in (1, 2, 3, K_INF):
        for batch in (1, 7, q.n):
            got, ph, sc = oracle.select_dynamic(q.tokens, q.off, q.len, q.arrival, m, k, batch, phase=1)
            want, ph_want, sc_want = _dynamic_literal(q, q.arrival, m, k, batch, 1)
            assert got.tolist() == want and ph == ph_want and sc.tolist() == sc_want
            if batch == 1:  # one pick: nothing to rescore
                st, _ = oracle.select(q.arrival, m, k, 1, 1)
                assert got.tolist() == st.tolist()
    # one bin with rescoring == the same number of single-query steps through the tree without
    # eviction (each step matches against cache + everything processed so far)
    for k in (2, 3, K_INF):
        got, _, sc = oracle.select_dynamic(q.tokens, q.off, q.len, q.arrival, m, k, q.n, phase=0)
        t2 = oracle.OracleTree()
        t2.build(w.cache)
        waiting, phase, order, at_pick = np.arange(q.n), 0, [], []
        while waiting.shape[0]:
            mm = t2.match(q.tokens, q.off[waiting], q.len[waiting])
            idx, phase = oracle.select(q.arrival[waiting], mm, k, 1, phase)
            t2.commit(q.tokens, q.off[waiting], q.len[waiting], idx, 1 << 60)
            order.append(int(waiting[idx[0]]))
            at_pick.append(int(mm[idx[0]]))
            waiting = np.delete(waiting, idx[0])
        assert got.tolist() == order and sc[got].tolist() == at_pick


def test_dynamic_select_reproduces_the_worked_example_in_one_bin():
    """Sec. 4.2's example with an empty cache and all four queries in one bin: static scores are all
    zero (arrival order), rescoring gives the LPM order x1, x3, x2, x4 and the overlaps 0, 5, 0, 5
    that make up the printed TTFTs 10, 15, 25, 30."""
    g = _golden()
    p = W.toy_example(0)
    zero = np.zeros(4, np.int32)
    static, _ = oracle.select(p.arrival, zero, K_INF, 4)
    assert (static + 1).tolist() == g["s0_fcfs_order"]
    for k in (2, K_INF):
        got, _, sc = oracle.select_dynamic(p.tokens, p.off, p.len, p.arrival, zero, k, 4)
        assert (got + 1).tolist() == g["s0_lpm_order"]
        cost = p.len[got] - sc[got]
        assert np.cumsum(cost).tolist() == g["s0_lpm_ttft_in_processing_order"]
    got, _, sc = oracle.select_dynamic(p.tokens, p.off, p.len, p.arrival, zero, 1, 4)
    # FCFS order; a cache that keeps all of the bin's prompts (not only the last one, as Def. 2's
    # model does when it prints 30 and 40) still holds x1 when x3 comes, and x2 when x4 comes
    assert (got + 1).tolist() == g["s0_fcfs_order"] and np.cumsum(p.len[got] - sc[got]).tolist() == [10, 20, 25, 30]


# ----------------------------------------------------------------------------- serving-side variants
@pytest.mark.parametrize("seed", range(8))
def test_eviction_protects_prompts_in_flight(seed):
    rng = np.random.default_rng(900 + seed)
    w = W.random_small(seed + 700, n_cache=10, n_query=30, vocab=3, max_len=8)
    tree, model = oracle.OracleTree(), PathModel()
    tree.build(w.cache)
    model.commit([w.cache.tokens[int(o): int(o) + int(l)] for o, l in zip(w.cache.off, w.cache.len)], 1 << 60)
    q = w.queries
    history = []
    for step in range(5):
        idx = rng.choice(q.n, size=4, replace=False).astype(np.int32)
        budget, protect = int(rng.integers(0, 25)), int(rng.integers(0, 7))
        st = tree.commit(q.tokens, q.off, q.len, idx, budget, protect=protect)
        xs = [q.tokens[int(q.off[i]): int(q.off[i]) + int(q.len[i])].tolist() for i in idx]
        model.commit(xs, budget, protect)
        assert tree.snapshot() == model.snapshot()
        history.extend(xs)
        # whatever the budget, the last `protect` admitted prompts are still cached in full
        for x in history[len(history) - protect:] if protect else []:
            arr = np.array(x, np.int32)
            assert tree.match(arr, np.zeros(1, np.int64), np.array([len(x)], np.int32))[0] == len(x)
        # and eviction went as far as it could: either within budget, or nothing unprotected is left
        if st.total_tokens > budget:
            rec = parse_snapshot(tree.snapshot())[3]
            assert protect > 0 and all(int(t) >= st.clock - protect for t in rec["tick"])
    # protect = 0 is the plain rule
    a, b = oracle.OracleTree(), oracle.OracleTree()
    a.build(w.cache), b.build(w.cache)
    idx = np.arange(6, dtype=np.int32)
    a.commit(q.tokens, q.off, q.len, idx, 12)
    b.commit(q.tokens, q.off, q.len, idx, 12, protect=0)
    assert a.snapshot() == b.snapshot()


def test_eviction_protection_edge_windows():
    """Protection windows of one prompt, of exactly and of more than all admitted prompts, under a budget of
    zero: the window is the last `protect` ticks (ticks >= clock - protect), tick 0 included when the
    window reaches back that far."""
    # three prompts that share nothing: each is one leaf stamped with its own tick 0, 1, 2
    toks = np.array([1, 1, 1, 2, 2, 3, 3, 3, 3], np.int32)
    off, ln = np.array([0, 3, 5], np.int64), np.array([3, 2, 4], np.int32)
    def after(protect):
        t = oracle.OracleTree()
        st = t.commit(toks, off, ln, np.arange(3, dtype=np.int32), 0, protect=protect)
        return sorted(snapshot_paths(t.snapshot()).items()), st
    paths, st = after(1)
    assert paths == [((3, 3, 3, 3), 2)] and (st.evicted_nodes, st.evicted_tokens, st.total_tokens) == (2, 5, 4)
    paths, st = after(2)
    assert paths == [((2, 2), 1), ((3, 3, 3, 3), 2)] and st.evicted_nodes == 1
    for protect in (3, 4, 1000):  # the window covers every admitted prompt, the one with tick 0 too
        paths, st = after(protect)
        assert paths == [((1, 1, 1), 0), ((2, 2), 1), ((3, 3, 3, 3), 2)] and st.evicted_nodes == 0 and st.total_tokens == 9
    paths, st = after(0)
    assert paths == [] and (st.evicted_nodes, st.evicted_tokens, st.total_tokens, st.n_nodes) == (3, 9, 0, 0)


def test_token_budget_cut_and_phase():
    ln = np.array([10, 4, 7, 3, 9], np.int32)
    m = np.array([2, 4, 0, 1, 9], np.int32)   # costs 8, 0, 7, 2, 0
    order = np.array([0, 1, 2, 3, 4])
    assert [oracle.token_budget_cut(order, ln, m, b) for b in (0, 7, 8, 14, 15, 16, 17, 100)] == [1, 1, 2, 2, 3, 3, 5, 5]
    assert oracle.token_budget_cut(order[::-1], ln, m, 0) == 1  # pick 4 is free, pick 3 already overflows
    assert oracle.token_budget_cut(np.array([4, 1, 3]), ln, m, 0) == 2  # free picks ride along until something costs
    assert oracle.token_budget_cut(np.zeros(0, np.int64), ln, m, 5) == 0
    # brute force: the kept count is the largest prefix (of at least one pick) within the budget
    rng = np.random.default_rng(4)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        ln = rng.integers(1, 30, size=n)
        m = (rng.random(n) * (ln + 1)).astype(np.int64).clip(0, ln)
        order = rng.permutation(n)
        b = int(rng.integers(0, 80))
        cost = np.cumsum((ln - m)[order])
        want = max(1, int((cost <= b).sum()) if (np.diff((cost <= b).astype(int)) <= 0).all() else 0)
        assert oracle.token_budget_cut(order, ln, m, b) == want
    # handing picks back rewinds the k-cycle: selecting n_kept in the first place gives the same phase
    arrival = np.arange(20, dtype=np.uint64)
    mm = rng.integers(0, 9, size=20).astype(np.int32)
    for k in (1, 2, 3, 7, 0, K_INF):
        for phase in (0, 1, 5):
            full, ph_full = oracle.select(arrival, mm, k, 12, phase)
            for kept in (1, 5, 12):
                part, ph_part = oracle.select(arrival, mm, k, kept, phase)
                assert part.tolist() == full[:kept].tolist()
                assert oracle.phase_after_cut(ph_full, 12, kept, k) == ph_part


# ----------------------------------------------------------------------------- adaptive k (epsilon-greedy over a list of k values)
def _feed(ad, costs, window=None):
    """One pull per entry of `costs`: `window` steps, the cost carried by one admitted query."""
    arms = []
    for c in costs:
        arms.append(ad.arm)
        for i in range(ad.window):
            ad.observe([c] if i == ad.window // 2 else [])
    return arms


def test_adaptive_k_starts_round_robin_and_holds_an_arm_for_a_window():
    ad = oracle.AdaptiveK([1, 4, K_INF], window=5, explore=0, seed=1)
    ks = []
    for step in range(15):
        ks.append(ad.k())
        ad.observe([100 + step])
    assert ks == [1] * 5 + [4] * 5 + [K_INF] * 5
    assert ad.count == [1, 1, 1] and ad.cost == [104, 109, 114]  # the largest TTFT of each window


def test_adaptive_k_window_maximum_starts_from_zero_and_draws_follow_the_stated_words():
    # a window whose admitted queries all had TTFT 0 is a pull of cost 0 (the maximum starts from zero in
    # every window, it is not carried over and has no floor)
    ad = oracle.AdaptiveK([2, 8], window=2, explore=0, seed=3)
    ad.observe([7]); ad.observe([])          # arm 0: cost 7
    ad.observe([0, 0]); ad.observe([0])      # arm 1: cost 0
    assert ad.count == [1, 1] and ad.cost == [7, 0] and ad.arm == 1
    # the exploring draw: word 0 of Philox-4x32-10 at counter (pulls, 0, tag, 0) against `explore`, word 1
    # picks the arm - recomputed here from the known-answer-pinned generator for a run that always explores
    # and one that explores about half the time
    for explore in (1 << 32, 1 << 31):
        ad = oracle.AdaptiveK([1, 2, 4, 8, 16], window=1, explore=explore, seed=0x1234_5678_9ABC)
        costs = [50, 10, 40, 30, 20]
        for c in costs:
            ad.observe([c])                  # round robin first
        for pull in range(5, 60):
            w = oracle.philox4x32_10((pull, 0, oracle.ADAPT_TAG, 0), (0x5678_9ABC, 0x1234))
            mean = [ad.cost[a] / ad.count[a] for a in range(5)]
            want = w[1] % 5 if w[0] < explore else mean.index(min(mean))
            assert ad.arm == want, (explore, pull)
            ad.observe([costs[ad.arm]])      # every arm keeps its mean


def test_adaptive_k_greedy_is_the_exact_argmin_of_the_mean_cost():
    from fractions import Fraction

    rng = np.random.default_rng(5)
    for trial in range(20):
        A = int(rng.integers(2, 7))
        ad = oracle.AdaptiveK(list(range(1, A + 1)), window=int(rng.integers(1, 4)), explore=0, seed=trial)
        hist = [[] for _ in range(A)]
        for pull in range(60):
            arm = ad.arm
            if pull >= A:  # after the first round: what a table of per-arm cost lists says
                means = [Fraction(sum(h), len(h)) for h in hist]
                assert arm == min(range(A), key=lambda a: (means[a], a))
            c = int(rng.integers(0, 6)) * (1 << int(rng.integers(0, 45)))
            _feed(ad, [c])
            hist[arm].append(c)
    # equal means with different counts: 6/2 against 3/1 -> the lower index
    ad = oracle.AdaptiveK([7, 9], window=1, explore=0, seed=0)
    for c in (2, 3):  # arm 0: 2, arm 1: 3
        ad.observe([c])
    assert ad.arm == 0
    ad.observe([4])  # arm 0: (2 + 4) / 2 = 3 = arm 1
    assert ad.count == [2, 1] and ad.arm == 0
    ad.observe([10**15])  # arm 0 now far worse
    assert ad.arm == 1
    # means that differ by less than one part in 2^64: exact fractions still tell them apart
    ad = oracle.AdaptiveK([1, 2], window=1, explore=0, seed=0)
    big = (1 << 62) + 1
    ad.observe([big]); ad.observe([big - 1])
    assert ad.arm == 1
    ad.observe([big - 1]); assert ad.arm == 1
    ad.observe([big + 2]); assert ad.arm == 0  # arm 1: (3 big) / 3 = big, arm 0: big


def test_adaptive_k_windows_without_admissions_are_not_pulls():
    ad = oracle.AdaptiveK([1, 2, 3], window=2, explore=0, seed=3)
    for _ in range(6):
        ad.observe([])
    assert ad.arm == 0 and ad.pulls == 0 and ad.count == [0, 0, 0]
    ad.observe([]); ad.observe([8])
    assert ad.arm == 1 and ad.pulls == 1 and ad.count == [1, 0, 0] and ad.cost == [8, 0, 0]


def test_adaptive_k_exploration_rate_and_uniformity():
    A, n = 5, 20000
    # always explore: every arm equally often (chi-square, 4 degrees of freedom, 0.999 quantile 18.5)
    ad = oracle.AdaptiveK(list(range(1, A + 1)), window=1, explore=1 << 32, seed=11)
    arms = np.array(_feed(ad, [1] * n))[A:]
    cnt = np.bincount(arms, minlength=A)
    assert ((cnt - arms.size / A) ** 2 / (arms.size / A)).sum() < 18.5
    # pairs of consecutive draws are uniform too (no arm follows itself more than another)
    pair = np.bincount(arms[:-1] * A + arms[1:], minlength=A * A)
    assert ((pair - (arms.size - 1) / A**2) ** 2 / ((arms.size - 1) / A**2)).sum() < 52.6  # 24 dof, 0.999
    # arm 0 is the cheapest by far, so any other arm is an exploration: rate eps (A-1)/A within 4 sigma
    for eps_bits in (2, 4):
        ad = oracle.AdaptiveK(list(range(1, A + 1)), window=1, explore=(1 << 32) >> eps_bits, seed=12 + eps_bits)
        got = []
        for pull in range(n):
            got.append(ad.arm)
            ad.observe([1 if ad.arm == 0 else 1000])
        other = sum(1 for a in got[A:] if a != 0)
        pr = (A - 1) / A / (1 << eps_bits)
        m = n - A
        assert abs(other - m * pr) < 4 * math.sqrt(m * pr * (1 - pr))
    # never explore: after the first round only the cheapest arm
    ad = oracle.AdaptiveK(list(range(1, A + 1)), window=1, explore=0, seed=13)
    got = []
    for pull in range(200):
        got.append(ad.arm)
        ad.observe([1 if ad.arm == 2 else 50])
    assert got[:A] == list(range(A)) and set(got[A:]) == {2}


def test_timed_run_with_adaptive_k_uses_the_arm_of_each_window():
    n, u, rep, d = 48, 9, 4, 5
    p, _ = W.shuffled_queue(n, u, rep, d, 3, seed=6)
    # one arm is the fixed-k run; a window longer than the run never leaves the first arm
    for k in (1, rep, K_INF):
        fixed = oracle.simulate_timed(p, k, batch=2, budget=3 * (u + d))
        one = oracle.simulate_timed(p, 0, batch=2, budget=3 * (u + d), adaptive=oracle.AdaptiveK([k], 3, 1 << 31, 1))
        long_w = oracle.simulate_timed(p, 0, batch=2, budget=3 * (u + d),
                                       adaptive=oracle.AdaptiveK([k, 2, 7], 10**6, 1 << 31, 1))
        assert fixed.ttft.tolist() == one.ttft.tolist() == long_w.ttft.tolist()
        assert set(one.ks) == {k} and set(long_w.ks) == {k}
    # several arms: each step's batch is Algorithm 1 under that step's k (checked with the literal
    # loop on the step's own queue), k changes only at window boundaries, and the counters hold
    # the largest TTFT of every window
    ad = oracle.AdaptiveK([1, rep, K_INF, 2], window=3, explore=1 << 30, seed=2)
    r = oracle.simulate_timed(p, 0, batch=2, budget=3 * (u + d), t_start=40, adaptive=ad)
    phase = 0
    for step in range(r.steps):
        w, m = r.waiting_ids[step], r.match_lens[step]
        idx, phase = select_literal(p.arrival[w], m, r.ks[step], 2, phase)
        assert w[idx].tolist() == r.batches[step].tolist()
        if step % 3:
            assert r.ks[step] == r.ks[step - 1]
    assert len(set(r.ks)) > 1 and sum(ad.count) == r.steps // 3
    by_arm = {}
    for wdw in range(r.steps // 3):
        worst = max(int(r.ttft[g]) for s3 in range(3 * wdw, 3 * wdw + 3) for g in r.batches[s3])
        by_arm[r.ks[3 * wdw]] = by_arm.get(r.ks[3 * wdw], 0) + worst
    assert [by_arm.get(a, 0) for a in ad.arms] == ad.cost
