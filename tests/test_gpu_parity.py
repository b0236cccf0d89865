"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, bit-exact.

Compared after every step: match lengths, the ordered batch, the phase, the commit counters and
the canonical tree snapshot (byte for byte; node ids and pool layout are not part of the state).
"""
import hashlib

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2502_04677_amd as K
else:  # collected on a CPU-only host: every test here is deselected by the marker
    K = None

K_INF = W.K_LPM_ENDPOINT


def _say(msg):
    print(msg, flush=True)


def _setup(w, budget=None, max_batch=None, extra_prompts=0, max_len=None):
    budget = w.budget if budget is None else budget
    max_batch = max_batch or max(w.batch, 1)
    max_len = max_len or int(max(w.cache.len.max(initial=1), w.queries.len.max(initial=1)))
    cfg = K.size_config(int(w.cache.tokens.shape[0]), w.cache.n, budget, max_batch, max_len, extra_prompts,
                        extra_tokens=int(w.queries.tokens.shape[0]))
    cache = K.DeviceQueries.from_host(w.cache)
    q = K.DeviceQueries.from_host(w.queries)
    s = K.Scheduler(cfg, cache, max(q.n, 1))
    ref = oracle.OracleTree()
    ref.build(w.cache)
    return s, ref, q


def _same_tree(s, ref, big=False):
    a, b = s.snapshot(), ref.snapshot()
    if big:
        assert len(a) == len(b) and hashlib.sha256(a).digest() == hashlib.sha256(b).digest()
    else:
        assert a == b


_step_no = [0]


def _check_step(s, ref, q, hq, k, batch, phase, budget, big=False, fifo=False):
    """One match -> select -> commit step on both sides, compared at every stage.  Calls alternate
    between the commit that takes the step's match results and the one that matches again."""
    _step_no[0] += 1
    reuse = bool(_step_no[0] & 1)
    s.set_phase(phase)
    m = s.match(q).cpu().numpy()
    m_ref = ref.match(hq.tokens, hq.off, hq.len)
    assert (m == m_ref).all()
    s.select(q, k, batch, fifo=fifo)
    idx_ref, ph_ref = oracle.select(hq.arrival, m_ref, k, batch, phase)
    assert s.batch().tolist() == idx_ref.tolist()
    assert s.phase_value() == ph_ref
    K.kLPM_set_budget(s.tree, budget)
    s.commit(q, batch, reuse_match=reuse)
    st_ref = ref.commit(hq.tokens, hq.off, hq.len, idx_ref, budget)
    st = s.read_stats()
    assert st.device_error == 0
    got = (st.total_tokens, st.inserted_tokens, st.evicted_tokens, st.n_nodes, st.new_nodes, st.evicted_nodes, st.clock)
    want = (st_ref.total_tokens, st_ref.inserted_tokens, st_ref.evicted_tokens, st_ref.n_nodes, st_ref.new_nodes,
            st_ref.evicted_nodes, st_ref.clock)
    assert got == want
    _same_tree(s, ref, big)
    return ph_ref


# ----------------------------------------------------------------------------- small, dense cases
@pytest.mark.parametrize("seed", range(8))
def test_random_small_steps(seed):
    _say(f"random_small seed={seed}")
    w = W.random_small(seed + 900, n_cache=14, n_query=40, vocab=3, max_len=10)
    s, ref, q = _setup(w, max_batch=64, extra_prompts=400, max_len=16)
    _same_tree(s, ref)
    rng = np.random.default_rng(seed)
    phase = 0
    for step in range(6):
        k = int(rng.choice([1, 2, 3, 5, 1000, 0, K_INF]))
        batch = int(rng.integers(1, 48))
        budget = int(rng.integers(0, 2 * max(1, ref.total_tokens)))
        _say(f"  step={step} k={k} batch={batch} budget={budget} phase={phase}")
        phase = _check_step(s, ref, q, w.queries, k, batch, phase, budget)


def test_config0_single_step_and_more():
    w = W.config0()
    s, ref, q = _setup(w, extra_prompts=w.queries.n)
    _same_tree(s, ref)
    phase = _check_step(s, ref, q, w.queries, w.k, w.batch, 0, 1 << 50)
    # keep going on the same queue with a tight budget so that eviction and id reuse are exercised
    for step, budget in enumerate([14000, 9000, 15000, 4000, 20000]):
        _say(f"config0 extra step {step} budget={budget}")
        phase = _check_step(s, ref, q, w.queries, w.k, w.batch, phase, budget)


def test_select_sweep_on_config0():
    w = W.config0()
    s, ref, q = _setup(w, max_batch=64)
    m = s.match(q).cpu().numpy()
    m_ref = ref.match(w.queries.tokens, w.queries.off, w.queries.len)
    assert (m == m_ref).all()
    for k in (1, 2, 3, 4, 8, 31, 32, 33, 1000, 0, K_INF):
        for batch in (1, 2, 31, 32, 64):
            for phase in (0, 1, 7):
                idx_ref, ph_ref = oracle.select(w.queries.arrival, m_ref, k, batch, phase)
                for fifo in (False, True):  # config 0's queue is in arrival order
                    s.set_phase(phase)
                    s.select(q, k, batch, fifo=fifo)
                    assert s.batch().tolist() == idx_ref.tolist(), (k, batch, phase, fifo)
                    assert s.phase_value() == ph_ref


def test_select_ties_and_unsorted_arrivals():
    rng = np.random.default_rng(7)
    for n in (1, 2, 63, 64, 65, 2047, 2048, 2049, 5000):
        arrival = rng.integers(0, max(2, n // 3), size=n).astype(np.uint64)
        if n > 10:
            arrival[rng.integers(0, n, size=3)] = np.uint64(2**63 + 12345)  # exercise the top key bits
        m = rng.integers(0, 6, size=n).astype(np.int32)
        d_arr = torch.from_numpy(arrival.view(np.int64)).cuda()
        d_m = torch.from_numpy(m).cuda()
        ws_bytes = K.kLPM_select_workspace_bytes(n)
        ws = K.alloc_aligned(ws_bytes, "cuda:0")
        phase = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        nsel = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        for k in (1, 2, 4, 0):
            for batch in (1, 17, min(n, 700), n + 3):
                out = torch.full((min(batch, n),), -1, dtype=torch.int32, device="cuda:0")
                phase.fill_(1)
                K.kLPM_select(d_arr, d_m, n, k, batch, phase, out, nsel, ws, ws_bytes)
                idx_ref, ph_ref = oracle.select(arrival, m, k, batch, 1)
                assert int(nsel.item()) == idx_ref.shape[0]
                assert out.cpu().numpy().tolist() == idx_ref.tolist(), (n, k, batch)
                assert int(phase.cpu().numpy().view(np.uint32)[0]) == ph_ref


def test_select_arrival_ordered_queue_single_kernel():
    """The single-kernel path for a queue kept in arrival order, against the oracle; a queue that
    breaks the promise is refused (-1) instead of being mis-scheduled."""
    rng = np.random.default_rng(11)
    for n, mmax in ((1, 3), (64, 1), (1000, 6), (3000, 5000), (70000, 9000), (5000, 2**30), (20000, 2**30), (9000, 0)):
        arrival = np.sort(rng.integers(0, max(2, n // 2), size=n)).astype(np.uint64)  # sorted, many ties
        m = rng.integers(0, mmax + 1, size=n).astype(np.int32)
        if n >= 1000:
            m[rng.integers(0, n, size=n // 2)] = 0  # a big tie class at the bottom
            m[rng.integers(0, n, size=n // 4)] = mmax  # and one at the top
        d_arr = torch.from_numpy(arrival.view(np.int64)).cuda()
        d_m = torch.from_numpy(m).cuda()
        ws_bytes = K.kLPM_select_workspace_bytes(n)
        ws = K.alloc_aligned(ws_bytes, "cuda:0")
        phase = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        nsel = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        for k in (1, 2, 3, 8, 1000, 0):
            for batch in (1, 5, min(n, 1024), min(n, 4096)):
                out = torch.full((min(batch, n),), -1, dtype=torch.int32, device="cuda:0")
                phase.fill_(2)
                # (nothing in the workspace has to hold a particular value when a selection starts)
                ws[0].fill_(0xA5 if k & 1 else 0xFF) if batch == 5 else None
                K.kLPM_select(d_arr, d_m, n, k, batch, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO)
                idx_ref, ph_ref = oracle.select(arrival, m, k, batch, 2)
                assert int(nsel.item()) == idx_ref.shape[0], (n, k, batch)
                assert out.cpu().numpy().tolist() == idx_ref.tolist(), (n, mmax, k, batch)
                assert int(phase.cpu().numpy().view(np.uint32)[0]) == ph_ref
        if n >= 64:
            # a match length above the promised bound is refused like a broken arrival order
            K.kLPM_select(d_arr, d_m, n, 4, 8, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO,
                          max_match=max(1, int(m.max()) - 1))
            if n > 8192 and int(m.max()) >= 2:  # (the short-queue kernel needs no bound and ignores it)
                assert int(nsel.item()) == -1
            K.kLPM_select(d_arr, d_m, n, 4, 8, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO,
                          max_match=int(m.max()))
            assert int(nsel.item()) == min(8, n)
            bad = arrival.copy()
            bad[n // 2] = bad[n // 2 + 1] + 5
            phase.fill_(1)
            K.kLPM_select(torch.from_numpy(bad.view(np.int64)).cuda(), d_m, n, 4, 8, phase, out, nsel, ws, ws_bytes,
                          flags=K.KLPM_SELECT_FIFO)
            assert int(nsel.item()) == -1 and int(phase.item()) == 1


def test_degenerate_inputs():
    w = W.config0()
    s, ref, q = _setup(w)
    # batch = 0 and n = 0 select nothing and keep the phase
    s.set_phase(3)
    s.select(q, 4, 0)
    assert s.batch().tolist() == [] and s.phase_value() == 3
    s.select(q, 4, 8, n=0)
    assert s.batch().tolist() == [] and s.phase_value() == 3
    # ... on every path, and without a workspace
    for flags in (0, K.KLPM_SELECT_FIFO):
        for n, batch in ((0, 8), (q.n, 0), (0, 0)):
            s.n_selected.fill_(77)
            K.kLPM_select(q.arrival, s.match_len, n, 4, batch, s.phase, s.batch_idx, s.n_selected, (None, 0), 0, flags=flags)
            assert int(s.n_selected.item()) == 0 and s.phase_value() == 3
    # empty tree: every match is 0; committing into it equals the oracle
    cfg = K.size_config(0, 0, 1 << 50, 32, 1024, extra_prompts=64, extra_tokens=int(w.queries.tokens.shape[0]))
    s2 = K.Scheduler(cfg, None, q.n)
    assert not s2.match(q).cpu().numpy().any()
    ref2 = oracle.OracleTree()
    _check_step(s2, ref2, q, w.queries, 2, 32, 0, 1 << 50)
    # a prompt span outside the token buffer is reported, not followed
    bad = K.DeviceQueries(q.tokens, q.off.clone(), q.len.clone(), q.arrival, q.n)
    bad.off[5] = q.tokens.numel() - 3
    bad.len[5] = 64
    m = s.match(bad).cpu().numpy()
    assert m[5] == -1 and (K.kLPM_read_stats(s.tree).device_error & 4)


def test_pool_compaction_keeps_the_tree_intact():
    """A pool barely larger than budget + one batch: the bump allocator fills a half every few
    commits, so live spans are compacted into the other half again and again."""
    w = W.config0()
    hq = w.queries
    budget = 9000
    max_len = int(max(w.cache.len.max(), hq.len.max()))
    batch = 16
    cache_tokens = int(w.cache.tokens.shape[0])
    cfg = K.make_config(budget, cache_tokens + batch * max_len + 64, 2 * (w.cache.n + hq.n) + 4 * batch + 64, batch, max_len)
    s = K.Scheduler(cfg, K.DeviceQueries.from_host(w.cache), hq.n)
    ref = oracle.OracleTree()
    ref.build(w.cache)
    q = K.DeviceQueries.from_host(hq)
    _same_tree(s, ref)
    rng = np.random.default_rng(3)
    phase = 0
    for step in range(40):
        k = int(rng.choice([1, 2, 4, K_INF]))
        phase = _check_step(s, ref, q, hq, k, batch, phase, budget)


def test_compaction_and_table_rebuild_on_a_larger_tree():
    """The same squeeze on a tree with room for more nodes than the small-tree path takes, and a
    child table small enough that tombstones force rebuilds: the commit's closing kernel compacts
    the pool on some steps and refills the table on others."""
    w = W.config0()
    hq = w.queries
    budget = 9000
    max_len = int(max(w.cache.len.max(), hq.len.max()))
    batch = 16
    cache_tokens = int(w.cache.tokens.shape[0])
    cfg = K.make_config(budget, cache_tokens + batch * max_len + 64, 2100, batch, max_len)
    s = K.Scheduler(cfg, K.DeviceQueries.from_host(w.cache), hq.n)
    ref = oracle.OracleTree()
    ref.build(w.cache)
    q = K.DeviceQueries.from_host(hq)
    _same_tree(s, ref)
    rng = np.random.default_rng(4)
    phase = 0
    evicted = 0
    for step in range(150):
        k = int(rng.choice([1, 2, 4, K_INF]))
        phase = _check_step(s, ref, q, hq, k, batch, phase, (0, 500, budget)[step % 3])  # churn: most of the tree goes every step
        evicted += s.read_stats().evicted_nodes
    assert evicted > 2100  # more evictions than a quarter of the table's slots: it has been rebuilt


def test_commit_refusals_leave_the_tree_as_it_was():
    w = W.config0()
    hq = w.queries
    max_len = int(max(w.cache.len.max(), hq.len.max()))
    q = K.DeviceQueries.from_host(hq)
    cache = K.DeviceQueries.from_host(w.cache)
    ref = oracle.OracleTree()
    ref.build(w.cache)
    m_ref = ref.match(hq.tokens, hq.off, hq.len)

    def fresh(cfg):
        s = K.Scheduler(cfg, cache, hq.n)
        _same_tree(s, ref)
        s.match(q)
        s.select(q, 2, 32)
        return s

    big_pool = int(w.cache.tokens.shape[0]) + 64 * max_len
    # not enough free node ids for two per admitted prompt
    s = fresh(K.make_config(1 << 40, big_pool, ref.n_nodes + 1 + 40, 32, max_len))
    s.commit(q, 32)
    st = s.read_stats()
    assert st.device_error & 1 and st.inserted_tokens == 0 and st.clock == w.cache.n
    _same_tree(s, ref)
    # the pool runs out: commits of fresh slices of the queue succeed until one batch's tails no
    # longer fit even after compaction; that commit is refused and changes nothing
    s = fresh(K.make_config(1 << 40, ref.total_tokens + 13000, 4096, 32, max_len))
    ref_p = oracle.OracleTree()
    ref_p.build(w.cache)
    refused = False
    for i in range(hq.n // 32):
        idx = np.arange(32 * i, 32 * i + 32, dtype=np.int32)
        s.batch_idx[:32] = torch.from_numpy(idx).cuda()
        s.n_selected.fill_(32)
        before = ref_p.snapshot()
        s.commit(q, 32)
        st = s.read_stats()
        if st.device_error & 2:
            assert s.snapshot() == before and st.inserted_tokens == 0
            refused = True
            break
        ref_p.commit(hq.tokens, hq.off, hq.len, idx, 1 << 60)
        assert s.snapshot() == ref_p.snapshot()
    assert refused
    assert (s.match(q).cpu().numpy() == ref_p.match(hq.tokens, hq.off, hq.len)).all()
    # more selected entries than the capacity passed to commit
    s = fresh(K.make_config(1 << 40, big_pool, 4096, 32, max_len))
    s.commit(q, 8)
    st = s.read_stats()
    assert st.device_error & 8 and st.inserted_tokens == 0
    _same_tree(s, ref)
    # an admitted prompt whose span lies outside the token buffer
    s = fresh(K.make_config(1 << 40, big_pool, 4096, 32, max_len))
    first = int(s.batch()[0])
    bad = K.DeviceQueries(q.tokens, q.off.clone(), q.len.clone(), q.arrival, q.n)
    bad.off[first] = q.tokens.numel() - 2
    s.commit(bad, 32)
    st = s.read_stats()
    assert st.device_error & 4 and st.inserted_tokens == 0
    _same_tree(s, ref)
    # match results handed to the commit that are not this tree's: every entry one off, or naming a
    # node that cannot hold it, is refused
    idx_ref, _ = oracle.select(hq.arrival, m_ref, 2, 32, 0)
    inner = [int(i) for i in idx_ref if 2 <= m_ref[i] < hq.len[i]]
    zero = [int(i) for i in idx_ref if m_ref[i] == 0]
    assert inner and zero
    tampers = [("len+1", inner[0], +1, None), ("len-1", inner[0], -1, None), ("past the end", inner[0], 1 << 20, None),
               ("negative", inner[0], -(1 << 20), None), ("node out of range", inner[0], 0, 4096),
               ("node negative", inner[0], 0, -1), ("root with a match", inner[0], 0, 0),
               ("dead node", inner[0], 0, 4000), ("no match below the root", zero[0], 0, 1)]
    for name, qi, dlen, node in tampers:
        _say(f"  tampered match result: {name}")
        s = fresh(K.make_config(1 << 40, big_pool, 4096, 32, max_len))
        ml, ln = s.match_len.clone(), s.last_node.clone()
        ml[qi] += dlen
        if node is not None:
            ln[qi] = node
        K.kLPM_commit_matched(s.tree, q, ml, ln, s.batch_idx, s.n_selected, 32, s.stats)
        st = s.read_stats()
        assert st.device_error == 4 and st.inserted_tokens == 0 and st.clock == w.cache.n, name
        _same_tree(s, ref)
    # after a refusal the same tree still commits normally
    s.commit(q, 32)
    ref2 = oracle.OracleTree()
    ref2.build(w.cache)
    ref2.commit(hq.tokens, hq.off, hq.len, idx_ref, 1 << 60)
    assert s.snapshot() == ref2.snapshot()


# ----------------------------------------------------------------------------- the configurations
def test_config1_step():
    w = W.config1()
    _say(f"config1: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w, extra_prompts=w.batch)
    _same_tree(s, ref, big=True)
    _check_step(s, ref, q, w.queries, w.k, w.batch, 0, w.budget, big=True, fifo=True)


def test_config2_scaled_steps():
    w = W.config2(scale=1 / 16)
    _say(f"config2/16: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w, extra_prompts=4 * w.batch)
    _same_tree(s, ref, big=True)
    phase = 0
    for step in range(3):  # budget = initial size: every step evicts what it inserts
        phase = _check_step(s, ref, q, w.queries, w.k, w.batch, phase, w.budget, big=True, fifo=(step % 2 == 1))


def test_config2_deep_tree_variant():
    """Same token recipe as the large step but about one node per 50-90 tokens: long chains of
    child-table probes, many short edges, many prompts that add no token at all."""
    w = W.config2_deep(scale=1 / 16)
    _say(f"config2-deep/16: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w, extra_prompts=4 * w.batch)
    _say(f"  oracle tree: {ref.total_tokens} tokens, {ref.n_nodes} nodes")
    _same_tree(s, ref, big=True)
    phase = 0
    for step in range(3):
        phase = _check_step(s, ref, q, w.queries, w.k, w.batch, phase, w.budget, big=True, fifo=(step % 2 == 0))


def test_config3_scaled_k_sweep():
    w = W.config3(scale=1 / 16)
    _say(f"config3/16: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w)
    _same_tree(s, ref, big=True)
    m = s.match(q).cpu().numpy()
    m_ref = ref.match(w.queries.tokens, w.queries.off, w.queries.len)
    assert (m == m_ref).all()
    outs = []
    for k in w.ks:
        s.set_phase(0)
        s.select(q, k, w.batch)
        idx_ref, ph_ref = oracle.select(w.queries.arrival, m_ref, k, w.batch, 0)
        assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref
        outs.append(idx_ref.tolist())
    assert outs[0] == outs[4]  # "k = 1" and the FCFS endpoint are the same setting
    _check_step(s, ref, q, w.queries, 4, w.batch, 0, w.budget, big=True)


def test_config2_full_size_steps():
    """The large configuration at full size, in the launch shapes the benchmark times."""
    w = W.config2()
    _say(f"config2 full: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w, extra_prompts=4 * w.batch, max_len=8192)
    _say("  built both trees")
    _same_tree(s, ref, big=True)
    phase = 0
    for step in range(2):
        _say(f"  step {step}")
        phase = _check_step(s, ref, q, w.queries, w.k, w.batch, phase, w.budget, big=True, fifo=(step == 0))


def test_config2_deep_full_size_step():
    """The deep-tree variant at full size (100M tokens in 1.2M nodes, 65,536 waiting): one whole step
    with the canonical tree compared before and after (the oracle's eviction is a scan per evicted
    leaf there, about ten seconds for the one step)."""
    w = W.config2_deep()
    _say(f"config2-deep full: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w, extra_prompts=2 * w.batch, max_len=8192)
    _say(f"  built both trees: {ref.total_tokens} tokens, {ref.n_nodes} nodes")
    _same_tree(s, ref, big=True)
    _check_step(s, ref, q, w.queries, w.k, w.batch, 0, w.budget, big=True, fifo=True)


def test_config3_full_size_k_sweep():
    """The hierarchical configuration at full size: match once, select for every k of the sweep."""
    w = W.config3()
    _say(f"config3 full: cache {w.cache.n} prompts / {w.cache.tokens.shape[0]} tokens, {w.queries.n} queries")
    s, ref, q = _setup(w)
    _say("  built both trees")
    _same_tree(s, ref, big=True)
    m = s.match(q).cpu().numpy()
    m_ref = ref.match(w.queries.tokens, w.queries.off, w.queries.len)
    assert (m == m_ref).all()
    for k in w.ks:
        for fifo in (False, True):
            s.set_phase(0)
            s.select(q, k, w.batch, fifo=fifo)
            idx_ref, ph_ref = oracle.select(w.queries.arrival, m_ref, k, w.batch, 0)
            assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref, (k, fifo)
    _check_step(s, ref, q, w.queries, 4, w.batch, 0, w.budget, big=True)


def _run_stream(stream, cap, snapshot_every, check_every_step=True):
    r = oracle.simulate_stream(stream, snapshot_every=snapshot_every)
    hq = stream.queries
    q = K.DeviceQueries.from_host(hq)
    cfg = K.size_config(0, 0, stream.budget, stream.batch, int(hq.len.max()), extra_prompts=hq.n)
    s = K.Scheduler(cfg, None, cap)
    first = np.arange(int(stream.step_start[0]), int(stream.step_start[1]))
    run = K.OnlineRun(s, q, cap, first)
    for step in range(stream.steps):
        nxt = None
        if step + 1 < stream.steps:
            ids = np.arange(int(stream.step_start[step + 1]), int(stream.step_start[step + 2]), dtype=np.int32)
            nxt = torch.from_numpy(ids).cuda()
        n_before = run.n_host
        run.step(stream.k, stream.batch, nxt)
        if check_every_step or r.snapshots[step] is not None:
            torch.cuda.synchronize()
            assert s.match_len[:n_before].cpu().numpy().tolist() == r.match_lens[step].tolist(), step
            got_batch = s.batch()
            assert r.waiting_ids[step][got_batch].tolist() == r.batches[step].tolist(), step
            st = s.read_stats()
            want = r.stats[step]
            assert st.device_error == 0
            assert (st.total_tokens, st.evicted_tokens, st.n_nodes, st.clock) == (
                want.total_tokens, want.evicted_tokens, want.n_nodes, want.clock), step
        if r.snapshots[step] is not None:
            _say(f"  stream step {step}: snapshot compare")
            assert s.snapshot() == r.snapshots[step], step
    assert int(run.sim_clock.item()) == r.clock
    ttft = run.ttft.cpu().numpy()
    assert ttft.tolist() == r.ttft.tolist()
    assert int(run.dev_error.item()) == 0
    done = ttft[ttft >= 0]
    assert oracle.percentile_nearest_rank(done, 0.5) == oracle.percentile_nearest_rank(r.ttft[r.ttft >= 0], 0.5)
    assert oracle.percentile_nearest_rank(done, 0.99) == oracle.percentile_nearest_rank(r.ttft[r.ttft >= 0], 0.99)
    return r


def test_config4_scaled_online_stream():
    stream = W.config4_stream(steps=60, rate=24, groups=2000, budget=150_000, batch=32)
    _run_stream(stream, 4096, snapshot_every=10)


def test_config4_overloaded_stream_keeps_a_backlog():
    """More arrivals than the batch admits: the queue backs up, k matters, phases carry over."""
    stream = W.config4_stream(steps=40, rate=40, groups=300, budget=120_000, batch=24)
    stream.k = 3
    r = _run_stream(stream, 4096, snapshot_every=8)
    assert max(len(w) for w in r.waiting_ids) > 10 * stream.batch


def test_config4_full_size_online_stream():
    """1,000 steps, Poisson(128) arrivals per step, 4M-token budget; every step compared."""
    stream = W.config4_stream()
    _say(f"config4 full: {stream.queries.n} queries / {stream.queries.tokens.shape[0]} tokens over {stream.steps} steps")
    _run_stream(stream, 8192, snapshot_every=100)


def test_select_repeated_on_a_dirty_workspace():
    """The long-queue selection hands its winners from workgroup to workgroup through flags in the
    workspace; many calls in a row on the same input, the workspace overwritten with random bytes in
    between, must all give the oracle's batch."""
    rng = np.random.default_rng(5)
    dev = "cuda:0"
    for n, mmax, ties in ((65536, 8192, False), (40000, 100000, False), (30000, 6000, True)):
        arrival = np.sort(rng.integers(0, n, size=n)).astype(np.uint64)
        m = rng.integers(0, mmax + 1, size=n).astype(np.int32)
        m[rng.integers(0, n, size=n // 3)] = 0
        m[rng.choice(600, size=40, replace=False)] = mmax - 1  # old queries among the best matches
        tie = rng.integers(0, 2**32, size=n, dtype=np.uint64).astype(np.uint32) if ties else None
        d_arr = torch.from_numpy(arrival.view(np.int64)).to(dev)
        d_m = torch.from_numpy(m).to(dev)
        d_tie = None if tie is None else torch.from_numpy(tie.view(np.int32)).to(dev)
        ws_bytes = K.kLPM_select_workspace_bytes(n)
        ws = K.alloc_aligned(ws_bytes, dev)
        phase = torch.zeros(1, dtype=torch.int32, device=dev)
        nsel = torch.zeros(1, dtype=torch.int32, device=dev)
        ref, ph_ref = oracle.select(arrival, m, 8, 1024, 3, tie_key=tie)
        ref_t = torch.from_numpy(ref).to(dev)
        out = torch.empty(1024, dtype=torch.int32, device=dev)
        wrong = torch.zeros(1, dtype=torch.int64, device=dev)
        for it in range(400):
            phase.fill_(3)
            if it % 5 == 0:
                ws[0].random_(0, 255)
            K.kLPM_select(d_arr, d_m, n, 8, 1024, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO, max_match=mmax,
                          tie_key=d_tie)
            wrong += (out != ref_t).sum() + (nsel[0] != 1024).long() + (phase[0] != ph_ref).long()
        assert int(wrong.item()) == 0, (n, mmax, ties)


@pytest.mark.parametrize("n", [150_000, 1_000_000])
def test_select_long_arrival_ordered_queues(n):
    """Queues long enough that every workgroup of the sweeps takes several rounds over its stretch; plain
    scores (one level), scores beyond one level's range (two levels) and tie keys (five levels)."""
    rng = np.random.default_rng(77 + n)
    arrival = np.sort(rng.integers(0, n // 3, size=n)).astype(np.uint64)
    d_arr = torch.from_numpy(arrival.view(np.int64)).cuda()
    ws_bytes = K.kLPM_select_workspace_bytes(n)
    ws = K.alloc_aligned(ws_bytes, "cuda:0")
    phase = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    nsel = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for mmax, ties in ((6000, False), (300_000, False), (50, True)):
        m = rng.integers(0, mmax + 1, size=n).astype(np.int32)
        m[rng.integers(0, n, size=n // 2)] = 0
        m[rng.integers(0, n, size=n // 50)] = mmax  # a tie class at the top, larger than some batches
        tie = rng.integers(0, 2**32, size=n, dtype=np.uint64).astype(np.uint32) if ties else None
        d_m = torch.from_numpy(m).cuda()
        d_tie = None if tie is None else torch.from_numpy(tie.view(np.int32)).cuda()
        for k, batch in ((4, 300), (8, 4096), (0, 1000)):
            if n > 500_000 and batch > 1000:
                continue  # (the oracle's literal loop is O(batch x n))
            ph = int(rng.integers(0, max(k, 1)))
            out = torch.full((batch,), -1, dtype=torch.int32, device="cuda:0")
            phase.fill_(ph)
            ws[0].fill_(0x5A)
            K.kLPM_select(d_arr, d_m, n, k, batch, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO,
                          max_match=mmax, tie_key=d_tie)
            idx_ref, ph_ref = oracle.select(arrival, m, k, batch, ph, tie_key=tie)
            assert int(nsel.item()) == idx_ref.shape[0], (n, mmax, k, batch)
            assert out.cpu().numpy().tolist() == idx_ref.tolist(), (n, mmax, ties, k, batch, ph)
            assert int(phase.cpu().numpy().view(np.uint32)[0]) == ph_ref


@pytest.mark.parametrize("n,boost", [(9000, 0), (9000, 40), (30000, 8), (30000, 300), (70000, 0), (70000, 60)])
def test_select_when_both_orders_reach_the_same_queries(n, boost):
    """Alg. 1 on arrival-ordered queues in which some of the oldest queries are also among the longest
    matches (none, a handful, more than a wavefront's worth), so that either cursor steps over what the
    other took; every k, phase and batch size against the oracle."""
    rng = np.random.default_rng(1000 + n + boost)
    arrival = np.sort(rng.integers(0, n, size=n)).astype(np.uint64)
    m = rng.integers(0, 4000, size=n).astype(np.int32)
    m[rng.integers(0, n, size=n // 3)] = 0
    if boost:
        old = rng.choice(600, size=boost, replace=False)
        m[old] = rng.integers(3000, 4200, size=boost).astype(np.int32)  # old queries with long matches
    d_arr = torch.from_numpy(arrival.view(np.int64)).cuda()
    d_m = torch.from_numpy(m).cuda()
    ws_bytes = K.kLPM_select_workspace_bytes(n)
    ws = K.alloc_aligned(ws_bytes, "cuda:0")
    phase = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    nsel = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for k in (2, 3, 5, 8, 64, 1000):
        for batch in (7, 512, 1024, 4096):
            ph = int(rng.integers(0, k))
            out = torch.full((batch,), -1, dtype=torch.int32, device="cuda:0")
            phase.fill_(ph)
            K.kLPM_select(d_arr, d_m, n, k, batch, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO)
            idx_ref, ph_ref = oracle.select(arrival, m, k, batch, ph)
            assert int(nsel.item()) == idx_ref.shape[0], (n, k, batch)
            assert out.cpu().numpy().tolist() == idx_ref.tolist(), (n, boost, k, batch, ph)
            assert int(phase.cpu().numpy().view(np.uint32)[0]) == ph_ref


# ----------------------------------------------------------------------------- device-side queue length
def test_select_with_device_side_queue_length():
    """Buffers sized for a capacity, of which only the first *n_live entries exist: every selection
    path must ignore what lies beyond (filled here with entries that would win every pick)."""
    rng = np.random.default_rng(23)
    dev = "cuda:0"
    for cap in (300, 6000, 20000):
        ws_bytes = K.kLPM_select_workspace_bytes(cap)
        ws = K.alloc_aligned(ws_bytes, dev)
        phase = torch.zeros(1, dtype=torch.int32, device=dev)
        nsel = torch.zeros(1, dtype=torch.int32, device=dev)
        live_d = torch.zeros(1, dtype=torch.int32, device=dev)
        for live in (0, 1, 2, cap // 3, cap - 1, cap, cap + 50):
            n = min(live, cap)
            m = rng.integers(0, 400, size=cap).astype(np.int32)
            for fifo in (True, False):
                arrival = rng.integers(0, max(2, cap // 4), size=cap).astype(np.uint64)
                if fifo:
                    arrival[:n] = np.sort(arrival[:n])
                arrival[n:] = 0  # beyond the live part: older and longer than everything
                m[n:] = 400
                d_arr = torch.from_numpy(arrival.view(np.int64)).to(dev)
                d_m = torch.from_numpy(m).to(dev)
                live_d.fill_(live)
                for k in (1, 3, 0):
                    for batch in (1, 7, 256):
                        out = torch.full((batch,), -7, dtype=torch.int32, device=dev)
                        phase.fill_(1)
                        K.kLPM_select(d_arr, d_m, cap, k, batch, phase, out, nsel, ws, ws_bytes,
                                      flags=K.KLPM_SELECT_FIFO if fifo else 0, max_match=400, n_live=live_d)
                        idx_ref, ph_ref = oracle.select(arrival[:n], m[:n], k, batch, 1)
                        got_n = int(nsel.item())
                        assert got_n == idx_ref.shape[0], (cap, live, fifo, k, batch)
                        assert out[:got_n].cpu().numpy().tolist() == idx_ref.tolist(), (cap, live, fifo, k, batch)
                        assert int(phase.cpu().numpy().view(np.uint32)[0]) == ph_ref, (cap, live, fifo, k, batch)


def test_match_with_device_side_queue_length():
    w = W.config0()
    s, ref, q = _setup(w)
    want = ref.match(w.queries.tokens, w.queries.off, w.queries.len)
    live_d = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for live in (0, 1, 100, q.n, q.n + 9):
        live_d.fill_(live)
        s.match_len.fill_(-5)
        ql = K.DeviceQueries(q.tokens, q.off, q.len, q.arrival, q.n, n_live=live_d)
        got = s.match(ql).cpu().numpy()
        n = min(live, q.n)
        assert got[:n].tolist() == want[:n].tolist() and (got[n:q.n] == -5).all()  # the rest is untouched


# ----------------------------------------------------------------------------- Def. 2 timeline with timed arrivals
def _run_timed(p, k, batch, budget, c_num=0, c_den=1, t_start=0, cap=None, check_every=1, tie_seed=None,
               adaptive=None):
    """The device-resident timed run against the oracle's event loop: queue contents, match lengths
    and batch at the checked steps; TTFT of every query, final clock and step count at the end."""
    cap_o = p.n if cap is None else cap
    ad_ref = None if adaptive is None else oracle.AdaptiveK(*adaptive)
    r = oracle.simulate_timed(p, k, batch, budget, c_num=c_num, c_den=c_den, t_start=t_start, queue_cap=cap_o,
                              tie_seed=tie_seed, adaptive=ad_ref)
    q = K.DeviceQueries.from_host(p)
    cfg = K.size_config(0, 0, budget, batch, int(p.len.max()), extra_prompts=2 * batch)
    s = K.Scheduler(cfg, None, cap_o)
    run = K.TimedRun(s, q, cap_o, p.arrival, c_num=c_num, c_den=c_den, t_start=t_start, tie_seed=tie_seed)
    ad = None if adaptive is None else K.AdaptiveK(*adaptive)
    k_host = k if adaptive is None else 0x5EED  # with a device-side k the host's value must not matter
    for step in range(r.steps):
        check = check_every and (step % check_every == 0 or step == r.steps - 1)
        if check:
            n_live = int(run.queue.n.item())
            ids = run.queue.id[:n_live].cpu().numpy()
            assert ids.tolist() == r.waiting_ids[step].tolist(), step
        run.step(k_host, batch, adaptive=ad)
        if check:
            assert s.match_len[:n_live].cpu().numpy().tolist() == r.match_lens[step].tolist(), step
            assert ids[s.batch()].tolist() == r.batches[step].tolist(), step
    run.step(k_host, batch)  # one step past the end: nobody is waiting, nothing is pending, nothing changes
    torch.cuda.synchronize()
    if ad is not None:
        st = ad.read()
        A = len(ad_ref.arms)
        assert st.device_error == 0
        assert (list(st.count)[:A], list(st.cost)[:A], st.pulls, st.arm, st.k, st.steps_in_window) == (
            ad_ref.count, ad_ref.cost, ad_ref.pulls, ad_ref.arm, ad_ref.k(), ad_ref.steps)
    assert int(run.queue.n.item()) == 0 and int(run.queue.n_joined.item()) == p.n
    assert int(run.sim_clock.item()) == r.clock
    assert run.ttft[:p.n].cpu().numpy().tolist() == r.ttft.tolist()
    assert int(run.dev_error.item()) == 0 and s.read_stats().device_error == 0
    return r


@pytest.mark.parametrize("seed,n,u,rep,d", [(1, 24, 6, 3, 4), (2, 40, 9, 4, 3), (3, 64, 70, 2, 90)])
def test_timed_shuffled_queue_small(seed, n, u, rep, d):
    """Regular Arrival Shuffled Queue (Def. 3) served one query at a time with one prompt of cache
    (the last-prompt cache of Def. 2), from bursts (s = 0) to arrivals slower than the service."""
    for s_gap in (0, 1, (u + d) // 2, u // rep + d, 3 * (u + d)):
        for c_num, c_den in ((0, 1), (3, 64)):
            p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=seed)
            p.arrival[:] = p.arrival * np.uint64(c_den)
            for k in (1, rep, K_INF):
                _say(f"timed small: n={n} u={u} d={d} s={s_gap} c={c_num}/{c_den} k={k}")
                _run_timed(p, k, 1, u + d, c_num=c_num, c_den=c_den)


def test_timed_batches_bounded_queue_and_late_start():
    """Batches of several queries, a waiting queue smaller than the backlog (arrivals stay outside, in
    order), a cache of a few prompts, and a start time after part of the stream has arrived."""
    p, _ = W.shuffled_queue(96, 40, 4, 25, 30, seed=7)
    for k, batch, cap, t_start in ((2, 4, 16, 0), (K_INF, 3, 8, 500), (4, 8, 96, 1200), (1, 5, 7, 0)):
        _say(f"timed batched: k={k} B={batch} cap={cap} T={t_start}")
        _run_timed(p, k, batch, 4 * 65, c_num=1, c_den=128, t_start=t_start, cap=cap)


@pytest.mark.parametrize("u,d", [(1000, 5000), (3000, 3000), (5000, 1000)])
def test_timed_shuffled_queue_paper_shape(u, d):
    """n = 2000 queries, 4 per shared prefix, prompt length 6000 split as in the paper's table on
    varying the prefix-length ratio; arrival gap between the per-query cost with and without reuse,
    so that how much a policy reuses decides whether its backlog grows."""
    n, rep, c_num, c_den = 2000, 4, 1, 1 << 16
    gap = ((u // rep + d) + (u + d)) // 2
    p, _ = W.shuffled_queue(n, u, rep, d, gap, seed=11)
    p.arrival[:] = p.arrival * np.uint64(c_den)
    for t_start in (0, gap * n * c_den):  # served while arriving / after everything has arrived (setting of Thm. 2)
        res = {}
        for k in (1, rep, K_INF):
            _say(f"timed paper shape: u={u} d={d} k={k} T={t_start // c_den}")
            r = _run_timed(p, k, 1, u + d, c_num=c_num, c_den=c_den, t_start=t_start, cap=2048, check_every=500)
            res[k] = [oracle.percentile_nearest_rank(r.ttft, q) / c_den for q in (0.5, 0.9, 0.95, 0.99)]
            _say(f"   TTFT P50/P90/P95/P99 (token times): {res[k]}")
        # more reuse, lower median: LPM <= k-LPM <= FCFS at P50 (Sec. 4.2 and the discussion of the
        # table on varying the prefix-length ratio)
        assert res[K_INF][0] <= res[rep][0] <= res[1][0]


def test_timed_runs_with_random_ties():
    """The timed run with the uniformly random tie-break that the theory assumes for LPM (footnote of
    Sec. 4.2): keys are redrawn per query id and step on both sides."""
    for seed, (n, u, rep, d, s_gap) in enumerate([(24, 6, 3, 4, 0), (40, 9, 4, 3, 2), (64, 70, 2, 90, 40)]):
        p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=seed + 20)
        for k, batch, t_start in ((K_INF, 1, 0), (rep, 1, s_gap * n), (2, 3, 0), (1, 2, 5)):
            _say(f"timed random ties: n={n} k={k} B={batch} T={t_start}")
            _run_timed(p, k, batch, batch * (u + d), t_start=t_start, tie_seed=1000 + seed)
    p, _ = W.shuffled_queue(96, 40, 4, 25, 30, seed=8)
    _run_timed(p, K_INF, 4, 4 * 65, c_num=1, c_den=128, cap=16, tie_seed=5)


def test_timed_gap_sweep_separates_the_policies_as_the_theory_says():
    """Thm. 2's setting at the shape of the paper's table (n = 2000, 4 queries per shared prefix,
    u = d = 3000): everything has arrived when processing starts, LPM breaks ties at random.  For an
    arrival gap 0 < s < u, k-LPM with k = the replication has the lowest maximum TTFT of the three
    policies (Corollary 1) while the median orders them by reuse."""
    n, rep, u, d, c_num, c_den = 2000, 4, 3000, 3000, 1, 1 << 16
    for s_gap in (500, 2500):
        p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=12)
        p.arrival[:] = p.arrival * np.uint64(c_den)
        worst, median = {}, {}
        for k in (1, rep, K_INF):
            _say(f"timed gap sweep: s={s_gap} k={k}")
            r = _run_timed(p, k, 1, u + d, c_num=c_num, c_den=c_den, t_start=s_gap * n * c_den, cap=2048,
                           check_every=700, tie_seed=99)
            worst[k], median[k] = int(r.ttft.max()), oracle.percentile_nearest_rank(r.ttft, 0.5)
        assert worst[rep] < worst[K_INF] and worst[rep] < worst[1], (s_gap, worst)
        assert median[K_INF] <= median[rep] <= median[1], (s_gap, median)
    # served while arriving, at a gap between the cost of a query with full reuse and with none (an
    # overloaded request rate): k = 2 has the lowest P99, as in the paper's serving experiments (Sec. 5.1)
    s_gap = (u // rep + d + u + d) // 2
    p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=12)
    p.arrival[:] = p.arrival * np.uint64(c_den)
    p99, median = {}, {}
    for k in (1, 2, K_INF):
        _say(f"timed gap sweep while arriving: s={s_gap} k={k}")
        r = _run_timed(p, k, 1, u + d, c_num=c_num, c_den=c_den, cap=2048, check_every=700, tie_seed=99)
        p99[k], median[k] = (oracle.percentile_nearest_rank(r.ttft, x) for x in (0.99, 0.5))
    assert p99[2] < p99[1] and p99[2] < p99[K_INF], p99
    assert median[K_INF] < median[2] < median[1], median


# ----------------------------------------------------------------------------- k read from device memory, adaptive k
def test_select_reads_k_from_device_memory():
    """Every selection path with k taken from device memory (the host's k is then ignored): the short
    and the long arrival-ordered paths, the sorting path, in-batch rescoring and the token-budget cut."""
    dev = "cuda:0"
    w = W.config1(scale=0.125)
    s, ref, q = _setup(w, max_batch=256)
    hq = w.queries
    m_ref = ref.match(hq.tokens, hq.off, hq.len)
    s.match(q)
    order = np.argsort(hq.arrival, kind="stable")
    assert (order == np.arange(hq.n)).all()  # this queue is in arrival order
    k_d = torch.zeros(1, dtype=torch.int32, device=dev)
    dyn_bytes = K.kLPM_select_dynamic_workspace_bytes(q.n)
    dyn_ws = K.alloc_aligned(dyn_bytes, dev)
    dyn = torch.zeros(q.n, dtype=torch.int32, device=dev)
    for k in (1, 2, 3, 7, 300, 0, K_INF):
        k_d.copy_(torch.from_numpy(np.array([k], dtype=np.uint32).view(np.int32)))
        for n, fifo in ((300, True), (hq.n, True), (hq.n, False), (300, False)):
            for batch in (1, 64, 256):
                _say(f"device-side k={k} n={n} fifo={fifo} B={batch}")
                s.set_phase(5)
                s.select(q, 0x5EED, batch, n=n, fifo=fifo, k_dev=k_d.data_ptr())
                idx_ref, ph_ref = oracle.select(hq.arrival[:n], m_ref[:n], k, batch, 5)
                assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref
        # the token-budget cut rewinds the phase by the same k
        s.set_phase(5)
        s.select(q, 0x5EED, 64, fifo=True, k_dev=k_d.data_ptr())
        full_ref, ph_full = oracle.select(hq.arrival, m_ref, k, 64, 5)
        cost = (hq.len[full_ref] - m_ref[full_ref]).astype(np.int64)
        K.kLPM_batch_token_budget(q, s.match_len, s.batch_idx, s.n_selected, 64, int(cost.sum() // 2), 0x5EED, s.phase,
                                  k_dev=k_d.data_ptr())
        keep = oracle.token_budget_cut(full_ref, hq.len, m_ref, int(cost.sum() // 2))
        assert s.batch().tolist() == full_ref[:keep].tolist()
        assert s.phase_value() == oracle.phase_after_cut(ph_full, 64, keep, k)
        # in-batch rescoring
        sub = 1500
        qs = K.DeviceQueries(q.tokens, q.off, q.len, q.arrival, sub)
        s.set_phase(1)
        K.kLPM_select_dynamic(qs, s.match_len, s.last_node, 0x5EED, 48, s.phase, dyn, s.batch_idx, s.n_selected, dyn_ws,
                              dyn_bytes, k_dev=k_d.data_ptr())
        idx_ref, ph_ref, _ = oracle.select_dynamic(hq.tokens, hq.off[:sub], hq.len[:sub], hq.arrival[:sub], m_ref[:sub], k, 48, 1)
        assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref


def test_timed_runs_with_adaptive_k():
    """k chosen per window by the device-resident epsilon-greedy rule: the run (every TTFT, hence every
    batch and every k) and the bandit's counters equal the oracle's."""
    for seed, (n, u, rep, d, s_gap) in enumerate([(48, 9, 4, 5, 3), (64, 70, 2, 90, 40), (96, 40, 4, 25, 30)]):
        p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=seed + 30)
        for arms, window, explore, batch, t_start in (((1, rep, K_INF), 3, 1 << 30, 1, 0),
                                                      ((2, 1), 1, 0, 2, s_gap * n),
                                                      ((K_INF, 3, 1, 8, 2), 2, 1 << 32, 3, 0),
                                                      ((rep,), 4, 1 << 31, 1, 0),
                                                      ((1, 0), 5, 1 << 29, 4, 7)):
            _say(f"timed adaptive: n={n} arms={arms} window={window} explore={explore} B={batch}")
            _run_timed(p, 0, batch, batch * (u + d), c_num=1, c_den=32, t_start=t_start,
                       adaptive=(list(arms), window, explore, 100 + seed))
    # with random ties as well (the sorting path of the selection reads the same device-side k)
    p, _ = W.shuffled_queue(80, 30, 4, 20, 15, seed=40)
    _run_timed(p, 0, 2, 2 * 50, tie_seed=3, adaptive=([1, 4, K_INF], 2, 1 << 30, 9))


def test_adaptive_k_observe_flags_what_it_cannot_read():
    """Entries of a batch that cannot be read (queue index or query id out of range, a TTFT that was
    never written) are left out of the window and flagged; an over-long batch is cut to the capacity
    given.  The rest of the batch still counts."""
    dev = "cuda:0"
    cap = 16
    qd = K.DeviceQueue.empty(cap, dev)
    qd.id[:6] = torch.tensor([5, 2, 9, 40, -3, 1], dtype=torch.int32, device=dev)
    qd.n.fill_(6)
    ttft = torch.full((12,), -1, dtype=torch.int64, device=dev)
    ttft[5], ttft[2], ttft[9], ttft[1] = 700, 300, 1 << 40, 50
    n_sel = torch.zeros(1, dtype=torch.int32, device=dev)

    def pull(idx, n, batch_cap):
        ad = K.AdaptiveK([3, 7], 1, 0, 0)
        bi = torch.tensor(idx + [0] * (8 - len(idx)), dtype=torch.int32, device=dev)
        n_sel.fill_(n)
        ad.observe(qd, bi, n_sel, batch_cap, ttft)
        return ad.read()

    st = pull([0, 1], 2, 8)
    assert (st.device_error, st.pulls, st.count[0], st.cost[0], st.arm, st.k) == (0, 1, 1, 700, 1, 7)
    st = pull([1, 2, 0], 3, 8)
    assert (st.device_error, st.cost[0]) == (0, 1 << 40)
    st = pull([1, 3], 2, 8)  # id 40 has no TTFT slot
    assert (st.device_error, st.pulls, st.cost[0]) == (4, 1, 300)
    st = pull([4, 5], 2, 8)  # negative id
    assert (st.device_error, st.cost[0]) == (4, 50)
    st = pull([7, 1], 2, 8)  # queue index beyond the queue's length
    assert (st.device_error, st.cost[0]) == (4, 300)
    st = pull([-1, 0], 2, 8)
    assert (st.device_error, st.cost[0]) == (4, 700)
    qd.id[6] = 3  # a query that was never admitted: its TTFT is still -1
    qd.n.fill_(7)
    st = pull([6, 0], 2, 8)
    assert (st.device_error, st.cost[0]) == (4, 700)
    st = pull([0, 1, 5], 3, 2)  # more selected than the capacity given: the first two count
    assert (st.device_error, st.pulls, st.cost[0]) == (8, 1, 700)
    st = pull([0], 0, 8)  # nobody admitted: not a pull
    assert (st.device_error, st.pulls, st.arm, st.k, st.steps_in_window) == (0, 0, 0, 3, 0)
    st = pull([0], -5, 8)
    assert (st.device_error, st.pulls) == (0, 0)


def test_adaptive_k_at_the_paper_shape():
    """n = 2000, 4 queries per shared prefix, u = d = 3000, served after everything has arrived with
    random ties; five arms, windows of 20 steps, a quarter of the pulls exploring."""
    n, rep, u, d, c_num, c_den, s_gap = 2000, 4, 3000, 3000, 1, 1 << 16, 1500
    p, _ = W.shuffled_queue(n, u, rep, d, s_gap, seed=13)
    p.arrival[:] = p.arrival * np.uint64(c_den)
    r = _run_timed(p, 0, 1, u + d, c_num=c_num, c_den=c_den, t_start=s_gap * n * c_den, cap=2048, check_every=500,
                   tie_seed=99, adaptive=([1, 2, rep, 2 * rep, K_INF], 20, 1 << 30, 77))
    assert len(set(r.ks)) == 5


def test_online_stream_with_adaptive_k():
    """The online stream (arrivals per step, LRU eviction under a budget, batches of many queries)
    with k chosen on the device."""
    stream = W.config4_stream(steps=120, rate=40, groups=2000, budget=150_000, batch=32)  # more arrivals than a batch admits
    ad_ref = oracle.AdaptiveK([1, 4, K_INF, 2], 4, 1 << 30, 21)
    r = oracle.simulate_stream(stream, adaptive=ad_ref)
    hq = stream.queries
    q = K.DeviceQueries.from_host(hq)
    cap = 4096
    cfg = K.size_config(0, 0, stream.budget, stream.batch, int(hq.len.max()), extra_prompts=hq.n)
    s = K.Scheduler(cfg, None, cap)
    run = K.OnlineRun(s, q, cap, np.arange(int(stream.step_start[0]), int(stream.step_start[1])))
    ad = K.AdaptiveK([1, 4, K_INF, 2], 4, 1 << 30, 21)
    for step in range(stream.steps):
        nxt = None
        if step + 1 < stream.steps:
            nxt = torch.arange(int(stream.step_start[step + 1]), int(stream.step_start[step + 2]), dtype=torch.int32,
                               device="cuda:0")
        run.step(0x5EED, stream.batch, nxt, adaptive=ad)
    torch.cuda.synchronize()
    assert run.ttft.cpu().numpy().tolist() == r.ttft.tolist()
    assert int(run.sim_clock.item()) == r.clock and int(run.dev_error.item()) == 0
    st = ad.read()
    assert st.device_error == 0 and st.pulls == ad_ref.pulls > 8
    assert (list(st.count)[:4], list(st.cost)[:4], st.arm, st.k) == (ad_ref.count, ad_ref.cost, ad_ref.arm, ad_ref.k())
    assert s.snapshot() == oracle_tree_after(stream, ad=[1, 4, K_INF, 2])


def oracle_tree_after(stream, ad):
    tree = oracle.OracleTree()
    oracle.simulate_stream(stream, tree=tree, adaptive=oracle.AdaptiveK(ad, 4, 1 << 30, 21))
    return tree.snapshot()


# ----------------------------------------------------------------------------- score and tie variants of Algorithm 1
def test_hit_rate_score_and_tie_keys_match_the_oracle():
    rng = np.random.default_rng(31)
    dev = "cuda:0"
    for n in (1, 257, 5000):
        ln = rng.integers(1, 70000, size=n).astype(np.int32)
        m = (rng.random(n) * (ln + 1)).astype(np.int64).clip(0, ln).astype(np.int32)
        m[: n // 8], m[n // 8: n // 4] = 0, ln[n // 8: n // 4]
        d_m, d_ln = torch.from_numpy(m).to(dev), torch.from_numpy(ln).to(dev)
        score = torch.zeros(n, dtype=torch.int32, device=dev)
        for bits in (30, 20, 1):
            K.kLPM_score_hit_rate(d_m, d_ln, n, bits, score)
            assert score.cpu().numpy().tolist() == oracle.score_hit_rate(m, ln, bits).tolist(), (n, bits)
        tie = torch.zeros(n, dtype=torch.int32, device=dev)
        ids = rng.integers(0, 2**31 - 1, size=n).astype(np.int32)
        for seed, step in ((0, 0), (2502046770, 17), ((0xDEADBEEF << 32) | 0x12345678, (5 << 32) | 9)):
            K.kLPM_tie_keys(seed, step, None, n, tie)
            assert tie.cpu().numpy().view(np.uint32).tolist() == oracle.tie_keys(seed, step, np.arange(n)).tolist()
            K.kLPM_tie_keys(seed, step, torch.from_numpy(ids).to(dev), n, tie)
            assert tie.cpu().numpy().view(np.uint32).tolist() == oracle.tie_keys(seed, step, ids).tolist()


def test_select_with_random_ties_and_hit_rate_score():
    rng = np.random.default_rng(37)
    dev = "cuda:0"
    for n in (1, 40, 3000, 20000):
        ws_bytes = K.kLPM_select_workspace_bytes(n)
        ws = K.alloc_aligned(ws_bytes, dev)
        phase = torch.zeros(1, dtype=torch.int32, device=dev)
        nsel = torch.zeros(1, dtype=torch.int32, device=dev)
        live_d = torch.zeros(1, dtype=torch.int32, device=dev)
        ln = rng.integers(1, 3000, size=n).astype(np.int32)
        m = np.minimum(rng.integers(0, 6, size=n) * 500, ln).astype(np.int32)  # few distinct values: big tie classes
        arrival = np.sort(rng.integers(0, max(2, n // 3), size=n)).astype(np.uint64)
        d_arr = torch.from_numpy(arrival.view(np.int64)).to(dev)
        d_m, d_ln = torch.from_numpy(m).to(dev), torch.from_numpy(ln).to(dev)
        score = torch.zeros(n, dtype=torch.int32, device=dev)
        K.kLPM_score_hit_rate(d_m, d_ln, n, 30, score)
        sc_ref = oracle.score_hit_rate(m, ln, 30)
        tie = torch.zeros(n, dtype=torch.int32, device=dev)
        for step, live in ((0, n), (1, max(1, n // 2))):
            K.kLPM_tie_keys(99, step, None, n, tie)
            tie_ref = oracle.tie_keys(99, step, np.arange(n))
            assert tie.cpu().numpy().view(np.uint32).tolist() == tie_ref.tolist()
            live_d.fill_(live)
            for which, d_s, s_ref in (("length", d_m, m), ("rate", score, sc_ref)):
                for k in (1, 2, 7, 0):
                    for batch in (1, 33, 1024):
                        for flags in (0, K.KLPM_SELECT_FIFO):
                            out = torch.full((batch,), -3, dtype=torch.int32, device=dev)
                            phase.fill_(1)
                            K.kLPM_select(d_arr, d_s, n, k, batch, phase, out, nsel, ws, ws_bytes, flags=flags,
                                          max_match=1 << 30, n_live=live_d, tie_key=tie)
                            idx_ref, ph_ref = oracle.select(arrival[:live], s_ref[:live], k, batch, 1, tie_key=tie_ref[:live])
                            got_n = int(nsel.item())
                            assert got_n == idx_ref.shape[0]
                            assert out[:got_n].cpu().numpy().tolist() == idx_ref.tolist(), (n, which, k, batch, flags)
                            assert int(phase.cpu().numpy().view(np.uint32)[0]) == ph_ref
        # tie keys from a tiny range: most ties between equal scores fall through to arrival and index
        K.kLPM_tie_keys(99, 5, None, n, tie)
        tie.bitwise_and_(3)
        tie_ref = oracle.tie_keys(99, 5, np.arange(n)) & np.uint32(3)
        for k in (2, 0):
            for flags in (0, K.KLPM_SELECT_FIFO):
                out = torch.full((512,), -3, dtype=torch.int32, device=dev)
                phase.fill_(1)
                live_d.fill_(n)
                K.kLPM_select(d_arr, d_m, n, k, 512, phase, out, nsel, ws, ws_bytes, flags=flags, max_match=4096,
                              n_live=live_d, tie_key=tie)
                idx_ref, ph_ref = oracle.select(arrival, m, k, 512, 1, tie_key=tie_ref)
                assert out[: int(nsel.item())].cpu().numpy().tolist() == idx_ref.tolist(), (n, k, flags)
        # the hit-rate score without tie keys also runs on the arrival-ordered paths
        for k in (3, 0):
            out = torch.full((64,), -3, dtype=torch.int32, device=dev)
            phase.fill_(0)
            K.kLPM_select(d_arr, score, n, k, 64, phase, out, nsel, ws, ws_bytes, flags=K.KLPM_SELECT_FIFO,
                          max_match=1 << 30)
            idx_ref, _ = oracle.select(arrival, sc_ref, k, 64, 0)
            assert out[: int(nsel.item())].cpu().numpy().tolist() == idx_ref.tolist(), (n, k)


def test_steps_with_hit_rate_score_and_random_ties_keep_the_tree_in_step():
    """Whole steps (match -> score -> tie keys -> select -> commit) under the variant rules."""
    w = W.config0()
    s, ref, q = _setup(w, budget=9000)
    hq = w.queries
    score = torch.zeros(q.n, dtype=torch.int32, device="cuda:0")
    tie = torch.zeros(q.n, dtype=torch.int32, device="cuda:0")
    phase = 0
    for step in range(4):
        m = s.match(q).cpu().numpy()
        m_ref = ref.match(hq.tokens, hq.off, hq.len)
        assert (m == m_ref).all()
        K.kLPM_score_hit_rate(s.match_len, q.len, q.n, 24, score)
        K.kLPM_tie_keys(7, step, None, q.n, tie)
        s.set_phase(phase)
        K.kLPM_select(q.arrival, score, q.n, 3, 32, s.phase, s.batch_idx, s.n_selected, s.ws, s.ws_bytes, tie_key=tie)
        idx_ref, phase = oracle.select(hq.arrival, oracle.score_hit_rate(m_ref, hq.len, 24), 3, 32, phase,
                                       tie_key=oracle.tie_keys(7, step, np.arange(q.n)))
        assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == phase
        s.commit(q, 32)
        ref.commit(hq.tokens, hq.off, hq.len, idx_ref, 9000)
        assert s.read_stats().device_error == 0
        _same_tree(s, ref)


# ----------------------------------------------------------------------------- in-batch rescoring
def _check_dynamic(s, ref, q, hq, ks, batches, live=None, fifo_bound=0):
    """``fifo_bound`` > 0: the queue is promised to be in arrival order with match lengths up to that bound."""
    dev = "cuda:0"
    n = q.n if live is None else min(live, q.n)
    live_d = None if live is None else torch.full((1,), live, dtype=torch.int32, device=dev)
    ql = K.DeviceQueries(q.tokens, q.off, q.len, q.arrival, q.n, n_live=live_d)
    m = s.match(ql, want_nodes=True).cpu().numpy()[:n]
    m_ref = ref.match(hq.tokens, hq.off[:n], hq.len[:n])
    assert (m == m_ref).all()
    ws_bytes = K.kLPM_select_dynamic_workspace_bytes(q.n)
    ws = K.alloc_aligned(ws_bytes, dev)
    dyn = torch.zeros(max(q.n, 1), dtype=torch.int32, device=dev)
    for k in ks:
        for batch in batches:
            out = torch.full((max(batch, 1),), -9, dtype=torch.int32, device=dev)
            s.set_phase(1)
            dyn.fill_(-1)
            K.kLPM_select_dynamic(ql, s.match_len, s.last_node, k, batch, s.phase, dyn, out, s.n_selected, ws, ws_bytes,
                                  flags=K.KLPM_SELECT_FIFO if fifo_bound else 0, max_match=fifo_bound)
            idx_ref, ph_ref, sc_ref = oracle.select_dynamic(hq.tokens, hq.off[:n], hq.len[:n], hq.arrival[:n], m_ref, k,
                                                            batch, 1)
            got_n = int(s.n_selected.item())
            assert got_n == idx_ref.shape[0], (k, batch)
            assert out[:got_n].cpu().numpy().tolist() == idx_ref.tolist(), (k, batch)
            assert s.phase_value() == ph_ref
            assert dyn[:n].cpu().numpy().tolist() == sc_ref.tolist(), (k, batch)


@pytest.mark.parametrize("seed", range(6))
def test_dynamic_select_small_dense(seed):
    w = W.random_small(seed + 300, n_cache=8, n_query=90, vocab=3, max_len=9)
    s, ref, q = _setup(w, max_batch=128)
    _check_dynamic(s, ref, q, w.queries, (1, 2, 3, 70, K_INF), (0, 1, 7, 64, 90, 128))
    _check_dynamic(s, ref, q, w.queries, (2, K_INF), (5, 90), live=37)
    _check_dynamic(s, ref, q, w.queries, (3,), (5,), live=0)


def test_dynamic_select_shuffled_queue_and_duplicates():
    # Def. 3 queue on an empty cache: every query's group is its user's four queries
    p, _ = W.shuffled_queue(400, 50, 4, 30, 1, seed=3)
    w = W.Workload("def3", W.take_prompts(p, np.zeros(0, np.int64)), p, 4, 400, 1 << 40)
    s, ref, q = _setup(w, max_batch=400)
    _check_dynamic(s, ref, q, p, (1, 4, 9, K_INF), (1, 100, 400))
    # config 0 with a block of identical prompts and prompts that are prefixes of one another
    w0 = W.config0()
    hq = w0.queries
    big = int(np.argmax(hq.len))
    extra = [hq.tokens[int(hq.off[big]): int(hq.off[big]) + int(hq.len[big])]] * 12
    extra += [extra[0][: int(hq.len[big]) - 7 * i] for i in range(1, 6)]
    dup = W.generators._from_lists([e.tolist() for e in extra], [3] * len(extra))
    hq2 = W.concat_prompts(hq, dup)
    hq2.arrival[:] = np.sort(hq2.arrival)
    w2 = W.Workload("cfg0+dups", w0.cache, hq2, w0.k, w0.batch, w0.budget)
    s, ref, q = _setup(w2, max_batch=hq2.n)
    _check_dynamic(s, ref, q, hq2, (2, 5, K_INF), (32, hq2.n))


def test_dynamic_select_medium_queue_then_commit():
    """Config-1-like queue (scaled) plus injected near-duplicates; the batch chosen with rescoring
    is committed on both sides and the trees must agree."""
    w = W.config1(scale=0.125)
    hq = w.queries
    rng = np.random.default_rng(5)
    src = rng.integers(0, hq.n, size=300)
    extra = []
    for i in src:
        t = hq.tokens[int(hq.off[i]): int(hq.off[i]) + int(hq.len[i])].copy()
        cut = int(rng.integers(1, t.shape[0] + 1))
        extra.append(np.concatenate([t[:cut], rng.integers(0, 32000, size=int(rng.integers(0, 40))).astype(np.int32)]).tolist())
    hq2 = W.concat_prompts(hq, W.generators._from_lists(extra, rng.integers(0, 1000, size=300).tolist()))
    w2 = W.Workload("cfg1+near-dups", w.cache, hq2, w.k, 256, w.budget)
    s, ref, q = _setup(w2, max_batch=256, extra_prompts=256)
    _say(f"dynamic medium: {hq2.n} waiting, cache {w.cache.n} prompts")
    _check_dynamic(s, ref, q, hq2, (1, 4, K_INF), (256,))
    # the last call's batch (k = infinity, 256 picks) goes into the tree
    idx_ref, _, _ = oracle.select_dynamic(hq2.tokens, hq2.off, hq2.len, hq2.arrival,
                                          ref.match(hq2.tokens, hq2.off, hq2.len), K_INF, 256, 1)
    ws_bytes = K.kLPM_select_dynamic_workspace_bytes(q.n)
    ws = K.alloc_aligned(ws_bytes, "cuda:0")
    dyn = torch.zeros(q.n, dtype=torch.int32, device="cuda:0")
    s.set_phase(1)
    K.kLPM_select_dynamic(q, s.match_len, s.last_node, K_INF, 256, s.phase, dyn, s.batch_idx, s.n_selected, ws, ws_bytes)
    assert s.batch().tolist() == idx_ref.tolist()
    s.commit(q, 256)
    ref.commit(hq2.tokens, hq2.off, hq2.len, idx_ref, w.budget)
    assert s.read_stats().device_error == 0
    _same_tree(s, ref, big=True)


def test_dynamic_select_on_an_arrival_ordered_queue():
    """The same selection told that the queue is in arrival order and how long a match can be (no sort by
    arrival, fewer passes over the match lengths); a queue that breaks either promise is refused."""
    w = W.config1(scale=0.5)
    hq = w.queries
    order = np.argsort(hq.arrival, kind="stable")
    hq = W.take_prompts(hq, order)
    w2 = W.Workload("cfg1-sorted", w.cache, hq, w.k, 256, w.budget)
    s, ref, q = _setup(w2, max_batch=256)
    assert hq.n > 4096
    bound = int(hq.len.max())
    _say(f"dynamic, arrival-ordered: {hq.n} waiting, bound {bound}")
    _check_dynamic(s, ref, q, hq, (1, 4, K_INF), (256,), fifo_bound=bound)
    _check_dynamic(s, ref, q, hq, (3,), (100,), live=hq.n - 1000, fifo_bound=bound)
    ws_bytes = K.kLPM_select_dynamic_workspace_bytes(q.n)
    ws = K.alloc_aligned(ws_bytes, "cuda:0")
    dyn = torch.zeros(q.n, dtype=torch.int32, device="cuda:0")
    m = s.match(q, want_nodes=True).cpu().numpy()
    s.set_phase(2)
    K.kLPM_select_dynamic(q, s.match_len, s.last_node, 4, 64, s.phase, dyn, s.batch_idx, s.n_selected, ws, ws_bytes,
                          flags=K.KLPM_SELECT_FIFO, max_match=max(1, int(m.max()) - 1))
    assert int(s.n_selected.item()) == -1 and s.phase_value() == 2  # a match length above the bound
    arr = hq.arrival.copy()
    arr[hq.n // 2] = arr[hq.n // 2 + 1] + 7
    qbad = K.DeviceQueries(q.tokens, q.off, q.len, torch.from_numpy(arr.view(np.int64)).cuda(), q.n)
    K.kLPM_select_dynamic(qbad, s.match_len, s.last_node, 4, 64, s.phase, dyn, s.batch_idx, s.n_selected, ws, ws_bytes,
                          flags=K.KLPM_SELECT_FIFO, max_match=bound)
    assert int(s.n_selected.item()) == -1 and s.phase_value() == 2  # arrival order broken
    K.kLPM_select_dynamic(qbad, s.match_len, s.last_node, 4, 64, s.phase, dyn, s.batch_idx, s.n_selected, ws, ws_bytes)
    assert int(s.n_selected.item()) == 64  # (no promise made: any order is accepted)


# ----------------------------------------------------------------------------- serving-side variants
@pytest.mark.parametrize("seed", range(4))
def test_eviction_protection_small(seed):
    rng = np.random.default_rng(40 + seed)
    w = W.random_small(seed + 700, n_cache=10, n_query=40, vocab=3, max_len=8)
    s, ref, q = _setup(w, max_batch=8)
    hq = w.queries
    for step in range(8):
        idx = rng.choice(hq.n, size=int(rng.integers(1, 8)), replace=False).astype(np.int32)
        budget, protect = int(rng.integers(0, 30)), int(rng.integers(0, 10))
        s.batch_idx[: idx.shape[0]] = torch.from_numpy(idx).cuda()
        s.n_selected.fill_(idx.shape[0])
        K.kLPM_set_budget(s.tree, budget)
        K.kLPM_set_protect(s.tree, protect)
        s.commit(q, 8)
        st_ref = ref.commit(hq.tokens, hq.off, hq.len, idx, budget, protect=protect)
        st = s.read_stats()
        assert st.device_error == 0
        assert (st.total_tokens, st.evicted_tokens, st.n_nodes, st.evicted_nodes, st.clock) == (
            st_ref.total_tokens, st_ref.evicted_tokens, st_ref.n_nodes, st_ref.evicted_nodes, st_ref.clock), (step, budget, protect)
        _same_tree(s, ref)


def test_eviction_protection_stream():
    """Config-4-like stream with a budget far below what the prompts in flight need: the last two
    batches stay cached whatever the budget says."""
    stream = W.config4_stream(steps=30, rate=24, groups=400, budget=40_000, batch=16)
    hq = stream.queries
    q = K.DeviceQueries.from_host(hq)
    cfg = K.size_config(0, 0, 400_000, stream.batch, int(hq.len.max()), extra_prompts=hq.n)
    s = K.Scheduler(cfg, None, hq.n)
    K.kLPM_set_budget(s.tree, stream.budget)
    K.kLPM_set_protect(s.tree, 2 * stream.batch)
    ref = oracle.OracleTree()
    phase = 0
    for step in range(stream.steps):
        lo, hi = int(stream.step_start[step]), int(stream.step_start[step + 1])
        sub = W.take_prompts(hq, np.arange(lo, hi))
        dq = K.DeviceQueries.from_host(sub)
        m = s.match(dq).cpu().numpy()[: sub.n]
        m_ref = ref.match(sub.tokens, sub.off, sub.len)
        assert (m == m_ref).all()
        s.set_phase(phase)
        s.select(dq, stream.k, stream.batch)
        idx_ref, phase = oracle.select(sub.arrival, m_ref, stream.k, stream.batch, phase)
        assert s.batch().tolist() == idx_ref.tolist()
        s.commit(dq, stream.batch)
        st_ref = ref.commit(sub.tokens, sub.off, sub.len, idx_ref, stream.budget, protect=2 * stream.batch)
        st = s.read_stats()
        assert st.device_error == 0 and (st.total_tokens, st.n_nodes, st.evicted_tokens) == (
            st_ref.total_tokens, st_ref.n_nodes, st_ref.evicted_tokens), step
        if step % 6 == 5:
            _same_tree(s, ref)
    _same_tree(s, ref)


def test_batch_token_budget_cut():
    w = W.config1(scale=0.125)
    s, ref, q = _setup(w, max_batch=256)
    hq = w.queries
    m_ref = ref.match(hq.tokens, hq.off, hq.len)
    live_d = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for live in (hq.n, 100):
        live_d.fill_(live)
        ql = K.DeviceQueries(q.tokens, q.off, q.len, q.arrival, q.n, n_live=live_d)
        s.match(ql)
        for k in (1, 3, 4, K_INF):
            for batch in (1, 17, 256):
                full_ref, ph_full = oracle.select(hq.arrival[:live], m_ref[:live], k, batch, 2)
                cost = (hq.len[full_ref] - m_ref[full_ref]).astype(np.int64)
                for budget in (0, int(cost[0]), int(cost.sum() // 3), int(cost.sum()) - 1, int(cost.sum()), 1 << 40):
                    s.set_phase(2)
                    s.select(ql, k, batch)
                    K.kLPM_batch_token_budget(ql, s.match_len, s.batch_idx, s.n_selected, batch, budget, k, s.phase)
                    keep = oracle.token_budget_cut(full_ref, hq.len, m_ref, budget)
                    assert int(s.n_selected.item()) == keep, (live, k, batch, budget)
                    assert s.batch().tolist() == full_ref[:keep].tolist()
                    assert s.phase_value() == oracle.phase_after_cut(ph_full, full_ref.shape[0], keep, k)
    # a cut batch commits like any other batch
    s.commit(q, 256)
    ref.commit(hq.tokens, hq.off, hq.len, full_ref[:keep], w.budget)
    _same_tree(s, ref, big=True)


def test_kv_slots_identify_cached_tokens():
    """A slot is a function of the cached prefix string: it holds that prefix's last token, equal
    prefixes share it, different prefixes never do; a query has exactly match_len of them."""
    w = W.config0()
    s, ref, q = _setup(w)
    hq = w.queries
    K.kLPM_set_budget(s.tree, 9000)
    for step in range(3):
        m_ref = ref.match(hq.tokens, hq.off, hq.len)
        s.match(q)
        s.set_phase(0)
        s.select(q, 2, 32)
        idx_ref, _ = oracle.select(hq.arrival, m_ref, 2, 32, 0)
        idx = s.batch()
        assert idx.tolist() == idx_ref.tolist()
        stride = int(hq.len.max())
        n_matched = torch.full((32,), -7, dtype=torch.int32, device="cuda:0")
        slots = torch.full((32 * stride,), -1, dtype=torch.int64, device="cuda:0")
        K.kLPM_kv_slots(s.tree, q, s.batch_idx, s.n_selected, 32, stride, n_matched, slots)
        got_n = n_matched.cpu().numpy()
        assert got_n.tolist() == m_ref[idx].tolist()
        toks = torch.zeros(32 * stride, dtype=torch.int32, device="cuda:0")
        K.kLPM_gather_slots(s.tree, slots, toks)
        sl, tk = slots.cpu().numpy().reshape(32, stride), toks.cpu().numpy().reshape(32, stride)
        by_prefix, by_slot = {}, {}
        for j, qi in enumerate(idx.tolist()):
            x = hq.tokens[int(hq.off[qi]): int(hq.off[qi]) + int(hq.len[qi])]
            assert tk[j, : got_n[j]].tolist() == x[: got_n[j]].tolist()       # the slot holds the token
            assert (sl[j, got_n[j]:] == -1).all() and (tk[j, got_n[j]:] == -1).all()  # nothing written past the match
            for t in range(int(got_n[j])):
                key = x[: t + 1].tobytes()
                assert by_prefix.setdefault(key, int(sl[j, t])) == int(sl[j, t])  # same prefix, same slot
                assert by_slot.setdefault(int(sl[j, t]), key) == key              # same slot, same prefix
        s.commit(q, 32)
        ref.commit(hq.tokens, hq.off, hq.len, idx_ref, 9000)
    # fewer picks than the capacity: the rest of n_matched is 0; a short stride cuts the rows
    s.n_selected.fill_(3)
    K.kLPM_kv_slots(s.tree, q, s.batch_idx, s.n_selected, 32, 16, n_matched, slots)
    got = n_matched.cpu().numpy()
    want = np.minimum(ref.match(hq.tokens, hq.off, hq.len)[s.batch_idx[:3].cpu().numpy()], 16)
    assert got[:3].tolist() == want.tolist() and (got[3:] == 0).all()


# ----------------------------------------------------------------------------- replay from a captured HIP graph
def test_graph_replay_of_scheduling_steps():
    """A scheduling step with a device-side queue length has fixed launch shapes, so it can be
    captured once per queue buffer set and replayed; every replay must leave what the eager step
    leaves (checked against the oracle's run step by step, with host reads between replays)."""
    n, u, rep, d, gap = 96, 40, 4, 25, 30
    p, _ = W.shuffled_queue(n, u, rep, d, gap, seed=21)
    k, batch, budget, cap = 3, 2, 4 * (u + d), 32
    r = oracle.simulate_timed(p, k, batch, budget, c_num=1, c_den=128, queue_cap=cap)
    q = K.DeviceQueries.from_host(p)
    cfg = K.size_config(0, 0, budget, batch, int(p.len.max()), extra_prompts=2 * batch)
    s = K.Scheduler(cfg, None, cap)
    run = K.TimedRun(s, q, cap, p.arrival, c_num=1, c_den=128)
    K.kLPM_reserve_clock(s.tree, n + 8)
    # two eager steps first (they also bring every kernel's code onto the device)
    done = 0
    for _ in range(2):
        run.step(k, batch)
        done += 1
    torch.cuda.synchronize()
    graphs = {}
    for _ in range(2):  # one graph per buffer set; capturing enqueues nothing
        parity = run.cur
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run.step(k, batch)
        graphs[parity] = g
    assert set(graphs) == {0, 1} and run.cur in (0, 1)
    while done < r.steps:
        n_live = int(run.queue.n.item())
        ids = run.queue.id[:n_live].cpu().numpy()
        assert ids.tolist() == r.waiting_ids[done].tolist(), done
        graphs[run.cur].replay()
        run.cur = 1 - run.cur
        torch.cuda.synchronize()
        assert s.match_len[:n_live].cpu().numpy().tolist() == r.match_lens[done].tolist(), done
        assert ids[s.batch()].tolist() == r.batches[done].tolist(), done
        st = s.read_stats()  # host work between replays
        assert st.device_error == 0
        done += 1
    assert int(run.queue.n.item()) == 0 and int(run.sim_clock.item()) == r.clock
    assert run.ttft[:n].cpu().numpy().tolist() == r.ttft.tolist()


# ----------------------------------------------------------------------------- sizes at the far end
def _short_prompts(rng, n, vocab, lo, hi, arrival=None):
    ln = rng.integers(lo, hi + 1, size=n).astype(np.int32)
    off = np.zeros(n, np.int64)
    off[1:] = np.cumsum(ln[:-1])
    tok = rng.integers(0, vocab, size=int(ln.sum())).astype(np.int32)
    arr = np.arange(n, dtype=np.uint64) if arrival is None else arrival
    return W.Prompts(tok, off, ln, arr)


def test_million_query_queue():
    """A queue of a million short prompts (heavy prefix sharing over a small alphabet): match of all
    of them, selection on the arrival-ordered paths and on the sorting path."""
    rng = np.random.default_rng(61)
    cache = _short_prompts(rng, 3000, 6, 3, 14)
    n = 1_000_000
    hq = _short_prompts(rng, n, 6, 2, 12)
    w = W.Workload("million", cache, hq, 8, 1024, 1 << 40)
    s, ref, q = _setup(w, max_batch=4096)
    m = s.match(q).cpu().numpy()
    m_ref = ref.match(hq.tokens, hq.off, hq.len, threads=8)
    assert (m == m_ref).all()
    for k, batch, fifo in ((8, 1024, True), (K_INF, 4096, True), (3, 300, False)):
        _say(f"million queue: select k={k} B={batch} fifo={fifo}")
        s.set_phase(2)
        s.select(q, k, batch, fifo=fifo)
        idx_ref, ph_ref = oracle.select(hq.arrival, m_ref, k, batch, 2)
        assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref
    # unsorted arrival times with many ties: only the sorting path applies
    arr2 = rng.integers(0, 1000, size=n).astype(np.uint64)
    d_arr2 = torch.from_numpy(arr2.view(np.int64)).cuda()
    q2 = K.DeviceQueries(q.tokens, q.off, q.len, d_arr2, q.n)
    s.set_phase(0)
    s.select(q2, 5, 512)
    idx_ref, ph_ref = oracle.select(arr2, m_ref, 5, 512, 0)
    assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref


def test_groups_larger_than_a_wavefront():
    """Dozens to hundreds of admitted prompts that stop at the same place of the tree: stops inside one long
    edge at many depths (with and without an own tail; cut for all of them at once by one wavefront, one to
    four prompts per lane, or - beyond 256 - inserted one after the other, which makes more table entries
    than the wavefront keeps a record of), and a common new prefix below the root.  Both kinds of commit,
    then a second batch on top of the first."""
    rng = np.random.default_rng(83)
    long = rng.integers(0, 1000, size=600).astype(np.int32)
    cache = W.generators._from_lists([long.tolist()], [0])

    def batch_of(n_each):
        out = []
        for _ in range(n_each):  # tokens >= 1000 never continue the cached edge
            cut = int(rng.integers(1, 600))
            out.append(long[:cut].tolist() + (1000 + rng.integers(0, 3, size=int(rng.integers(0, 6)))).tolist())
        for _ in range(n_each):
            out.append([2000, 2001] + rng.integers(0, 3, size=int(rng.integers(0, 9))).tolist())
        order = rng.permutation(len(out))
        return [out[i] for i in order]

    for n_each in (40, 70, 130, 230, 300):  # one prompt per lane; two, three, four per lane; the serial road
        lists = batch_of(n_each) + batch_of(n_each)
        hq = W.generators._from_lists(lists, list(range(len(lists))))
        n = len(lists)
        w = W.Workload("one-group", cache, hq, 1, n // 2, 1 << 40)
        s, ref, q = _setup(w, max_batch=n // 2, extra_prompts=n)
        _say(f"large groups: {n_each} prompts inside one edge and {n_each} below a new prefix, twice")
        # FCFS takes the first half, then (the picks are not removed from this queue) longest match
        # takes those again or their equals: every prompt is present by then, ticks only
        ph = _check_step(s, ref, q, hq, 1, n // 2, 0, 1 << 40, fifo=True)
        _check_step(s, ref, q, hq, K_INF, n // 2, ph, 1 << 40, fifo=True)
        # the second half on top of the first: pieces of the old edge are cut again
        tail = W.take_prompts(hq, np.arange(n // 2, n))
        q2 = K.DeviceQueries.from_host(tail, "cuda:0")
        _check_step(s, ref, q2, tail, 1, n // 2, 0, 1 << 40, fifo=True)


@pytest.mark.parametrize("donor_len,n_members", [(160, 60), (160, 200), (1500, 40)])
def test_near_duplicates_of_an_uncached_prompt(donor_len, n_members):
    """One batch of prompts that all repeat the head of the same string, which the cache does not hold, each
    for a length of its own, before a tail of their own: they stop at one node boundary with the same next
    token and form one group whose members agree with each other for longer than with the group's first
    prompt, level after level (the classes that settle among themselves in the structure pass; with the
    long string the agreement exceeds what a lane compares by itself).  Exact duplicates, prompts that are
    prefixes of others and prompts that end inside the common part are among them."""
    rng = np.random.default_rng(1234 + donor_len + n_members)
    prefix = rng.integers(0, 1000, size=40).astype(np.int32)
    cache = W.generators._from_lists([prefix.tolist() + [5000, 5001]], [0])
    donor = rng.integers(1000, 2000, size=donor_len).astype(np.int32)
    lists = []
    for i in range(n_members):
        c = int(rng.integers(1, donor_len + 1))
        kind = int(rng.integers(0, 6))
        tail = [] if kind == 0 else (3000 + rng.integers(0, 3 if kind == 1 else 100000, size=int(rng.integers(1, 6)))).tolist()
        lists.append(prefix.tolist() + donor[:c].tolist() + tail)
    lists += [lists[3], lists[7], lists[3]]  # exact duplicates
    order = rng.permutation(len(lists))
    lists = [lists[i] for i in order]
    n = len(lists)
    hq = W.generators._from_lists(lists, list(range(n)))
    w = W.Workload("near-duplicates", cache, hq, 1, n, 1 << 40)
    s, ref, q = _setup(w, max_batch=n, extra_prompts=2 * n)
    _say(f"near duplicates: {n} prompts repeating up to {donor_len} tokens of one uncached string")
    ph = _check_step(s, ref, q, hq, 1, n, 0, 1 << 40, fifo=True)
    _check_step(s, ref, q, hq, K_INF, n, ph, 1 << 40, fifo=True)  # everything is cached by now: ticks only
    _check_step(s, ref, q, hq, 2, n // 2, 0, 300, fifo=True)      # and under eviction pressure


@pytest.mark.parametrize("n_prompts,batch", [(900, 450), (3000, 1500), (1100, 513), (2100, 1023), (4200, 2047), (4200, 2049)])
def test_batches_that_share_new_prefixes_at_several_levels(n_prompts, batch):
    """Admitted prompts of the shape prefix + first c tokens of a donor string + own tail, several per
    donor with different c, some equal, some a prefix of another: behind the place where they leave
    the old tree they share new prefixes of different lengths, level below level.  The cached prompt
    of a prefix either continues it (the batch stops inside that edge, at the prefix end and at
    other depths) or ends with it (the batch stops at a node boundary).  Batches of up to 512, 1,024
    and 2,048 prompts and larger ones take different plan kernels and structure passes; sizes that are
    no multiple of the plan's group of four leave its last workgroup a partial group."""
    rng = np.random.default_rng(97)
    n_pref = 12
    prefixes = [rng.integers(0, 50, size=int(rng.integers(40, 300))).tolist() for _ in range(n_pref)]
    for p_i in range(n_pref):
        prefixes[p_i][0] = 100 + p_i  # distinct first tokens
    cached = [p + (rng.integers(50, 60, size=int(rng.integers(5, 400))).tolist() if i % 2 else []) for i, p in enumerate(prefixes)]
    cache = W.generators._from_lists(cached, list(range(n_pref)))
    donors = [[rng.integers(60, 64, size=200).tolist() for _ in range(3)] for _ in range(n_pref)]
    lists = []
    for _ in range(n_prompts):
        g = int(rng.integers(0, n_pref))
        kind = rng.random()
        if kind < 0.15:   # stops somewhere inside the prefix (or the cached continuation)
            base = cached[g][: int(rng.integers(1, len(cached[g]) + 1))]
            lists.append(base + rng.integers(70, 73, size=int(rng.integers(0, 4))).tolist())
            continue
        d = donors[g][int(rng.integers(0, 3))]
        c = int(rng.choice([0, 1, 2, 5, 5, 17, 64, 64, 130, 200]))
        own = rng.integers(80, 83, size=int(rng.choice([0, 0, 1, 3, 40]))).tolist()
        lists.append(prefixes[g] + d[:c] + own)
    hq = W.generators._from_lists(lists, list(range(len(lists))))
    w = W.Workload("levels", cache, hq, 3, batch, 1 << 40)
    s, ref, q = _setup(w, max_batch=batch, extra_prompts=len(lists))
    ph = _check_step(s, ref, q, hq, 3, batch, 0, 1 << 40, fifo=True)
    rest = W.take_prompts(hq, np.setdiff1d(np.arange(hq.n), s.batch()))
    q2 = K.DeviceQueries.from_host(rest, "cuda:0")
    ph = _check_step(s, ref, q2, rest, 3, batch, ph, 1 << 40, fifo=True)
    # once more under a budget that evicts part of what the two batches built
    _check_step(s, ref, q, hq, K_INF, batch * 2 // 3, ph, ref.total_tokens // 2, fifo=True)


def test_largest_batch_and_very_long_prompts():
    """A commit of 65,536 prompts at once (the largest batch a configuration may name), and prompts
    of several hundred thousand tokens (edges far longer than any window of the match kernel)."""
    rng = np.random.default_rng(67)
    # 65,536 tiny prompts over 3,000 first tokens: about 20 prompts per root child, deep sharing
    hq = _short_prompts(rng, 65536, 3000, 1, 4)
    empty = W.take_prompts(hq, np.zeros(0, np.int64))
    w = W.Workload("max-batch", empty, hq, 4, 65536, 1 << 40)
    s, ref, q = _setup(w, max_batch=65536)
    m = s.match(q).cpu().numpy()
    assert (m == 0).all()
    s.set_phase(0)
    s.select(q, 4, 65536)  # more than the arrival-ordered kernels take: the sorting path
    idx_ref, ph_ref = oracle.select(hq.arrival, m, 4, 65536, 0)
    assert s.batch().tolist() == idx_ref.tolist() and s.phase_value() == ph_ref
    s.commit(q, 65536)
    st_ref = ref.commit(hq.tokens, hq.off, hq.len, idx_ref, 1 << 40)
    st = s.read_stats()
    assert st.device_error == 0 and (st.total_tokens, st.n_nodes, st.clock) == (st_ref.total_tokens, st_ref.n_nodes, st_ref.clock)
    _same_tree(s, ref, big=True)
    # then evict most of it in one go
    K.kLPM_set_budget(s.tree, 5000)
    s.n_selected.fill_(0)
    s.commit(q, 0)
    ref.commit(hq.tokens, hq.off, hq.len, np.zeros(0, np.int32), 5000)
    assert s.read_stats().total_tokens <= 5000
    _same_tree(s, ref, big=True)

    # very long prompts: a 400,000-token prompt, a copy that differs in its last token, a copy cut in
    # the middle of the edge, one diverging at token 300,001, and an unrelated one
    base = rng.integers(0, 32000, size=400_000).astype(np.int32)
    a = base.copy()
    b = base.copy(); b[-1] ^= 1
    c = base[:123_457].copy()
    d = np.concatenate([base[:300_001], rng.integers(0, 32000, size=50_000).astype(np.int32)]); d[300_001] = (base[300_001] + 1) % 32000
    e = rng.integers(0, 32000, size=200_000).astype(np.int32); e[0] = (base[0] + 1) % 32000
    hq = W.generators._from_lists([a, b, c, d, e], [0, 1, 2, 3, 4])
    empty = W.take_prompts(hq, np.zeros(0, np.int64))
    w = W.Workload("long", empty, hq, 1, 5, 1 << 40)
    s, ref, q = _setup(w, max_batch=5, max_len=400_000)
    _check_step(s, ref, q, hq, 1, 5, 0, 1 << 40, big=True)   # all five in one batch, in arrival order
    m = s.match(q).cpu().numpy()
    assert m.tolist() == hq.len.tolist() == ref.match(hq.tokens, hq.off, hq.len).tolist()
    # and a budget that keeps only the most recent path
    _check_step(s, ref, q, hq, K_INF, 1, 0, 250_000, big=True)


def test_eviction_cut_inside_a_tick_with_thousands_of_nodes():
    """A chain of 9,000 one-token nodes, all stamped by one prompt (the full string inserted last):
    the eviction cut then falls among more nodes of a single tick than the sorting pass holds, and
    the search has to finish with digit passes over the depth."""
    rng = np.random.default_rng(71)
    n = 9000
    base = rng.integers(0, 32000, size=n).astype(np.int32)
    # prompts = prefixes of one string, shortest first: every insertion appends a one-token node
    ln = np.arange(1, n + 1, dtype=np.int32)
    off = np.zeros(n, np.int64)
    tok = np.tile(base, 1)
    cache = W.Prompts(tok, off, ln, np.arange(n, dtype=np.uint64))  # all prompts share the one token buffer
    other = _short_prompts(rng, 64, 32000, 40, 80)
    full = W.generators._from_lists([base.tolist()], [0])
    hq = W.concat_prompts(full, other)
    w = W.Workload("chain", cache, hq, 1, 8, 1 << 40)
    s, ref, q = _setup(w, max_batch=64, max_len=n)
    assert K.kLPM_read_stats(s.tree).n_nodes == n
    # the full string stamps all 9,000 nodes with one tick; then a few unrelated prompts
    for batch_ids, budget in (([0], 1 << 40), (list(range(1, 9)), n - 100), (list(range(9, 17)), 5000),
                              (list(range(17, 25)), 4321), (list(range(25, 33)), 700), (list(range(33, 41)), 0)):
        idx = np.array(batch_ids, dtype=np.int32)
        s.batch_idx[: idx.shape[0]] = torch.from_numpy(idx).cuda()
        s.n_selected.fill_(idx.shape[0])
        K.kLPM_set_budget(s.tree, budget)
        s.commit(q, 64)
        st_ref = ref.commit(hq.tokens, hq.off, hq.len, idx, budget)
        st = s.read_stats()
        assert st.device_error == 0
        assert (st.total_tokens, st.evicted_tokens, st.n_nodes, st.evicted_nodes) == (
            st_ref.total_tokens, st_ref.evicted_tokens, st_ref.n_nodes, st_ref.evicted_nodes), budget
        _same_tree(s, ref, big=True)


# ----------------------------------------------------------------------------- everything mixed
@pytest.mark.parametrize("seed", range(6))
def test_mixed_operations_against_the_oracle(seed, n_query=120, max_batch=32, steps=25, max_len=10):
    """Random sequences of scheduling steps over small, densely sharing workloads, each step drawing
    its own variant: score (length / hit rate), ties (arrival / random keys), rescoring (per step /
    in batch), queue promise (arrival-ordered or not), prefill token budget, KV budget, protection
    window, a device-side queue length, k from the host or from device memory, and a commit that
    matches again or takes the step's match.  Batch, phase and tree are compared after every step."""
    rng = np.random.default_rng(8800 + seed)
    w = W.random_small(seed + 900, n_cache=12, n_query=n_query, vocab=3, max_len=max_len, arrival_hi=1000)
    hq = w.queries
    order = np.argsort(hq.arrival, kind="stable")
    hq = W.take_prompts(hq, order)  # a queue in arrival order, so that either selection path applies
    w = W.Workload("mixed", w.cache, hq, 2, 16, 1 << 40)
    s, ref, q = _setup(w, max_batch=max_batch, extra_prompts=steps * max_batch)
    dev = "cuda:0"
    score = torch.zeros(q.n, dtype=torch.int32, device=dev)
    tie = torch.zeros(q.n, dtype=torch.int32, device=dev)
    dyn = torch.zeros(q.n, dtype=torch.int32, device=dev)
    dws_bytes = K.kLPM_select_dynamic_workspace_bytes(q.n)
    dws = K.alloc_aligned(dws_bytes, dev)
    live_d = torch.zeros(1, dtype=torch.int32, device=dev)
    k_d = torch.zeros(1, dtype=torch.int32, device=dev)
    phase = 0
    for step in range(steps):
        live = int(rng.integers(1, q.n + 1))
        k = int(rng.choice([1, 2, 3, 5, K_INF]))
        k_d.copy_(torch.from_numpy(np.array([k], dtype=np.uint32).view(np.int32)))
        k_dev = k_d.data_ptr() if rng.integers(0, 3) == 0 else None
        k_arg = 0x5EED if k_dev is not None else k  # with a device-side k the host's value must not matter
        batch = int(rng.integers(1, max_batch + 1))
        budget = int(rng.choice([1 << 40, 400, 150, 60]))
        protect = int(rng.choice([0, 0, 5, 40]))
        variant = rng.choice(["plain", "fifo", "rate", "ties", "dynamic", "token_budget"])
        live_d.fill_(live)
        ql = K.DeviceQueries(q.tokens, q.off, q.len, q.arrival, q.n, n_live=live_d)
        m = s.match(ql, want_nodes=True).cpu().numpy()[:live]
        m_ref = ref.match(hq.tokens, hq.off[:live], hq.len[:live])
        assert (m == m_ref).all(), (step, variant)
        s.set_phase(phase)
        arr = hq.arrival[:live]
        if variant == "dynamic":
            K.kLPM_select_dynamic(ql, s.match_len, s.last_node, k_arg, batch, s.phase, dyn, s.batch_idx, s.n_selected, dws,
                                  dws_bytes, k_dev=k_dev)
            idx_ref, phase, sc_ref = oracle.select_dynamic(hq.tokens, hq.off[:live], hq.len[:live], arr, m_ref, k, batch, phase)
            assert dyn[:live].cpu().numpy().tolist() == sc_ref.tolist(), (step, variant)
        elif variant == "rate":
            K.kLPM_score_hit_rate(s.match_len, q.len, q.n, 20, score, n_live=live_d)
            s.select(ql, k_arg, batch, fifo=bool(rng.integers(0, 2)), score=score, score_max=1 << 20, k_dev=k_dev)
            idx_ref, phase = oracle.select(arr, oracle.score_hit_rate(m_ref, hq.len[:live], 20), k, batch, phase)
        elif variant == "ties":
            K.kLPM_tie_keys(seed, step, None, q.n, tie, n_live=live_d)
            s.select(ql, k_arg, batch, tie_key=tie, fifo=bool(rng.integers(0, 2)), k_dev=k_dev)
            idx_ref, phase = oracle.select(arr, m_ref, k, batch, phase, tie_key=oracle.tie_keys(seed, step, np.arange(live)))
        else:
            s.select(ql, k_arg, batch, fifo=(variant != "plain"), k_dev=k_dev)
            idx_ref, ph = oracle.select(arr, m_ref, k, batch, phase)
            if variant == "token_budget":
                tb = int(rng.integers(0, 60))
                K.kLPM_batch_token_budget(ql, s.match_len, s.batch_idx, s.n_selected, batch, tb, k_arg, s.phase, k_dev=k_dev)
                keep = oracle.token_budget_cut(idx_ref, hq.len, m_ref, tb)
                ph = oracle.phase_after_cut(ph, idx_ref.shape[0], keep, k)
                idx_ref = idx_ref[:keep]
            phase = ph
        assert s.batch().tolist() == idx_ref.tolist(), (step, variant, k, batch, live)
        assert s.phase_value() == phase, (step, variant)
        K.kLPM_set_budget(s.tree, budget)
        K.kLPM_set_protect(s.tree, protect)
        s.commit(ql, max_batch, reuse_match=bool(rng.integers(0, 2)))
        st_ref = ref.commit(hq.tokens, hq.off, hq.len, idx_ref, budget, protect=protect)
        st = s.read_stats()
        assert st.device_error == 0
        assert (st.total_tokens, st.n_nodes, st.evicted_tokens, st.clock) == (
            st_ref.total_tokens, st_ref.n_nodes, st_ref.evicted_tokens, st_ref.clock), (step, variant, budget, protect)
        _same_tree(s, ref)
