"""CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrapper over ``klpm_oracle.c`` plus the pure-Python parts of the
reference: the online-stream simulation (waiting queue bookkeeping, simulated
clock, TTFT) and the nearest-rank percentile.  Only tests, the smoke check and
the benchmark's CPU-baseline leg may import this package; the GPU library and
its binding never do.

Paper passages followed: Algorithm 1 (k-LPM), Def. 1 (query stream), Def. 2
(completion-time model, used with c_attn = 0 for the simulated prefill cost),
Sec. 2.1 (bins of B queries finish together; fixed memory pool), Sec. 1
(radix-tree prefix cache with LRU eviction); ``simulate_timed`` follows Def. 2's
timeline with the attention term (c_attn >= 0) on queries that arrive at their
own times (Def. 1, Def. 3); ``score_hit_rate`` and ``tie_keys`` are the hit-rate
score of Algorithm 1's wording and the uniformly random tie-break assumed by the
theory (footnote of Sec. 4.2), the latter drawn from Philox-4x32-10 (SC'11).
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "klpm_oracle.c")
_LIB = os.path.join(_HERE, "libklpm_oracle.so")

K_INF = 0xFFFFFFFF


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-pthread", "-o", _LIB, _SRC])
    return _LIB


class _Stats(C.Structure):
    _fields_ = [
        ("total_tokens", C.c_int64), ("inserted_tokens", C.c_int64), ("evicted_tokens", C.c_int64),
        ("n_nodes", C.c_int32), ("new_nodes", C.c_int32), ("evicted_nodes", C.c_int32), ("pad", C.c_int32),
        ("clock", C.c_uint64),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, i32, i64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32
        L.orc_tree_new.restype = vp
        L.orc_tree_free.argtypes = [vp]
        L.orc_total_tokens.restype = i64; L.orc_total_tokens.argtypes = [vp]
        L.orc_n_nodes.restype = i64; L.orc_n_nodes.argtypes = [vp]
        L.orc_clock.restype = C.c_uint64; L.orc_clock.argtypes = [vp]
        L.orc_match.argtypes = [vp, vp, vp, vp, i32, vp]
        L.orc_match_mt.argtypes = [vp, vp, vp, vp, i32, vp, i32]
        L.orc_select.restype = i32
        L.orc_select.argtypes = [vp, vp, vp, i32, u32, i32, C.POINTER(u32), vp]
        L.orc_commit.argtypes = [vp, vp, vp, vp, vp, i32, i64, i64, C.POINTER(_Stats)]
        L.orc_snapshot_bytes.restype = C.c_size_t; L.orc_snapshot_bytes.argtypes = [vp]
        L.orc_snapshot.restype = C.c_size_t; L.orc_snapshot.argtypes = [vp, vp, C.c_size_t]
        L.orc_select_dynamic.restype = i32
        L.orc_select_dynamic.argtypes = [vp, vp, vp, vp, vp, i32, u32, i32, C.POINTER(u32), vp]
        L.orc_def2.argtypes = [vp, vp, vp, vp, vp, i32, C.c_double, C.c_double, vp]
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


@dataclass
class CommitStats:
    total_tokens: int
    inserted_tokens: int
    evicted_tokens: int
    n_nodes: int
    new_nodes: int
    evicted_nodes: int
    clock: int


class OracleTree:
    """Pointer-based radix tree over token strings with per-node last-use ticks."""

    def __init__(self):
        self._L = _load()
        self._t = self._L.orc_tree_new()

    def __del__(self):
        try:
            if self._t:
                self._L.orc_tree_free(self._t)
                self._t = None
        except Exception:
            pass

    @property
    def total_tokens(self) -> int:
        return int(self._L.orc_total_tokens(self._t))

    @property
    def n_nodes(self) -> int:
        return int(self._L.orc_n_nodes(self._t))

    @property
    def clock(self) -> int:
        return int(self._L.orc_clock(self._t))

    def match(self, tokens, off, length, threads: int = 1) -> np.ndarray:
        tokens, off, length = _c(tokens, np.int32), _c(off, np.int64), _c(length, np.int32)
        out = np.zeros(length.shape[0], dtype=np.int32)
        if threads <= 1:
            self._L.orc_match(self._t, _p(tokens), _p(off), _p(length), length.shape[0], _p(out))
        else:
            self._L.orc_match_mt(self._t, _p(tokens), _p(off), _p(length), length.shape[0], _p(out), threads)
        return out

    def commit(self, tokens, off, length, batch_idx, budget: int, protect: int = 0) -> CommitStats:
        """``protect``: the paths of that many most recently admitted prompts (this batch included)
        are in flight and are never evicted, even if the total then stays above the budget."""
        tokens, off, length = _c(tokens, np.int32), _c(off, np.int64), _c(length, np.int32)
        batch_idx = _c(batch_idx, np.int32)
        st = _Stats()
        self._L.orc_commit(self._t, _p(tokens), _p(off), _p(length), _p(batch_idx), batch_idx.shape[0],
                           int(min(budget, (1 << 62))), int(protect), C.byref(st))
        return CommitStats(st.total_tokens, st.inserted_tokens, st.evicted_tokens, st.n_nodes, st.new_nodes,
                           st.evicted_nodes, st.clock)

    def build(self, prompts) -> CommitStats:
        """Insert the initial cached prompts in order, ticks 0..P-1, no eviction."""
        return self.commit(prompts.tokens, prompts.off, prompts.len, np.arange(prompts.n, dtype=np.int32), 1 << 62)

    def snapshot(self) -> bytes:
        n = int(self._L.orc_snapshot_bytes(self._t))
        buf = np.zeros(n, dtype=np.uint8)
        got = int(self._L.orc_snapshot(self._t, _p(buf), n))
        assert got == n
        return buf.tobytes()


def select(arrival, match_len, k: int, batch: int, phase: int = 0, tie_key=None) -> Tuple[np.ndarray, int]:
    """Algorithm 1 over a static score vector, cut at ``batch`` picks. Returns (batch_idx, phase_out).

    ``match_len`` is the score (any int32 vector: match lengths, or ``score_hit_rate``); ``tie_key``
    (uint32 per query, optional) decides between equal scores before the arrival time does.
    """
    L = _load()
    arrival, match_len = _c(arrival, np.uint64), _c(match_len, np.int32)
    n = arrival.shape[0]
    tie = None if tie_key is None else _c(tie_key, np.uint32)
    assert tie is None or tie.shape[0] == n
    out = np.zeros(max(0, min(batch, n)), dtype=np.int32)
    ph = C.c_uint32(phase)
    got = L.orc_select(_p(arrival), _p(match_len), None if tie is None else _p(tie), n, C.c_uint32(k & 0xFFFFFFFF),
                       batch, C.byref(ph), _p(out))
    return out[:got], int(ph.value)


def select_dynamic(prompts_tokens, off, length, arrival, match_len, k: int, batch: int,
                   phase: int = 0) -> Tuple[np.ndarray, int, np.ndarray]:
    """Algorithm 1 with in-batch rescoring: after every pick p the score of each remaining query i
    becomes max(score_i, overlap(x_i, x_p)) - the cache holds what it has processed (Sec. 1), and
    Def. 2 credits a query with what the prompts before it left there.  Returns (batch_idx,
    phase_out, scores): a picked query's entry of ``scores`` is its score when it was picked."""
    L = _load()
    tok, off, ln = _c(prompts_tokens, np.int32), _c(off, np.int64), _c(length, np.int32)
    arrival = _c(arrival, np.uint64)
    score = np.array(match_len, dtype=np.int32, copy=True)
    n = arrival.shape[0]
    assert off.shape[0] == n and ln.shape[0] == n and score.shape[0] == n
    out = np.zeros(max(0, min(batch, n)), dtype=np.int32)
    ph = C.c_uint32(phase)
    got = L.orc_select_dynamic(_p(tok), _p(off), _p(ln), _p(arrival), _p(score), n, C.c_uint32(k & 0xFFFFFFFF), batch,
                               C.byref(ph), _p(out))
    return out[:got], int(ph.value), score


def token_budget_cut(batch_idx, length, match_len, token_budget: int) -> int:
    """Dynamic batch size (Sec. 2.1): of the picks in order, keep the longest prefix whose uncached
    tokens sum(|x| - m) fit the prefill token budget; the first pick always stays (a prompt longer
    than the budget must still run some time).  Returns how many picks are kept."""
    total, keep = 0, 0
    for j, i in enumerate(np.asarray(batch_idx).tolist()):
        total += max(0, int(length[i]) - max(0, int(match_len[i])))
        if j > 0 and total > token_budget:
            break
        keep = j + 1
    return keep


def phase_after_cut(phase_after: int, n_selected: int, n_kept: int, k: int) -> int:
    """Position in the k-cycle once the picks beyond ``n_kept`` have been handed back."""
    if k in (0, K_INF):
        return 0
    return (phase_after - (n_selected - n_kept)) % k


def score_hit_rate(match_len, length, scale_bits: int = 30) -> np.ndarray:
    """Prefix-cache hit *rate* of each query (the wording of Algorithm 1) as an integer score:
    floor(m * 2^scale_bits / |x|).  Exact as an order of the rationals m/|x| whenever
    |x| <= 2^(scale_bits/2); beyond that nearly equal rates may share a score."""
    m = np.maximum(np.asarray(match_len, dtype=np.int64), 0)
    ln = np.asarray(length, dtype=np.int64)
    assert 1 <= scale_bits <= 30 and (ln >= 1).all() and (m <= ln).all()
    return ((m << scale_bits) // ln).astype(np.int32)


_PHILOX_M0, _PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key) -> Tuple[int, int, int, int]:
    """Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as
    1, 2, 3", SC'11): a keyed bijection of a 128-bit counter; each round multiplies two counter
    words by fixed odd constants, swaps the halves around and mixes in the key, which moves on by a
    Weyl constant per round."""
    c0, c1, c2, c3 = (int(v) & 0xFFFFFFFF for v in counter)
    k0, k1 = (int(v) & 0xFFFFFFFF for v in key)
    for r in range(10):
        if r:
            k0, k1 = (k0 + _PHILOX_W0) & 0xFFFFFFFF, (k1 + _PHILOX_W1) & 0xFFFFFFFF
        p0, p1 = _PHILOX_M0 * c0, _PHILOX_M1 * c2
        c0, c1, c2, c3 = (p1 >> 32) ^ c1 ^ k0, p1 & 0xFFFFFFFF, (p0 >> 32) ^ c3 ^ k1, p0 & 0xFFFFFFFF
    return c0, c1, c2, c3


def tie_keys(seed: int, step: int, ids) -> np.ndarray:
    """One uniform 32-bit tie key per query and scheduling step: word 0 of Philox-4x32-10 at counter
    (id, 0, step low, step high) under the key (seed low, seed high).  Redrawn every step, so a
    query's luck does not persist; independent of where the query sits in the queue.
    (The same rounds as ``philox4x32_10``, on numpy arrays of 64-bit words.)"""
    mask = np.uint64(0xFFFFFFFF)
    c0 = np.asarray(ids, dtype=np.int64).astype(np.uint64) & mask
    c1 = np.zeros_like(c0)
    c2 = np.full_like(c0, step & 0xFFFFFFFF)
    c3 = np.full_like(c0, (step >> 32) & 0xFFFFFFFF)
    k0, k1 = seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF
    for r in range(10):
        if r:
            k0, k1 = (k0 + _PHILOX_W0) & 0xFFFFFFFF, (k1 + _PHILOX_W1) & 0xFFFFFFFF
        p0, p1 = np.uint64(_PHILOX_M0) * c0, np.uint64(_PHILOX_M1) * c2
        c0, c1, c2, c3 = ((p1 >> np.uint64(32)) ^ c1 ^ np.uint64(k0), p1 & mask,
                          (p0 >> np.uint64(32)) ^ c3 ^ np.uint64(k1), p0 & mask)
    return c0.astype(np.uint32)


ADAPT_TAG = 0x6B4C504D  # third counter word of the draws below ("kLPM"), keeps them apart from the tie keys


class AdaptiveK:
    """k chosen per window of scheduling steps by an epsilon-greedy bandit over a list of k values.

    Sec. 4.2 says that k can be set by back-testing or by an adaptive multi-armed bandit and leaves
    the method open; this is the textbook epsilon-greedy rule with these choices: a pull lasts
    ``window`` scheduling steps; its cost is the largest TTFT among the queries admitted during
    those steps (the tail is what k-LPM is about, Thm. 2); a window that admitted nobody is not a
    pull and leaves everything as it was.  After a pull: an arm never pulled yet goes next (lowest
    index first); otherwise words (w0, w1, ., .) of Philox-4x32-10 at counter (pulls low, pulls high,
    ADAPT_TAG, 0) under key (seed low, seed high) decide - explore arm w1 mod A if w0 < ``explore``
    (probability explore / 2^32), else the arm with the smallest mean cost, compared as exact
    fractions, the lower index on equality.
    """

    def __init__(self, arms, window: int, explore: int, seed: int):
        assert len(arms) >= 1 and window >= 1 and 0 <= explore <= 1 << 32
        self.arms = [int(a) for a in arms]
        self.window, self.explore, self.seed = int(window), int(explore), int(seed)
        self.count = [0] * len(self.arms)
        self.cost = [0] * len(self.arms)
        self.arm, self.steps, self.pulls = 0, 0, 0
        self.cur_max, self.cur_n = 0, 0

    def k(self) -> int:
        return self.arms[self.arm]

    def observe(self, ttfts) -> None:
        """Called once per scheduling step with the TTFT of every query that step admitted."""
        for t in ttfts:
            self.cur_max = max(self.cur_max, int(t))
            self.cur_n += 1
        self.steps += 1
        if self.steps < self.window:
            return
        self.steps = 0
        if self.cur_n > 0:
            self.count[self.arm] += 1
            self.cost[self.arm] += self.cur_max
            self.pulls += 1
            self.arm = self._next_arm()
        self.cur_max, self.cur_n = 0, 0

    def _next_arm(self) -> int:
        from fractions import Fraction

        A = len(self.arms)
        for a in range(A):
            if self.count[a] == 0:
                return a
        w = philox4x32_10((self.pulls & 0xFFFFFFFF, (self.pulls >> 32) & 0xFFFFFFFF, ADAPT_TAG, 0),
                          (self.seed & 0xFFFFFFFF, (self.seed >> 32) & 0xFFFFFFFF))
        if w[0] < self.explore:
            return w[1] % A
        best = 0
        for a in range(1, A):
            if Fraction(self.cost[a], self.count[a]) < Fraction(self.cost[best], self.count[best]):
                best = a
        return best


def def2_completion(prompts, order, c_attn: float = 0.0, t_start: float = 0.0) -> np.ndarray:
    """Completion time R(.) of every query (indexed by query, not by position) under Def. 2."""
    L = _load()
    order = _c(order, np.int32)
    out = np.zeros(prompts.n, dtype=np.float64)
    L.orc_def2(_p(_c(prompts.tokens, np.int32)), _p(_c(prompts.off, np.int64)), _p(_c(prompts.len, np.int32)),
               _p(_c(prompts.arrival, np.uint64)), _p(order), order.shape[0], float(c_attn), float(t_start), _p(out))
    return out


def percentile_nearest_rank(values, p: float) -> int:
    """Nearest-rank percentile of an integer array: sorted[ceil(p*n) - 1]."""
    v = np.sort(np.asarray(values))
    if v.shape[0] == 0:
        return 0
    r = max(1, int(math.ceil(p * v.shape[0])))
    return int(v[r - 1])


def schedule_with_tree(prompts, k: int, budget: int, t_start: int = 0, batch: int = 1) -> np.ndarray:
    """Run match -> select -> commit over a fixed queue until it is empty.

    With ``batch = 1`` and ``budget`` = one prompt length this is the
    last-prompt cache of Def. 2 driven through the radix-tree pipeline.  All
    queries are taken to be waiting from the start (processing begins at
    ``t_start`` >= every arrival).  Returns the processing order.
    """
    tree = OracleTree()
    waiting = np.arange(prompts.n, dtype=np.int64)
    phase = 0
    order: List[int] = []
    while waiting.shape[0]:
        off, ln, arr = prompts.off[waiting], prompts.len[waiting], prompts.arrival[waiting]
        m = tree.match(prompts.tokens, off, ln)
        idx, phase = select(arr, m, k, batch, phase)
        tree.commit(prompts.tokens, off, ln, idx, budget)
        order.extend(int(waiting[i]) for i in idx)
        keep = np.ones(waiting.shape[0], dtype=bool)
        keep[idx] = False
        waiting = waiting[keep]
    return np.array(order, dtype=np.int32)


@dataclass
class StreamResult:
    ttft: np.ndarray  # int64 per query (-1 if never admitted)
    admitted_step: np.ndarray  # int32 per query
    batches: List[np.ndarray]  # global query ids in pick order, per step
    match_lens: List[np.ndarray]  # match lengths of the waiting queue, per step
    waiting_ids: List[np.ndarray]  # global query ids of the waiting queue, per step
    clock: int  # simulated time after the last step
    stats: List[CommitStats]
    snapshots: List[Optional[bytes]]


def simulate_stream(stream, snapshot_every: int = 0, tree: Optional[OracleTree] = None,
                    adaptive: Optional[AdaptiveK] = None) -> StreamResult:
    """Online simulation: each step, enqueue that step's arrivals at the current simulated
    time, score the whole waiting queue, pick a k-LPM batch (phase persists across steps),
    commit it under the KV budget, then advance time by the batch's prefill cost.

    Prefill cost of a query is its uncached token count |x| - m (Def. 2 with c_attn = 0,
    m measured at step start); a batch finishes together (Sec. 2.1); time advances by
    max(1, total cost); TTFT = finish time - enqueue time.  With ``adaptive`` each step runs with
    the k that object holds and reports the TTFT of the queries it admitted to it.
    """
    q = stream.queries
    tree = tree or OracleTree()
    n = q.n
    ttft = np.full(n, -1, dtype=np.int64)
    adm = np.full(n, -1, dtype=np.int32)
    enq = np.zeros(n, dtype=np.uint64)
    waiting = np.zeros(0, dtype=np.int64)
    clock = 0
    phase = 0
    res = StreamResult(ttft, adm, [], [], [], 0, [], [])
    for s in range(stream.steps):
        new = np.arange(int(stream.step_start[s]), int(stream.step_start[s + 1]), dtype=np.int64)
        enq[new] = clock
        waiting = np.concatenate([waiting, new])
        off, ln, arr = q.off[waiting], q.len[waiting], enq[waiting]
        m = tree.match(q.tokens, off, ln)
        k_now = stream.k if adaptive is None else adaptive.k()
        idx, phase = select(arr, m, k_now, stream.batch, phase)
        st = tree.commit(q.tokens, off, ln, idx, stream.budget)
        cost = int((ln[idx].astype(np.int64) - m[idx].astype(np.int64)).sum())
        clock += max(1, cost)
        gids = waiting[idx]
        ttft[gids] = clock - enq[gids].astype(np.int64)
        adm[gids] = s
        if adaptive is not None:
            adaptive.observe(ttft[gids].tolist())
        res.batches.append(gids.copy())
        res.match_lens.append(m)
        res.waiting_ids.append(waiting.copy())
        res.stats.append(st)
        res.snapshots.append(tree.snapshot() if snapshot_every and (s + 1) % snapshot_every == 0 else None)
        keep = np.ones(waiting.shape[0], dtype=bool)
        keep[idx] = False
        waiting = waiting[keep]
    res.clock = clock
    return res


@dataclass
class TimedResult:
    ttft: np.ndarray  # int64 per query, in clock units (-1 if never admitted)
    order: np.ndarray  # query ids in processing order
    batches: List[np.ndarray]  # query ids in pick order, per step
    match_lens: List[np.ndarray]  # match lengths of the waiting queue, per step
    waiting_ids: List[np.ndarray]  # query ids of the waiting queue, per step
    clock: int  # time at which the last batch finished
    steps: int
    ks: List[int] = field(default_factory=list)  # the k each step ran with


def simulate_timed(prompts, k: int, batch: int, budget: int, c_num: int = 0, c_den: int = 1, t_start: int = 0,
                   queue_cap: Optional[int] = None, tree: Optional[OracleTree] = None,
                   tie_seed: Optional[int] = None, adaptive: Optional[AdaptiveK] = None) -> TimedResult:
    """Def. 2's timeline driven through match -> select -> commit, with queries that become
    visible to the scheduler only once they have arrived (Def. 1: arrival time t_i).

    Time is an integer count of units of 1/c_den of one token's linear prefill time; arrival times
    are given in that unit.  A query costs (|x| - m)(c_den + c_num |x|) units, i.e.
    (1 + c_attn |x|)(|x| - m) token times with c_attn = c_num / c_den (Def. 2); m is its match
    length at the start of the step; the batch finishes together (Sec. 2.1), and nothing starts
    before it has arrived: when nobody is waiting the clock jumps to the next arrival
    (the max(R, t) of Def. 2).  With batch = 1 and budget = one prompt this is Def. 2 itself.
    ``queue_cap`` bounds the waiting queue; arrivals that find it full stay outside, in arrival
    order, keeping their arrival time.  With ``tie_seed`` equal match lengths are ordered by the
    uniformly random keys of ``tie_keys`` (drawn per query id and step; footnote of Sec. 4.2).
    With ``adaptive`` each step runs with the k that object holds (``k`` is ignored) and reports the
    TTFT of the queries it admitted to it.
    """
    n = prompts.n
    arr = np.asarray(prompts.arrival, dtype=np.uint64)
    pending = np.lexsort((np.arange(n), arr))  # by (arrival, id)
    cap = n if queue_cap is None else int(queue_cap)
    tree = tree or OracleTree()
    ttft = np.full(n, -1, dtype=np.int64)
    res = TimedResult(ttft, np.zeros(0, np.int32), [], [], [], int(t_start), 0)
    waiting: List[int] = []
    cursor, clock, phase = 0, int(t_start), 0
    order: List[int] = []
    while True:
        while cursor < n and len(waiting) < cap and int(arr[pending[cursor]]) <= clock:
            waiting.append(int(pending[cursor]))
            cursor += 1
        if not waiting:
            if cursor == n:
                break
            clock = int(arr[pending[cursor]])  # idle until the next arrival
            continue
        w = np.array(waiting, dtype=np.int64)
        off, ln = prompts.off[w], prompts.len[w]
        m = tree.match(prompts.tokens, off, ln)
        tk = None if tie_seed is None else tie_keys(tie_seed, res.steps, w)
        k_now = k if adaptive is None else adaptive.k()
        idx, phase = select(arr[w], m, k_now, batch, phase, tie_key=tk)
        tree.commit(prompts.tokens, off, ln, idx, budget)
        cost = 0
        for i in idx.tolist():
            x = int(ln[i])
            cost += (x - int(m[i])) * (c_den + c_num * x)
        clock += cost
        gids = w[idx]
        ttft[gids] = clock - arr[gids].astype(np.int64)
        res.ks.append(k_now)
        if adaptive is not None:
            adaptive.observe(ttft[gids].tolist())
        order.extend(int(g) for g in gids)
        res.batches.append(gids.astype(np.int32))
        res.match_lens.append(m)
        res.waiting_ids.append(w.astype(np.int32))
        res.steps += 1
        gone = set(idx.tolist())
        waiting = [q for i, q in enumerate(waiting) if i not in gone]
    res.order = np.array(order, dtype=np.int32)
    res.clock = clock
    return res
