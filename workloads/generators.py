"""Synthetic prefix-sharing workloads (inputs only, no scheduling arithmetic).

All token strings are returned in CSR form: one flat ``int32`` token array plus
``off`` (int64 start), ``len`` (int32 length) and ``arrival`` (uint64 integer
ticks, the t_i of the query-stream definition, Def. 1).  Every generator is a
pure function of its seed.

The shapes follow the paper's workload model: tree-structured prompts of low
height, ``(base_prompt)(user_context)(doc)`` (Sec. 4.1), a few prompts per long
shared prefix with context lengths of several thousand tokens (Sec. 5), and the
Regular Arrival Shuffled Queue (Def. 3).  Token values are i.i.d. uniform over
a 32,000-word vocabulary unless copied, so distinct prefixes share a first
token now and then, the "non-zero negligible reuse" the paper's appendix C.2
footnote mentions for its own random strings.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

VOCAB = 32000
SEED_BASE = 2502046770
# Encodes "k = infinity" (pure longest-prefix-match order) for the scheduler.
K_LPM_ENDPOINT = 0xFFFFFFFF


@dataclass
class Prompts:
    """A set of token strings with arrival ticks, in CSR layout."""

    tokens: np.ndarray  # int32 [sum(len)]
    off: np.ndarray  # int64 [n]
    len: np.ndarray  # int32 [n]
    arrival: np.ndarray  # uint64 [n]

    @property
    def n(self) -> int:
        return int(self.len.shape[0])

    def prompt(self, i: int) -> np.ndarray:
        o = int(self.off[i])
        return self.tokens[o : o + int(self.len[i])]

    def as_lists(self) -> List[List[int]]:
        return [self.prompt(i).tolist() for i in range(self.n)]


@dataclass
class Workload:
    name: str
    cache: Prompts  # prompts already processed (initial tree contents, in order)
    queries: Prompts  # the waiting queue
    k: int
    batch: int
    budget: int  # KV budget in tokens; a value >= all tokens means "no eviction"
    ks: Sequence[int] = field(default_factory=tuple)  # optional sweep over k
    extra: Optional[Prompts] = None  # later arrivals (used to refill the queue)


@dataclass
class Stream:
    """An online stream: query i arrives at scheduling step ``step_of[i]``."""

    name: str
    queries: Prompts  # arrival field is unused (assigned by the simulation)
    step_start: np.ndarray  # int64 [steps+1]; step s owns [step_start[s], step_start[s+1])
    k: int
    batch: int
    budget: int

    @property
    def steps(self) -> int:
        return int(self.step_start.shape[0] - 1)


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------

def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


def _from_lists(seqs: Sequence[Sequence[int]], arrival: Optional[Sequence[int]] = None) -> Prompts:
    lens = np.array([len(s) for s in seqs], dtype=np.int32)
    off = np.zeros(len(seqs), dtype=np.int64)
    if len(seqs):
        off[1:] = np.cumsum(lens[:-1], dtype=np.int64)
    toks = np.zeros(int(lens.sum()), dtype=np.int32)
    for i, s in enumerate(seqs):
        toks[off[i] : off[i] + lens[i]] = np.asarray(s, dtype=np.int32)
    if arrival is None:
        arr = np.arange(len(seqs), dtype=np.uint64)
    else:
        arr = np.asarray(arrival, dtype=np.uint64)
    return Prompts(toks, off, lens, arr)


def concat_prompts(a: Prompts, b: Prompts) -> Prompts:
    """``a`` followed by ``b`` sharing one token array."""
    toks = np.concatenate([a.tokens, b.tokens])
    off = np.concatenate([a.off, b.off + a.tokens.shape[0]])
    return Prompts(toks, off, np.concatenate([a.len, b.len]), np.concatenate([a.arrival, b.arrival]))


def concat_all(parts: Sequence[Prompts]) -> Prompts:
    """The prompt sets one after the other, sharing one token array."""
    base = np.cumsum([0] + [p.tokens.shape[0] for p in parts[:-1]])
    return Prompts(np.concatenate([p.tokens for p in parts]),
                   np.concatenate([p.off + b for p, b in zip(parts, base)]),
                   np.concatenate([p.len for p in parts]), np.concatenate([p.arrival for p in parts]))


def take_prompts(p: Prompts, idx: np.ndarray) -> Prompts:
    """Sub-selection that keeps sharing the token array (offsets are re-used)."""
    idx = np.asarray(idx, dtype=np.int64)
    return Prompts(p.tokens, p.off[idx].copy(), p.len[idx].copy(), p.arrival[idx].copy())


def _zipf_cdf(groups: int, s: float) -> np.ndarray:
    w = np.arange(1, groups + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def _zipf_draw(rng: np.random.Generator, cdf: np.ndarray, n: int) -> np.ndarray:
    g = np.searchsorted(cdf, rng.random(n), side="right")
    return np.minimum(g, cdf.shape[0] - 1).astype(np.int64)


def _csr_offsets(lens: np.ndarray) -> np.ndarray:
    off = np.zeros(lens.shape[0], dtype=np.int64)
    if lens.shape[0] > 1:
        off[1:] = np.cumsum(lens[:-1], dtype=np.int64)
    return off


class _Fresh:
    """Hands out slices of one big uniform-random token array."""

    def __init__(self, rng: np.random.Generator, total: int):
        self.buf = rng.integers(0, VOCAB, size=int(total), dtype=np.int32)
        self.pos = 0

    def take(self, n: int) -> np.ndarray:
        out = self.buf[self.pos : self.pos + n]
        self.pos += n
        return out


def _grouped_cache(rng, group_of: np.ndarray, prefix_tok, prefix_off, prefix_len, suffix_len: np.ndarray) -> Prompts:
    """Cached prompts: group prefix followed by a fresh suffix."""
    n = group_of.shape[0]
    lens = (prefix_len[group_of] + suffix_len).astype(np.int32)
    off = _csr_offsets(lens)
    toks = np.empty(int(lens.sum(dtype=np.int64)), dtype=np.int32)
    fresh = _Fresh(rng, int(suffix_len.sum(dtype=np.int64)))
    for i in range(n):
        g = int(group_of[i])
        pl = int(prefix_len[g])
        o = int(off[i])
        po = int(prefix_off[g])
        toks[o : o + pl] = prefix_tok[po : po + pl]
        sl = int(suffix_len[i])
        toks[o + pl : o + pl + sl] = fresh.take(sl)
    return Prompts(toks, off, lens, np.arange(n, dtype=np.uint64))


def _grouped_queries(
    rng,
    n: int,
    derived: np.ndarray,  # bool [n]
    group_of: np.ndarray,  # int64 [n] (ignored where not derived)
    prefix_tok,
    prefix_off,
    prefix_len,
    donors_by_group,  # dict: group -> list of (kind, ref, suffix start, suffix len)
    copy_max: int,
    tail_lo: int,
    tail_hi: int,
    fresh_lo: int,
    fresh_hi: int,
    register_as_donor: bool = False,
) -> Prompts:
    """Waiting queries: either group prefix + copied suffix head + fresh tail, or fully fresh."""
    copy_want = rng.integers(0, copy_max + 1, size=n)
    tail_len = rng.integers(tail_lo, tail_hi + 1, size=n)
    fresh_len = rng.integers(fresh_lo, fresh_hi + 1, size=n)
    donor_pick = rng.random(n)
    # first pass: lengths
    copy_len = np.zeros(n, dtype=np.int64)
    donor_sel: List[Optional[tuple]] = [None] * n
    lens = np.empty(n, dtype=np.int64)
    toks_parts_total = 0
    for i in range(n):
        if derived[i]:
            g = int(group_of[i])
            dl = donors_by_group.get(g)
            c = 0
            if dl:
                d = dl[int(donor_pick[i] * len(dl)) % len(dl)]
                c = min(int(copy_want[i]), d[3])
                donor_sel[i] = d
            copy_len[i] = c
            lens[i] = int(prefix_len[g]) + c + int(tail_len[i])
            if register_as_donor:
                # the suffix of this prompt (copy + tail) becomes a donor for later ones;
                # its tokens live in the output array, filled in below, so remember (i, start, len)
                donors_by_group.setdefault(g, []).append((1, i, int(prefix_len[g]), c + int(tail_len[i])))
        else:
            lens[i] = int(fresh_len[i])
        toks_parts_total += int(lens[i])
    lens32 = lens.astype(np.int32)
    off = _csr_offsets(lens32)
    toks = np.empty(toks_parts_total, dtype=np.int32)
    n_fresh_tokens = int(np.where(derived, tail_len, fresh_len).sum())
    fresh = _Fresh(rng, n_fresh_tokens)
    for i in range(n):
        o = int(off[i])
        if derived[i]:
            g = int(group_of[i])
            pl = int(prefix_len[g])
            po = int(prefix_off[g])
            toks[o : o + pl] = prefix_tok[po : po + pl]
            c = int(copy_len[i])
            if c:
                d = donor_sel[i]
                if d[0] == 1:  # donor is an earlier prompt of this same output array
                    src_o = int(off[d[1]]) + d[2]
                    toks[o + pl : o + pl + c] = toks[src_o : src_o + c]
                else:  # donor is a suffix inside an external token array
                    toks[o + pl : o + pl + c] = d[1][d[2] : d[2] + c]
            tl = int(tail_len[i])
            toks[o + pl + c : o + pl + c + tl] = fresh.take(tl)
        else:
            fl = int(fresh_len[i])
            toks[o : o + fl] = fresh.take(fl)
    return Prompts(toks, off, lens32, np.arange(n, dtype=np.uint64))


def _donors_from_cache(cache: Prompts, group_of: np.ndarray, prefix_len: np.ndarray):
    donors = {}
    for i in range(cache.n):
        g = int(group_of[i])
        pl = int(prefix_len[g])
        donors.setdefault(g, []).append((0, cache.tokens, int(cache.off[i]) + pl, int(cache.len[i]) - pl))
    return donors


def _make_prefixes(rng, lens: np.ndarray):
    off = _csr_offsets(lens.astype(np.int32))
    tok = rng.integers(0, VOCAB, size=int(lens.sum(dtype=np.int64)), dtype=np.int32)
    return tok, off, lens.astype(np.int64)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config0(seed: int = SEED_BASE + 0) -> Workload:
    """Tiny single step: 16 groups x 128-token prefix, 64 cached prompts, 256 queries."""
    groups = 16
    ptok, poff, plen = _make_prefixes(_rng(seed, 0), np.full(groups, 128))
    rc = _rng(seed, 1)
    group_of = np.repeat(np.arange(groups, dtype=np.int64), 4)
    suffix = rc.integers(64, 257, size=group_of.shape[0])
    cache = _grouped_cache(rc, group_of, ptok, poff, plen, suffix)
    rq = _rng(seed, 2)
    n = 256
    derived = rq.random(n) < 0.75
    qgroup = rq.integers(0, groups, size=n)
    donors = _donors_from_cache(cache, group_of, plen)
    queries = _grouped_queries(rq, n, derived, qgroup, ptok, poff, plen, donors, 128, 32, 256, 64, 512)
    return Workload("cfg0-tiny", cache, queries, k=2, batch=32, budget=1 << 40)


def config1(seed: int = SEED_BASE + 1, scale: float = 1.0) -> Workload:
    """Medium Zipf step: 200 groups (Zipf 1.1), 1024-token prefix, 10,000 cached prompts, 16,384 queries."""
    groups = 200
    n_cache = max(8, int(round(10000 * scale)))
    n = max(8, int(round(16384 * scale)))
    cdf = _zipf_cdf(groups, 1.1)
    ptok, poff, plen = _make_prefixes(_rng(seed, 0), np.full(groups, 1024))
    rc = _rng(seed, 1)
    group_of = _zipf_draw(rc, cdf, n_cache)
    suffix = rc.integers(128, 2049, size=n_cache)
    cache = _grouped_cache(rc, group_of, ptok, poff, plen, suffix)
    rq = _rng(seed, 2)
    derived = rq.random(n) < 0.90
    qgroup = _zipf_draw(rq, cdf, n)
    donors = _donors_from_cache(cache, group_of, plen)
    queries = _grouped_queries(rq, n, derived, qgroup, ptok, poff, plen, donors, 128, 32, 2944, 256, 4096)
    ra = _rng(seed, 3)
    gaps = ra.exponential(1.0, size=n)
    queries.arrival = np.floor(np.cumsum(gaps) * float(1 << 20)).astype(np.uint64)
    return Workload("cfg1-medium-zipf", cache, queries, k=4, batch=256, budget=1 << 40)


def config2(seed: int = SEED_BASE + 2, scale: float = 1.0, extra_queries: int = 0) -> Workload:
    """Large single step: ~100M-token cache from 50,000 Zipf(1.0) groups, 65,536 queries.

    ``scale`` shrinks the token target, the group count and the queue together
    (used by tests); ``extra_queries`` generates later arrivals from the same
    recipe so a harness can keep the queue full over several steps.
    """
    groups = max(16, int(round(50000 * scale)))
    target = int(100_000_000 * scale)
    n = max(16, int(round(65536 * scale)))
    batch = max(4, int(round(1024 * scale)))
    cdf = _zipf_cdf(groups, 1.0)
    rp = _rng(seed, 0)
    plen_draw = rp.integers(512, 4097, size=groups)
    ptok, poff, plen = _make_prefixes(rp, plen_draw)
    rc = _rng(seed, 1)
    # draw candidates, then cut where the tree would first hold >= target tokens
    # (a group's prefix counts once, every suffix counts in full)
    cand = max(64, int(target / 2000) + 1024)
    group_of = _zipf_draw(rc, cdf, cand)
    suffix = rc.integers(256, 4097, size=cand)
    first = np.zeros(cand, dtype=bool)
    _, first_idx = np.unique(group_of, return_index=True)
    first[first_idx] = True
    tree_tokens = np.cumsum(suffix + np.where(first, plen[group_of], 0))
    n_cache = int(np.searchsorted(tree_tokens, target, side="left")) + 1
    n_cache = min(n_cache, cand)
    group_of = group_of[:n_cache]
    suffix = suffix[:n_cache]
    cache = _grouped_cache(rc, group_of, ptok, poff, plen, suffix)
    donors = _donors_from_cache(cache, group_of, plen)

    def draw(rq, nq):
        derived = rq.random(nq) < 0.85
        qgroup = _zipf_draw(rq, cdf, nq)
        return _grouped_queries(rq, nq, derived, qgroup, ptok, poff, plen, donors, 128, 32, 3968, 64, 8192)

    # (the later arrivals are drawn batch by batch from streams of their own, so the queue and the
    # first arrivals are the same whatever the number asked for)
    queries = draw(_rng(seed, 2), n)
    parts = [draw(_rng(seed, 1000 + c), min(batch, int(extra_queries) - c * batch))
             for c in range((int(extra_queries) + batch - 1) // batch)]
    extra = concat_all(parts) if parts else None
    return Workload("cfg2-large", cache, queries, k=8, batch=batch, budget=target, extra=extra)


def config2_deep(seed: int = SEED_BASE + 12, scale: float = 1.0, extra_queries: int = 0) -> Workload:
    """Deep-tree variant of the large step: same token target, about 50 tokens per node.

    Suffixes are short walks over a per-group pool of 32-64-token segments, so
    many prompts share whole segments and the tree gets one to two new nodes
    per prompt with only a segment or two of new tokens each.
    """
    groups = max(8, int(round(8192 * scale)))
    target = int(100_000_000 * scale)
    n = max(16, int(round(65536 * scale)))
    batch = max(4, int(round(1024 * scale)))
    pool_segments = 16
    cdf = _zipf_cdf(groups, 1.0)
    rp = _rng(seed, 0)
    ptok, poff, plen = _make_prefixes(rp, rp.integers(512, 4097, size=groups))
    seg_len = rp.integers(32, 65, size=(groups, pool_segments))
    seg_off = _csr_offsets(seg_len.reshape(-1).astype(np.int32)).reshape(groups, pool_segments)
    seg_tok = rp.integers(0, VOCAB, size=int(seg_len.sum()), dtype=np.int32)
    rc = _rng(seed, 1)
    seen = set()
    tree_tokens = 0
    plist = []
    chunk = 65536
    while tree_tokens < target:
        gs = _zipf_draw(rc, cdf, chunk)
        depth = rc.integers(1, 5, size=chunk)
        picks = rc.integers(0, pool_segments, size=(chunk, 4))
        for i in range(chunk):
            g = int(gs[i])
            if (g,) not in seen:
                seen.add((g,))
                tree_tokens += int(plen[g])
            key = (g,)
            for lvl in range(int(depth[i])):
                key = key + (int(picks[i, lvl]),)
                if key not in seen:
                    seen.add(key)
                    tree_tokens += int(seg_len[g, picks[i, lvl]])
            plist.append((g, tuple(int(v) for v in picks[i, : int(depth[i])])))
            if tree_tokens >= target:
                break

    def assemble(items):
        lens = np.array([int(plen[g]) + sum(int(seg_len[g, s]) for s in segs) for g, segs in items], dtype=np.int32)
        off = _csr_offsets(lens)
        toks = np.empty(int(lens.sum(dtype=np.int64)), dtype=np.int32)
        for i, (g, segs) in enumerate(items):
            o = int(off[i])
            pl = int(plen[g])
            toks[o : o + pl] = ptok[int(poff[g]) : int(poff[g]) + pl]
            o += pl
            for s in segs:
                sl = int(seg_len[g, s])
                so = int(seg_off[g, s])
                toks[o : o + sl] = seg_tok[so : so + sl]
                o += sl
        return Prompts(toks, off, lens, np.arange(len(items), dtype=np.uint64))

    cache = assemble(plist)
    def draw(rq, nq):
        qg = _zipf_draw(rq, cdf, nq)
        qdepth = rq.integers(1, 7, size=nq)
        qpicks = rq.integers(0, pool_segments, size=(nq, 6))
        return assemble([(int(qg[i]), tuple(int(v) for v in qpicks[i, : int(qdepth[i])])) for i in range(nq)])

    # (the later arrivals are drawn batch by batch from streams of their own, so the queue and the
    # first arrivals are the same whatever the number asked for)
    queries = draw(_rng(seed, 2), n)
    parts = [draw(_rng(seed, 1000 + c), min(batch, int(extra_queries) - c * batch))
             for c in range((int(extra_queries) + batch - 1) // batch)]
    extra = concat_all(parts) if parts else None
    return Workload("cfg2-deep", cache, queries, k=8, batch=batch, budget=target, extra=extra)


def config3(seed: int = SEED_BASE + 3, scale: float = 1.0) -> Workload:
    """Hierarchical prefixes: 8 system prompts x 64 few-shot blocks x user turns."""
    n_sys, n_blk = 8, 64
    n_cache = max(64, int(round(200000 * scale)))
    n = max(16, int(round(32768 * scale)))
    batch = max(4, int(round(512 * scale)))
    rp = _rng(seed, 0)
    sys_tok = rp.integers(0, VOCAB, size=(n_sys, 2048), dtype=np.int32)
    blk_tok = rp.integers(0, VOCAB, size=(n_sys * n_blk, 512), dtype=np.int32)
    cdf = _zipf_cdf(n_sys * n_blk, 1.0)
    # rank -> (system, block) pair through a fixed shuffle so popular pairs spread over systems
    perm = rp.permutation(n_sys * n_blk)

    def build(rng, pairs, turn_parts):
        """turn_parts[i] = list of arrays forming the user turn of prompt i."""
        lens = np.array([2048 + 512 + sum(p.shape[0] for p in parts) for parts in turn_parts], dtype=np.int32)
        off = _csr_offsets(lens)
        toks = np.empty(int(lens.sum(dtype=np.int64)), dtype=np.int32)
        for i, parts in enumerate(turn_parts):
            o = int(off[i])
            pr = int(pairs[i])
            toks[o : o + 2048] = sys_tok[pr // n_blk]
            toks[o + 2048 : o + 2560] = blk_tok[pr]
            o += 2560
            for p in parts:
                toks[o : o + p.shape[0]] = p
                o += p.shape[0]
        return Prompts(toks, off, lens, np.arange(len(turn_parts), dtype=np.uint64))

    rc = _rng(seed, 1)
    cpairs = perm[_zipf_draw(rc, cdf, n_cache)]
    cturn = rc.integers(32, 513, size=n_cache)
    fresh = _Fresh(rc, int(cturn.sum()))
    cparts = [[fresh.take(int(t))] for t in cturn]
    cache = build(rc, cpairs, cparts)
    by_pair = {}
    for i in range(n_cache):
        by_pair.setdefault(int(cpairs[i]), []).append(i)
    rq = _rng(seed, 2)
    qpairs = perm[_zipf_draw(rq, cdf, n)]
    reuse = rq.random(n) < 0.5
    cwant = rq.integers(0, 129, size=n)
    qturn = rq.integers(32, 513, size=n)
    dpick = rq.random(n)
    qfresh = _Fresh(rq, int(qturn.sum()))
    qparts = []
    for i in range(n):
        parts = []
        lst = by_pair.get(int(qpairs[i]))
        if reuse[i] and lst:
            j = lst[int(dpick[i] * len(lst)) % len(lst)]
            c = min(int(cwant[i]), int(cturn[j]))
            if c:
                parts.append(cparts[j][0][:c])
        parts.append(qfresh.take(int(qturn[i])))
        qparts.append(parts)
    queries = build(rq, qpairs, qparts)
    ks = (1, 2, 4, 8, 1, K_LPM_ENDPOINT)  # "k=1" and the FCFS endpoint are the same setting
    return Workload("cfg3-hierarchical", cache, queries, k=4, batch=batch, budget=1 << 40, ks=ks)


def config4_stream(seed: int = SEED_BASE + 4, steps: int = 1000, rate: float = 128.0,
                   groups: int = 50000, budget: int = 4_000_000, batch: int = 256) -> Stream:
    """Online stream: Poisson(rate) arrivals per step from the large-step group recipe.

    The cache starts empty; a group-derived query copies the head of the suffix
    of an earlier stream prompt of its group (if there is one).
    """
    cdf = _zipf_cdf(groups, 1.0)
    rp = _rng(seed, 0)
    ptok, poff, plen = _make_prefixes(rp, rp.integers(512, 4097, size=groups))
    ra = _rng(seed, 3)
    per_step = ra.poisson(rate, size=steps).astype(np.int64)
    step_start = np.zeros(steps + 1, dtype=np.int64)
    step_start[1:] = np.cumsum(per_step)
    n = int(step_start[-1])
    rq = _rng(seed, 2)
    derived = rq.random(n) < 0.85
    qgroup = _zipf_draw(rq, cdf, n)
    donors = {}
    queries = _grouped_queries(rq, n, derived, qgroup, ptok, poff, plen, donors, 128, 32, 3968, 64, 8192,
                               register_as_donor=True)
    queries.arrival = np.zeros(n, dtype=np.uint64)
    return Stream("cfg4-online", queries, step_start, k=4, batch=batch, budget=budget)


def refill_arrivals(w: Workload, step: int, count: int) -> Prompts:
    """The ``count`` later arrivals that join the queue after scheduling step ``step``."""
    assert w.extra is not None and (step + 1) * count <= w.extra.n
    return take_prompts(w.extra, np.arange(step * count, (step + 1) * count))


# --------------------------------------------------------------------------
# the paper's analytic workloads
# --------------------------------------------------------------------------

def shuffled_queue(n: int, u: int, k: int, d: int, s: int, seed: int = SEED_BASE + 100):
    """Regular Arrival Shuffled Queue (Def. 3).

    ``n/k`` user substrings of length ``u`` each shared by exactly ``k``
    queries, ``n`` unique doc substrings of length ``d``; every substring
    starts with its own distinct token, the rest is random.  Query j (in
    generation order, user ``j // k``) gets arrival time ``s * sigma(j)`` for a
    uniform random permutation sigma of 1..n.  Returns (prompts, user_of).
    """
    assert n % k == 0 and u >= 1 and d >= 1
    rng = _rng(seed, 0)
    n_user = n // k
    first_user = np.arange(n_user, dtype=np.int32)
    first_doc = np.arange(n_user, n_user + n, dtype=np.int32)
    seqs = []
    users = rng.integers(n_user + n, n_user + n + VOCAB, size=(n_user, u), dtype=np.int32)
    users[:, 0] = first_user
    docs = rng.integers(n_user + n, n_user + n + VOCAB, size=(n, d), dtype=np.int32)
    docs[:, 0] = first_doc
    user_of = np.arange(n) // k
    for j in range(n):
        seqs.append(np.concatenate([users[user_of[j]], docs[j]]))
    sigma = rng.permutation(n) + 1
    return _from_lists(seqs, (s * sigma).astype(np.uint64)), user_of


def toy_example(s: int) -> Prompts:
    """The four-query example of Sec. 4.2: n=4, replication 2, u=d=5, arrivals s*i.

    x1=(user1)(doc1), x2=(user2)(doc2), x3=(user1)(doc3), x4=(user2)(doc4).
    """
    user1 = [1, 11, 12, 13, 14]
    user2 = [2, 21, 22, 23, 24]
    doc = {i: [100 + i, 30 + i, 40 + i, 50 + i, 60 + i] for i in (1, 2, 3, 4)}
    seqs = [user1 + doc[1], user2 + doc[2], user1 + doc[3], user2 + doc[4]]
    return _from_lists(seqs, [s * (i + 1) for i in range(4)])


def random_small(seed: int, n_cache: int = 12, n_query: int = 20, vocab: int = 3,
                 max_len: int = 10, arrival_hi: int = 6) -> Workload:
    """Tiny random strings over a tiny alphabet: dense prefix sharing, many ties."""
    rng = _rng(seed, 7)

    def strings(m):
        out = []
        for _ in range(m):
            length = int(rng.integers(1, max_len + 1))
            out.append(rng.integers(0, vocab, size=length).tolist())
        return out

    cache = _from_lists(strings(n_cache))
    q = strings(n_query)
    arrival = rng.integers(0, arrival_hi, size=n_query)
    queries = _from_lists(q, arrival)
    return Workload("random-small", cache, queries, k=int(rng.integers(1, 5)), batch=int(rng.integers(1, n_query + 2)),
                    budget=1 << 40)
