"""Buffer ownership around the C ABI: one object per tree that keeps the per-step device buffers.

Nothing here computes: each method forwards to one library call on the current stream.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


def size_config(cache_tokens: int, cache_prompts: int, budget: int, max_batch: int, max_prompt_len: int,
                extra_prompts: int = 0, extra_tokens: int = 0, slack_batches: int = 32) -> B.Config:
    """A configuration with room for the initial cache plus commits of ``max_batch`` prompts.

    The tree is built without eviction, so one pool half must hold the whole initial cache; under a
    finite budget it later holds at most the budget plus one batch, otherwise the initial cache plus
    ``extra_tokens`` of later insertions.
    """
    finite = budget < (1 << 36)  # anything larger cannot be reached and means "never evict"
    live = max(int(cache_tokens), int(budget)) if finite else int(cache_tokens) + int(extra_tokens)
    # (room for ``slack_batches`` worst-case batches between two pool compactions, which move every cached
    # token once: the pool is cheap next to the HBM size, a compaction costs a step a few hundred microseconds)
    pool = int(live * 1.05) + slack_batches * max_batch * max_prompt_len + 4096
    nodes = 2 * (cache_prompts + extra_prompts) + 4 * max_batch + 64
    return B.make_config(budget, pool, nodes, max_batch, max_prompt_len)


class Scheduler:
    def __init__(self, cfg: B.Config, initial: Optional[B.DeviceQueries], n_max: int, device="cuda:0"):
        self.device = torch.device(device)
        self.cfg = cfg
        self.tree = B.kLPM_build_tree(cfg, initial, device=device)
        self.n_max = int(n_max)
        self.match_len = torch.zeros(max(self.n_max, 1), dtype=torch.int32, device=device)
        self.last_node = torch.zeros(max(self.n_max, 1), dtype=torch.int32, device=device)
        self.batch_idx = torch.zeros(max(cfg.max_batch, 1), dtype=torch.int32, device=device)
        self.n_selected = torch.zeros(1, dtype=torch.int32, device=device)
        self.phase = torch.zeros(1, dtype=torch.int32, device=device)  # bits of a uint32
        self.stats = torch.zeros(B.STATS_BYTES, dtype=torch.uint8, device=device)
        self.ws_bytes = B.kLPM_select_workspace_bytes(self.n_max)
        self.ws = B.alloc_aligned(self.ws_bytes, device)
        self._matched_q = None  # the query set whose match (lengths and nodes) is still valid for the tree

    def match(self, q: B.DeviceQueries, want_nodes: bool = True) -> torch.Tensor:
        assert q.n <= self.n_max
        out = B.kLPM_match(self.tree, q, self.match_len, self.last_node if want_nodes else None)
        self._matched_q = q if want_nodes else None
        return out

    def select(self, q: B.DeviceQueries, k: int, batch: int, n: Optional[int] = None, fifo: bool = False,
               score: Optional[torch.Tensor] = None, score_max: int = 0, tie_key: Optional[torch.Tensor] = None,
               k_dev: Optional[int] = None) -> None:
        """``fifo`` promises that the queue is in arrival order (checked on the device).  ``score``
        (default: the match lengths of the last ``match``) is what longest-match picks maximise,
        ``score_max`` its upper bound; ``tie_key`` decides between equal scores; ``k_dev`` is the device
        address of a k that replaces ``k`` (``AdaptiveK.k_dev``)."""
        assert batch <= self.cfg.max_batch
        B.kLPM_select(q.arrival, self.match_len if score is None else score, q.n if n is None else n, k, batch,
                      self.phase, self.batch_idx, self.n_selected, self.ws, self.ws_bytes,
                      flags=B.KLPM_SELECT_FIFO if fifo else 0,
                      max_match=self.cfg.max_prompt_len if score is None else score_max, n_live=q.n_live,
                      tie_key=tie_key, k_dev=k_dev)

    def commit(self, q: B.DeviceQueries, batch_cap: Optional[int] = None, reuse_match: bool = True) -> None:
        """Commits the selected batch.  When ``q`` is the very object last passed to ``match`` and no
        commit has happened since, the admitted prompts' matches are taken from that call."""
        cap = self.cfg.max_batch if batch_cap is None else batch_cap
        if reuse_match and self._matched_q is q:
            B.kLPM_commit_matched(self.tree, q, self.match_len, self.last_node, self.batch_idx, self.n_selected, cap,
                                  self.stats)
        else:
            B.kLPM_commit(self.tree, q, self.batch_idx, self.n_selected, cap, self.stats)
        self._matched_q = None

    def step(self, q: B.DeviceQueries, k: int, batch: int) -> None:
        self.match(q)
        self.select(q, k, batch)
        self.commit(q, batch)

    # ---- host read-back helpers (synchronise) ----
    def batch(self) -> np.ndarray:
        n = int(self.n_selected.cpu().item())
        return self.batch_idx[:n].cpu().numpy()

    def phase_value(self) -> int:
        return int(self.phase.cpu().numpy().view(np.uint32)[0])

    def set_phase(self, v: int) -> None:
        self.phase.copy_(torch.from_numpy(np.array([v], dtype=np.uint32).view(np.int32)))

    def read_stats(self) -> B.Stats:
        torch.cuda.synchronize(self.device)
        return B.stats_from_tensor(self.stats)

    def snapshot(self) -> bytes:
        return B.kLPM_snapshot(self.tree)


class AdaptiveK:
    """Device-resident epsilon-greedy choice of k: the state buffer and the address of its current k."""

    def __init__(self, arms, window: int, explore: int, seed: int, device="cuda:0"):
        nbytes = B.kLPM_adapt_state_bytes()
        self.buf, self.state = B.alloc_aligned(nbytes, device)
        B.kLPM_adapt_init(self.state, nbytes, arms, window, explore, seed)
        self.k_dev = B.kLPM_adapt_k(self.state)
        self.n_arms = len(arms)

    def observe(self, served: B.DeviceQueue, batch_idx: torch.Tensor, n_selected: torch.Tensor, batch_cap: int,
                ttft: torch.Tensor) -> None:
        B.kLPM_adapt_observe(self.state, served, batch_idx, n_selected, batch_cap, ttft)

    def read(self) -> B.AdaptStats:
        return B.kLPM_adapt_read(self.state)


class OnlineRun:
    """Device-resident waiting queue for an online stream (arrivals per scheduling step).

    Two buffer sets are used in turn: each step reads the current queue and writes the next one.
    The queue length evolves deterministically (admitted = min(batch, waiting)), so the host tracks
    it without reading anything back.
    """

    def __init__(self, sched: Scheduler, all_q: B.DeviceQueries, cap: int, first_ids: np.ndarray,
                 first_arrival: Optional[np.ndarray] = None):
        dev = sched.device
        self.s = sched
        self.all_q = all_q
        self.cap = int(cap)
        self.queues = [B.DeviceQueue.empty(cap, dev), B.DeviceQueue.empty(cap, dev)]
        self.cur = 0
        self.ttft = torch.full((max(all_q.n, 1),), -1, dtype=torch.int64, device=dev)
        self.matched = torch.zeros(1, dtype=torch.int64, device=dev)
        self.dev_error = torch.zeros(1, dtype=torch.int32, device=dev)
        n0 = int(first_ids.shape[0])
        assert n0 <= self.cap
        q0 = self.queues[0]
        q0.id[:n0] = torch.from_numpy(first_ids.astype(np.int32)).to(dev)
        if first_arrival is not None:
            q0.arrival[:n0] = torch.from_numpy(np.ascontiguousarray(first_arrival, dtype=np.uint64).view(np.int64)).to(dev)
        q0.n.fill_(n0)
        self.n_host = n0
        B.kLPM_queue_gather(q0, all_q)

    @property
    def queue(self) -> B.DeviceQueue:
        return self.queues[self.cur]

    @property
    def sim_clock(self) -> torch.Tensor:
        """Simulated time of the current queue state (one-element int64 device tensor)."""
        return self.queue.clock

    def view(self) -> B.DeviceQueries:
        """The current queue as a query set sharing the stream's token pool."""
        q = self.queue
        return B.DeviceQueries(self.all_q.tokens, q.off, q.len, q.arrival, self.n_host)

    def advance(self, batch: int, new_ids: Optional[torch.Tensor], matched: Optional[torch.Tensor] = None) -> None:
        """Retire the batch and enqueue ``new_ids``; the queue's summed match length is added to
        ``matched`` (a one-element int64 device tensor; default: this run's own accumulator)."""
        s = self.s
        n_new = 0 if new_ids is None else int(new_ids.shape[0])
        B.kLPM_queue_advance(self.queues[self.cur], self.queues[1 - self.cur], self.all_q, s.match_len, s.batch_idx,
                             s.n_selected, batch, new_ids, n_new, self.ttft,
                             self.matched if matched is None else matched, self.dev_error)
        self.cur = 1 - self.cur
        self.n_host = min(self.cap, self.n_host - min(batch, self.n_host) + n_new)

    def step(self, k: int, batch: int, new_ids: Optional[torch.Tensor], adaptive: Optional[AdaptiveK] = None) -> None:
        """One scheduling step: match, select, commit, then retire the batch and enqueue ``new_ids``.
        With ``adaptive`` the step runs with the k that object holds on the device and reports the
        TTFT of the queries it admitted to it."""
        s = self.s
        q = self.view()
        served = self.queue
        s.match(q)
        # this queue is append-only with stable removal
        s.select(q, k, batch, fifo=True, k_dev=None if adaptive is None else adaptive.k_dev)
        # (the host knows the queue length here, so the commit is sized for what can be admitted: its
        # bound on the LRU clock, which sets the number of eviction passes, then grows no faster than
        # the clock itself)
        s.commit(q, min(batch, self.n_host))
        self.advance(batch, new_ids)
        if adaptive is not None:
            adaptive.observe(served, s.batch_idx, s.n_selected, batch, self.ttft)


class TimedRun:
    """Def. 2's timeline on the device: queries join the waiting queue when their arrival time has
    come, a batch costs (1 + c_attn |x|)(|x| - match) token times per query, an idle scheduler waits
    for the next arrival.  The queue length lives on the device (``n_live``), so a step never reads
    anything back; a step on an empty queue with nothing pending is a no-op.

    Times (arrivals, clock, TTFT) count units of 1/c_den of one token's linear prefill time.
    """

    def __init__(self, sched: Scheduler, all_q: B.DeviceQueries, cap: int, arrival: np.ndarray, c_num: int = 0,
                 c_den: int = 1, t_start: int = 0, tie_seed: Optional[int] = None):
        """With ``tie_seed`` equal match lengths are ordered by uniformly random keys redrawn every
        step (per query id and step number) instead of by arrival."""
        dev = sched.device
        self.s = sched
        self.all_q = all_q
        self.cap = int(cap)
        self.queues = [B.DeviceQueue.empty(cap, dev, clock=t_start), B.DeviceQueue.empty(cap, dev, clock=t_start)]
        self.cur = 0
        self.pending = B.DeviceArrivals.from_host(arrival, c_num, c_den, dev)
        self.ttft = torch.full((max(all_q.n, 1),), -1, dtype=torch.int64, device=dev)
        self.matched = torch.zeros(1, dtype=torch.int64, device=dev)
        self.dev_error = torch.zeros(1, dtype=torch.int32, device=dev)
        self.tie_seed = tie_seed
        self.tie = torch.zeros(max(self.cap, 1), dtype=torch.int32, device=dev) if tie_seed is not None else None
        self.steps_done = 0
        sched.n_selected.zero_()
        self._advance(0)  # initial fill: everything that has arrived by t_start, or the first arrival

    @property
    def queue(self) -> B.DeviceQueue:
        return self.queues[self.cur]

    @property
    def sim_clock(self) -> torch.Tensor:
        return self.queue.clock

    def view(self) -> B.DeviceQueries:
        q = self.queue
        return B.DeviceQueries(self.all_q.tokens, q.off, q.len, q.arrival, self.cap, n_live=q.n)

    def _advance(self, batch: int) -> None:
        s = self.s
        B.kLPM_queue_advance_timed(self.queues[self.cur], self.queues[1 - self.cur], self.all_q, s.match_len,
                                   s.batch_idx, s.n_selected, batch, self.pending, self.ttft, self.matched,
                                   self.dev_error)
        self.cur = 1 - self.cur

    def step(self, k: int, batch: int, adaptive: Optional[AdaptiveK] = None) -> None:
        """With ``adaptive`` the step runs with the k that object holds on the device (``k`` is ignored)
        and reports the TTFT of the queries it admitted to it."""
        s = self.s
        q = self.view()
        served = self.queue
        k_dev = None if adaptive is None else adaptive.k_dev
        s.match(q)
        if self.tie is None:
            s.select(q, k, batch, fifo=True, k_dev=k_dev)  # arrivals join in time order, removal is stable
        else:
            B.kLPM_tie_keys(self.tie_seed, self.steps_done, self.queue.id, self.cap, self.tie, n_live=self.queue.n)
            s.select(q, k, batch, tie_key=self.tie, k_dev=k_dev)
        s.commit(q, batch)
        self._advance(batch)
        if adaptive is not None:
            adaptive.observe(served, s.batch_idx, s.n_selected, batch, self.ttft)
        self.steps_done += 1
