"""Buffer ownership around the C ABI: one object per tree that keeps the per-step device buffers.

Nothing here computes: each method forwards to one library call on the current stream.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B


def size_config(cache_tokens: int, cache_prompts: int, budget: int, max_batch: int, max_prompt_len: int,
                extra_prompts: int = 0) -> B.Config:
    """A configuration with room for the given cache plus commits of ``max_batch`` prompts."""
    live = min(int(cache_tokens), int(budget)) if budget < (1 << 60) else int(cache_tokens)
    pool = int(live * 1.05) + 2 * max_batch * max_prompt_len + 4096
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

    def match(self, q: B.DeviceQueries, want_nodes: bool = False) -> torch.Tensor:
        assert q.n <= self.n_max
        return B.kLPM_match(self.tree, q, self.match_len, self.last_node if want_nodes else None)

    def select(self, q: B.DeviceQueries, k: int, batch: int, n: Optional[int] = None) -> None:
        assert batch <= self.cfg.max_batch
        B.kLPM_select(q.arrival, self.match_len, q.n if n is None else n, k, batch, self.phase, self.batch_idx,
                      self.n_selected, self.ws, self.ws_bytes)

    def commit(self, q: B.DeviceQueries, batch_cap: Optional[int] = None) -> None:
        B.kLPM_commit(self.tree, q, self.batch_idx, self.n_selected,
                      self.cfg.max_batch if batch_cap is None else batch_cap, self.stats)

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


class OnlineRun:
    """Device-resident waiting queue for an online stream (arrivals per scheduling step)."""

    def __init__(self, sched: Scheduler, all_q: B.DeviceQueries, cap: int, first_ids: np.ndarray):
        dev = sched.device
        self.s = sched
        self.all_q = all_q
        self.cap = int(cap)
        self.wait_id = torch.zeros(self.cap, dtype=torch.int32, device=dev)
        self.wait_arr = torch.zeros(self.cap, dtype=torch.int64, device=dev)
        self.n_wait = torch.zeros(1, dtype=torch.int32, device=dev)
        self.off_w = torch.zeros(self.cap, dtype=torch.int64, device=dev)
        self.len_w = torch.zeros(self.cap, dtype=torch.int32, device=dev)
        self.sim_clock = torch.zeros(1, dtype=torch.int64, device=dev)
        self.ttft = torch.full((max(all_q.n, 1),), -1, dtype=torch.int64, device=dev)
        self.dev_error = torch.zeros(1, dtype=torch.int32, device=dev)
        self.scratch_bytes = 16 * max(self.cap, 1) + 768
        self.scratch = B.alloc_aligned(self.scratch_bytes, dev)
        n0 = int(first_ids.shape[0])
        assert n0 <= self.cap
        self.wait_id[:n0] = torch.from_numpy(first_ids.astype(np.int32)).to(dev)
        self.n_wait.fill_(n0)
        self.n_host = n0

    def step(self, k: int, batch: int, new_ids: Optional[torch.Tensor]) -> None:
        """One scheduling step: gather the queue view, match, select, commit, then retire the
        batch and enqueue ``new_ids``.  The queue length evolves deterministically (admitted =
        min(batch, waiting)), so the host tracks it without reading anything back."""
        s = self.s
        n = self.n_host
        B.kLPM_queue_gather(self.wait_id, self.n_wait, n, self.all_q.off, self.all_q.len, self.all_q.n,
                            self.off_w, self.len_w)
        q = B.DeviceQueries(self.all_q.tokens, self.off_w, self.len_w, self.wait_arr, n)
        s.match(q)
        s.select(q, k, batch)
        s.commit(q, batch)
        n_new = 0 if new_ids is None else int(new_ids.shape[0])
        B.kLPM_queue_advance(self.wait_id, self.wait_arr, self.n_wait, self.cap, s.match_len, self.all_q.len,
                             self.all_q.n, s.batch_idx, s.n_selected, batch, new_ids, n_new, self.sim_clock,
                             self.ttft, self.scratch, self.scratch_bytes, self.dev_error)
        self.n_host = min(self.cap, n - min(batch, n) + n_new)
