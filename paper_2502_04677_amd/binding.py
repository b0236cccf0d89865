"""Thin Python binding of the C ABI in ``include/klpm.h`` (argument marshalling only).

Every step of the scheduling path runs inside the HIP library; PyTorch is used for device memory
and streams.  There is no CPU fallback: if the library cannot be loaded the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# KLPM_LIBRARY may point at another build of the same library (same ABI)
_LIB_PATH = os.environ.get("KLPM_LIBRARY") or os.path.join(_PKG, "libklpm.so")

KLPM_OK = 0
KLPM_K_INFINITY = 0xFFFFFFFF
KLPM_SELECT_FIFO = 1
DEV_NODES_FULL, DEV_POOL_FULL, DEV_BAD_INPUT, DEV_BATCH_OVERFLOW = 1, 2, 4, 8

EXPORTS = (
    "kLPM_arena_bytes", "kLPM_build_tree", "kLPM_match", "kLPM_select_workspace_bytes", "kLPM_select", "kLPM_select_static",
    "kLPM_score_hit_rate", "kLPM_tie_keys", "kLPM_select_dynamic_workspace_bytes", "kLPM_select_dynamic",
    "kLPM_commit", "kLPM_commit_matched", "kLPM_set_budget", "kLPM_set_protect", "kLPM_reserve_clock", "kLPM_batch_token_budget", "kLPM_kv_slots", "kLPM_gather_slots", "kLPM_queue_advance", "kLPM_queue_advance_timed", "kLPM_queue_gather",
    "kLPM_read_stats", "kLPM_probe_read",
    "kLPM_adapt_state_bytes", "kLPM_adapt_init", "kLPM_adapt_k", "kLPM_adapt_observe", "kLPM_adapt_read",
    "kLPM_snapshot_bytes", "kLPM_snapshot", "kLPM_destroy", "kLPM_strerror",
)


class Queries(C.Structure):
    _fields_ = [("tokens", C.c_void_p), ("off", C.c_void_p), ("len", C.c_void_p), ("arrival", C.c_void_p),
                ("n_tokens", C.c_int64), ("n", C.c_int32), ("n_live", C.c_void_p)]


class Arrivals(C.Structure):
    _fields_ = [("id", C.c_void_p), ("time", C.c_void_p), ("n", C.c_int32), ("c_num", C.c_uint32), ("c_den", C.c_uint32)]


class Queue(C.Structure):
    _fields_ = [("id", C.c_void_p), ("arrival", C.c_void_p), ("off", C.c_void_p), ("len", C.c_void_p),
                ("n", C.c_void_p), ("clock", C.c_void_p), ("n_joined", C.c_void_p), ("cap", C.c_int32)]


class Config(C.Structure):
    _fields_ = [("budget_tokens", C.c_int64), ("pool_tokens", C.c_int64), ("max_nodes", C.c_int32),
                ("max_batch", C.c_int32), ("max_prompt_len", C.c_int32), ("flags", C.c_uint32)]


class Stats(C.Structure):
    _fields_ = [("total_tokens", C.c_int64), ("inserted_tokens", C.c_int64), ("evicted_tokens", C.c_int64),
                ("n_nodes", C.c_int32), ("new_nodes", C.c_int32), ("evicted_nodes", C.c_int32),
                ("device_error", C.c_uint32), ("clock", C.c_uint64)]


STATS_BYTES = C.sizeof(Stats)
ADAPT_MAX_ARMS = 16


class AdaptConfig(C.Structure):
    _fields_ = [("arms", C.c_uint32 * ADAPT_MAX_ARMS), ("n_arms", C.c_int32), ("window", C.c_int32),
                ("explore", C.c_uint64), ("seed", C.c_uint64)]


class AdaptStats(C.Structure):
    _fields_ = [("count", C.c_uint64 * ADAPT_MAX_ARMS), ("cost", C.c_uint64 * ADAPT_MAX_ARMS), ("pulls", C.c_uint64),
                ("arm", C.c_int32), ("k", C.c_uint32), ("steps_in_window", C.c_int32), ("device_error", C.c_uint32)]


def load_library() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        from . import build as _build  # compiles with hipcc; raises if that is impossible
        _build.build()
    lib = C.CDLL(_LIB_PATH)
    missing = [name for name in EXPORTS if not hasattr(lib, name)]
    if missing:
        raise ImportError(f"{_LIB_PATH} is older than its sources (no {', '.join(missing)}): rebuild it with "
                          "`python paper_2502_04677_amd/build.py` or __graft_entry__.build()")
    vp, i32, i64, u32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_size_t
    lib.kLPM_arena_bytes.argtypes = [C.POINTER(Config), C.POINTER(sz)]
    lib.kLPM_build_tree.argtypes = [C.POINTER(vp), C.POINTER(Config), vp, sz, C.POINTER(Queries), vp]
    lib.kLPM_match.argtypes = [vp, C.POINTER(Queries), vp, vp, vp]
    lib.kLPM_select_workspace_bytes.argtypes = [i32, C.POINTER(sz)]
    lib.kLPM_select.argtypes = [vp, vp, vp, i32, vp, u32, vp, i32, u32, i32, vp, vp, vp, vp, sz, vp]
    lib.kLPM_select_static.argtypes = [vp, vp, vp, i32, vp, u32, vp, i32, u32, i32, vp, vp, vp, vp]
    lib.kLPM_adapt_state_bytes.argtypes = [C.POINTER(sz)]
    lib.kLPM_adapt_init.argtypes = [vp, sz, C.POINTER(AdaptConfig), vp]
    lib.kLPM_adapt_k.argtypes = [vp, C.POINTER(vp)]
    lib.kLPM_adapt_observe.argtypes = [vp, C.POINTER(Queue), vp, vp, i32, vp, i32, vp]
    lib.kLPM_adapt_read.argtypes = [vp, C.POINTER(AdaptStats), vp]
    lib.kLPM_select_dynamic_workspace_bytes.argtypes = [i32, C.POINTER(sz)]
    lib.kLPM_select_dynamic.argtypes = [C.POINTER(Queries), vp, vp, u32, vp, i32, u32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.kLPM_score_hit_rate.argtypes = [vp, vp, i32, vp, i32, vp, vp]
    lib.kLPM_tie_keys.argtypes = [C.c_uint64, C.c_uint64, vp, i32, vp, vp, vp]
    lib.kLPM_commit.argtypes = [vp, C.POINTER(Queries), vp, vp, i32, vp, vp]
    lib.kLPM_commit_matched.argtypes = [vp, C.POINTER(Queries), vp, vp, vp, vp, i32, vp, vp]
    lib.kLPM_set_budget.argtypes = [vp, i64]
    lib.kLPM_set_protect.argtypes = [vp, i64]
    lib.kLPM_reserve_clock.argtypes = [vp, C.c_uint64]
    lib.kLPM_batch_token_budget.argtypes = [C.POINTER(Queries), vp, vp, vp, i32, i64, u32, vp, vp, vp]
    lib.kLPM_kv_slots.argtypes = [vp, C.POINTER(Queries), vp, vp, i32, i32, vp, vp, vp]
    lib.kLPM_gather_slots.argtypes = [vp, vp, i64, vp, vp]
    lib.kLPM_queue_advance.argtypes = [C.POINTER(Queue), C.POINTER(Queue), C.POINTER(Queries), vp, vp, vp, i32, vp, i32,
                                       vp, vp, vp, vp]
    lib.kLPM_queue_advance_timed.argtypes = [C.POINTER(Queue), C.POINTER(Queue), C.POINTER(Queries), vp, vp, vp, i32,
                                             C.POINTER(Arrivals), vp, vp, vp, vp]
    lib.kLPM_queue_gather.argtypes = [C.POINTER(Queue), C.POINTER(Queries), vp]
    lib.kLPM_probe_read.argtypes = [vp, sz, vp, vp]
    lib.kLPM_read_stats.argtypes = [vp, C.POINTER(Stats), vp]
    lib.kLPM_snapshot_bytes.argtypes = [vp, C.POINTER(sz), vp]
    lib.kLPM_snapshot.argtypes = [vp, vp, sz, C.POINTER(sz), vp]
    lib.kLPM_destroy.argtypes = [vp]
    lib.kLPM_strerror.argtypes = [C.c_int]
    lib.kLPM_strerror.restype = C.c_char_p
    for name in EXPORTS:
        if name != "kLPM_strerror":
            getattr(lib, name).restype = C.c_int
    return lib


_lib = load_library()


class KlpmError(RuntimeError):
    pass


def _check(rc: int, what: str) -> None:
    if rc != KLPM_OK:
        raise KlpmError(f"{what}: {_lib.kLPM_strerror(rc).decode()} ({rc})")


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype, dtype)
    return t


@dataclass
class DeviceQueries:
    """Device-resident CSR prompts: tokens int32, off int64, len int32, arrival int64 (bits of uint64)."""

    tokens: torch.Tensor
    off: torch.Tensor
    len: torch.Tensor
    arrival: Optional[torch.Tensor]
    n: int
    n_live: Optional[torch.Tensor] = None  # int32 [1] on the device: how many of the n entries exist

    @staticmethod
    def from_host(p, device="cuda:0") -> "DeviceQueries":
        tok = torch.from_numpy(np.ascontiguousarray(p.tokens, dtype=np.int32)).to(device)
        if tok.numel() == 0:
            tok = torch.zeros(1, dtype=torch.int32, device=device)
        off = torch.from_numpy(np.ascontiguousarray(p.off, dtype=np.int64)).to(device)
        ln = torch.from_numpy(np.ascontiguousarray(p.len, dtype=np.int32)).to(device)
        arr = torch.from_numpy(np.ascontiguousarray(p.arrival, dtype=np.uint64).view(np.int64)).to(device)
        return DeviceQueries(tok, off, ln, arr, int(p.len.shape[0]))

    def c_struct(self) -> Queries:
        return Queries(_dev(self.tokens, torch.int32).data_ptr(), _dev(self.off, torch.int64).data_ptr() if self.n else 0,
                       _dev(self.len, torch.int32).data_ptr() if self.n else 0,
                       0 if self.arrival is None else self.arrival.data_ptr(), int(self.tokens.numel()), int(self.n),
                       0 if self.n_live is None else _dev(self.n_live, torch.int32).data_ptr())


class Tree:
    """Owner of the arena tensor and the library handle."""

    def __init__(self, handle: int, arena: torch.Tensor, cfg: Config):
        self.handle = C.c_void_p(handle)
        self.arena = arena
        self.cfg = cfg

    def close(self) -> None:
        if self.handle:
            _lib.kLPM_destroy(self.handle)
            self.handle = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def make_config(budget_tokens: int, pool_tokens: int, max_nodes: int, max_batch: int, max_prompt_len: int) -> Config:
    return Config(int(min(budget_tokens, (1 << 62))), int(pool_tokens), int(max_nodes), int(max_batch),
                  int(max_prompt_len), 0)


def kLPM_arena_bytes(cfg: Config) -> int:
    out = C.c_size_t(0)
    _check(_lib.kLPM_arena_bytes(C.byref(cfg), C.byref(out)), "kLPM_arena_bytes")
    return int(out.value)


def kLPM_build_tree(cfg: Config, initial: Optional[DeviceQueries], device="cuda:0", stream=None) -> Tree:
    nbytes = kLPM_arena_bytes(cfg)
    arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    base = (arena.data_ptr() + 255) // 256 * 256
    handle = C.c_void_p(0)
    q = initial.c_struct() if initial is not None else None
    rc = _lib.kLPM_build_tree(C.byref(handle), C.byref(cfg), C.c_void_p(base), nbytes,
                              C.byref(q) if q is not None else None, _stream(stream))
    _check(rc, "kLPM_build_tree")
    return Tree(handle.value, arena, cfg)


def kLPM_match(tree: Tree, q: DeviceQueries, match_len: Optional[torch.Tensor] = None,
               last_node: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    if match_len is None:
        match_len = torch.empty(max(q.n, 1), dtype=torch.int32, device=q.tokens.device)
    qs = q.c_struct()
    _check(_lib.kLPM_match(tree.handle, C.byref(qs), _ptr(match_len), _ptr(last_node), _stream(stream)), "kLPM_match")
    return match_len[: q.n]


def kLPM_select_workspace_bytes(n: int) -> int:
    out = C.c_size_t(0)
    _check(_lib.kLPM_select_workspace_bytes(int(n), C.byref(out)), "kLPM_select_workspace_bytes")
    return int(out.value)


def alloc_aligned(nbytes: int, device) -> Tuple[torch.Tensor, int]:
    buf = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=device)
    return buf, (buf.data_ptr() + 255) // 256 * 256


def kLPM_select(arrival: torch.Tensor, match_len: torch.Tensor, n: int, k: int, batch: int,
                phase_inout: torch.Tensor, batch_idx: torch.Tensor, n_selected: torch.Tensor,
                workspace: Tuple[torch.Tensor, int], workspace_bytes: int, stream=None, flags: int = 0,
                max_match: int = 0, n_live: Optional[torch.Tensor] = None,
                tie_key: Optional[torch.Tensor] = None, k_dev: Optional[int] = None) -> None:
    """``k_dev``: device address of a uint32 holding k (``AdaptiveK.k_dev``); ``k`` is then ignored."""
    _check(_lib.kLPM_select(_ptr(arrival), _ptr(match_len), _ptr(tie_key), int(n), _ptr(n_live), C.c_uint32(k & 0xFFFFFFFF),
                            C.c_void_p(k_dev), int(batch),
                            C.c_uint32(flags), int(max_match), _ptr(phase_inout), _ptr(batch_idx), _ptr(n_selected), C.c_void_p(workspace[1]),
                            int(workspace_bytes), _stream(stream)), "kLPM_select")


KLPM_SELECT_STATIC_MAX_N = 131072
KLPM_ELIMIT = -5


def kLPM_select_static(arrival: torch.Tensor, match_len: torch.Tensor, n: int, k: int, batch: int,
                       phase_inout: torch.Tensor, batch_idx: torch.Tensor, n_selected: torch.Tensor, stream=None,
                       flags: int = 0, max_match: int = 0, n_live: Optional[torch.Tensor] = None,
                       tie_key: Optional[torch.Tensor] = None, k_dev: Optional[int] = None) -> None:
    """``kLPM_select`` with the library's own fixed scratch array as workspace (allocates nothing)."""
    _check(_lib.kLPM_select_static(_ptr(arrival), _ptr(match_len), _ptr(tie_key), int(n), _ptr(n_live),
                                   C.c_uint32(k & 0xFFFFFFFF), C.c_void_p(k_dev), int(batch), C.c_uint32(flags),
                                   int(max_match), _ptr(phase_inout), _ptr(batch_idx), _ptr(n_selected),
                                   _stream(stream)), "kLPM_select_static")


def kLPM_select_dynamic_workspace_bytes(n: int) -> int:
    out = C.c_size_t(0)
    _check(_lib.kLPM_select_dynamic_workspace_bytes(int(n), C.byref(out)), "kLPM_select_dynamic_workspace_bytes")
    return int(out.value)


def kLPM_select_dynamic(q: DeviceQueries, match_len: torch.Tensor, last_node: torch.Tensor, k: int, batch: int,
                        phase_inout: torch.Tensor, dyn_match: torch.Tensor, batch_idx: torch.Tensor,
                        n_selected: torch.Tensor, workspace: Tuple[torch.Tensor, int], workspace_bytes: int,
                        stream=None, k_dev: Optional[int] = None, flags: int = 0, max_match: int = 0) -> None:
    qs = q.c_struct()
    _check(_lib.kLPM_select_dynamic(C.byref(qs), _ptr(match_len), _ptr(last_node), C.c_uint32(k & 0xFFFFFFFF),
                                    C.c_void_p(k_dev), int(batch), C.c_uint32(flags), int(max_match),
                                    _ptr(phase_inout), _ptr(dyn_match), _ptr(batch_idx), _ptr(n_selected),
                                    C.c_void_p(workspace[1]), int(workspace_bytes), _stream(stream)),
           "kLPM_select_dynamic")


def kLPM_score_hit_rate(match_len: torch.Tensor, length: torch.Tensor, n: int, scale_bits: int, score: torch.Tensor,
                        n_live: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(_lib.kLPM_score_hit_rate(_ptr(match_len), _ptr(length), int(n), _ptr(n_live), int(scale_bits), _ptr(score),
                                    _stream(stream)), "kLPM_score_hit_rate")


def kLPM_tie_keys(seed: int, step: int, ids: Optional[torch.Tensor], n: int, tie_key: torch.Tensor,
                  n_live: Optional[torch.Tensor] = None, stream=None) -> None:
    _check(_lib.kLPM_tie_keys(C.c_uint64(seed & (2**64 - 1)), C.c_uint64(step & (2**64 - 1)), _ptr(ids), int(n),
                              _ptr(n_live), _ptr(tie_key), _stream(stream)), "kLPM_tie_keys")


def kLPM_commit(tree: Tree, q: DeviceQueries, batch_idx: Optional[torch.Tensor], n_selected: Optional[torch.Tensor],
                batch_cap: int, stats: Optional[torch.Tensor] = None, stream=None) -> None:
    qs = q.c_struct()
    _check(_lib.kLPM_commit(tree.handle, C.byref(qs), _ptr(batch_idx), _ptr(n_selected), int(batch_cap), _ptr(stats),
                            _stream(stream)), "kLPM_commit")


def kLPM_commit_matched(tree: Tree, q: DeviceQueries, match_len: torch.Tensor, last_node: torch.Tensor,
                        batch_idx: Optional[torch.Tensor], n_selected: Optional[torch.Tensor], batch_cap: int,
                        stats: Optional[torch.Tensor] = None, stream=None) -> None:
    assert match_len.shape[0] >= q.n and last_node.shape[0] >= q.n
    qs = q.c_struct()
    _check(_lib.kLPM_commit_matched(tree.handle, C.byref(qs), _ptr(match_len), _ptr(last_node), _ptr(batch_idx),
                                    _ptr(n_selected), int(batch_cap), _ptr(stats), _stream(stream)),
           "kLPM_commit_matched")


def kLPM_adapt_state_bytes() -> int:
    need = C.c_size_t(0)
    _check(_lib.kLPM_adapt_state_bytes(C.byref(need)), "kLPM_adapt_state_bytes")
    return int(need.value)


def kLPM_adapt_init(state: int, state_bytes: int, arms, window: int, explore: int, seed: int, stream=None) -> None:
    """``state``: device address (8-byte aligned) of at least ``kLPM_adapt_state_bytes()`` bytes."""
    cfg = AdaptConfig()
    if not 1 <= len(arms) <= ADAPT_MAX_ARMS:
        raise KlpmError("kLPM_adapt_init: between 1 and 16 arms")
    for i, a in enumerate(arms):
        cfg.arms[i] = int(a) & 0xFFFFFFFF
    cfg.n_arms, cfg.window, cfg.explore, cfg.seed = len(arms), int(window), int(explore), int(seed) & (2**64 - 1)
    _check(_lib.kLPM_adapt_init(C.c_void_p(state), int(state_bytes), C.byref(cfg), _stream(stream)), "kLPM_adapt_init")


def kLPM_adapt_k(state: int) -> int:
    """Device address of the current k (the ``k_dev`` argument of the selection calls)."""
    kp = C.c_void_p(0)
    _check(_lib.kLPM_adapt_k(C.c_void_p(state), C.byref(kp)), "kLPM_adapt_k")
    return int(kp.value)


def kLPM_adapt_observe(state: int, served: "DeviceQueue", batch_idx: torch.Tensor, n_selected: torch.Tensor,
                       batch_cap: int, ttft: torch.Tensor, stream=None) -> None:
    qs = served.c_struct()
    _check(_lib.kLPM_adapt_observe(C.c_void_p(state), C.byref(qs), _ptr(batch_idx), _ptr(n_selected), int(batch_cap),
                                   _ptr(ttft), int(ttft.shape[0]), _stream(stream)), "kLPM_adapt_observe")


def kLPM_adapt_read(state: int, stream=None) -> AdaptStats:
    out = AdaptStats()
    _check(_lib.kLPM_adapt_read(C.c_void_p(state), C.byref(out), _stream(stream)), "kLPM_adapt_read")
    return out


def kLPM_reserve_clock(tree: Tree, extra_prompts: int) -> None:
    _check(_lib.kLPM_reserve_clock(tree.handle, C.c_uint64(int(extra_prompts))), "kLPM_reserve_clock")


def kLPM_set_protect(tree: Tree, recent_prompts: int) -> None:
    _check(_lib.kLPM_set_protect(tree.handle, int(recent_prompts)), "kLPM_set_protect")


def kLPM_batch_token_budget(q: DeviceQueries, match_len: torch.Tensor, batch_idx: torch.Tensor, n_selected: torch.Tensor,
                            batch_cap: int, token_budget: int, k: int, phase_inout: torch.Tensor, stream=None,
                            k_dev: Optional[int] = None) -> None:
    qs = q.c_struct()
    _check(_lib.kLPM_batch_token_budget(C.byref(qs), _ptr(match_len), _ptr(batch_idx), _ptr(n_selected), int(batch_cap),
                                        int(token_budget), C.c_uint32(k & 0xFFFFFFFF), C.c_void_p(k_dev),
                                        _ptr(phase_inout), _stream(stream)),
           "kLPM_batch_token_budget")


def kLPM_kv_slots(tree: Tree, q: DeviceQueries, batch_idx: torch.Tensor, n_selected: torch.Tensor, batch_cap: int,
                  stride: int, n_matched: torch.Tensor, slots: torch.Tensor, stream=None) -> None:
    qs = q.c_struct()
    assert slots.dtype == torch.int64 and slots.numel() >= batch_cap * stride and n_matched.numel() >= batch_cap
    _check(_lib.kLPM_kv_slots(tree.handle, C.byref(qs), _ptr(batch_idx), _ptr(n_selected), int(batch_cap), int(stride),
                              _ptr(n_matched), _ptr(slots), _stream(stream)), "kLPM_kv_slots")


def kLPM_gather_slots(tree: Tree, slots: torch.Tensor, tokens_out: torch.Tensor, stream=None) -> None:
    assert slots.dtype == torch.int64 and tokens_out.dtype == torch.int32 and tokens_out.numel() >= slots.numel()
    _check(_lib.kLPM_gather_slots(tree.handle, _ptr(slots), int(slots.numel()), _ptr(tokens_out), _stream(stream)),
           "kLPM_gather_slots")


def kLPM_set_budget(tree: Tree, budget_tokens: int) -> None:
    _check(_lib.kLPM_set_budget(tree.handle, int(min(budget_tokens, 1 << 62))), "kLPM_set_budget")


@dataclass
class DeviceQueue:
    """Device buffers of one waiting queue (ids, enqueue times, CSR view, count)."""

    id: torch.Tensor  # int32 [cap]
    arrival: torch.Tensor  # int64 [cap] (bits of uint64)
    off: torch.Tensor  # int64 [cap]
    len: torch.Tensor  # int32 [cap]
    n: torch.Tensor  # int32 [1]
    clock: torch.Tensor  # int64 [1] (bits of uint64): simulated time of this queue state
    n_joined: torch.Tensor  # int32 [1]: timed runs, arrivals that have joined so far
    cap: int

    @staticmethod
    def empty(cap: int, device, clock: int = 0) -> "DeviceQueue":
        c = max(int(cap), 1)
        return DeviceQueue(torch.zeros(c, dtype=torch.int32, device=device), torch.zeros(c, dtype=torch.int64, device=device),
                           torch.zeros(c, dtype=torch.int64, device=device), torch.zeros(c, dtype=torch.int32, device=device),
                           torch.zeros(1, dtype=torch.int32, device=device),
                           torch.full((1,), int(clock), dtype=torch.int64, device=device),
                           torch.zeros(1, dtype=torch.int32, device=device), int(cap))

    def c_struct(self) -> Queue:
        return Queue(self.id.data_ptr(), self.arrival.data_ptr(), self.off.data_ptr(), self.len.data_ptr(),
                     self.n.data_ptr(), self.clock.data_ptr(), self.n_joined.data_ptr(), self.cap)


def kLPM_queue_advance(cur: DeviceQueue, nxt: DeviceQueue, all_q: DeviceQueries, match_len, batch_idx, n_selected,
                       batch_cap: int, new_id, n_new: int, ttft, matched_accum, dev_error, stream=None) -> None:
    c, n, a = cur.c_struct(), nxt.c_struct(), all_q.c_struct()
    _check(_lib.kLPM_queue_advance(C.byref(c), C.byref(n), C.byref(a), _ptr(match_len), _ptr(batch_idx),
                                   _ptr(n_selected), int(batch_cap), _ptr(new_id), int(n_new), _ptr(ttft),
                                   _ptr(matched_accum), _ptr(dev_error), _stream(stream)), "kLPM_queue_advance")


@dataclass
class DeviceArrivals:
    """Arrivals in time order, resident on the device."""

    id: torch.Tensor  # int32 [n], ordered by (time, id)
    time: torch.Tensor  # int64 [n] (bits of uint64), non-decreasing
    n: int
    c_num: int = 0
    c_den: int = 1

    @staticmethod
    def from_host(arrival: np.ndarray, c_num: int, c_den: int, device) -> "DeviceArrivals":
        arrival = np.ascontiguousarray(arrival, dtype=np.uint64)
        order = np.lexsort((np.arange(arrival.shape[0]), arrival)).astype(np.int32)
        t = arrival[order].view(np.int64)
        n = int(order.shape[0])
        pad = max(n, 1)
        ids = torch.zeros(pad, dtype=torch.int32, device=device)
        tim = torch.zeros(pad, dtype=torch.int64, device=device)
        ids[:n] = torch.from_numpy(order).to(device)
        tim[:n] = torch.from_numpy(np.ascontiguousarray(t)).to(device)
        return DeviceArrivals(ids, tim, n, int(c_num), int(c_den))

    def c_struct(self) -> Arrivals:
        return Arrivals(self.id.data_ptr(), self.time.data_ptr(), self.n, self.c_num, self.c_den)


def kLPM_queue_advance_timed(cur: DeviceQueue, nxt: DeviceQueue, all_q: DeviceQueries, match_len, batch_idx, n_selected,
                             batch_cap: int, pending: DeviceArrivals, ttft, matched_accum, dev_error, stream=None) -> None:
    c, n, a, p = cur.c_struct(), nxt.c_struct(), all_q.c_struct(), pending.c_struct()
    _check(_lib.kLPM_queue_advance_timed(C.byref(c), C.byref(n), C.byref(a), _ptr(match_len), _ptr(batch_idx),
                                         _ptr(n_selected), int(batch_cap), C.byref(p), _ptr(ttft), _ptr(matched_accum),
                                         _ptr(dev_error), _stream(stream)), "kLPM_queue_advance_timed")


def kLPM_queue_gather(q: DeviceQueue, all_q: DeviceQueries, stream=None) -> None:
    c, a = q.c_struct(), all_q.c_struct()
    _check(_lib.kLPM_queue_gather(C.byref(c), C.byref(a), _stream(stream)), "kLPM_queue_gather")


def kLPM_probe_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    assert sink.dtype == torch.int64 and src.is_contiguous()
    _check(_lib.kLPM_probe_read(_ptr(src), int(src.numel() * src.element_size()), _ptr(sink), _stream(stream)),
           "kLPM_probe_read")


def kLPM_read_stats(tree: Tree, stream=None) -> Stats:
    st = Stats()
    _check(_lib.kLPM_read_stats(tree.handle, C.byref(st), _stream(stream)), "kLPM_read_stats")
    return st


def stats_from_tensor(t: torch.Tensor) -> Stats:
    """Decode a device kLPM_stats record (uint8 tensor of STATS_BYTES) after synchronising."""
    raw = t.cpu().numpy().tobytes()
    return Stats.from_buffer_copy(raw[:STATS_BYTES])


def kLPM_snapshot(tree: Tree, stream=None) -> bytes:
    need = C.c_size_t(0)
    _check(_lib.kLPM_snapshot_bytes(tree.handle, C.byref(need), _stream(stream)), "kLPM_snapshot_bytes")
    buf = np.zeros(int(need.value), dtype=np.uint8)
    got = C.c_size_t(0)
    _check(_lib.kLPM_snapshot(tree.handle, buf.ctypes.data_as(C.c_void_p), buf.shape[0], C.byref(got), _stream(stream)),
           "kLPM_snapshot")
    assert got.value == need.value
    return buf.tobytes()


def kLPM_destroy(tree: Tree) -> None:
    tree.close()
