"""Test-side helpers: canonical-snapshot parsing and brute-force models.

The brute-force models here are deliberately independent of both the C oracle
and the GPU library: plain Python over lists, tuples and dicts.
"""
from __future__ import annotations

import struct
from typing import Dict, List, Sequence, Tuple

import numpy as np

REC = np.dtype([("depth_start", "<i4"), ("edge_len", "<i4"), ("tick", "<u8"), ("n_children", "<i4"), ("pad", "<i4")])


def parse_snapshot(buf: bytes):
    """-> (n_nodes, total_tokens, clock, records[REC], tokens[int32])."""
    n_nodes, total, clock = struct.unpack_from("<qqQ", buf, 0)
    rec = np.frombuffer(buf, dtype=REC, count=n_nodes, offset=24)
    tok = np.frombuffer(buf, dtype="<i4", count=total, offset=24 + n_nodes * REC.itemsize)
    assert len(buf) == 24 + n_nodes * REC.itemsize + total * 4
    return n_nodes, total, clock, rec, tok


def snapshot_paths(buf: bytes) -> Dict[Tuple[int, ...], int]:
    """Node end-path (tuple of tokens from the root) -> tick, rebuilt from the DFS order."""
    n_nodes, total, clock, rec, tok = parse_snapshot(buf)
    out = {}
    stack: List[Tuple[int, ...]] = []  # path strings of the current ancestors
    pos = 0
    for r in rec:
        ds, el = int(r["depth_start"]), int(r["edge_len"])
        while stack and len(stack[-1]) > ds:
            stack.pop()
        base = stack[-1] if stack else ()
        assert len(base) == ds, "pre-order depth mismatch"
        path = base + tuple(int(t) for t in tok[pos : pos + el])
        pos += el
        out[path] = int(r["tick"])
        stack.append(path)
    assert pos == total
    return out


def lcp(a: Sequence[int], b: Sequence[int]) -> int:
    j = 0
    lim = min(len(a), len(b))
    while j < lim and a[j] == b[j]:
        j += 1
    return j


class PathModel:
    """Dictionary-of-paths model of the prefix cache.

    A node is identified by the full token string from the root to its end;
    its edge starts where its nearest proper-prefix node ends.  Everything is
    quadratic brute force.
    """

    def __init__(self):
        self.nodes: Dict[Tuple[int, ...], int] = {}
        self.clock = 0

    def _parent_len(self, key) -> int:
        best = 0
        for other in self.nodes:
            if len(other) < len(key) and key[: len(other)] == other:
                best = max(best, len(other))
        return best

    def total(self) -> int:
        return sum(len(k) - self._parent_len(k) for k in self.nodes)

    def match(self, x) -> int:
        return max((lcp(x, k) for k in self.nodes), default=0)

    def insert(self, x) -> None:
        x = tuple(int(t) for t in x)
        tick = self.clock
        self.clock += 1
        m = self.match(x)
        if m > 0 and x[:m] not in self.nodes:
            self.nodes[x[:m]] = tick
        if len(x) > m:
            self.nodes[x] = tick
        for k in self.nodes:
            if len(k) <= len(x) and x[: len(k)] == k:
                self.nodes[k] = tick

    def leaves(self):
        ks = list(self.nodes)
        return [k for k in ks if not any(len(o) > len(k) and o[: len(k)] == k for o in ks)]

    def evict(self, budget: int, protect: int = 0) -> int:
        n = 0
        while self.nodes and self.total() > budget:
            victim = min(self.leaves(), key=lambda k: self.nodes[k])
            if protect > 0 and self.nodes[victim] >= self.clock - protect:
                break  # the least recently used leaf belongs to a prompt still in flight
            del self.nodes[victim]
            n += 1
        return n

    def commit(self, prompts: Sequence[Sequence[int]], budget: int, protect: int = 0) -> None:
        for x in prompts:
            self.insert(x)
        self.evict(budget, protect)

    def snapshot(self) -> bytes:
        keys = sorted(self.nodes)
        rec = np.zeros(len(keys), dtype=REC)
        toks: List[int] = []
        for i, k in enumerate(keys):
            ds = self._parent_len(k)
            nch = sum(1 for o in keys if len(o) > len(k) and o[: len(k)] == k and self._parent_len(o) == len(k))
            rec[i] = (ds, len(k) - ds, self.nodes[k], nch, 0)
            toks.extend(k[ds:])
        head = struct.pack("<qqQ", len(keys), len(toks), self.clock)
        return head + rec.tobytes() + np.asarray(toks, dtype="<i4").tobytes()


def select_literal(arrival, match_len, k, batch, phase, tie_key=None):
    """Algorithm 1 as a loop over a Python list of waiting queries."""
    tie = [0] * len(arrival) if tie_key is None else [int(v) for v in tie_key]
    inf = k in (0, 0xFFFFFFFF)
    remaining = list(range(len(arrival)))
    out = []
    ph = 0 if inf else phase % k
    for j in range(min(batch, len(arrival))):
        if not inf and (ph + j) % k == 0:
            p = min(remaining, key=lambda i: (int(arrival[i]), i))
        else:
            p = min(remaining, key=lambda i: (-int(match_len[i]), tie[i], int(arrival[i]), i))
        out.append(p)
        remaining.remove(p)
    return out, (0 if inf else (ph + len(out)) % k)
