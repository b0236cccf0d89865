"""Writes tests/golden/workload_digests.txt: SHA-256 fingerprints of what the seeded input generators produce.

The generators draw from numpy's PCG64 through `numpy.random.Generator`; the fingerprints make a change of
those streams (another numpy version, an edit of a recipe) show up as a failing test instead of as silently
different inputs.  They are fingerprints of inputs only - no value of the scheduling method is stored here.
Run from the repository root: python tests/golden/make_workload_digests.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import workloads as W  # noqa: E402


def digest_prompts(p) -> str:
    h = hashlib.sha256()
    for a in (p.tokens, p.off, p.len, p.arrival):
        a = np.ascontiguousarray(a)
        h.update(str(a.dtype).encode() + b"|" + str(a.shape).encode() + b"|")
        h.update(a.tobytes())
    return h.hexdigest()


def cases():
    """(name, digest) pairs; sizes chosen so that the whole list takes a few seconds."""
    w = W.config0()
    yield "config0.cache", digest_prompts(w.cache)
    yield "config0.queries", digest_prompts(w.queries)
    w = W.config1(scale=0.05)
    yield "config1(scale=0.05).cache", digest_prompts(w.cache)
    yield "config1(scale=0.05).queries", digest_prompts(w.queries)
    w = W.config2(scale=1.0 / 64, extra_queries=64)
    yield "config2(scale=1/64).cache", digest_prompts(w.cache)
    yield "config2(scale=1/64).queries", digest_prompts(w.queries)
    yield "config2(scale=1/64).extra", digest_prompts(w.extra)
    w = W.config2_deep(scale=1.0 / 64)
    yield "config2_deep(scale=1/64).cache", digest_prompts(w.cache)
    yield "config2_deep(scale=1/64).queries", digest_prompts(w.queries)
    w = W.config3(scale=0.02)
    yield "config3(scale=0.02).cache", digest_prompts(w.cache)
    yield "config3(scale=0.02).queries", digest_prompts(w.queries)
    s = W.config4_stream(steps=40, rate=24, groups=2000, budget=150_000, batch=32)
    yield "config4_stream(steps=40,rate=24,groups=2000).queries", digest_prompts(s.queries)
    yield "config4_stream(steps=40,rate=24,groups=2000).step_start", hashlib.sha256(np.ascontiguousarray(s.step_start).tobytes()).hexdigest()
    p, user_of = W.shuffled_queue(200, 30, 4, 20, 7, seed=5)
    yield "shuffled_queue(200,30,4,20,7,seed=5).prompts", digest_prompts(p)
    yield "shuffled_queue(200,30,4,20,7,seed=5).user_of", hashlib.sha256(np.ascontiguousarray(user_of).tobytes()).hexdigest()
    w = W.random_small(901, n_cache=14, n_query=40, vocab=3, max_len=10)
    yield "random_small(901).cache", digest_prompts(w.cache)
    yield "random_small(901).queries", digest_prompts(w.queries)


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_digests.txt")
    with open(out, "w") as f:
        f.write("# SHA-256 of the arrays the seeded generators produce (written by make_workload_digests.py; inputs only)\n")
        f.write(f"# numpy {np.__version__} when written\n")
        for name, d in cases():
            f.write(f"{d}  {name}\n")
    print(open(out).read())
