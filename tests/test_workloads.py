"""The seeded input generators: their outputs are pinned by fingerprint, and their stated shapes hold.

The generators draw from numpy's PCG64 through numpy.random.Generator, whose distribution methods are not
promised to stay bit-identical across numpy versions.  Parity never depends on that (both sides always get
the arrays of one and the same call), but measured figures are quoted for particular inputs: a changed
stream must fail here, visibly, rather than move those figures silently.
"""
import importlib.util
import os

import numpy as np

import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def _digest_module():
    spec = importlib.util.spec_from_file_location("make_workload_digests", os.path.join(HERE, "golden", "make_workload_digests.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_generators_reproduce_their_recorded_fingerprints():
    want = {}
    for line in open(os.path.join(HERE, "golden", "workload_digests.txt")):
        if line.startswith("#") or not line.strip():
            continue
        d, name = line.rstrip("\n").split("  ", 1)
        want[name] = d
    got = dict(_digest_module().cases())
    assert set(got) == set(want)
    changed = [n for n in want if got[n] != want[n]]
    assert not changed, f"generator output changed (numpy {np.__version__}): {changed}"


def test_generators_are_deterministic_and_seeded():
    a, b = W.config0(), W.config0()
    assert np.array_equal(a.queries.tokens, b.queries.tokens) and np.array_equal(a.cache.tokens, b.cache.tokens)
    c = W.config0(seed=W.SEED_BASE + 77)
    assert not np.array_equal(a.queries.tokens[:1000], c.queries.tokens[:1000])


def test_config0_has_the_stated_shape():
    w = W.config0()
    assert (w.cache.n, w.queries.n, w.k, w.batch) == (64, 256, 2, 32)
    assert w.queries.arrival.tolist() == list(range(256))
    assert 0 <= int(w.queries.tokens.min()) and int(w.queries.tokens.max()) < W.VOCAB
    # cached prompts: a 128-token group prefix and a suffix of 64 to 256 tokens, four prompts per group
    assert ((w.cache.len >= 128 + 64) & (w.cache.len <= 128 + 256)).all()
    heads = {tuple(w.cache.prompt(i)[:128].tolist()) for i in range(w.cache.n)}
    assert len(heads) == 16
    # queries: every length the recipe allows, and roughly three quarters start with a cached group prefix
    assert ((w.queries.len >= 64) & (w.queries.len <= 128 + 128 + 256)).all()
    derived = sum(tuple(w.queries.prompt(i)[:128].tolist()) in heads for i in range(w.queries.n))
    assert 0.6 * 256 <= derived <= 0.9 * 256


def test_shuffled_queue_is_definition_3():
    n, u, rep, d, s = 48, 9, 4, 5, 3
    p, user_of = W.shuffled_queue(n, u, rep, d, s, seed=11)
    assert p.n == n and (p.len == u + d).all()
    # arrivals are s * sigma(j) for a permutation sigma of 1..n
    assert sorted((p.arrival // s).tolist()) == list(range(1, n + 1))
    # n / rep user strings of length u, each shared by exactly rep queries; all document strings differ
    users = [tuple(p.prompt(i)[:u].tolist()) for i in range(n)]
    docs = [tuple(p.prompt(i)[u:].tolist()) for i in range(n)]
    assert len(set(users)) == n // rep and all(users.count(x) == rep for x in set(users))
    assert len(set(docs)) == n
    assert all(users[i] == users[j] for i in range(n) for j in range(n) if user_of[i] == user_of[j])
    # strings start with tokens of their own, so that different users (documents) share nothing
    assert len({x[0] for x in set(users)}) == n // rep and len({x[0] for x in docs}) == n
