"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, and its
host-side argument validation and sizing logic behave (no kernel is launched here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "klpm.h")


@pytest.fixture(scope="module")
def K():
    import paper_2502_04677_amd as K

    return K


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kLPM_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol(K):
    from paper_2502_04677_amd import binding

    lib = C.CDLL(os.path.join(ROOT, "paper_2502_04677_amd", "libklpm.so"))
    names = declared_functions()
    assert {"kLPM_build_tree", "kLPM_match", "kLPM_select", "kLPM_commit"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTS)
    for n in names:  # the binding carries the same names
        assert hasattr(K, n) or n in ("kLPM_snapshot_bytes", "kLPM_strerror"), n


def test_struct_layouts_match_header(K):
    from paper_2502_04677_amd import binding

    assert C.sizeof(binding.Queries) == 56
    assert C.sizeof(binding.Arrivals) == 32 and C.sizeof(binding.Queue) == 64
    assert C.sizeof(binding.Config) == 32
    assert C.sizeof(binding.Stats) == 48 and binding.STATS_BYTES == 48
    assert C.sizeof(binding.AdaptConfig) == 88 and C.sizeof(binding.AdaptStats) == 280


def test_arena_sizing_and_config_validation(K):
    from paper_2502_04677_amd import binding

    small = K.kLPM_arena_bytes(K.make_config(1000, 10_000, 100, 16, 64))
    big = K.kLPM_arena_bytes(K.make_config(1000, 20_000, 100, 16, 64))
    assert big - small >= 2 * 10_000 * 4 - 256  # two pool halves of int32 tokens (sub-ranges are 256-byte aligned)
    assert small % 256 == 0
    for bad in (K.make_config(-1, 10, 10, 1, 8), K.make_config(10, 0, 10, 1, 8), K.make_config(10, 10, 1, 1, 8),
                K.make_config(10, 10, 10, 0, 8), K.make_config(10, 10, 10, 1, 0), K.make_config(10, 10, 10, 70000, 8)):
        with pytest.raises(K.KlpmError):
            K.kLPM_arena_bytes(bad)
    lib = binding._lib
    assert lib.kLPM_arena_bytes(None, None) == -1
    assert lib.kLPM_strerror(0) == b"ok" and b"invalid" in lib.kLPM_strerror(-1)
    assert b"arena" in lib.kLPM_strerror(-2) and b"unknown" in lib.kLPM_strerror(-77)


def test_select_workspace_grows_with_n(K):
    a, b = K.kLPM_select_workspace_bytes(0), K.kLPM_select_workspace_bytes(100_000)
    assert 0 < a < b and b >= 100_000 * (8 + 8 + 4 * 5)
    with pytest.raises(K.KlpmError):
        K.kLPM_select_workspace_bytes(-1)


def test_null_and_negative_arguments_are_rejected_before_any_launch(K):
    from paper_2502_04677_amd import binding

    lib = binding._lib
    cfg = K.make_config(100, 1000, 16, 4, 32)
    out = C.c_void_p(0)
    assert lib.kLPM_build_tree(C.byref(out), C.byref(cfg), None, 0, None, None) == -1  # no arena
    assert lib.kLPM_build_tree(None, C.byref(cfg), C.c_void_p(256), 1 << 30, None, None) == -1
    # misaligned / too small arena
    assert lib.kLPM_build_tree(C.byref(out), C.byref(cfg), C.c_void_p(264), 1 << 30, None, None) == -2
    assert lib.kLPM_build_tree(C.byref(out), C.byref(cfg), C.c_void_p(256), 16, None, None) == -2
    q = binding.Queries(0, 0, 0, 0, 0, -1)
    assert lib.kLPM_match(None, C.byref(q), None, None, None) == -1
    assert lib.kLPM_commit(None, C.byref(q), None, None, 0, None, None) == -1
    assert lib.kLPM_set_budget(None, 5) == -1
    # timed queue advance: no arrival list, zero denominator of the attention coefficient
    qa, qb = binding.Queue(8, 8, 8, 8, 8, 8, 8, 0), binding.Queue(16, 16, 16, 16, 16, 16, 16, 0)
    q0 = binding.Queries(0, 0, 0, 0, 0, 0, 0)
    args = (C.byref(qa), C.byref(qb), C.byref(q0), None, None, C.c_void_p(8), 0)
    tail = (C.c_void_p(8), None, None, None)
    assert lib.kLPM_queue_advance_timed(*args, None, *tail) == -1
    bad = binding.Arrivals(0, 0, 0, 1, 0)
    assert lib.kLPM_queue_advance_timed(*args, C.byref(bad), *tail) == -1
    ok = binding.Arrivals(0, 0, 0, 0, 1)
    # the two buffer sets must be distinct, and a timed run needs the joined counters
    assert lib.kLPM_queue_advance_timed(C.byref(qa), C.byref(qa), C.byref(q0), None, None, C.c_void_p(8), 0, C.byref(ok), *tail) == -1
    no_join = binding.Queue(16, 16, 16, 16, 16, 16, 0, 0)
    assert lib.kLPM_queue_advance_timed(C.byref(qa), C.byref(no_join), C.byref(q0), None, None, C.c_void_p(8), 0, C.byref(ok), *tail) == -1
    assert lib.kLPM_read_stats(None, None, None) == -1
    assert lib.kLPM_snapshot(None, None, 0, None, None) == -1
    # in-batch rescoring: no queue, a queue beyond the limit of the state bits, no workspace
    dyn_tail = (2, None, 8, K.KLPM_SELECT_FIFO, 100, C.c_void_p(8), C.c_void_p(8), C.c_void_p(8), C.c_void_p(8))
    assert lib.kLPM_select_dynamic(None, None, None, *dyn_tail, None, 0, None) == -1
    big = binding.Queries(8, 8, 8, 8, 1 << 20, 300_000)
    assert lib.kLPM_select_dynamic(C.byref(big), C.c_void_p(8), C.c_void_p(8), *dyn_tail, C.c_void_p(256), 1 << 40, None) == -1
    some = binding.Queries(8, 8, 8, 8, 1 << 20, 5000)
    assert lib.kLPM_select_dynamic(C.byref(some), C.c_void_p(8), C.c_void_p(8), *dyn_tail, None, 0, None) == -2
    assert lib.kLPM_select_dynamic(C.byref(some), C.c_void_p(8), C.c_void_p(8), *dyn_tail, C.c_void_p(256), 64, None) == -2
    assert lib.kLPM_destroy(None) == 0


def test_size_config_leaves_room_for_a_batch(K):
    cfg = K.size_config(cache_tokens=1_000_000, cache_prompts=500, budget=600_000, max_batch=64, max_prompt_len=4096)
    assert cfg.pool_tokens >= 600_000 + 64 * 4096 and cfg.max_nodes >= 2 * 500 + 2 * 64
    assert cfg.budget_tokens == 600_000


def test_adaptive_k_arguments_are_validated_on_the_host(K):
    from paper_2502_04677_amd import binding

    lib = binding._lib
    assert K.kLPM_adapt_state_bytes() % 256 == 0 and K.kLPM_adapt_state_bytes() >= 384
    fake = 0x1000  # never dereferenced: every call below is refused before anything is enqueued

    def init(n_arms, window, explore, nbytes=4096, addr=fake):
        cfg = binding.AdaptConfig()
        cfg.n_arms, cfg.window, cfg.explore, cfg.seed = n_arms, window, explore, 0
        return lib.kLPM_adapt_init(C.c_void_p(addr), nbytes, C.byref(cfg), None)

    assert init(0, 1, 0) != 0 and init(17, 1, 0) != 0 and init(-1, 1, 0) != 0
    assert init(2, 0, 0) != 0 and init(2, 1, (1 << 32) + 1) != 0
    assert init(2, 1, 0, nbytes=64) != 0 and init(2, 1, 0, addr=fake + 4) != 0 and init(2, 1, 0, addr=0) != 0
    assert lib.kLPM_adapt_init(C.c_void_p(fake), 4096, None, None) != 0
    assert K.kLPM_adapt_k(fake) == fake  # the current k is the first word of the state
    assert lib.kLPM_adapt_k(None, None) != 0 and lib.kLPM_adapt_read(None, None, None) != 0
    assert lib.kLPM_adapt_observe(None, None, None, None, 0, None, 0, None) != 0


def test_select_static_refuses_sizes_beyond_its_maximum_on_the_host(K):
    """The limit check comes before anything touches a GPU, so it can be seen on a CPU-only host."""
    from paper_2502_04677_amd import binding

    rc = binding._lib.kLPM_select_static(None, None, None, K.KLPM_SELECT_STATIC_MAX_N + 1, None, 2, None, 8, 0, 0, None,
                                         None, None, None)
    assert rc == K.KLPM_ELIMIT and b"maximum" in binding._lib.kLPM_strerror(rc)
