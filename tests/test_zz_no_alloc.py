"""The selection entry point that allocates nothing (its workspace is a fixed array in the
library's device image) against kLPM_select with a caller workspace: same inputs, same outputs,
bit for bit, on consecutive calls of different sizes that share the one array."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2502_04677_amd as K
else:
    K = None


def _inputs(rng, n, ordered):
    arrival = np.sort(rng.integers(0, 4 * n, size=n)) if ordered else rng.integers(0, n // 2 + 2, size=n)
    # clustered scores with many ties, some zero, as match lengths of a queue look
    score = rng.choice([0, 0, 17, 128, 128, 129, 1024, 4095], size=n) + (rng.integers(0, 3, size=n) == 0) * rng.integers(0, 50, size=n)
    tie = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    dev = "cuda:0"
    return (torch.from_numpy(arrival.astype(np.uint64).view(np.int64)).to(dev),
            torch.from_numpy(score.astype(np.int32)).to(dev),
            torch.from_numpy(tie.view(np.int32)).to(dev))


def _both(n, k, batch, flags, ordered, use_tie, phase0, rng, n_live=None):
    arr, score, tie = _inputs(rng, n, ordered)
    tk = tie if use_tie else None
    live = None if n_live is None else torch.tensor([n_live], dtype=torch.int32, device="cuda:0")
    outs = []
    for static in (False, True):
        phase = torch.tensor([phase0], dtype=torch.int32, device="cuda:0")
        idx = torch.full((max(batch, 1),), -7, dtype=torch.int32, device="cuda:0")
        nsel = torch.full((1,), -7, dtype=torch.int32, device="cuda:0")
        if static:
            K.kLPM_select_static(arr, score, n, k, batch, phase, idx, nsel, flags=flags, max_match=8192, n_live=live,
                                 tie_key=tk)
        else:
            nbytes = K.kLPM_select_workspace_bytes(n)
            ws = K.alloc_aligned(nbytes, "cuda:0")
            K.kLPM_select(arr, score, n, k, batch, phase, idx, nsel, ws, nbytes, flags=flags, max_match=8192,
                          n_live=live, tie_key=tk)
        torch.cuda.synchronize()
        outs.append((int(nsel.item()), int(phase.item()), idx.cpu().numpy().copy()))
    (n0, p0, i0), (n1, p1, i1) = outs
    assert n0 == n1 and p0 == p1, (n, k, batch, flags, outs[0][:2], outs[1][:2])
    assert n0 == min(batch, n if n_live is None else min(n, n_live))
    assert (i0 == i1).all(), (n, k, batch, flags)


def test_select_static_equals_select_on_calls_in_a_row():
    rng = np.random.default_rng(7)
    F = K.KLPM_SELECT_FIFO
    # (n, k, batch, flags, arrival-ordered, tie keys, phase): each pair of lines is two calls in a
    # row on the shared array, the second one smaller; all paths of the selection take part
    cases = [
        (70_000, 8, 1024, F, True, False, 3),    # long arrival-ordered queue: histogram levels in the workspace
        (9_000, 8, 1024, F, True, False, 5),     # the same path, smaller
        (50_000, 4, 512, 0, False, False, 1),    # general queue: radix sorts in the workspace
        (6_000, 4, 512, 0, False, False, 2),     # smaller
        (40_000, 3, 700, F, True, True, 0),      # arrival-ordered with tie keys
        (5_000, 3, 700, F, True, True, 1),
        (30_000, 2, 300, 0, False, True, 1),     # radix sorts with tie keys
        (3_000, 2, 300, 0, False, True, 0),      # one-workgroup sort of both orders
        (K.KLPM_SELECT_STATIC_MAX_N, 8, 4096, F, True, False, 0),  # the largest size accepted
        (K.KLPM_SELECT_STATIC_MAX_N, 0, 2048, 0, False, False, 0),
        (2_000, 1, 64, F, True, False, 0),
        (100, K.KLPM_K_INFINITY, 100, 0, False, False, 0),
    ]
    for c in cases:
        print("select_static case", c, flush=True)
        _both(*c, rng)
    print("device-side queue length", flush=True)
    _both(20_000, 4, 256, F, True, False, 2, rng, n_live=11_111)
    _both(20_000, 4, 256, 0, False, False, 2, rng, n_live=9_999)


def test_select_static_limits_and_empty_calls():
    dev = "cuda:0"
    phase = torch.tensor([2], dtype=torch.int32, device=dev)
    idx = torch.zeros(8, dtype=torch.int32, device=dev)
    nsel = torch.full((1,), 9, dtype=torch.int32, device=dev)
    arr = torch.zeros(8, dtype=torch.int64, device=dev)
    m = torch.zeros(8, dtype=torch.int32, device=dev)
    with pytest.raises(K.KlpmError, match="maximum"):
        K.kLPM_select_static(arr, m, K.KLPM_SELECT_STATIC_MAX_N + 1, 2, 8, phase, idx, nsel)
    torch.cuda.synchronize()
    assert int(nsel.item()) == 9 and int(phase.item()) == 2  # nothing was enqueued
    K.kLPM_select_static(arr, m, 0, 2, 8, phase, idx, nsel)
    torch.cuda.synchronize()
    assert int(nsel.item()) == 0 and int(phase.item()) == 2
