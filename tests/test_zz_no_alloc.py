"""tc_merge_noalloc (the entry point for callers that cannot allocate) against tc_merge, through the raw C ABI."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _setup():
    from paper_2503_10501_amd import binding as tc
    from workloads.configs import Workload
    tc.load_library()
    assert torch.cuda.is_available()
    return tc, Workload


def _inputs(tc, w, seed):
    """Metric rows, hidden-state rows and a score order for `w` (any values do: both entry points get the same)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    p = tc.params_for(w)
    sd = tc.storage_dtype(p)
    B, N, D = w.batch, w.n_vis, w.hidden
    metric = torch.randn(B, N, D, generator=g).to(sd).cuda()
    X = torch.randn(B, N, D, generator=g).to(sd).cuda()
    order = torch.stack([torch.randperm(N, generator=g)[:w.k_prune] for _ in range(B)]).to(torch.int32).cuda()
    return p, sd, X, metric, order


def _run_both(tc, p, sd, X, metric, order):
    lib = tc.load_library()
    B, N = p.batch, p.n_vis
    outs = []
    for which in ("ws", "noalloc"):
        X_out = torch.full((B, p.k_final, p.hidden_dim), 7.0, dtype=sd, device="cuda")
        kept = torch.full((B, p.k_final), -5, dtype=torch.int32, device="cuda")
        dst = torch.full((B, N), -5, dtype=torch.int32, device="cuda")
        st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        args = [ctypes.byref(p)] + [ctypes.c_void_p(t.data_ptr()) for t in (X, metric, order, X_out, kept, dst)]
        if which == "ws":
            ws = tc.new_workspace(p)
            rc = lib.tc_merge(*args, ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel()), st)
        else:
            rc = lib.tc_merge_noalloc(*args, st)
        assert rc == 0, (which, rc)
        torch.cuda.synchronize()
        outs.append((X_out, kept, dst))
    return outs


def test_noalloc_merge_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    tc, Workload = _setup()
    # first a larger input, then a smaller one: the second call finds the first call's contents in the scratch
    big = Workload("na_big", 31, 3, 300, 4, 2, 2, 128, "bf16", 120, 70, 8, "powerlaw", 0.05, "iid")
    small = Workload("na_small", 32, 2, 90, 4, 2, 2, 64, "bf16", 31, 20, 8, "powerlaw", 0.05, "iid")
    for w, seed in ((big, 1), (small, 2)):
        p, sd, X, metric, order = _inputs(tc, w, seed)
        (Xa, ka, da), (Xb, kb, db) = _run_both(tc, p, sd, X, metric, order)
        assert torch.equal(ka, kb) and torch.equal(da, db), w.name      # index work: bit exact
        assert torch.equal(Xa, Xb), w.name                              # same kernels, same arithmetic: bit exact
        assert int((da >= 0).sum()) == w.batch * w.k_prune
        assert int((ka >= 0).sum()) == w.batch * w.k_final


def test_noalloc_merge_rejects_sizes_beyond_its_scratch():
    tc, Workload = _setup()
    lib = tc.load_library()
    # |A| |B| B floats = 4 * 1024 * 1024 * 8 = 32 MiB > 16 MiB; the check is on the host, nothing is launched
    w = Workload("na_huge", 33, 8, 2048, 0, 0, 1, 64, "bf16", 2048, 1024, 8, "powerlaw", 0.05, "iid")
    p = tc.params_for(w)
    dummy = torch.zeros(64, dtype=torch.int32, device="cuda")
    a = ctypes.c_void_p(dummy.data_ptr())
    rc = lib.tc_merge_noalloc(ctypes.byref(p), a, a, a, a, a, a, None)
    assert rc == -8
    assert b"scratch" in lib.tc_status_string(rc)
