"""GPU parity tests for the entry points beyond the compression path: information quantity (matrix
rank), sequence re-assembly with original position ids and rotary tables, KV-cache share."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _mods():
    from oracle import tokencarve_oracle as orc
    from paper_2503_10501_amd import binding as tc
    from tests import gpu_utils as gu
    from workloads import CONFIGS, make_batch
    tc.load_library()
    assert torch.cuda.is_available()
    return tc, gu, orc, CONFIGS, make_batch


def _rank(tc, p, O_dev, rows=None, rtol=0.0, want_sigma=True):
    B = p.batch
    n = rows.shape[1] if rows is not None else p.n_vis
    rank = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    sigma = torch.empty(B, n, dtype=torch.float32, device="cuda") if want_sigma and n > 0 else None
    info = torch.empty(B, dtype=torch.int32, device="cuda")
    ws = tc.new_workspace(p)
    tc.tc_info_rank(p, O_dev, rank, ws, rows=rows, rtol=rtol, sigma=sigma, info=info)
    torch.cuda.synchronize()
    return rank.cpu().numpy(), None if sigma is None else sigma.cpu().numpy().astype(np.float64), info.cpu().numpy()


def _check_rank(orc, O_host, rows_host, rtol, rank, sigma, info):
    """Rank must equal the oracle's count unless a singular value lies within 1e-3 of the threshold;
    sigma to 1e-5 sigma_max."""
    for i in range(len(rank)):
        assert info[i] > 0
        rt = None if rtol == 0.0 else float(np.float32(rtol))
        r, s = orc.info_rank(O_host[i], None if rows_host is None else rows_host[i], rt)
        n = len(s)
        if sigma is not None:
            assert np.abs(sigma[i][:n] - s).max() <= 1e-5 * s[0]
            assert np.all(sigma[i][n:] <= 1e-5 * s[0])   # more rows than columns: the surplus is zero
        n_rows = O_host[i].shape[0] if rows_host is None else len(rows_host[i])
        thr = (rt if rt is not None else max(O_host[i].shape[1], n_rows) * 2.0 ** -23) * s[0]
        # a singular value within 1e-3 of the threshold may be counted either way
        lo, hi = int((s > thr * (1 + 1e-3)).sum()), int((s > thr * (1 - 1e-3)).sum())
        assert lo <= rank[i] <= hi, (i, rank[i], lo, hi)
        if lo == hi:
            assert rank[i] == r


def test_rank_of_planted_low_rank_rows_float32():
    tc, gu, orc, CONFIGS, _ = _mods()
    from workloads.generate import planted_lowrank
    g = np.random.Generator(np.random.Philox(91))
    O = np.stack([planted_lowrank(g, 64, 256, np.linspace(10.0, 1.0, r), 0.01).astype(np.float32) for r in (8, 3)])
    p = tc.params_for(CONFIGS["tiny"], batch=2)
    Od = torch.from_numpy(O).cuda()
    rank, sigma, info = _rank(tc, p, Od, rtol=0.05)       # between noise (about 0.24) and signal (>= 1)
    assert rank.tolist() == [8, 3]
    _check_rank(orc, O.astype(np.float64), None, 0.05, rank, sigma, info)
    rank, sigma, info = _rank(tc, p, Od)                   # default threshold: the noise makes it full rank
    assert rank.tolist() == [64, 64]
    _check_rank(orc, O.astype(np.float64), None, 0.0, rank, sigma, info)


def test_rank_of_kept_rows_on_ragged_subsets():
    tc, gu, orc, CONFIGS, _ = _mods()
    from workloads.generate import planted_lowrank
    g = np.random.Generator(np.random.Philox(92))
    B, N, D = 3, 200, 512
    O = np.stack([planted_lowrank(g, N, D, 30.0 * np.arange(1, 25.0) ** -0.8, 0.02).astype(np.float32) for _ in range(B)])
    from workloads.configs import Workload
    w = Workload("rk", 31, B, N, 4, 4, 4, 128, "f32", 50, 40, 24, "powerlaw", 0.02, "iid")
    p = tc.params_for(w)
    Od = torch.from_numpy(O).cuda()
    for k in (200, 130, 65, 64, 17, 5, 1):
        rows = np.stack([np.sort(g.permutation(N)[:k]) for _ in range(B)]).astype(np.int32)
        rank, sigma, info = _rank(tc, p, Od, rows=torch.from_numpy(rows).cuda(), rtol=0.03)
        _check_rank(orc, O.astype(np.float64), rows, 0.03, rank, sigma, info)
        assert np.all(rank <= k)
    # no rows at all
    rank, _, _ = _rank(tc, p, Od, rows=torch.empty(B, 0, dtype=torch.int32, device="cuda"))
    assert rank.tolist() == [0, 0, 0]


def test_rank_before_and_after_compression_llava7b_single_image():
    """The rank-versus-kept-tokens curve of Section 3.2.2 at the paper's token counts, on the rows the
    GPU path itself keeps (bf16 storage, 576 x 4096)."""
    tc, gu, orc, CONFIGS, make_batch = _mods()
    w = CONFIGS["llava7b_b1"]
    b = make_batch(w, [0])
    counts = [(192, 128), (96, 64)]
    p0 = tc.params_for(w, batch=1)
    Q, K, V = gu.dev(b["Q"], p0), gu.dev(b["K"], p0), gu.dev(b["V"], p0)
    Xv = gu.dev(b["X"][:, w.n_sys:w.n_sys + w.n_vis], p0)
    ranks = []
    for kp, kf in counts:
        p = tc.params_for(w, batch=1, k_prune=kp, k_final=kf)
        out = gu.compress(p, Q, K, V, Xv)
        Oh = gu.host(out["O"]).astype(np.float64)
        kept = out["kept_idx"]
        rank, sigma, info = _rank(tc, p, out["O"], rows=kept, rtol=0.02)
        _check_rank(orc, Oh, kept.cpu().numpy(), 0.02, rank, sigma, info)
        ranks.append(int(rank[0]))
    rank_all, sigma_all, info = _rank(tc, p0, out["O"], rtol=0.02)
    _check_rank(orc, Oh, None, 0.02, rank_all, sigma_all, info)
    assert rank_all[0] >= ranks[0] >= ranks[1] > 0          # dropping tokens never raises the rank


def test_rank_rejects_bad_arguments():
    tc, gu, orc, CONFIGS, _ = _mods()
    p = tc.params_for(CONFIGS["tiny"], batch=1)
    O = torch.zeros(1, 64, 256, device="cuda")
    rank = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = tc.new_workspace(p)
    with pytest.raises(tc.TokenCarveError):
        tc.tc_info_rank(p, O, rank, ws, rtol=1e-9)
    with pytest.raises(tc.TokenCarveError):
        tc.tc_info_rank(p, O, rank, ws, rows=torch.zeros(1, 65, dtype=torch.int32, device="cuda"))
    tc.tc_info_rank(p, O, rank, ws, rtol=0.1)             # an all-zero matrix has rank 0
    torch.cuda.synchronize()
    assert rank.item() == 0


@pytest.mark.parametrize("name", ["tiny", "llava7b_b1"])
def test_assembled_sequence_positions_and_rotary_tables(name):
    tc, gu, orc, CONFIGS, make_batch = _mods()
    w = CONFIGS[name]
    nb = min(w.batch, 2)
    b = make_batch(w, list(range(nb)))
    p = tc.params_for(w, batch=nb)
    sd = tc.storage_dtype(p)
    H = gu.dev(b["X"], p)                                   # [B, L, hidden]
    out = gu.compress(p, gu.dev(b["Q"], p), gu.dev(b["K"], p), gu.dev(b["V"], p),
                      H[:, w.n_sys:w.n_sys + w.n_vis].contiguous())
    L = w.n_sys + w.n_vis + w.n_prompt
    Ln = L - w.n_vis + w.k_final
    H_new = torch.empty(nb, Ln, w.hidden, dtype=sd, device="cuda")
    pos = torch.empty(nb, Ln, dtype=torch.int32, device="cuda")
    rc = torch.empty(nb, Ln, w.head_dim // 2, dtype=torch.float32, device="cuda")
    rs = torch.empty_like(rc)
    tc.tc_assemble_sequence(p, H, out["X_out"], out["kept_idx"], H_new, pos, 10000.0, rc, rs)
    torch.cuda.synchronize()
    Hh, Xo, kept = gu.host(H), gu.host(out["X_out"]), out["kept_idx"].cpu().numpy()
    for i in range(nb):
        Hn, pid = orc.assemble_sequence(Hh[i], Xo[i], kept[i], w.n_sys, w.n_vis)
        assert np.array_equal(gu.host(H_new)[i], Hn.astype(np.float32))       # rows are copied bit for bit
        assert np.array_equal(pos[i].cpu().numpy(), pid)
        c, s = orc.rope_tables(pid, w.head_dim, 10000.0)
        assert np.abs(rc[i].cpu().numpy() - c).max() <= 1.2e-7               # float64 evaluation, one rounding to float32
        assert np.abs(rs[i].cpu().numpy() - s).max() <= 1.2e-7
    # without rotary tables, and keeping every visual token: the sequence comes back unchanged
    pa = tc.params_for(w, batch=nb, k_prune=w.n_vis, k_final=w.n_vis)
    ident = torch.arange(w.n_vis, dtype=torch.int32, device="cuda").repeat(nb, 1).contiguous()
    H_same = torch.empty(nb, L, w.hidden, dtype=sd, device="cuda")
    pos2 = torch.empty(nb, L, dtype=torch.int32, device="cuda")
    tc.tc_assemble_sequence(pa, H, H[:, w.n_sys:w.n_sys + w.n_vis].contiguous(), ident, H_same, pos2)
    torch.cuda.synchronize()
    assert torch.equal(H_same, H)
    assert torch.equal(pos2, torch.arange(L, dtype=torch.int32, device="cuda").repeat(nb, 1))
    with pytest.raises(tc.TokenCarveError):
        tc.tc_assemble_sequence(p, H, out["X_out"], out["kept_idx"], H_new, pos, 10000.0, rc, None)


def test_kv_cache_share_matches_the_oracle():
    tc, gu, orc, CONFIGS, _ = _mods()
    for args in ((80, 576, 192, 32, 2), (80, 576, 64, 32, 2), (64, 2880, 640, 40, 2), (0, 1, 0, 1, 0)):
        assert abs(tc.tc_kv_cache_fraction(*args) - orc.kv_cache_fraction(*args)) < 1e-15
    assert tc.tc_kv_cache_fraction(80, 576, 577, 32, 2) == -1.0
