"""Helpers for the GPU parity tests: move seeded numpy inputs to the device, run the C ABI
through the binding, bring results back as numpy.  No method arithmetic lives here."""
import numpy as np
import torch

from paper_2503_10501_amd import binding as tc


def dev(a, p):
    """float32 numpy (already rounded to the storage type) -> device tensor of the storage type."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(tc.storage_dtype(p)).contiguous()


def host(t):
    if isinstance(t, np.ndarray):   # already on the host (the large configurations convert once, not per image)
        return t
    return t.detach().to(torch.float32).cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def storage_name(p):
    return {tc.TC_F32: "f32", tc.TC_BF16: "bf16", tc.TC_F16: "f16"}[p.dtype]


def attn_output(p, Q, K, V):
    ws = tc.new_workspace(p)
    O = torch.empty(p.batch, p.n_vis, p.n_heads * p.head_dim, dtype=tc.storage_dtype(p), device="cuda")
    S = torch.empty(p.batch, p.n_vis, dtype=torch.float32, device="cuda")
    tc.tc_attn_output(p, dev(Q, p), dev(K, p), dev(V, p), O, S, ws)
    torch.cuda.synchronize()
    return O, S


def ipgs_score(p, O_dev, S_dev):
    ws = tc.new_workspace(p)
    B, N = p.batch, p.n_vis
    E = torch.empty(B, N, dtype=torch.float32, device="cuda")
    C = torch.empty(B, N, dtype=torch.float32, device="cuda")
    sig = torch.empty(B, N, dtype=torch.float32, device="cuda")
    info = torch.empty(B, dtype=torch.int32, device="cuda")
    tc.tc_ipgs_score(p, O_dev, S_dev, E, C, sig, info, ws)
    torch.cuda.synchronize()
    return E, C, sig, info


def select_topk(p, E_dev):
    ws = tc.new_workspace(p)
    order = torch.empty(p.batch, p.k_prune, dtype=torch.int32, device="cuda")
    tc.tc_select_topk(p, E_dev, order, ws)
    torch.cuda.synchronize()
    return order


def similarity(p, metric_dev, order_dev):
    ws = tc.new_workspace(p)
    nA = p.k_prune // 2
    nB = p.k_prune - nA
    sim = torch.empty(p.batch, nB, max(nA, 1), dtype=torch.float32, device="cuda")
    tc.tc_similarity(p, metric_dev, order_dev, sim, ws)
    torch.cuda.synchronize()
    return sim


def merge(p, X_dev, metric_dev, order_dev):
    ws = tc.new_workspace(p)
    B = p.batch
    X_out = torch.empty(B, p.k_final, p.hidden_dim, dtype=tc.storage_dtype(p), device="cuda")
    kept = torch.empty(B, p.k_final, dtype=torch.int32, device="cuda")
    dst = torch.empty(B, p.n_vis, dtype=torch.int32, device="cuda")
    tc.tc_merge(p, X_dev, metric_dev, order_dev, X_out, kept, dst, ws)
    torch.cuda.synchronize()
    return X_out, kept, dst


def compress(p, Q, K, V, Xvis):
    ws = tc.new_workspace(p)
    B, N = p.batch, p.n_vis
    sd = tc.storage_dtype(p)
    out = {
        "X_out": torch.empty(B, p.k_final, p.hidden_dim, dtype=sd, device="cuda"),
        "kept_idx": torch.empty(B, p.k_final, dtype=torch.int32, device="cuda"),
        "merge_dst": torch.empty(B, N, dtype=torch.int32, device="cuda"),
        "O": torch.empty(B, N, p.n_heads * p.head_dim, dtype=sd, device="cuda"),
        "E": torch.empty(B, N, dtype=torch.float32, device="cuda"),
        "order": torch.empty(B, p.k_prune, dtype=torch.int32, device="cuda"),
        "info": torch.empty(B, dtype=torch.int32, device="cuda"),
    }
    tc.tc_compress(p, Q, K, V, Xvis, out["X_out"], out["kept_idx"], out["merge_dst"], ws, O=out["O"],
                   score=out["E"], order=out["order"], info=out["info"])
    torch.cuda.synchronize()
    return out
