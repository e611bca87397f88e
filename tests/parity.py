"""Stage-wise comparison of the HIP path with the float64 oracle on identical inputs.

Every stage of the library is fed what the previous GPU stage produced, and the oracle is fed the
same bits, so that a rounding-level difference in one stage cannot cascade through the discrete
choices (sort, argmax) of the next one.  Tolerances:
  O      bf16 storage: 1 unit in the last place, |dO| <= 2^-7 |O| + 1e-5 rms;
         float32 storage (accumulated in float32): |dO| <= 2^-22 |O| + 1e-5 rms
  S      1e-4 relative
  C      1e-3 relative per token (spec tolerance; `tight` asks for 1e-4 on the fp64 solver,
         whose eigenvectors are accumulated in float32)
  E      1e-3 of max|E|; sigma: 1e-3 sigma_1
  order  exact on the GPU's own E; against the oracle's E exact outside the 1e-4 tie band
  kept_idx / merge_dst exact unless an argmax or top-m margin of the oracle is <= 1e-4
  X_out  1 unit in the last place of the storage type
"""
import numpy as np
import torch

from oracle import tokencarve_oracle as orc
from paper_2503_10501_amd import binding as tc
from tests import gpu_utils as gu


def ulp_bound(ref, dtype, rms):
    if dtype == "bf16":
        return 2.0 ** -7 * np.abs(ref) + 1e-5 * rms
    if dtype == "f16":
        return 2.0 ** -10 * np.abs(ref) + 1e-5 * rms
    return 2.0 ** -22 * np.abs(ref) + 1e-5 * rms   # float32 storage: sums are accumulated in float32


def check_attention(p, w, batch, images, O_dev, S_dev, report):
    Oh, Sh = gu.host(O_dev), gu.host(S_dev)
    sn = gu.storage_name(p)
    for i in images:
        Z, S = orc.attn_output(batch["Q"][i], batch["K"][i], batch["V"][i], w.n_sys, w.n_vis, bool(p.causal),
                               p.softmax_scale or None)
        O = orc.to_storage(Z, sn)
        rms = float(np.sqrt((O ** 2).mean()))
        # compare against the unrounded Z with half an ulp of slack on top of the final rounding
        err = np.abs(Oh[i] - O)
        viol = err > ulp_bound(O, sn, rms)
        assert not viol.any(), "image %d: %d entries of O off by more than one ulp (max %.3e, rms %.3e)" % (
            i, viol.sum(), err.max(), rms)
        rel = np.abs(Sh[i] - S) / np.maximum(S, 1e-12)
        assert rel.max() <= 1e-4, "image %d: attention score rel err %.3e" % (i, rel.max())
        report.setdefault("O_exact_frac", []).append(float((Oh[i] == O).mean()))
        report.setdefault("S_rel", []).append(float(rel.max()))


def check_ipgs(p, w, images, O_dev, S_dev, E_dev, C_dev, sig_dev, info_dev, report, tight=True):
    Oh, Sh = gu.host(O_dev).astype(np.float64), gu.host(S_dev).astype(np.float64) if S_dev is not None else None
    Eh, Ch, sh, ih = gu.host(E_dev), gu.host(C_dev), gu.host(sig_dev), gu.host(info_dev)
    c_tol = 1e-4 if tight else 1e-3
    for i in images:
        assert ih[i] > 0, "image %d: eigensolver reported %d" % (i, ih[i])
        E, C, s = orc.ipgs_score(Oh[i], None if Sh is None else Sh[i], p.lambda_, p.norm_mode, p.sv_rtol)
        c_rel = np.abs(Ch[i] - C) / C
        assert c_rel.max() <= c_tol, "image %d: C rel err %.3e (tol %.1e)" % (i, c_rel.max(), c_tol)
        e_err = np.abs(Eh[i] - E).max() / max(np.abs(E).max(), 1e-30)
        assert e_err <= (1e-4 if tight else 1e-3), "image %d: E err %.3e" % (i, e_err)
        n = min(len(s), sh.shape[1])
        s_err = np.abs(sh[i][:n] - s[:n]).max() / s[0]
        assert s_err <= (1e-5 if tight else 1e-3), "image %d: sigma err %.3e sigma_1" % (i, s_err)
        # Frobenius identity on the GPU's own spectrum: sum sigma^2 = ||O||_F^2
        fro = (Oh[i] ** 2).sum()
        assert abs((sh[i].astype(np.float64) ** 2).sum() - fro) <= (1e-5 if tight else 1e-4) * fro
        report.setdefault("C_rel", []).append(float(c_rel.max()))
        report.setdefault("sweeps", []).append(int(ih[i]))


def check_topk(p, images, E_dev, order_dev, E_oracle=None, report=None):
    Eh, oh = gu.host(E_dev).astype(np.float64), gu.host(order_dev)
    for i in images:
        expect = orc.select_topk(Eh[i], p.k_prune)
        assert np.array_equal(oh[i], expect), "image %d: order differs from the stable sort of the same scores" % i
        if E_oracle is not None:
            Eo = E_oracle[i]
            srt = np.sort(Eo)[::-1]
            cut = srt[p.k_prune - 1]
            band = 1e-4 * max(np.abs(Eo).max(), 1e-30)
            sure_in = set(np.nonzero(Eo > cut + band)[0].tolist())
            sure_out = set(np.nonzero(Eo < cut - band)[0].tolist())
            got = set(oh[i].tolist())
            assert sure_in <= got and not (sure_out & got), "image %d: kept set differs outside the tie band" % i
            if report is not None:
                report.setdefault("tie_band_tokens", []).append(len(Eo) - len(sure_in) - len(sure_out))


def check_merge(p, w, images, X_np, O_dev, order_dev, Xout_dev, kept_dev, dst_dev, report):
    Oh, oh = gu.host(O_dev).astype(np.float64), gu.host(order_dev)
    Xo, kh, dh = gu.host(Xout_dev), gu.host(kept_dev), gu.host(dst_dev)
    sn = gu.storage_name(p)
    for i in images:
        ref = orc.merge(X_np[i], Oh[i], oh[i], p.k_final, out_dtype=sn)
        # margins of the oracle's discrete choices
        tie = False
        if len(ref["set_a"]) and len(ref["set_b"]):
            sim = orc.similarity(Oh[i], ref["set_a"], ref["set_b"])
            if sim.shape[1] > 1:
                part = np.sort(sim, axis=1)
                tie |= bool((part[:, -1] - part[:, -2]).min() <= 1e-4)
            m = p.k_prune - p.k_final
            v = np.sort(ref["val"])[::-1]
            if 0 < m < len(v):
                tie |= bool(v[m - 1] - v[m] <= 1e-4)
        same = np.array_equal(kh[i], ref["kept_idx"]) and np.array_equal(dh[i], ref["merge_dst"])
        if tie and not same:
            report.setdefault("merge_ties", []).append(i)   # documented tie: several results are valid
            continue
        assert same, "image %d: kept_idx / merge_dst differ from the oracle with no tie at the margin" % i
        rms = float(np.sqrt((ref["X_out"] ** 2).mean()))
        err = np.abs(Xo[i] - ref["X_out"])
        assert not (err > ulp_bound(ref["X_out"], sn, rms)).any(), "image %d: X_out max err %.3e" % (i, err.max())
        report.setdefault("Xout_exact_frac", []).append(float((Xo[i] == ref["X_out"]).mean()))


def run_all_stages(w, images=None, eig=tc.TC_EIG_F64, oracle_images=None, tight=True, **param_overrides):
    """GPU path stage by stage on `images` of workload w, each stage checked against the oracle."""
    from workloads import make_batch
    images = list(range(w.batch)) if images is None else list(images)
    batch = make_batch(w, images)
    idx = list(range(len(images))) if oracle_images is None else list(oracle_images)
    p = tc.params_for(w, batch=len(images), eig_dtype=eig, **param_overrides)
    report = {}
    O, S = gu.attn_output(p, batch["Q"], batch["K"], batch["V"])
    check_attention(p, w, batch, idx, O, S, report)
    E, C, sig, info = gu.ipgs_score(p, O, S)
    check_ipgs(p, w, idx, O, S, E, C, sig, info, report, tight)
    order = gu.select_topk(p, E)
    Eo = {}
    for i in idx:
        Z, So = orc.attn_output(batch["Q"][i], batch["K"][i], batch["V"][i], w.n_sys, w.n_vis, bool(p.causal),
                                p.softmax_scale or None)
        Eo[i] = orc.ipgs_score(orc.to_storage(Z, gu.storage_name(p)), So, p.lambda_, p.norm_mode, p.sv_rtol)[0]
    check_topk(p, idx, E, order, Eo, report)
    Xv = np.ascontiguousarray(batch["X"][:, w.n_sys:w.n_sys + w.n_vis])
    Xd = gu.dev(Xv, p)
    X_out, kept, dst = gu.merge(p, Xd, O, order)
    check_merge(p, w, idx, Xv, O, order, X_out, kept, dst, report)
    # the one-call path must reproduce the staged path bit for bit
    whole = gu.compress(p, gu.dev(batch["Q"], p), gu.dev(batch["K"], p), gu.dev(batch["V"], p), Xd)
    assert torch.equal(whole["O"], O) and torch.equal(whole["E"], E) and torch.equal(whole["order"], order)
    assert torch.equal(whole["kept_idx"], kept) and torch.equal(whole["merge_dst"], dst)
    assert torch.equal(whole["X_out"], X_out) and torch.equal(whole["info"], info)
    # un-gated: overlap of the final kept sets with a fully independent oracle run
    jac = []
    for i in idx:
        full = orc.compress(batch["Q"][i], batch["K"][i], batch["V"][i], Xv[i], w.n_sys, w.n_vis, p.k_prune,
                            p.k_final, lam=p.lambda_, norm=p.norm_mode, causal=bool(p.causal),
                            dtype=gu.storage_name(p), sv_rtol=p.sv_rtol, scale=p.softmax_scale or None)
        a, b = set(gu.host(kept)[i].tolist()), set(full["kept_idx"].tolist())
        jac.append(len(a & b) / len(a | b))
    report["jaccard_vs_independent_oracle"] = jac
    return report
