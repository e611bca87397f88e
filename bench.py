#!/usr/bin/env python3
"""Benchmark of the TokenCarve compression path on one MI355X.

One step = one tc_compress call (attention output -> IPGS score -> prune -> merge) over one batch of
synthetic LLaVA-1.5-7B-shaped inputs (batch 64, 576 visual + 64 text tokens, D = 4096, bf16,
576 -> 128 -> 64 tokens), inputs resident in HBM, library default parameters.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llava7b_b64] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"hbm_gbps": 8000.0, "mfma_bf16": 2500.0, "mfma_f64": 78.6, "mfma_f32": 157.3, "vec_f64": 78.6, "vec_f32": 157.3}


# ---- algorithmic work per batch (what the method must move or compute) ---------------------------------------
def panel_ends(n_vis):
    """Last column + 1 of every panel of the reduction to tridiagonal form: the panel width is what fits the 160 KB of
    LDS of a compute unit next to two vectors and the partial sums of the matrix-vector product (the library's sizing
    rule, csrc/tridiag.hip)."""
    nr = (n_vis + 15) // 16 * 16
    row_sums = sum(nr - k for k in range(128, nr, 128))   # row sums of the matrix-vector product, one double each
    nb = min(32, ((160 * 1024 - 1024 - 2048 * 8 - 2 * nr * 8 - 8 * row_sums) // (16 * nr)) & ~3)
    return [min(j0 + nb, n_vis - 1) for j0 in range(0, n_vis - 1, max(nb, 1))]


def work_model(w):
    B, N, D, H, dh, Ls = w.batch, w.n_vis, w.hidden, w.n_heads, w.head_dim, w.n_sys
    es = 4 if w.dtype == "f32" else 2
    kp, kf = w.k_prune, w.k_final
    nA = kp // 2
    nB = kp - nA
    pairs = N * Ls + N * (N + 1) // 2 if w.causal else N * (Ls + N + w.n_prompt)     # (query, key) pairs per head
    keys = Ls + N if w.causal else Ls + N + w.n_prompt
    return {
        # Eq. 3-1/3-2: QK^T and PV, 2 * 2 * d_h flops per pair
        "attn_flops": B * H * pairs * 4 * dh,
        "attn_bytes": B * es * D * (N + 2 * keys + N),            # Q rows, K and V rows, O written
        # Gram: lower triangle of 2 N^2 D
        "gram_flops": B * N * N * D,
        "gram_bytes": B * (es * N * D + 8 * N * N),
        # reduction to tridiagonal form: per column the symmetric trailing matrix once (its lower half),
        # plus the rank-2 updates (read and write of the lower half once per column pair v, w): N^3/6 * 8 * (1 + 2/nb)
        "tridiag_bytes": B * 8 * sum((N - j - 1) * (N - j) // 2 for j in range(N - 1)),
        "tridiag_flops": B * 4 * N ** 3 // 3,
        # rank-2nb update of the trailing matrix after every panel: its lower half read and written once
        "tridiag_update_bytes": B * 16 * sum((N - je) * (N - je + 1) // 2 for je in panel_ends(N)),
        # twisted factorisations: pivots and multipliers written and read once (2 * 8 N^2 each way), vectors written (4 N^2)
        "twisted_bytes": B * N * N * (16 + 16 + 4),
        # back-transformation: 4 N^3 / 2 ... each reflector touches (N-j-1) rows of N columns, 4 flops each
        "backtf_flops": B * 4 * N * sum(N - j - 1 for j in range(N - 1)),
        "backtf_bytes": B * N * N * (4 + 4),                      # vectors of T and reflectors read once
        # Eq. 3-10 similarity and the merge
        "sim_flops": B * 2 * nA * nB * D,
        "sim_bytes": B * (kp * D * es + 4 * nA * nB),
        "rownorm_bytes": B * kp * D * es,
        "average_bytes": B * (kp + kf) * w.hidden * es,
        # Jacobi method (when it runs): Eq. 3-6 reads U once
        "ics_bytes": B * 4 * N * N,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llava7b_b64")
    ap.add_argument("--method", default="auto", choices=["auto", "jacobi", "tridiagonal"])
    ap.add_argument("--groups", type=int, default=0, help="Jacobi method: stream groups (0 = library default, 1 = one stream)")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--path-only", action="store_true",
                    help="time the compression path only: no rate probe, no other workloads or methods, no entry points "
                         "beyond the path (keeps kernel traces clean)")
    ap.add_argument("--cpu-sample", type=int, default=12, help="images timed through the CPU oracle")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards by image with no exchange "
              "between GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_10501_amd import binding as tc
    from workloads import CONFIGS, make_batch

    tc.load_library()  # fails loudly when the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    w = CONFIGS[args.workload]
    t0 = time.time()
    batch = make_batch(w)
    gen_s = time.time() - t0
    method = {"auto": tc.TC_EIG_AUTO, "jacobi": tc.TC_EIG_JACOBI, "tridiagonal": tc.TC_EIG_TRIDIAGONAL}[args.method]
    p = tc.params_for(w, eig_method=method, stream_groups=args.groups)
    sd = tc.storage_dtype(p)

    def dev(a):
        return torch.from_numpy(a).cuda().to(sd).contiguous()

    Q, K, V = dev(batch["Q"]), dev(batch["K"]), dev(batch["V"])
    X = dev(np.ascontiguousarray(batch["X"][:, w.n_sys:w.n_sys + w.n_vis]))
    B, N = w.batch, w.n_vis

    def outputs(pp):
        return (torch.empty(B, pp.k_final, w.hidden, dtype=sd, device="cuda"),
                torch.empty(B, pp.k_final, dtype=torch.int32, device="cuda"),
                torch.empty(B, N, dtype=torch.int32, device="cuda"),
                torch.empty(B, dtype=torch.int32, device="cuda"))

    X_out, kept, dst, info = outputs(p)
    ws = tc.new_workspace(p)
    if args.copy_calib:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst_c = torch.empty_like(src)
        dst_c.copy_(src)            # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst_c

    def timed_steps(pp, outs, wsp, steps, warmup):
        """ms per tc_compress call, and host time per call spent enqueuing it."""
        for _ in range(warmup):
            tc.tc_compress(pp, Q, K, V, X, outs[0], outs[1], outs[2], wsp, info=outs[3])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        host = 0.0
        for _ in range(steps):
            h0 = time.perf_counter()
            tc.tc_compress(pp, Q, K, V, X, outs[0], outs[1], outs[2], wsp, info=outs[3])
            host += time.perf_counter() - h0
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, host * 1e3 / steps

    # the timed region: library default parameters, nothing calibrated
    tc.tc_compress(p, Q, K, V, X, X_out, kept, dst, ws, info=info)
    torch.cuda.synchronize()
    status = info.cpu().numpy()
    if (status <= 0).any():
        print("bench.py: eigensolver failed for some image: %s" % status, file=sys.stderr)
        sys.exit(1)
    kept_ref = kept.clone()
    ms_per_step, host_ms = timed_steps(p, (X_out, kept, dst, info), ws, args.steps, args.warmup)
    if (info.cpu().numpy() <= 0).any() or not torch.equal(kept, kept_ref):
        print("bench.py: timed runs disagree with the first run", file=sys.stderr)
        sys.exit(1)

    # per-kernel durations, measured live with HIP events on the launch stream (kernels run one at a time)
    kinds, _ = tc.tc_profile_compress(p, Q, K, V, X, X_out, kept, dst, info, ws)
    kinds, _ = tc.tc_profile_compress(p, Q, K, V, X, X_out, kept, dst, info, ws)
    tiles_done = kinds.pop("jacobi_update_tiles")[1]
    rot_steps = kinds.pop("jacobi_rotation_steps")[1]
    kernel_ms = {k: round(v[0], 4) for k, v in kinds.items() if v[1] > 0}
    launches = {k: v[1] for k, v in kinds.items() if v[1] > 0}
    wm = work_model(w)

    def ms(k):
        return kinds[k][0] if kinds[k][1] > 0 else None

    def rate(work, k, unit):   # work / time of kernel kind k; unit "T" = 1e12 per s, "G" = 1e9 per s
        t = ms(k)
        return None if not t else work / (t * 1e-3) / (1e12 if unit == "T" else 1e9)

    def entry(kernel, bound, achieved, peak, unit, **extra):
        d = {"kernel": kernel, "bound": bound, "achieved": None if achieved is None else round(achieved, 3),
             "peak": peak, "unit": unit, "frac": None if achieved is None else round(achieved / peak, 4)}
        d.update(extra)
        return d

    # ---- per row of the path: achieved rate against the peak of the unit that bounds it -------------------
    attn_t = rate(wm["attn_flops"], "attn", "T")
    attn_ai = wm["attn_flops"] / wm["attn_bytes"]
    attn_cap = min(PEAK["mfma_bf16"], attn_ai * PEAK["hbm_gbps"] / 1e3)       # TFLOP/s the HBM can feed at this intensity
    per_row = {
        "a1_a2_attention": entry("attn", "mfma", attn_t, PEAK["mfma_bf16"] if w.dtype != "f32" else PEAK["vec_f32"], "TFLOP/s",
                                 ms=ms("attn"), flop_per_byte=round(attn_ai, 1),
                                 frac_of_min_mfma_hbm=None if attn_t is None else round(attn_t / attn_cap, 4)),
        "a3_gram": entry("gram", "mfma", rate(wm["gram_flops"], "gram", "T"), PEAK["mfma_f64"], "TFLOP/s", ms=ms("gram"),
                         hbm_gbps=None if not ms("gram") else round(rate(wm["gram_bytes"], "gram", "G"), 1)),
        "a8_similarity": entry("sim", "hbm", rate(wm["sim_bytes"], "sim", "G"), PEAK["hbm_gbps"], "GB/s", ms=ms("sim"),
                               mfma_tflops=None if not ms("sim") else round(rate(wm["sim_flops"], "sim", "T"), 2)),
        "a8_rownorm_gather": entry("rownorm", "hbm", rate(wm["rownorm_bytes"], "rownorm", "G"), PEAK["hbm_gbps"], "GB/s",
                                   ms=ms("rownorm")),
        "a9_average": entry("average", "hbm", rate(wm["average_bytes"], "average", "G"), PEAK["hbm_gbps"], "GB/s",
                            ms=ms("average")),
        "a7_topk": {"kernel": "topk", "bound": "lds/latency", "ms": ms("topk")},
        "a9_assign": {"kernel": "assign", "bound": "lds/latency", "ms": ms("assign")},
    }
    if kinds["tridiag"][1] > 0:   # the tridiagonal route ran
        per_row["a4_tridiagonal_reduction"] = entry("tridiag", "hbm", rate(wm["tridiag_bytes"], "tridiag", "G"), PEAK["hbm_gbps"],
                                                    "GB/s", ms=ms("tridiag"))
        per_row["a4_trailing_update"] = entry("tridiag_update", "hbm", rate(wm["tridiag_update_bytes"], "tridiag_update", "G"),
                                              PEAK["hbm_gbps"], "GB/s", ms=ms("tridiag_update"))
        per_row["a4_bisection"] = {"kernel": "bisect", "bound": "alu (float64 divisions, one lane per eigenvalue)", "ms": ms("bisect")}
        per_row["a4_twisted_factorisation"] = entry("twisted", "hbm", rate(wm["twisted_bytes"], "twisted", "G"), PEAK["hbm_gbps"],
                                                    "GB/s", ms=ms("twisted"))
        per_row["a4_a5_backtransform_ics"] = entry("backtransform", "alu", rate(wm["backtf_flops"], "backtransform", "T"),
                                                   PEAK["vec_f32"], "TFLOP/s", ms=ms("backtransform"))
    else:
        per_row["a5_ics"] = entry("ics", "hbm", rate(wm["ics_bytes"], "ics", "G"), PEAK["hbm_gbps"], "GB/s", ms=ms("ics"))
        solve_flops = rot_steps * (528 * 24 + 4096 * 3)
        per_row["a4_jacobi_solve"] = entry("jacobi_solve", "alu", rate(solve_flops, "jacobi_solve", "T"), PEAK["vec_f64"], "TFLOP/s",
                                           ms=ms("jacobi_solve"))
        per_row["a4_jacobi_update_g"] = entry("jacobi_update", "mfma", rate(tiles_done * 4 * 64 ** 3, "jacobi_update", "T"),
                                              PEAK["mfma_f64"], "TFLOP/s", ms=ms("jacobi_update"))
        per_row["a4_jacobi_update_u"] = {"kernel": "jacobi_update_u", "bound": "mfma", "ms": ms("jacobi_update_u")}

    # ---- roofline of the dominant kernel: the one with the largest summed time ------------------------------
    dominant = max(kernel_ms, key=kernel_ms.get)
    dom_row = next((v for v in per_row.values() if v.get("kernel") == dominant and "achieved" in v), None)
    traffic = None   # HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel and workload, if any
    pmc = os.path.join(ROOT, "profiles", "%s.%s.pmc.txt" % (dominant, w.name))
    if os.path.exists(pmc):
        for line in open(pmc):
            if line.startswith("hbm_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
    roofline = {"kernel": dominant, "bound": dom_row["bound"] if dom_row else None,
                "achieved": dom_row["achieved"] if dom_row else None, "peak": dom_row["peak"] if dom_row else None,
                "unit": dom_row["unit"] if dom_row else None, "frac": dom_row["frac"] if dom_row else None,
                "traffic": traffic, "launches": launches[dominant],
                "avg_launch_us": round(kernel_ms[dominant] * 1e3 / launches[dominant], 2)}

    out = {
        "metric": "images/sec compressed (576x4096 -> k_prune -> k_final tokens, batch 64)",
        "value": round(B / (ms_per_step * 1e-3), 2),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "host_enqueue_ms_per_step": round(host_ms, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 storage; fp32-accumulate bf16 MFMA (attention, similarity); f64 Gram + eigensolver",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "n_vis": N, "n_text": w.n_sys + w.n_prompt,
                   "hidden": w.hidden, "heads": w.n_heads, "head_dim": w.head_dim,
                   "k_prune": w.k_prune, "k_final": w.k_final, "lambda": w.lam, "causal": w.causal,
                   "qkv": w.qkv_mode, "params": "library defaults", "eig_method": args.method,
                   "eig_method_used": "tridiagonal" if kinds["tridiag"][1] > 0 else "jacobi",
                   "eigensolver_status_min_max": [int(status.min()), int(status.max())],
                   "input_generation_s": round(gen_s, 1)},
        "roofline": roofline,
        "per_row": per_row,
        "kernel_ms": kernel_ms,
        "kernel_launches": launches,
        "kernel_ms_total": round(sum(kernel_ms.values()), 3),
    }

    if not args.path_only:
        out["sustained_rates"] = {k: round(v, 1) for k, v in tc.tc_probe_rates().items()}
        # the counts of the metric string (576 -> 256 -> 192 tokens) at the same batch
        p2 = tc.params_for(w.with_(k_prune=256, k_final=192), eig_method=method, stream_groups=args.groups)
        o2 = outputs(p2)
        ms2, _ = timed_steps(p2, o2, ws if tc.tc_workspace_bytes(p2) <= ws.numel() else tc.new_workspace(p2), max(args.steps // 2, 3), 2)
        out["metric_string_counts"] = {"k_prune": 256, "k_final": 192, "ms_per_step": round(ms2, 3),
                                       "value": round(B / (ms2 * 1e-3), 2), "unit": "images/s"}
        # Not the headline: the same K steps issued round-robin on several streams, each with its own workspace and
        # outputs.  Behind the Gram matrix a step keeps 64 to 768 wavefronts busy, so independent batches overlap;
        # a serving loop with more than one batch queued would see this rate.
        def in_flight(n_streams, steps):
            pf = tc.params_for(w, eig_method=method, stream_groups=1)
            streams = [torch.cuda.Stream() for _ in range(n_streams)]
            sets = [(outputs(pf), tc.new_workspace(pf)) for _ in range(n_streams)]
            for (o, wsp) in sets:
                tc.tc_compress(pf, Q, K, V, X, o[0], o[1], o[2], wsp, info=o[3])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                o, wsp = sets[i % n_streams]
                tc.tc_compress(pf, Q, K, V, X, o[0], o[1], o[2], wsp, info=o[3], stream=streams[i % n_streams].cuda_stream)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) * 1e3 / steps
            ok = all(torch.equal(o[1], kept_ref) and bool((o[3] > 0).all()) for o, _ in sets)
            return {"streams": n_streams, "ms_per_step": round(dt, 3), "value": round(B / (dt * 1e-3), 2),
                    "unit": "images/s", "results_equal_to_single_stream": ok}
        out["several_batches_in_flight"] = [in_flight(2, 2 * max(args.steps // 2, 4)), in_flight(4, 4 * max(args.steps // 4, 2))]
        # the iterative method on the same workload: default parameters (30 sweeps enqueued, converged images skip)
        # and with the sweep count set to what the slowest image needed
        pj = tc.params_for(w, eig_method=tc.TC_EIG_JACOBI, stream_groups=args.groups)
        oj = outputs(pj)
        wj = tc.new_workspace(pj)
        msj, hostj = timed_steps(pj, oj, wj, max(args.steps // 4, 3), 1)
        sweeps = oj[3].cpu().numpy()
        jac = {"ms_per_step_default_params": round(msj, 3), "host_enqueue_ms_default_params": round(hostj, 3),
               "sweeps_used_min_max": [int(sweeps.min()), int(sweeps.max())]}
        if (sweeps > 0).all():
            pj.jacobi_max_sweeps = int(sweeps.max())
            msc, hostc = timed_steps(pj, oj, wj, max(args.steps // 4, 3), 1)
            jac.update({"ms_per_step_calibrated_sweeps": round(msc, 3), "host_enqueue_ms_calibrated": round(hostc, 3)})
        out["jacobi_method"] = jac
        del wj
        next_rows(args, tc, torch, w, p, batch, dev, sd, Q, K, V, X, X_out, kept, dst, info, ws, out)

    if not args.no_cpu_baseline:
        from oracle import tokencarve_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count() or 1
        n = min(args.cpu_sample, B)
        t0 = time.perf_counter()
        for i in range(n):
            orc.compress(batch["Q"][i], batch["K"][i], batch["V"][i], batch["X"][i, w.n_sys:w.n_sys + w.n_vis],
                         w.n_sys, w.n_vis, w.k_prune, w.k_final, lam=w.lam, causal=bool(w.causal), dtype=w.dtype)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(n / cpu_s, 3), "unit": "images/s", "cores": int(cores),
                               "kind": "oracle",
                               "sample": "first %d images of the same batch, float64 numpy oracle, one image at a "
                                         "time with BLAS/LAPACK threads" % n}
    print(json.dumps(out))


def next_rows(args, tc, torch, w, p, batch, dev, sd, Q, K, V, X, X_out, kept, dst, info, ws, out):
    """The entry points beyond the compression path, timed with events on the launch stream."""
    B, N = w.batch, w.n_vis

    def timed(fn, reps=5):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    O_all = torch.empty(B, N, w.n_heads * w.head_dim, dtype=sd, device="cuda")
    tc.tc_compress(p, Q, K, V, X, X_out, kept, dst, ws, O=O_all, info=info)
    rank = torch.empty(B, dtype=torch.int32, device="cuda")
    ms_rank_all = timed(lambda: tc.tc_info_rank(p, O_all, rank, ws, rtol=0.02))
    ms_rank_kept = timed(lambda: tc.tc_info_rank(p, O_all, rank, ws, rows=kept, rtol=0.02))
    L = w.n_sys + w.n_vis + w.n_prompt
    Ln = L - N + w.k_final
    Hfull = dev(batch["X"])
    H_new = torch.empty(B, Ln, w.hidden, dtype=sd, device="cuda")
    pos = torch.empty(B, Ln, dtype=torch.int32, device="cuda")
    rc_t = torch.empty(B, Ln, w.head_dim // 2, dtype=torch.float32, device="cuda")
    rs_t = torch.empty_like(rc_t)
    ms_asm = timed(lambda: tc.tc_assemble_sequence(p, Hfull, X_out, kept, H_new, pos, 10000.0, rc_t, rs_t), reps=20)
    asm_bytes = 2 * B * Ln * w.hidden * Hfull.element_size() + 2 * rc_t.numel() * 4 + pos.numel() * 4
    out["next_rows"] = {
        "info_rank_all_rows_ms": round(ms_rank_all, 3), "info_rank_kept_rows_ms": round(ms_rank_kept, 3),
        "assemble_sequence_ms": round(ms_asm, 4),
        "assemble_sequence_roofline": {"bound": "hbm", "achieved": round(asm_bytes / (ms_asm * 1e-3) / 1e9, 1),
                                       "peak": 8000.0, "unit": "GB/s",
                                       "frac": round(asm_bytes / (ms_asm * 1e-3) / 1e9 / 8000.0, 4)},
        "kv_cache_share": round(tc.tc_kv_cache_fraction(w.n_sys + w.n_prompt, N, w.k_final, 32, 2), 4),
    }


if __name__ == "__main__":
    main()
