#!/usr/bin/env python3
"""Benchmark of the TokenCarve compression path on one MI355X.

One step = one tc_compress call (attention output -> IPGS score -> prune -> merge) over one batch of
synthetic LLaVA-1.5-7B-shaped inputs (batch 64, 576 visual + 64 text tokens, D = 4096, bf16,
576 -> 128 -> 64 tokens), inputs resident in HBM.  Prints ONE JSON line.

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

PEAK_FP64_MFMA_TFLOPS = 78.6   # MI355X dense fp64 matrix-core peak
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_FP64_VECTOR_TFLOPS = 78.6  # 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz
PEAK_FP32_VECTOR_TFLOPS = 157.3
FULL_EVERY = 6                   # one rotation launch in six sweeps all 64 indices of its pair (csrc/jacobi.hip)


def jacobi_solve_flops_per_image_sweep(n_vis):
    """Algorithmic flops of the rotation kernel for one image and sweep.

    One step of a pair's 64x64 subproblem applies 32 disjoint plane rotations from both sides to the
    symmetric S (528 2x2 blocks of its upper triangle, 4 results of 2 x 3 flops each) and from the right
    to the accumulated R (4096 entries, 3 flops each).  A launch runs 32 such steps (63 at every
    FULL_EVERY-th step of a sweep); a sweep has Np/32 - 1 launches of Np/64 pairs.
    """
    np_ = (n_vis + 63) // 64 * 64
    P, steps = np_ // 64, np_ // 32 - 1
    per_step = 528 * 24 + 4096 * 3
    full = len(range(0, steps, FULL_EVERY))
    return P * per_step * (full * 63 + (steps - full) * 32)


def jacobi_update_flops_per_image_step(n_vis):
    """Algorithmic flops of one block-Jacobi tile-update step of G for one image.

    b = 32, a pair tile is 64x64.  With P pairs, symmetry leaves the P(P-1)/2 tiles I < J of G to
    this kernel, each two 64x64x64 products (R_I^T G_IJ, then times R_J); the P tiles on the block
    diagonal come back from the rotation kernel, which holds them rotated at its end.  (The float32
    eigenvector update is a separate kernel: (Np/64) x P tiles with one product each.)
    """
    np_ = (n_vis + 63) // 64 * 64
    P = np_ // 64
    gemm = 2 * 64 ** 3
    return P * (P - 1) // 2 * 2 * gemm


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llava7b_b64")
    ap.add_argument("--eig", default="f64", choices=["f64", "f32"])
    ap.add_argument("--sweeps", type=int, default=0,
                    help="eigensolver sweeps to launch; 0 = find the number the slowest image needs with one untimed run")
    ap.add_argument("--groups", type=int, default=0, help="eigensolver stream groups (0 = library default, 1 = one stream)")
    ap.add_argument("--copy-calib", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--path-only", action="store_true",
                    help="skip the timings of the entry points beyond the compression path (keeps kernel traces clean)")
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
    eig = tc.TC_EIG_F64 if args.eig == "f64" else tc.TC_EIG_F32
    p = tc.params_for(w, eig_dtype=eig, stream_groups=args.groups)
    sd = tc.storage_dtype(p)

    def dev(a):
        return torch.from_numpy(a).cuda().to(sd).contiguous()

    Q, K, V = dev(batch["Q"]), dev(batch["K"]), dev(batch["V"])
    X = dev(np.ascontiguousarray(batch["X"][:, w.n_sys:w.n_sys + w.n_vis]))
    B, N = w.batch, w.n_vis
    X_out = torch.empty(B, w.k_final, w.hidden, dtype=sd, device="cuda")
    kept = torch.empty(B, w.k_final, dtype=torch.int32, device="cuda")
    dst = torch.empty(B, N, dtype=torch.int32, device="cuda")
    info = torch.empty(B, dtype=torch.int32, device="cuda")
    ws = tc.new_workspace(p)
    if args.copy_calib:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst_c = torch.empty_like(src)
        dst_c.copy_(src)            # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst_c

    # How many eigensolver sweeps to launch.  The library default (30) enqueues launches that find every
    # image converged and return at once; here the count is fixed to what the slowest image needs,
    # found by one untimed run unless --sweeps gives it.  Convergence of every image is checked below.
    if args.sweeps > 0:
        p.jacobi_max_sweeps = args.sweeps
    tc.tc_compress(p, Q, K, V, X, X_out, kept, dst, ws, info=info)
    torch.cuda.synchronize()
    sweeps = info.cpu().numpy()
    if (sweeps <= 0).any():
        print("bench.py: eigensolver did not converge for some image: %s" % sweeps, file=sys.stderr)
        sys.exit(1)
    p.jacobi_max_sweeps = int(sweeps.max())
    kept_ref = kept.clone()

    for _ in range(args.warmup):
        tc.tc_compress(p, Q, K, V, X, X_out, kept, dst, ws, info=info)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tc.tc_compress(p, Q, K, V, X, X_out, kept, dst, ws, info=info)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    if (info.cpu().numpy() <= 0).any() or not torch.equal(kept, kept_ref):
        print("bench.py: timed runs disagree with the calibration run", file=sys.stderr)
        sys.exit(1)

    # per-kernel durations, measured live with HIP events on the launch stream
    kinds, upd_by_sweep = tc.tc_profile_compress(p, Q, K, V, X, X_out, kept, dst, info, ws)
    kinds, upd_by_sweep = tc.tc_profile_compress(p, Q, K, V, X, X_out, kept, dst, info, ws)
    upd_ms, upd_launches = kinds["jacobi_update"]
    tiles_done = kinds.pop("jacobi_update_tiles")[1]   # counted by the kernel: tiles between two converged block pairs are skipped
    rot_steps = kinds.pop("jacobi_rotation_steps")[1]  # likewise: visits of converged block pairs apply no rotations
    steps_per_sweep = (N + 63) // 64 * 2 - 1
    per_img = jacobi_update_flops_per_image_step(N)
    Pp = (N + 63) // 64
    tiles_full = 0
    for s in range(p.jacobi_max_sweeps):
        active = int((sweeps > s).sum())            # images still iterating in sweep s
        tiles_full += active * (Pp * (Pp - 1) // 2) * steps_per_sweep
    flops = tiles_done * (per_img / max(Pp * (Pp - 1) // 2, 1))
    achieved = flops / (upd_ms * 1e-3) / 1e12 if upd_launches else 0.0   # a single block pair (N <= 64) has no tile update
    peak = PEAK_FP64_MFMA_TFLOPS if args.eig == "f64" else PEAK_FP32_MFMA_TFLOPS
    # the rotation kernel: plain vector arithmetic (the float32 solver sweeps all 64 indices in every launch)
    solve_ms, solve_launches = kinds["jacobi_solve"]
    solve_flops = rot_steps * (528 * 24 + 4096 * 3)
    if args.eig == "f64":
        solve_full = jacobi_solve_flops_per_image_sweep(N)
    else:
        solve_full = ((N + 63) // 64) * (528 * 24 + 4096 * 3) * 63 * steps_per_sweep
    solve_full *= sum(int((sweeps > s).sum()) for s in range(p.jacobi_max_sweeps))
    solve_achieved = solve_flops / (solve_ms * 1e-3) / 1e12
    solve_peak = PEAK_FP64_VECTOR_TFLOPS if args.eig == "f64" else PEAK_FP32_VECTOR_TFLOPS
    total_kernel_ms = sum(v[0] for v in kinds.values())
    sustained = tc.tc_probe_rates()   # what this GPU delivers on register-only MFMA loops and a plain copy
    traffic = None   # HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary
    pmc = os.path.join(ROOT, "profiles", "jacobi_update_g.%s.pmc.txt" % w.name)
    if os.path.exists(pmc) and args.eig == "f64":
        for line in open(pmc):
            if line.startswith("hbm_bytes_per_launch:"):
                traffic = float(line.split(":")[1])

    out = {
        "metric": "images/sec compressed (576x4096 -> k_prune -> k_final tokens, batch 64)",
        "value": round(B / (ms_per_step * 1e-3), 2),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 storage; fp32-accumulate bf16 MFMA (attention, similarity); %s Gram + eigensolver" % args.eig,
        "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "n_vis": N, "n_text": w.n_sys + w.n_prompt,
                   "hidden": w.hidden, "heads": w.n_heads, "head_dim": w.head_dim,
                   "k_prune": w.k_prune, "k_final": w.k_final, "lambda": w.lam, "causal": w.causal,
                   "qkv": w.qkv_mode, "stream_groups": args.groups, "jacobi_max_sweeps": int(p.jacobi_max_sweeps),
                   "sweeps_used_min_max": [int(sweeps.min()), int(sweeps.max())],
                   "input_generation_s": round(gen_s, 1)},
        "roofline": {"kernel": "jacobi_update", "bound": "mfma", "achieved": round(achieved, 3), "peak": peak,
                     "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": traffic,
                     "avg_launch_us": round(upd_ms * 1e3 / max(upd_launches, 1), 2), "launches": upd_launches,
                     "tiles_processed": tiles_done, "tiles_without_skipping": tiles_full,
                     "frac_of_sustained_mfma": round(achieved / sustained["mfma_f64_tflops" if args.eig == "f64" else "mfma_f32_tflops"], 4)},
        "roofline_alu": {"kernel": "jacobi_solve", "bound": "alu", "achieved": round(solve_achieved, 3),
                         "peak": solve_peak, "unit": "TFLOP/s", "frac": round(solve_achieved / solve_peak, 4),
                         "avg_launch_us": round(solve_ms * 1e3 / max(solve_launches, 1), 2),
                         "launches": solve_launches, "flops_counted": solve_flops, "flops_without_skipping": solve_full},
        "sustained_rates": {k: round(v, 1) for k, v in sustained.items()},
        "kernel_ms": {k: round(v[0], 3) for k, v in kinds.items()},
        "kernel_ms_total": round(total_kernel_ms, 3),
    }

    if not args.path_only:
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
