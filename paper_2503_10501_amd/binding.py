"""ctypes binding of libtokencarve.so: same names as the C ABI, argument marshalling only.

Every function takes torch tensors that already live on the GPU (contiguous, the
dtype the C header states), passes their device pointers through, and returns
nothing; a non-zero tc_status raises TokenCarveError.  Work is enqueued on
torch's current stream unless `stream` (a raw hipStream_t integer) is given.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtokencarve.so")

TC_F32, TC_BF16, TC_F16 = 0, 1, 2
_DTYPES = {"f32": TC_F32, "bf16": TC_BF16, "f16": TC_F16}
TC_NORM_NONE, TC_NORM_MINMAX = 0, 1
TC_EIG_F64, TC_EIG_F32 = 0, 1
TC_EIG_AUTO, TC_EIG_JACOBI, TC_EIG_TRIDIAGONAL = 0, 1, 2

SYMBOLS = ("tc_workspace_bytes", "tc_status_string", "tc_attn_output", "tc_ipgs_score", "tc_select_topk",
           "tc_merge", "tc_merge_noalloc", "tc_similarity", "tc_compress", "tc_profile_compress", "tc_probe_rates", "tc_info_rank",
           "tc_assemble_sequence", "tc_kv_cache_fraction")
PROF_KINDS = ("attn", "attn_reduce", "gram", "jacobi_init", "jacobi_solve", "jacobi_update", "jacobi_update_u", "jacobi_sweep_end",
              "sigma", "ics", "combine", "topk", "rownorm", "sim", "assign", "average", "tridiag", "bisect", "twisted",
              "backtransform", "tridiag_update")


class TokenCarveError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("libtokencarve: %s (status %d)" % (text, status))
        self.status = status


class tc_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("vis_start", ctypes.c_int32),
        ("n_vis", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("hidden_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("lambda_", ctypes.c_float), ("norm_mode", ctypes.c_int32),
        ("sv_rtol", ctypes.c_float), ("k_prune", ctypes.c_int32), ("k_final", ctypes.c_int32),
        ("jacobi_max_sweeps", ctypes.c_int32), ("jacobi_tol", ctypes.c_float), ("eig_dtype", ctypes.c_int32),
        ("eig_method", ctypes.c_int32), ("stream_groups", ctypes.c_int32), ("n_prompt_queries", ctypes.c_int32),
    ]


def make_params(batch, seq_len, vis_start, n_vis, n_heads, head_dim, hidden_dim, dtype, k_prune, k_final,
                lam=0.5, causal=1, norm_mode=TC_NORM_MINMAX, sv_rtol=0.0, softmax_scale=0.0,
                jacobi_max_sweeps=0, jacobi_tol=0.0, eig_dtype=TC_EIG_F64, stream_groups=0, eig_method=0,
                n_prompt_queries=0):
    return tc_params(batch, seq_len, vis_start, n_vis, n_heads, head_dim, hidden_dim, dtype, causal,
                     softmax_scale, lam, norm_mode, sv_rtol, k_prune, k_final, jacobi_max_sweeps, jacobi_tol,
                     eig_dtype, eig_method, stream_groups, n_prompt_queries)


def params_for(w, batch=None, **overrides):
    """tc_params for a workloads.Workload."""
    kw = dict(batch=w.batch if batch is None else batch, seq_len=w.seq_len, vis_start=w.n_sys, n_vis=w.n_vis,
              n_heads=w.n_heads, head_dim=w.head_dim, hidden_dim=w.hidden,
              dtype=_DTYPES[w.dtype], k_prune=w.k_prune, k_final=w.k_final, lam=w.lam,
              causal=w.causal)
    kw.update(overrides)
    return make_params(**kw)


_lib = None


def load_library():
    """Load libtokencarve.so (built by `python -m paper_2503_10501_amd.build`); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s not found: build it with `python -m paper_2503_10501_amd.build` "
                          "(there is no CPU fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, pp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(tc_params)
    lib.tc_workspace_bytes.restype = sz
    lib.tc_workspace_bytes.argtypes = [pp]
    lib.tc_status_string.restype = ctypes.c_char_p
    lib.tc_status_string.argtypes = [ctypes.c_int]
    lib.tc_attn_output.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tc_ipgs_score.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tc_select_topk.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.tc_merge.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tc_merge_noalloc.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
    lib.tc_similarity.argtypes = [pp, vp, vp, vp, vp, sz, vp]
    lib.tc_compress.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tc_profile_compress.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, ctypes.c_int32, vp]
    lib.tc_probe_rates.argtypes = [vp, sz, vp, vp]
    lib.tc_info_rank.argtypes = [pp, vp, vp, ctypes.c_int32, ctypes.c_float, vp, vp, vp, vp, sz, vp]
    lib.tc_assemble_sequence.argtypes = [pp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp]
    lib.tc_kv_cache_fraction.argtypes = [ctypes.c_int32] * 5
    for name in SYMBOLS[2:]:
        getattr(lib, name).restype = ctypes.c_int
    lib.tc_kv_cache_fraction.restype = ctypes.c_double
    _lib = lib
    return lib


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous and on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream(stream):
    return torch.cuda.current_stream().cuda_stream if stream is None else stream


def _check(rc):
    if rc != 0:
        raise TokenCarveError(rc, load_library().tc_status_string(rc).decode())


def storage_dtype(p):
    return {TC_F32: torch.float32, TC_BF16: torch.bfloat16, TC_F16: torch.float16}[p.dtype]


def tc_status_string(status):
    return load_library().tc_status_string(status).decode()


def tc_workspace_bytes(p):
    return int(load_library().tc_workspace_bytes(ctypes.byref(p)))


def new_workspace(p, device="cuda"):
    n = tc_workspace_bytes(p)
    if n == 0:
        raise TokenCarveError(-4, "invalid tc_params")
    return torch.empty(n, dtype=torch.uint8, device=device)


def tc_attn_output(p, Q, K, V, O, attn_score, ws, stream=None):
    sd = storage_dtype(p)
    _check(load_library().tc_attn_output(ctypes.byref(p), _ptr(Q, sd), _ptr(K, sd), _ptr(V, sd), _ptr(O, sd),
                                         _ptr(attn_score, torch.float32), _ptr(ws), ws.numel(), _stream(stream)))


def tc_ipgs_score(p, O, attn_score, score, ics, sigma, info, ws, stream=None):
    sd = storage_dtype(p)
    _check(load_library().tc_ipgs_score(ctypes.byref(p), _ptr(O, sd), _ptr(attn_score, torch.float32),
                                        _ptr(score, torch.float32), _ptr(ics, torch.float32),
                                        _ptr(sigma, torch.float32), _ptr(info, torch.int32), _ptr(ws), ws.numel(),
                                        _stream(stream)))


def tc_select_topk(p, score, order, ws, stream=None):
    _check(load_library().tc_select_topk(ctypes.byref(p), _ptr(score, torch.float32), _ptr(order, torch.int32),
                                         _ptr(ws), ws.numel(), _stream(stream)))


def tc_merge(p, X, metric, order, X_out, kept_idx, merge_dst, ws, stream=None):
    sd = storage_dtype(p)
    _check(load_library().tc_merge(ctypes.byref(p), _ptr(X, sd), _ptr(metric, sd), _ptr(order, torch.int32),
                                   _ptr(X_out, sd), _ptr(kept_idx, torch.int32), _ptr(merge_dst, torch.int32),
                                   _ptr(ws), ws.numel(), _stream(stream)))


def tc_merge_noalloc(p, X, metric, order, X_out, kept_idx, merge_dst, stream=None):
    sd = storage_dtype(p)
    _check(load_library().tc_merge_noalloc(ctypes.byref(p), _ptr(X, sd), _ptr(metric, sd), _ptr(order, torch.int32),
                                           _ptr(X_out, sd), _ptr(kept_idx, torch.int32),
                                           _ptr(merge_dst, torch.int32), _stream(stream)))


def tc_similarity(p, metric, order, sim, ws, stream=None):
    _check(load_library().tc_similarity(ctypes.byref(p), _ptr(metric, storage_dtype(p)), _ptr(order, torch.int32),
                                        _ptr(sim, torch.float32), _ptr(ws), ws.numel(), _stream(stream)))


def tc_compress(p, Q, K, V, X, X_out, kept_idx, merge_dst, ws, O=None, score=None, order=None, info=None,
                stream=None):
    sd = storage_dtype(p)
    _check(load_library().tc_compress(ctypes.byref(p), _ptr(Q, sd), _ptr(K, sd), _ptr(V, sd), _ptr(X, sd),
                                      _ptr(X_out, sd), _ptr(kept_idx, torch.int32), _ptr(merge_dst, torch.int32),
                                      _ptr(O, sd), _ptr(score, torch.float32), _ptr(order, torch.int32),
                                      _ptr(info, torch.int32), _ptr(ws), ws.numel(), _stream(stream)))


def tc_profile_compress(p, Q, K, V, X, X_out, kept_idx, merge_dst, info, ws, max_sweeps_out=64, stream=None):
    """Returns ({kind: (total_ms, launches)}, [jacobi_update ms per sweep]); blocks until the stream is idle.
    The extra keys "jacobi_update_tiles" and "jacobi_rotation_steps" hold (0.0, count): the 64x64 tiles the
    tile update processed and the rotation steps the rotation kernel applied."""
    sd = storage_dtype(p)
    n = len(PROF_KINDS)
    ms = (ctypes.c_float * n)()
    cnt = (ctypes.c_int32 * n)()
    per_sweep = (ctypes.c_float * max_sweeps_out)()
    work = (ctypes.c_int64 * 2)()
    _check(load_library().tc_profile_compress(ctypes.byref(p), _ptr(Q, sd), _ptr(K, sd), _ptr(V, sd), _ptr(X, sd),
                                              _ptr(X_out, sd), _ptr(kept_idx, torch.int32),
                                              _ptr(merge_dst, torch.int32), _ptr(info, torch.int32), _ptr(ws),
                                              ws.numel(), _stream(stream), ms, cnt, per_sweep, max_sweeps_out,
                                              work))
    kinds = {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(PROF_KINDS)}
    kinds["jacobi_update_tiles"] = (0.0, int(work[0]))
    kinds["jacobi_rotation_steps"] = (0.0, int(work[1]))
    return kinds, [float(x) for x in per_sweep]


def tc_probe_rates(stream=None):
    """Sustained {fp64, fp32, bf16} matrix-core TFLOP/s and streaming-copy GB/s of the current GPU."""
    ws = torch.empty(1 << 31, dtype=torch.uint8, device="cuda")
    rates = (ctypes.c_float * 5)()
    _check(load_library().tc_probe_rates(_ptr(ws), ws.numel(), _stream(stream), rates))
    return {"mfma_f64_tflops": float(rates[0]), "mfma_f32_tflops": float(rates[1]),
            "mfma_bf16_tflops": float(rates[2]), "copy_gbps": float(rates[3]),
            "mfma_f64_4x4x4_tflops": float(rates[4])}


def tc_info_rank(p, O, rank, ws, rows=None, rtol=0.0, sigma=None, info=None, stream=None):
    n_rows = int(rows.shape[1]) if rows is not None else int(p.n_vis)
    if rows is not None and rows.numel() == 0:   # an empty tensor has no address; NULL would mean "all rows"
        rows = torch.zeros(4, dtype=torch.int32, device="cuda")
    _check(load_library().tc_info_rank(ctypes.byref(p), _ptr(O), _ptr(rows, torch.int32), n_rows, float(rtol),
                                       _ptr(rank, torch.int32), _ptr(sigma, torch.float32), _ptr(info, torch.int32),
                                       _ptr(ws), ws.numel(), _stream(stream)))


def tc_assemble_sequence(p, H, X_out, kept_idx, H_new, pos_ids, rope_base=10000.0, rope_cos=None, rope_sin=None,
                         stream=None):
    _check(load_library().tc_assemble_sequence(ctypes.byref(p), _ptr(H), _ptr(X_out), _ptr(kept_idx, torch.int32),
                                               _ptr(H_new), _ptr(pos_ids, torch.int32), float(rope_base),
                                               _ptr(rope_cos, torch.float32), _ptr(rope_sin, torch.float32),
                                               _stream(stream)))


def tc_kv_cache_fraction(n_text, n_vis, n_kept, n_layers, n_layers_before):
    return float(load_library().tc_kv_cache_fraction(n_text, n_vis, n_kept, n_layers, n_layers_before))
