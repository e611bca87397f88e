"""Seeded generators for hidden states and layer-2 Q, K, V.

Every array returned here is float32 whose values are already representable in
the workload's storage type (bf16 values are float32 with the low 16 mantissa
bits zero), so the CPU oracle and the GPU path consume identical numbers.
Random numbers come from numpy's counter-based Philox generator; image `b` of
config `c` uses seed 10_000*c + b, the projection weights of a config use seed
10_000*c + 9_999.
"""
import numpy as np


def _rng(seed):
    return np.random.Generator(np.random.Philox(int(seed)))


def round_to_storage(a, dtype):
    """Round a float array to the storage type and return it as float32.

    "f32": plain cast.  "bf16": round-to-nearest-even on the upper 16 bits of
    the float32 pattern.  "f16": IEEE half, round-to-nearest-even (storage-format
    conversions, not part of the method).
    """
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a32
    if dtype == "f16":
        return np.asarray(a, dtype=np.float64).astype(np.float16).astype(np.float32)
    if dtype != "bf16":
        raise ValueError(dtype)
    u = a32.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(a32.shape)


def _orthonormal(rng, rows, cols):
    q, _ = np.linalg.qr(rng.standard_normal((rows, cols)))
    return q


def spectrum(kind, rank, n_rows, n_cols):
    """Planted singular values s_1 >= ... >= s_rank."""
    if kind == "linspace":
        return np.linspace(10.0, 1.0, rank)
    if kind == "powerlaw":
        s = np.arange(1, rank + 1, dtype=np.float64) ** -0.8
        # unit-RMS signal: sum s_i^2 = n_rows * n_cols
        return s * np.sqrt(n_rows * n_cols / np.sum(s * s))
    raise ValueError(kind)


def planted_lowrank(rng, n_rows, n_cols, s, noise):
    """U_r diag(s) V_r^T + noise * N(0,1) with orthonormal U_r, V_r (float64)."""
    r = len(s)
    u = _orthonormal(rng, n_rows, r)
    v = _orthonormal(rng, n_cols, r)
    m = (u * s) @ v.T
    if noise:
        m = m + noise * rng.standard_normal((n_rows, n_cols))
    return m


def projection_weights(w):
    """W_q, W_k, W_v ~ N(0, 1/D), float32, one set per config."""
    rng = _rng(w.seed(9_999))
    d = w.hidden
    return [(rng.standard_normal((d, d), dtype=np.float32) / np.float32(np.sqrt(d))) for _ in range(3)]


def make_image(w, image, weights=None):
    """One image's inputs.

    Returns a dict of float32 arrays already rounded to w.dtype:
      X   [L, D]        hidden states of the whole sequence
      Q,K,V [H, L, d_h] layer-2 query/key/value (rotary embedding already applied)
    """
    rng = _rng(w.seed(image))
    L, D, H, dh = w.seq_len, w.hidden, w.n_heads, w.head_dim
    x = rng.standard_normal((L, D))
    s = spectrum(w.spectrum, w.rank, w.n_vis, D)
    x[w.n_sys:w.n_sys + w.n_vis] = planted_lowrank(rng, w.n_vis, D, s, w.noise)
    x = round_to_storage(x, w.dtype)
    if w.qkv_mode == "iid":
        q, k, v = (rng.standard_normal((H, L, dh)) for _ in range(3))
    elif w.qkv_mode == "proj":
        if weights is None:
            weights = projection_weights(w)
        q, k, v = ((x @ wm).reshape(L, H, dh).transpose(1, 0, 2) for wm in weights)
    else:
        raise ValueError(w.qkv_mode)
    return {
        "X": x,
        "Q": round_to_storage(q, w.dtype),
        "K": round_to_storage(k, w.dtype),
        "V": round_to_storage(v, w.dtype),
    }


def make_batch(w, images=None):
    """Stack `images` (default: range(w.batch)) into [B, ...] arrays."""
    if images is None:
        images = range(w.batch)
    weights = projection_weights(w) if w.qkv_mode == "proj" else None
    items = [make_image(w, b, weights) for b in images]
    return {k: np.stack([it[k] for it in items]) for k in ("X", "Q", "K", "V")}
