"""Float64 CPU oracle for the TokenCarve compression path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and the cpu_baseline leg of bench.py may
import this file.  It shares no code with the HIP library and never imports it.
Everything is numpy float64, one image at a time, written in the order and
notation of the paper (Section 3.1 Eq. 3-1/3-2; Section 3.3.1 Eq. 3-5..3-8;
Section 3.3.2 Eq. 3-9/3-10 and the merge paragraph after it).  No blocking,
fusion or re-ordering: each function is the definition or the algorithm step.

Library primitives used as steps: numpy matmul, numpy.linalg.svd (the paper's
own step "apply Singular Value Decomposition"), numpy stable argsort.

Readings taken where the paper is silent (each mirrored by the HIP path):
  * Eq. 3-1 carries no mask but the LLM is autoregressive: `causal` flag,
    query at sequence position p sees keys 0..p.  Q and K arrive with the rotary
    embedding already applied.
  * A^2 in Eq. 3-7 is the visual-by-visual block of the full-sequence softmax
    (system-token keys take part in the softmax, no re-normalisation); the mean
    runs over all H*L_v*L_v entries of that block, masked zeros included.
  * d in Section 3.3.1 is the concatenation of heads, before any output
    projection: Z = A V.
  * r in Eq. 3-6: every singular value is summed (zero ones add nothing);
    `sv_rtol` optionally drops sigma_i <= sv_rtol * sigma_max.
  * C and S live on very different scales; `norm` = "minmax" rescales each to
    [0,1] over the image's visual tokens with the only normalisation the paper
    writes (Eq. 3-3); "none" is Eq. 3-8 taken literally.
  * "IndexSort" in Eq. 3-9 sorts the IPGS score E, descending; every tie
    (sort, argmax, top-m) goes to the lower original visual index.
  * Eq. 3-10: Norm = per-row L2 normalisation (cosine similarity) of Z.
  * Merge: unweighted mean of a Set-A token and all Set-B tokens sent to it
    (ToMe's average with unit sizes); similarity is measured on Z, the
    averaging acts on the rows handed in as X; output rows in ascending
    original position.

Beyond the compression path (Section 3.2 and the Conclusion):
  * Information quantity = matrix rank of the attention output of the visual
    tokens (Section 3.2.2): the number of singular values above rtol * sigma_max.
    The paper names no tolerance: the default is max(rows, cols) * 2^-23, the
    usual numerical-rank threshold for float32 data; callers may pass their own.
    The curve "rank versus kept tokens" is normalised with Eq. 3-3 (minmax()).
    The paper evaluates it on the last layer's Z after running the compressed
    sequence through the model; with no model here it is evaluated on the rows
    of the given Z that survive (kept_idx), which is the same quantity at the
    layer where compression happens.
  * Sequence after compression: [system | kept visual | prompt], every token
    keeps its original position id (Conclusion: rotary encodings are recomputed
    from the original position ids).  Rotary tables follow the standard
    definition theta_i = base^(-2i/d_h), angle = position * theta_i.
  * KV cache share (CUDA Time Test table): layers in front of the compression
    point keep the full sequence, the others the shortened one.

PARITY UNPINNED: when two singular values coincide, U is not unique inside
that subspace and Eq. 3-6 depends on the basis chosen; there only the
invariants (sum_i (u_xi sigma_i)^2 = ||Z_x||^2, bounds on C) are pinned.
"""
import numpy as np

NORM_NONE = 0
NORM_MINMAX = 1


# ----------------------------------------------------------------------------
# storage rounding (stage boundary: Z is stored in the workload's dtype)
# ----------------------------------------------------------------------------
def to_storage(a, dtype):
    """Round float64 values to the nearest bf16 / IEEE half / float32 value (ties to even); returns float64."""
    a = np.asarray(a, dtype=np.float64)
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float64)
    if dtype != "bf16":
        raise ValueError(dtype)
    # bf16 has 8 significand bits: round x to a multiple of 2^(e-7), e = floor(log2|x|).
    out = np.zeros_like(a)
    nz = a != 0
    m, e = np.frexp(a[nz])            # a = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0    # 8 significant bits; numpy rint is ties-to-even
    out[nz] = np.ldexp(q, e)
    return out


# ----------------------------------------------------------------------------
# Eq. 3-1, 3-2, 3-7: attention output and attention score of the visual tokens
# ----------------------------------------------------------------------------
def attn_output(Q, K, V, n_sys, n_vis, causal=True, scale=None, n_prompt_q=0):
    """Q, K, V: [H, L, d_h].  Returns Z_visual [N, H*d_h] and S [N] (float64).

    Eq. 3-1: A = softmax(Q K^T / sqrt(d_k)) row-wise over the allowed keys.
    Eq. 3-2: Z = A V; its rows L_s .. L_s+L_v are Z_visual (Section 3.2.2).
    Eq. 3-7: S(x) = mean over heads and visual queries of A[:, :, x].
    Text-guided variant of Eq. 3-7 (not in the paper, which keeps A^2 visual-by-visual): with
    n_prompt_q = P > 0 the mean also runs over the P query rows that follow the visual block (the
    first P prompt tokens), i.e. over the H * (L_v + P) entries of column x; P = 0 is Eq. 3-7.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    H, L, dh = Q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(dh)
    if n_prompt_q < 0 or n_sys + n_vis + n_prompt_q > L:
        raise ValueError("n_prompt_q rows must lie inside the sequence, after the visual block")
    rows = np.arange(n_sys, n_sys + n_vis + n_prompt_q)        # visual queries, then the prompt queries
    Z = np.zeros((n_vis, H * dh))
    S = np.zeros(n_vis)
    for h in range(H):
        logits = (Q[h, rows] @ K[h].T) * scale                 # [N + P, L]
        if causal:
            allowed = np.arange(L)[None, :] <= rows[:, None]
            logits = np.where(allowed, logits, -np.inf)
        logits = logits - logits.max(axis=1, keepdims=True)
        A = np.exp(logits)
        A = A / A.sum(axis=1, keepdims=True)
        Z[:, h * dh:(h + 1) * dh] = A[:n_vis] @ V[h]
        S += A[:, n_sys:n_sys + n_vis].sum(axis=0)
    S /= H * (n_vis + n_prompt_q)
    return Z, S


# ----------------------------------------------------------------------------
# Section 3.3.1: SVD, Eq. 3-6 information contribution score, Eq. 3-8
# ----------------------------------------------------------------------------
def left_svd(O):
    """Z_visual = U Sigma V^T.  Returns U [N, min(N,d)] and sigma (descending)."""
    U, s, _ = np.linalg.svd(np.asarray(O, dtype=np.float64), full_matrices=False)
    return U, s


def ics(O, sv_rtol=0.0):
    """Eq. 3-6: C(x) = sum_i |u_xi sigma_i|.  Returns C [N], sigma, U."""
    U, s = left_svd(O)
    keep = s > sv_rtol * s[0] if sv_rtol > 0 else np.ones_like(s, dtype=bool)
    C = (np.abs(U[:, keep]) * s[keep]).sum(axis=1)
    return C, s, U


def minmax(v):
    """Eq. 3-3 applied to a score vector; a constant vector maps to zeros."""
    lo, hi = v.min(), v.max()
    if hi == lo:
        return np.zeros_like(v)
    return (v - lo) / (hi - lo)


def combined_score(C, S, lam, norm=NORM_MINMAX):
    """Eq. 3-8: E = (1 - lambda) C + lambda S (each min-max scaled when norm == NORM_MINMAX)."""
    if norm == NORM_MINMAX:
        C, S = minmax(C), minmax(S)
    return (1.0 - lam) * C + lam * S


def ipgs_score(O, S, lam, norm=NORM_MINMAX, sv_rtol=0.0):
    """Returns E, C, sigma for one image's stored attention output O [N, d]."""
    C, s, _ = ics(O, sv_rtol)
    if S is None:
        S = np.zeros_like(C)
    return combined_score(C, S, lam, norm), C, s


# ----------------------------------------------------------------------------
# Stage I prune, Eq. 3-9 split
# ----------------------------------------------------------------------------
def select_topk(E, k_prune):
    """Indices of the k_prune highest scores, score descending, ties to the lower index."""
    order = np.argsort(-np.asarray(E, dtype=np.float64), kind="stable")
    return order[:k_prune].astype(np.int64)


def split_sets(order):
    """Eq. 3-9: SetA = first half of the score-ordered survivors, SetB = the rest."""
    half = len(order) // 2
    return order[:half], order[half:]


# ----------------------------------------------------------------------------
# Eq. 3-10 and the merge
# ----------------------------------------------------------------------------
def similarity(metric, set_a, set_b):
    """Eq. 3-10: Simi_AB[j, i] = <z_Bj/|z_Bj|, z_Ai/|z_Ai|>."""
    Zm = np.asarray(metric, dtype=np.float64)
    nrm = np.maximum(np.linalg.norm(Zm, axis=1, keepdims=True), 1e-30)
    Zn = Zm / nrm
    return Zn[set_b] @ Zn[set_a].T


def merge(X, metric, order, k_final, out_dtype=None):
    """Stage II.  X [N, hidden] rows to be averaged, metric [N, d] rows compared (Z).

    Returns dict with
      X_out    [k_final, hidden]  (float64; rounded to out_dtype when given)
      kept_idx [k_final]          ascending original visual indices of the output rows
      merge_dst[N]                -1 pruned, x kept as itself, a when x was merged into a
      val, best, merged           per Set-B diagnostics used by the tie rules of the tests
    """
    X = np.asarray(X, dtype=np.float64)
    n = X.shape[0]
    order = np.asarray(order, dtype=np.int64)
    k_prune = len(order)
    m = k_prune - k_final
    set_a, set_b = split_sets(order)
    if not (0 <= m <= len(set_b)):
        raise ValueError("k_prune - k_final must lie in [0, |SetB|]")
    merge_dst = np.full(n, -1, dtype=np.int64)
    merge_dst[order] = order
    best = np.zeros(len(set_b), dtype=np.int64)
    val = np.zeros(len(set_b))
    if len(set_a) and len(set_b):
        sim = similarity(metric, set_a, set_b)
        for j in range(len(set_b)):
            top = sim[j].max()
            cands = set_a[sim[j] == top]
            best[j] = cands.min()               # tie: lower original index
            val[j] = top
    # the m Set-B tokens with the highest similarity; ties to the lower original index
    rank = sorted(range(len(set_b)), key=lambda j: (-val[j], set_b[j]))
    merged = np.array(sorted(rank[:m]), dtype=np.int64)
    for j in merged:
        merge_dst[set_b[j]] = best[j]
    kept_idx, X_out = average_rows(X, merge_dst, out_dtype)
    return {"X_out": X_out, "kept_idx": kept_idx, "merge_dst": merge_dst,
            "val": val, "best": best, "merged": merged, "set_a": set_a, "set_b": set_b}


def average_rows(X, merge_dst, out_dtype=None):
    """The averaging step of the merge for a given assignment: merge_dst[x] = -1 (pruned), x (output
    row) or a (x is averaged into output row a).  Output row a is the unweighted mean of X[a] and of
    every row sent to it; rows come out in ascending original position.  Returns (kept_idx, X_out)."""
    X = np.asarray(X, dtype=np.float64)
    merge_dst = np.asarray(merge_dst, dtype=np.int64)
    kept_idx = np.nonzero(merge_dst == np.arange(len(merge_dst)))[0].astype(np.int64)
    X_out = np.zeros((len(kept_idx), X.shape[1]))
    for r, a in enumerate(kept_idx):
        members = np.nonzero(merge_dst == a)[0]   # a itself and everything merged into it
        X_out[r] = X[members].sum(axis=0) / len(members)
    if out_dtype is not None:
        X_out = to_storage(X_out, out_dtype)
    return kept_idx, X_out


# ----------------------------------------------------------------------------
# whole path for one image
# ----------------------------------------------------------------------------
def compress(Q, K, V, X_vis, n_sys, n_vis, k_prune, k_final, lam=0.5, norm=NORM_MINMAX,
             causal=True, dtype="bf16", sv_rtol=0.0, scale=None, n_prompt_q=0):
    """attention output -> stored O -> IPGS score -> prune -> merge, for one image."""
    Z, S = attn_output(Q, K, V, n_sys, n_vis, causal, scale, n_prompt_q)
    O = to_storage(Z, dtype)
    E, C, sigma = ipgs_score(O, S, lam, norm, sv_rtol)
    order = select_topk(E, k_prune)
    out = merge(X_vis, O, order, k_final, out_dtype=dtype)
    out.update({"O": O, "S": S, "C": C, "E": E, "sigma": sigma, "order": order})
    return out


# ----------------------------------------------------------------------------
# diagnostics (conditioning of Eq. 3-6; not part of the method)
# ----------------------------------------------------------------------------
def min_relative_gap(sigma, floor=1e-6):
    """min_i (sigma_i - sigma_{i+1}) / sigma_1 over sigma_i > floor * sigma_1."""
    s = np.asarray(sigma)
    s = s[s > floor * s[0]]
    if len(s) < 2:
        return np.inf
    return float(np.min(s[:-1] - s[1:]) / s[0])


def gram_precision_floor(O, gram_dtype=np.float32):
    """Largest relative change of C(x) when the Gram matrix O O^T is rounded to
    `gram_dtype` before an otherwise float64 eigen-decomposition: how much of a
    mismatch is conditioning of Eq. 3-6 rather than arithmetic error."""
    O = np.asarray(O, dtype=np.float64)
    C_ref, _, _ = ics(O)
    G = (O @ O.T).astype(gram_dtype).astype(np.float64)
    lam, U = np.linalg.eigh(G)
    C = (np.abs(U) * np.sqrt(np.maximum(lam, 0.0))).sum(axis=1)
    return float(np.max(np.abs(C - C_ref) / C_ref))


# ----------------------------------------------------------------------------
# Information quantity (Section 3.2.2, "Attention Output Matrix Rank")
# ----------------------------------------------------------------------------
def info_rank(O, rows=None, rtol=None):
    """Numerical rank of the rows `rows` (all if None) of O [N, D]; returns (rank, sigma descending)."""
    A = np.asarray(O, dtype=np.float64)
    if rows is not None:
        A = A[np.asarray(rows, dtype=np.int64)]
    if A.shape[0] == 0:
        return 0, np.zeros(0)
    sigma = np.linalg.svd(A, compute_uv=False)
    if rtol is None:
        rtol = max(A.shape) * 2.0 ** -23
    if sigma[0] <= 0.0:
        return 0, sigma
    return int(np.count_nonzero(sigma > rtol * sigma[0])), sigma


def visual_token_information(ranks):
    """The rank curve of Section 3.2.2, normalised with Eq. 3-3."""
    return minmax(np.asarray(ranks, dtype=np.float64))


# ----------------------------------------------------------------------------
# Sequence after compression (Fig. 2; Conclusion on position ids)
# ----------------------------------------------------------------------------
def assemble_sequence(H, X_out, kept_idx, n_sys, n_vis):
    """H [L, D] hidden states of the full sequence, X_out [k_f, D] compressed visual rows.

    Returns (H_new [L - n_vis + k_f, D], pos_ids): system rows, compressed visual rows, prompt
    rows, each with the position it had in the full sequence.
    """
    H = np.asarray(H, dtype=np.float64)
    kept_idx = np.asarray(kept_idx, dtype=np.int64)
    L = H.shape[0]
    H_new = np.concatenate([H[:n_sys], np.asarray(X_out, dtype=np.float64), H[n_sys + n_vis:]], axis=0)
    pos = np.concatenate([np.arange(n_sys), n_sys + kept_idx, np.arange(n_sys + n_vis, L)])
    return H_new, pos.astype(np.int64)


def rope_tables(pos_ids, head_dim, base=10000.0):
    """cos and sin [len(pos_ids), head_dim/2] of the rotary embedding R(theta) of Eq. 3-1."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    theta = base ** (-2.0 * i / head_dim)
    ang = np.asarray(pos_ids, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang), np.sin(ang)


def apply_rope(x, cos, sin):
    """Rotate x [n, head_dim] pairwise (x_i, x_{i+d/2}), the LLaMA layout."""
    x = np.asarray(x, dtype=np.float64)
    h = x.shape[1] // 2
    a, b = x[:, :h], x[:, h:]
    return np.concatenate([a * cos - b * sin, a * sin + b * cos], axis=1)


def kv_cache_fraction(n_text, n_vis, n_kept, n_layers, n_layers_before):
    """KV-cache size relative to the uncompressed run (CUDA Time Test table)."""
    full = n_text + n_vis
    short = n_text + n_kept
    return (n_layers_before * full + (n_layers - n_layers_before) * short) / (n_layers * full)
