"""Independent CPU helpers used to pin the oracle (nothing here is imported by oracle/)."""
import itertools
import math

import numpy as np


def hestenes_svd(M, tol=1e-15, max_sweeps=60):
    """One-sided Jacobi (Hestenes) on the rows of M: returns U, sigma with M = U diag(sigma) W^T.

    A second, independent route to the left singular vectors: plane rotations
    are applied to pairs of rows until all rows are mutually orthogonal; the row
    norms are then the singular values and the accumulated rotations give U.
    """
    A = np.array(M, dtype=np.float64)
    n = A.shape[0]
    J = np.eye(n)
    for _ in range(max_sweeps):
        rotated = False
        for p in range(n - 1):
            for q in range(p + 1, n):
                a = A[p] @ A[p]
                b = A[q] @ A[q]
                g = A[p] @ A[q]
                if abs(g) <= tol * math.sqrt(a * b) or g == 0.0:
                    continue
                rotated = True
                zeta = (b - a) / (2.0 * g)
                t = math.copysign(1.0, zeta) / (abs(zeta) + math.sqrt(1.0 + zeta * zeta))
                c = 1.0 / math.sqrt(1.0 + t * t)
                s = c * t
                Ap, Aq = A[p].copy(), A[q].copy()
                A[p], A[q] = c * Ap - s * Aq, s * Ap + c * Aq
                Jp, Jq = J[p].copy(), J[q].copy()
                J[p], J[q] = c * Jp - s * Jq, s * Jp + c * Jq
        if not rotated:
            break
    sigma = np.linalg.norm(A, axis=1)
    order = np.argsort(-sigma, kind="stable")
    return J.T[:, order], sigma[order]          # J M = diag(sigma) W^T  =>  M = J^T diag(sigma) W^T


def softmax_attention_loops(Q, K, V, n_sys, n_vis, causal, scale, n_prompt_q=0):
    """Eq. 3-1/3-2/3-7 with scalar Python loops (tiny sizes only); n_prompt_q more query rows after the
    visual block enter the column means (they produce no row of Z)."""
    H, L, dh = Q.shape
    Z = np.zeros((n_vis, H * dh))
    S = np.zeros(n_vis)
    for h in range(H):
        for q in range(n_vis + n_prompt_q):
            p = n_sys + q
            last = p if causal else L - 1
            logit = [sum(float(Q[h, p, e]) * float(K[h, k, e]) for e in range(dh)) * scale
                     for k in range(last + 1)]
            mx = max(logit)
            w = [math.exp(v - mx) for v in logit]
            tot = sum(w)
            for k, wk in enumerate(w):
                a = wk / tot
                if q < n_vis:
                    for e in range(dh):
                        Z[q, h * dh + e] += a * float(V[h, k, e])
                if n_sys <= k < n_sys + n_vis:
                    S[k - n_sys] += a
    return Z, S / (H * (n_vis + n_prompt_q))


def best_subset_by_sum(E, k):
    """Brute force: the size-k subset with the largest score sum."""
    best, best_set = -math.inf, None
    for comb in itertools.combinations(range(len(E)), k):
        tot = sum(E[i] for i in comb)
        if tot > best:
            best, best_set = tot, comb
    return set(best_set)


def rank_by_elimination(A, tol=1e-9):
    """Rank of a small matrix by Gaussian elimination with full pivoting (independent of any SVD)."""
    M = np.array(A, dtype=np.float64)
    scale = np.abs(M).max() if M.size else 0.0
    if scale == 0.0:
        return 0
    rank = 0
    rows, cols = M.shape
    for _ in range(min(rows, cols)):
        sub = np.abs(M[rank:, rank:])
        i, j = np.unravel_index(np.argmax(sub), sub.shape)
        if sub[i, j] <= tol * scale:
            break
        M[[rank, rank + i]] = M[[rank + i, rank]]
        M[:, [rank, rank + j]] = M[:, [rank + j, rank]]
        M[rank + 1:, rank:] -= np.outer(M[rank + 1:, rank] / M[rank, rank], M[rank, rank:])
        rank += 1
    return rank
