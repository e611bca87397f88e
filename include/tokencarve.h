/*
 * tokencarve.h -- C ABI of the MI355X (gfx950) TokenCarve compression library.
 *
 * TokenCarve (arXiv 2503.10501) compresses the visual tokens of a multimodal LLM
 * between LLM layers 2 and 3 during prefill (Section 3.3): it scores every visual
 * token by its contribution to the singular spectrum of the layer-2 attention
 * output (Eq. 3-6) mixed with its attention score (Eq. 3-7, 3-8), prunes to the
 * best L_vc(1+rho) tokens (Stage I), then merges the L_vc*rho lower-scored
 * survivors that are most similar to a higher-scored one into it (Stage II,
 * Eq. 3-9, 3-10), leaving L_vc tokens.
 *
 * Conventions for every entry point
 *   - `p` is a HOST pointer.  Every other pointer is a DEVICE pointer owned by the
 *     caller, contiguous row-major, 16-byte aligned.  The library allocates no
 *     memory, frees none and keeps no pointer after the call returns.  The only
 *     state it keeps is up to three helper streams per device, created the first
 *     time a batch is split into stream groups (see tc_params.stream_groups) and
 *     kept until the process ends; their work is ordered after what is already on
 *     `stream` and `stream` waits for it before the next stage.
 *   - All scratch memory comes from `ws` (`ws_bytes` >= tc_workspace_bytes(p)).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without waiting for it.  Two calls may
 *     overlap only if they use different workspaces.
 *   - The return value is a tc_status.  Argument errors are detected on the host
 *     before anything is launched: a failing call launches nothing and writes
 *     nothing.  Data-dependent conditions (eigensolver not converged) are reported
 *     in the device array `info`, never by the return code.
 *   - Outputs are fully overwritten; inputs are never modified.
 *   - Token indices are int32, local to the image's visual tokens (0 .. n_vis-1);
 *     the sequence position of visual token x is vis_start + x.
 *   - Notation: B batch, L sequence length, L_s = vis_start, N = n_vis, H heads,
 *     d_h head_dim, D = H*d_h, k_p = k_prune = L_vc(1+rho), k_f = k_final = L_vc,
 *     |A| = k_p/2 (integer division), |B| = k_p - |A|, m = k_p - k_f <= |B|.
 */
#ifndef TOKENCARVE_H
#define TOKENCARVE_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define TC_API __attribute__((visibility("default")))
#else
#define TC_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TC_OK = 0,
  TC_ERR_NULL = -1,      /* a required pointer is NULL                               */
  TC_ERR_SHAPE = -2,     /* unsupported or inconsistent sizes                        */
  TC_ERR_DTYPE = -3,     /* dtype / eig_dtype not one of the enumerators             */
  TC_ERR_PARAM = -4,     /* lambda, k_prune, k_final, tolerances out of range        */
  TC_ERR_WORKSPACE = -5, /* ws_bytes < tc_workspace_bytes(p)                         */
  TC_ERR_ALIGN = -6,     /* a pointer is not 16-byte aligned                         */
  TC_ERR_HIP = -7,       /* a HIP launch failed (hipGetLastError was not hipSuccess) */
  TC_ERR_SCRATCH = -8    /* tc_merge_noalloc: the sizes need more than TC_NOALLOC_SCRATCH_BYTES */
} tc_status;

typedef enum { TC_F32 = 0, TC_BF16 = 1, TC_F16 = 2 } tc_dtype;  /* storage of Q,K,V,O,X,X_out (TC_F16: IEEE half) */
typedef enum { TC_NORM_NONE = 0, TC_NORM_MINMAX = 1 } tc_norm;
/* arithmetic of the Gram matrix and of the eigenvalue iteration (the eigenvectors are accumulated in
   float32 either way); TC_EIG_F32 is only accurate enough for well-conditioned spectra */
typedef enum { TC_EIG_F64 = 0, TC_EIG_F32 = 1 } tc_eig_dtype;
/* how the eigen-decomposition of the Gram matrix (the SVD of Section 3.3.1) is computed:
   TC_EIG_TRIDIAGONAL  Householder reduction to tridiagonal form, eigenvalues by bisection, eigenvectors from
                       twisted factorisations, back-transformation; float64 only, n_vis <= 1024;
   TC_EIG_JACOBI       two-sided block Jacobi iteration (any n_vis, float64 or float32);
   TC_EIG_AUTO         the tridiagonal route where it applies, else Jacobi */
typedef enum { TC_EIG_AUTO = 0, TC_EIG_JACOBI = 1, TC_EIG_TRIDIAGONAL = 2 } tc_eig_method;

typedef struct {
  int32_t batch;        /* B >= 0 (B == 0: nothing is launched, TC_OK)                         */
  int32_t seq_len;      /* L                                                                    */
  int32_t vis_start;    /* L_s ; vis_start + n_vis <= seq_len                                   */
  int32_t n_vis;        /* N, 1 .. 4096                                                         */
  int32_t n_heads;      /* H                                                                    */
  int32_t head_dim;     /* d_h in {64, 128}; D = H * d_h                                        */
  int32_t hidden_dim;   /* row width of X and X_out, a multiple of 8                            */
  int32_t dtype;        /* tc_dtype                                                             */
  int32_t causal;       /* 1: query at position p attends keys 0..p ; 0: all L keys             */
  float softmax_scale;  /* 0 => 1/sqrt(head_dim)                                                */
  float lambda;         /* Eq. 3-8 weight of the attention score, in [0,1]                      */
  int32_t norm_mode;    /* tc_norm: min-max scale C and S over the image before Eq. 3-8, or not */
  float sv_rtol;        /* Eq. 3-6 drops terms with sigma_i <= sv_rtol * sigma_max; 0 keeps all */
  int32_t k_prune;      /* k_p: 1 <= k_final <= k_prune <= n_vis, k_prune - k_final <= |B|      */
  int32_t k_final;      /* k_f                                                                  */
  int32_t jacobi_max_sweeps; /* 0 => 30 (Jacobi method only)                                    */
  float jacobi_tol;     /* an image stops after the first sweep that leaves off(G)/||G||_F < tol
                           (off = Frobenius norm of the off-diagonal part);
                           0 => 2e-9 * min(1, 576 / N) (3e-6 for TC_EIG_F32)                    */
  int32_t eig_dtype;    /* tc_eig_dtype                                                         */
  int32_t eig_method;   /* tc_eig_method; TC_EIG_TRIDIAGONAL with TC_EIG_F32 or n_vis > 1024 is rejected (TC_ERR_PARAM) */
  int32_t stream_groups; /* groups of images whose eigensolver work (tridiagonal route: attention and Gram matrix
                            too) runs on helper streams and overlaps: 0 = the library chooses (Jacobi: 1, 2 or 4 by
                            the amount of work; tridiagonal: 2 from 16 images on), 1 = everything on `stream`,
                            2..4 = that many groups.  Results do not depend on it.                      */
  int32_t n_prompt_queries; /* P, text-guided variant of Eq. 3-7: the P query rows after the visual block (positions
                            vis_start + n_vis .. + P - 1) join the visual query rows in the column mean, which
                            then runs over H * (n_vis + P) entries; 0 <= P <= seq_len - vis_start - n_vis.
                            0 = Eq. 3-7 as printed.  The attention output O is that of the visual rows either way. */
} tc_params;

/* Bytes of scratch that any entry point may need for `p` (0 if p is invalid). */
TC_API size_t tc_workspace_bytes(const tc_params* p);

/* Static text for a tc_status value. */
TC_API const char* tc_status_string(int status);

/*
 * Eq. 3-1, 3-2 restricted to the visual query rows (Section 3.2.2 slice), and Eq. 3-7.
 *   Q, K, V     [B, H, L, d_h]  dtype; rotary embedding already applied to Q and K
 *   O           [B, N, D]       dtype; O[b, x, h*d_h + e] = sum_k A[b,h,L_s+x,k] V[b,h,k,e],
 *                               A = softmax over the allowed keys of Q K^T * scale, rounded once
 *   attn_score  [B, N]          float; S[b,x] = mean over h and over visual queries q of
 *                               A[b,h,L_s+q,L_s+x] (masked entries count as 0); may be NULL
 */
TC_API int tc_attn_output(const tc_params* p, const void* Q, const void* K, const void* V, void* O,
                   float* attn_score, void* ws, size_t ws_bytes, void* stream);

/*
 * Section 3.3.1.  SVD of O[b] = U Sigma V^T is realised as the eigen-decomposition of the Gram
 * matrix O O^T = U Sigma^2 U^T (batched block-Jacobi); Eq. 3-6 then Eq. 3-8.
 *   O           [B, N, D] dtype
 *   attn_score  [B, N] float, may be NULL only when lambda == 0
 *   score       [B, N] float  E of Eq. 3-8
 *   ics         [B, N] float  C of Eq. 3-6 (before any normalisation); optional (NULL)
 *   sigma       [B, N] float  singular values, descending; optional
 *   info        [B] int32     > 0: done, < 0: failed, never 0.  Jacobi method: the number of sweeps used
 *                             (1 for an all-zero matrix, which needs none), negated if the tolerance was
 *                             not reached within jacobi_max_sweeps.  Tridiagonal method: 1, or -1 if an
 *                             eigenvector came out non-finite or two eigenvalues closer than 1e-10 of the
 *                             spectral norm could not be given independent vectors.  Optional
 */
TC_API int tc_ipgs_score(const tc_params* p, const void* O, const float* attn_score, float* score,
                  float* ics, float* sigma, int32_t* info, void* ws, size_t ws_bytes, void* stream);

/*
 * Stage I (end of Section 3.3.1) and the ordering used by Eq. 3-9.
 *   score  [B, N] float
 *   order  [B, k_prune] int32  visual indices of the k_prune best scores, score descending,
 *                              equal scores in ascending index order
 */
TC_API int tc_select_topk(const tc_params* p, const float* score, int32_t* order, void* ws,
                   size_t ws_bytes, void* stream);

/*
 * Eq. 3-10 on its own: SetA = order[0 : k_p/2], SetB = the rest (Eq. 3-9);
 *     sim[b, j, i] = <z_Bj, z_Ai> / (|z_Bj| |z_Ai|),   z = rows of `metric`, |z| >= 1e-30 enforced.
 *   metric  [B, N, D] dtype            (the attention output O)
 *   order   [B, k_prune] int32         from tc_select_topk; an entry outside [0, N) is clamped
 *   sim     [B, |B|, |A|] float        written; nothing is written when |A| = 0 (k_prune = 1)
 * tc_merge computes the same matrix into its workspace.
 */
TC_API int tc_similarity(const tc_params* p, const void* metric, const int32_t* order, float* sim, void* ws,
                         size_t ws_bytes, void* stream);

/*
 * Stage II (Section 3.3.2).  SetA = order[0 : k_p/2], SetB = the rest (Eq. 3-9); cosine
 * similarity of `metric` rows (Eq. 3-10); the m SetB tokens with the highest best-similarity are
 * averaged into their most similar SetA token (unweighted mean of the destination and all of its
 * sources); every tie goes to the lower visual index.
 *   X          [B, N, hidden_dim] dtype  rows that are averaged (hidden states of the visual tokens)
 *   metric     [B, N, D] dtype           rows that are compared (the attention output O); may alias X
 *   order      [B, k_prune] int32        from tc_select_topk; entries must be distinct, in [0, N)
 *   X_out      [B, k_final, hidden_dim]  dtype, rows in ascending visual index
 *   kept_idx   [B, k_final] int32        ascending visual indices of the rows of X_out
 *   merge_dst  [B, N] int32              -1 pruned; x if x is an output row; a if x was merged into a
 */
TC_API int tc_merge(const tc_params* p, const void* X, const void* metric, const int32_t* order,
             void* X_out, int32_t* kept_idx, int32_t* merge_dst, void* ws, size_t ws_bytes,
             void* stream);

/*
 * tc_merge for callers that cannot allocate or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as tc_merge, but
 * the scratch (row norms, similarity matrix, merge list) comes from a static device array of
 * TC_NOALLOC_SCRATCH_BYTES inside the library, which every GPU the library is used on holds from the
 * first call until the process ends.  The call allocates and frees nothing and enqueues kernels only
 * (no memset nodes).  It needs 4 B k_p + 4 B |A| |B| + 8 B max(m, 1) bytes (each term rounded up to 256) and returns
 * TC_ERR_SCRATCH, launching nothing, when that exceeds the array.  All calls on one GPU share the array:
 * calls that overlap in time on the same GPU (different streams or host threads) race; calls ordered on
 * one stream are safe.
 */
#define TC_NOALLOC_SCRATCH_BYTES (16u << 20)
TC_API int tc_merge_noalloc(const tc_params* p, const void* X, const void* metric, const int32_t* order,
                            void* X_out, int32_t* kept_idx, int32_t* merge_dst, void* stream);

/*
 * The whole path of Section 3.3 on one stream: tc_attn_output -> tc_ipgs_score ->
 * tc_select_topk -> tc_merge (metric = O).
 *   X                      [B, N, hidden_dim] dtype (visual rows of the hidden states)
 *   O_opt, score_opt, order_opt, info_opt: optional outputs ([B,N,D] dtype, [B,N] float,
 *                          [B,k_prune] int32, [B] int32); NULL keeps the intermediate in `ws` only
 */
TC_API int tc_compress(const tc_params* p, const void* Q, const void* K, const void* V, const void* X,
                void* X_out, int32_t* kept_idx, int32_t* merge_dst, void* O_opt, float* score_opt,
                int32_t* order_opt, int32_t* info_opt, void* ws, size_t ws_bytes, void* stream);

/*
 * Measurement aid (not part of the method): runs tc_compress with a pair of HIP events around every
 * kernel launch, waits for the stream, and returns on the HOST the summed duration in milliseconds
 * and the number of launches per kernel kind (arrays of TC_PROF_KINDS entries, order of tc_prof_kind).
 * jacobi_update_ms_by_sweep (host, max_sweeps_out floats, may be NULL) receives the tile-update time
 * of each eigensolver sweep; jacobi_work (host, 2 entries, may be NULL) the work the eigensolver has
 * actually done in all sweeps and images together: [0] the number of 64x64 tiles of G the tile update
 * has processed, [1] the number of rotation steps (32 plane rotations of a 64x64 subproblem each) the
 * rotation kernel has applied (towards the end the eigensolver leaves converged block pairs alone;
 * their visits and the tiles between two such pairs are not counted).  Unlike every
 * other entry point this one blocks the calling thread, creates and destroys HIP events and copies a
 * few bytes per image from the workspace to the host.
 */
typedef enum {
  TC_PROF_ATTN = 0, TC_PROF_ATTN_REDUCE, TC_PROF_GRAM, TC_PROF_JACOBI_INIT, TC_PROF_JACOBI_SOLVE,
  TC_PROF_JACOBI_UPDATE, TC_PROF_JACOBI_UPDATE_U, TC_PROF_JACOBI_SWEEP_END, TC_PROF_SIGMA, TC_PROF_ICS, TC_PROF_COMBINE, TC_PROF_TOPK,
  TC_PROF_ROWNORM, TC_PROF_SIM, TC_PROF_ASSIGN, TC_PROF_AVERAGE, TC_PROF_TRIDIAG, TC_PROF_BISECT, TC_PROF_TWISTED,
  TC_PROF_BACKTRANSFORM, TC_PROF_TRIDIAG_UPDATE, TC_PROF_KINDS
} tc_prof_kind;
TC_API int tc_profile_compress(const tc_params* p, const void* Q, const void* K, const void* V, const void* X,
                               void* X_out, int32_t* kept_idx, int32_t* merge_dst, int32_t* info, void* ws,
                               size_t ws_bytes, void* stream, float* ms_by_kind, int32_t* launches_by_kind,
                               float* jacobi_update_ms_by_sweep, int32_t max_sweeps_out,
                               int64_t* jacobi_work);

/*
 * Information quantity of a set of visual tokens (Section 3.2.2, "matrix rank as a proxy metric"; the
 * appendix "Attention Output Matrix Rank"): for every image the numerical rank of the attention
 * output rows O[b, rows[b, :], :],
 *     rank[b] = #{ i : sigma_i > rtol * sigma_max },
 * sigma = singular values of the n_rows x D matrix (D = n_heads * head_dim), obtained as the square
 * roots of the eigenvalues of its Gram matrix with the eigensolver of tc_ipgs_score (p->eig_dtype,
 * jacobi_* as there; TC_EIG_F64 recommended).
 *   O      [B, n_vis, D]  device, p->dtype, as written by tc_attn_output
 *   rows   [B, n_rows]    device int32, distinct visual indices in [0, n_vis) (e.g. kept_idx of
 *                         tc_merge); NULL = all n_vis rows (n_rows is then ignored).  An index out of
 *                         range is clamped, not reported.
 *   rtol   threshold relative to sigma_max; 0 = max(n_rows, D) * 2^-23 (numerical rank of float32
 *          data).  Values in (0, 1e-7) are rejected with TC_ERR_PARAM: the Gram route cannot resolve
 *          singular values that far below the largest one.
 *   rank   [B] device int32, written
 *   sigma  [B, n_rows] device float, optional: the singular values, descending
 *   info   [B] device int32, optional: sweeps used, negative if not converged
 *   ws     workspace of tc_workspace_bytes(p) bytes (its contents are destroyed)
 * n_rows = 0 gives rank 0.  Errors as for tc_ipgs_score; 0 <= n_rows <= n_vis else TC_ERR_SHAPE.
 */
TC_API int tc_info_rank(const tc_params* p, const void* O, const int32_t* rows, int32_t n_rows, float rtol,
                        int32_t* rank, float* sigma, int32_t* info, void* ws, size_t ws_bytes, void* stream);

/*
 * The sequence handed to the next layer after compression (Fig. 2, lower panel; Conclusion: kept
 * tokens keep their original position ids and the rotary encodings are recomputed from them):
 *     H_new[b] = [ H[b, 0 : vis_start] | X_out[b] | H[b, vis_start + n_vis : seq_len] ]
 *     pos_ids[b] = [ 0 .. vis_start-1 | vis_start + kept_idx[b, :] | vis_start + n_vis .. seq_len-1 ]
 * with L' = seq_len - n_vis + k_final rows, and optionally the rotary tables of Eq. 3-1's R(theta),
 *     rope_cos[b, j, i] = cos(pos_ids[b, j] * rope_base^(-2 i / head_dim)),  i < head_dim / 2
 * (rope_sin alike), evaluated in float64 and rounded once.
 *   H        [B, seq_len, hidden_dim]  device, p->dtype: hidden states of the full sequence
 *   X_out    [B, k_final, hidden_dim]  device, p->dtype: compressed visual rows (tc_merge / tc_compress)
 *   kept_idx [B, k_final]              device int32, ascending (tc_merge / tc_compress)
 *   H_new    [B, L', hidden_dim]       device, written; must not overlap H or X_out
 *   pos_ids  [B, L']                   device int32, written
 *   rope_cos, rope_sin [B, L', head_dim/2] device float, both given or both NULL; rope_base > 1
 *                                      (10000 for LLaMA) is only read when they are given
 * Needs no workspace.  Text rows are copied bit for bit.
 */
TC_API int tc_assemble_sequence(const tc_params* p, const void* H, const void* X_out, const int32_t* kept_idx,
                                void* H_new, int32_t* pos_ids, float rope_base, float* rope_cos, float* rope_sin,
                                void* stream);

/*
 * Host arithmetic, no GPU work: size of the KV cache relative to the uncompressed run when the
 * n_layers_before layers in front of the compression point hold the full sequence (n_text + n_vis
 * tokens) and the remaining layers n_text + n_kept tokens (the "KV Cache (%)" row of the paper's
 * latency table).  Returns -1 for arguments out of range.
 */
TC_API double tc_kv_cache_fraction(int32_t n_text, int32_t n_vis, int32_t n_kept, int32_t n_layers,
                                   int32_t n_layers_before);

/*
 * Measurement aid: sustained rates of this GPU, for reading roofline fractions against what the part
 * actually delivers.  Runs register-only loops of independent matrix-core products (fp64 16x16x4,
 * fp32 16x16x4, bf16 32x32x16) and a streaming copy of 1 GiB inside `ws` (ws_bytes >= 2 GiB,
 * contents destroyed), waits for them, and writes to the HOST array rates[5]:
 * TFLOP/s fp64 (16x16x4), TFLOP/s fp32, TFLOP/s bf16, GB/s copied (read + written), TFLOP/s fp64 with
 * the 4x4x4 four-block product.  Blocks the calling thread.
 */
TC_API int tc_probe_rates(void* ws, size_t ws_bytes, void* stream, float* rates);

#ifdef __cplusplus
}
#endif
#endif /* TOKENCARVE_H */
