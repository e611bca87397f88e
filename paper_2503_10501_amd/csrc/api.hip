// C ABI entry points of libtokencarve: argument checks, workspace carving, stage sequencing.
// The operations are defined in include/tokencarve.h (Section 3.3 of the TokenCarve paper).
#include <cmath>

#include "tc_internal.h"

namespace tc {

int make_plan(const tc_params* p, Plan* pl) {
  if (!p) return TC_ERR_NULL;
  if (p->dtype != TC_F32 && p->dtype != TC_BF16 && p->dtype != TC_F16) return TC_ERR_DTYPE;
  if (p->eig_dtype != TC_EIG_F64 && p->eig_dtype != TC_EIG_F32) return TC_ERR_DTYPE;
  if (p->batch < 0 || p->seq_len < 1 || p->vis_start < 0 || p->n_vis < 1 || p->n_vis > MAX_NVIS ||
      (int64_t)p->vis_start + p->n_vis > p->seq_len || p->n_heads < 1 || p->n_heads > 1024 ||
      (p->head_dim != 64 && p->head_dim != 128) || p->hidden_dim < 8 || (p->hidden_dim % 8) != 0 ||
      p->hidden_dim > (1 << 20) || p->seq_len > (1 << 20) || p->batch > (1 << 16))
    return TC_ERR_SHAPE;
  if (!(p->lambda >= 0.f && p->lambda <= 1.f) || (p->norm_mode != TC_NORM_NONE && p->norm_mode != TC_NORM_MINMAX) ||
      !(p->sv_rtol >= 0.f && p->sv_rtol < 1.f) || (p->causal != 0 && p->causal != 1) || !(p->softmax_scale >= 0.f) ||
      !std::isfinite(p->softmax_scale) || p->jacobi_max_sweeps < 0 || p->jacobi_max_sweeps > 1000 ||
      !(p->jacobi_tol >= 0.f) || !(p->jacobi_tol < 1.f) || p->stream_groups < 0 || p->stream_groups > 4 ||
      p->eig_method < TC_EIG_AUTO || p->eig_method > TC_EIG_TRIDIAGONAL || p->n_prompt_queries < 0 ||
      (int64_t)p->vis_start + p->n_vis + p->n_prompt_queries > p->seq_len)
    return TC_ERR_PARAM;
  // the tridiagonal route works in float64 and keeps its panels in the LDS of one compute unit
  const bool direct_ok = p->eig_dtype == TC_EIG_F64 && p->n_vis <= 1024 && tridiag_panel_width(p->n_vis) >= 4;
  if (p->eig_method == TC_EIG_TRIDIAGONAL && !direct_ok) return TC_ERR_PARAM;
  if (p->k_final < 1 || p->k_final > p->k_prune || p->k_prune > p->n_vis) return TC_ERR_PARAM;
  const int nA = p->k_prune / 2, nB = p->k_prune - nA;
  if (p->k_prune - p->k_final > nB) return TC_ERR_PARAM;

  Plan& q = *pl;
  q.B = p->batch; q.batch_call = p->batch; q.L = p->seq_len; q.Ls = p->vis_start; q.N = p->n_vis; q.H = p->n_heads; q.dh = p->head_dim;
  q.D = q.H * q.dh; q.hidden = p->hidden_dim; q.kp = p->k_prune; q.kf = p->k_final; q.m = q.kp - q.kf;
  q.nA = nA; q.nB = nB;
  q.Np = round_up(q.N, JT); q.nblk = q.Np / JB; q.P = q.nblk / 2; q.steps = q.nblk - 1;
  q.Nq = q.N + p->n_prompt_queries;
  q.q_tile = 128; q.n_qtiles = (q.Nq + q.q_tile - 1) / q.q_tile;
  q.esize = p->dtype == TC_F32 ? 4 : 2;
  q.tsize = p->eig_dtype == TC_EIG_F64 ? 8 : 4;
  q.groups = p->stream_groups;
  q.method = (p->eig_method == TC_EIG_JACOBI || !direct_ok) ? TC_EIG_JACOBI : TC_EIG_TRIDIAGONAL;
  q.max_sweeps = p->jacobi_max_sweeps > 0 ? p->jacobi_max_sweeps : 30;
  // The error of Eq. 3-6 grows like off(G) / (gap between neighbouring eigenvalues), and with more tokens the
  // gaps shrink like 1/N: the default tolerance found at N = 576 is scaled accordingly for larger N.
  const double tol_scale = q.Np > 576 ? 576.0 / q.Np : 1.0;
  q.tol = p->jacobi_tol > 0.f ? (double)p->jacobi_tol : (p->eig_dtype == TC_EIG_F64 ? 2e-9 * tol_scale : 3e-6);
  q.scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / std::sqrt((float)q.dh);

  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  const size_t B = (size_t)q.B, N = (size_t)q.N, Np = (size_t)q.Np;
  q.off_O = take(B * N * q.D * q.esize);
  q.off_S = take(B * N * 4);
  // per (head, query tile) column sums; the float path keeps a (max, sum) pair per (head, query row) there instead
  q.spart_stride = (size_t)q.H * ((size_t)q.n_qtiles * N > 2 * (size_t)q.Nq ? (size_t)q.n_qtiles * N : 2 * (size_t)q.Nq);
  q.off_Spart = take(B * q.spart_stride * 4);
  q.off_G = take(B * Np * Np * q.tsize);
  q.off_U = take(B * Np * Np * 4);  // eigenvectors are kept in float32
  q.off_R = take(B * q.P * JT * JT * q.tsize);
  q.off_offpart = take(B * (size_t)q.nblk * 8);
  q.off_state = take(B * sizeof(EigState));
  q.off_sig = take(B * Np * 8);
  q.off_C = take(B * N * 4);
  q.off_E = take(B * N * 4);
  q.off_order = take(B * q.kp * 4);
  q.off_rnorm = take(B * q.kp * 4);
  q.off_sim = take(B * (size_t)q.nB * (q.nA > 0 ? q.nA : 1) * 4);
  q.off_mlist = take(B * (size_t)(q.m > 0 ? q.m : 1) * 8);
  q.off_info = take(B * 4);
  if (q.method == TC_EIG_TRIDIAGONAL) {
    const size_t nstrip = (N + 15) / 16;   // strips of the back-transformation are 16 to 64 eigenvectors wide
    q.off_td_d = take(B * Np * 8);
    q.off_td_e = take(B * Np * 8);
    q.off_td_tau = take(B * Np * 4);
    q.off_td_lam = take(B * Np * 8);
    q.off_td_blk = take(B * Np * 8);
    q.off_td_tnorm = take(B * 8);
    q.off_td_rn = take(B * Np * 8);
    q.off_td_bad = take(B * 4);
    q.off_td_wgt = take(B * Np * 8);
    q.off_td_W = take(B * Np * Np * 4);        // eigenvectors of T (the reflectors use the region of U)
    q.off_td_tw = take(B * Np * Np * 16);      // pivots and multipliers of the twisted factorisations
    q.off_td_Cpart = take(B * nstrip * Np * 8);
    q.off_td_Tf = take(B * ((N + 15) / 16) * 256 * 4);   // T factors of the blocks of 16 reflectors
    q.off_td_tab = take(B * Np * 24 * 4);                // wavefront assignments of the reduction, one table per image slot
  }
  q.total = off > 0 ? off : 256;
  return TC_OK;
}

// Eigenvalues (and, with `vectors`, Eq. 3-6) by the tridiagonal route for the images img0 .. img0 + sub.B - 1 of the
// batch whose plan is `pl` (`sub` = the same plan with B = the number of images of this group); every
// workspace region is addressed per image, so groups of images can run side by side on different streams.
static int direct_chain(const Plan& pl, const Plan& sub, int img0, const tc_params* p, bool vectors, float* C_ws,
                        float* ics, float* sigma, int32_t* info, void* ws, hipStream_t st) {
  const size_t Np = pl.Np, i0 = img0, nstrip = (pl.N + 15) / 16, npanel = (pl.N + 15) / 16;
  double* G = at<double>(ws, pl.off_G) + i0 * Np * Np;
  double* dvec = at<double>(ws, pl.off_td_d) + i0 * Np;
  double* evec = at<double>(ws, pl.off_td_e) + i0 * Np;
  float* tauv = at<float>(ws, pl.off_td_tau) + i0 * Np;
  float* Vc = at<float>(ws, pl.off_U) + i0 * Np * Np;
  double* tw = at<double>(ws, pl.off_td_tw);
  // (the panels of the reduction pass through the start of the image's pivot scratch, which is idle until stage 2)
  int rc = launch_tridiag(sub, G, dvec, evec, tauv, Vc, tw + i0 * Np * Np, Np * Np, at<int>(ws, pl.off_td_tab) + i0 * Np * 24, st);
  if (rc != TC_OK) return rc;
  return launch_td_eigen(sub, dvec, evec, tauv, Vc, at<double>(ws, pl.off_td_lam) + i0 * Np, at<int2>(ws, pl.off_td_blk) + i0 * Np,
                         at<double>(ws, pl.off_td_tnorm) + i0, tw + i0 * Np * Np, tw + ((size_t)pl.B + i0) * Np * Np,
                         at<float>(ws, pl.off_td_W) + i0 * Np * Np, at<double>(ws, pl.off_td_rn) + i0 * Np,
                         at<int32_t>(ws, pl.off_td_bad) + i0, at<double>(ws, pl.off_sig) + i0 * Np,
                         at<double>(ws, pl.off_td_wgt) + i0 * Np, at<double>(ws, pl.off_td_Cpart) + i0 * nstrip * Np,
                         at<float>(ws, pl.off_td_Tf) + i0 * npanel * 256, p->sv_rtol, vectors, C_ws ? C_ws + i0 * pl.N : nullptr,
                         ics ? ics + i0 * pl.N : nullptr, sigma ? sigma + i0 * pl.N : nullptr, info ? info + i0 : nullptr, st);
}

// Attention (when Q is given), Gram matrix, eigen-decomposition and Eq. 3-6 / 3-8.
// Tridiagonal route: the batch is cut into groups of images (two by default from 16 images on, up to four on
// request) whose chains run on the library's helper streams, each group starting when the one before it has
// formed its Gram matrices.  The reduction to tridiagonal form keeps one compute unit per image busy for most
// of the call and is bound by latency, so the kernels of the other groups fill the rest of the chip meanwhile.
// The gain is small (about 2 % at 64 images): every kernel after the reduction is latency-bound as well and
// takes as long for half the batch as for all of it.
static int front_chain(const Plan& pl, const tc_params* p, const void* Q, const void* K, const void* V, void* O,
                       float* S, float* score, float* ics, float* sigma, int32_t* info, void* ws, hipStream_t st) {
  if (pl.method != TC_EIG_TRIDIAGONAL) {
    int rc = TC_OK;
    if (Q && (rc = launch_attention(pl, p->dtype, p->causal, Q, K, V, O, S, at<float>(ws, pl.off_Spart), st)) != TC_OK) return rc;
    void* G = at<char>(ws, pl.off_G);
    void* U = at<char>(ws, pl.off_U);
    EigState* state = at<EigState>(ws, pl.off_state);
    if ((rc = launch_gram(pl, p->dtype, p->eig_dtype, O, G, st)) != TC_OK) return rc;
    if ((rc = launch_jacobi(pl, p->eig_dtype, G, U, at<char>(ws, pl.off_R), at<double>(ws, pl.off_offpart), state, st)) != TC_OK)
      return rc;
    return launch_scores(pl, p->eig_dtype, G, U, state, S, p->lambda, p->norm_mode, p->sv_rtol, at<char>(ws, pl.off_sig),
                         at<float>(ws, pl.off_C), score, ics, sigma, info, st);
  }
  int groups = pl.groups > 0 ? pl.groups : (pl.B >= 16 ? 2 : 1);
  if (groups > pl.B) groups = pl.B;
  if (profiling_active()) groups = 1;  // per-kernel timing wants kernels that run alone
  hipStream_t streams[4];
  groups = fork_streams(st, groups, streams);
  int first[5];
  for (int g = 0; g <= groups; g++) first[g] = (int)((long long)pl.B * g / groups);
  int rc = TC_OK;
  for (int g = 0; g < groups && rc == TC_OK; g++) {
    const int img0 = first[g], nimg = first[g + 1] - img0;
    if (nimg <= 0) continue;
    Plan sub = pl;
    sub.B = nimg;
    const size_t i0 = img0, N = pl.N, es = pl.esize;
    char* Og = static_cast<char*>(O) + i0 * N * pl.D * es;
    float* Sg = S ? S + i0 * N : nullptr;
    if (Q) {
      const size_t qoff = i0 * pl.H * pl.L * pl.dh * es;
      rc = launch_attention(sub, p->dtype, p->causal, static_cast<const char*>(Q) + qoff, static_cast<const char*>(K) + qoff,
                            static_cast<const char*>(V) + qoff, Og, Sg,
                            at<float>(ws, pl.off_Spart) + i0 * pl.spart_stride, streams[g]);
      if (rc != TC_OK) break;
    }
    rc = launch_gram(sub, p->dtype, p->eig_dtype, Og, at<double>(ws, pl.off_G) + i0 * pl.Np * pl.Np, streams[g]);
    if (rc != TC_OK) break;
    // the next group's attention and Gram kernels (which fill the chip) start when this group's are done, so
    // that the groups' reductions start one after the other and their tails do not all come at the end
    stagger_streams(st, g, groups);
    float* C_ws = at<float>(ws, pl.off_C);
    rc = direct_chain(pl, sub, img0, p, true, C_ws, ics, sigma, info, ws, streams[g]);
    if (rc != TC_OK) break;
    rc = launch_combine(sub, C_ws + i0 * N, Sg, p->lambda, p->norm_mode, score + i0 * N, streams[g]);
  }
  join_streams(st, groups);
  return rc;
}

int direct_eigenvalues(const Plan& pl, const tc_params* p, float* sigma, int32_t* info, void* ws, hipStream_t st) {
  return direct_chain(pl, pl, 0, p, false, nullptr, nullptr, sigma, info, ws, st);
}

}  // namespace tc

using namespace tc;

extern "C" {

size_t tc_workspace_bytes(const tc_params* p) {
  Plan pl;
  if (make_plan(p, &pl) != TC_OK) return 0;
  return pl.total;
}

const char* tc_status_string(int status) {
  switch (status) {
    case TC_OK: return "ok";
    case TC_ERR_NULL: return "a required pointer is NULL";
    case TC_ERR_SHAPE: return "unsupported or inconsistent sizes";
    case TC_ERR_DTYPE: return "unknown dtype";
    case TC_ERR_PARAM: return "parameter out of range";
    case TC_ERR_WORKSPACE: return "workspace too small";
    case TC_ERR_ALIGN: return "pointer not 16-byte aligned";
    case TC_ERR_HIP: return "HIP launch failed";
    case TC_ERR_SCRATCH: return "sizes exceed the static scratch of tc_merge_noalloc (TC_NOALLOC_SCRATCH_BYTES)";
    default: return "unknown status";
  }
}

int tc_attn_output(const tc_params* p, const void* Q, const void* K, const void* V, void* O, float* attn_score,
                   void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;  // an empty batch: nothing to check, nothing to launch
  if (!Q || !K || !V || !O) return TC_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(attn_score)) return TC_ERR_ALIGN;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  return launch_attention(pl, p->dtype, p->causal, Q, K, V, O, attn_score, at<float>(ws, pl.off_Spart),
                          (hipStream_t)stream);
}

int tc_ipgs_score(const tc_params* p, const void* O, const float* attn_score, float* score, float* ics, float* sigma,
                  int32_t* info, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;  // an empty batch: nothing to check, nothing to launch
  if (!O || !score) return TC_ERR_NULL;
  if (!attn_score && p->lambda != 0.f) return TC_ERR_NULL;
  if (misaligned(O) || misaligned(attn_score) || misaligned(score) || misaligned(ics) || misaligned(sigma) ||
      misaligned(info))
    return TC_ERR_ALIGN;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  return front_chain(pl, p, nullptr, nullptr, nullptr, const_cast<void*>(O), const_cast<float*>(attn_score), score, ics, sigma,
                     info, ws, (hipStream_t)stream);
}

int tc_select_topk(const tc_params* p, const float* score, int32_t* order, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;  // an empty batch: nothing to check, nothing to launch
  if (!score || !order) return TC_ERR_NULL;
  if (misaligned(score) || misaligned(order)) return TC_ERR_ALIGN;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  return launch_topk(pl, score, order, (hipStream_t)stream);
}

int tc_merge(const tc_params* p, const void* X, const void* metric, const int32_t* order, void* X_out,
             int32_t* kept_idx, int32_t* merge_dst, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;  // an empty batch: nothing to check, nothing to launch
  if (!X || !metric || !order || !X_out || !kept_idx || !merge_dst) return TC_ERR_NULL;
  if (misaligned(X) || misaligned(metric) || misaligned(order) || misaligned(X_out) || misaligned(kept_idx) ||
      misaligned(merge_dst))
    return TC_ERR_ALIGN;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  return launch_merge(pl, p->dtype, X, metric, order, X_out, kept_idx, merge_dst, at<float>(ws, pl.off_rnorm),
                      at<float>(ws, pl.off_sim), at<int32_t>(ws, pl.off_mlist), (hipStream_t)stream);
}

int tc_similarity(const tc_params* p, const void* metric, const int32_t* order, float* sim, void* ws, size_t ws_bytes,
                  void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;  // an empty batch: nothing to check, nothing to launch
  if (!metric || !order || !sim) return TC_ERR_NULL;
  if (misaligned(metric) || misaligned(order) || misaligned(sim)) return TC_ERR_ALIGN;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  return launch_similarity(pl, p->dtype, metric, order, at<float>(ws, pl.off_rnorm), sim, (hipStream_t)stream);
}

int tc_compress(const tc_params* p, const void* Q, const void* K, const void* V, const void* X, void* X_out,
                int32_t* kept_idx, int32_t* merge_dst, void* O_opt, float* score_opt, int32_t* order_opt,
                int32_t* info_opt, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;  // an empty batch: nothing to check, nothing to launch
  if (!Q || !K || !V || !X || !X_out || !kept_idx || !merge_dst) return TC_ERR_NULL;
  if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(X) || misaligned(X_out) || misaligned(kept_idx) ||
      misaligned(merge_dst) || misaligned(O_opt) || misaligned(score_opt) || misaligned(order_opt) ||
      misaligned(info_opt))
    return TC_ERR_ALIGN;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  void* O = O_opt ? O_opt : at<char>(ws, pl.off_O);
  float* S = at<float>(ws, pl.off_S);
  float* E = score_opt ? score_opt : at<float>(ws, pl.off_E);
  int32_t* order = order_opt ? order_opt : at<int32_t>(ws, pl.off_order);
  int32_t* info = info_opt ? info_opt : at<int32_t>(ws, pl.off_info);
  rc = front_chain(pl, p, Q, K, V, O, S, E, nullptr, nullptr, info, ws, st);
  if (rc != TC_OK) return rc;
  rc = launch_topk(pl, E, order, st);
  if (rc != TC_OK) return rc;
  return launch_merge(pl, p->dtype, X, O, order, X_out, kept_idx, merge_dst, at<float>(ws, pl.off_rnorm),
                      at<float>(ws, pl.off_sim), at<int32_t>(ws, pl.off_mlist), st);
}

}  // extern "C"
