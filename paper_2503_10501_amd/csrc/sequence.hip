// The token sequence after compression (Fig. 2 of the TokenCarve paper): system tokens, the
// compressed visual tokens, prompt tokens, every token with the position id it had before
// (Conclusion: rotary position encodings are recomputed from the original position ids), and the
// rotary tables cos/sin(position * theta_i), theta_i = base^(-2i/d_h), for those positions.
#include "tc_internal.h"

namespace tc {

// One workgroup per row of the new sequence.
__global__ __launch_bounds__(256) void assemble_kernel(const uint4* __restrict__ H, const uint4* __restrict__ Xc,
                                                       const int32_t* __restrict__ kept, uint4* __restrict__ Hn,
                                                       int32_t* __restrict__ pos_ids, float* __restrict__ rcos,
                                                       float* __restrict__ rsin, int L, int Ls, int N, int kf, int vec,
                                                       int dh, double log_base) {
  const int b = blockIdx.y, j = blockIdx.x, Ln = L - N + kf;
  const uint4* src;
  int pos;
  if (j < Ls) {
    pos = j;
    src = H + ((size_t)b * L + j) * vec;
  } else if (j < Ls + kf) {
    int x = kept[(size_t)b * kf + (j - Ls)];
    x = x < 0 ? 0 : (x >= N ? N - 1 : x);
    pos = Ls + x;
    src = Xc + ((size_t)b * kf + (j - Ls)) * vec;
  } else {
    pos = j + N - kf;
    src = H + ((size_t)b * L + pos) * vec;
  }
  uint4* dst = Hn + ((size_t)b * Ln + j) * vec;
  for (int i = threadIdx.x; i < vec; i += 256) dst[i] = src[i];
  if (threadIdx.x == 0) pos_ids[(size_t)b * Ln + j] = pos;
  if (rcos) {
    const int half = dh / 2;
    for (int i = threadIdx.x; i < half; i += 256) {
      const double theta = exp(-2.0 * (double)i / (double)dh * log_base);
      const double ang = (double)pos * theta;
      rcos[((size_t)b * Ln + j) * half + i] = (float)cos(ang);
      rsin[((size_t)b * Ln + j) * half + i] = (float)sin(ang);
    }
  }
}

}  // namespace tc

using namespace tc;

extern "C" int tc_assemble_sequence(const tc_params* p, const void* H, const void* X_out, const int32_t* kept_idx,
                                    void* H_new, int32_t* pos_ids, float rope_base, float* rope_cos, float* rope_sin,
                                    void* stream) {
  Plan pl;
  int rc = make_plan(p, &pl);
  if (rc != TC_OK) return rc;
  if (pl.B == 0) return TC_OK;
  if (!H || !X_out || !kept_idx || !H_new || !pos_ids) return TC_ERR_NULL;
  if ((rope_cos == nullptr) != (rope_sin == nullptr)) return TC_ERR_NULL;
  if (rope_cos && !(rope_base > 1.f)) return TC_ERR_PARAM;
  if (misaligned(H) || misaligned(X_out) || misaligned(kept_idx) || misaligned(H_new) || misaligned(pos_ids) ||
      misaligned(rope_cos) || misaligned(rope_sin))
    return TC_ERR_ALIGN;
  const int Ln = pl.L - pl.N + pl.kf;
  const int vec = pl.hidden * pl.esize / 16;
  assemble_kernel<<<dim3(Ln, pl.B), 256, 0, (hipStream_t)stream>>>(
      (const uint4*)H, (const uint4*)X_out, kept_idx, (uint4*)H_new, pos_ids, rope_cos, rope_sin, pl.L, pl.Ls, pl.N,
      pl.kf, vec, pl.dh, rope_cos ? std::log((double)rope_base) : 0.0);
  return check_launch();
}

extern "C" double tc_kv_cache_fraction(int32_t n_text, int32_t n_vis, int32_t n_kept, int32_t n_layers,
                                       int32_t n_layers_before) {
  if (n_text < 0 || n_vis < 1 || n_kept < 0 || n_kept > n_vis || n_layers < 1 || n_layers_before < 0 ||
      n_layers_before > n_layers)
    return -1.0;
  const double full = (double)n_text + n_vis, kept = (double)n_text + n_kept;
  return (n_layers_before * full + (n_layers - n_layers_before) * kept) / (n_layers * full);
}
