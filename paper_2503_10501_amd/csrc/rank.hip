// Information quantity of a set of visual tokens (Section 3.2.2 of the TokenCarve paper): the matrix
// rank of their attention-output rows, counted as the singular values above rtol * sigma_max.  The
// singular values come from the same Gram matrix + Jacobi eigensolver as Eq. 3-6, without the
// eigenvectors.
#include "tc_internal.h"

namespace tc {

// dst[b][j][:] = src[b][rows[b][j]][:], rows of `bytes` bytes (a multiple of 16); an index outside
// [0, N) is clamped.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ rows,
                                                          uint4* __restrict__ dst, int N, int n_rows, int vec_per_row) {
  const int b = blockIdx.y, j = blockIdx.x;
  int r = rows[(size_t)b * n_rows + j];
  r = r < 0 ? 0 : (r >= N ? N - 1 : r);
  const uint4* s = src + ((size_t)b * N + r) * vec_per_row;
  uint4* d = dst + ((size_t)b * n_rows + j) * vec_per_row;
  for (int i = threadIdx.x; i < vec_per_row; i += 256) d[i] = s[i];
}

// rank[b] = #{ i : sigma_i > rtol * max_i sigma_i }, compared in float64.
__global__ __launch_bounds__(256) void rank_kernel(const double* __restrict__ sig, double rtol, int32_t* __restrict__ rank,
                                                   int Np) {
  __shared__ double smax[4];
  __shared__ int cnt[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* sb = sig + (size_t)b * Np;
  double mx = 0.0;
  for (int i = tid; i < Np; i += 256) mx = fmax(mx, sb[i]);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o, 64));
  if (lane == 0) smax[wave] = mx;
  __syncthreads();
  mx = fmax(fmax(smax[0], smax[1]), fmax(smax[2], smax[3]));
  const double thr = rtol * mx;
  int c = 0;
  for (int i = tid; i < Np; i += 256) c += (mx > 0.0 && sb[i] > thr) ? 1 : 0;
  c = wave_sum(c);
  if (lane == 0) cnt[wave] = c;
  __syncthreads();
  if (tid == 0) rank[b] = cnt[0] + cnt[1] + cnt[2] + cnt[3];
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

}  // namespace tc

using namespace tc;

extern "C" int tc_info_rank(const tc_params* p, const void* O, const int32_t* rows, int32_t n_rows, float rtol,
                            int32_t* rank, float* sigma, int32_t* info, void* ws, size_t ws_bytes, void* stream) {
  Plan full;
  int rc = make_plan(p, &full);
  if (rc != TC_OK) return rc;
  if (full.B == 0) return TC_OK;
  if (!rows) n_rows = full.N;
  if (n_rows < 0 || n_rows > full.N) return TC_ERR_SHAPE;
  if (!(rtol >= 0.f) || rtol >= 1.f || (rtol > 0.f && rtol < 1e-7f)) return TC_ERR_PARAM;  // the Gram route resolves sigma down to about 1e-7 sigma_max
  if (!O || !rank) return TC_ERR_NULL;
  if (misaligned(O) || misaligned(rows) || misaligned(rank) || misaligned(sigma) || misaligned(info)) return TC_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  if (n_rows == 0) {  // no rows: rank 0, no workspace needed
    fill_i32_kernel<<<(full.B + 255) / 256, 256, 0, st>>>(rank, 0, full.B);
    if (info) fill_i32_kernel<<<(full.B + 255) / 256, 256, 0, st>>>(info, 1, full.B);
    return check_launch();
  }
  tc_params q = *p;  // the same problem on n_rows tokens; selection and merge sizes are irrelevant here
  q.n_vis = n_rows;
  q.k_prune = q.k_final = 1;
  Plan pl;
  if ((rc = make_plan(&q, &pl)) != TC_OK) return rc;
  if ((rc = check_ws(pl, ws, ws_bytes)) != TC_OK) return rc;
  const void* Osub = O;
  if (rows) {
    const int vec = pl.D * pl.esize / 16;
    gather_rows_kernel<<<dim3(n_rows, pl.B), 256, 0, st>>>((const uint4*)O, rows, at<uint4>(ws, pl.off_O), full.N, n_rows, vec);
    Osub = at<char>(ws, pl.off_O);
  }
  void* G = at<char>(ws, pl.off_G);
  EigState* state = at<EigState>(ws, pl.off_state);
  if ((rc = launch_gram(pl, p->dtype, p->eig_dtype, Osub, G, st)) != TC_OK) return rc;
  if (pl.method == TC_EIG_TRIDIAGONAL) {  // eigenvalues only: reduction and bisection, no vectors
    if ((rc = direct_eigenvalues(pl, &q, sigma, info, ws, st)) != TC_OK) return rc;
  } else {
    if ((rc = launch_jacobi(pl, p->eig_dtype, G, nullptr, at<char>(ws, pl.off_R), at<double>(ws, pl.off_offpart), state, st)) != TC_OK)
      return rc;
    if ((rc = launch_sigma(pl, p->eig_dtype, G, state, at<double>(ws, pl.off_sig), sigma, info, st)) != TC_OK) return rc;
  }
  const double tol = rtol > 0.f ? (double)rtol : (double)(n_rows > pl.D ? n_rows : pl.D) * 1.1920928955078125e-07;  // 2^-23
  rank_kernel<<<pl.B, 256, 0, st>>>(at<double>(ws, pl.off_sig), tol, rank, pl.Np);
  return check_launch();
}
