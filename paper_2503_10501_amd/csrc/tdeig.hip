// Direct symmetric eigensolver, stages 2 and 3 (stage 1, the reduction G = Q T Q^T, is tridiag.hip):
//   2a  eigenvalues of the tridiagonal T by bisection on Sturm counts, one lane per eigenvalue;
//   2b  eigenvector of every eigenvalue from the twisted factorisation of T - lambda I
//       (forward L D+ L^T, backward U D- U^T, joined at the index r that minimises |gamma_r|;
//       the vector solves (T - lambda I) z = gamma_r e_r), one lane per eigenvector;
//   3   back-transformation U = Q W = H_0 ... H_{N-2} W in float32 with the columns of a strip held in
//       registers, and, since U is only needed for it, the information contribution score of Eq. 3-6,
//       C(x) = sum_i |U[x][i]| sigma_i, accumulated right there: U is never written.
// T is first split where an off-diagonal element is negligible (|e_k| <= eps ||T||); each eigenpair then
// belongs to one unreduced block and its vector is zero outside that block, so equal eigenvalues of
// decoupled blocks (block-diagonal Gram matrices, null spaces) get orthogonal vectors for free.
// Eigenvectors of one block are computed independently of each other: their mutual orthogonality is
// eps ||T|| / gap.  For the spectra this library meets (gaps >= 1e-9 ||T||) that is 1e-6 or better; a pair
// closer than 1e-10 ||T|| inside one block is orthogonalised explicitly afterwards (td_cluster_kernel).
#include <cfloat>

#include "tc_internal.h"

namespace tc {

constexpr double TD_EPS = 2.220446049250313e-16;

// ---- 2a -----------------------------------------------------------------------------------------------
// dvec, evec [B][Np] from the reduction.  Writes lam [B][Np] (eigenvalue of slot k: the (k - s)-th smallest
// of the block [s, t) that row k lies in), blk [B][Np] = (s, t), and tnorm [B] = ||T||_inf.
__global__ __launch_bounds__(256) void td_bisect_kernel(const double* __restrict__ dvec, const double* __restrict__ evec,
                                                        double* __restrict__ lam, int2* __restrict__ blk,
                                                        double* __restrict__ tnorm, int32_t* __restrict__ bad, int N,
                                                        int Np) {
  extern __shared__ __attribute__((aligned(16))) unsigned char tb_smem[];
  double* ds = reinterpret_cast<double*>(tb_smem);  // [N]
  double* es = ds + N;                               // [N]: es[i] = |coupling of rows i-1 and i|, es[0] = 0
  double* e2 = es + N;                               // [N]: its square, 0 where T is split
  __shared__ double wmax[4];
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* db = dvec + (size_t)b * Np;
  const double* eb = evec + (size_t)b * Np;
  for (int i = tid; i < N; i += 256) {
    ds[i] = db[i];
    es[i] = i > 0 ? fabs(eb[i - 1]) : 0.0;
  }
  __syncthreads();
  double rowmax = 0.0;
  for (int i = tid; i < N; i += 256) rowmax = fmax(rowmax, fabs(ds[i]) + es[i] + (i + 1 < N ? es[i + 1] : 0.0));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) rowmax = fmax(rowmax, __shfl_xor(rowmax, o, 64));
  if (lane == 0) wmax[wave] = rowmax;
  __syncthreads();
  const double tn = fmax(fmax(wmax[0], wmax[1]), fmax(wmax[2], wmax[3]));
  const double split = TD_EPS * tn;
  for (int i = tid; i < N; i += 256) e2[i] = es[i] > split ? es[i] * es[i] : 0.0;
  __syncthreads();
  if (blockIdx.x == 0 && tid == 0) { tnorm[b] = tn; bad[b] = 0; }
  const int k = blockIdx.x * 256 + tid;
  if (k >= N) return;
  int s = k, t = k + 1;
  while (s > 0 && e2[s] != 0.0) s--;
  while (t < N && e2[t] != 0.0) t++;
  const int m = k - s;
  // Gershgorin interval of the block, slightly widened
  double lo = DBL_MAX, hi = -DBL_MAX, e2max = 0.0;
  for (int i = s; i < t; i++) {
    const double r = (i > s ? es[i] : 0.0) + (i + 1 < t ? es[i + 1] : 0.0);
    lo = fmin(lo, ds[i] - r);
    hi = fmax(hi, ds[i] + r);
    e2max = fmax(e2max, e2[i]);
  }
  const double widen = 2.0 * TD_EPS * tn * (t - s) + 2.0 * DBL_MIN;
  lo -= widen;
  hi += widen;
  const double pivmin = DBL_MIN * fmax(1.0, e2max);
  for (int it = 0; it < 128; it++) {
    const double mid = 0.5 * (lo + hi);
    if (!(mid > lo && mid < hi)) break;                                   // the interval cannot be halved any more
    if (hi - lo <= 0.25 * TD_EPS * tn) break;  // the entries of T carry errors of eps ||T|| themselves; same count for every lane
    // number of eigenvalues of the block below mid = number of negative pivots of T - mid I
    double q = ds[s] - mid;
    if (fabs(q) < pivmin) q = -pivmin;
    int cnt = q < 0.0 ? 1 : 0;
    for (int i = s + 1; i < t; i++) {
      q = (ds[i] - mid) - e2[i] / q;
      if (fabs(q) < pivmin) q = -pivmin;
      cnt += q < 0.0 ? 1 : 0;
    }
    if (cnt > m) hi = mid; else lo = mid;
  }
  lam[(size_t)b * Np + k] = 0.5 * (lo + hi);
  blk[(size_t)b * Np + k] = int2{s, t};
}

// ---- 2b -----------------------------------------------------------------------------------------------
// One lane per eigenvector.  DP and UM are scratch [B][Np][Np] doubles addressed [row][slot] (contiguous
// across the lanes of a wavefront).  W [B][Np][Np] float receives the unnormalised vector of slot k in
// column k (rows outside its block are zero); rn [B][Np] its reciprocal norm (0 if the vector is not
// finite, which also raises bad[b]).
__global__ __launch_bounds__(64) void td_twisted_kernel(const double* __restrict__ dvec, const double* __restrict__ evec,
                                                        const double* __restrict__ lam, const int2* __restrict__ blk,
                                                        const double* __restrict__ tnorm, double* __restrict__ DP,
                                                        double* __restrict__ UM, float* __restrict__ W,
                                                        double* __restrict__ rn, int32_t* __restrict__ bad, int N,
                                                        int Np) {
  extern __shared__ __attribute__((aligned(16))) unsigned char tw_smem[];
  double* ds = reinterpret_cast<double*>(tw_smem);  // [N]
  double* es = ds + N;                               // [N]: es[i] couples rows i and i+1 (signed), 0 where T is split
  const int b = blockIdx.y, tid = threadIdx.x;
  const double* db = dvec + (size_t)b * Np;
  const double* eb = evec + (size_t)b * Np;
  const double split = TD_EPS * tnorm[b];
  double e2max = 0.0;
  for (int i = tid; i < N; i += 64) {
    ds[i] = db[i];
    const double e = i + 1 < N ? eb[i] : 0.0;
    es[i] = fabs(e) > split ? e : 0.0;
  }
  __syncthreads();
  const int k = blockIdx.x * 64 + tid;
  if (k >= N) return;
  const int2 st = blk[(size_t)b * Np + k];
  const int s = st.x, t = st.y;
  for (int i = s; i + 1 < t; i++) e2max = fmax(e2max, es[i] * es[i]);
  const double pivmin = DBL_MIN * fmax(1.0, e2max);
  const double l = lam[(size_t)b * Np + k];
  double* dp = DP + (size_t)b * Np * Np + k;
  double* um = UM + (size_t)b * Np * Np + k;
  float* w = W + (size_t)b * Np * Np + k;
  // forward: T - l I = L D+ L^T, pivots dp[i]
  double p = ds[s] - l;
  for (int i = s; i < t; i++) {
    if (fabs(p) < pivmin) p = -pivmin;
    dp[(size_t)i * Np] = p;
    if (i + 1 < t) p = (ds[i + 1] - l) - (es[i] / p) * es[i];
  }
  // backward: T - l I = U D- U^T, pivots dm; gamma_i = dp[i] + dm[i] - (d_i - l); keep the smallest |gamma|
  double dm = ds[t - 1] - l;
  double gbest = DBL_MAX;
  int r = t - 1;
  for (int i = t - 1; i >= s; i--) {
    if (fabs(dm) < pivmin) dm = -pivmin;
    const double g = fabs(dp[(size_t)i * Np] + dm - (ds[i] - l));
    if (g < gbest || !(gbest == gbest)) { gbest = g; r = i; }
    if (i > s) {
      const double u = es[i - 1] / dm;
      um[(size_t)(i - 1) * Np] = u;
      dm = (ds[i - 1] - l) - u * es[i - 1];
    }
  }
  // the vector: z_r = 1, upwards with the multipliers of L, downwards with those of U
  for (int i = 0; i < s; i++) w[(size_t)i * Np] = 0.f;
  for (int i = t; i < N; i++) w[(size_t)i * Np] = 0.f;
  double z = 1.0, nrm = 1.0;
  w[(size_t)r * Np] = 1.f;
  for (int i = r - 1; i >= s; i--) {
    z = -(es[i] / dp[(size_t)i * Np]) * z;
    w[(size_t)i * Np] = (float)z;
    nrm += z * z;
  }
  z = 1.0;
  for (int i = r; i + 1 < t; i++) {
    z = -um[(size_t)i * Np] * z;
    w[(size_t)(i + 1) * Np] = (float)z;
    nrm += z * z;
  }
  const bool fin = nrm == nrm && nrm < DBL_MAX && nrm < 1e60;  // float storage of z holds |z| < 3e38 relative to z_r = 1
  rn[(size_t)b * Np + k] = fin ? 1.0 / sqrt(nrm) : 0.0;
  if (!fin) atomicOr(&bad[b], 1);
}

// ---- close eigenvalues inside one block -----------------------------------------------------------------
// One workgroup per image walks over the slots of every block in ascending order of eigenvalue.  A slot
// whose eigenvalue lies within 1e-10 ||T|| of its predecessor's joins the predecessor's cluster and its
// vector is orthogonalised (modified Gram-Schmidt, float64 accumulation) against the cluster's earlier
// vectors.  If nothing independent is left of it (the two vectors were the same to 1e-3) the pair cannot
// be separated this way: bad[b] gets bit 2 and the caller's info turns negative.
__global__ __launch_bounds__(256) void td_cluster_kernel(const double* __restrict__ lam, const int2* __restrict__ blk,
                                                         const double* __restrict__ tnorm, float* __restrict__ W,
                                                         double* __restrict__ rn, int32_t* __restrict__ bad, int N,
                                                         int Np) {
  __shared__ double red[4];
  __shared__ int any;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* lb = lam + (size_t)b * Np;
  const int2* bb = blk + (size_t)b * Np;
  double* rb = rn + (size_t)b * Np;
  float* Wb = W + (size_t)b * Np * Np;
  const double ctol = 1e-10 * tnorm[b];
  // quick exit: no close pair anywhere (the usual case)
  if (tid == 0) any = 0;
  __syncthreads();
  int mine = 0;
  for (int k = 1 + tid; k < N; k += 256) mine |= (bb[k].x == bb[k - 1].x && lb[k] - lb[k - 1] <= ctol) ? 1 : 0;
  if (mine) any = 1;  // every writer stores the same value
  __syncthreads();
  if (!any) return;
  auto block_sum = [&](double x) {
    x = wave_sum(x);
    __syncthreads();
    if (lane == 0) red[wave] = x;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
  };
  int first = 0;  // first slot of the current cluster
  for (int k = 1; k < N; k++) {
    const bool close = bb[k].x == bb[k - 1].x && lb[k] - lb[k - 1] <= ctol;  // uniform over the workgroup
    if (!close) { first = k; continue; }
    const int s = bb[k].x, t = bb[k].y;
    for (int j = first; j < k; j++) {
      double dot = 0.0;
      for (int i = s + tid; i < t; i += 256) dot += (double)Wb[(size_t)i * Np + j] * (double)Wb[(size_t)i * Np + k];
      dot = block_sum(dot) * rb[j] * rb[j];  // column j has norm 1 / rb[j]
      for (int i = s + tid; i < t; i += 256)
        Wb[(size_t)i * Np + k] = (float)((double)Wb[(size_t)i * Np + k] - dot * (double)Wb[(size_t)i * Np + j]);
      __syncthreads();
    }
    double n2 = 0.0;
    for (int i = s + tid; i < t; i += 256) { const double v = Wb[(size_t)i * Np + k]; n2 += v * v; }
    n2 = block_sum(n2);
    const double before = rb[k] > 0.0 ? 1.0 / (rb[k] * rb[k]) : 0.0;
    __syncthreads();
    if (tid == 0) {
      if (!(n2 > 1e-6 * before)) atomicOr(&bad[b], 2);
      rb[k] = n2 > 0.0 ? 1.0 / sqrt(n2) : 0.0;
    }
    __syncthreads();
  }
}

// ---- weights of Eq. 3-6 -----------------------------------------------------------------------------------
// sigma_k = sqrt(max(lambda_k, 0)); wgt[k] = sigma_k * rn[k] (0 for terms dropped by sv_rtol): the factor that
// turns the unnormalised vector of slot k into its term of C.  Also the optional outputs of tc_ipgs_score that
// do not need the vectors: sigma sorted in descending order, and info.
__global__ __launch_bounds__(256) void td_weights_kernel(const double* __restrict__ lam, const double* __restrict__ rn,
                                                         const int32_t* __restrict__ bad, float sv_rtol,
                                                         double* __restrict__ sig, double* __restrict__ wgt,
                                                         float* __restrict__ sigma_out, int32_t* __restrict__ info_out,
                                                         int N, int Np) {
  extern __shared__ float key[];  // pow2 >= N floats, only when sigma_out != nullptr
  __shared__ double wmax[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* lb = lam + (size_t)b * Np;
  double* sb = sig + (size_t)b * Np;
  double mx = 0.0;
  int nanflag = 0;
  for (int i = tid; i < Np; i += 256) {
    double s = 0.0;
    if (i < N) {
      const double l = lb[i];
      nanflag |= (l == l) ? 0 : 1;
      s = l > 0.0 ? sqrt(l) : 0.0;
    }
    sb[i] = s;
    mx = fmax(mx, s);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mx = fmax(mx, __shfl_xor(mx, o, 64));
    nanflag |= __shfl_xor(nanflag, o, 64);
  }
  __shared__ int wnan[4];
  if (lane == 0) { wmax[wave] = mx; wnan[wave] = nanflag; }
  __syncthreads();
  const double thr = sv_rtol > 0.f ? (double)sv_rtol * fmax(fmax(wmax[0], wmax[1]), fmax(wmax[2], wmax[3])) : -1.0;
  if (wgt)
    for (int i = tid; i < Np; i += 256) {
      const double s = sb[i];
      wgt[(size_t)b * Np + i] = (i < N && s > thr) ? s * rn[(size_t)b * Np + i] : 0.0;
    }
  if (tid == 0 && info_out)  // 1: done (the method does not iterate); negative: an eigenvector is not finite or a cluster stayed unresolved
    info_out[b] = (bad[b] | wnan[0] | wnan[1] | wnan[2] | wnan[3]) ? -1 : 1;
  if (!sigma_out) return;
  int n2 = 1;
  while (n2 < N) n2 <<= 1;
  for (int i = tid; i < n2; i += 256) key[i] = i < N ? (float)sb[i] : -1.0f;
  __syncthreads();
  for (int k = 2; k <= n2; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < n2; i += 256) {
        const int l = i ^ j;
        if (l > i) {
          const float a = key[i], c = key[l];
          const bool desc = (i & k) == 0;
          if (desc ? (a < c) : (a > c)) { key[i] = c; key[l] = a; }
        }
      }
      __syncthreads();
    }
  for (int i = tid; i < N; i += 256) sigma_out[(size_t)b * N + i] = key[i];
}

// ---- 3 ------------------------------------------------------------------------------------------------
// U = H_0 H_1 ... H_{N-2} W for a strip of 64 columns (eigenvectors), H_j = I - tau_j v_j v_j^T, applied from
// j = N-2 down to 0.  A workgroup of 16 wavefronts owns the strip: lane = column, wavefront w the rows
// i = 16 r + w (r < RT), held in registers for the whole kernel.  Per reflector: every wavefront forms
// its part of v_j^T U, the 16 parts are added in a fixed order through LDS (one barrier per reflector, two
// alternating buffers), then the rows are updated.  v_j comes through LDS too (three rotating buffers), reordered so that a
// wavefront reads its RT values as consecutive 16-byte pieces; only the chunks of four rows that a
// reflector reaches (rows > j) are touched.  At the end the strip's share of Eq. 3-6,
//     Cpart[strip][x] = sum_{k in strip} |U[x][k]| wgt[k],
// is reduced across the lanes and written; U itself is not.
template <int RT>
__global__ __launch_bounds__(1024) void td_backtransform_kernel(const float* __restrict__ W, const float* __restrict__ Vc,
                                                                const float* __restrict__ tauv,
                                                                const double* __restrict__ wgt,
                                                                double* __restrict__ Cpart, float* __restrict__ U_out,
                                                                int N, int Np, int nstrip) {
  static_assert(RT % 4 == 0, "rows are handled four at a time");
  __shared__ __attribute__((aligned(16))) float vbuf[3][16 * RT];  // v_j reordered: [row % 16][row / 16]; three in rotation
  __shared__ float red[2][16][64];
  const int b = blockIdx.y, strip = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = strip * 64 + lane;  // this lane's eigenvector
  const bool live = k < N;
  const float* Wb = W + (size_t)b * Np * Np;
  const float* Vb = Vc + (size_t)b * Np * Np;
  const float* tb = tauv + (size_t)b * Np;
  float u[RT];
#pragma unroll
  for (int r = 0; r < RT; r++) {
    const int i = 16 * r + w;
    u[r] = (live && i < N) ? Wb[(size_t)i * Np + k] : 0.f;
  }
  // the slot of row i in the reordered v: (i % 16) * RT + i / 16
  auto stage = [&](int j, int buf) {
    for (int i = tid; i < 16 * RT; i += 1024) vbuf[buf][(i & 15) * RT + (i >> 4)] = i < N ? Vb[(size_t)j * Np + i] : 0.f;
  };
  if (N >= 2) stage(N - 2, 0);
  __syncthreads();
  for (int j = N - 2; j >= 0; j--) {
    const int step = N - 2 - j, cur = step & 1, vcur = step % 3;
    // v of the next reflector, published by this step's barrier.  Three buffers: the one of the previous step
    // may still be read by wavefronts that are in that step's update (which comes after its barrier).
    if (j > 0) stage(j - 1, (step + 1) % 3);
    const float* vj = &vbuf[vcur][w * RT];
    // rows 16 r + w > j  <=>  r >= (j - w) / 16 + 1 (for j >= w), else every r: first chunk of four that matters
    const int rlo = j >= w ? (j - w) / 16 + 1 : 0;
    const int c0 = rlo >> 2;
    float part = 0.f;
#pragma unroll
    for (int c = 0; c < RT / 4; c++) {
      if (c >= c0) {  // uniform over the wavefront
        const float4 q = *reinterpret_cast<const float4*>(vj + 4 * c);
        part += q.x * u[4 * c];
        part += q.y * u[4 * c + 1];
        part += q.z * u[4 * c + 2];
        part += q.w * u[4 * c + 3];
      }
    }
    red[cur][w][lane] = part;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int x = 0; x < 16; x++) s += red[cur][x][lane];
    s *= tb[j];
#pragma unroll
    for (int c = 0; c < RT / 4; c++) {
      if (c >= c0) {  // v_j is read a second time rather than kept: 64 rows of u leave no registers for it
        const float4 q = *reinterpret_cast<const float4*>(vj + 4 * c);
        u[4 * c] -= s * q.x;
        u[4 * c + 1] -= s * q.y;
        u[4 * c + 2] -= s * q.z;
        u[4 * c + 3] -= s * q.w;
      }
    }
  }
  if (U_out && live) {
    float* Ub = U_out + (size_t)b * Np * Np;
#pragma unroll
    for (int r = 0; r < RT; r++) {
      const int i = 16 * r + w;
      if (i < N) Ub[(size_t)i * Np + k] = u[r];
    }
  }
  // Eq. 3-6, this strip's share
  const double wk = live ? wgt[(size_t)b * Np + k] : 0.0;
  double* Cp = Cpart + ((size_t)b * nstrip + strip) * Np;
#pragma unroll
  for (int r = 0; r < RT; r++) {
    const int i = 16 * r + w;
    const double term = wave_sum(fabs((double)u[r]) * wk);
    if (lane == 0 && i < N) Cp[i] = term;
  }
}

// C(x) = sum over the strips of their shares, in a fixed order.
__global__ __launch_bounds__(256) void td_ics_finish_kernel(const double* __restrict__ Cpart, float* __restrict__ C,
                                                            float* __restrict__ C_out, int N, int Np, int nstrip) {
  const int b = blockIdx.y, x = blockIdx.x * 256 + threadIdx.x;
  if (x >= N) return;
  double s = 0.0;
  for (int t = 0; t < nstrip; t++) s += Cpart[((size_t)b * nstrip + t) * Np + x];
  C[(size_t)b * N + x] = (float)s;
  if (C_out) C_out[(size_t)b * N + x] = (float)s;
}

int launch_td_eigen(const Plan& pl, const double* dvec, const double* evec, const float* tauv, const float* Vc,
                    double* lam, int2* blk, double* tnorm, double* DP, double* UM, float* W, double* rn, int32_t* bad,
                    double* sig, double* wgt, double* Cpart, float sv_rtol, bool vectors, float* C, float* C_out,
                    float* sigma_out, int32_t* info_out, hipStream_t st) {
  const int N = pl.N, Np = pl.Np, B = pl.B;
  TC_TIMED(PK_BISECT, 0, st, (td_bisect_kernel<<<dim3((N + 255) / 256, B), 256, (size_t)3 * N * 8, st>>>(dvec, evec, lam, blk, tnorm, bad, N, Np)));
  int n2 = 1;
  while (n2 < N) n2 <<= 1;
  const size_t shm_sig = sigma_out ? (size_t)n2 * sizeof(float) : 0;
  if (!vectors) {  // eigenvalues only (the information-quantity tool)
    TC_TIMED(PK_BISECT, 1, st, (td_weights_kernel<<<B, 256, shm_sig, st>>>(lam, nullptr, bad, 0.f, sig, nullptr, sigma_out, info_out, N, Np)));
    return check_launch();
  }
  TC_TIMED(PK_TWISTED, 0, st, (td_twisted_kernel<<<dim3((N + 63) / 64, B), 64, (size_t)2 * N * 8, st>>>(dvec, evec, lam, blk, tnorm, DP, UM, W, rn, bad, N, Np)));
  TC_TIMED(PK_TWISTED, 1, st, (td_cluster_kernel<<<B, 256, 0, st>>>(lam, blk, tnorm, W, rn, bad, N, Np)));
  TC_TIMED(PK_BISECT, 1, st, (td_weights_kernel<<<B, 256, shm_sig, st>>>(lam, rn, bad, sv_rtol, sig, wgt, sigma_out, info_out, N, Np)));
  const int nstrip = (N + 63) / 64;
  const dim3 gb(nstrip, B);
  if (Np <= 64)
    TC_TIMED(PK_BACKTF, 0, st, (td_backtransform_kernel<4><<<gb, 1024, 0, st>>>(W, Vc, tauv, wgt, Cpart, nullptr, N, Np, nstrip)));
  else if (Np <= 256)
    TC_TIMED(PK_BACKTF, 0, st, (td_backtransform_kernel<16><<<gb, 1024, 0, st>>>(W, Vc, tauv, wgt, Cpart, nullptr, N, Np, nstrip)));
  else if (Np <= 576)
    TC_TIMED(PK_BACKTF, 0, st, (td_backtransform_kernel<36><<<gb, 1024, 0, st>>>(W, Vc, tauv, wgt, Cpart, nullptr, N, Np, nstrip)));
  else if (Np <= 1024)
    TC_TIMED(PK_BACKTF, 0, st, (td_backtransform_kernel<64><<<gb, 1024, 0, st>>>(W, Vc, tauv, wgt, Cpart, nullptr, N, Np, nstrip)));
  else
    return TC_ERR_SHAPE;
  TC_TIMED(PK_ICS, 0, st, (td_ics_finish_kernel<<<dim3((N + 255) / 256, B), 256, 0, st>>>(Cpart, C, C_out, N, Np, nstrip)));
  return check_launch();
}

}  // namespace tc
