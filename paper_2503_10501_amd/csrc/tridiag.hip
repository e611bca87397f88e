// Direct symmetric eigensolver, stage 1: reduction of the Gram matrix to tridiagonal form,
//     G = Q T Q^T,   Q = H_0 H_1 ... H_{N-3},   H_j = I - tau_j v_j v_j^T  (Householder reflectors),
// so that the singular vectors of Section 3.3.1 (Z = U Sigma V^T, Z Z^T = U Sigma^2 U^T) become
// U = Q W with T W = W Sigma^2 (stages 2 and 3: tdeig.hip).
//
// One workgroup of 16 wavefronts reduces one image; nothing is exchanged between workgroups.  The
// reduction is bound by memory: column j needs the product of the trailing (N-j-1)^2 matrix with v_j.
// Measured on MI355X a single workgroup streams 150 GB/s out of its L2 and 64 of them together 6 TB/s,
// which is what the fabric delivers to any number of compute units for a working set of this size, so
// one compute unit per image is enough at batch 64.
//
// The trailing matrix is only rewritten once per panel of nb columns (the scheme of LAPACK's
// dlatrd/dsytrd): inside a panel the reflectors v and the vectors w of the rank-2 updates
// A <- A - v w^T - w v^T are kept in LDS (panels Vp, Wp) and applied on the fly to the column being
// reduced and to the matrix-vector product; at the end of the panel the trailing matrix gets the
// rank-2nb update on the matrix cores (both triangles: the matrix-vector product reads whole rows).
// G is symmetric and stored in full, so the product p = A v is formed as column sums over rows,
// p_c = sum_i A[i][c] v_i: a lane owns two neighbouring columns, loads are 16 bytes wide and contiguous
// across the wavefront, and no cross-lane reduction is needed; 4 row groups x 4 column groups of
// wavefronts leave four partial sums per column, added in a fixed order (results are bit-reproducible).
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(2))) double d2;
typedef __attribute__((ext_vector_type(4))) double d4;

constexpr int TD_THREADS = 1024;
constexpr int TD_WAVES = TD_THREADS / 64;
constexpr int TD_LDS_BYTES = 160 * 1024;  // LDS of one compute unit, all of it for the one workgroup

// Panel width that fits the LDS next to the vectors: v, p and four rows of partial sums (7 vectors of Nr
// doubles), the two panels (2 nb Nr doubles) and 1 KB of small scratch.
int tridiag_panel_width(int N) {
  const int Nr = round_up(N, 16);
  long nb = ((long)TD_LDS_BYTES - 1024 - 7L * Nr * 8) / (16L * Nr);
  nb &= ~3L;
  return nb > 32 ? 32 : (int)nb;
}
size_t tridiag_lds_bytes(int N, int nb) {
  const int Nr = round_up(N, 16);
  return (size_t)(2 * nb + 7) * Nr * 8 + 1024;
}

// Sum over the workgroup in a fixed order: lanes by the butterfly of lane 0, wavefronts left to right.
__device__ inline double td_block_sum(double x, double* scratch, int wave, int lane) {
  x = wave_sum(x);
  if (lane == 0) scratch[wave] = x;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < TD_WAVES; k++) s += scratch[k];
  __syncthreads();
  return s;
}

// G      [B][Np][Np]  in: the Gram matrix, symmetric, stored in full; destroyed
// dvec   [B][Np]      out: diagonal of T
// evec   [B][Np]      out: evec[j] = T[j+1][j], j < N-1
// tauv   [B][Np]      out: tau_j (0 for a reflector that is the identity)
// Vc     [B][Np][Np]  out, float: row j holds v_j (zeros up to index j, 1 at j+1); rows j >= N-1 are not written
__global__ __launch_bounds__(TD_THREADS) void tridiag_kernel(double* __restrict__ G, int N, int Np, int nb,
                                                             double* __restrict__ dvec, double* __restrict__ evec,
                                                             float* __restrict__ tauv, float* __restrict__ Vc) {
  extern __shared__ __attribute__((aligned(16))) unsigned char td_smem[];
  const int Nr = round_up(N, 16);
  double* Vp = reinterpret_cast<double*>(td_smem);  // [Nr][nb] reflectors of the panel
  double* Wp = Vp + (size_t)Nr * nb;                 // [Nr][nb] their update vectors
  double* vs = Wp + (size_t)Nr * nb;                 // [Nr] current reflector
  double* as = vs + Nr;                              // [Nr] current column
  double* red = as + Nr;                             // [4][Nr] partial column sums of the four row groups
  double* dots = red + 4 * (size_t)Nr;               // [64] W^T v and V^T v
  double* wsum = dots + 64;                          // [16] wavefront partials of td_block_sum
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  double* A = G + (size_t)b * Np * Np;
  double* dout = dvec + (size_t)b * Np;
  double* eout = evec + (size_t)b * Np;
  float* tout = tauv + (size_t)b * Np;
  float* Vout = Vc + (size_t)b * Np * Np;
  const int l15 = lane & 15, q4 = lane >> 4;

  for (int j0 = 0; j0 < N - 1; j0 += nb) {
    const int jend = min(j0 + nb, N - 1);  // this panel reduces columns j0 .. jend-1
    for (int j = j0; j < jend; j++) {
      const int jj = j - j0;
      // ---- column j of the matrix as it would be with the panel's updates applied (row j, by symmetry) ----
      const int i1 = j + tid;
      double x = 0.0;
      if (i1 < N) {
        x = A[(size_t)j * Np + i1];
        for (int c = 0; c < jj; c++) x -= Vp[i1 * nb + c] * Wp[j * nb + c] + Wp[i1 * nb + c] * Vp[j * nb + c];
        as[i1] = x;
      }
      if (tid == 0) dout[j] = x;
      // ---- Householder reflector that maps x[j+1:] onto beta e_1 ------------------------------------------
      const double xn2 = td_block_sum((tid >= 2 && i1 < N) ? x * x : 0.0, wsum, wave, lane);  // (its barriers also publish as[])
      const double alpha = as[j + 1];
      double beta = alpha, tau = 0.0, scal = 0.0;
      if (xn2 > 0.0) {
        beta = -copysign(sqrt(alpha * alpha + xn2), alpha);
        tau = (beta - alpha) / beta;
        scal = 1.0 / (alpha - beta);
      }
      if (tid >= 1 && i1 < N) {
        const double v = tid == 1 ? 1.0 : x * scal;
        vs[i1] = v;
        Vp[i1 * nb + jj] = v;
      }
      if (tid == 0) {
        eout[j] = beta;
        tout[j] = (float)tau;
      }
      __syncthreads();
      // ---- p = A v over the trailing matrix (rows and columns j+1 .. N-1), as column sums -------------------
      const int r0 = j + 1;
      const int cbase = r0 & ~1;                 // column pairs start at an even column (16-byte loads)
      const int npair = (N - cbase + 1) >> 1;
      const int np4 = (npair + 3) >> 2;          // pairs per column group, <= 128
      {
        const int rg = wave & 3, cg = wave >> 2;
        const int qa = cg * np4 + lane, qb = qa + 64;
        const bool oka = lane < np4 && qa < npair, okb = lane + 64 < np4 && qb < npair;
        const double* cola = A + cbase + 2 * (oka ? qa : 0);
        const double* colb = A + cbase + 2 * (okb ? qb : 0);
        d2 acca = d2{0.0, 0.0}, accb = d2{0.0, 0.0};
        const bool two = np4 > 64;  // uniform: only matrices with more than 512 trailing columns need the second pair
        for (int ib = r0 + rg; ib < N; ib += 32) {
          d2 xa[8], xb[8];
          double vi[8];
#pragma unroll
          for (int u = 0; u < 8; u++) {
            const int i = ib + 4 * u;
            const bool in = i < N;
            const size_t ro = (size_t)(in ? i : r0) * Np;  // a row past the end is replaced by a valid one and gets weight 0
            vi[u] = in ? vs[i] : 0.0;
            xa[u] = *reinterpret_cast<const d2*>(cola + ro);
            if (two) xb[u] = *reinterpret_cast<const d2*>(colb + ro);
          }
#pragma unroll
          for (int u = 0; u < 8; u++) {
            acca += xa[u] * vi[u];
            if (two) accb += xb[u] * vi[u];
          }
        }
        if (oka) { red[rg * Nr + cbase + 2 * qa] = acca.x; red[rg * Nr + cbase + 2 * qa + 1] = acca.y; }
        if (okb) { red[rg * Nr + cbase + 2 * qb] = accb.x; red[rg * Nr + cbase + 2 * qb + 1] = accb.y; }
      }
      // ---- W^T v and V^T v for the panel's earlier columns: one wavefront per dot product ------------------
      for (int id = wave; id < 2 * jj; id += TD_WAVES) {
        const double* P = id < jj ? Wp + id : Vp + (id - jj);
        double s = 0.0;
        for (int i = r0 + lane; i < N; i += 64) s += P[i * nb] * vs[i];
        s = wave_sum(s);
        if (lane == 0) dots[id] = s;
      }
      __syncthreads();
      // ---- p <- tau (A v - V (W^T v) - W (V^T v)),  w = p - (tau/2) (p^T v) v -------------------------------
      const int c = r0 + tid;
      double pc = 0.0, vc = 0.0;
      if (c < N) {
        pc = (red[c] + red[Nr + c]) + (red[2 * Nr + c] + red[3 * Nr + c]);
        for (int k = 0; k < jj; k++) pc -= Vp[c * nb + k] * dots[k] + Wp[c * nb + k] * dots[jj + k];
        pc *= tau;
        vc = vs[c];
      }
      const double pv = td_block_sum(pc * vc, wsum, wave, lane);
      if (c < N) Wp[c * nb + jj] = pc - 0.5 * tau * pv * vc;
      __syncthreads();
    }
    // ---- end of the panel ----------------------------------------------------------------------------------
    const int cnt = jend - j0;          // columns reduced in this panel
    const int kcols = round_up(cnt, 4); // contraction length per factor, padded with zero columns
    // the reflectors leave as float rows (stage 3 applies them in float32)
    for (int jj = 0; jj < cnt; jj++) {
      const int j = j0 + jj;
      for (int i = tid; i < N; i += TD_THREADS)
        Vout[(size_t)j * Np + i] = i > j ? (float)Vp[i * nb + jj] : 0.f;
    }
    if (kcols > cnt) {  // a last, shorter panel: columns cnt .. kcols-1 still hold the previous panel
      for (int e = tid; e < Nr * (kcols - cnt); e += TD_THREADS) {
        const int i = e / (kcols - cnt), k = cnt + e % (kcols - cnt);
        Vp[i * nb + k] = 0.0;
        Wp[i * nb + k] = 0.0;
      }
    }
    __syncthreads();
    // trailing matrix (rows and columns jend .. N-1) <- itself - Vp Wp^T - Wp Vp^T on the matrix cores.
    // A task is a strip of 16 rows x 64 columns; product ks contracts over k = 4 ks + lane / 16 of the
    // 2 kcols columns of [Vp | Wp] (rows) against [Wp | Vp] (columns).
    {
      const int base = jend & ~15;
      const int nrt = (N - base + 15) >> 4, ncc = (N - base + 63) >> 6;
      const int ksteps = kcols >> 2;
      for (int task = wave; task < nrt * ncc; task += TD_WAVES) {
        const int rt = base + 16 * (task / ncc), ct = base + 64 * (task % ncc);
        d4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; t++) {
          const int cc = ct + 16 * t + l15;
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const int rr = rt + 4 * e + q4;
            acc[t][e] = (rr < N && cc < N) ? A[(size_t)rr * Np + cc] : 0.0;
          }
        }
        const int arow = min(rt + l15, Nr - 1);
        for (int half = 0; half < 2; half++) {
          const double* L = half == 0 ? Vp : Wp;   // row factor
          const double* R = half == 0 ? Wp : Vp;   // column factor
          for (int ks = 0; ks < ksteps; ks++) {
            const int k = 4 * ks + q4;
            const double a = -L[arow * nb + k];
#pragma unroll
            for (int t = 0; t < 4; t++) {
              const int crow = min(ct + 16 * t + l15, Nr - 1);
              acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, R[crow * nb + k], acc[t], 0, 0, 0);
            }
          }
        }
#pragma unroll
        for (int t = 0; t < 4; t++) {
          const int cc = ct + 16 * t + l15;
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const int rr = rt + 4 * e + q4;
            if (rr >= jend && cc >= jend && rr < N && cc < N) A[(size_t)rr * Np + cc] = acc[t][e];
          }
        }
      }
    }
    __syncthreads();  // the rewritten matrix is visible to the whole workgroup
  }
  if (tid == 0) {
    dout[N - 1] = A[(size_t)(N - 1) * Np + (N - 1)];
    eout[N - 1] = 0.0;
    tout[N - 1] = 0.f;
  }
}

int launch_tridiag(const Plan& pl, double* G, double* dvec, double* evec, float* tauv, float* Vc, hipStream_t st) {
  const int nb = tridiag_panel_width(pl.N);
  if (nb < 4) return TC_ERR_SHAPE;
  const size_t lds = tridiag_lds_bytes(pl.N, nb);
  // more than 64 KB of dynamic LDS has to be allowed per function (a cheap host call, repeated so that it
  // holds on whichever device is current)
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(tridiag_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          TD_LDS_BYTES) != hipSuccess)
    return TC_ERR_HIP;
  TC_TIMED(PK_TRIDIAG, 0, st, (tridiag_kernel<<<pl.B, TD_THREADS, lds, st>>>(G, pl.N, pl.Np, nb, dvec, evec, tauv, Vc)));
  return check_launch();
}

}  // namespace tc
