// Direct symmetric eigensolver, stage 1: reduction of the Gram matrix to tridiagonal form,
//     G = Q T Q^T,   Q = H_0 H_1 ... H_{N-3},   H_j = I - tau_j v_j v_j^T  (Householder reflectors),
// so that the singular vectors of Section 3.3.1 (Z = U Sigma V^T, Z Z^T = U Sigma^2 U^T) become
// U = Q W with T W = W Sigma^2 (stages 2 and 3: tdeig.hip).
//
// The columns of an image are reduced by one workgroup of 16 wavefronts.  The reduction is bound by
// memory: column j needs the product of the trailing (N-j-1)^2 matrix with v_j.  Measured on MI355X a
// single workgroup streams 150 GB/s out of its L2 and 64 of them together 6 TB/s, which is what the
// fabric delivers to any number of compute units for a working set of this size, so one compute unit per
// image is enough for the products at batch 64.
//
// The trailing matrix is only rewritten once per panel of nb columns (the scheme of LAPACK's
// dlatrd/dsytrd): inside a panel the reflectors v and the vectors w of the rank-2 updates
// A <- A - v w^T - w v^T are kept in LDS (panels Vp, Wp) and applied on the fly to the column being
// reduced and to the matrix-vector product (tridiag_panel_kernel, one launch per panel).  The panels then
// go to global memory and the trailing matrix gets the rank-2nb update on the matrix cores from a launch
// of its own that spreads over the whole chip (tridiag_update_kernel: computed for the lower triangle,
// stored to both, since the matrix-vector product reads whole rows): inside the panel kernel the update
// ran on one compute unit per image, 2 of its 10.7 ms per batch of 64 and of its 9.3 ms for one image.
// G is symmetric and stored in full, so the product p = A v is formed as column sums over rows,
// p_c = sum_i A[i][c] v_i: a lane owns two neighbouring columns, loads are 16 bytes wide and contiguous
// across the wavefront, and no cross-lane reduction is needed; 4 row groups x 4 column groups of
// wavefronts leave four partial sums per column, added in a fixed order (results are bit-reproducible).
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(2))) double d2;
typedef __attribute__((ext_vector_type(4))) double d4;

#ifndef TD_INFLIGHT
#define TD_INFLIGHT 12
#endif
constexpr int TD_THREADS = 1024;
constexpr int TD_WAVES = TD_THREADS / 64;
constexpr int TD_LDS_BYTES = 160 * 1024;  // LDS of one compute unit, all of it for the one workgroup

constexpr int TD_RED = 2048;              // partial column sums of the matrix-vector product

// Panel width that fits the LDS next to the current reflector and column (2 vectors of Nr doubles), the
// partial sums, the two panels (2 nb Nr doubles) and 1 KB of small scratch.
int tridiag_panel_width(int N) {
  const int Nr = round_up(N, 16);
  long nb = ((long)TD_LDS_BYTES - 1024 - TD_RED * 8 - 2L * Nr * 8) / (16L * Nr);
  nb &= ~3L;
  return nb > 32 ? 32 : (int)nb;
}
size_t tridiag_lds_bytes(int N, int nb) {
  const int Nr = round_up(N, 16);
  return (size_t)(2 * nb + 2) * Nr * 8 + TD_RED * 8 + 1024;
}

// Sum over the workgroup in a fixed order: lanes as above, wavefronts left to right.  One barrier: the caller
// must not use the same scratch array for its next sum unless another barrier lies in between (the two sums of
// a column step use two arrays).
__device__ inline double td_block_sum(double x, double* scratch, int wave, int lane) {
  x = wave_sum_dpp(x);
  if (lane == 0) scratch[wave] = x;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < TD_WAVES; k++) s += scratch[k];
  return s;
}

// One task of the rank-2nb update: trailing matrix (rows and columns jend .. N-1) <- itself - Vp Wp^T - Wp Vp^T on
// the matrix cores, for the strip of 16 rows x 64 columns (a, bch) counted from base = jend rounded down to 16;
// product ks contracts over k = 4 ks + lane / 16 of the 2 kcols columns of [Vp | Wp] (rows) against [Wp | Vp]
// (columns).  Only strips that reach the diagonal or lie below it are computed (64 bch <= 16 a + 15); a strip
// strictly below the diagonal also writes its mirror image, which is a strip that is skipped.  Vp, Wp: [Nr][nb]
// in LDS or in global memory.
__device__ inline void td_update_strip(double* __restrict__ A, int N, int Np, int Nr, int nb, int jend, int kcols,
                                       const double* Vp, const double* Wp, int a, int bch, int lane) {
  const int l15 = lane & 15, q4 = lane >> 4;
  const int base = jend & ~15;
  const int rt = base + 16 * a, ct = base + 64 * bch;
  const bool below = 64 * bch + 63 < 16 * a;
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
  const int ksteps = kcols >> 2;
  for (int half = 0; half < 2; half++) {
    const double* L = half == 0 ? Vp : Wp;   // row factor
    const double* R = half == 0 ? Wp : Vp;   // column factor
    for (int ks = 0; ks < ksteps; ks++) {
      const int k = 4 * ks + q4;
      const double av = -L[arow * nb + k];
#pragma unroll
      for (int t = 0; t < 4; t++) {
        const int crow = min(ct + 16 * t + l15, Nr - 1);
        acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, R[crow * nb + k], acc[t], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 4; t++) {
    const int cc = ct + 16 * t + l15;
#pragma unroll
    for (int e = 0; e < 4; e++) {
      const int rr = rt + 4 * e + q4;
      if (rr >= jend && cc >= jend && rr < N && cc < N) {
        A[(size_t)rr * Np + cc] = acc[t][e];
        if (below) A[(size_t)cc * Np + rr] = acc[t][e];
      }
    }
  }
}

// G      [B][Np][Np]  in: the Gram matrix, symmetric, stored in full; destroyed
// dvec   [B][Np]      out: diagonal of T
// evec   [B][Np]      out: evec[j] = T[j+1][j], j < N-1
// tauv   [B][Np]      out: tau_j (0 for a reflector that is the identity)
// Vc     [B][Np/16][Np][16] out, float: the reflectors in blocks of sixteen, Vc[j / 16][i][j % 16] = v_j[i] (zeros up to
//                     i = j, 1 at j + 1) -- the layout stage 3 copies into LDS; reflectors j >= N-1 are not written
// panels [B][2][Nr][nb] out: the panel's Vp and Wp (zero beyond the panel's columns, up to kcols) for the update
// One launch reduces the panels that start at j0, j0 + nb, ... below j0_stop.  fused != 0: the update after each
// panel runs inside the kernel, on this image's compute unit (the whole reduction in one launch: better from about
// a hundred images on, where the chip is full anyway); fused == 0: one panel per launch, the panels go to global
// memory and tridiag_update_kernel follows.
__global__ __launch_bounds__(TD_THREADS) void tridiag_panel_kernel(double* __restrict__ G, int N, int Np, int nb, int j0_first,
                                                                   int j0_stop, int fused,
                                                                   double* __restrict__ dvec, double* __restrict__ evec,
                                                                   float* __restrict__ tauv, float* __restrict__ Vc,
                                                                   double* __restrict__ panels, size_t panels_stride) {
  extern __shared__ __attribute__((aligned(16))) unsigned char td_smem[];
  const int Nr = round_up(N, 16);
  double* Vp = reinterpret_cast<double*>(td_smem);  // [Nr][nb] reflectors of the panel
  double* Wp = Vp + (size_t)Nr * nb;                 // [Nr][nb] their update vectors
  double* vs = Wp + (size_t)Nr * nb;                 // [Nr] current reflector
  double* as = vs + Nr;                              // [Nr] current column
  double* red = as + Nr;                             // [nrg][128 ncg] partial column sums of the row groups, <= 2048 in all
  double* dots = red + TD_RED;                       // [64] W^T v and V^T v
  double* wsum = dots + 64;                          // [2][16] wavefront partials of td_block_sum
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  double* A = G + (size_t)b * Np * Np;
  double* dout = dvec + (size_t)b * Np;
  double* eout = evec + (size_t)b * Np;
  float* tout = tauv + (size_t)b * Np;
  float* Vout = Vc + (size_t)b * Np * Np;
  const int l15 = lane & 15, q4 = lane >> 4;

  for (int j0 = j0_first; j0 < j0_stop; j0 += nb) {
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
      // Wavefront (rg, cg): column group cg = 128 columns (a lane owns two neighbours, one 16-byte load per row),
      // row group rg = every nrg-th row.  As the trailing matrix shrinks there are fewer column groups and more
      // row groups; up to TD_INFLIGHT rows are in flight per wavefront.
      const int r0 = j + 1;
      const int cbase = r0 & ~1;                 // column pairs start at an even column
      const int ncols = N - cbase;
      const int ncg = (ncols + 127) >> 7;        // <= 8 for N <= 1024
      const int nrg = TD_WAVES / ncg;            // >= 2
      const int pitch = ncg << 7;                // nrg * pitch <= 2048 partial sums
      if (wave < ncg * nrg) {
        const int cg = wave % ncg, rg = wave / ncg;
        const int c = cbase + (cg << 7) + 2 * lane;
        const bool ok = c < N;                   // (an odd N reads the zero padding column N as the pair's second half)
        const double* col = A + (ok ? c : cbase);
        d2 acc = d2{0.0, 0.0};
        // whole chunks of TD_INFLIGHT rows with all their loads in flight together, then chunks of 4, then single rows:
        // no row is fetched that does not count (a chunk padded with repeated rows cost up to a tenth of the kernel)
        int ib = r0 + rg;
        for (; ib + (TD_INFLIGHT - 1) * nrg < N; ib += TD_INFLIGHT * nrg) {
          d2 x[TD_INFLIGHT];
#pragma unroll
          for (int u = 0; u < TD_INFLIGHT; u++) x[u] = *reinterpret_cast<const d2*>(col + (size_t)(ib + u * nrg) * Np);
#pragma unroll
          for (int u = 0; u < TD_INFLIGHT; u++) acc += x[u] * vs[ib + u * nrg];
        }
        for (; ib + 3 * nrg < N; ib += 4 * nrg) {
          d2 x[4];
#pragma unroll
          for (int u = 0; u < 4; u++) x[u] = *reinterpret_cast<const d2*>(col + (size_t)(ib + u * nrg) * Np);
#pragma unroll
          for (int u = 0; u < 4; u++) acc += x[u] * vs[ib + u * nrg];
        }
        {
          d2 x[3];
#pragma unroll
          for (int u = 0; u < 3; u++)
            if (ib + u * nrg < N) x[u] = *reinterpret_cast<const d2*>(col + (size_t)(ib + u * nrg) * Np);  // uniform over the wavefront
#pragma unroll
          for (int u = 0; u < 3; u++)
            if (ib + u * nrg < N) acc += x[u] * vs[ib + u * nrg];
        }
        if (ok) {
          red[rg * pitch + (c - cbase)] = acc.x;
          red[rg * pitch + (c - cbase) + 1] = acc.y;
        }
      }
      // ---- W^T v and V^T v for the panel's earlier columns: one wavefront per dot product ------------------
      for (int id = wave; id < 2 * jj; id += TD_WAVES) {
        const double* P = id < jj ? Wp + id : Vp + (id - jj);
        double s = 0.0;
        for (int i = r0 + lane; i < N; i += 64) s += P[i * nb] * vs[i];
        s = wave_sum_dpp(s);
        if (lane == 0) dots[id] = s;
      }
      __syncthreads();
      // ---- p <- tau (A v - V (W^T v) - W (V^T v)),  w = p - (tau/2) (p^T v) v -------------------------------
      const int c = r0 + tid;
      double pc = 0.0, vc = 0.0;
      if (c < N) {
        for (int g = 0; g < nrg; g++) pc += red[g * pitch + (c - cbase)];  // fixed order
        for (int k = 0; k < jj; k++) pc -= Vp[c * nb + k] * dots[k] + Wp[c * nb + k] * dots[jj + k];
        pc *= tau;
        vc = vs[c];
      }
      const double pv = td_block_sum(pc * vc, wsum + TD_WAVES, wave, lane);
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
        Vout[((size_t)(j >> 4) * Np + i) * 16 + (j & 15)] = i > j ? (float)Vp[i * nb + jj] : 0.f;
    }
    if (kcols > cnt) {  // a last, shorter panel: columns cnt .. kcols-1 still hold the previous panel
      for (int e = tid; e < Nr * (kcols - cnt); e += TD_THREADS) {
        const int i = e / (kcols - cnt), k = cnt + e % (kcols - cnt);
        Vp[i * nb + k] = 0.0;
        Wp[i * nb + k] = 0.0;
      }
    }
    __syncthreads();
    if (fused) {  // strips are dealt to the wavefronts round-robin
      const int base = jend & ~15;
      const int nrt = (N - base + 15) >> 4, ncc = (N - base + 63) >> 6;
      int idx = 0;
      for (int a = 0; a < nrt; a++) {
        const int n_a = min(ncc, (a >> 2) + 1);
        for (int bch = 0; bch < n_a; bch++, idx++)
          if ((idx & (TD_WAVES - 1)) == wave) td_update_strip(A, N, Np, Nr, nb, jend, kcols, Vp, Wp, a, bch, lane);
      }
      __syncthreads();  // the rewritten matrix is visible to the whole workgroup
    } else {
      // the panels for the update of the trailing matrix (rows that the update does not store are written as zero)
      double* Vg = panels + (size_t)b * panels_stride;
      double* Wg = Vg + (size_t)Nr * nb;
      for (int e = tid; e < Nr * kcols; e += TD_THREADS) {
        const int i = e / kcols, k = e % kcols;
        Vg[i * nb + k] = (i >= jend && i < N) ? Vp[i * nb + k] : 0.0;
        Wg[i * nb + k] = (i >= jend && i < N) ? Wp[i * nb + k] : 0.0;
      }
    }
  }
  if (fused && tid == 0) {
    dout[N - 1] = A[(size_t)(N - 1) * Np + (N - 1)];
    eout[N - 1] = 0.0;
    tout[N - 1] = 0.f;
  }
}

// The update of the trailing matrix after a panel as a launch of its own: one wavefront per strip (td_update_strip),
// panels read from global memory.
__global__ __launch_bounds__(256) void tridiag_update_kernel(double* __restrict__ G, int N, int Np, int nb, int jend,
                                                             int kcols, const double* __restrict__ panels,
                                                             size_t panels_stride, int ntasks) {
  const int b = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  const int task = blockIdx.x * 4 + (tid >> 6);
  if (task >= ntasks) return;  // uniform over the wavefront; no barrier in this kernel
  const int Nr = round_up(N, 16);
  const int base = jend & ~15;
  const int ncc = (N - base + 63) >> 6;
  int a = 0, rest = task;  // row tile a has min(ncc, a / 4 + 1) strips
  for (;;) {
    const int n_a = min(ncc, (a >> 2) + 1);
    if (rest < n_a) break;
    rest -= n_a;
    a++;
  }
  const double* Vg = panels + (size_t)b * panels_stride;
  td_update_strip(G + (size_t)b * Np * Np, N, Np, Nr, nb, jend, kcols, Vg, Vg + (size_t)Nr * nb, a, rest, lane);
}

// The last diagonal entry, after the last update.
__global__ __launch_bounds__(64) void tridiag_last_kernel(const double* __restrict__ G, int N, int Np,
                                                          double* __restrict__ dvec, double* __restrict__ evec,
                                                          float* __restrict__ tauv) {
  const int b = blockIdx.x;
  if (threadIdx.x == 0) {
    dvec[(size_t)b * Np + N - 1] = G[(size_t)b * Np * Np + (size_t)(N - 1) * Np + (N - 1)];
    evec[(size_t)b * Np + N - 1] = 0.0;
    tauv[(size_t)b * Np + N - 1] = 0.f;
  }
}

int launch_tridiag(const Plan& pl, double* G, double* dvec, double* evec, float* tauv, float* Vc, double* panels,
                   size_t panels_stride, hipStream_t st) {
  const int N = pl.N, nb = tridiag_panel_width(N);
  if (nb < 4) return TC_ERR_SHAPE;
  if ((size_t)2 * round_up(N, 16) * nb > panels_stride) return TC_ERR_WORKSPACE;
  const size_t lds = tridiag_lds_bytes(N, nb);
  // more than 64 KB of dynamic LDS has to be allowed per function (a cheap host call, repeated so that it
  // holds on whichever device is current)
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(tridiag_panel_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          TD_LDS_BYTES) != hipSuccess)
    return TC_ERR_HIP;
  if (pl.batch_call >= 96) {  // the chip is full of images: the whole reduction in one launch, updates on the image's own compute unit
    TC_TIMED(PK_TRIDIAG, 0, st, (tridiag_panel_kernel<<<pl.B, TD_THREADS, lds, st>>>(G, N, pl.Np, nb, 0, N - 1, 1, dvec, evec, tauv, Vc, panels, panels_stride)));
    return check_launch();
  }
  for (int j0 = 0; j0 < N - 1; j0 += nb) {
    const int jend = j0 + nb < N - 1 ? j0 + nb : N - 1;
    const int kcols = round_up(jend - j0, 4);
    TC_TIMED(PK_TRIDIAG, 0, st, (tridiag_panel_kernel<<<pl.B, TD_THREADS, lds, st>>>(G, N, pl.Np, nb, j0, j0 + 1, 0, dvec, evec, tauv, Vc, panels, panels_stride)));
    const int base = jend & ~15;
    const int nrt = (N - base + 15) >> 4, ncc = (N - base + 63) >> 6;
    int ntasks = 0;
    for (int a = 0; a < nrt; a++) ntasks += ncc < (a >> 2) + 1 ? ncc : (a >> 2) + 1;
    TC_TIMED(PK_TRIDIAG_UPDATE, 0, st, (tridiag_update_kernel<<<dim3((ntasks + 3) / 4, pl.B), 256, 0, st>>>(G, N, pl.Np, nb, jend, kcols, panels, panels_stride, ntasks)));
  }
  TC_TIMED(PK_TRIDIAG_UPDATE, 1, st, (tridiag_last_kernel<<<pl.B, 64, 0, st>>>(G, N, pl.Np, dvec, evec, tauv)));
  return check_launch();
}

}  // namespace tc
