// Direct symmetric eigensolver, stage 1: reduction of the Gram matrix to tridiagonal form,
//     G = Q T Q^T,   Q = H_0 H_1 ... H_{N-3},   H_j = I - tau_j v_j v_j^T  (Householder reflectors),
// so that the singular vectors of Section 3.3.1 (Z = U Sigma V^T, Z Z^T = U Sigma^2 U^T) become
// U = Q W with T W = W Sigma^2 (stages 2 and 3: tdeig.hip).
//
// The columns of an image are reduced by one workgroup of 16 wavefronts.  The reduction is bound by
// memory: column j needs the product of the trailing (N-j-1)^2 matrix with v_j.  Measured on MI355X a
// single workgroup streams 110 to 150 GB/s out of its L2 and 64 of them together 5 to 6 TB/s, which is what
// the fabric delivers to any number of compute units for a working set of this size, so one compute unit
// per image is enough for the products at batch 64.
//
// The trailing matrix is only rewritten once per panel of nb columns (the scheme of LAPACK's
// dlatrd/dsytrd): inside a panel the reflectors v and the vectors w of the rank-2 updates
// A <- A - v w^T - w v^T are kept in LDS (panels Vp, Wp) and applied on the fly to the column being
// reduced and to the matrix-vector product (tridiag_panel_kernel, one launch per panel).  The panels then
// go to global memory and the trailing matrix gets the rank-2nb update on the matrix cores from a launch
// of its own that spreads over the whole chip (tridiag_update_kernel: computed for the lower triangle,
// stored to both): inside the panel kernel the update ran on one compute unit per image, 2 of its 10.7 ms
// per batch of 64 and of its 9.3 ms for one image.
//
// G is symmetric and stored in full.  The product p = A v reads 128-column groups of rows (a lane owns two
// neighbouring columns, loads are 16 bytes wide and contiguous across the wavefront).  Inside the diagonal
// block of a column group both triangles are read and a row only adds to the column sums
// p_c += A[r][c] v_r, which need no exchange between lanes; a row below the block is fetched once and used
// twice, for the column sums and for its own row sum sum_c A[r][c] v_c over the group's columns (the mirror
// image above the diagonal is never read), added up over the lanes eight rows at a time.  That is 0.58 of
// the elements of the full trailing matrices at 576 tokens.  The 16 wavefronts are dealt to the column
// groups in proportion to their rows (tridiag_table_kernel); every partial sum has one writer and the sums
// are added in a fixed order (results are bit-reproducible).
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(2))) double d2;
typedef __attribute__((ext_vector_type(4))) double d4;

constexpr int TD_THREADS = 1024;
constexpr int TD_WAVES = TD_THREADS / 64;
constexpr int TD_LDS_BYTES = 160 * 1024;  // LDS of one compute unit, all of it for the one workgroup

constexpr int TD_RED = 2048;              // partial column sums of the matrix-vector product
constexpr int TD_TAB = 24;                // ints per column in the table of wavefront assignments

// Row sums of the matrix-vector product (the part of a row left of its diagonal block): one double per row and
// column group, at most sum_k max(0, Nr - 128 k), k >= 1.
__host__ __device__ inline int tridiag_rowsum_len(int Nr) {
  int n = 0;
  for (int k = 128; k < Nr; k += 128) n += Nr - k;
  return n;
}

// Panel width that fits the LDS next to the current reflector and column (2 vectors of Nr doubles), the
// partial sums of the matrix-vector product (columns and rows), the two panels (2 nb Nr doubles) and 1 KB of small scratch.
int tridiag_panel_width(int N) {
  const int Nr = round_up(N, 16);
  long nb = ((long)TD_LDS_BYTES - 1024 - TD_RED * 8 - 2L * Nr * 8 - 8L * tridiag_rowsum_len(Nr)) / (16L * Nr);
  nb &= ~3L;
  return nb > 32 ? 32 : (int)nb;
}
size_t tridiag_lds_bytes(int N, int nb) {
  const int Nr = round_up(N, 16);
  return (size_t)(2 * nb + 2) * Nr * 8 + TD_RED * 8 + (size_t)tridiag_rowsum_len(Nr) * 8 + 1024;
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

// Totals over the 64 lanes of eight values at once (recursive halving, fixed order): lane L returns the total of
// part[L / 8].  The halves of the wavefront and the rows of 16 lanes trade registers with the swap instructions,
// lanes L and L^8 through a rotation of the row, the last eight lanes through quad and half-row permutations.
__device__ inline double td_sum8(const double* part, int lane) {
  typedef __attribute__((ext_vector_type(2))) unsigned int u2;
  double q[4], s[2];
#pragma unroll
  for (int u = 0; u < 4; u++) {  // lanes < 32: part[u] of L and L+32; lanes >= 32: part[u + 4]
    const u2 lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(part[u]), (unsigned)__double2loint(part[u + 4]), false, false);
    const u2 hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(part[u]), (unsigned)__double2hiint(part[u + 4]), false, false);
    q[u] = __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
  }
#pragma unroll
  for (int u = 0; u < 2; u++) {  // even rows of 16 lanes: q[u] of L and L+16; odd rows: q[u + 2]
    const u2 lo = __builtin_amdgcn_permlane16_swap((unsigned)__double2loint(q[u]), (unsigned)__double2loint(q[u + 2]), false, false);
    const u2 hi = __builtin_amdgcn_permlane16_swap((unsigned)__double2hiint(q[u]), (unsigned)__double2hiint(q[u + 2]), false, false);
    s[u] = __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
  }
  const bool up = (lane & 8) != 0;
  double t = (up ? s[1] : s[0]) + dpp_f64<0x128>(up ? s[0] : s[1]);  // row_ror:8, L <-> L^8
  t += dpp_f64<0xB1>(t);   // quad_perm [1,0,3,2]
  t += dpp_f64<0x4E>(t);   // quad_perm [2,3,0,1]
  t += dpp_f64<0x141>(t);  // row_half_mirror
  return t;
}

// Which wavefront works on which part of the matrix-vector product of column j: column group g (128 columns from
// cbase + 128 g) takes the rows from its diagonal block down, R_g of them, and the 16 wavefronts are dealt so that
// the largest R_g / n_g is as small as it can be.  tab[j][w] = g | rg << 4 | n_g << 12 for wavefront w (row group
// rg of n_g), tab[j][16 + g] = first wavefront of g | n_g << 8.
__global__ __launch_bounds__(256) void tridiag_table_kernel(int N, int* __restrict__ tab) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= N - 1) return;
  const int r0 = j + 1, cbase = r0 & ~1;
  const int ncg = (N - cbase + 127) >> 7;
  int R[8], n[8];
  for (int g = 0; g < 8; g++) {
    R[g] = g < ncg ? N - max(cbase + 128 * g, r0) : 0;
    n[g] = g < ncg ? 1 : 0;
  }
  for (int k = ncg; k < TD_WAVES; k++) {
    int best = 0;
    for (int g = 1; g < ncg; g++)
      if (R[g] * n[best] > R[best] * n[g]) best = g;
    n[best]++;
  }
  int* row = tab + (size_t)j * TD_TAB;
  int w = 0;
  for (int g = 0; g < 8; g++) {
    row[16 + g] = w | (n[g] << 8);
    for (int rg = 0; rg < n[g]; rg++) row[w++] = g | (rg << 4) | (n[g] << 12);
  }
}

// One task of the rank-2nb update: trailing matrix (rows and columns jend .. N-1) <- itself - Vp Wp^T - Wp Vp^T on
// the matrix cores, for the strip of 16 rows x 64 columns (a, bch) counted from base = jend rounded down to 16;
// product ks contracts over k = 4 ks + lane / 16 of the 2 kcols columns of [Vp | Wp] (rows) against [Wp | Vp]
// (columns).  Only strips that reach the diagonal or lie below it are computed (64 bch <= 16 a + 15); a strip
// strictly below the diagonal also writes its mirror image (in a strip that is skipped) where somebody reads it:
// within 128 columns of the diagonal (the diagonal blocks of the matrix-vector product) and in the rows of the next
// panel (a column is formed from its row).  Vp, Wp: [Nr][nb] in LDS or in global memory.
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
        if (below && (rr - cc < 128 || cc < jend + nb)) A[(size_t)cc * Np + rr] = acc[t][e];
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
                                                                   double* __restrict__ panels, size_t panels_stride,
                                                                   const int* __restrict__ tab) {
  extern __shared__ __attribute__((aligned(16))) unsigned char td_smem[];
  const int Nr = round_up(N, 16);
  double* Vp = reinterpret_cast<double*>(td_smem);  // [Nr][nb] reflectors of the panel
  double* Wp = Vp + (size_t)Nr * nb;                 // [Nr][nb] their update vectors
  double* vs = Wp + (size_t)Nr * nb;                 // [Nr] current reflector
  double* as = vs + Nr;                              // [Nr] current column
  double* red = as + Nr;                             // [16][128] partial column sums, one set per wavefront
  double* yrow = red + TD_RED;                       // row sums left of the diagonal blocks, per column group
  double* dots = yrow + tridiag_rowsum_len(Nr);      // [64] W^T v and V^T v
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
      // this column's table entries, asked for early: the wavefront's task and, for the thread's own element of p,
      // the wavefronts of its column group
      const int* trow = tab + (size_t)j * TD_TAB;
      const int ent = trow[wave];
      const int cbase = (j + 1) & ~1;            // column pairs start at an even column
      const int ent_c = (j + 1 + tid < N) ? trow[16 + ((j + 1 + tid - cbase) >> 7)] : 0;
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
      // ---- p = A v over the trailing matrix (rows and columns j+1 .. N-1) -----------------------------------
      // The matrix is symmetric and stored in full; an element below the diagonal blocks is fetched once and used
      // twice.  Column group g = 128 columns from cbase + 128 g (a lane owns two neighbours, one 16-byte load per
      // row).  Its rows run from the top of its diagonal block down: inside the block (128 rows, both triangles)
      // a row only adds to the column sums p_c += A[r][c] v_r; a row r below the block also gives the part of p_r
      // that lies in these columns, sum_c A[r][c] v_c, summed over the lanes eight rows at a time.  The rows of a
      // group are dealt to its wavefronts in turn (table: more wavefronts for the groups with more rows).
      const int r0 = j + 1;
      {
        const int cg = ent & 15, rg = (ent >> 4) & 255, nrg = ent >> 12;
        const int C0 = cbase + (cg << 7);
        const int c = C0 + 2 * lane;
        const bool ok = c < N;                   // (an odd N reads the zero padding column N as the pair's second half)
        const double* col = A + (ok ? c : cbase);
        const double vc0 = (ok && c >= r0) ? vs[c] : 0.0, vc1 = (c + 1 < N) ? vs[c + 1] : 0.0;
        const int dend = min(C0 + 128, N);       // rows below dend lie under the diagonal block
        int yoff = 0;                            // where this group's row sums start
        for (int g = 0; g < cg; g++) yoff += N - (cbase + 128 * g + 128);
        d2 acc = d2{0.0, 0.0};
        // Chunks of eight rows with all their loads in flight together, then a last chunk of fewer rows fetched four
        // at a time: no row is fetched that does not count.  A chunk that reaches below the diagonal block also
        // forms the row sums of its rows there.
        double* yg = yrow + yoff - (C0 + 128);
        int ib = max(C0, r0) + rg;
        for (; ib + 7 * nrg < N; ib += 8 * nrg) {
          d2 x[8];
#pragma unroll
          for (int u = 0; u < 8; u++) x[u] = *reinterpret_cast<const d2*>(col + (size_t)(ib + u * nrg) * Np);
#pragma unroll
          for (int u = 0; u < 8; u++) acc += x[u] * vs[ib + u * nrg];
          if (ib >= dend) {  // all eight rows below the block (uniform over the wavefront)
            double part[8];
#pragma unroll
            for (int u = 0; u < 8; u++) part[u] = x[u].x * vc0 + x[u].y * vc1;
            const double tot = td_sum8(part, lane);
            if ((lane & 7) == 0) yg[ib + (lane >> 3) * nrg] = tot;
          } else if (ib + 7 * nrg >= dend) {  // some of them
            double part[8];
#pragma unroll
            for (int u = 0; u < 8; u++) part[u] = ib + u * nrg >= dend ? x[u].x * vc0 + x[u].y * vc1 : 0.0;
            const double tot = td_sum8(part, lane);
            const int r = ib + (lane >> 3) * nrg;
            if ((lane & 7) == 0 && r >= dend) yg[r] = tot;
          }
        }
        if (ib < N) {
          double part[8];
#pragma unroll
          for (int h = 0; h < 2; h++) {
            d2 x[4];
#pragma unroll
            for (int u = 0; u < 4; u++)
              if (ib + (4 * h + u) * nrg < N) x[u] = *reinterpret_cast<const d2*>(col + (size_t)(ib + (4 * h + u) * nrg) * Np);  // uniform over the wavefront
#pragma unroll
            for (int u = 0; u < 4; u++) {
              const int r = ib + (4 * h + u) * nrg;
              part[4 * h + u] = 0.0;
              if (r < N) {
                acc += x[u] * vs[r];
                if (r >= dend) part[4 * h + u] = x[u].x * vc0 + x[u].y * vc1;
              }
            }
          }
          const double tot = td_sum8(part, lane);
          const int r = ib + (lane >> 3) * nrg;
          if ((lane & 7) == 0 && r >= dend && r < N) yg[r] = tot;
        }
        red[(wave << 7) + 2 * lane] = acc.x;
        red[(wave << 7) + 2 * lane + 1] = acc.y;
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
        const int cgc = (c - cbase) >> 7;
        const int w0 = ent_c & 255, w1 = w0 + (ent_c >> 8), cl = c - cbase - (cgc << 7);
        for (int w = w0; w < w1; w++) pc += red[(w << 7) + cl];  // fixed order: the wavefronts of the column's group,
        int yoff = 0;                                            // then the row sums of the groups to its left
        for (int g = 0; g < cgc; g++) {
          const int top = cbase + 128 * g + 128;
          pc += yrow[yoff + (c - top)];
          yoff += N - top;
        }
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
    // the reflectors leave as float rows (stage 3 applies them in float32), four columns per 16-byte store: j0 is a
    // multiple of 4, so the four lie in one block of sixteen; slots of a last group past column jend - 1 get zeros
    // (stage 3 does not use them)
    for (int g4 = 0; g4 < kcols; g4 += 4) {
      const int j = j0 + g4;
      for (int i = tid; i < N; i += TD_THREADS) {
        float4 v;
        v.x = (g4 < cnt && i > j) ? (float)Vp[i * nb + g4] : 0.f;
        v.y = (g4 + 1 < cnt && i > j + 1) ? (float)Vp[i * nb + g4 + 1] : 0.f;
        v.z = (g4 + 2 < cnt && i > j + 2) ? (float)Vp[i * nb + g4 + 2] : 0.f;
        v.w = (g4 + 3 < cnt && i > j + 3) ? (float)Vp[i * nb + g4 + 3] : 0.f;
        *reinterpret_cast<float4*>(&Vout[((size_t)(j >> 4) * Np + i) * 16 + (j & 15)]) = v;
      }
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
      // (the update reads rows from jend rounded down to 16 on; sixteen lanes per row, no index divisions)
      for (int k = tid & 15; k < kcols; k += 16)
        for (int i = (jend & ~15) + (tid >> 4); i < Nr; i += TD_THREADS / 16) {
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
                   size_t panels_stride, int* tab, hipStream_t st) {
  const int N = pl.N, nb = tridiag_panel_width(N);
  if (nb < 4) return TC_ERR_SHAPE;
  if ((size_t)2 * round_up(N, 16) * nb > panels_stride) return TC_ERR_WORKSPACE;
  const size_t lds = tridiag_lds_bytes(N, nb);
  // more than 64 KB of dynamic LDS has to be allowed per function (a cheap host call, repeated so that it
  // holds on whichever device is current)
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(tridiag_panel_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          TD_LDS_BYTES) != hipSuccess)
    return TC_ERR_HIP;
  TC_TIMED(PK_TRIDIAG_UPDATE, 2, st, (tridiag_table_kernel<<<(N + 255) / 256, 256, 0, st>>>(N, tab)));
  if (pl.batch_call >= 96) {  // the chip is full of images: the whole reduction in one launch, updates on the image's own compute unit
    TC_TIMED(PK_TRIDIAG, 0, st, (tridiag_panel_kernel<<<pl.B, TD_THREADS, lds, st>>>(G, N, pl.Np, nb, 0, N - 1, 1, dvec, evec, tauv, Vc, panels, panels_stride, tab)));
    return check_launch();
  }
  for (int j0 = 0; j0 < N - 1; j0 += nb) {
    const int jend = j0 + nb < N - 1 ? j0 + nb : N - 1;
    const int kcols = round_up(jend - j0, 4);
    TC_TIMED(PK_TRIDIAG, 0, st, (tridiag_panel_kernel<<<pl.B, TD_THREADS, lds, st>>>(G, N, pl.Np, nb, j0, j0 + 1, 0, dvec, evec, tauv, Vc, panels, panels_stride, tab)));
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
