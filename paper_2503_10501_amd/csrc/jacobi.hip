// Batched symmetric eigensolver for the Gram matrices: two-sided block-Jacobi.
//
// G (Np x Np, Np a multiple of 64) is split into blocks of b = 32 rows/columns.  One step pairs the
// blocks by a round-robin tournament; for every pair (p,q) the 64x64 subproblem
// [[G_pp G_pq][G_qp G_qq]] is diagonalised approximately by one cyclic sweep of plane rotations held
// in LDS (jacobi_solve), giving an orthogonal 64x64 matrix R.  Then every 64x64 tile of G that the
// step's pairs (I,J) span is replaced by R_I^T G_IJ R_J and the eigenvector columns by U_J R_J
// (jacobi_update), both as small matrix products on the matrix cores.  nblk-1 steps make a sweep;
// sweeps repeat until the off-diagonal mass measured during a sweep is below the tolerance, per
// image, with the iteration count fixed on the host and converged images skipped on the device.
// On exit diag(G) holds the eigenvalues sigma_i^2 and U the left singular vectors of O
// (Section 3.3.1: Z = U Sigma V^T  =>  Z Z^T = U Sigma^2 U^T).
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(4))) double d4;
typedef __attribute__((ext_vector_type(4))) float f4;

// 16x16x4 matrix-core product for both element types.  A: lane holds A[lane%16][lane/16];
// B: lane holds B[lane/16][lane%16]; accumulator element j of a lane is C[row(j)][lane%16].
template <typename T> struct MM;
template <> struct MM<double> {
  typedef d4 acc_t;
  __device__ static inline acc_t mma(double a, double b, acc_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
  }
  __device__ static inline int row(int j, int lane) { return 4 * j + (lane >> 4); }
};
template <> struct MM<float> {
  typedef f4 acc_t;
  __device__ static inline acc_t mma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  __device__ static inline int row(int j, int lane) { return 4 * (lane >> 4) + j; }
};

constexpr int SLD = JT + 1;  // padded leading dimension of the LDS tiles

// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void jacobi_init_u(T* __restrict__ U, int Np) {
  const size_t n2 = (size_t)Np * Np;
  T* Ub = U + (size_t)blockIdx.y * n2;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += (size_t)gridDim.x * blockDim.x)
    Ub[i] = (i / Np == i % Np) ? T(1) : T(0);
}

template <typename T>
__global__ __launch_bounds__(1024) void jacobi_init_state(const T* __restrict__ G, EigState* __restrict__ state,
                                                          int Np) {
  __shared__ double red[16];
  const size_t n2 = (size_t)Np * Np;
  const T* Gb = G + (size_t)blockIdx.x * n2;
  double s = 0.0;
  for (size_t i = threadIdx.x; i < n2; i += 1024) { double v = (double)Gb[i]; s += v * v; }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int i = 0; i < 16; i++) tot += red[i];
    state[blockIdx.x].norm2 = tot;
    state[blockIdx.x].done = tot > 0.0 ? 0 : 1;
    state[blockIdx.x].sweeps = 0;
  }
}

// ---------------------------------------------------------------------------------------
// One workgroup per block pair: load the 64x64 subproblem, one cyclic sweep of rotations, emit R.
template <typename T>
__global__ __launch_bounds__(256) void jacobi_solve(const T* __restrict__ G, T* __restrict__ R,
                                                    double* __restrict__ offpart, const EigState* __restrict__ state,
                                                    int Np, int nblk, int step) {
  const int b = blockIdx.y, pair = blockIdx.x, P = nblk / 2;
  if (state[b].done) return;
  __shared__ T S[JT][SLD];
  __shared__ T Rm[JT][SLD];
  __shared__ T rc[JB], rs[JB];
  __shared__ int ri[JB], rj[JB];
  __shared__ double red[4];
  int p, q;
  round_robin_pair(nblk, step, pair, &p, &q);
  const T* Gb = G + (size_t)b * Np * Np;
  const int tid = threadIdx.x;
  {
    const int c = tid & 63, gc = (c < JB ? p * JB + c : q * JB + c - JB);
    double off = 0.0;
    for (int r = tid >> 6; r < JT; r += 4) {
      const int gr = (r < JB ? p * JB + r : q * JB + r - JB);
      const T v = Gb[(size_t)gr * Np + gc];
      S[r][c] = v;
      Rm[r][c] = (r == c) ? T(1) : T(0);
      const double dv = (double)v;
      if ((r < JB) != (c < JB)) off += dv * dv;                       // the G_pq / G_qp blocks
      else if (r != c) off += dv * dv / (double)(nblk - 1);           // inside G_pp, G_qq (seen nblk-1 times)
    }
    off = wave_sum(off);
    if ((tid & 63) == 0) red[tid >> 6] = off;
  }
  __syncthreads();
  if (tid == 0) offpart[((size_t)b * (nblk - 1) + step) * P + pair] = red[0] + red[1] + red[2] + red[3];

  for (int st = 0; st < JT - 1; st++) {
    if (tid < JB) {
      int i, j;
      round_robin_pair(JT, st, tid, &i, &j);
      const T aii = S[i][i], ajj = S[j][j], aij = S[i][j];
      T c = T(1), s = T(0);
      if (aij != T(0)) {
        const T zeta = (ajj - aii) / (T(2) * aij);
        const T az = fabs(zeta);
        T t = T(1) / (az + sqrt(T(1) + az * az));  // az = inf gives t = 0
        if (!(az < T(1e150))) t = T(0);            // also catches NaN
        if (zeta < T(0)) t = -t;
        c = T(1) / sqrt(T(1) + t * t);
        s = c * t;
      }
      rc[tid] = c; rs[tid] = s; ri[tid] = i; rj[tid] = j;
    }
    __syncthreads();
    // S <- J^T S J on 2x2 blocks (rows of pair I) x (columns of pair J); R <- R J
    {
      const int J = tid & 31;
      const int jc0 = ri[J], jc1 = rj[J];
      const T cJ = rc[J], sJ = rs[J];
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int I = (tid >> 5) + 8 * u;
        const int ir0 = ri[I], ir1 = rj[I];
        const T cI = rc[I], sI = rs[I];
        const T a = S[ir0][jc0], bb = S[ir0][jc1], cc = S[ir1][jc0], d = S[ir1][jc1];
        const T a1 = cI * a - sI * cc, b1 = cI * bb - sI * d, c1 = sI * a + cI * cc, d1 = sI * bb + cI * d;
        S[ir0][jc0] = cJ * a1 - sJ * b1;
        S[ir0][jc1] = sJ * a1 + cJ * b1;
        S[ir1][jc0] = cJ * c1 - sJ * d1;
        S[ir1][jc1] = sJ * c1 + cJ * d1;
      }
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int r = (tid >> 5) + 8 * u;
        const T x = Rm[r][jc0], y = Rm[r][jc1];
        Rm[r][jc0] = cJ * x - sJ * y;
        Rm[r][jc1] = sJ * x + cJ * y;
      }
    }
    __syncthreads();
  }
  T* Rb = R + ((size_t)b * P + pair) * JT * JT;
  for (int e = tid; e < JT * JT; e += 256) Rb[e] = Rm[e >> 6][e & 63];
}

// ---------------------------------------------------------------------------------------
// Tile update.  blockIdx.x < P*P: tile (I,J) of G becomes R_I^T G_IJ R_J.  The remaining
// (Np/64)*P workgroups update a 64-row slab of U's columns of pair J: U_J <- U_J R_J.
template <typename T>
__global__ __launch_bounds__(256) void jacobi_update(T* __restrict__ G, T* __restrict__ U, const T* __restrict__ R,
                                                     const EigState* __restrict__ state, int Np, int nblk, int step) {
  typedef typename MM<T>::acc_t acc_t;
  const int b = blockIdx.y, P = nblk / 2;
  if (state[b].done) return;
  __shared__ T X[JT][SLD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const bool isG = (int)blockIdx.x < P * P;
  int I, J;
  T* M;
  int rowbase[2];  // global row of local rows 0..31 and 32..63
  if (isG) {
    I = blockIdx.x / P; J = blockIdx.x % P;
    M = G + (size_t)b * Np * Np;
    int p, q;
    round_robin_pair(nblk, step, I, &p, &q);
    rowbase[0] = p * JB; rowbase[1] = q * JB;
  } else {
    const int t = blockIdx.x - P * P;
    I = -1; J = t % P;
    M = U + (size_t)b * Np * Np;
    rowbase[0] = (t / P) * JT; rowbase[1] = rowbase[0] + JB;
  }
  int colbase[2];
  {
    int p, q;
    round_robin_pair(nblk, step, J, &p, &q);
    colbase[0] = p * JB; colbase[1] = q * JB;
  }
  const T* RJ = R + ((size_t)b * P + J) * JT * JT;
  // Right factor as matrix-core B fragments kept in registers: this wave needs R_J[:, wc*32 .. +32).
  T rjf[16][2];
#pragma unroll
  for (int ks = 0; ks < 16; ks++) {
    const int k = 4 * ks + (lane >> 4);
    rjf[ks][0] = RJ[k * JT + wc * 32 + (lane & 15)];
    rjf[ks][1] = RJ[k * JT + wc * 32 + 16 + (lane & 15)];
  }
  // Left factor R_I^T as A fragments: A[i][k] = R_I[k][i], rows i in wr*32 .. +32.
  T rif[16][2];
  if (isG) {
    const T* RI = R + ((size_t)b * P + I) * JT * JT;
#pragma unroll
    for (int ks = 0; ks < 16; ks++) {
      const int k = 4 * ks + (lane >> 4);
      rif[ks][0] = RI[k * JT + wr * 32 + (lane & 15)];
      rif[ks][1] = RI[k * JT + wr * 32 + 16 + (lane & 15)];
    }
  }
  // Gather the tile: lanes 0..15 read 16 consecutive columns of one row.
  {
    const int c = (lane & 15) + 16 * wave;
    const int gc = colbase[c >> 5] + (c & 31);
#pragma unroll
    for (int it = 0; it < 16; it++) {
      const int r = (lane >> 4) + 4 * it;
      X[r][c] = M[(size_t)(rowbase[r >> 5] + (r & 31)) * Np + gc];
    }
  }
  __syncthreads();
  acc_t acc[2][2];
  if (isG) {
    // W = R_I^T X
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++) acc[i][j] = acc_t{0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < 16; ks++) {
      const int k = 4 * ks + (lane >> 4);
      const T b0 = X[k][wc * 32 + (lane & 15)], b1 = X[k][wc * 32 + 16 + (lane & 15)];
      acc[0][0] = MM<T>::mma(rif[ks][0], b0, acc[0][0]);
      acc[0][1] = MM<T>::mma(rif[ks][0], b1, acc[0][1]);
      acc[1][0] = MM<T>::mma(rif[ks][1], b0, acc[1][0]);
      acc[1][1] = MM<T>::mma(rif[ks][1], b1, acc[1][1]);
    }
    __syncthreads();  // every wave has finished reading X
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int nt = 0; nt < 2; nt++)
#pragma unroll
        for (int j = 0; j < 4; j++)
          X[wr * 32 + mt * 16 + MM<T>::row(j, lane)][wc * 32 + nt * 16 + (lane & 15)] = acc[mt][nt][j];
    __syncthreads();
  }
  // Y = X R_J
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) acc[i][j] = acc_t{0, 0, 0, 0};
#pragma unroll
  for (int ks = 0; ks < 16; ks++) {
    const int k = 4 * ks + (lane >> 4);
    const T a0 = X[wr * 32 + (lane & 15)][k], a1 = X[wr * 32 + 16 + (lane & 15)][k];
    acc[0][0] = MM<T>::mma(a0, rjf[ks][0], acc[0][0]);
    acc[0][1] = MM<T>::mma(a0, rjf[ks][1], acc[0][1]);
    acc[1][0] = MM<T>::mma(a1, rjf[ks][0], acc[1][0]);
    acc[1][1] = MM<T>::mma(a1, rjf[ks][1], acc[1][1]);
  }
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int r = wr * 32 + mt * 16 + MM<T>::row(j, lane);
        const int c = wc * 32 + nt * 16 + (lane & 15);
        M[(size_t)(rowbase[r >> 5] + (r & 31)) * Np + colbase[c >> 5] + (c & 31)] = acc[mt][nt][j];
      }
}

// ---------------------------------------------------------------------------------------
__global__ void jacobi_sweep_end(const double* __restrict__ offpart, EigState* __restrict__ state, int count,
                                 double tol, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B || state[b].done) return;
  const double* op = offpart + (size_t)b * count;
  double s = 0.0;
  for (int i = 0; i < count; i++) s += op[i];  // fixed order: the decision is reproducible
  state[b].sweeps += 1;
  if (s <= tol * tol * state[b].norm2) state[b].done = 1;
}

template <typename T>
static int run_jacobi(const Plan& pl, T* G, T* U, T* R, double* offpart, EigState* state, hipStream_t st) {
  const int Np = pl.Np, nblk = pl.nblk, P = pl.P;
  TC_TIMED(PK_JINIT, 0, st, (jacobi_init_u<T><<<dim3(Np * Np / 1024 > 0 ? Np * Np / 1024 : 1, pl.B), 256, 0, st>>>(U, Np)));
  TC_TIMED(PK_JINIT, 1, st, (jacobi_init_state<T><<<pl.B, 1024, 0, st>>>(G, state, Np)));
  const dim3 gs(P, pl.B), gu(P * P + (Np / JT) * P, pl.B);
  for (int sweep = 0; sweep < pl.max_sweeps; sweep++) {
    for (int step = 0; step < pl.steps; step++) {
      TC_TIMED(PK_JSOLVE, sweep, st, (jacobi_solve<T><<<gs, 256, 0, st>>>(G, R, offpart, state, Np, nblk, step)));
      TC_TIMED(PK_JUPDATE, sweep, st, (jacobi_update<T><<<gu, 256, 0, st>>>(G, U, R, state, Np, nblk, step)));
    }
    TC_TIMED(PK_JSWEEPEND, sweep, st, (jacobi_sweep_end<<<(pl.B + 63) / 64, 64, 0, st>>>(offpart, state, P * pl.steps, pl.tol, pl.B)));
  }
  return check_launch();
}

int launch_jacobi(const Plan& pl, int eig_dtype, void* G, void* U, void* R, double* offpart, EigState* state,
                  hipStream_t st) {
  if (eig_dtype == TC_EIG_F64) return run_jacobi<double>(pl, (double*)G, (double*)U, (double*)R, offpart, state, st);
  return run_jacobi<float>(pl, (float*)G, (float*)U, (float*)R, offpart, state, st);
}

}  // namespace tc
