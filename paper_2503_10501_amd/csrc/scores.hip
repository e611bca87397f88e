// Information contribution score (Eq. 3-6) from the eigen-decomposition of the Gram matrix, and
// the combined IPGS score (Eq. 3-8).
#include "tc_internal.h"

namespace tc {

// sigma_i = sqrt(max(lambda_i, 0)) from diag(G); optional descending copy and the sweep count.
template <typename T>
__global__ __launch_bounds__(256) void sigma_kernel(const T* __restrict__ G, const EigState* __restrict__ state,
                                                    double* __restrict__ sig, float* __restrict__ sigma_out,
                                                    int32_t* __restrict__ info_out, int N, int Np) {
  extern __shared__ float key[];  // pow2 >= Np floats, only when sigma_out != nullptr
  const int b = blockIdx.x, tid = threadIdx.x;
  const T* Gb = G + (size_t)b * Np * Np;
  double* sb = sig + (size_t)b * Np;
  for (int i = tid; i < Np; i += 256) {
    const double lam = (double)Gb[(size_t)i * Np + i];
    sb[i] = lam > 0.0 ? sqrt(lam) : 0.0;
  }
  if (tid == 0 && info_out) {  // > 0: converged (an all-zero matrix needs no sweep and reports 1); < 0: not converged
    const int sw = state[b].sweeps > 0 ? state[b].sweeps : 1;
    info_out[b] = state[b].done ? sw : -sw;
  }
  if (!sigma_out) return;
  int n2 = 1;
  while (n2 < Np) n2 <<= 1;
  __syncthreads();
  // the Np - N padded directions carry sigma = 0 and sort to the end
  for (int i = tid; i < n2; i += 256) key[i] = i < Np ? (float)sb[i] : -1.0f;
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

// C(x) = sum_i |U[x][i]| sigma_i (Eq. 3-6), one wavefront per token, float64 accumulation.
__global__ __launch_bounds__(256) void ics_kernel(const float* __restrict__ U, const double* __restrict__ sig,
                                                  float sv_rtol, float* __restrict__ C, float* __restrict__ C_out,
                                                  int N, int Np) {
  __shared__ double smax[4];
  const int b = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const double* sb = sig + (size_t)b * Np;
  double thr = -1.0;
  if (sv_rtol > 0.f) {  // uniform branch
    double mx = 0.0;
    for (int i = threadIdx.x; i < Np; i += 256) mx = fmax(mx, sb[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o, 64));
    if (lane == 0) smax[wave] = mx;
    __syncthreads();
    thr = (double)sv_rtol * fmax(fmax(smax[0], smax[1]), fmax(smax[2], smax[3]));
  }
  const int x = blockIdx.x * 4 + wave;
  if (x >= N) return;
  const float* Ub = U + (size_t)b * Np * Np;  // stored by block columns
  double acc = 0.0;
  for (int i = lane; i < Np; i += 64) {
    const double s = sb[i];
    if (s > thr) acc += fabs((double)Ub[u_index(x, i, Np)]) * s;
  }
  acc = wave_sum(acc);
  if (lane == 0) {
    C[(size_t)b * N + x] = (float)acc;
    if (C_out) C_out[(size_t)b * N + x] = (float)acc;
  }
}

// E = (1-lambda) n(C) + lambda n(S), n = identity or min-max over the image's tokens.
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ C, const float* __restrict__ S,
                                                      float lambda, int norm_mode, float* __restrict__ E, int N) {
  __shared__ float red[4][4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* Cb = C + (size_t)b * N;
  const float* Sb = S ? S + (size_t)b * N : nullptr;
  float cmin = INFINITY, cmax = -INFINITY, smin = INFINITY, smax = -INFINITY;
  if (norm_mode == TC_NORM_MINMAX) {
    for (int i = tid; i < N; i += 256) {
      const float c = Cb[i], s = Sb ? Sb[i] : 0.f;
      cmin = fminf(cmin, c); cmax = fmaxf(cmax, c); smin = fminf(smin, s); smax = fmaxf(smax, s);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      cmin = fminf(cmin, __shfl_xor(cmin, o, 64)); cmax = fmaxf(cmax, __shfl_xor(cmax, o, 64));
      smin = fminf(smin, __shfl_xor(smin, o, 64)); smax = fmaxf(smax, __shfl_xor(smax, o, 64));
    }
    if (lane == 0) { red[wave][0] = cmin; red[wave][1] = cmax; red[wave][2] = smin; red[wave][3] = smax; }
    __syncthreads();
    cmin = fminf(fminf(red[0][0], red[1][0]), fminf(red[2][0], red[3][0]));
    cmax = fmaxf(fmaxf(red[0][1], red[1][1]), fmaxf(red[2][1], red[3][1]));
    smin = fminf(fminf(red[0][2], red[1][2]), fminf(red[2][2], red[3][2]));
    smax = fmaxf(fmaxf(red[0][3], red[1][3]), fmaxf(red[2][3], red[3][3]));
  }
  for (int i = tid; i < N; i += 256) {
    double c = Cb[i], s = Sb ? Sb[i] : 0.f;
    if (norm_mode == TC_NORM_MINMAX) {
      c = cmax > cmin ? (c - (double)cmin) / ((double)cmax - (double)cmin) : 0.0;
      s = smax > smin ? (s - (double)smin) / ((double)smax - (double)smin) : 0.0;
    }
    E[(size_t)b * N + i] = (float)((1.0 - (double)lambda) * c + (double)lambda * s);
  }
}

template <typename T>
static int run_scores(const Plan& pl, const T* G, const float* U, const EigState* state, const float* S, float lambda,
                      int norm_mode, float sv_rtol, double* sig, float* C_ws, float* E, float* C_out, float* sigma_out,
                      int32_t* info_out, hipStream_t st) {
  int n2 = 1;
  while (n2 < pl.Np) n2 <<= 1;
  TC_TIMED(PK_SIGMA, 0, st, (sigma_kernel<T><<<pl.B, 256, sigma_out ? n2 * sizeof(float) : 0, st>>>(G, state, sig, sigma_out, info_out, pl.N, pl.Np)));
  TC_TIMED(PK_ICS, 0, st, (ics_kernel<<<dim3((pl.N + 3) / 4, pl.B), 256, 0, st>>>(U, sig, sv_rtol, C_ws, C_out, pl.N, pl.Np)));
  TC_TIMED(PK_COMBINE, 0, st, (combine_kernel<<<pl.B, 256, 0, st>>>(C_ws, S, lambda, norm_mode, E, pl.N)));
  return check_launch();
}

int launch_combine(const Plan& pl, const float* C_ws, const float* S, float lambda, int norm_mode, float* E, hipStream_t st) {
  TC_TIMED(PK_COMBINE, 0, st, (combine_kernel<<<pl.B, 256, 0, st>>>(C_ws, S, lambda, norm_mode, E, pl.N)));
  return check_launch();
}

// Singular values only (no eigenvectors): sqrt of the eigenvalues into sig_ws, optional sorted copy and sweep count.
int launch_sigma(const Plan& pl, int eig_dtype, const void* G, const EigState* state, double* sig_ws, float* sigma_out,
                 int32_t* info_out, hipStream_t st) {
  int n2 = 1;
  while (n2 < pl.Np) n2 <<= 1;
  const size_t shm = sigma_out ? n2 * sizeof(float) : 0;
  if (eig_dtype == TC_EIG_F64)
    sigma_kernel<double><<<pl.B, 256, shm, st>>>((const double*)G, state, sig_ws, sigma_out, info_out, pl.N, pl.Np);
  else
    sigma_kernel<float><<<pl.B, 256, shm, st>>>((const float*)G, state, sig_ws, sigma_out, info_out, pl.N, pl.Np);
  return check_launch();
}

int launch_scores(const Plan& pl, int eig_dtype, const void* G, const void* U, const EigState* state, const float* S,
                  float lambda, int norm_mode, float sv_rtol, void* sig_ws, float* C_ws, float* E, float* C_out,
                  float* sigma_out, int32_t* info_out, hipStream_t st) {
  if (eig_dtype == TC_EIG_F64)
    return run_scores<double>(pl, (const double*)G, (const float*)U, state, S, lambda, norm_mode, sv_rtol,
                              (double*)sig_ws, C_ws, E, C_out, sigma_out, info_out, st);
  return run_scores<float>(pl, (const float*)G, (const float*)U, state, S, lambda, norm_mode, sv_rtol, (double*)sig_ws,
                           C_ws, E, C_out, sigma_out, info_out, st);
}

}  // namespace tc
