// Gram matrix G[b] = O[b] O[b]^T (the route to the SVD of Section 3.3.1: O = U Sigma V^T gives
// O O^T = U Sigma^2 U^T).  Products and sums are formed in float64 on the fp64 matrix cores so that
// small singular values are not drowned by the rounding of the large ones; G is stored in the
// eigensolver's type, zero padded to Np x Np.
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(4))) double d4;

constexpr int GK = 32;   // K chunk staged in LDS
constexpr int GLD = 64;  // panel leading dimension: panel[k][row]

template <typename TIn>
__device__ inline void load8(const TIn* src, double* dst);

template <>
__device__ inline void load8<uint16_t>(const uint16_t* src, double* dst) {
  uint4 v = *reinterpret_cast<const uint4*>(src);
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; i++) {
    dst[2 * i] = (double)__uint_as_float(w[i] << 16);
    dst[2 * i + 1] = (double)__uint_as_float(w[i] & 0xffff0000u);
  }
}
template <>
__device__ inline void load8<f16_t>(const f16_t* src, double* dst) {
  uint4 v = *reinterpret_cast<const uint4*>(src);
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; i++) {
    float lo, hi;
    unpack2<f16_t>(w[i], &lo, &hi);
    dst[2 * i] = (double)lo;
    dst[2 * i + 1] = (double)hi;
  }
}
template <>
__device__ inline void load8<float>(const float* src, double* dst) {
  float4 a = *reinterpret_cast<const float4*>(src);
  float4 b = *reinterpret_cast<const float4*>(src + 4);
  dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w;
  dst[4] = b.x; dst[5] = b.y; dst[6] = b.z; dst[7] = b.w;
}

// One workgroup: a 64x64 tile (ti >= tj) of G for image blockIdx.y, mirrored into (tj, ti).
template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void gram_kernel(const TIn* __restrict__ O, TOut* __restrict__ G, int N, int D,
                                                   int Np, int B) {
  __shared__ double As[GK][GLD];
  __shared__ double Bs[GK][GLD];
  const int ntile = Np / 64;
  int b, t;
  if (!group_on_xcd(blockIdx.x, ntile * (ntile + 1) / 2, B, &b, &t)) return;
  int ti = 0;  // decode the lower-triangular tile index
  while (t >= ti + 1) { t -= ti + 1; ti++; }
  const int tj = t;
  const TIn* Ob = O + (size_t)b * N * D;
  TOut* Gb = G + (size_t)b * Np * Np;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int lrow = tid & 63, kc = tid >> 6;  // loader: row within the panel, which 8-wide k chunk
  d4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++) acc[i][j] = d4{0, 0, 0, 0};
  const int rowA = ti * 64 + lrow, rowB = tj * 64 + lrow;
  const bool diag = ti == tj;
  for (int k0 = 0; k0 < D; k0 += GK) {
    double va[8], vb[8];
    if (rowA < N) load8<TIn>(Ob + (size_t)rowA * D + k0 + kc * 8, va);
    else
#pragma unroll
      for (int i = 0; i < 8; i++) va[i] = 0.0;
    if (!diag) {
      if (rowB < N) load8<TIn>(Ob + (size_t)rowB * D + k0 + kc * 8, vb);
      else
#pragma unroll
        for (int i = 0; i < 8; i++) vb[i] = 0.0;
    }
    __syncthreads();  // previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < 8; i++) {
      As[kc * 8 + i][lrow] = va[i];
      if (!diag) Bs[kc * 8 + i][lrow] = vb[i];
    }
    __syncthreads();
    const double(*Bp)[GLD] = diag ? As : Bs;
#pragma unroll
    for (int kk = 0; kk < GK; kk += 4) {
      const int k = kk + (lane >> 4);
      double a0 = As[k][wr * 32 + (lane & 15)], a1 = As[k][wr * 32 + 16 + (lane & 15)];
      double b0 = Bp[k][wc * 32 + (lane & 15)], b1 = Bp[k][wc * 32 + 16 + (lane & 15)];
      acc[0][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b1, acc[1][1], 0, 0, 0);
    }
  }
  // accumulator element j of a lane sits at row 4*j + lane/16, column lane%16 of its 16x16 tile
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int r = ti * 64 + wr * 32 + mt * 16 + 4 * j + (lane >> 4);
        const int c = tj * 64 + wc * 32 + nt * 16 + (lane & 15);
        const TOut v = (TOut)acc[mt][nt][j];
        Gb[(size_t)r * Np + c] = v;
        if (!diag) Gb[(size_t)c * Np + r] = v;
      }
}

int launch_gram(const Plan& pl, int dtype, int eig_dtype, const void* O, void* G, hipStream_t st) {
  const int nt = pl.Np / 64;
  dim3 grid(grid_for_groups(nt * (nt + 1) / 2, pl.B)), block(256);
  if (dtype == TC_BF16) {
    if (eig_dtype == TC_EIG_F64)
      TC_TIMED(PK_GRAM, 0, st, (gram_kernel<uint16_t, double><<<grid, block, 0, st>>>((const uint16_t*)O, (double*)G, pl.N, pl.D, pl.Np, pl.B)));
    else
      TC_TIMED(PK_GRAM, 0, st, (gram_kernel<uint16_t, float><<<grid, block, 0, st>>>((const uint16_t*)O, (float*)G, pl.N, pl.D, pl.Np, pl.B)));
  } else if (dtype == TC_F16) {
    if (eig_dtype == TC_EIG_F64)
      TC_TIMED(PK_GRAM, 0, st, (gram_kernel<f16_t, double><<<grid, block, 0, st>>>((const f16_t*)O, (double*)G, pl.N, pl.D, pl.Np, pl.B)));
    else
      TC_TIMED(PK_GRAM, 0, st, (gram_kernel<f16_t, float><<<grid, block, 0, st>>>((const f16_t*)O, (float*)G, pl.N, pl.D, pl.Np, pl.B)));
  } else {
    if (eig_dtype == TC_EIG_F64)
      TC_TIMED(PK_GRAM, 0, st, (gram_kernel<float, double><<<grid, block, 0, st>>>((const float*)O, (double*)G, pl.N, pl.D, pl.Np, pl.B)));
    else
      TC_TIMED(PK_GRAM, 0, st, (gram_kernel<float, float><<<grid, block, 0, st>>>((const float*)O, (float*)G, pl.N, pl.D, pl.Np, pl.B)));
  }
  return check_launch();
}

}  // namespace tc
