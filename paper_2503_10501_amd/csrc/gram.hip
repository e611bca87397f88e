// Gram matrix G[b] = O[b] O[b]^T (the route to the SVD of Section 3.3.1: O = U Sigma V^T gives
// O O^T = U Sigma^2 U^T).  Products and sums are formed in float64 on the fp64 matrix cores so that
// small singular values are not drowned by the rounding of the large ones; G is stored in the
// eigensolver's type, zero padded to Np x Np.
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(4))) double d4;

constexpr int GK = 32;   // K chunk staged in LDS
constexpr int GLD = 66;  // panel leading dimension: panel[k][row]; 66 keeps the four contraction rows a wavefront reads at once in different banks

// Eight consecutive stored elements of a row, still in the storage type (converted on the way into LDS).
template <typename TIn> struct Raw8;
template <> struct Raw8<uint16_t> { uint4 v; };
template <> struct Raw8<f16_t> { uint4 v; };
template <> struct Raw8<float> { float4 a, b; };

template <typename TIn>
__device__ inline Raw8<TIn> fetch8(const TIn* src) {
  Raw8<TIn> r;
  if constexpr (sizeof(TIn) == 2) {
    r.v = *reinterpret_cast<const uint4*>(src);
  } else {
    r.a = *reinterpret_cast<const float4*>(src);
    r.b = *reinterpret_cast<const float4*>(src + 4);
  }
  return r;
}
template <typename TIn>
__device__ inline Raw8<TIn> zero8() {
  Raw8<TIn> r;
  if constexpr (sizeof(TIn) == 2) r.v = uint4{0, 0, 0, 0};
  else { r.a = float4{0, 0, 0, 0}; r.b = float4{0, 0, 0, 0}; }
  return r;
}
template <typename TIn>
__device__ inline void widen8(const Raw8<TIn>& r, double* dst) {
  if constexpr (sizeof(TIn) == 2) {
    const uint32_t w[4] = {r.v.x, r.v.y, r.v.z, r.v.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      float lo, hi;
      unpack2<TIn>(w[i], &lo, &hi);
      dst[2 * i] = (double)lo;
      dst[2 * i + 1] = (double)hi;
    }
  } else {
    dst[0] = r.a.x; dst[1] = r.a.y; dst[2] = r.a.z; dst[3] = r.a.w;
    dst[4] = r.b.x; dst[5] = r.b.y; dst[6] = r.b.z; dst[7] = r.b.w;
  }
}

// One workgroup: a 64x64 tile (ti >= tj) of G for one image, mirrored into (tj, ti).  Wavefront w
// owns quadrant (w / 2, w % 2).  The products run on v_mfma_f64_4x4x4 (four independent 4x4x4 blocks
// per instruction), which sustains half as much again as the 16x16x4 form on this chip; a plain
// product with a long contraction can feed it: lane l = p + 4 q + 16 k holds A[p][k] of block q
// (here the same for all four blocks), B[k][p] of block q, and gets D[k][p] of block q, so with
//   A = rows 8 p + r of the quadrant (r = 0..7: eight products share one 16-byte-aligned run of LDS),
//   B = columns 2 (4 q + p) + s    (s = 0, 1: both in one 16-byte read),
// sixteen products per four contraction indices take five 16-byte LDS reads, and a lane ends with
// rows 8 k + r, columns 2 (4 q + p) + s: 16-byte pairs along the row for the tile, runs of eight
// along the column for its mirror.  The next 32 columns of O are fetched into registers meanwhile.
template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void gram_kernel(const TIn* __restrict__ O, TOut* __restrict__ G, int N, int D,
                                                   int Np, int B) {
  typedef __attribute__((ext_vector_type(2))) double d2;
  typedef __attribute__((ext_vector_type(2))) TOut o2;
  __shared__ __attribute__((aligned(16))) double As[GK][GLD];
  __shared__ __attribute__((aligned(16))) double Bs[GK][GLD];
  const int ntile = Np / 64;
  int b, t;
  if (!group_on_xcd(blockIdx.x, ntile * (ntile + 1) / 2, B, &b, &t)) return;
  int ti = 0;  // decode the lower-triangular tile index
  while (t >= ti + 1) { t -= ti + 1; ti++; }
  const int tj = t;
  const TIn* Ob = O + (size_t)b * N * D;
  TOut* Gb = G + (size_t)b * Np * Np;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l15 = lane & 15, q4 = lane >> 4;
  const int wr = wave >> 1, wc = wave & 1;
  const int lrow = tid & 63, kc = tid >> 6;  // loader: row within the panel, which 8-wide k chunk
  const int p4 = lane & 3, blk = (lane >> 2) & 3, kq = lane >> 4;
  double acc[8][2];
#pragma unroll
  for (int r = 0; r < 8; r++) acc[r][0] = acc[r][1] = 0.0;
  const int rowA = ti * 64 + lrow, rowB = tj * 64 + lrow;
  const bool diag = ti == tj;
  const TIn* srcA = Ob + (size_t)rowA * D + kc * 8;
  const TIn* srcB = Ob + (size_t)rowB * D + kc * 8;
  Raw8<TIn> ra = rowA < N ? fetch8<TIn>(srcA) : zero8<TIn>();
  Raw8<TIn> rb = (!diag && rowB < N) ? fetch8<TIn>(srcB) : zero8<TIn>();
  for (int k0 = 0; k0 < D; k0 += GK) {
    double va[8], vb[8];
    widen8<TIn>(ra, va);
    if (!diag) widen8<TIn>(rb, vb);
    __syncthreads();  // previous chunk fully consumed
#pragma unroll
    for (int i = 0; i < 8; i++) {
      As[kc * 8 + i][lrow] = va[i];
      if (!diag) Bs[kc * 8 + i][lrow] = vb[i];
    }
    __syncthreads();
    if (k0 + GK < D) {  // in flight during the products
      if (rowA < N) ra = fetch8<TIn>(srcA + k0 + GK);
      if (!diag && rowB < N) rb = fetch8<TIn>(srcB + k0 + GK);
    }
    const double(*Bp)[GLD] = diag ? As : Bs;
#pragma unroll
    for (int kk = 0; kk < GK; kk += 4) {
      const double* arow = &As[kk + kq][wr * 32 + 8 * p4];
      const d2 a01 = *reinterpret_cast<const d2*>(arow), a23 = *reinterpret_cast<const d2*>(arow + 2);
      const d2 a45 = *reinterpret_cast<const d2*>(arow + 4), a67 = *reinterpret_cast<const d2*>(arow + 6);
      const d2 bb = *reinterpret_cast<const d2*>(&Bp[kk + kq][wc * 32 + 2 * (4 * blk + p4)]);
      const double a[8] = {a01.x, a01.y, a23.x, a23.y, a45.x, a45.y, a67.x, a67.y};
#pragma unroll
      for (int r = 0; r < 8; r++) {
        acc[r][0] = __builtin_amdgcn_mfma_f64_4x4x4f64(a[r], bb.x, acc[r][0], 0, 0, 0);
        acc[r][1] = __builtin_amdgcn_mfma_f64_4x4x4f64(a[r], bb.y, acc[r][1], 0, 0, 0);
      }
    }
  }
  // the lane holds rows 8 kq + r, columns 2 (4 blk + p4) + s of its quadrant
  const int r0 = ti * 64 + wr * 32 + 8 * kq, c0 = tj * 64 + wc * 32 + 2 * (4 * blk + p4);
#pragma unroll
  for (int r = 0; r < 8; r++)
    *reinterpret_cast<o2*>(&Gb[(size_t)(r0 + r) * Np + c0]) = o2{(TOut)acc[r][0], (TOut)acc[r][1]};
  if (!diag) {
#pragma unroll
    for (int sc = 0; sc < 2; sc++)
#pragma unroll
      for (int r = 0; r < 8; r += 2)
        *reinterpret_cast<o2*>(&Gb[(size_t)(c0 + sc) * Np + r0 + r]) = o2{(TOut)acc[r][sc], (TOut)acc[r + 1][sc]};
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
