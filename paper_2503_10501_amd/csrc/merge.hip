// Stage II (Section 3.3.2): cosine similarity between SetB and SetA rows of the metric (Eq. 3-10),
// choice of the merged tokens and their destinations, and the averaging pass that writes the
// compressed token rows in ascending position.
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf8;
typedef __attribute__((ext_vector_type(8))) _Float16 h8;
typedef __attribute__((ext_vector_type(16))) float f16v;

// ---- 1 / ||metric row||_2 for the k_prune surviving rows, in score order -----------------------
template <typename TIn>
__global__ __launch_bounds__(256) void rownorm_kernel(const TIn* __restrict__ metric, const int32_t* __restrict__ order,
                                                      float* __restrict__ rnorm, int N, int D, int kp) {
  const int b = blockIdx.y, lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= kp) return;
  const int x = min(max(order[(size_t)b * kp + r], 0), N - 1);
  const TIn* row = metric + ((size_t)b * N + x) * D;
  float ss = 0.f;
  if constexpr (sizeof(TIn) == 2) {
    for (int k = lane * 8; k < D; k += 512) {
      const uint4 v = *reinterpret_cast<const uint4*>(row + k);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float lo, hi;
        unpack2<TIn>(w[i], &lo, &hi);
        ss += lo * lo;
        ss += hi * hi;
      }
    }
  } else {
    for (int k = lane * 4; k < D; k += 256) {
      const float4 v = *reinterpret_cast<const float4*>(row + k);
      ss += v.x * v.x; ss += v.y * v.y; ss += v.z * v.z; ss += v.w * v.w;
    }
  }
  ss = wave_sum(ss);
  if (lane == 0) rnorm[(size_t)b * kp + r] = 1.0f / fmaxf(sqrtf(ss), 1e-30f);
}

// ---- Sim[b][j][i] = <z_Bj, z_Ai> / (|z_Bj| |z_Ai|), 16-bit rows (bf16 or half) on the matrix cores ---
constexpr int SK = 64;       // K chunk
constexpr int SP = SK + 8;   // padded LDS row (bf16 elements)

template <bool F16>
__global__ __launch_bounds__(256) void sim_bf16_kernel(const uint16_t* __restrict__ metric,
                                                       const int32_t* __restrict__ order,
                                                       const float* __restrict__ rnorm, float* __restrict__ sim, int N,
                                                       int D, int kp, int nA, int nB) {
  __shared__ __attribute__((aligned(16))) uint16_t Bj[64][SP];
  __shared__ __attribute__((aligned(16))) uint16_t Ai[64][SP];
  const int b = blockIdx.y;
  const int tilesA = (nA + 63) / 64;
  const int tj = blockIdx.x / tilesA, ti = blockIdx.x % tilesA;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wr = wave >> 1, wc = wave & 1;
  const int32_t* ord = order + (size_t)b * kp;
  const int lrow = tid >> 2, piece = tid & 3;  // loader: 64 rows x 4 pieces of 16 bf16
  const int j_l = tj * 64 + lrow, i_l = ti * 64 + lrow;
  const uint16_t* srcB = j_l < nB ? metric + ((size_t)b * N + min(max(ord[nA + j_l], 0), N - 1)) * D : nullptr;
  const uint16_t* srcA = i_l < nA ? metric + ((size_t)b * N + min(max(ord[i_l], 0), N - 1)) * D : nullptr;
  f16v acc;
#pragma unroll
  for (int i = 0; i < 16; i++) acc[i] = 0.f;
  const uint4 zero = {0, 0, 0, 0};
  for (int k0 = 0; k0 < D; k0 += SK) {
    uint4 b0 = zero, b1 = zero, a0 = zero, a1 = zero;
    if (srcB) { b0 = *reinterpret_cast<const uint4*>(srcB + k0 + piece * 16); b1 = *reinterpret_cast<const uint4*>(srcB + k0 + piece * 16 + 8); }
    if (srcA) { a0 = *reinterpret_cast<const uint4*>(srcA + k0 + piece * 16); a1 = *reinterpret_cast<const uint4*>(srcA + k0 + piece * 16 + 8); }
    __syncthreads();
    *reinterpret_cast<uint4*>(&Bj[lrow][piece * 16]) = b0;
    *reinterpret_cast<uint4*>(&Bj[lrow][piece * 16 + 8]) = b1;
    *reinterpret_cast<uint4*>(&Ai[lrow][piece * 16]) = a0;
    *reinterpret_cast<uint4*>(&Ai[lrow][piece * 16 + 8]) = a1;
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < SK; kk += 16) {
      if constexpr (F16) {
        const h8 fa = *reinterpret_cast<const h8*>(&Bj[wr * 32 + (lane & 31)][kk + 8 * (lane >> 5)]);
        const h8 fb = *reinterpret_cast<const h8*>(&Ai[wc * 32 + (lane & 31)][kk + 8 * (lane >> 5)]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa, fb, acc, 0, 0, 0);
      } else {
        const bf8 fa = *reinterpret_cast<const bf8*>(&Bj[wr * 32 + (lane & 31)][kk + 8 * (lane >> 5)]);
        const bf8 fb = *reinterpret_cast<const bf8*>(&Ai[wc * 32 + (lane & 31)][kk + 8 * (lane >> 5)]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc, 0, 0, 0);
      }
    }
  }
  const int i = ti * 64 + wc * 32 + (lane & 31);
  if (i < nA) {
    const float rn_i = rnorm[(size_t)b * kp + i];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int j = tj * 64 + wr * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (j < nB) sim[((size_t)b * nB + j) * nA + i] = acc[r] * rnorm[(size_t)b * kp + nA + j] * rn_i;
    }
  }
}

// float rows: plain LDS-tiled FMA (the float32 storage type is a correctness path, not a fast one)
__global__ __launch_bounds__(256) void sim_f32_kernel(const float* __restrict__ metric,
                                                      const int32_t* __restrict__ order,
                                                      const float* __restrict__ rnorm, float* __restrict__ sim, int N,
                                                      int D, int kp, int nA, int nB) {
  __shared__ float Bj[16][33];
  __shared__ float Ai[16][33];
  const int b = blockIdx.y;
  const int tilesA = (nA + 15) / 16;
  const int tj = blockIdx.x / tilesA, ti = blockIdx.x % tilesA;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int32_t* ord = order + (size_t)b * kp;
  const int lrow = tid >> 4, lk = tid & 15;
  const int j_l = tj * 16 + lrow, i_l = ti * 16 + lrow;
  const float* srcB = j_l < nB ? metric + ((size_t)b * N + min(max(ord[nA + j_l], 0), N - 1)) * D : nullptr;
  const float* srcA = i_l < nA ? metric + ((size_t)b * N + min(max(ord[i_l], 0), N - 1)) * D : nullptr;
  double acc = 0.0;
  for (int k0 = 0; k0 < D; k0 += 32) {
    __syncthreads();
    for (int h = 0; h < 2; h++) {
      const int k = k0 + lk + 16 * h;
      Bj[lrow][lk + 16 * h] = (srcB && k < D) ? srcB[k] : 0.f;
      Ai[lrow][lk + 16 * h] = (srcA && k < D) ? srcA[k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 32; k++) acc += (double)Bj[ty][k] * (double)Ai[tx][k];
  }
  const int j = tj * 16 + ty, i = ti * 16 + tx;
  if (j < nB && i < nA)
    sim[((size_t)b * nB + j) * nA + i] = (float)acc * rnorm[(size_t)b * kp + nA + j] * rnorm[(size_t)b * kp + i];
}

// ---- per image: argmax over SetA, top-m of SetB, index bookkeeping -------------------------------
// LDS: dst[N] | val[nB] | best[nB] | cnt[256]
__global__ __launch_bounds__(256) void assign_kernel(const float* __restrict__ sim, const int32_t* __restrict__ order,
                                                     int32_t* __restrict__ kept_idx, int32_t* __restrict__ merge_dst,
                                                     int32_t* __restrict__ mlist, int N, int kp, int kf, int nA,
                                                     int nB) {
  extern __shared__ int smem_i[];
  int* dst = smem_i;
  float* val = reinterpret_cast<float*>(smem_i + N);
  int* best = smem_i + N + nB;
  int* cnt = smem_i + N + 2 * nB;
  int* cnt2 = cnt + 256;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* ord = order + (size_t)b * kp;
  const int m = kp - kf;
  for (int x = tid; x < N; x += 256) dst[x] = -1;
  __syncthreads();
  for (int r = tid; r < kp; r += 256) {
    const int x = ord[r];
    if ((unsigned)x < (unsigned)N) dst[x] = x;  // entries outside [0,N) violate the contract and are ignored
  }
  // most similar SetA token of every SetB token; equal similarity -> lower visual index
  for (int j = wave; j < nB; j += 4) {
    const float* row = sim + ((size_t)b * nB + j) * nA;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int i = lane; i < nA; i += 64) {
      float v = row[i];
      if (v != v) v = -INFINITY;  // a NaN similarity (a NaN in the metric row) loses against everything
      const int a = ord[i];
      if (v > bv || (v == bv && a < bi)) { bv = v; bi = a; }  // v == bv == -inf still takes the lowest index: the destination is always a Set-A token
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { val[j] = bv; best[j] = bi; }
  }
  __syncthreads();
  // the m SetB tokens with the highest similarity; equal similarity -> lower visual index
  for (int j = tid; j < nB; j += 256) {
    const float v = val[j];
    const int xj = ord[nA + j];
    int rank = 0;
    for (int k = 0; k < nB; k++) {
      const float vk = val[k];
      rank += (vk > v || (vk == v && ord[nA + k] < xj)) ? 1 : 0;
    }
    if (rank < m && (unsigned)xj < (unsigned)N) dst[xj] = best[j];
  }
  __syncthreads();
  // compact, in ascending position: output rows (dst[x] == x) and merged sources (dst[x] != x, >= 0)
  const int chunk = (N + 255) / 256;
  const int x0 = tid * chunk, x1 = min(N, x0 + chunk);
  int nk = 0, nm = 0;
  for (int x = x0; x < x1; x++) {
    const int d = dst[x];
    nk += d == x;
    nm += d >= 0 && d != x;
  }
  cnt[tid] = nk; cnt2[tid] = nm;
  __syncthreads();
  if (tid == 0) {
    int a = 0, c = 0;
    for (int t = 0; t < 256; t++) {
      const int ta = cnt[t], tc_ = cnt2[t];
      cnt[t] = a; cnt2[t] = c;
      a += ta; c += tc_;
    }
  }
  __syncthreads();
  int pk = cnt[tid], pm = cnt2[tid];
  for (int x = x0; x < x1; x++) {
    const int d = dst[x];
    if (d == x) { if (pk < kf) kept_idx[(size_t)b * kf + pk++] = x; }
    else if (d >= 0 && pm < m) { mlist[((size_t)b * (m > 0 ? m : 1) + pm) * 2] = x; mlist[((size_t)b * (m > 0 ? m : 1) + pm) * 2 + 1] = d; pm++; }
  }
  for (int x = tid; x < N; x += 256) merge_dst[(size_t)b * N + x] = dst[x];
}

// ---- averaging pass: one workgroup per output row ------------------------------------------------
template <typename TIn>
__global__ __launch_bounds__(256) void average_kernel(const TIn* __restrict__ X, const int32_t* __restrict__ kept_idx,
                                                      const int32_t* __restrict__ mlist, TIn* __restrict__ X_out,
                                                      int N, int hidden, int kf, int m) {
  constexpr int V = 16 / sizeof(TIn);  // elements per 16-byte access
  __shared__ int srcs[MAX_NVIS / 2];   // sources merged into this row, ascending position
  __shared__ int wave_cnt[4];
  const int b = blockIdx.y, r = blockIdx.x, tid = threadIdx.x;
  const int a = kept_idx[(size_t)b * kf + r];
  const int32_t* ml = mlist + (size_t)b * (m > 0 ? m : 1) * 2;
  const TIn* Xb = X + (size_t)b * N * hidden;
  TIn* out = X_out + ((size_t)b * kf + r) * hidden;
  int nsrc = 0;
  for (int base = 0; base < m; base += 256) {  // uniform trip count; order of mlist is kept
    const int e = base + tid;
    const bool hit = e < m && ml[2 * e + 1] == a;
    const unsigned long long mask = __ballot(hit);
    __syncthreads();
    if ((tid & 63) == 0) wave_cnt[tid >> 6] = __popcll(mask);
    __syncthreads();
    int off = nsrc;
    for (int w = 0; w < (tid >> 6); w++) off += wave_cnt[w];
    if (hit) srcs[off + __popcll(mask & ((1ull << (tid & 63)) - 1ull))] = ml[2 * e];
    nsrc += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
  }
  __syncthreads();
  const float fc = (float)(1 + nsrc);
  for (int v0 = tid * V; v0 < hidden; v0 += 256 * V) {
    float acc[V];
    auto add_row = [&](const TIn* row, bool first) {
      const uint4 raw = *reinterpret_cast<const uint4*>(row + v0);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
      if constexpr (sizeof(TIn) == 2) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
          float lo, hi;
          unpack2<TIn>(w[i], &lo, &hi);
          acc[2 * i] = first ? lo : acc[2 * i] + lo;
          acc[2 * i + 1] = first ? hi : acc[2 * i + 1] + hi;
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; i++) acc[i] = first ? __uint_as_float(w[i]) : acc[i] + __uint_as_float(w[i]);
      }
    };
    add_row(Xb + (size_t)a * hidden, true);
    for (int s = 0; s < nsrc; s++) add_row(Xb + (size_t)srcs[s] * hidden, false);
    uint32_t w[4];
    if constexpr (sizeof(TIn) == 2) {
#pragma unroll
      for (int i = 0; i < 4; i++) w[i] = pack2<TIn>(acc[2 * i] / fc, acc[2 * i + 1] / fc);
    } else {
#pragma unroll
      for (int i = 0; i < 4; i++) w[i] = __float_as_uint(acc[i] / fc);
    }
    *reinterpret_cast<uint4*>(out + v0) = uint4{w[0], w[1], w[2], w[3]};
  }
}

// Eq. 3-10: row norms of the k_prune surviving rows, then Sim [B, |B|, |A|].
int launch_similarity(const Plan& pl, int dtype, const void* metric, const int32_t* order, float* rnorm, float* sim,
                      hipStream_t st) {
  if (pl.nA == 0) return TC_OK;  // a single survivor: Set A is empty, there is nothing to compare
  const dim3 gn((pl.kp + 3) / 4, pl.B);
  if (dtype == TC_BF16 || dtype == TC_F16) {
    const dim3 gsim(((pl.nB + 63) / 64) * ((pl.nA + 63) / 64), pl.B);
    if (dtype == TC_F16) {
      TC_TIMED(PK_ROWNORM, 0, st, (rownorm_kernel<f16_t><<<gn, 256, 0, st>>>((const f16_t*)metric, order, rnorm, pl.N, pl.D, pl.kp)));
      TC_TIMED(PK_SIM, 0, st, (sim_bf16_kernel<true><<<gsim, 256, 0, st>>>((const uint16_t*)metric, order, rnorm, sim, pl.N, pl.D, pl.kp, pl.nA, pl.nB)));
    } else {
      TC_TIMED(PK_ROWNORM, 0, st, (rownorm_kernel<uint16_t><<<gn, 256, 0, st>>>((const uint16_t*)metric, order, rnorm, pl.N, pl.D, pl.kp)));
      TC_TIMED(PK_SIM, 0, st, (sim_bf16_kernel<false><<<gsim, 256, 0, st>>>((const uint16_t*)metric, order, rnorm, sim, pl.N, pl.D, pl.kp, pl.nA, pl.nB)));
    }
  } else {
    TC_TIMED(PK_ROWNORM, 0, st, (rownorm_kernel<float><<<gn, 256, 0, st>>>((const float*)metric, order, rnorm, pl.N, pl.D, pl.kp)));
    const dim3 gsim(((pl.nB + 15) / 16) * ((pl.nA + 15) / 16), pl.B);
    TC_TIMED(PK_SIM, 0, st, (sim_f32_kernel<<<gsim, 256, 0, st>>>((const float*)metric, order, rnorm, sim, pl.N, pl.D, pl.kp, pl.nA, pl.nB)));
  }
  return check_launch();
}

int launch_merge(const Plan& pl, int dtype, const void* X, const void* metric, const int32_t* order, void* X_out,
                 int32_t* kept_idx, int32_t* merge_dst, float* rnorm, float* sim, int32_t* mlist, hipStream_t st) {
  const int rc = launch_similarity(pl, dtype, metric, order, rnorm, sim, st);
  if (rc != TC_OK) return rc;
  const size_t lds = ((size_t)pl.N + 2 * (size_t)pl.nB + 512) * 4;
  TC_TIMED(PK_ASSIGN, 0, st, (assign_kernel<<<pl.B, 256, lds, st>>>(sim, order, kept_idx, merge_dst, mlist, pl.N, pl.kp, pl.kf, pl.nA, pl.nB)));
  const dim3 ga(pl.kf, pl.B);
  if (dtype == TC_F16)
    TC_TIMED(PK_AVERAGE, 0, st, (average_kernel<f16_t><<<ga, 256, 0, st>>>((const f16_t*)X, kept_idx, mlist, (f16_t*)X_out, pl.N, pl.hidden, pl.kf, pl.m)));
  else if (dtype == TC_BF16)
    TC_TIMED(PK_AVERAGE, 0, st, (average_kernel<uint16_t><<<ga, 256, 0, st>>>((const uint16_t*)X, kept_idx, mlist, (uint16_t*)X_out, pl.N, pl.hidden,
                                                pl.kf, pl.m)));
  else
    TC_TIMED(PK_AVERAGE, 0, st, (average_kernel<float><<<ga, 256, 0, st>>>((const float*)X, kept_idx, mlist, (float*)X_out, pl.N, pl.hidden, pl.kf,
                                             pl.m)));
  return check_launch();
}

}  // namespace tc
