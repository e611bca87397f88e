// Stage I pruning and the ordering of Eq. 3-9: per image, a bitonic sort of (score, index) held in
// LDS; the first k_prune entries are written out (score descending, equal scores by ascending index).
#include "tc_internal.h"

namespace tc {

__device__ inline bool precedes(float ka, int ia, float kb, int ib) { return ka > kb || (ka == kb && ia < ib); }

__global__ __launch_bounds__(1024) void topk_kernel(const float* __restrict__ E, int32_t* __restrict__ order, int N,
                                                    int n2, int kp) {
  extern __shared__ unsigned char smem[];
  float* key = reinterpret_cast<float*>(smem);
  int* idx = reinterpret_cast<int*>(smem + (size_t)n2 * sizeof(float));
  const int b = blockIdx.x, tid = threadIdx.x, nt = blockDim.x;
  for (int i = tid; i < n2; i += nt) {
    float v = i < N ? E[(size_t)b * N + i] : -INFINITY;
    if (v != v) v = -INFINITY;  // NaN scores rank last
    key[i] = v;
    idx[i] = i;                 // padding carries indices >= N and loses every tie
  }
  __syncthreads();
  for (int k = 2; k <= n2; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < n2; i += nt) {
        const int l = i ^ j;
        if (l > i) {
          const float ka = key[i], kb = key[l];
          const int ia = idx[i], ib = idx[l];
          const bool fwd = (i & k) == 0;  // this subsequence is sorted "best first"
          const bool swap = fwd ? precedes(kb, ib, ka, ia) : precedes(ka, ia, kb, ib);
          if (swap) { key[i] = kb; key[l] = ka; idx[i] = ib; idx[l] = ia; }
        }
      }
      __syncthreads();
    }
  for (int i = tid; i < kp; i += nt) order[(size_t)b * kp + i] = idx[i];
}

int launch_topk(const Plan& pl, const float* E, int32_t* order, hipStream_t st) {
  int n2 = 64;
  while (n2 < pl.N) n2 <<= 1;
  const int threads = n2 / 2 < 1024 ? (n2 / 2 < 64 ? 64 : n2 / 2) : 1024;
  TC_TIMED(PK_TOPK, 0, st, (topk_kernel<<<pl.B, threads, (size_t)n2 * 8, st>>>(E, order, pl.N, n2, pl.kp)));
  return check_launch();
}

}  // namespace tc
