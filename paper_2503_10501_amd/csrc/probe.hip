// Measurement aid: what this GPU sustains on the matrix cores and on HBM, from register-only loops
// of independent matrix-core products and from a plain streaming copy.  Used by bench.py to print the
// sustained rates next to the published peaks.
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(4))) double d4;
typedef __attribute__((ext_vector_type(4))) float f4;
typedef __attribute__((ext_vector_type(16))) float f16v;
typedef __attribute__((ext_vector_type(8))) __bf16 bf8;

// MODE 0: v_mfma_f64_16x16x4 (2048 flop), 1: v_mfma_f32_16x16x4 (2048 flop), 2: v_mfma_f32_32x32x16_bf16 (32768 flop),
// 3: v_mfma_f64_4x4x4, four blocks (512 flop)
template <int MODE>
__global__ __launch_bounds__(256) void mfma_loop(float* __restrict__ out, int n) {
  const int tid = threadIdx.x;
  const double a = tid * 1e-3, b = tid * 2e-3;
  d4 c[4];
  double s4[4] = {0.0, 0.0, 0.0, 0.0};
  f4 e[4];
  f16v g[4];
  bf8 ha, hb;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    c[i] = d4{0, 0, 0, 0};
    e[i] = f4{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 16; j++) g[i][j] = 0.f;
  }
#pragma unroll
  for (int i = 0; i < 8; i++) { ha[i] = (__bf16)(float)(tid + i); hb[i] = (__bf16)(float)i; }
  for (int it = 0; it < n; it++) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if (MODE == 0) c[i] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c[i], 0, 0, 0);
      if (MODE == 1) e[i] = __builtin_amdgcn_mfma_f32_16x16x4f32((float)a, (float)b, e[i], 0, 0, 0);
      if (MODE == 2) g[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ha, hb, g[i], 0, 0, 0);
      if (MODE == 3) s4[i] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, s4[i], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    s += (float)c[i][0] + e[i][0] + g[i][0] + (float)s4[i];
  }
  out[(size_t)blockIdx.x * 256 + tid] = s;
}

__global__ __launch_bounds__(256) void copy_loop(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

template <int MODE>
static float time_mfma(float* buf, int blocks, int iters, hipStream_t st) {
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.f;
  float best = 1e30f;
  for (int rep = 0; rep < 3; rep++) {
    (void)hipEventRecord(e0, st);
    mfma_loop<MODE><<<blocks, 256, 0, st>>>(buf, iters);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess) { best = -1.f; break; }
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    if (rep > 0 && ms < best) best = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return best;
}

}  // namespace tc

using namespace tc;

extern "C" int tc_probe_rates(void* ws, size_t ws_bytes, void* stream, float* rates) {
  if (!ws || !rates) return TC_ERR_NULL;
  if (misaligned(ws)) return TC_ERR_ALIGN;
  const size_t need = (size_t)1 << 31;  // two 1 GiB halves for the copy: four times the 256 MB last-level cache, so the rate is an HBM rate
  if (ws_bytes < need) return TC_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int blocks = 2048, iters = 20000;
  float* buf = static_cast<float*>(ws);
  const double mfmas = 4.0 * iters * 4.0 * blocks;  // per wavefront 4 per iteration, 4 wavefronts per workgroup
  const float t0 = time_mfma<0>(buf, blocks, iters, st);
  const float t1 = time_mfma<1>(buf, blocks, iters, st);
  const float t2 = time_mfma<2>(buf, blocks, iters, st);
  const float t3 = time_mfma<3>(buf, blocks, iters, st);
  if (t0 <= 0.f || t1 <= 0.f || t2 <= 0.f || t3 <= 0.f) return TC_ERR_HIP;
  rates[0] = (float)(mfmas * 2048.0 / (t0 * 1e-3) / 1e12);
  rates[1] = (float)(mfmas * 2048.0 / (t1 * 1e-3) / 1e12);
  rates[2] = (float)(mfmas * 32768.0 / (t2 * 1e-3) / 1e12);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return TC_ERR_HIP;
  const size_t half = need / 2, n16 = half / 16;
  float best = 1e30f;
  for (int rep = 0; rep < 4; rep++) {
    (void)hipEventRecord(e0, st);
    copy_loop<<<4096, 256, 0, st>>>(static_cast<const uint4*>(ws), reinterpret_cast<uint4*>(static_cast<char*>(ws) + half), n16);
    (void)hipEventRecord(e1, st);
    if (hipEventSynchronize(e1) != hipSuccess) { best = -1.f; break; }
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    if (rep > 0 && ms < best) best = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (best <= 0.f) return TC_ERR_HIP;
  rates[3] = (float)(2.0 * half / (best * 1e-3) / 1e9);  // GB/s, bytes read + bytes written
  rates[4] = (float)(mfmas * 512.0 / (t3 * 1e-3) / 1e12);
  return check_launch();
}
