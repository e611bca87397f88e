// Internal declarations shared by the HIP translation units of libtokencarve.
// Nothing here is part of the C ABI (see include/tokencarve.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tokencarve.h"

namespace tc {

// ---- block-Jacobi geometry -------------------------------------------------------------
constexpr int JB = 32;      // block size b of the block-Jacobi eigensolver
constexpr int JT = 2 * JB;  // a block pair spans a 64 x 64 tile
constexpr int MAX_NVIS = 4096;

__host__ __device__ inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// The eigenvector matrix U of an image (Np x Np, float32) is stored by block columns: the JB columns
// of block column c / JB are kept together, row after row, so that the two block columns a step's
// pair rotates are two contiguous streams (a 64-row slab of one is 8 KB in a row).
__host__ __device__ inline size_t u_index(int r, int c, int Np) {
  return ((size_t)(c / JB) * Np + r) * JB + (c % JB);
}
inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Per-image eigensolver state kept in the workspace.
struct EigState {
  double norm2;    // ||G||_F^2, fixed for the whole solve
  double thr2;     // a visit of a block pair is skipped when the mass it would remove is <= thr2 (0: never)
  int32_t done;    // 1 once the off-diagonal measure fell below the tolerance
  int32_t sweeps;  // sweeps executed so far
  uint32_t tiles;  // 64x64 tiles the tile update has processed (skipped ones not counted); for the profiler
  uint32_t rot_steps[MAX_NVIS / JT];  // rotation steps (32 plane rotations each) the rotation kernel has applied at pair slot i; for the profiler
  int32_t skip[MAX_NVIS / JT];  // per pair of the current step: 1 = the rotation kernel left it alone (R = I)
};

// Everything an entry point needs to know about sizes and where its scratch lives.
struct Plan {
  int B, L, Ls, N, H, dh, D, hidden, kp, kf, m, nA, nB;
  int Np;        // N rounded up to a multiple of JT (zero padded rows/columns of G)
  int nblk;      // Np / JB, always even
  int P;         // nblk / 2 block pairs per step
  int steps;     // nblk - 1 steps per sweep
  int q_tile;    // query rows per attention workgroup
  int n_qtiles;
  int batch_call;        // images of the whole call (B is the group's share when the batch is cut into stream groups)
  int Nq;                // query rows whose probabilities enter the attention score: N + prompt rows
  size_t spart_stride;   // floats of the partial-score region per image
  int esize;     // bytes of one stored element (2 or 4)
  int tsize;     // bytes of one eigensolver element (4 or 8)
  int max_sweeps;
  int groups;    // requested stream groups (0 = automatic)
  int method;    // eigensolver actually used: TC_EIG_JACOBI or TC_EIG_TRIDIAGONAL
  double tol;
  float scale;
  size_t off_O, off_S, off_Spart, off_G, off_U, off_R, off_offpart, off_state, off_sig, off_C, off_E, off_order,
      off_rnorm, off_sim, off_mlist, off_info;
  size_t off_td_d, off_td_e, off_td_tau, off_td_lam, off_td_blk, off_td_tnorm, off_td_rn, off_td_bad, off_td_wgt,
      off_td_W, off_td_tw, off_td_Cpart, off_td_Tf, off_td_tab;  // direct eigensolver only
  size_t total;
};

int make_plan(const tc_params* p, Plan* plan);  // validates p; returns tc_status

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

template <typename T>
inline T* at(void* ws, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(ws) + off); }

inline int check_ws(const Plan& pl, const void* ws, size_t ws_bytes) {
  if (!ws) return TC_ERR_NULL;
  if (misaligned(ws)) return TC_ERR_ALIGN;
  if (ws_bytes < pl.total) return TC_ERR_WORKSPACE;
  return TC_OK;
}

// ---- stage launchers (each returns a tc_status; all work is enqueued on `st`) ----------
int launch_attention(const Plan& pl, int dtype, int causal, const void* Q, const void* K, const void* V, void* O,
                     float* S, float* Spart, hipStream_t st);
int launch_gram(const Plan& pl, int dtype, int eig_dtype, const void* O, void* G, hipStream_t st);
int launch_jacobi(const Plan& pl, int eig_dtype, void* G, void* U /* nullptr: eigenvalues only */, void* R,
                  double* offpart, EigState* state, hipStream_t st);
int launch_scores(const Plan& pl, int eig_dtype, const void* G, const void* U, const EigState* state,
                  const float* S, float lambda, int norm_mode, float sv_rtol, void* sig_ws, float* C_ws, float* E,
                  float* C_out, float* sigma_out, int32_t* info_out, hipStream_t st);
int launch_sigma(const Plan& pl, int eig_dtype, const void* G, const EigState* state, double* sig_ws, float* sigma_out,
                 int32_t* info_out, hipStream_t st);
int launch_combine(const Plan& pl, const float* C_ws, const float* S, float lambda, int norm_mode, float* E, hipStream_t st);
// direct eigensolver (tridiag.hip, tdeig.hip)
int tridiag_panel_width(int N);
int launch_tridiag(const Plan& pl, double* G, double* dvec, double* evec, float* tauv, float* Vc, double* panels,
                   size_t panels_stride, int* tab, hipStream_t st);
int launch_td_eigen(const Plan& pl, const double* dvec, const double* evec, const float* tauv, const float* Vc,
                    double* lam, int2* blk, double* tnorm, double* DP, double* DM, float* W, double* rn, int32_t* bad,
                    double* sig, double* wgt, double* Cpart, float* Tf, float sv_rtol, bool vectors, float* C, float* C_out,
                    float* sigma_out, int32_t* info_out, hipStream_t st);
int direct_eigenvalues(const Plan& pl, const tc_params* p, float* sigma, int32_t* info, void* ws, hipStream_t st);  // api.hip
// helper streams of the library (jacobi.hip): up to 4 streams that run side by side and meet again
int fork_streams(hipStream_t st, int groups, hipStream_t* streams);
void stagger_streams(hipStream_t st, int g, int groups);
void join_streams(hipStream_t st, int groups);
int launch_topk(const Plan& pl, const float* E, int32_t* order, hipStream_t st);
int launch_similarity(const Plan& pl, int dtype, const void* metric, const int32_t* order, float* rnorm, float* sim,
                      hipStream_t st);
int launch_merge(const Plan& pl, int dtype, const void* X, const void* metric, const int32_t* order, void* X_out,
                 int32_t* kept_idx, int32_t* merge_dst, float* rnorm, float* sim, int32_t* mlist, hipStream_t st);

// ---- optional per-kernel timing (only active inside tc_profile_compress) ----------------------
enum ProfKind {
  PK_ATTN = 0, PK_ATTN_REDUCE, PK_GRAM, PK_JINIT, PK_JSOLVE, PK_JUPDATE, PK_JUPDATE_U, PK_JSWEEPEND, PK_SIGMA, PK_ICS, PK_COMBINE,
  PK_TOPK, PK_ROWNORM, PK_SIM, PK_ASSIGN, PK_AVERAGE, PK_TRIDIAG, PK_BISECT, PK_TWISTED, PK_BACKTF, PK_TRIDIAG_UPDATE, PK_COUNT
};
static_assert((int)PK_COUNT == (int)TC_PROF_KINDS, "internal and public kernel kinds must match");
void prof_begin(int kind, int tag, hipStream_t st);  // no-ops unless a profile run is active on this thread
void prof_end(hipStream_t st);
bool profiling_active();
#define TC_TIMED(kind, tag, st, ...) \
  do {                               \
    tc::prof_begin(kind, tag, st);   \
    __VA_ARGS__;                     \
    tc::prof_end(st);                \
  } while (0)

inline int check_launch() { return hipGetLastError() == hipSuccess ? TC_OK : TC_ERR_HIP; }

// ---- small device helpers ---------------------------------------------------------------
__device__ inline float bf16_bits_to_float(uint16_t h) { return __uint_as_float(uint32_t(h) << 16); }

__device__ inline uint16_t float_to_bf16_bits(float f) {  // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

// IEEE half precision storage (TC_F16): conversions by the hardware, round to nearest even.
struct f16_t { uint16_t bits; };  // tag type for templates; bf16 storage uses plain uint16_t
__device__ inline float f16_bits_to_float(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ inline uint16_t float_to_f16_bits(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// The two 16-bit elements packed in a 32-bit word, and the way back (T = uint16_t: bf16, f16_t: half).
template <typename T> __device__ inline void unpack2(uint32_t w, float* lo, float* hi);
template <> __device__ inline void unpack2<uint16_t>(uint32_t w, float* lo, float* hi) {
  *lo = __uint_as_float(w << 16);
  *hi = __uint_as_float(w & 0xffff0000u);
}
template <> __device__ inline void unpack2<f16_t>(uint32_t w, float* lo, float* hi) {
  *lo = f16_bits_to_float((uint16_t)(w & 0xffffu));
  *hi = f16_bits_to_float((uint16_t)(w >> 16));
}
template <typename T> __device__ inline uint32_t pack2(float lo, float hi);
template <> __device__ inline uint32_t pack2<uint16_t>(float lo, float hi) {
  return (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
}
template <> __device__ inline uint32_t pack2<f16_t>(float lo, float hi) {
  return (uint32_t)float_to_f16_bits(lo) | ((uint32_t)float_to_f16_bits(hi) << 16);
}

// Round-robin tournament on n (even) players: pair `i` (0 <= i < n/2) of round `s` (0 <= s < n-1).
__host__ __device__ inline void round_robin_pair(int n, int s, int i, int* a, int* b) {
  const int m = n - 1;
  int x, y;
  if (i == 0) {
    x = n - 1;
    y = s % m;
  } else {
    x = (s + i) % m;
    y = (s - i + m) % m;
  }
  *a = x < y ? x : y;
  *b = x < y ? y : x;
}

// The hardware deals workgroups to the 8 XCDs (each with its own L2) round-robin by linear id.
// group_on_xcd() maps a linear id to (group, item) so that all `items` workgroups of a group land
// on one XCD and run back to back there (what they share -- rotation blocks, K/V of a head, row
// panels -- is then fetched into that L2 once).  Groups are taken eight at a time, one per XCD; the
// groups left over when their number is not a multiple of 8 keep the plain order, spread over all
// XCDs (one XCD with an extra group would finish long after the others).  Launch grid_for_groups()
// workgroups; the function returns false for an id outside the grid.
__host__ __device__ inline int grid_for_groups(int items, int groups) { return items * groups; }
__device__ inline bool group_on_xcd(int id, int items, int groups, int* group, int* item) {
  const int full = groups & ~7, lim = items * full;
  if (id >= lim) {
    const int r = id - lim;
    *group = full + r / items;
    *item = r % items;
    return *group < groups;
  }
  const int k = id >> 3;
  *item = k % items;
  *group = (k / items) * 8 + (id & 7);
  return true;
}

template <typename T>
__device__ inline T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Sum over the 64 lanes with data-parallel lane permutations (no LDS round trips): partners L^1, L^2, 7-L and
// 15-L inside a row of 16, then the four row totals through scalar registers, in a fixed order.  Every lane
// returns the same bits.
template <int CTRL>
__device__ inline double dpp_f64(double x) {
  // (every lane is written -- all rows and banks enabled, and the controls used read lanes inside the wavefront --,
  // so the form without a previous value will do: no register has to be cleared first)
  const int lo = __builtin_amdgcn_mov_dpp(__double2loint(x), CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_mov_dpp(__double2hiint(x), CTRL, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}
__device__ inline double readlane_f64(double x, int l) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l), __builtin_amdgcn_readlane(__double2loint(x), l));
}
// total of each row of 16 lanes, in every lane of the row
__device__ inline double row16_sum_dpp(double x) {
  x += dpp_f64<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_f64<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_f64<0x141>(x);  // row_half_mirror
  x += dpp_f64<0x140>(x);  // row_mirror
  return x;
}
__device__ inline double wave_sum_dpp(double x) {
  x = row16_sum_dpp(x);
  return (readlane_f64(x, 0) + readlane_f64(x, 16)) + (readlane_f64(x, 32) + readlane_f64(x, 48));
}


}  // namespace tc
