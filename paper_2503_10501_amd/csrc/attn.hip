// Attention output of the visual query rows (Eq. 3-1, 3-2 and the slice of Section 3.2.2) and the
// attention score of every visual token (Eq. 3-7).
//
// 16-bit storage (bf16 or half): one workgroup = one (image, head, 128-query tile); each wavefront owns 32 queries.
// Scores are formed transposed, S^T = K Q^T, so that a lane owns one query (softmax statistics stay
// in the lane) and the probabilities feed O^T = V^T P^T straight from the accumulator registers.
// Two passes over the keys: pass 1 finds the row maximum and normaliser, pass 2 recomputes the
// scores, forms the exact probabilities, accumulates O^T and the column sums of the probabilities
// (the attention matrix itself is never stored).  Column sums leave the workgroup as one partial
// row per (head, query tile) and are added in a fixed order by a second small kernel.
#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf8;
typedef __attribute__((ext_vector_type(8))) _Float16 h8;
typedef __attribute__((ext_vector_type(16))) float f16v;

// The 16-bit element type of the matrix-core operands: bf16 (F16 = false) or IEEE half.
template <bool F16> struct Elem16;
template <> struct Elem16<false> {
  typedef __bf16 elem;
  typedef bf8 vec8;
  __device__ static inline f16v mma(vec8 a, vec8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
  __device__ static inline uint16_t bits(float f) { return float_to_bf16_bits(f); }
  // a and b as packed 16-bit heads (a in the low half) and the packed heads of what the first rounding left
  __device__ static inline void split2(float a, float b, uint32_t& head, uint32_t& rem) {
    typedef __attribute__((ext_vector_type(2))) float f2;
    typedef __attribute__((ext_vector_type(2))) __bf16 b2;
    union { b2 v; uint32_t w; } h, r;
    h.v = __builtin_convertvector(f2{a, b}, b2);
    r.v = __builtin_convertvector(f2{a - __uint_as_float(h.w << 16), b - __uint_as_float(h.w & 0xffff0000u)}, b2);
    head = h.w;
    rem = r.w;
  }
};
template <> struct Elem16<true> {
  typedef _Float16 elem;
  typedef h8 vec8;
  __device__ static inline f16v mma(vec8 a, vec8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
  __device__ static inline uint16_t bits(float f) { return float_to_f16_bits(f); }
  __device__ static inline void split2(float a, float b, uint32_t& head, uint32_t& rem) {
    typedef __attribute__((ext_vector_type(2))) float f2;
    typedef __attribute__((ext_vector_type(2))) _Float16 h2;
    union { h2 v; uint32_t w; } h, r;
    h.v = __builtin_convertvector(f2{a, b}, h2);
    r.v = __builtin_convertvector(f2{a - (float)h.v[0], b - (float)h.v[1]}, h2);
    head = h.w;
    rem = r.w;
  }
};

typedef __attribute__((ext_vector_type(2))) unsigned int u2v;
typedef __attribute__((ext_vector_type(4))) unsigned int u4v;  // 16 bytes in registers (a native vector: no struct copies)

// v of the lane that a data-parallel permutation control pairs this lane with (0x140: 15-L within a
// row of 16 lanes, 0x141: 7-L within 8, 0x4E: L^2, 0xB1: L^1).  All lanes of the wavefront must be active.
template <int CTRL>
__device__ inline float lane_perm(float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), CTRL, 0xf, 0xf, false));
}

// 2^x by the hardware instruction alone: results below the smallest normal number come out as 0, which
// a softmax term of that size may (the library routine spends five more instructions per call on them)
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int AQ = 128;  // queries per workgroup
constexpr int AK = 64;   // keys per LDS tile

// LDS: two stages of (K tile, transposed V tile), so that the next tile is written while this one is read
// (one barrier per tile), and two sets of per-wavefront column sums.
template <int DH>
struct AttnSmem {
  static constexpr int KLD = DH + 8;  // bf16 elements per K row in LDS
  static constexpr int VLD = AK + 8;  // bf16 elements per V^T row in LDS
  static constexpr int K_BYTES = AK * KLD * 2;
  static constexpr int V_BYTES = DH * VLD * 2;
  static constexpr int STAGE = K_BYTES + V_BYTES;
  static constexpr int O_BYTES = 4 * 32 * KLD * 2;
  static constexpr int MAIN = 2 * STAGE > O_BYTES ? 2 * STAGE : O_BYTES;
  static constexpr int CS_BYTES = 2 * 4 * AK * 4;
  static constexpr int TOTAL = MAIN + CS_BYTES;
};

// Keys past the end of the sequence are read as the last key (no branch around a load, so that the compiler
// counts the loads in flight exactly); they are masked out of every result.
template <int DH>
__device__ inline void load_k_tile(const uint16_t* __restrict__ Kh, int k0, int L, u4v* regs) {
  constexpr int CH = DH / 8, ITER = AK * CH / 256;
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int idx = threadIdx.x + 256 * it, key = idx / CH, ch = idx % CH;
    regs[it] = *reinterpret_cast<const u4v*>(Kh + (size_t)min(k0 + key, L - 1) * DH + ch * 8);
  }
}
template <int DH>
__device__ inline void store_k_tile(uint16_t* Ks, const u4v* regs) {
  constexpr int CH = DH / 8, ITER = AK * CH / 256, KLD = AttnSmem<DH>::KLD;
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int idx = threadIdx.x + 256 * it, key = idx / CH, ch = idx % CH;
    *reinterpret_cast<u4v*>(Ks + key * KLD + ch * 8) = regs[it];
  }
}
template <int DH>
__device__ inline void load_v_tile(const uint16_t* __restrict__ Vh, int k0, int L, u4v* regs) {
  constexpr int ITER = DH / 32;
  const int key = threadIdx.x & 63;
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int ch = (threadIdx.x >> 6) + 4 * it;
    regs[it] = *reinterpret_cast<const u4v*>(Vh + (size_t)min(k0 + key, L - 1) * DH + ch * 8);
  }
}
template <int DH>
__device__ inline void store_v_tile_transposed(uint16_t* Vt, const u4v* regs) {
  constexpr int ITER = DH / 32, VLD = AttnSmem<DH>::VLD;
  const int key = threadIdx.x & 63;
  // Within a row the keys are stored with bits 2 and 3 swapped: the eight keys that one lane feeds
  // to a matrix-core product (16u + 4*half + {0..3} and those plus 8) are then 16 contiguous bytes.
  const int pos = (key & ~12) | ((key & 4) << 1) | ((key & 8) >> 1);
#pragma unroll
  for (int it = 0; it < ITER; it++) {
    const int ch = (threadIdx.x >> 6) + 4 * it;
    const uint32_t w[4] = {regs[it].x, regs[it].y, regs[it].z, regs[it].w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      Vt[(ch * 8 + 2 * i) * VLD + pos] = (uint16_t)(w[i] & 0xffffu);
      Vt[(ch * 8 + 2 * i + 1) * VLD + pos] = (uint16_t)(w[i] >> 16);
    }
  }
}

// One word of every 128-byte line of a K tile (threads 0 .. 127) and of a V tile (threads 128 .. 255), so that
// the lines are on their way into the L2 well before the tile itself is fetched (a first read comes from HBM
// and takes longer than the work on one tile).  Keys are clamped to [0, kcap): a touch past the end repeats a line.
template <int DH>
__device__ inline uint32_t touch_lines(const uint16_t* __restrict__ Kh, const uint16_t* __restrict__ Vh, int k_key0,
                                       int v_key0, int kcap) {
  constexpr int LPR = DH * 2 / 128;  // lines per row
  const int i = min((int)(threadIdx.x & 127), AK * LPR - 1);
  const bool is_v = threadIdx.x >= 128;
  const int key = min(max(is_v ? v_key0 : k_key0, 0) + i / LPR, kcap - 1);
  return *reinterpret_cast<const uint32_t*>((is_v ? Vh : Kh) + (size_t)key * DH + (i % LPR) * 64);
}

// The two S^T sub-tiles of a key tile, each 32 keys (rows) x 32 queries (columns); accumulator element r of a
// lane is key 8*(r/4) + 4*(lane/32) + r%4, query lane%32.  The two chains of dependent matrix-core products
// alternate, so that one runs while the other waits for its accumulator.
template <int DH, bool F16>
__device__ inline void score_pair(const uint16_t* Ks, const typename Elem16<F16>::vec8* qf, int lane, f16v& s0, f16v& s1) {
  typedef typename Elem16<F16>::vec8 vec8;
  constexpr int KLD = AttnSmem<DH>::KLD;
#pragma unroll
  for (int i = 0; i < 16; i++) s0[i] = s1[i] = 0.f;
  const uint16_t* row0 = Ks + (lane & 31) * KLD + 8 * (lane >> 5);
  const uint16_t* row1 = row0 + 32 * KLD;
#pragma unroll
  for (int ks = 0; ks < DH / 16; ks++) {
    const vec8 a0 = *reinterpret_cast<const vec8*>(row0 + 16 * ks);
    const vec8 a1 = *reinterpret_cast<const vec8*>(row1 + 16 * ks);
    s0 = Elem16<F16>::mma(a0, qf[ks], s0);
    s1 = Elem16<F16>::mma(a1, qf[ks], s1);
  }
}

// Pass 1 on one key tile: running row maximum and normaliser (log2 domain).  MASKED = the tile crosses the
// causal edge of some query of the wavefront; the arithmetic on the visible keys is the same in both
// forms, so a query's statistics do not depend on where the query tiles fall.
template <int DH, bool F16, bool MASKED>
__device__ inline void stats_tile(const uint16_t* Ks, const typename Elem16<F16>::vec8* qf, int k0, int kend_q,
                                  float scale_log2e, float& m_run, float& l_run, int lane) {
  const int half = lane >> 5;
  f16v s[2];
  score_pair<DH, F16>(Ks, qf, lane, s[0], s[1]);
  float mx = -INFINITY;
#pragma unroll
  for (int sub = 0; sub < 2; sub++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int key = k0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      if (!MASKED || key < kend_q) mx = fmaxf(mx, s[sub][r]);
    }
  if (!MASKED || mx > -INFINITY) {
    const float m_new = fmaxf(m_run, mx * scale_log2e);  // the scale is positive
    float sum = 0.f;
#pragma unroll
    for (int sub = 0; sub < 2; sub++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int key = k0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
        const float e = fast_exp2(fmaf(s[sub][r], scale_log2e, -m_new));
        sum += (!MASKED || key < kend_q) ? e : 0.f;
      }
    l_run = l_run * fast_exp2(m_run - m_new) + sum;
    m_run = m_new;
  }
}

// One tile of pass 1 with its data movement: statistics from this stage, the next tile into the other stage,
// one barrier, then the fetch of the tile after the next and a touch of lines further ahead (K four tiles on,
// V one tile on for pass 2).  `touch` is the touch issued two tiles ago: it is waited for here, behind the
// fetch that was issued after it.
template <int DH, bool F16>
__device__ __forceinline__ void stats_step(unsigned char* smem, const uint16_t* __restrict__ Kh, const uint16_t* __restrict__ Vh,
                                           const typename Elem16<F16>::vec8* qf, u4v (&kr)[AK * (DH / 8) / 256],
                                           uint32_t& touch, int t, int n_tiles, int kvis_all, int kend_q, int kcap, int L,
                                           float scale_log2e, float& m_run, float& l_run) {
  typedef AttnSmem<DH> SM;
  const int k0 = t * AK, lane = threadIdx.x & 63;
  const uint16_t* Ks = reinterpret_cast<const uint16_t*>(smem + (t & 1) * SM::STAGE);
  if (k0 + AK <= kvis_all)
    stats_tile<DH, F16, false>(Ks, qf, k0, kend_q, scale_log2e, m_run, l_run, lane);
  else
    stats_tile<DH, F16, true>(Ks, qf, k0, kend_q, scale_log2e, m_run, l_run, lane);
  // (no branches in this part: behind the last tile the other stage takes a tile that nobody reads)
  store_k_tile<DH>(reinterpret_cast<uint16_t*>(smem + ((t + 1) & 1) * SM::STAGE), kr);
  asm volatile("" ::"v"(touch));
  __syncthreads();
  load_k_tile<DH>(Kh, t + 2 < n_tiles ? k0 + 2 * AK : 0, L, kr);
  touch = touch_lines<DH>(Kh, Vh, k0 + 4 * AK, k0 + AK, kcap);
}

// O^T += V^T P^T for one 32-key sub-tile.  Matrix-core k-slot (half, i) of product u is key
// sub*32 + 16u + 8*(i/4) + 4*half + i%4, which is accumulator element 8u+i of the score sub-tile.
template <int DH, bool F16>
__device__ inline void pv_subtile(const uint16_t* Vt, int sub, const float* pr, f16v* oacc, int lane) {
  typedef typename Elem16<F16>::vec8 vec8;
  constexpr int VLD = AttnSmem<DH>::VLD;
  const int half = lane >> 5;
#pragma unroll
  for (int u = 0; u < 2; u++) {
    // probabilities enter the matrix cores as a 16-bit head plus a 16-bit remainder (16 or more
    // significant bits), so O is accurate to its own final rounding
    union { uint32_t w[4]; vec8 v; } pb, pl;
#pragma unroll
    for (int i = 0; i < 4; i++) Elem16<F16>::split2(pr[8 * u + 2 * i], pr[8 * u + 2 * i + 1], pb.w[i], pl.w[i]);
#pragma unroll
    for (int mt = 0; mt < DH / 32; mt++) {
      union { u4v u4; vec8 v; } va;  // V^T row 32 mt + lane%32, the lane's eight keys (stored side by side)
      va.u4 = *reinterpret_cast<const u4v*>(Vt + (32 * mt + (lane & 31)) * VLD + sub * 32 + 16 * u + 8 * half);
      oacc[mt] = Elem16<F16>::mma(va.v, pb.v, oacc[mt]);
      oacc[mt] = Elem16<F16>::mma(va.v, pl.v, oacc[mt]);
    }
  }
}

// Column sums of one sub-tile over this wavefront's 32 queries (the 32 lanes of each half): recursive
// halving, 16 values -> 1 value per lane pair.  First the two 16-lane rows of a half trade eight values
// with the row-swap instruction (after it, one register holds a value's two row parts in the even row and
// the other the partner value's in the odd row), then lanes L and 15-L, L and 7-L, L and L^2 trade through
// data-parallel lane permutations, and the two lanes of a pair are added.  pr is used up.
__device__ inline void colsum_subtile(float* pr, float* cs_sub, int lane) {
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const u2v sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(pr[i]), __float_as_uint(pr[i + 8]), false, false);
    pr[i] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  }
  {
    const bool up = (lane & 8) != 0;
#pragma unroll
    for (int i = 0; i < 4; i++) pr[i] = (up ? pr[i + 4] : pr[i]) + lane_perm<0x140>(up ? pr[i] : pr[i + 4]);  // L <-> 15-L
  }
  {
    const bool up = (lane & 4) != 0;
#pragma unroll
    for (int i = 0; i < 2; i++) pr[i] = (up ? pr[i + 2] : pr[i]) + lane_perm<0x141>(up ? pr[i] : pr[i + 2]);  // L <-> 7-L
  }
  {
    const bool up = (lane & 2) != 0;
    pr[0] = (up ? pr[1] : pr[0]) + lane_perm<0x4E>(up ? pr[0] : pr[1]);  // L <-> L^2
  }
  pr[0] += lane_perm<0xB1>(pr[0]);  // L <-> L^1
  if ((lane & 1) == 0) {
    const int r = (lane >> 1) & 15;  // accumulator element whose column sum this lane pair holds
    cs_sub[8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)] = pr[0];
  }
}

// Pass 2 on one key tile: exact probabilities, O^T accumulation (WANT_O), column sums.  The scores of both
// sub-tiles come first so that the exponentials of one overlap the matrix-core work of the other.
template <int DH, bool F16, bool MASKED, bool WANT_O>
__device__ inline void probs_tile(const uint16_t* Ks, const uint16_t* Vt, const typename Elem16<F16>::vec8* qf, f16v* oacc,
                                  float* cs_wave, int k0, int kend_q, float scale_log2e, float m_fold, int lane) {
  const int half = lane >> 5;
  f16v s[2];
  score_pair<DH, F16>(Ks, qf, lane, s[0], s[1]);
#pragma unroll
  for (int sub = 0; sub < 2; sub++) {
    float pr[16];
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int key = k0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
      const float e = fast_exp2(fmaf(s[sub][r], scale_log2e, -m_fold));
      pr[r] = (!MASKED || key < kend_q) ? e : 0.f;
    }
    if (WANT_O) pv_subtile<DH, F16>(Vt, sub, pr, oacc, lane);
    colsum_subtile(pr, cs_wave + sub * 32, lane);
  }
}

template <int DH, bool F16, bool WANT_O>
__device__ inline void probs_pass(unsigned char* smem, const uint16_t* __restrict__ Kh, const uint16_t* __restrict__ Vh,
                                  const typename Elem16<F16>::vec8* qf, f16v* oacc, u4v* kr, u4v* vr, float* sp_row,
                                  int n_tiles, int kvis_all, int kend_q, float scale_log2e, float m_fold, int L, int Ls,
                                  int N) {
  typedef AttnSmem<DH> SM;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* cs = reinterpret_cast<float*>(smem + SM::MAIN);  // [2][4][AK]
  store_k_tile<DH>(reinterpret_cast<uint16_t*>(smem), kr);
  store_v_tile_transposed<DH>(reinterpret_cast<uint16_t*>(smem + SM::K_BYTES), vr);
  __syncthreads();
  if (n_tiles > 1) {
    load_k_tile<DH>(Kh, AK, L, kr);
    load_v_tile<DH>(Vh, AK, L, vr);
  }
  for (int t = 0; t < n_tiles; t++) {
    const int k0 = t * AK;
    unsigned char* stage = smem + (t & 1) * SM::STAGE;
    unsigned char* other = smem + ((t + 1) & 1) * SM::STAGE;
    const uint16_t* Ks = reinterpret_cast<const uint16_t*>(stage);
    const uint16_t* Vt = reinterpret_cast<const uint16_t*>(stage + SM::K_BYTES);
    float* cs_t = cs + (t & 1) * 4 * AK;
    if (k0 + AK <= kvis_all)  // every key visible to every query of the wavefront: no masks
      probs_tile<DH, F16, false, WANT_O>(Ks, Vt, qf, oacc, cs_t + wave * AK, k0, kend_q, scale_log2e, m_fold, lane);
    else
      probs_tile<DH, F16, true, WANT_O>(Ks, Vt, qf, oacc, cs_t + wave * AK, k0, kend_q, scale_log2e, m_fold, lane);
    if (t + 1 < n_tiles) {  // the other stage was last read before the previous barrier
      store_k_tile<DH>(reinterpret_cast<uint16_t*>(other), kr);
      store_v_tile_transposed<DH>(reinterpret_cast<uint16_t*>(other + SM::K_BYTES), vr);
    }
    __syncthreads();
    if (t + 2 < n_tiles) {
      load_k_tile<DH>(Kh, k0 + 2 * AK, L, kr);
      load_v_tile<DH>(Vh, k0 + 2 * AK, L, vr);
    }
    if (tid < AK) {  // this set of column sums is written again two tiles on, behind the next barrier
      const int x = k0 + tid - Ls;
      if (x >= 0 && x < N) sp_row[x] = (cs_t[tid] + cs_t[AK + tid]) + (cs_t[2 * AK + tid] + cs_t[3 * AK + tid]);
    }
  }
}

template <int DH, bool F16>
__global__ __launch_bounds__(256, 2) void attn_bf16_kernel(const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K,
                                                        const uint16_t* __restrict__ V, uint16_t* __restrict__ O,
                                                        float* __restrict__ Spart, int L, int Ls, int N, int Nq, int H,
                                                        int causal, float scale_log2e, int n_qtiles, int B, size_t stride) {
  typedef AttnSmem<DH> SM;
  typedef typename Elem16<F16>::vec8 vec8;
  extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
  unsigned char* smem = attn_smem;
  int bh, qt;  // the query tiles of one (image, head) share K and V: keep them on one XCD
  if (!group_on_xcd(blockIdx.x, n_qtiles, B * H, &bh, &qt)) return;
  qt = n_qtiles - 1 - qt;  // longest (latest) query tile first
  const int h = bh % H, b = bh / H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const size_t head_off = ((size_t)b * H + h) * (size_t)L * DH;
  const uint16_t* Qh = Q + head_off;
  const uint16_t* Kh = K + head_off;
  const uint16_t* Vh = V + head_off;
  // The tiles are laid so that the last one is full: a ragged query count leaves its empty rows in the first
  // tile, the one with the fewest visible keys under the causal mask.
  const int qbase = qt * AQ - (n_qtiles * AQ - Nq);
  const int q = qbase + wave * 32 + (lane & 31);
  // query rows 0 .. N-1 are the visual tokens; rows N .. Nq-1 (prompt tokens) only add to the column sums
  const bool qvalid = q >= 0;
  const int p = Ls + (qvalid ? q : 0);                // sequence position of this lane's query
  const int kend_q = causal ? p + 1 : L;              // keys [0, kend_q) are visible to it
  const int kend = causal ? min(L, Ls + qbase + AQ) : L;  // the tile's last query sees the most
  const int n_tiles = (kend + AK - 1) / AK;
  // keys [0, kvis_all) are visible to every query of this wavefront (its first query sees the fewest)
  const int kvis_all = causal ? min(L, Ls + max(qbase + wave * 32, 0) + 1) : L;

  vec8 qf[DH / 16];
#pragma unroll
  for (int ks = 0; ks < DH / 16; ks++)
    qf[ks] = *reinterpret_cast<const vec8*>(Qh + (size_t)p * DH + 16 * ks + 8 * half);

  // ---------------- pass 1: row maximum and normaliser (log2 domain) ----------------
  // Both passes keep the tile after the next in registers (fetched while the matrix cores work on this one)
  // and write it into the LDS stage that is not being read; one barrier per tile.
  float m_run = -INFINITY, l_run = 0.f;
  u4v kr[AK * (DH / 8) / 256], vr[DH / 32];
  load_k_tile<DH>(Kh, 0, L, kr);
  store_k_tile<DH>(reinterpret_cast<uint16_t*>(smem), kr);
  __syncthreads();
  load_k_tile<DH>(Kh, n_tiles > 1 ? AK : 0, L, kr);  // after the last tile of this pass: tile 0 for pass 2
  // Lines of K four tiles ahead and of V (for pass 2) are touched while this pass runs; a touch is waited
  // for two tiles later, behind the tile fetch that was issued after it.
  const int kcap = min(L, n_tiles * AK);
  uint32_t touch_a = touch_lines<DH>(Kh, Vh, 2 * AK, 0, kcap), touch_b = touch_lines<DH>(Kh, Vh, 3 * AK, 0, kcap);
  for (int t = 0; t < n_tiles; t += 2) {
    stats_step<DH, F16>(smem, Kh, Vh, qf, kr, touch_a, t, n_tiles, kvis_all, kend_q, kcap, L, scale_log2e, m_run, l_run);
    if (t + 1 < n_tiles)
      stats_step<DH, F16>(smem, Kh, Vh, qf, kr, touch_b, t + 1, n_tiles, kvis_all, kend_q, kcap, L, scale_log2e, m_run, l_run);
  }
  asm volatile("" ::"v"(touch_a), "v"(touch_b));
  load_v_tile<DH>(Vh, 0, L, vr);
  {
    const float m_o = __shfl_xor(m_run, 32, 64), l_o = __shfl_xor(l_run, 32, 64);
    const float M = fmaxf(m_run, m_o);  // finite: key 0 is visible to every query
    l_run = l_run * fast_exp2(m_run - M) + l_o * fast_exp2(m_o - M);
    m_run = M;
  }
  // p = 2^(s - m) / l = 2^(s - (m + log2 l)); rows before the first query contribute nothing (2^-inf = 0)
  const float m_fold = qvalid ? m_run + log2f(l_run) : INFINITY;

  // ---------------- pass 2: probabilities, O^T accumulation, column sums ----------------
  f16v oacc[DH / 32];
#pragma unroll
  for (int mt = 0; mt < DH / 32; mt++)
#pragma unroll
    for (int i = 0; i < 16; i++) oacc[mt][i] = 0.f;
  float* sp_row = Spart + (size_t)b * stride + ((size_t)h * n_qtiles + qt) * N;
  if (qbase < N)  // the tile holds visual rows: their output is wanted
    probs_pass<DH, F16, true>(smem, Kh, Vh, qf, oacc, kr, vr, sp_row, n_tiles, kvis_all, kend_q, scale_log2e, m_fold, L, Ls, N);
  else
    probs_pass<DH, F16, false>(smem, Kh, Vh, qf, oacc, kr, vr, sp_row, n_tiles, kvis_all, kend_q, scale_log2e, m_fold, L, Ls, N);
  // visual tokens behind the last key tile received no attention from this query tile
  for (int x = max(0, n_tiles * AK - Ls) + tid; x < N; x += 256) sp_row[x] = 0.f;

  // ---------------- write O: transpose through LDS, 16-byte rows stores ----------------
  if (qbase >= N) return;
  __syncthreads();
  uint16_t* Os = reinterpret_cast<uint16_t*>(smem) + wave * 32 * SM::KLD;
#pragma unroll
  for (int mt = 0; mt < DH / 32; mt++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int d = 32 * mt + 8 * (r >> 2) + 4 * half + (r & 3);
      Os[(lane & 31) * SM::KLD + d] = Elem16<F16>::bits(oacc[mt][r]);
    }
  __syncthreads();
  constexpr int CH = DH / 8;
  for (int idx = lane; idx < 32 * CH; idx += 64) {
    const int ql = idx / CH, ch = idx % CH;
    const int qq = qbase + wave * 32 + ql;
    if (qq >= 0 && qq < N)
      *reinterpret_cast<u4v*>(O + ((size_t)b * N + qq) * ((size_t)H * DH) + (size_t)h * DH + ch * 8) =
          *reinterpret_cast<const u4v*>(Os + ql * SM::KLD + ch * 8);
  }
}

// S[b][x] = (1 / (H Nq)) sum_h sum_tiles partial column sums, in a fixed order: four threads per token take a
// quarter of the partial rows each (the loads of one thread depend on nothing but are issued one after the other),
// their float64 sums are added in order.
__global__ __launch_bounds__(256) void attn_score_reduce(const float* __restrict__ Spart, float* __restrict__ S, int N,
                                                         int Nq, int H, int n_qtiles, size_t stride) {
  __shared__ double part[4][64];
  const int b = blockIdx.y, xl = threadIdx.x & 63, q = threadIdx.x >> 6, x = blockIdx.x * 64 + xl;
  const int rows = H * n_qtiles, per = (rows + 3) / 4;
  double acc = 0.0;
  if (x < N) {
    const float* sp = Spart + (size_t)b * stride + x;
    const int i1 = min(rows, (q + 1) * per);
    for (int i = q * per; i < i1; i++) acc += (double)sp[(size_t)i * N];
  }
  part[q][xl] = acc;
  __syncthreads();
  if (q == 0 && x < N)
    S[(size_t)b * N + x] = (float)(((part[0][xl] + part[1][xl]) + (part[2][xl] + part[3][xl])) / ((double)H * (double)Nq));
}

// ---------------- float32 storage: plain-ALU correctness path ----------------
// One wavefront per (image, head, query): two passes over the keys, float accumulation.
template <int DH>
__global__ __launch_bounds__(64) void attn_f32_rows(const float* __restrict__ Q, const float* __restrict__ K,
                                                    const float* __restrict__ V, float* __restrict__ O,
                                                    float* __restrict__ stats, int L, int Ls, int N, int Nq, int H,
                                                    int causal, float scale, size_t stride) {
  __shared__ float qs[DH];
  const int q = blockIdx.x, h = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  const size_t head_off = ((size_t)b * H + h) * (size_t)L * DH;
  const int p = Ls + q, kend = causal ? p + 1 : L;
  for (int d = lane; d < DH; d += 64) qs[d] = Q[head_off + (size_t)p * DH + d];
  __syncthreads();
  float m = -INFINITY, l = 0.f;
  for (int k = lane; k < kend; k += 64) {
    const float* kr = K + head_off + (size_t)k * DH;
    float s = 0.f;
    for (int d = 0; d < DH; d++) s += qs[d] * kr[d];
    s *= scale;
    const float mn = fmaxf(m, s);
    l = l * expf(m - mn) + expf(s - mn);
    m = mn;
  }
  float M = m;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
  l = (m > -INFINITY) ? l * expf(m - M) : 0.f;
  l = wave_sum(l);
  float acc[DH];
#pragma unroll
  for (int d = 0; d < DH; d++) acc[d] = 0.f;
  for (int k = lane; k < kend; k += 64) {
    const float* kr = K + head_off + (size_t)k * DH;
    const float* vr = V + head_off + (size_t)k * DH;
    float s = 0.f;
    for (int d = 0; d < DH; d++) s += qs[d] * kr[d];
    const float pk = expf(s * scale - M) / l;
#pragma unroll
    for (int d = 0; d < DH; d++) acc[d] += pk * vr[d];
  }
  if (q < N) {  // prompt rows (q >= N) only leave their softmax statistics
    float* out = O + ((size_t)b * N + q) * ((size_t)H * DH) + (size_t)h * DH;
#pragma unroll
    for (int d = 0; d < DH; d++) {
      const float v = wave_sum(acc[d]);
      if (lane == (d & 63)) out[d] = v;
    }
  }
  if (lane == 0) {
    stats[(size_t)b * stride + ((size_t)h * Nq + q) * 2] = M;
    stats[(size_t)b * stride + ((size_t)h * Nq + q) * 2 + 1] = l;
  }
}

// One workgroup per (image, visual key x): S[b][x] = mean over heads and the Nq query rows of A[.., q, x].
template <int DH>
__global__ __launch_bounds__(256) void attn_f32_cols(const float* __restrict__ Q, const float* __restrict__ K,
                                                     const float* __restrict__ stats, float* __restrict__ S, int L,
                                                     int Ls, int N, int Nq, int H, int causal, float scale, size_t stride) {
  __shared__ double red[256];
  const int x = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  double acc = 0.0;
  for (int idx = tid; idx < H * Nq; idx += 256) {
    const int h = idx / Nq, q = idx % Nq;
    if (causal && x > q) continue;
    const size_t head_off = ((size_t)b * H + h) * (size_t)L * DH;
    const float* qr = Q + head_off + (size_t)(Ls + q) * DH;
    const float* kr = K + head_off + (size_t)(Ls + x) * DH;
    float s = 0.f;
    for (int d = 0; d < DH; d++) s += qr[d] * kr[d];
    const float M = stats[(size_t)b * stride + ((size_t)h * Nq + q) * 2], l = stats[(size_t)b * stride + ((size_t)h * Nq + q) * 2 + 1];
    acc += (double)(expf(s * scale - M) / l);
  }
  red[tid] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  if (tid == 0) S[(size_t)b * N + x] = (float)(red[0] / ((double)H * (double)Nq));
}

int launch_attention(const Plan& pl, int dtype, int causal, const void* Q, const void* K, const void* V, void* O,
                     float* S, float* Spart, hipStream_t st) {
  if (dtype == TC_BF16 || dtype == TC_F16) {
    const dim3 grid(grid_for_groups(pl.n_qtiles, pl.B * pl.H));
    const float sl2 = pl.scale * 1.4426950408889634f;
    const uint16_t *q = (const uint16_t*)Q, *k = (const uint16_t*)K, *v = (const uint16_t*)V;
    uint16_t* o = (uint16_t*)O;
#define TC_ATTN16(DH_, F16_) \
  do {                                                                                                                  \
    constexpr int shm = AttnSmem<DH_>::TOTAL;                                                                             \
    if (shm > 64 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel<DH_, F16_>),                \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, shm) != hipSuccess)            \
      return TC_ERR_HIP;                                                                                                  \
    TC_TIMED(PK_ATTN, 0, st, (attn_bf16_kernel<DH_, F16_><<<grid, 256, shm, st>>>(q, k, v, o, Spart, pl.L, pl.Ls, pl.N, pl.Nq, pl.H, causal, sl2, pl.n_qtiles, pl.B, pl.spart_stride))); \
  } while (0)
    if (pl.dh == 128) {
      if (dtype == TC_F16) TC_ATTN16(128, true); else TC_ATTN16(128, false);
    } else {
      if (dtype == TC_F16) TC_ATTN16(64, true); else TC_ATTN16(64, false);
    }
#undef TC_ATTN16
    if (S) TC_TIMED(PK_ATTN_REDUCE, 0, st, (attn_score_reduce<<<dim3((pl.N + 63) / 64, pl.B), 256, 0, st>>>(Spart, S, pl.N, pl.Nq, pl.H, pl.n_qtiles, pl.spart_stride)));
  } else {
    const dim3 grid(pl.Nq, pl.H, pl.B);
    if (pl.dh == 128) {
      TC_TIMED(PK_ATTN, 0, st, (attn_f32_rows<128><<<grid, 64, 0, st>>>((const float*)Q, (const float*)K, (const float*)V, (float*)O, Spart,
                                              pl.L, pl.Ls, pl.N, pl.Nq, pl.H, causal, pl.scale, pl.spart_stride)));
      if (S) TC_TIMED(PK_ATTN_REDUCE, 0, st, (attn_f32_cols<128><<<dim3(pl.N, pl.B), 256, 0, st>>>((const float*)Q, (const float*)K, Spart, S, pl.L,
                                                                   pl.Ls, pl.N, pl.Nq, pl.H, causal, pl.scale, pl.spart_stride)));
    } else {
      TC_TIMED(PK_ATTN, 0, st, (attn_f32_rows<64><<<grid, 64, 0, st>>>((const float*)Q, (const float*)K, (const float*)V, (float*)O, Spart, pl.L,
                                             pl.Ls, pl.N, pl.Nq, pl.H, causal, pl.scale, pl.spart_stride)));
      if (S) TC_TIMED(PK_ATTN_REDUCE, 0, st, (attn_f32_cols<64><<<dim3(pl.N, pl.B), 256, 0, st>>>((const float*)Q, (const float*)K, Spart, S, pl.L,
                                                                  pl.Ls, pl.N, pl.Nq, pl.H, causal, pl.scale, pl.spart_stride)));
    }
  }
  return check_launch();
}

}  // namespace tc
