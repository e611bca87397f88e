// Batched symmetric eigensolver for the Gram matrices: two-sided block-Jacobi.
//
// G (Np x Np, Np a multiple of 64) is split into blocks of b = 32 rows/columns.  One step pairs the
// blocks by a round-robin tournament; for every pair (p,q) the 64x64 subproblem
// [[G_pp G_pq][G_qp G_qq]] is diagonalised approximately by one cyclic sweep of plane rotations held
// in LDS (jacobi_solve), giving an orthogonal 64x64 matrix R.  Then every 64x64 tile of G that the
// step's pairs (I,J) span is replaced by R_I^T G_IJ R_J and the eigenvector columns by U_J R_J
// (jacobi_update), both as small matrix products on the matrix cores.  nblk-1 steps make a sweep;
// sweeps repeat until the off-diagonal mass of G, measured after every sweep, is below the
// tolerance, per image, with the iteration count fixed on the host and converged images skipped on
// the device.  Close to convergence the rotation kernel also leaves alone every pair whose visit would
// remove a negligible mass (R = I and a flag in the solver state), and the updates skip what such
// pairs span.
// After the Gram kernel has filled G in full, only its upper triangle is maintained: the blocks above
// the block diagonal by the tile update, the blocks of a pair itself by the rotation kernel.
// On exit diag(G) holds the eigenvalues sigma_i^2 and U the left singular vectors of O
// (Section 3.3.1: Z = U Sigma V^T  =>  Z Z^T = U Sigma^2 U^T).
#include <mutex>

#include "tc_internal.h"

namespace tc {

typedef __attribute__((ext_vector_type(4))) double d4;
typedef __attribute__((ext_vector_type(4))) float f4;

// 16x16x4 matrix-core product for both element types.  A: lane holds A[lane%16][lane/16];
// B: lane holds B[lane/16][lane%16]; accumulator element j of a lane is C[row(j)][lane%16].
// Which four of the 64 contraction indices one product covers is free as long as A and B agree:
// both updates give product ks the indices 4 ks .. 4 ks + 3 (lane / 16 picks one of them), and pad
// their LDS rows (66 doubles, 68 floats) so that the operand reads of a wavefront are conflict-free.
template <typename T> struct MM;
template <> struct MM<double> {
  typedef d4 acc_t;
  typedef __attribute__((ext_vector_type(2))) double pair_t;
  __device__ static inline acc_t mma(double a, double b, acc_t c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
  }
  __device__ static inline int row(int j, int lane) { return 4 * j + (lane >> 4); }
};
template <> struct MM<float> {
  typedef f4 acc_t;
  typedef __attribute__((ext_vector_type(2))) float pair_t;
  __device__ static inline acc_t mma(float a, float b, acc_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  __device__ static inline int row(int j, int lane) { return 4 * (lane >> 4) + j; }
};

constexpr int SLD = JT + 1;  // padded leading dimension of the LDS tiles

// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void jacobi_init_u(float* __restrict__ U, int Np) {
  const size_t n2 = (size_t)Np * Np;
  float* Ub = U + (size_t)blockIdx.y * n2;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += (size_t)gridDim.x * blockDim.x)
    Ub[i] = ((i / JB) % Np == (i / ((size_t)JB * Np)) * JB + i % JB) ? 1.f : 0.f;  // row == column in the block-column layout
}

// ||G||_F^2 of every image, in two steps with fixed summation orders: one workgroup per 32 rows
// writes a partial sum, then one wavefront per image adds the partials and sets up the solver state.
template <typename T>
__global__ __launch_bounds__(256) void jacobi_norm_partial(const T* __restrict__ G, double* __restrict__ part, int Np,
                                                           int nblk) {
  __shared__ double red[4];
  const T* rows = G + ((size_t)blockIdx.y * Np + (size_t)blockIdx.x * JB) * Np;
  double s = 0.0;
  for (int i = threadIdx.x; i < JB * Np; i += 256) { const double v = (double)rows[i]; s += v * v; }
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) part[(size_t)blockIdx.y * nblk + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}
__global__ void jacobi_init_state(const double* __restrict__ part, EigState* __restrict__ state, int nblk) {
  const int b = blockIdx.x, lane = threadIdx.x;  // one wavefront per image
  double s = 0.0;
  for (int i = lane; i < nblk; i += 64) s += part[(size_t)b * nblk + i];
  s = wave_sum(s);
  for (int i = lane; i < MAX_NVIS / JT; i += 64) state[b].rot_steps[i] = 0u;
  if (lane == 0) {
    state[b].norm2 = s;
    state[b].thr2 = 0.0;
    state[b].done = s > 0.0 ? 0 : 1;
    state[b].sweeps = 0;
    state[b].tiles = 0u;
  }
}

// ---------------------------------------------------------------------------------------
// Plane rotation that annihilates a_ij of [[a_ii a_ij][a_ij a_jj]] (i < j): J = [[c s][-s c]].
// tan(theta) only has to be accurate to single precision (a less exact angle leaves a residual of
// relative size 1e-7, removed by the next sweep), so it comes from the hardware reciprocal and
// square-root approximations in float; c is then refined to full precision so that c^2 + s^2 = 1
// holds to the rounding of T and the accumulated transformation stays orthogonal.
// Of the two rotations that annihilate a_ij the one that leaves the larger diagonal entry at the
// smaller index is taken (it differs from the small-angle one by a quarter turn): keeping the
// diagonal sorted while it converges saves sweeps.
__device__ inline void rotation(double aii, double ajj, double aij, double* c, double* s) {
  // tan(theta) and the first guess of cos(theta) in float (the difference a_jj - a_ii is formed in
  // double first); out-of-range ratios end as inf or NaN and mean "no rotation"
  float tf = 0.f;
  if (aij != 0.0) {
    const float zf = (float)(ajj - aii) * __builtin_amdgcn_rcpf((float)(2.0 * aij));
    const float az = fabsf(zf);
    if (az < 1e18f) {  // false for inf and NaN
      tf = __builtin_amdgcn_rcpf(az + __builtin_amdgcn_sqrtf(fmaf(az, az, 1.f)));
      tf = zf < 0.f ? -tf : tf;
    }
  }
  const double t = (double)tf;
  const double x = 1.0 + t * t;  // in [1, 2]
  double y = (double)__builtin_amdgcn_rsqf(fmaf(tf, tf, 1.f));
  y = y * (1.5 - 0.5 * x * y * y);
  y = y * (1.5 - 0.5 * x * y * y);
  const double cc = y, ss = y * t;
  const bool swap = (aii - t * aij) < (ajj + t * aij);  // new a_ii < new a_jj
  *c = swap ? -ss : cc;
  *s = swap ? cc : ss;
}
__device__ inline void rotation(float aii, float ajj, float aij, float* c, float* s) {
  float t = 0.f;
  if (aij != 0.f) {
    const float z = (ajj - aii) * __builtin_amdgcn_rcpf(2.f * aij);
    const float az = fabsf(z);
    if (az < 1e18f) {
      t = __builtin_amdgcn_rcpf(az + __builtin_amdgcn_sqrtf(1.f + az * az));
      t = z < 0.f ? -t : t;
    }
  }
  const float x = 1.f + t * t;
  float y = __builtin_amdgcn_rsqf(x);
  y = y * (1.5f - 0.5f * x * y * y);
  const float cc = y, ss = y * t;
  const bool swap = (aii - t * aij) < (ajj + t * aij);
  *c = swap ? -ss : cc;
  *s = swap ? cc : ss;
}

// One workgroup (8 wavefronts) per block pair: load the 64x64 subproblem, one cyclic sweep of plane
// rotations in the round-robin order, emit the accumulated orthogonal matrix R.
//
// The 64 indices sit in 32 "seats": the 32 seats of a step are its 32 disjoint rotations.  In a
// full sweep (CROSS = false, 63 steps, every index pair once) the seats follow a round-robin
// tournament: seat i of step st holds top = (st+i) mod 63 (63 for seat 0) and bottom = (st-i) mod 63,
// every index advances by one per step (the pairs round_robin_pair() enumerates).  In a cross sweep
// (CROSS = true, 32 steps) only pairs with one index in each of the two blocks are rotated:
// top = i, bottom = 32 + (i + st) mod 32.  A rotation is stored in seat orientation: top' = c top - s bottom,
// bottom' = s top + c bottom.
//   * S is symmetric and lives in LDS as 2x2 blocks (rows of seat I) x (columns of seat J), I <= J.
//     Storage is by seat, not by index: plane 0 holds the (top,top),(top,bottom) pair of every
//     block, plane 1 the (bottom,top),(bottom,bottom) pair, so a lane reads a block with two
//     16-byte loads that are contiguous across lanes.  Since the indices move between seats by the
//     same permutation every step, each rotated element has a fixed destination slot (computed once
//     per lane); it is written there in a second buffer, and the two buffers swap roles every step.
//     Of a diagonal block (I,I) only tt, tb and bb are kept.
//   * The 496 off-diagonal blocks have one lane each on eight wavefronts, the seat pair of a lane
//     fixed for the whole kernel.
//   * R never touches LDS for arithmetic: lane r holds row r of R in registers with the columns in
//     seat order -- wavefront w owns seats 4w..4w+3 -- so every step rotates fixed register pairs;
//     afterwards the columns move one seat along the tournament cycle, a register renaming inside a
//     wavefront plus one column handed to each neighbouring wavefront through a small LDS buffer.
//     After 63 steps the seats are back in their starting order.
//   * One barrier per step.  While the eight wavefronts apply the rotations of step st to S and to
//     R, a ninth computes the rotations of step st+1: lane i evaluates the three elements of seat
//     i's next pivot straight from the old S and the current rotations (three 2x2 blocks, 18
//     multiply-adds, same operation order as the block lanes) instead of waiting for the updated
//     S.  These lanes also own the diagonal blocks: the two diagonal elements they evaluate are
//     the new diagonal of their seat, and the element a rotation annihilates is stored as zero.
//     The rotation table and the hand-over buffers alternate between two copies like S.
//     Measured alternatives that were slower on MI355X: rotations computed after the S update (two
//     barriers per step), every lane computing its own rotation, wavefronts specialised for S and
//     for R, one block per lane on 12 wavefronts, and index/address lookup tables in LDS or global
//     memory.  Alone on a compute unit a workgroup is bound by the latency chain of the rotation
//     wavefront, three per compute unit by LDS bandwidth.
// Value held by lane `l` (l uniform over the wavefront), delivered through a scalar register.
__device__ inline float lane_value(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ inline double lane_value(double v, int l) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), l);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
  return __hiloint2double(hi, lo);
}

constexpr int SOLVE_WAVES = 8;                          // wavefronts that hold blocks of S and columns of R
constexpr int SOLVE_THREADS = 64 * (SOLVE_WAVES + 1);   // plus the rotation wavefront
// Declared bound of the kernel.  With a bound of 9 wavefronts the compiler derives "at most 7
// wavefronts per SIMD" from the wave slots and pads the register allocation to 65 (72 allocated),
// after which only two workgroups fit a compute unit; a bound of 10 leaves the allocation alone and
// three fit as long as the kernel needs no more than 64 registers (which waves_per_eu(8) on the
// kernel makes the register allocator's budget).
constexpr int SOLVE_BOUND = 64 * (SOLVE_WAVES + 2);
constexpr int SEATS = JB / SOLVE_WAVES;                 // seats per wavefront
constexpr int N_BLOCKS = JB * (JB + 1) / 2;             // stored blocks, diagonal ones included
constexpr int N_OFFDIAG = JB * (JB - 1) / 2;            // blocks with a lane of their own
static_assert(N_OFFDIAG <= 64 * SOLVE_WAVES, "one off-diagonal block per lane");

__device__ inline int next63(int x) { return x == 62 ? 0 : x + 1; }

template <typename T>
struct alignas(2 * sizeof(T)) Pair2 {
  T x, y;
};

// Seat position p in [0,64): p < 32 is the top of seat p, p >= 32 the bottom of seat p - 32.
// Where the index sitting at position p moves in one step, and where the index that arrives at p
// comes from.
template <bool CROSS>
__device__ inline int next_position(int p) {
  if (CROSS) return p < JB ? p : JB + ((p - JB) + JB - 1) % JB;  // tops stay, bottoms move one seat down
  if (p == 0) return 0;                                          // seat 0's top never moves
  if (p == 1) return JB;                                         // top of seat 1 -> bottom of seat 0
  if (p < JB) return p - 1;                                      // tops move towards seat 1
  if (p == JT - 1) return JB - 1;                                // bottom of seat 31 -> top of seat 31
  return p + 1;                                                  // bottoms move away from seat 0
}
template <bool CROSS>
__device__ inline int prev_position(int p) {
  if (CROSS) return p < JB ? p : JB + ((p - JB) + 1) % JB;
  if (p == 0) return 0;
  if (p == JB) return 1;
  if (p < JB - 1) return p + 1;
  if (p == JB - 1) return JT - 1;
  return p - 1;
}

__device__ inline int block_id(int I, int J) { return I * JB - I * (I - 1) / 2 + (J - I); }  // I <= J

// Slot (in elements of one buffer) of the symmetric element whose row sits at position a and whose
// column sits at position b.
__device__ inline int slot_of(int a, int b) {
  int I = a & (JB - 1), kr = a >> 5, J = b & (JB - 1), kc = b >> 5;
  if (I > J || (I == J && kr > kc)) { int t = I; I = J; J = t; t = kr; kr = kc; kc = t; }
  return kr * (2 * N_BLOCKS) + 2 * block_id(I, J) + kc;
}

template <typename T, bool CROSS>
__global__ __launch_bounds__(SOLVE_BOUND) __attribute__((amdgpu_waves_per_eu(8, 8))) void jacobi_solve(T* __restrict__ G, T* __restrict__ R,
                                                            EigState* __restrict__ state, int Np, int nblk,
                                                            int step, int img0, int nimg, int inner_steps, int count_work) {
  // all pairs of an image on the XCD that runs the image's tile updates: the blocks they have just
  // written are read from that L2, and so is R by the updates that follow
  const int P = nblk / 2;
  int img, pair;
  if (!group_on_xcd(blockIdx.x, P, nimg, &img, &pair)) return;
  const int b = img0 + img;
  const int done = state[b].done;  // tested after the loads below have been issued
  const double thr2 = state[b].thr2;
  constexpr int BUF = 4 * N_BLOCKS;  // elements of one buffer: two planes of N_BLOCKS pairs
  constexpr int STAGE = JT * SLD;    // the finished R is staged here for row-contiguous stores
  constexpr int XCOPIES = CROSS ? 1 : 2;
  __shared__ __attribute__((aligned(16))) T SB[(2 * BUF > STAGE ? 2 * BUF : STAGE)];
  __shared__ T xch[2][XCOPIES][SOLVE_WAVES][JT];  // columns of R handed to the neighbouring wavefront: [parity][top/bottom]
  __shared__ Pair2<T> rcs[2][JB];                  // (c, z) of every seat, [parity]
  __shared__ double mass[SOLVE_WAVES + 1];         // what this visit would remove, per wavefront
  int p, q;
  round_robin_pair(nblk, step, pair, &p, &q);
  T* Gb = G + (size_t)b * Np * Np;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool rwave = wave == SOLVE_WAVES;  // the rotation wavefront
  // Indices at step 0.  Full sweep: top_i = i, top_0 = 63, bottom_i = (63 - i) mod 63.
  // Cross sweep: top_i = i stays, bottom_i = 32 + (i + st) mod 32.
  auto top0 = [](int i) { return CROSS ? i : (i == 0 ? 63 : i); };
  auto bot0 = [](int i) { return CROSS ? JB + i : (63 - i) % 63; };
  auto next_top = [](int x) { return CROSS || x == 63 ? x : next63(x); };
  auto next_bot = [](int x) { return CROSS ? (x == JT - 1 ? JB : x + 1) : next63(x); };
  // Element {r,c} of the subproblem, r and c in 0..63 (first the rows and columns of block p, then
  // of block q), lives in memory at its place in the upper triangle: block (q,p) is not stored, and of
  // the diagonal blocks only the upper triangle is kept up to date.
  auto gaddr = [&](int r, int c) {
    if (r > c) { const int t = r; r = c; c = t; }
    const int gr = (r < JB ? p * JB + r : q * JB + r - JB), gc = (c < JB ? p * JB + c : q * JB + c - JB);
    return Gb + (size_t)gr * Np + gc;
  };
  auto gload = [&](int r, int c) { return *gaddr(r, c); };
  // the off-diagonal block of S this lane owns (wavefronts 0..7): row I of the strict upper triangle holds JB-1-I blocks
  const bool act = !rwave && tid < N_OFFDIAG;
  int sI = 0, sJ = act ? tid : 0;
  while (sJ >= JB - 1 - sI) { sJ -= JB - 1 - sI; sI++; }
  sJ += sI + 1;
  // the seat of a rotation lane
  const int seat = lane & (JB - 1);
  int rt = top0(seat), rb = bot0(seat);  // indices in the seat
  if (rwave) sI = sJ = seat;
  const int rd = 2 * block_id(sI, sJ);  // this lane's (tt,tb) pair; (bt,bb) sits 2*N_BLOCKS further
  // destinations of the rotated elements in the other buffer (a rotation lane only uses wtb: where
  // the element it annihilates goes)
  const int pTI = next_position<CROSS>(sI), pBI = next_position<CROSS>(JB + sI);
  const int pTJ = next_position<CROSS>(sJ), pBJ = next_position<CROSS>(JB + sJ);
  const int wtt = slot_of(pTI, pTJ), wtb = slot_of(pTI, pBJ), wbt = slot_of(pBI, pTJ), wbb = slot_of(pBI, pBJ);
  // rotation lanes: the next pivot of the seat consists of a_xx, a_xy, a_yy, where x and y are the
  // positions whose indices arrive in this seat (always in two different seats Sx, Sy).  a_xx and
  // a_yy come from the diagonal blocks of Sx and Sy, a_xy from the block of the two seats.
  const int px = prev_position<CROSS>(seat), py = prev_position<CROSS>(JB + seat);
  const int Sx = px & (JB - 1), Sy = py & (JB - 1);
  const bool kx = px >= JB, ky = py >= JB;  // bottom of its seat?
  const bool swp = Sx > Sy;                 // the stored block is (Sy,Sx): a_xy is read as a_yx
  const int rdx = 2 * block_id(Sx, Sx), rdy = 2 * block_id(Sy, Sy);
  const int rdxy = 2 * (swp ? block_id(Sy, Sx) : block_id(Sx, Sy));

  T d_tt = T(0), d_tb = T(0), d_bb = T(0);
  double m = 0.0;  // squares of the elements this visit annihilates: a cross sweep's tops are in block p, its bottoms in block q
  if (act) {
    const int iTI = top0(sI), iBI = bot0(sI), iTJ = top0(sJ), iBJ = bot0(sJ);
    const T ett = gload(iTI, iTJ), etb = gload(iTI, iBJ), ebt = gload(iBI, iTJ), ebb = gload(iBI, iBJ);
    if (done) return;  // uniform over the workgroup
    *reinterpret_cast<Pair2<T>*>(&SB[rd]) = Pair2<T>{ett, etb};
    *reinterpret_cast<Pair2<T>*>(&SB[2 * N_BLOCKS + rd]) = Pair2<T>{ebt, ebb};
    m = (double)etb * etb + (double)ebt * ebt;
    if (!CROSS) m += (double)ett * ett + (double)ebb * ebb;
  } else if (rwave && lane < JB) {  // the diagonal block of the seat
    d_tt = gload(rt, rt); d_tb = gload(rt, rb); d_bb = gload(rb, rb);
    if (done) return;
    *reinterpret_cast<Pair2<T>*>(&SB[rd]) = Pair2<T>{d_tt, d_tb};
    SB[2 * N_BLOCKS + rd + 1] = d_bb;
    m = (double)d_tb * d_tb;
  } else if (done) {
    return;
  }
  if (thr2 > 0.0) {  // uniform over the workgroup
    m = wave_sum(m);
    if (lane == 0) mass[wave] = m;
  }
  T rtop[SEATS], rbot[SEATS];  // columns of R in seat order (wavefronts 0..7), R = I at the start
#pragma unroll
  for (int k = 0; k < SEATS; k++) {
    const int i = SEATS * (rwave ? 0 : wave) + k;
    rtop[k] = (lane == top0(i)) ? T(1) : T(0);
    rbot[k] = (lane == bot0(i)) ? T(1) : T(0);
  }
  auto store_rotation = [&](int par, T att, T atb, T abb) {
    // rotation() wants the pair ordered by index; a rotation is stored in seat orientation
    // (top' = c top - z bottom, bottom' = z top + c bottom)
    const bool flip = rt > rb;
    T c, s;
    rotation(flip ? abb : att, flip ? att : abb, atb, &c, &s);
    rcs[par][seat] = Pair2<T>{c, flip ? -s : s};
    rt = next_top(rt);
    rb = next_bot(rb);
  };
  if (rwave && lane < JB && inner_steps > 0) store_rotation(0, d_tt, d_tb, d_bb);  // rotations of step 0
  __syncthreads();
  if (thr2 > 0.0) {
    double tot = 0.0;
#pragma unroll
    for (int k = 0; k <= SOLVE_WAVES; k++) tot += mass[k];
    if (2.0 * tot <= thr2) {  // nothing worth removing: R = I, G stays as it is, the updates skip this pair
      T* Rb = R + ((size_t)b * P + pair) * JT * JT;
      for (int e = tid; e < JT * JT; e += SOLVE_THREADS) Rb[e] = (e >> 6) == (e & 63) ? T(1) : T(0);
      if (tid == 0) state[b].skip[pair] = 1;
      return;
    }
  }
  if (tid == 0) {  // no other workgroup touches this pair's slots during the launch
    state[b].skip[pair] = 0;
    if (count_work) state[b].rot_steps[pair] += (unsigned)inner_steps;  // only under the profiling entry point, which reads it
  }

  for (int st = 0; st < inner_steps; st++) {  // a whole sweep brings the seats back to their starting order
    const int par = st & 1, cur = par * BUF, nxt = BUF - cur;
    const bool more = st + 1 < inner_steps;  // after the last step no further rotations are needed
    if (rwave) {
      if (lane < JB) {
        // ---- the next pivot, evaluated from the current S and the current rotations ---------------
        // element (kr, kc) of J_I^T B J_J for the block at pair slot r, in the order the block lanes use
        auto element = [&](int r, bool isdiag, Pair2<T> rI, Pair2<T> rJ, bool kr, bool kc) {
          const Pair2<T> et = *reinterpret_cast<const Pair2<T>*>(&SB[cur + r]);
          const Pair2<T> eb = *reinterpret_cast<const Pair2<T>*>(&SB[cur + 2 * N_BLOCKS + r]);
          const T ebt = isdiag ? et.y : eb.x;
          const T uI0 = kr ? rI.y : rI.x, uI1 = kr ? rI.x : -rI.y;
          const T uJ0 = kc ? rJ.y : rJ.x, uJ1 = kc ? rJ.x : -rJ.y;
          const T f0 = uI0 * et.x + uI1 * ebt, f1 = uI0 * et.y + uI1 * eb.y;
          return uJ0 * f0 + uJ1 * f1;
        };
        const Pair2<T> rX = rcs[par][Sx], rY = rcs[par][Sy];
        const T axx = element(rdx, true, rX, rX, kx, kx), ayy = element(rdy, true, rY, rY, ky, ky);
        SB[nxt + rd] = axx;                      // the seat's new diagonal ((top,bottom) comes from a block lane)
        SB[nxt + 2 * N_BLOCKS + rd + 1] = ayy;
        // the element this step's rotation annihilates, at its new place: not an exact zero (the angle
        // is only good to single precision), and since this S goes back to G, what is left of the
        // element has to stay in it (dropping it would not be a similarity transformation)
        const Pair2<T> rM = rcs[par][seat];
        SB[nxt + wtb] = element(rd, true, rM, rM, false, true);
        if (more) {
          const T axy = element(rdxy, false, swp ? rY : rX, swp ? rX : rY, swp ? ky : kx, swp ? kx : ky);
          store_rotation(par ^ 1, axx, axy, ayy);
        }
      }
    } else {
      // ---- S <- J^T S J ---------------------------------------------------------------------------
      if (act) {
        const Pair2<T> rI = rcs[par][sI], rJ = rcs[par][sJ];
        const Pair2<T> et = *reinterpret_cast<const Pair2<T>*>(&SB[cur + rd]);
        const Pair2<T> eb = *reinterpret_cast<const Pair2<T>*>(&SB[cur + 2 * N_BLOCKS + rd]);
        const T cI = rI.x, zI = rI.y, cJ = rJ.x, zJ = rJ.y;
        const T ftt = cI * et.x - zI * eb.x, fbt = zI * et.x + cI * eb.x;  // rows of seat I
        const T ftb = cI * et.y - zI * eb.y, fbb = zI * et.y + cI * eb.y;
        SB[nxt + wtt] = cJ * ftt - zJ * ftb;                                // columns of seat J
        SB[nxt + wtb] = zJ * ftt + cJ * ftb;
        SB[nxt + wbt] = cJ * fbt - zJ * fbb;
        SB[nxt + wbb] = zJ * fbt + cJ * fbb;
      }
      // ---- R <- R J on this wavefront's seats -----------------------------------------------------
      // one LDS read per lane, then scalar broadcasts: lane k (k < SEATS) holds the rotation of seat k
      const Pair2<T> mine = rcs[par][SEATS * wave + (lane & (SEATS - 1))];
      if (st > 0) {  // columns handed over by the neighbours during the previous step
        if (CROSS) {
          rbot[SEATS - 1] = xch[par ^ 1][0][(wave + 1) % SOLVE_WAVES][lane];
        } else {
          if (wave < SOLVE_WAVES - 1) rtop[SEATS - 1] = xch[par ^ 1][0][wave + 1][lane];
          if (wave > 0) rbot[0] = xch[par ^ 1][XCOPIES - 1][wave - 1][lane];
        }
      }
#pragma unroll
      for (int k = 0; k < SEATS; k++) {
        const T c = lane_value(mine.x, k), z = lane_value(mine.y, k);
        const T x = rtop[k], y = rbot[k];
        rtop[k] = c * x - z * y;
        rbot[k] = z * x + c * y;
      }
      // move the columns one seat along the cycle
      if (CROSS) {  // tops stay, every bottom moves to the seat before it (seat 0's to seat 31)
        const T out_bot = rbot[0];
#pragma unroll
        for (int k = 0; k < SEATS - 1; k++) rbot[k] = rbot[k + 1];
        xch[par][0][wave][lane] = out_bot;  // becomes the last bottom of the wavefront before
      } else {  // tops move towards seat 1, bottoms away from seat 0
        const T out_top = rtop[0], out_bot = rbot[SEATS - 1], top1 = rtop[1];
        if (wave == 0) {
#pragma unroll
          for (int k = 1; k < SEATS - 1; k++) rtop[k] = rtop[k + 1];  // seat 0's top (index 63) never moves
        } else {
#pragma unroll
          for (int k = 0; k < SEATS - 1; k++) rtop[k] = rtop[k + 1];
        }
        if (wave == SOLVE_WAVES - 1) rtop[SEATS - 1] = rbot[SEATS - 1];  // top_31 <- bottom_31
#pragma unroll
        for (int k = SEATS - 1; k > 0; k--) rbot[k] = rbot[k - 1];
        if (wave == 0) rbot[0] = top1;                                    // bottom_0 <- top_1
        if (wave > 0) xch[par][0][wave][lane] = out_top;                  // becomes the last top of wave-1
        if (wave < SOLVE_WAVES - 1) xch[par][XCOPIES - 1][wave][lane] = out_bot;  // becomes the first bottom of wave+1
      }
    }
    __syncthreads();  // the other S buffer, the next rotations and the handed-over columns are complete
  }
  // The rotated subproblem itself is R^T [[G_pp G_pq][G_qp G_qq]] R: it goes back to G from here (the
  // tile update leaves the tiles on the block diagonal alone).  After a whole sweep the seats are
  // back in their step-0 order, so every lane finds its elements where it put them at the start.
  const int fin = ((inner_steps - 1) & 1) ? 0 : BUF;  // the buffer the last step wrote
  Pair2<T> s_t = Pair2<T>{T(0), T(0)}, s_b = Pair2<T>{T(0), T(0)};
  if (act || (rwave && lane < JB)) {
    s_t = *reinterpret_cast<const Pair2<T>*>(&SB[fin + rd]);
    s_b = *reinterpret_cast<const Pair2<T>*>(&SB[fin + 2 * N_BLOCKS + rd]);
  }
  if (!rwave) {
    if (inner_steps > 0) {
      const int par = (inner_steps - 1) & 1;
      if (CROSS) {
        rbot[SEATS - 1] = xch[par][0][(wave + 1) % SOLVE_WAVES][lane];
      } else {
        if (wave < SOLVE_WAVES - 1) rtop[SEATS - 1] = xch[par][0][wave + 1][lane];
        if (wave > 0) rbot[0] = xch[par][XCOPIES - 1][wave - 1][lane];
      }
    }
  }
  __syncthreads();  // every lane holds its elements of S: the buffers are free
  if (!rwave) {
    // stage R through LDS for row-contiguous stores
#pragma unroll
    for (int k = 0; k < SEATS; k++) {
      const int i = SEATS * wave + k;
      SB[lane * SLD + top0(i)] = rtop[k];
      SB[lane * SLD + bot0(i)] = rbot[k];
    }
  }
  if (act) {
    const int iTI = top0(sI), iBI = bot0(sI), iTJ = top0(sJ), iBJ = bot0(sJ);
    *gaddr(iTI, iTJ) = s_t.x; *gaddr(iTI, iBJ) = s_t.y;
    *gaddr(iBI, iTJ) = s_b.x; *gaddr(iBI, iBJ) = s_b.y;
  } else if (rwave && lane < JB) {
    const int it = top0(seat), ib = bot0(seat);
    *gaddr(it, it) = s_t.x; *gaddr(it, ib) = s_t.y; *gaddr(ib, ib) = s_b.y;
  }
  __syncthreads();
  T* Rb = R + ((size_t)b * P + pair) * JT * JT;
  for (int e = tid; e < JT * JT; e += SOLVE_THREADS) Rb[e] = SB[(e >> 6) * SLD + (e & 63)];
}

// ---------------------------------------------------------------------------------------
// Tile update of G.  Only the 32x32 blocks (r,c) with r <= c are kept up to date (of the diagonal
// blocks the upper triangle), which halves the traffic and keeps the working set of a step inside
// the last-level cache.  The three blocks of a pair itself come back from the rotation kernel, which
// holds R_I^T G_II R_I at its end anyway; here one workgroup takes pairs of block pairs I < J: the
// 64x64 tile spanned by the rows of pair I and the columns of pair J is gathered (a quadrant whose
// block lies below the diagonal is read from its mirror block and transposed on the way into LDS),
// becomes R_I^T G_IJ R_J, and goes back to the stored blocks.  The mirror tile (J,I) is never formed.
constexpr double SKIP_START = 500.0;  // converged block pairs are skipped once off(G) < SKIP_START * tolerance
constexpr int FULL_EVERY = 6;  // one solve in FULL_EVERY is a full 63-step sweep of its subproblem
constexpr int G_CHUNK = 3;  // consecutive tiles handled by one workgroup (2 or 1 when the launch would not fill the chip)

// Tile index t (row-major over the pairs of pairs I < J, row I holds P - 1 - I tiles) -> (I, J).
__device__ inline void decode_tile(int t, int P, int* I, int* J) {
  int i = 0;
  while (t >= P - 1 - i) { t -= P - 1 - i; i++; }
  *I = i;
  *J = t + i + 1;
}

// A workgroup walks over `gchunk` consecutive tiles and software-pipelines them: while the matrix
// cores work on tile k, tile k+1 and its right factor are already in flight in registers, so only
// the first tile of a chunk waits for memory.
//
// Wavefront w owns quadrant (wr, wc) = (w / 2, w % 2) of the tile: it gathers it, and it holds that
// quadrant of both products in its accumulators, as 2 x 2 matrix-core tiles of 16 x 16.  The 16 tile
// columns n of column tile nt are the quadrant's columns 2 n + nt, so the two column tiles of a lane
// are neighbours in memory: right factor, tile rows in LDS, W and the stored Y all move as 16-byte
// pairs.  The left factor stays in registers while consecutive tiles share it; the right factor
// goes through LDS (fetched once per workgroup, and the register file has no room for both factors,
// the next tile and the accumulators: a spilled register costs a full wait on the memory counter in
// the middle of the tile).  Product ks contracts over k = 4 ks + lane / 16.
constexpr int GLDP = JT + 2;  // row pitch of the tile in LDS: even (pairs stay 16-byte aligned), conflict-free reads

template <typename T>
__global__ __launch_bounds__(256, 2) void jacobi_update_g(T* __restrict__ G, const T* __restrict__ R,
                                                       EigState* __restrict__ state, int Np, int nblk, int step,
                                                       int img0, int nimg, int gchunk, int count_work) {
  typedef typename MM<T>::acc_t acc_t;
  typedef typename MM<T>::pair_t T2;  // two neighbouring elements, moved as one 16-byte (8-byte) access
  const int P = nblk / 2, ntiles = P * (P - 1) / 2, nchunks = (ntiles + gchunk - 1) / gchunk;
  int img, chunk;
  if (!group_on_xcd(blockIdx.x, nchunks, nimg, &img, &chunk)) return;
  const int b = img0 + img;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int myskip = tid < P ? state[b].skip[tid] : 0;  // in flight together with the load of `done`
  if (state[b].done) return;
  __shared__ __attribute__((aligned(16))) T X[JT][GLDP];   // the tile, then W
  __shared__ __attribute__((aligned(16))) T RJs[JT][GLDP]; // the right factor R_J
  __shared__ int2 pairs[MAX_NVIS / JT];                     // the two blocks of every pair of this step
  __shared__ int skipped[MAX_NVIS / JT + 1];                // pairs the rotation kernel left alone (R = I)
  const int wr = wave >> 1, wc = wave & 1, l15 = lane & 15, q4 = lane >> 4;
  T* M = G + (size_t)b * Np * Np;
  const T* Rimg = R + (size_t)b * P * JT * JT;
  const int t0 = chunk * gchunk, t1 = min(ntiles, t0 + gchunk);
  if (tid < P) {
    int x, y;
    round_robin_pair(nblk, step, tid, &x, &y);
    pairs[tid] = int2{x, y};
    skipped[tid] = myskip;
  }
  if (count_work && chunk == 0 && wave == 0) {  // under the profiling entry point one wavefront per image counts the tiles processed
    const unsigned sk = __builtin_popcountll(__ballot(myskip != 0));  // P <= 64: all flags sit in this wavefront
    if (lane == 0) state[b].tiles += (unsigned)ntiles - sk * (sk - 1) / 2;
  }
  __syncthreads();
  // a tile between two skipped pairs stays as it is (uniform over the workgroup)
  auto active = [&](int i, int j) { return __builtin_amdgcn_readfirstlane(skipped[i] & skipped[j]) == 0; };
  auto advance = [&](int* i, int* j) {  // the next tile of the row, or the first of the next row
    if (++*j == P) { ++*i; *j = *i + 1; }
  };
  auto blocks_of = [&](int pr, int* blk) {  // uniform over the workgroup
    const int2 v = pairs[pr];
    blk[0] = __builtin_amdgcn_readfirstlane(v.x);
    blk[1] = __builtin_amdgcn_readfirstlane(v.y);
  };
  // Gather of quadrant (wr, wc): for it = 0..7 the column pair 2 l15, 2 l15 + 1 of row q4 + 4 it of
  // the stored block -- the quadrant's own block, or its mirror block when that lies below the
  // block diagonal (then the pair is transposed on the way into LDS).
  auto gather = [&](const int* rowblk, const int* colblk, T2* x) {
    const int br = rowblk[wr], bc = colblk[wc];
    const T* src = (br <= bc ? M + (size_t)(br * JB) * Np + bc * JB : M + (size_t)(bc * JB) * Np + br * JB) + 2 * l15;
#pragma unroll
    for (int it = 0; it < 8; it++) x[it] = *reinterpret_cast<const T2*>(src + (size_t)(q4 + 4 * it) * Np);
  };
  auto load_left = [&](int I, T (*f)[2]) {  // R_I^T as A fragments: A[i][k] = R_I[k][i], rows wr*32 .. +32
    const T* RI = Rimg + (size_t)I * JT * JT + wr * 32 + l15;
#pragma unroll
    for (int ks = 0; ks < 16; ks++) {
      f[ks][0] = RI[(4 * ks + q4) * JT];
      f[ks][1] = RI[(4 * ks + q4) * JT + 16];
    }
  };
  // R_J on its way to LDS: thread moves, for it = 0..7, the column pair 2 (tid % 32) of row tid / 32 + 8 it
  auto fetch_right = [&](int J, T2* x) {
    const T* RJ = Rimg + (size_t)J * JT * JT + (tid >> 5) * JT + 2 * (tid & 31);
#pragma unroll
    for (int it = 0; it < 8; it++) x[it] = *reinterpret_cast<const T2*>(RJ + 8 * it * JT);
  };
  int I, J, rowblk[2], colblk[2], t = t0;
  decode_tile(t0, P, &I, &J);
  while (t < t1 && !active(I, J)) { t++; advance(&I, &J); }
  if (t >= t1) return;
  blocks_of(I, rowblk);
  blocks_of(J, colblk);
  T left[16][2];
  T2 xpre[8], rpre[8];
  // The first left factor goes through the R_J buffer: fetched once per workgroup with 16-byte loads
  // (as fragments straight from memory each wavefront would fetch its half, the workgroup all of it
  // twice, in 8-byte pieces), while the first tile and its right factor are already on their way.
  fetch_right(I, rpre);
  gather(rowblk, colblk, xpre);
#pragma unroll
  for (int it = 0; it < 8; it++) *reinterpret_cast<T2*>(&RJs[(tid >> 5) + 8 * it][2 * (tid & 31)]) = rpre[it];
  fetch_right(J, rpre);
  __syncthreads();
#pragma unroll
  for (int ks = 0; ks < 16; ks++) {
    left[ks][0] = RJs[4 * ks + q4][wr * 32 + l15];
    left[ks][1] = RJs[4 * ks + q4][wr * 32 + 16 + l15];
  }
  asm volatile("" ::: "memory");  // the optimiser may not sink these reads behind the barrier: the buffer is reused after it
  __syncthreads();
  // The prefetched quadrant and right factor go from registers into LDS (a quadrant read from its
  // mirror block is transposed here).  Done for the first tile before the loop and for every later
  // tile at the end of the previous iteration, behind that tile's stores: on that path the compiler
  // can count the eight stores issued after the prefetch loads and leave them in flight (the memory
  // counter is in order; a wait placed at the top of the loop would have to assume the path from the
  // prologue, with nothing behind the loads, and so wait for the stores to be acknowledged).
  auto stage = [&](const int* rowblk, const int* colblk) {
    if (rowblk[wr] <= colblk[wc]) {
#pragma unroll
      for (int it = 0; it < 8; it++) *reinterpret_cast<T2*>(&X[wr * JB + q4 + 4 * it][wc * JB + 2 * l15]) = xpre[it];
    } else {
#pragma unroll
      for (int it = 0; it < 8; it++) {
        X[wr * JB + 2 * l15][wc * JB + q4 + 4 * it] = xpre[it].x;
        X[wr * JB + 2 * l15 + 1][wc * JB + q4 + 4 * it] = xpre[it].y;
      }
    }
#pragma unroll
    for (int it = 0; it < 8; it++) *reinterpret_cast<T2*>(&RJs[(tid >> 5) + 8 * it][2 * (tid & 31)]) = rpre[it];
  };
  stage(rowblk, colblk);
  for (;;) {
    __syncthreads();  // tile and right factor complete in LDS
    // memory traffic for later: the next tile of the chunk that has work to do, and its right factor
    int In = I, Jn = J, tn = t + 1, rowblk_n[2] = {rowblk[0], rowblk[1]}, colblk_n[2];
    advance(&In, &Jn);
    while (tn < t1 && !active(In, Jn)) { tn++; advance(&In, &Jn); }
    const bool more = tn < t1;
    if (more) {
      if (In != I) blocks_of(In, rowblk_n);
      blocks_of(Jn, colblk_n);
    }
    acc_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++) acc[i][j] = acc_t{0, 0, 0, 0};
    // W = R_I^T X.  The operand of product ks + 1 is read from LDS while product ks runs, and the 16
    // loads of the next tile and its right factor are issued one per product step: issued in one
    // burst by all four wavefronts they queue up in the memory pipeline and stall the products.
    const T* gsrc = M;
    const T* rsrc = Rimg;
    if (more) {
      const int br = rowblk_n[wr], bc = colblk_n[wc];
      gsrc = (br <= bc ? M + (size_t)(br * JB) * Np + bc * JB : M + (size_t)(bc * JB) * Np + br * JB) + 2 * l15 + (size_t)q4 * Np;
      rsrc = Rimg + (size_t)Jn * JT * JT + (tid >> 5) * JT + 2 * (tid & 31);
    }
    T2 bb = *reinterpret_cast<const T2*>(&X[q4][wc * 32 + 2 * l15]);
#define TC_PRODUCT1_STEP(ks, PREFETCH)                                                                          \
  {                                                                                                             \
    const T2 cb = bb;                                                                                           \
    if ((ks) + 1 < 16) bb = *reinterpret_cast<const T2*>(&X[4 * ((ks) + 1) + q4][wc * 32 + 2 * l15]);            \
    if (PREFETCH) { /* one running address per stream: sixteen precomputed ones would spill */                   \
      if ((ks) < 8) {                                                                                           \
        xpre[(ks) & 7] = *reinterpret_cast<const T2*>(gsrc);                                                    \
        gsrc += (size_t)4 * Np;                                                                                 \
        asm volatile("" : "+v"(gsrc));                                                                          \
      } else {                                                                                                  \
        rpre[(ks) & 7] = *reinterpret_cast<const T2*>(rsrc + 8 * ((ks) - 8) * JT);                              \
      }                                                                                                         \
    }                                                                                                           \
    __builtin_amdgcn_sched_barrier(0); /* keep the reads ahead of the products (the scheduler would sink them) */ \
    acc[0][0] = MM<T>::mma(left[ks][0], cb.x, acc[0][0]);                                                       \
    acc[0][1] = MM<T>::mma(left[ks][0], cb.y, acc[0][1]);                                                       \
    acc[1][0] = MM<T>::mma(left[ks][1], cb.x, acc[1][0]);                                                       \
    acc[1][1] = MM<T>::mma(left[ks][1], cb.y, acc[1][1]);                                                       \
  }
#pragma unroll
    for (int ks = 0; ks < 16; ks++) TC_PRODUCT1_STEP(ks, more)
#undef TC_PRODUCT1_STEP
    if (more && In != I) load_left(In, left);  // next tile starts a new row of tiles
    __syncthreads();  // every wave has finished reading X
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int j = 0; j < 4; j++)
        *reinterpret_cast<T2*>(&X[wr * 32 + mt * 16 + MM<T>::row(j, lane)][wc * 32 + 2 * l15]) = T2{acc[mt][0][j], acc[mt][1][j]};
    __syncthreads();
    // Y = W R_J
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int j = 0; j < 2; j++) acc[i][j] = acc_t{0, 0, 0, 0};
    {  // operands of product ks + 1 are read from LDS while product ks runs
      T a0 = X[wr * 32 + l15][q4], a1 = X[wr * 32 + 16 + l15][q4];
      T2 bb = *reinterpret_cast<const T2*>(&RJs[q4][wc * 32 + 2 * l15]);
#pragma unroll
      for (int ks = 0; ks < 16; ks++) {
        const T c0 = a0, c1 = a1;
        const T2 cb = bb;
        if (ks + 1 < 16) {
          a0 = X[wr * 32 + l15][4 * (ks + 1) + q4];
          a1 = X[wr * 32 + 16 + l15][4 * (ks + 1) + q4];
          bb = *reinterpret_cast<const T2*>(&RJs[4 * (ks + 1) + q4][wc * 32 + 2 * l15]);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the products (the scheduler would sink them)
        acc[0][0] = MM<T>::mma(c0, cb.x, acc[0][0]);
        acc[0][1] = MM<T>::mma(c0, cb.y, acc[0][1]);
        acc[1][0] = MM<T>::mma(c1, cb.x, acc[1][0]);
        acc[1][1] = MM<T>::mma(c1, cb.y, acc[1][1]);
      }
    }
    __syncthreads();  // W and R_J fully consumed
    // The quadrant of Y goes from the accumulators to its block (rows of block rowblk[wr], columns
    // of block colblk[wc]) as 16-byte column pairs.  A quadrant whose block is only stored as its
    // mirror is first transposed inside the wavefront's own quarter of X (nobody else touches that
    // quarter before the next barrier, and the LDS serves one wavefront's accesses in order).  This
    // way every wavefront issues exactly eight stores per tile on every path: the wait for the
    // prefetched next tile can then leave them in flight (the memory counter is in order and the
    // compiler has to assume the path with the fewest stores behind the loads).
    const int br = rowblk[wr], bc = colblk[wc];
    if (br <= bc) {
      T* dst = M + (size_t)(br * JB) * Np + bc * JB + 2 * l15;
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int j = 0; j < 4; j++)
          *reinterpret_cast<T2*>(dst + (size_t)(mt * 16 + MM<T>::row(j, lane)) * Np) = T2{acc[mt][0][j], acc[mt][1][j]};
    } else {
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int nt = 0; nt < 2; nt++)
#pragma unroll
          for (int j = 0; j < 4; j++) X[wr * 32 + 2 * l15 + nt][wc * 32 + mt * 16 + MM<T>::row(j, lane)] = acc[mt][nt][j];
      T* dst = M + (size_t)(bc * JB) * Np + br * JB + 2 * l15;
#pragma unroll
      for (int it = 0; it < 8; it++)
        *reinterpret_cast<T2*>(dst + (size_t)(q4 + 4 * it) * Np) = *reinterpret_cast<const T2*>(&X[wr * 32 + q4 + 4 * it][wc * 32 + 2 * l15]);
    }
    if (!more) break;
    stage(rowblk_n, colblk_n);
    I = In; J = Jn; t = tn;
    rowblk[0] = rowblk_n[0]; rowblk[1] = rowblk_n[1];
    colblk[0] = colblk_n[0]; colblk[1] = colblk_n[1];
  }
}

// Eigenvector update in float32: U_J <- U_J R_J on the columns of pair J, 64-row slabs.
// U only feeds Eq. 3-6, where an absolute error of 1e-6 per entry is far below the tolerance, so it
// is stored and multiplied in float32 whatever the type of G; R is rounded to float32 on load.
// A workgroup keeps its fragments of R_J in registers and walks over `uchunk` consecutive slabs,
// fetching the next slab into registers while the matrix cores work on the current one (3 slabs
// when the launch has enough workgroups to fill the chip that way, else one slab per workgroup).
// Wavefront w owns rows 16 w .. 16 w + 15 of the slab and all 64 columns, as four matrix-core column
// tiles whose 16 columns n are the slab's columns 4 n + nt: a lane's four results of a row are
// neighbours in memory, and the slab moves in and out as 16-byte accesses (128-byte row pieces).
constexpr int ULD = JT + 4;  // LDS pitch of the slab: 16-byte aligned rows, conflict-free operand reads

template <typename T>
__global__ __launch_bounds__(256) void jacobi_update_u(float* __restrict__ U, const T* __restrict__ R,
                                                       const EigState* __restrict__ state, int Np, int nblk, int step,
                                                       int img0, int nimg, int uchunk) {
  typedef typename MM<T>::pair_t T2;
  const int P = nblk / 2, nslab = Np / JT, nchunk = (nslab + uchunk - 1) / uchunk;
  int img, tile;
  if (!group_on_xcd(blockIdx.x, nchunk * P, nimg, &img, &tile)) return;
  const int b = img0 + img;
  const int J = tile % P, chunk = tile / P;
  const int done = state[b].done, skipJ = state[b].skip[J];  // both loads in flight together
  if (done | skipJ) return;  // skipped by the rotation kernel: R_J = I
  __shared__ __attribute__((aligned(16))) float X[JT][ULD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l15 = lane & 15, q4 = lane >> 4;
  const int slab0 = chunk * uchunk, slab1 = min(nslab, slab0 + uchunk);
  float* M = U + (size_t)b * Np * Np;
  int colblk[2];
  round_robin_pair(nblk, step, J, &colblk[0], &colblk[1]);
  const T* RJ = R + ((size_t)b * P + J) * JT * JT;
  // moving the slab: thread handles columns 4 (tid % 16) .. + 3 of rows tid / 16 + 16 it; U is
  // stored by block columns (u_index), so a row of a block column is JB floats from the next
  const int mrow = tid >> 4, mcol = 4 * (tid & 15);
  const float* src = M + (size_t)colblk[mcol >> 5] * Np * JB + (mcol & 31);
  f4 xpre[4];
  auto fetch = [&](int slab) {
#pragma unroll
    for (int it = 0; it < 4; it++) xpre[it] = *reinterpret_cast<const f4*>(src + (size_t)(slab * JT + mrow + 16 * it) * JB);
  };
  fetch(slab0);
  // R_J, rounded to float32, goes through the slab buffer once per workgroup (every wavefront needs
  // all of it): thread handles columns 4 (tid % 16) .. + 3 of rows tid / 16 + 16 it
#pragma unroll
  for (int it = 0; it < 4; it++) {
    const T* rp = RJ + (mrow + 16 * it) * JT + mcol;
    const T2 v0 = *reinterpret_cast<const T2*>(rp), v1 = *reinterpret_cast<const T2*>(rp + 2);
    *reinterpret_cast<f4*>(&X[mrow + 16 * it][mcol]) = f4{(float)v0.x, (float)v0.y, (float)v1.x, (float)v1.y};
  }
  __syncthreads();
  float rf[16][4];  // B fragments: product ks contracts over k = 4 ks + q4; column tile nt holds columns 4 n + nt
#pragma unroll
  for (int ks = 0; ks < 16; ks++) {
    const f4 v = *reinterpret_cast<const f4*>(&X[4 * ks + q4][4 * l15]);
    rf[ks][0] = v[0]; rf[ks][1] = v[1]; rf[ks][2] = v[2]; rf[ks][3] = v[3];
  }
  // The fragments are only used inside the slab loop, and the optimiser would sink these reads to
  // the loop's entry, behind the barrier below, where other wavefronts already overwrite the buffer.
  asm volatile("" ::: "memory");
  __syncthreads();  // the buffer is free for the first slab
  float* dst = M + (size_t)colblk[(4 * l15) >> 5] * Np * JB + ((4 * l15) & 31);  // the lane's four columns of a result row
  for (int slab = slab0; slab < slab1; slab++) {
#pragma unroll
    for (int it = 0; it < 4; it++) *reinterpret_cast<f4*>(&X[mrow + 16 * it][mcol]) = xpre[it];
    __syncthreads();
    if (slab + 1 < slab1) fetch(slab + 1);
    f4 acc[4];
#pragma unroll
    for (int i = 0; i < 4; i++) acc[i] = f4{0, 0, 0, 0};
    {  // the operand of product ks + 1 is read from LDS while product ks runs
      float a = X[wave * 16 + l15][q4];
#pragma unroll
      for (int ks = 0; ks < 16; ks++) {
        const float ca = a;
        if (ks + 1 < 16) a = X[wave * 16 + l15][4 * (ks + 1) + q4];
        __builtin_amdgcn_sched_barrier(0);  // keep the read ahead of the products (the scheduler would sink it)
#pragma unroll
        for (int nt = 0; nt < 4; nt++) acc[nt] = MM<float>::mma(ca, rf[ks][nt], acc[nt]);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; j++)
      *reinterpret_cast<f4*>(dst + (size_t)(slab * JT + wave * 16 + MM<float>::row(j, lane)) * JB) =
          f4{acc[0][j], acc[1][j], acc[2][j], acc[3][j]};
    __syncthreads();  // every wave has finished reading X
  }
}

// ---------------------------------------------------------------------------------------
// Off-diagonal mass of G after a sweep, from the blocks that are maintained: block row i of image b
// gives  2 sum_{c > r} G_rc^2  over its rows (what lies below the diagonal mirrors what lies above
// and is not kept up to date).  One workgroup per (block row, image); every thread adds its
// elements in a fixed order and the partial sums are combined in a fixed order, so the stopping
// decision is reproducible.
template <typename T>
__global__ __launch_bounds__(256) void jacobi_offnorm(const T* __restrict__ G, const EigState* __restrict__ state,
                                                      double* __restrict__ offpart, int Np, int nblk, int img0) {
  const int i = blockIdx.x, b = img0 + blockIdx.y, tid = threadIdx.x;
  if (state[b].done) return;
  __shared__ double red[4];
  const T* Gb = G + (size_t)b * Np * Np;
  const int c0 = i * JB, width = Np - c0;
  double s = 0.0;
  for (int r = tid >> 6; r < JB; r += 4) {  // a wavefront takes every fourth row, its lanes consecutive columns
    const T* row = Gb + (size_t)(c0 + r) * Np + c0;
    for (int c = r + 1 + (tid & 63); c < width; c += 64) {  // strictly above the diagonal; the mirror half is not kept up to date
      const double v = (double)row[c];
      s += 2.0 * v * v;
    }
  }
  s = wave_sum(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) offpart[(size_t)b * nblk + i] = (red[0] + red[1]) + (red[2] + red[3]);
}

// One wavefront per image: add the block-row partials, count the sweep, decide.
__global__ void jacobi_sweep_end(const double* __restrict__ offpart, EigState* __restrict__ state, int count,
                                 double tol, int img0) {
  const int b = img0 + blockIdx.x, lane = threadIdx.x;
  if (state[b].done) return;
  const double* op = offpart + (size_t)b * count;
  double s = 0.0;
  for (int i = lane; i < count; i += 64) s += op[i];
  s = wave_sum(s);
  if (lane == 0) {
    const double limit = tol * tol * state[b].norm2;
    state[b].sweeps += 1;
    if (s <= limit) state[b].done = 1;
    // Close to the end most block pairs have already converged far below the tolerance while a few still
    // carry the remaining mass (convergence is quadratic pair by pair).  From here on a visit is skipped
    // when it would remove less than limit / (64 nblk^2): all skipped visits of a sweep together
    // leave less than 1/128 of the squared stopping threshold, and the stopping test itself keeps measuring G.
    if (s <= SKIP_START * SKIP_START * limit) state[b].thr2 = limit / (64.0 * count * count);
  }
}

// ---------------------------------------------------------------------------------------
// Helper streams.  The rotation kernel is bound by the vector ALUs and by latency, the tile updates
// by the matrix cores, and images are independent, so the batch is cut into up to MAX_GROUPS groups
// whose step sequences run on different streams and overlap on the GPU.  The helper streams are
// created once per device and kept for the life of the process (no device memory); the events that
// tie them to the caller's stream live only for the duration of one call.
constexpr int MAX_GROUPS = 4;
struct StreamPool {
  hipStream_t s[MAX_GROUPS - 1];
  hipEvent_t fork, join[MAX_GROUPS - 1], stage[MAX_GROUPS - 1];  // re-recorded by every call (a wait captures the state at the time it is enqueued)
  bool ok = false;
};
static std::mutex g_pool_mutex;
static StreamPool g_pools[64];

static StreamPool* helper_streams() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(g_pool_mutex);
  StreamPool& pool = g_pools[dev];
  if (!pool.ok) {
    int ns = 0, ne = 0, nst = 0;
    bool good = hipEventCreateWithFlags(&pool.fork, hipEventDisableTiming) == hipSuccess;
    const bool have_fork = good;
    while (good && ns < MAX_GROUPS - 1) {
      good = hipStreamCreateWithFlags(&pool.s[ns], hipStreamNonBlocking) == hipSuccess;
      if (good) ns++;
    }
    while (good && ne < MAX_GROUPS - 1) {
      good = hipEventCreateWithFlags(&pool.join[ne], hipEventDisableTiming) == hipSuccess;
      if (good) ne++;
    }
    while (good && nst < MAX_GROUPS - 1) {
      good = hipEventCreateWithFlags(&pool.stage[nst], hipEventDisableTiming) == hipSuccess;
      if (good) nst++;
    }
    if (!good) {  // release what was created; the caller falls back to one stream
      if (have_fork) (void)hipEventDestroy(pool.fork);
      for (int i = 0; i < ns; i++) (void)hipStreamDestroy(pool.s[i]);
      for (int i = 0; i < ne; i++) (void)hipEventDestroy(pool.join[i]);
      for (int i = 0; i < nst; i++) (void)hipEventDestroy(pool.stage[i]);
      return nullptr;
    }
    pool.ok = true;
  }
  return &pool;
}

// Fork: streams[0] = st, streams[1 .. n-1] = helper streams that wait for what is already enqueued on st.
// Returns the number of streams available (1 if the helpers could not be created).  The pool's events are
// shared by all calls on the device, so the pool stays locked until join_streams(): two host threads enqueuing
// at the same time cannot interleave their record/wait pairs.
static std::unique_lock<std::mutex>& pool_lock() {
  static thread_local std::unique_lock<std::mutex> lock(g_pool_mutex, std::defer_lock);
  return lock;
}
int fork_streams(hipStream_t st, int groups, hipStream_t* streams) {
  streams[0] = st;
  if (groups > MAX_GROUPS) groups = MAX_GROUPS;
  StreamPool* pool = groups > 1 ? helper_streams() : nullptr;
  if (!pool) return 1;
  pool_lock().lock();
  (void)hipEventRecord(pool->fork, st);
  for (int g = 1; g < groups; g++) {
    streams[g] = pool->s[g - 1];
    (void)hipStreamWaitEvent(streams[g], pool->fork, 0);
  }
  return groups;
}
// Between a fork and its join: what is enqueued on stream g + 1 from now on waits for what is on stream g now
// (g = 0 is the caller's stream).  Lets the groups start one after the other instead of all at once.
void stagger_streams(hipStream_t st, int g, int groups) {
  if (g + 1 >= groups) return;
  int dev = 0;
  (void)hipGetDevice(&dev);
  StreamPool& pool = g_pools[dev];
  (void)hipEventRecord(pool.stage[g], g == 0 ? st : pool.s[g - 1]);
  (void)hipStreamWaitEvent(pool.s[g], pool.stage[g], 0);
}
// Join: st waits for everything enqueued on the helper streams since the fork.
void join_streams(hipStream_t st, int groups) {
  if (groups <= 1) return;
  int dev = 0;
  (void)hipGetDevice(&dev);
  StreamPool& pool = g_pools[dev];
  for (int g = 0; g < groups - 1; g++) {
    (void)hipEventRecord(pool.join[g], pool.s[g]);
    (void)hipStreamWaitEvent(st, pool.join[g], 0);
  }
  pool_lock().unlock();
}

template <typename T>
static void enqueue_group(const Plan& pl, T* G, float* U, T* R, double* offpart, EigState* state, int img0, int nimg,
                          hipStream_t st) {
  const int Np = pl.Np, nblk = pl.nblk, P = pl.P;
  const int gs = grid_for_groups(P, nimg);
  const int ntiles = P * (P - 1) / 2, gchunk = ntiles * nimg >= 1024 ? G_CHUNK : (ntiles * nimg >= 512 ? 2 : 1);  // smaller launches: fewer tiles per workgroup, so that the chip is still filled
  const int gg = grid_for_groups((ntiles + gchunk - 1) / gchunk, nimg), uchunk = (Np / JT) * P * nimg >= 512 ? 3 : 1,
            gu = grid_for_groups(((Np / JT + uchunk - 1) / uchunk) * P, nimg);
  const int count_work = profiling_active() ? 1 : 0;  // the kernels keep count of the work they really do only for the profiler
  for (int sweep = 0; sweep < pl.max_sweeps; sweep++) {
    for (int step = 0; step < pl.steps; step++) {
      // Step 0 of a sweep visits every block, and its full 63-step solve leaves the diagonal blocks
      // nearly diagonal: most later visits only rotate index pairs across the two blocks (32 steps
      // instead of 63); a full solve every FULL_EVERY-th step keeps the entries inside the diagonal
      // blocks converging (cross-only sweeps stall).
      // (float32 solver: always full sweeps; its rounding noise inside the diagonal blocks needs them)
      if (step % FULL_EVERY == 0 || sizeof(T) == 4)
        TC_TIMED(PK_JSOLVE, sweep, st, (jacobi_solve<T, false><<<gs, SOLVE_THREADS, 0, st>>>(G, R, state, Np, nblk, step, img0, nimg, JT - 1, count_work)));
      else
        TC_TIMED(PK_JSOLVE, sweep, st, (jacobi_solve<T, true><<<gs, SOLVE_THREADS, 0, st>>>(G, R, state, Np, nblk, step, img0, nimg, JB, count_work)));
      if (ntiles > 0)  // a single pair: the rotation kernel has done it all
        TC_TIMED(PK_JUPDATE, sweep, st, (jacobi_update_g<T><<<gg, 256, 0, st>>>(G, R, state, Np, nblk, step, img0, nimg, gchunk, count_work)));
      if (U) TC_TIMED(PK_JUPDATE_U, sweep, st, (jacobi_update_u<T><<<gu, 256, 0, st>>>(U, R, state, Np, nblk, step, img0, nimg, uchunk)));
    }
    TC_TIMED(PK_JSWEEPEND, sweep, st, (jacobi_offnorm<T><<<dim3(nblk, nimg), 256, 0, st>>>(G, state, offpart, Np, nblk, img0)));
    TC_TIMED(PK_JSWEEPEND, sweep, st, (jacobi_sweep_end<<<nimg, 64, 0, st>>>(offpart, state, nblk, pl.tol, img0)));
  }
}

template <typename T>
static int run_jacobi(const Plan& pl, T* G, float* U, T* R, double* offpart, EigState* state, hipStream_t st) {
  const int Np = pl.Np;
  if (U) TC_TIMED(PK_JINIT, 0, st, (jacobi_init_u<<<dim3(Np * Np / 1024 > 0 ? Np * Np / 1024 : 1, pl.B), 256, 0, st>>>(U, Np)));  // U == nullptr: eigenvalues only
  TC_TIMED(PK_JINIT, 1, st, (jacobi_norm_partial<T><<<dim3(pl.nblk, pl.B), 256, 0, st>>>(G, offpart, Np, pl.nblk)));
  TC_TIMED(PK_JINIT, 2, st, (jacobi_init_state<<<pl.B, 64, 0, st>>>(offpart, state, pl.nblk)));
  // Splitting pays once every group still fills the chip with its tile updates (measured at N = 576:
  // one stream up to 12 images, two from 16, four from 32; N = 2880: four at 8 images)
  const long tiles = (long)pl.B * pl.P * (pl.P - 1) / 2;
  int groups = pl.groups > 0 ? pl.groups : (tiles >= 1152 ? 4 : (tiles >= 576 ? 2 : 1));
  if (groups > pl.B) groups = pl.B;
  if (profiling_active()) groups = 1;  // per-kernel timing wants kernels that run alone
  hipStream_t streams[MAX_GROUPS];
  groups = fork_streams(st, groups, streams);
  const int per = (pl.B + groups - 1) / groups;
  for (int g = 0; g < groups; g++) {
    const int img0 = g * per, nimg = pl.B - img0 < per ? pl.B - img0 : per;
    if (nimg <= 0) continue;
    enqueue_group<T>(pl, G, U, R, offpart, state, img0, nimg, streams[g]);
  }
  join_streams(st, groups);
  return check_launch();
}

int launch_jacobi(const Plan& pl, int eig_dtype, void* G, void* U, void* R, double* offpart, EigState* state,
                  hipStream_t st) {
  if (eig_dtype == TC_EIG_F64) return run_jacobi<double>(pl, (double*)G, (float*)U, (double*)R, offpart, state, st);
  return run_jacobi<float>(pl, (float*)G, (float*)U, (float*)R, offpart, state, st);
}

}  // namespace tc
