// Direct symmetric eigensolver, stages 2 and 3 (stage 1, the reduction G = Q T Q^T, is tridiag.hip):
//   2a  eigenvalues of the tridiagonal T by bisection on Sturm counts, one lane per eigenvalue;
//   2b  eigenvector of every eigenvalue from the twisted factorisation of T - lambda I
//       (forward L D+ L^T, backward U D- U^T, joined at the index r that minimises |gamma_r|;
//       the vector solves (T - lambda I) z = gamma_r e_r), one lane per eigenvector;
//   3   back-transformation U = Q W = H_0 ... H_{N-2} W in float32 on the matrix cores, the reflectors sixteen
//       at a time in compact WY form, a strip of 64 eigenvectors held in accumulator registers; since U is
//       only needed for it, the information contribution score of Eq. 3-6, C(x) = sum_i |U[x][i]| sigma_i,
//       is accumulated right there: U is never written.
// T is first split where an off-diagonal element is negligible (|e_k| <= eps ||T||); each eigenpair then
// belongs to one unreduced block and its vector is zero outside that block, so equal eigenvalues of
// decoupled blocks (block-diagonal Gram matrices, null spaces) get orthogonal vectors for free.
// Eigenvectors of one block are computed independently of each other: their mutual orthogonality is
// eps ||T|| / gap.  For the spectra this library meets (gaps >= 1e-9 ||T||) that is 1e-6 or better; a pair
// closer than 1e-10 ||T|| inside one block is orthogonalised explicitly afterwards (td_cluster_kernel).
#include <cfloat>

#include "tc_internal.h"

namespace tc {

constexpr double TD_EPS = 2.220446049250313e-16;

// ---- 2a -----------------------------------------------------------------------------------------------
// dvec, evec [B][Np] from the reduction.  Writes lam [B][Np] (eigenvalue of slot k: the (k - s)-th smallest
// of the block [s, t) that row k lies in), blk [B][Np] = (s, t), and tnorm [B] = ||T||_inf.
//
// The number of eigenvalues below x is the number of sign changes in the sequence of leading principal
// minors p_0 = 1, p_1 = d_s - x, p_i = (d_i - x) p_{i-1} - e_{i-1}^2 p_{i-2}.  In this form the chain from one step to the next is a single fused multiply-add;
// the quotient form q_i = d_i - x - e^2 / q_{i-1} puts a float64 division (thirty dependent instructions)
// on it, and with one eigenvalue per lane there is nothing to hide that latency behind: measured 3.4 ms
// per batch against 0.2.  T is scaled by a power of two to ||T|| <= 1 so that the minors change by at most a
// factor 3 per step, and they are brought back into range every eight steps.
typedef double tb_pair __attribute__((ext_vector_type(2)));

// Scaled copy of T for the bisection, one workgroup per image: prep [B][prep_stride] doubles holds
// (d_i, e_i^2) pairs for rows 0 .. N-1 (e_i = |coupling of rows i-1 and i|, e_0 = 0; the square is 0 where T
// is split), sixteen zero pairs behind them, then the N scaled |e_i|.  Also tnorm [B] = ||T||_inf, and bad[b]
// is cleared.
__global__ __launch_bounds__(256) void td_prepare_kernel(const double* __restrict__ dvec, const double* __restrict__ evec,
                                                         double* __restrict__ prep, size_t prep_stride,
                                                         double* __restrict__ tnorm, int32_t* __restrict__ bad, int N,
                                                         int Np) {
  __shared__ double wmax[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* db = dvec + (size_t)b * Np;
  const double* eb = evec + (size_t)b * Np;
  double rowmax = 0.0;
  for (int i = tid; i < N; i += 256)
    rowmax = fmax(rowmax, fabs(db[i]) + (i > 0 ? fabs(eb[i - 1]) : 0.0) + (i + 1 < N ? fabs(eb[i]) : 0.0));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) rowmax = fmax(rowmax, __shfl_xor(rowmax, o, 64));
  if (lane == 0) wmax[wave] = rowmax;
  __syncthreads();
  const double tn = fmax(fmax(wmax[0], wmax[1]), fmax(wmax[2], wmax[3]));
  const double split = TD_EPS * tn;
  // power of two that brings ||T|| into (1/2, 1] (exact); a zero or non-finite norm leaves T as it is
  int ex = 0;
  if (tn > 0.0 && tn < DBL_MAX) (void)frexp(tn, &ex);
  const double down = ldexp(1.0, -ex);
  tb_pair* pr = reinterpret_cast<tb_pair*>(prep + (size_t)b * prep_stride);
  double* esc = reinterpret_cast<double*>(pr + N + 16);
  for (int i = tid; i < N + 16; i += 256) {
    const double e = i > 0 && i < N ? fabs(eb[i - 1]) : 0.0;
    pr[i] = i < N ? tb_pair{db[i] * down, e > split ? (e * down) * (e * down) : 0.0} : tb_pair{0.0, 0.0};
    if (i < N) esc[i] = e * down;
  }
  if (tid == 0) { tnorm[b] = tn; bad[b] = 0; }
}

// G = 1 << gs lanes per eigenvalue; blockIdx.y = image.  A step evaluates the number of eigenvalues below G
// points that cut the interval into G + 1 equal parts, one point per lane, and keeps the part that holds the
// eigenvalue: log2(G + 1) bits per walk over the rows instead of one (the walk is a chain of dependent
// operations that a wavefront alone on its SIMD cannot hide; with few images the chip has lanes to spare).
// The usual case, T not split anywhere (or every lane of the
// wavefront in the same block), reads the rows through the scalar unit: the coefficients are the same for all
// lanes, and fetched per lane from LDS the sixteen bytes per row and lane made the LDS the limit of the kernel.
__global__ __launch_bounds__(256) void td_bisect_kernel(const double* __restrict__ prep, size_t prep_stride,
                                                        const double* __restrict__ tnorm, double* __restrict__ lam,
                                                        int2* __restrict__ blk, int N, int Np, int gs) {
  extern __shared__ __attribute__((aligned(16))) unsigned char tb_smem[];
  double* ds = reinterpret_cast<double*>(tb_smem);  // [N], scaled
  double* es = ds + N;                               // [N]: es[i] = |coupling of rows i-1 and i|, es[0] = 0, scaled
  double* e2 = es + N;                               // [N]: its square, 0 where T is split
  tb_pair* de = reinterpret_cast<tb_pair*>(e2 + N);  // [N + 16]: (ds[i], e2[i]) side by side, one 16-byte read per row; zero padding
  const int b = blockIdx.y, tid = threadIdx.x;
  const tb_pair* __restrict__ pr = reinterpret_cast<const tb_pair*>(prep + (size_t)b * prep_stride);
  const double* __restrict__ esc = reinterpret_cast<const double*>(pr + N + 16);
  for (int i = tid; i < N + 16; i += 256) {
    const tb_pair v = pr[i];
    de[i] = v;
    if (i < N) {
      ds[i] = v.x;
      e2[i] = v.y;
      es[i] = esc[i];
    }
  }
  const double tn = tnorm[b];
  int ex = 0;
  if (tn > 0.0 && tn < DBL_MAX) (void)frexp(tn, &ex);
  const double up = ldexp(1.0, ex);
  __syncthreads();
  const int G = 1 << gs, sec = tid & (G - 1);  // this lane's point: the (sec + 1)-th of G
  const int k = (blockIdx.x * 256 + tid) >> gs;
  if (k >= N) return;                          // (whole groups of G lanes leave together)
  const double inv = 1.0 / (double)(G + 1);
  const int gshift = (tid & 63) & ~(G - 1);    // first lane of the group within the wavefront
  int s = k, t = k + 1;
  while (s > 0 && e2[s] != 0.0) s--;
  while (t < N && e2[t] != 0.0) t++;
  const int m = k - s;
  // Gershgorin interval of the block, slightly widened (scaled units: ||T|| <= 1)
  double lo = DBL_MAX, hi = -DBL_MAX;
  for (int i = s; i < t; i++) {
    const double r = (i > s && e2[i] != 0.0 ? es[i] : 0.0) + (i + 1 < t && e2[i + 1] != 0.0 ? es[i + 1] : 0.0);
    lo = fmin(lo, ds[i] - r);
    hi = fmax(hi, ds[i] + r);
  }
  const double widen = 2.0 * TD_EPS * (t - s) + 2.0 * DBL_MIN;
  lo -= widen;
  hi += widen;
  const double BIG = 0x1p256, SMALL = 0x1p-256;
  const double d_s = ds[s];
  const int s0 = __builtin_amdgcn_readfirstlane(s), t0 = __builtin_amdgcn_readfirstlane(t);
  const bool uniform = __all(s == s0 && t == t0);
  for (int it = 0; it < 128; it++) {
    const double mid = 0.5 * (lo + hi);
    if (!(mid > lo && mid < hi)) break;     // the interval cannot be halved any more
    if (hi - lo <= 0.25 * TD_EPS) break;    // the entries of T carry errors of eps ||T|| themselves; same count for every lane
    const double width = hi - lo;
    const double x = gs ? lo + width * ((double)(sec + 1) * inv) : mid;  // the lane's point
    double pp = 1.0, p = d_s - x;           // p_{i-2}, p_{i-1}
    // Sign changes are counted on the sign bits.  The signs of the minors are shifted into one register, a bit
    // per row (bit 0 = the newest); after eight rows the changes among them and against the minor before them
    // are the set bits of (signs xor signs >> 1) in its low byte.  An exact zero needs no special case: its
    // successor is -e^2 times its predecessor, so the three minors around it contain one sign change whichever
    // sign the zero is given.  Eight rows at a time: their coefficients are fetched from LDS together and one
    // chunk ahead (read one by one inside the chain, each read would cost its full latency); rows past the
    // block's end are replaced by the identity step p_i = p_{i-1}, which changes no sign; then the pair of
    // minors is brought back into range (a common factor does not change any sign).
    unsigned signs = (unsigned)__double2hiint(p) >> 31;  // p_0 = 1 is positive: bit 1 = 0
    int cnt = (int)signs;
    if (uniform) {
      // every lane of the wavefront walks over the same block: the row index is a scalar, the coefficients come
      // through the scalar unit (loaded one chunk ahead), and no row needs a select.  (Two recurrences per
      // lane, at one third and two thirds of the interval, were measured too: no gain, the kernel is bound by
      // the rate at which one wavefront issues float64 operations, not by their latency.)
      int i0 = s0 + 1;
      tb_pair ca[8], cb[8];
#pragma unroll
      for (int u = 0; u < 8; u++) ca[u] = pr[i0 + u];
#define TB_UCHUNK(CUR, NXT)                                                                    \
  {                                                                                            \
    _Pragma("unroll") for (int u = 0; u < 8; u++) NXT[u] = pr[i0 + 8 + u];                     \
    _Pragma("unroll") for (int u = 0; u < 8; u++) {                                            \
      const double pn = fma(CUR[u].x - x, p, -(CUR[u].y * pp));                              \
      signs = __builtin_amdgcn_alignbit(signs, (unsigned)__double2hiint(pn), 31);              \
      pp = p;                                                                                  \
      p = pn;                                                                                  \
    }                                                                                          \
    cnt += __popc((signs ^ (signs >> 1)) & 0xffu);                                             \
    const double mag = fmax(fabs(p), fabs(pp));                                                \
    const double f = mag > BIG ? SMALL : (mag < SMALL && mag > 0.0 ? BIG : 1.0);               \
    p *= f;                                                                                    \
    pp *= f;                                                                                   \
    i0 += 8;                                                                                   \
  }
      while (i0 + 8 <= t0) {
        TB_UCHUNK(ca, cb)
        if (i0 + 8 > t0) {
#pragma unroll
          for (int u = 0; u < 8; u++) ca[u] = cb[u];
          break;
        }
        TB_UCHUNK(cb, ca)
      }
#undef TB_UCHUNK
      // the last, shorter chunk (ca holds rows i0 .. i0 + 7)
#pragma unroll
      for (int u = 0; u < 8; u++) {
        if (i0 + u < t0) {
          const double pn = fma(ca[u].x - x, p, -(ca[u].y * pp));
          cnt += (int)((unsigned)(__double2hiint(pn) ^ __double2hiint(p)) >> 31);
          pp = p;
          p = pn;
        }
      }
    } else {
    // (two chunk buffers that trade places: no register copies)
    tb_pair ca[8], cb[8];
    int i0 = s + 1;
#pragma unroll
    for (int u = 0; u < 8; u++) ca[u] = de[i0 + u];
#define TB_CHUNK(CUR, NXT)                                                                                                \
  {                                                                                                                       \
    _Pragma("unroll") for (int u = 0; u < 8; u++) NXT[u] = de[i0 + 8 + u];                                                \
    /* the eight reads of this chunk have arrived; those of the next stay in flight */                                   \
    asm volatile("" : "+v"(CUR[0].x), "+v"(CUR[1].x), "+v"(CUR[2].x), "+v"(CUR[3].x), "+v"(CUR[4].x), "+v"(CUR[5].x),     \
                      "+v"(CUR[6].x), "+v"(CUR[7].x), "+v"(CUR[0].y), "+v"(CUR[1].y), "+v"(CUR[2].y), "+v"(CUR[3].y),     \
                      "+v"(CUR[4].y), "+v"(CUR[5].y), "+v"(CUR[6].y), "+v"(CUR[7].y));                                    \
    if (i0 + 8 <= t) { /* a whole chunk: no selects */                                                                    \
      _Pragma("unroll") for (int u = 0; u < 8; u++) {                                                                     \
        const double pn = fma(CUR[u].x - x, p, -(CUR[u].y * pp));                                                       \
        signs = __builtin_amdgcn_alignbit(signs, (unsigned)__double2hiint(pn), 31);                                       \
        pp = p;                                                                                                           \
        p = pn;                                                                                                           \
      }                                                                                                                   \
    } else {                                                                                                              \
      _Pragma("unroll") for (int u = 0; u < 8; u++) {                                                                     \
        const bool in = i0 + u < t;                                                                                       \
        const double pn = fma(in ? CUR[u].x - x : 1.0, p, -((in ? CUR[u].y : 0.0) * pp));                               \
        signs = __builtin_amdgcn_alignbit(signs, (unsigned)__double2hiint(pn), 31);                                       \
        pp = p;                                                                                                           \
        p = pn;                                                                                                           \
      }                                                                                                                   \
    }                                                                                                                     \
    cnt += __popc((signs ^ (signs >> 1)) & 0xffu);                                                                        \
    const double mag = fmax(fabs(p), fabs(pp));                                                                           \
    const double f = mag > BIG ? SMALL : (mag < SMALL && mag > 0.0 ? BIG : 1.0);                                          \
    p *= f;                                                                                                               \
    pp *= f;                                                                                                              \
    i0 += 8;                                                                                                              \
  }
    while (i0 < t) {
      TB_CHUNK(ca, cb)
      if (i0 >= t) break;
      TB_CHUNK(cb, ca)
    }
#undef TB_CHUNK
    }
    if (gs == 0) {
      if (cnt > m) hi = mid; else lo = mid;
    } else {
      // points with at most m eigenvalues below them lie left of the eigenvalue: their number (the counts rise
      // with the point) picks the part; the new ends are points that lanes of the group evaluated, bit for bit
      const unsigned long long left = __ballot(cnt <= m);
      const int ms = __popcll((left >> gshift) & ((1ull << G) - 1ull));
      const double nlo = ms == 0 ? lo : lo + width * ((double)ms * inv);
      const double nhi = ms == G ? hi : lo + width * ((double)(ms + 1) * inv);
      lo = nlo;
      hi = nhi;
    }
  }
  if (sec == 0) {
    lam[(size_t)b * Np + k] = 0.5 * (lo + hi) * up;
    blk[(size_t)b * Np + k] = int2{s, t};
  }
}

// ---- 2b -----------------------------------------------------------------------------------------------
// One lane per eigenvector.  DP and DM are scratch [B][Np][Np] doubles addressed [row][slot] (contiguous
// across the lanes of a wavefront): the pivots of the two factorisations.  W [B][Np][Np] float receives the
// unnormalised vector of slot k in column k (rows outside its block are zero); rn [B][Np] its reciprocal
// norm (0 if the vector is not finite, which also raises bad[b]).
//
// All lanes of a wavefront walk over the same row at the same time, whatever block their eigenvalue belongs
// to and wherever its twist index lies (a lane ignores the rows that are not its own): every access to the
// scratch arrays and to W is one contiguous run per row.  With per-lane rows (each lane starting at its own
// twist index) a wavefront touched up to 64 rows per instruction and the kernel took six times as long.
// The two factorisations are independent chains with a division per row: they run in one loop, side by side.
// So do the two halves of the vector.  Loads from the scratch arrays are issued one chunk of eight rows ahead.
__global__ __launch_bounds__(64) void td_twisted_kernel(const double* __restrict__ dvec, const double* __restrict__ evec,
                                                        const double* __restrict__ lam, const int2* __restrict__ blk,
                                                        const double* __restrict__ tnorm, double* __restrict__ DP,
                                                        double* __restrict__ DM, float* __restrict__ W,
                                                        double* __restrict__ rn, int32_t* __restrict__ bad, int N,
                                                        int Np) {
  extern __shared__ __attribute__((aligned(16))) unsigned char tw_smem[];
  double* ds = reinterpret_cast<double*>(tw_smem);  // [N]
  double* es = ds + N;                               // [N]: es[i] couples rows i and i+1 (signed), 0 where T is split
  const int b = blockIdx.y, tid = threadIdx.x;
  const double* db = dvec + (size_t)b * Np;
  const double* eb = evec + (size_t)b * Np;
  const double split = TD_EPS * tnorm[b];
  for (int i = tid; i < N; i += 64) {
    ds[i] = db[i];
    const double e = i + 1 < N ? eb[i] : 0.0;
    es[i] = fabs(e) > split ? e : 0.0;
  }
  __syncthreads();
  const int k = blockIdx.x * 64 + tid;
  if (k >= N) return;  // (no barrier below)
  const int2 st = blk[(size_t)b * Np + k];
  const int s = st.x, t = st.y;
  double e2max = 0.0;
  for (int i = s; i + 1 < t; i++) e2max = fmax(e2max, es[i] * es[i]);
  const double pivmin = DBL_MIN * fmax(1.0, e2max);
  const double l = lam[(size_t)b * Np + k];
  double* dp = DP + (size_t)b * Np * Np + k;
  double* dmv = DM + (size_t)b * Np * Np + k;
  float* w = W + (size_t)b * Np * Np + k;

  // forward, rows ascending:   T - l I = L D+ L^T, pivots dp[i] (the chain starts anew at row s);
  // backward, rows descending: T - l I = U D- U^T, pivots dm[j] (the chain starts anew at row t - 1)
  {
    double p = 1.0, dm = 1.0;
    auto row = [&](int i) {
      const int j = N - 1 - i;
      const double a = ds[i] - l, ep = i > 0 ? es[i - 1] : 0.0;
      double pn = a - (ep / p) * ep;
      pn = i == s ? a : pn;
      if (fabs(pn) < pivmin) pn = -pivmin;
      p = pn;
      if (i >= s && i < t) dp[(size_t)i * Np] = p;
      const double aj = ds[j] - l, ej = es[j];
      double dn = aj - (ej / dm) * ej;
      dn = j == t - 1 ? aj : dn;
      if (fabs(dn) < pivmin) dn = -pivmin;
      dm = dn;
      if (j >= s && j < t) dmv[(size_t)j * Np] = dm;
    };
    int i0 = 0;
    for (; i0 + 8 <= N; i0 += 8) {
#pragma unroll
      for (int u = 0; u < 8; u++) row(i0 + u);
    }
    for (; i0 < N; i0++) row(i0);
  }

#define TD_ARRIVED8(f) \
  asm volatile("" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
  // twist index: gamma_i = dp[i] + dm[i] - (d_i - l), the row with the smallest |gamma| (rows descending, the
  // first of equal ones wins).  Rows outside the block hold whatever the scratch memory held: not looked at.
  double gbest = DBL_MAX;
  int r = t - 1;
  {
    double f[8], h[8], fn[8], hn[8];
#pragma unroll
    for (int u = 0; u < 8; u++) {
      const size_t row = (size_t)max(N - 1 - u, 0) * Np;
      f[u] = dp[row];
      h[u] = dmv[row];
    }
    for (int hi = N - 1; hi >= 0; hi -= 8) {
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const size_t row = (size_t)max(hi - 8 - u, 0) * Np;
        fn[u] = dp[row];
        hn[u] = dmv[row];
      }
      TD_ARRIVED8(f)
      TD_ARRIVED8(h)
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int i = hi - u;
        const double g = fabs(f[u] + h[u] - (ds[max(i, 0)] - l));
        const bool take = i >= s && i < t && (g < gbest || !(gbest == gbest));
        gbest = take ? g : gbest;
        r = take ? i : r;
      }
#pragma unroll
      for (int u = 0; u < 8; u++) { f[u] = fn[u]; h[u] = hn[u]; }
    }
  }

  // the vector: z_r = 1; upwards from r with the multipliers e_i / dp[i] of L (rows descending), downwards with
  // the multipliers e_{i-1} / dm[i] of U (rows ascending); zero outside the block
  double zu = 1.0, zd = 1.0, nrm = 1.0;
  {
    double f[8], h[8], fn[8], hn[8];
#pragma unroll
    for (int u = 0; u < 8; u++) {
      f[u] = dp[(size_t)max(N - 1 - u, 0) * Np];
      h[u] = dmv[(size_t)min(u, N - 1) * Np];
    }
    for (int c0 = 0; c0 < N; c0 += 8) {
#pragma unroll
      for (int u = 0; u < 8; u++) {
        fn[u] = dp[(size_t)max(N - 1 - c0 - 8 - u, 0) * Np];
        hn[u] = dmv[(size_t)min(c0 + 8 + u, N - 1) * Np];
      }
      TD_ARRIVED8(f)
      TD_ARRIVED8(h)
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int c = c0 + u;
        const bool in = c < N;
        const int iu = max(N - 1 - c, 0), id = min(c, N - 1);
        {  // rows iu <= r
          const double q = es[iu] / f[u];
          const bool act = in && iu >= s && iu < r;
          const double zn = -q * zu;
          zu = act ? zn : zu;
          nrm += act ? zn * zn : 0.0;
          if (in && iu <= r) w[(size_t)iu * Np] = iu < s ? 0.f : (iu == r ? 1.f : (float)zu);
        }
        {  // rows id > r
          const double q = es[max(id - 1, 0)] / h[u];
          const bool act = in && id > r && id < t;
          const double zn = -q * zd;
          zd = act ? zn : zd;
          nrm += act ? zn * zn : 0.0;
          if (in && id > r) w[(size_t)id * Np] = id >= t ? 0.f : (float)zd;
        }
      }
#pragma unroll
      for (int u = 0; u < 8; u++) { f[u] = fn[u]; h[u] = hn[u]; }
    }
  }
#undef TD_ARRIVED8
  const bool fin = nrm == nrm && nrm < DBL_MAX && nrm < 1e60;  // float storage of z holds |z| < 3e38 relative to z_r = 1
  rn[(size_t)b * Np + k] = fin ? 1.0 / sqrt(nrm) : 0.0;
  if (!fin) atomicOr(&bad[b], 1);
}

// ---- close eigenvalues inside one block -----------------------------------------------------------------
// One workgroup per image walks over the slots of every block in ascending order of eigenvalue.  A slot
// whose eigenvalue lies within 1e-10 ||T|| of its predecessor's joins the predecessor's cluster and its
// vector is orthogonalised (modified Gram-Schmidt, float64 accumulation) against the cluster's earlier
// vectors.  If nothing independent is left of it (the two vectors were the same to 1e-3) the pair cannot
// be separated this way: bad[b] gets bit 2 and the caller's info turns negative.
__global__ __launch_bounds__(256) void td_cluster_kernel(const double* __restrict__ lam, const int2* __restrict__ blk,
                                                         const double* __restrict__ tnorm, float* __restrict__ W,
                                                         double* __restrict__ rn, int32_t* __restrict__ bad, int N,
                                                         int Np) {
  __shared__ double red[4];
  __shared__ int any;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* lb = lam + (size_t)b * Np;
  const int2* bb = blk + (size_t)b * Np;
  double* rb = rn + (size_t)b * Np;
  float* Wb = W + (size_t)b * Np * Np;
  const double ctol = 1e-10 * tnorm[b];
  // vectors of eigenvalues that count as zero (below the resolution of the reduction) get weight 0 in Eq. 3-6: they
  // are left as they are, however many of them there are (the null space of a rank-deficient matrix)
  const double floor0 = tnorm[b] > 0.0 ? 8.0 * TD_EPS * tnorm[b] : DBL_MAX;
  // quick exit: no close pair anywhere (the usual case)
  if (tid == 0) any = 0;
  __syncthreads();
  int mine = 0;
  for (int k = 1 + tid; k < N; k += 256) mine |= (bb[k].x == bb[k - 1].x && lb[k] - lb[k - 1] <= ctol && lb[k] > floor0) ? 1 : 0;
  if (mine) any = 1;  // every writer stores the same value
  __syncthreads();
  if (!any) return;
  auto block_sum = [&](double x) {
    x = wave_sum(x);
    __syncthreads();
    if (lane == 0) red[wave] = x;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
  };
  int first = 0;  // first slot of the current cluster
  for (int k = 1; k < N; k++) {
    const bool close = bb[k].x == bb[k - 1].x && lb[k] - lb[k - 1] <= ctol && lb[k] > floor0;  // uniform over the workgroup
    if (!close) { first = k; continue; }
    const int s = bb[k].x, t = bb[k].y;
    for (int j = first; j < k; j++) {
      double dot = 0.0;
      for (int i = s + tid; i < t; i += 256) dot += (double)Wb[(size_t)i * Np + j] * (double)Wb[(size_t)i * Np + k];
      dot = block_sum(dot) * rb[j] * rb[j];  // column j has norm 1 / rb[j]
      for (int i = s + tid; i < t; i += 256)
        Wb[(size_t)i * Np + k] = (float)((double)Wb[(size_t)i * Np + k] - dot * (double)Wb[(size_t)i * Np + j]);
      __syncthreads();
    }
    double n2 = 0.0;
    for (int i = s + tid; i < t; i += 256) { const double v = Wb[(size_t)i * Np + k]; n2 += v * v; }
    n2 = block_sum(n2);
    const double before = rb[k] > 0.0 ? 1.0 / (rb[k] * rb[k]) : 0.0;
    __syncthreads();
    if (tid == 0) {
      if (!(n2 > 1e-6 * before)) atomicOr(&bad[b], 2);
      rb[k] = n2 > 0.0 ? 1.0 / sqrt(n2) : 0.0;
    }
    __syncthreads();
  }
}

// ---- weights of Eq. 3-6 -----------------------------------------------------------------------------------
// sigma_k = sqrt(max(lambda_k, 0)); wgt[k] = sigma_k * rn[k] (0 for terms dropped by sv_rtol): the factor that
// turns the unnormalised vector of slot k into its term of C.  Also the optional outputs of tc_ipgs_score that
// do not need the vectors: sigma sorted in descending order, and info.
__global__ __launch_bounds__(256) void td_weights_kernel(const double* __restrict__ lam, const double* __restrict__ rn,
                                                         const double* __restrict__ tnorm,
                                                         const int32_t* __restrict__ bad, float sv_rtol,
                                                         double* __restrict__ sig, double* __restrict__ wgt,
                                                         float* __restrict__ sigma_out, int32_t* __restrict__ info_out,
                                                         int N, int Np) {
  extern __shared__ float key[];  // pow2 >= N floats, only when sigma_out != nullptr
  __shared__ double wmax[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double* lb = lam + (size_t)b * Np;
  double* sb = sig + (size_t)b * Np;
  // Eigenvalues come out of the reduction and the bisection with an absolute error of a few eps ||T||: what lies
  // below that is zero (an all-zero matrix, the null space of a rank-deficient one).
  const double floor0 = tnorm[b] > 0.0 ? 8.0 * TD_EPS * tnorm[b] : DBL_MAX;  // (every eigenvalue of an all-zero matrix is zero)
  double mx = 0.0;
  int nanflag = 0;
  for (int i = tid; i < Np; i += 256) {
    double s = 0.0;
    if (i < N) {
      const double l = lb[i];
      nanflag |= (l == l) ? 0 : 1;
      s = l > floor0 ? sqrt(l) : 0.0;
    }
    sb[i] = s;
    mx = fmax(mx, s);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mx = fmax(mx, __shfl_xor(mx, o, 64));
    nanflag |= __shfl_xor(nanflag, o, 64);
  }
  __shared__ int wnan[4];
  if (lane == 0) { wmax[wave] = mx; wnan[wave] = nanflag; }
  __syncthreads();
  const double thr = sv_rtol > 0.f ? (double)sv_rtol * fmax(fmax(wmax[0], wmax[1]), fmax(wmax[2], wmax[3])) : -1.0;
  if (wgt)
    for (int i = tid; i < Np; i += 256) {
      const double s = sb[i];
      wgt[(size_t)b * Np + i] = (i < N && s > thr) ? s * rn[(size_t)b * Np + i] : 0.0;
    }
  if (tid == 0 && info_out)  // 1: done (the method does not iterate); negative: an eigenvector is not finite or a cluster stayed unresolved
    info_out[b] = (bad[b] | wnan[0] | wnan[1] | wnan[2] | wnan[3]) ? -1 : 1;
  if (!sigma_out) return;
  int n2 = 1;
  while (n2 < N) n2 <<= 1;
  for (int i = tid; i < n2; i += 256) key[i] = i < N ? (float)sb[i] : -1.0f;
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

// ---- 3 ------------------------------------------------------------------------------------------------
// U = H_0 H_1 ... H_{N-2} W, sixteen reflectors at a time in compact WY form (the scheme of LAPACK's
// dlarft/dlarfb): H_j0 ... H_j0+15 = I - V T V^T with V the 16 reflectors and T upper triangular,
//     T[c][c] = tau_c,   T[0:c, c] = -tau_c T[0:c, 0:c] (V[:, 0:c]^T v_c).
typedef __attribute__((ext_vector_type(4))) float f4;
constexpr int BT_K = 16;  // reflectors per block

// T of every block of 16 reflectors: one workgroup per (block, image).  The block goes through LDS once
// (16-byte accesses); thread (a, c) then forms v_a^T v_c from there.
__global__ __launch_bounds__(256) void td_tfactor_kernel(const float* __restrict__ Vc, const float* __restrict__ tauv,
                                                         float* __restrict__ Tf, int N, int Np, int npanel) {
  constexpr int VP = BT_K + 1;
  extern __shared__ __attribute__((aligned(16))) float tf_smem[];  // [N - j0][VP]
  __shared__ float S[BT_K][BT_K];   // S[a][c] = v_a^T v_c, a < c
  __shared__ float T[BT_K][BT_K];
  const int p = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j0 = BT_K * p, rows = N - j0;
  const f4* src = reinterpret_cast<const f4*>(Vc + (size_t)b * Np * Np + (size_t)p * Np * BT_K + (size_t)j0 * BT_K);
  for (int e = tid; e < rows * 4; e += 256) {
    const int i = e >> 2, m = 4 * (e & 3);
    const f4 v = src[e];
    float* d = &tf_smem[i * VP + m];
#pragma unroll
    for (int u = 0; u < 4; u++) d[u] = j0 + m + u <= N - 2 ? v[u] : 0.f;  // reflectors past N-2 do not exist: their slots were never written
  }
  __syncthreads();
  {
    const int a = tid / BT_K, c = tid % BT_K;
    float dot = 0.f;
    if (a < c)  // v_c is zero up to row j0 + c
      for (int i = c + 1; i < rows; i++) dot += tf_smem[i * VP + a] * tf_smem[i * VP + c];
    S[a][c] = dot;
    T[a][c] = 0.f;
  }
  __syncthreads();
  if (wave == 0) {  // column by column; lane a owns row a
    for (int c = 0; c < BT_K; c++) {
      const float tau = j0 + c <= N - 2 ? tauv[(size_t)b * Np + j0 + c] : 0.f;
      float acc = 0.f;
      if (lane < c)
        for (int r = lane; r < c; r++) acc += T[lane][r] * S[r][c];
      if (lane < c) T[lane][c] = -tau * acc;
      if (lane == c) T[c][c] = tau;
      // (a wavefront runs in lockstep and the LDS serves its accesses in order: column c is complete before c + 1 reads it)
      __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
      __builtin_amdgcn_wave_barrier();
    }
  }
  __syncthreads();
  Tf[((size_t)b * npanel + p) * (BT_K * BT_K) + tid] = T[tid / BT_K][tid % BT_K];
}

// A strip of 16 CT eigenvectors (columns k0 .. k0 + 16 CT - 1 of W) lives in the accumulator registers of the four
// wavefronts of a workgroup for the whole kernel: wavefront w owns the row tiles rt = 4 t + w (16 rows each),
// as CT 16x16 column tiles; element j of a lane is (row 4 (lane / 16) + j, column lane % 16) of its tile.
// Per block of reflectors, last block first:
//   Z  = V^T U     contraction over rows; the B operand of matrix-core step j is accumulator element j itself
//                  (rows j, 4 + j, 8 + j, 12 + j of the tile), the A operand the matching rows of V;
//                  the four wavefronts' parts are added in a fixed order through LDS
//   Z2 = T Z       one 16x16x16 product per column tile, same trick on the accumulator of Z
//   U -= V Z2      likewise on the accumulator of Z2.
// V of the block goes through LDS, transposed to [row][reflector].  Only row tiles that the block reaches
// (rows > j0) take part.  At the end the strip's share of Eq. 3-6, Cpart[strip][x] = sum_k |U[x][k]| wgt[k],
// is reduced across the 16 lanes of a row and written; U itself is not.  CT is chosen by the launcher so that
// the workgroups fill the chip in whole rounds and the accumulators fit the register file.
template <int TPW, int CT>
__global__ __launch_bounds__(256) void td_backtransform_kernel(const float* __restrict__ W, const float* __restrict__ Vc,
                                                               const float* __restrict__ Tf,
                                                               const double* __restrict__ wgt,
                                                               double* __restrict__ Cpart, int N, int Np, int nstrip,
                                                               int npanel) {
  constexpr int VP = BT_K + 1;       // LDS pitch of a row of V
  constexpr int ROWS = 64 * TPW;     // rows covered by the workgroup (>= Np)
  extern __shared__ __attribute__((aligned(16))) float bt_smem[];
  float* vt = bt_smem;                         // [ROWS][VP]
  constexpr int SW = 16 * CT;                  // width of the strip
  float* zbuf = vt + ROWS * VP;                // [4][16][SW] the wavefronts' parts of Z
  float* tl = zbuf + 4 * BT_K * SW;            // [16][16]
  const int b = blockIdx.y, strip = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l15 = lane & 15, q4 = lane >> 4;
  const int k0 = strip * SW;
  const float* Wb = W + (size_t)b * Np * Np;
  const float* Vb = Vc + (size_t)b * Np * Np;
  f4 acc[TPW][CT];
#pragma unroll
  for (int t = 0; t < TPW; t++)
#pragma unroll
    for (int ct = 0; ct < CT; ct++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int row = 16 * (4 * t + wave) + 4 * q4 + j, col = k0 + 16 * ct + l15;
        acc[t][ct][j] = (row < N && col < N) ? Wb[(size_t)row * Np + col] : 0.f;
      }
  // The block's reflectors [row][16] are a straight copy, 16 bytes per access; the copy of the next block is
  // in flight (in registers) while the matrix cores work on this one.
  constexpr int PER = ROWS * 4 / 256;  // 16-byte pieces per thread when the block covers every row
  f4 piece[PER];
  float t_next;
  auto fetch = [&](int p) {
    const f4* src = reinterpret_cast<const f4*>(Vb + (size_t)p * Np * BT_K);
#pragma unroll
    for (int u = 0; u < PER; u++) {
      const int e = tid + 256 * u, i = e >> 2;      // row i, quarter e & 3
      piece[u] = (i >= BT_K * p && i < N) ? src[e] : f4{0.f, 0.f, 0.f, 0.f};
    }
    t_next = Tf[((size_t)b * npanel + p) * (BT_K * BT_K) + tid];
  };
  fetch(npanel - 1);
  for (int p = npanel - 1; p >= 0; p--) {
    const int j0 = BT_K * p;
    __syncthreads();  // the previous block no longer reads vt, tl, zbuf
#pragma unroll
    for (int u = 0; u < PER; u++) {
      const int e = tid + 256 * u, i = e >> 2, m = 4 * (e & 3);
      if (i >= j0) {
        const bool last = j0 + m + 3 > N - 2;  // reflectors past N-2 do not exist: their slots were never written
        float* d = &vt[i * VP + m];
        d[0] = (!last || j0 + m <= N - 2) ? piece[u][0] : 0.f;
        d[1] = (!last || j0 + m + 1 <= N - 2) ? piece[u][1] : 0.f;
        d[2] = (!last || j0 + m + 2 <= N - 2) ? piece[u][2] : 0.f;
        d[3] = (!last || j0 + m + 3 <= N - 2) ? piece[u][3] : 0.f;
      }
    }
    tl[tid] = t_next;
    if (p > 0) fetch(p - 1);
    __syncthreads();
    f4 z[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ct++) z[ct] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < TPW; t++) {
      const int rt = 4 * t + wave;
      if (rt >= p) {  // uniform: rows 16 rt .. 16 rt + 15 reach beyond j0 = 16 p
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const float a = vt[(16 * rt + 4 * q4 + j) * VP + l15];
#pragma unroll
          for (int ct = 0; ct < CT; ct++) z[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, acc[t][ct][j], z[ct], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int ct = 0; ct < CT; ct++)
#pragma unroll
      for (int j = 0; j < 4; j++) zbuf[(wave * BT_K + 4 * q4 + j) * SW + 16 * ct + l15] = z[ct][j];
    __syncthreads();
#pragma unroll
    for (int ct = 0; ct < CT; ct++)
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int o = (4 * q4 + j) * SW + 16 * ct + l15;
        z[ct][j] = (zbuf[o] + zbuf[BT_K * SW + o]) + (zbuf[2 * BT_K * SW + o] + zbuf[3 * BT_K * SW + o]);
      }
    f4 z2[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ct++) z2[ct] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const float a = tl[l15 * BT_K + 4 * q4 + j];
#pragma unroll
      for (int ct = 0; ct < CT; ct++) z2[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, z[ct][j], z2[ct], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < TPW; t++) {
      const int rt = 4 * t + wave;
      if (rt >= p) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const float a = -vt[(16 * rt + l15) * VP + 4 * q4 + j];
#pragma unroll
          for (int ct = 0; ct < CT; ct++) acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, z2[ct][j], acc[t][ct], 0, 0, 0);
        }
      }
    }
  }
  // Eq. 3-6, this strip's share
  double wk[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ct++) {
    const int col = k0 + 16 * ct + l15;
    wk[ct] = col < N ? wgt[(size_t)b * Np + col] : 0.0;
  }
  double* Cp = Cpart + ((size_t)b * nstrip + strip) * Np;
#pragma unroll
  for (int t = 0; t < TPW; t++)
#pragma unroll
    for (int j = 0; j < 4; j++) {
      double term = 0.0;
#pragma unroll
      for (int ct = 0; ct < CT; ct++) term += fabs((double)acc[t][ct][j]) * wk[ct];
      term = row16_sum_dpp(term);
      const int row = 16 * (4 * t + wave) + 4 * q4 + j;
      if (l15 == 0 && row < N) Cp[row] = term;
    }
}

// C(x) = sum over the strips of their shares, in a fixed order.
__global__ __launch_bounds__(256) void td_ics_finish_kernel(const double* __restrict__ Cpart, float* __restrict__ C,
                                                            float* __restrict__ C_out, int N, int Np, int nstrip) {
  const int b = blockIdx.y, x = blockIdx.x * 256 + threadIdx.x;
  if (x >= N) return;
  double s = 0.0;
  for (int t = 0; t < nstrip; t++) s += Cpart[((size_t)b * nstrip + t) * Np + x];
  C[(size_t)b * N + x] = (float)s;
  if (C_out) C_out[(size_t)b * N + x] = (float)s;
}

int launch_td_eigen(const Plan& pl, const double* dvec, const double* evec, const float* tauv, const float* Vc,
                    double* lam, int2* blk, double* tnorm, double* DP, double* DM, float* W, double* rn, int32_t* bad,
                    double* sig, double* wgt, double* Cpart, float* Tf, float sv_rtol, bool vectors, float* C, float* C_out,
                    float* sigma_out, int32_t* info_out, hipStream_t st) {
  const int N = pl.N, Np = pl.Np, B = pl.B;
  // (the scaled copy of T lives at the start of each image's region of DP until the factorisations overwrite it)
  const size_t prep_stride = (size_t)Np * Np;
  TC_TIMED(PK_BISECT, 0, st, (td_prepare_kernel<<<B, 256, 0, st>>>(dvec, evec, DP, prep_stride, tnorm, bad, N, Np)));
  // lanes per eigenvalue: as many as keep the launch near one wavefront per SIMD (by the size of the whole call, so
  // that an image's result does not depend on how the call is cut into stream groups)
  const int gs = pl.batch_call <= 16 ? 3 : pl.batch_call <= 32 ? 2 : pl.batch_call <= 128 ? 1 : 0;
  TC_TIMED(PK_BISECT, 0, st, (td_bisect_kernel<<<dim3(((N << gs) + 255) / 256, B), 256, (size_t)5 * N * 8 + 256, st>>>(DP, prep_stride, tnorm, lam, blk, N, Np, gs)));
  int n2 = 1;
  while (n2 < N) n2 <<= 1;
  const size_t shm_sig = sigma_out ? (size_t)n2 * sizeof(float) : 0;
  if (!vectors) {  // eigenvalues only (the information-quantity tool)
    TC_TIMED(PK_BISECT, 1, st, (td_weights_kernel<<<B, 256, shm_sig, st>>>(lam, nullptr, tnorm, bad, 0.f, sig, nullptr, sigma_out, info_out, N, Np)));
    return check_launch();
  }
  TC_TIMED(PK_TWISTED, 0, st, (td_twisted_kernel<<<dim3((N + 63) / 64, B), 64, (size_t)2 * N * 8, st>>>(dvec, evec, lam, blk, tnorm, DP, DM, W, rn, bad, N, Np)));
  TC_TIMED(PK_TWISTED, 1, st, (td_cluster_kernel<<<B, 256, 0, st>>>(lam, blk, tnorm, W, rn, bad, N, Np)));
  TC_TIMED(PK_BISECT, 1, st, (td_weights_kernel<<<B, 256, shm_sig, st>>>(lam, rn, tnorm, bad, sv_rtol, sig, wgt, sigma_out, info_out, N, Np)));
  const int npanel = (N + BT_K - 1) / BT_K;
  {
    const size_t shm = (size_t)N * (BT_K + 1) * sizeof(float);
    if (shm > 64 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(td_tfactor_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)
      return TC_ERR_HIP;
    TC_TIMED(PK_BACKTF, 0, st, (td_tfactor_kernel<<<dim3(npanel, B), 256, shm, st>>>(Vc, tauv, Tf, N, Np, npanel)));
  }
  // Width of the strips (16 CT eigenvectors per workgroup, one workgroup per compute unit at a time): the one
  // with the least (rounds over the chip) x (work of a workgroup: CT column tiles plus a fixed part of about
  // one); above 576 rows at most two column tiles fit the registers next to the row tiles.
  int ct_best = 1;
  {
    long best = -1;
    for (int ct = Np > 576 ? 2 : 4; ct >= 1; ct--) {
      const long wgs = (long)((N + 16 * ct - 1) / (16 * ct)) * B, rounds = (wgs + 255) / 256;
      const long cost = rounds * (ct + 1);
      if (best < 0 || cost < best) { best = cost; ct_best = ct; }
    }
  }
  const int nstrip = (N + 16 * ct_best - 1) / (16 * ct_best);
  const dim3 gb(nstrip, B);
#define TC_BACKTF2(TPW_, CT_)                                                                                               \
  {                                                                                                                         \
    const size_t shm = ((size_t)64 * TPW_ * (BT_K + 1) + 4 * BT_K * 16 * CT_ + BT_K * BT_K) * sizeof(float);                \
    if (shm > 64 * 1024 &&                                                                                                  \
        hipFuncSetAttribute(reinterpret_cast<const void*>(td_backtransform_kernel<TPW_, CT_>),                              \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)                            \
      return TC_ERR_HIP;                                                                                                    \
    TC_TIMED(PK_BACKTF, 1, st, (td_backtransform_kernel<TPW_, CT_><<<gb, 256, shm, st>>>(W, Vc, Tf, wgt, Cpart, N, Np, nstrip, npanel))); \
  }
#define TC_BACKTF(TPW_)                                    \
  {                                                        \
    if (ct_best == 4) TC_BACKTF2(TPW_, 4)                  \
    else if (ct_best == 3) TC_BACKTF2(TPW_, 3)             \
    else if (ct_best == 2) TC_BACKTF2(TPW_, 2)             \
    else TC_BACKTF2(TPW_, 1)                               \
  }
  if (Np <= 64) TC_BACKTF(1)
  else if (Np <= 128) TC_BACKTF(2)
  else if (Np <= 256) TC_BACKTF(4)
  else if (Np <= 576) TC_BACKTF(9)
  else if (Np <= 1024) {
    if (ct_best == 2) TC_BACKTF2(16, 2) else TC_BACKTF2(16, 1)
  } else return TC_ERR_SHAPE;
#undef TC_BACKTF
#undef TC_BACKTF2
  TC_TIMED(PK_ICS, 0, st, (td_ics_finish_kernel<<<dim3((N + 255) / 256, B), 256, 0, st>>>(Cpart, C, C_out, N, Np, nstrip)));
  return check_launch();
}

}  // namespace tc
