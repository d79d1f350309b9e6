// phi of the linear block code (paper Sec. 3.4, Lemma 1, Lemma l9) for all groups:
//   1. rho_j = f R_j, accumulated in fp64 with a fixed reduction tree (project_kernel + reduce_kernel);
//   2. per group, one wavefront builds and solves the error-locator system
//        [W_{m+s-1}, -W_{s-1} .* (rho 1^T)] a = rho .* w^s
//      (written in the Chebyshev basis, rows equilibrated) and orders the points by |D(w_i)| (corrupted points
//      are roots of the locator D).  V is the smallest set of points without which the others lie within
//      tau * median|rho| of one polynomial P_j of degree m-1 (Lemma 1; the sparse-recovery appendix): the
//      leading roots of D are tried first, then - because in floating point a weakly corrupted point's |D| can
//      come out larger than an honest neighbour's - every subset of at most s points in the order of the position
//      of its last point among the roots, one candidate set per lane;
//   3. the same wavefront prepares psi (Lemma 2): m well-spread honest nodes of the group and the
//      inverse of their m x m Vandermonde (Lagrange basis coefficients), left on the device for decode.
#include <math.h>

#include "solon_internal.h"
#include "wave_ops.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define SOLON_TAU 1e-4          // residual threshold relative to the group's median |rho|
#define SOLON_RANK_TOL 1e-12    // a column whose remaining norm falls below this fraction is dependent
#define SOLON_INV_NORM_MAX 1e6  // largest accepted infinity norm of the inverse m x m Vandermonde
#define SOLON_SEARCH_LIMIT 65536      // candidate sets tried beyond the locator's leading roots before a group is given up
#define SOLON_SPEC_SEARCH_LIMIT 1024  // the same for the guess of the one-pass entry (a wrong guess only costs time)
#define SOLON_LANE_TEST_MAX 8         // largest locator degree whose candidate sets are tested one per lane
#define SOLON_Y_CLAMP 1e8             // projections are clamped to this many medians in the per-lane test (see lane_test)
#define SOLON_CHOL_MIN 1e-13          // smallest accepted pivot of the per-lane Cholesky factorisation

// ------------------------------------------------------------------------------------------------
// Projection.  grid = (row bunches, column tiles); a bunch is RB consecutive rows of R (the last bunch may hold
// fewer), a tile a contiguous run of `seg` 256-wide strips of columns.  A thread keeps one fp64 accumulator per
// row of its bunch and walks its strips with 16-byte loads, so f is loaded once per RB rows of R.  All RB loads of
// a strip are issued back to back with no branch between them: a bunch with fewer rows re-reads its last row
// (in bounds, served by the cache) and drops those sums.
//
// sample_total > 0 turns the launch into a SAMPLE of the columns (the guess of the one-pass locate + decode): tile t then
// covers the hashed position h(key, t) among the sample_total whole tiles of a row, with the key taken from the bits of
// this call's f - which a sender of R cannot know, so no node can keep its corruption out of the sample on purpose.
// A position drawn twice only weights its columns twice: the projections of honest rows stay values of one polynomial.
template <int RB, bool VEC, bool XCD_MAP>
__global__ __launch_bounds__(256) void project_kernel(const float* __restrict__ R, int64_t ldr, const float* __restrict__ f,
                                                       int64_t d_c, int P, int seg, int nbunch, int ntiles, double* __restrict__ partials,
                                                       uint32_t sample_total) {
  // Block -> (tile, bunch).  Workgroups are handed to the eight XCDs round-robin, each with its own L2: block L runs
  // on XCD L % 8 as that XCD's (L / 8)-th block.  Numbering the work so that consecutive blocks OF ONE XCD are the
  // bunches of one tile lets all bunches of a tile find its piece of f in that XCD's L2.
  int bunch, tile;
  if (XCD_MAP) {
    const int64_t total = (int64_t)nbunch * ntiles;
    const int64_t per_xcd = (total + 7) / 8;
    const int64_t v = (int64_t)(blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((int64_t)(blockIdx.x >> 3) >= per_xcd || v >= total) return;
    tile = (int)(v / nbunch);
    bunch = (int)(v - (int64_t)tile * nbunch);
  } else {
    bunch = blockIdx.x % nbunch;
    tile = blockIdx.x / nbunch;
  }
  const int row0 = bunch * RB;
  const int nrows = min(RB, P - row0);
  const int tid = threadIdx.x;
  double acc[RB];
  const float* rp[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    acc[i] = 0.0;
    rp[i] = R + (int64_t)(row0 + min(i, nrows - 1)) * ldr;
  }
  int64_t tpos = tile;
  if (sample_total > 0) {
    const uint32_t key = __float_as_uint(f[0]) ^ (__float_as_uint(f[1]) << 11 | __float_as_uint(f[1]) >> 21) ^
                         (__float_as_uint(f[2]) << 22 | __float_as_uint(f[2]) >> 10) ^ (__float_as_uint(f[3]) * 0x9E3779B9u);
    uint32_t h = key + 0x9E3779B9u * (uint32_t)(tile + 1);  // the 32-bit finaliser of MurmurHash3
    h ^= h >> 16; h *= 0x85EBCA6Bu; h ^= h >> 13; h *= 0xC2B2AE35u; h ^= h >> 16;
    tpos = (int64_t)(((uint64_t)h * (uint64_t)sample_total) >> 32);
  }
  const int64_t first = tpos * seg * 256 + tid;
  if (VEC) {
    const int64_t nvec = d_c / 4;
    for (int it = 0; it < seg; ++it) {
      const int64_t u = first + (int64_t)it * 256;
      if (u >= nvec) break;
      const f32x4 fv = *reinterpret_cast<const f32x4*>(f + 4 * u);
      f32x4 rv[RB];
#pragma unroll
      for (int i = 0; i < RB; ++i) rv[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(rp[i] + 4 * u));
      const double f0 = fv.x, f1 = fv.y, f2 = fv.z, f3 = fv.w;
#pragma unroll
      for (int i = 0; i < RB; ++i) {
        acc[i] = fma(f0, (double)rv[i].x, acc[i]);
        acc[i] = fma(f1, (double)rv[i].y, acc[i]);
        acc[i] = fma(f2, (double)rv[i].z, acc[i]);
        acc[i] = fma(f3, (double)rv[i].w, acc[i]);
      }
    }
    if (sample_total == 0 && tile == 0 && tid < (int)(d_c - nvec * 4)) {  // fewer than four trailing columns
      const int64_t c = nvec * 4 + tid;
      const double fc = f[c];
#pragma unroll
      for (int i = 0; i < RB; ++i) acc[i] = fma(fc, (double)rp[i][c], acc[i]);
    }
  } else {
    for (int it = 0; it < seg; ++it) {
      const int64_t c = first + (int64_t)it * 256;
      if (c >= d_c) break;
      const double fc = f[c];
#pragma unroll
      for (int i = 0; i < RB; ++i) acc[i] = fma(fc, (double)rp[i][c], acc[i]);
    }
  }
  // fixed-order reduction: butterfly inside each wavefront, then the four wavefronts in order
  __shared__ double sm[4][RB];
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int i = 0; i < RB; ++i) {
    double v = acc[i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) sm[wave][i] = v;
  }
  __syncthreads();
  if (tid < nrows) partials[(int64_t)tile * P + row0 + tid] = ((sm[0][tid] + sm[1][tid]) + sm[2][tid]) + sm[3][tid];
}

// rho_j = sum over tiles of partials[tile][j]: one block per node, strided partial sums, then a fixed tree.
__global__ __launch_bounds__(256) void reduce_kernel(const double* __restrict__ partials, int ntiles, int P, double* __restrict__ rho) {
  __shared__ double sm[4];
  const int j = blockIdx.x, tid = threadIdx.x;
  double v = 0.0;
  for (int t = tid; t < ntiles; t += 256) v += partials[(int64_t)t * P + j];
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  if ((tid & 63) == 0) sm[tid >> 6] = v;
  __syncthreads();
  if (tid == 0) rho[j] = ((sm[0] + sm[1]) + sm[2]) + sm[3];
}

template <int RB>
static void project_launch(bool vec, bool xcd_map, int nbunch, int ntiles, hipStream_t st, const float* R, int64_t ldr, const float* f,
                           int64_t d_c, int P, int seg, double* partials, uint32_t sample_total) {
  const int64_t total = (int64_t)nbunch * ntiles;
  const dim3 grid((unsigned)(xcd_map ? (total + 7) / 8 * 8 : total));
#define SOLON_LAUNCH(V, X) hipLaunchKernelGGL((project_kernel<RB, V, X>), grid, dim3(256), 0, st, R, ldr, f, d_c, P, seg, nbunch, ntiles, partials, sample_total)
  if (vec && xcd_map) SOLON_LAUNCH(true, true);
  else if (vec) SOLON_LAUNCH(true, false);
  else if (xcd_map) SOLON_LAUNCH(false, true);
  else SOLON_LAUNCH(false, false);
#undef SOLON_LAUNCH
}

int solon_project_partials_on(const solon_plan* plan, const solon_dev& D, int max_tiles, const float* R, int64_t ldr, const float* f,
                              int64_t ncols, int tile_base, int* ntiles_out, hipStream_t st, int64_t sample_of) {
  const int P = plan->P;
  // rows per bunch: the fewest bunches of at most 4 rows, of equal size where P allows.  With the XCD-aware block
  // numbering the bunches of a tile share f through one L2, so more rows per bunch buy nothing, and fewer rows mean more,
  // lighter blocks (measured, whole solon_locate call: P = 15, rows of 22 MB: 16 rows 70.5 us, 8 rows 68.2, 4 rows 66.0;
  // P = 63, 11 MB: 127.8 / 121.4 / 118.6; P = 100, 124 MB: 2244 / 2227 / 2208; 2 or 3 rows are no better than 4;
  // 25 rows leave too few resident waves: 5.7 against 6.75 TB/s).
  const int rb_max = std::max(1, std::min(SOLON_PROJ_ROWS, solon_tuning("project_rows", 4)));
  const int nbunch0 = (P + rb_max - 1) / rb_max;
  const int rb = (P + nbunch0 - 1) / nbunch0;
  const int nbunch = (P + rb - 1) / rb;
  const bool vec = ((uintptr_t)R % 16 == 0) && (ldr % 4 == 0) && ((uintptr_t)f % 16 == 0);
  const int64_t work = vec ? ncols / 4 : ncols;
  const int64_t strips = std::max<int64_t>(1, (work + 255) / 256);
  // strips per tile: 4 to 32 (measured best: 32 once there are well over 6000 blocks, 4 for small inputs), and
  // enough to keep the partial-sum table within its allocation
  const int64_t room = max_tiles - tile_base;
  int64_t seg = solon_tuning("project_seg", 0);
  if (seg <= 0) seg = std::min<int64_t>(32, std::max<int64_t>(4, strips * nbunch / 6000));
  if (sample_of > 0) seg = 1;  // a sample: many small tiles, each at a hashed position of the row
  seg = std::max<int64_t>(seg, (strips + room - 1) / room);
  const int64_t ntiles = (strips + seg - 1) / seg;
  *ntiles_out = (int)ntiles;
  // whole tiles in a row of sample_of columns (the caller makes sure there is at least one)
  const uint32_t sample_total = sample_of > 0 ? (uint32_t)std::min<int64_t>((vec ? sample_of / 4 : sample_of) / (seg * 256), 0x7fffffff) : 0u;
  const int64_t row_cols = sample_of > 0 ? sample_of : ncols;
  const bool xcd_map = solon_tuning("project_xcd_map", 1) != 0 && nbunch > 1;
  double* partials = D.partials + (int64_t)tile_base * P;
  switch (rb) {
#define SOLON_CASE(N) case N: project_launch<N>(vec, xcd_map, nbunch, (int)ntiles, st, R, ldr, f, row_cols, P, (int)seg, partials, sample_total); break;
    SOLON_CASE(1) SOLON_CASE(2) SOLON_CASE(3) SOLON_CASE(4) SOLON_CASE(5) SOLON_CASE(6) SOLON_CASE(7) SOLON_CASE(8)
    SOLON_CASE(9) SOLON_CASE(10) SOLON_CASE(11) SOLON_CASE(12) SOLON_CASE(13) SOLON_CASE(14) SOLON_CASE(15) SOLON_CASE(16)
    SOLON_CASE(17) SOLON_CASE(18) SOLON_CASE(19) SOLON_CASE(20) SOLON_CASE(21) SOLON_CASE(22) SOLON_CASE(23) SOLON_CASE(24)
    SOLON_CASE(25) SOLON_CASE(26) SOLON_CASE(27) SOLON_CASE(28) SOLON_CASE(29) SOLON_CASE(30) SOLON_CASE(31) SOLON_CASE(32)
#undef SOLON_CASE
    default:
      solon_set_error("solon_locate: no projection kernel for %d rows per block", rb);
      return SOLON_E_INVAL;
  }
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

int solon_project_reduce_on(const solon_plan* plan, const solon_dev& D, int ntiles, hipStream_t st) {
  hipLaunchKernelGGL(reduce_kernel, dim3(plan->P), dim3(256), 0, st, D.partials, ntiles, plan->P, D.rho);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

int solon_project_partials(solon_plan* plan, const float* R, int64_t ldr, const float* f, int64_t ncols, int tile_base, int* ntiles_out,
                           hipStream_t st, int64_t sample_of) {
  return solon_project_partials_on(plan, plan->dev, SOLON_PROJ_MAX_TILES, R, ldr, f, ncols, tile_base, ntiles_out, st, sample_of);
}

int solon_project_reduce(solon_plan* plan, int ntiles, hipStream_t st) { return solon_project_reduce_on(plan, plan->dev, ntiles, st); }

int solon_launch_project(solon_plan* plan, const float* R, int64_t ldr, const float* f, hipStream_t st) {
  int ntiles = 0;
  const int rc = solon_project_partials(plan, R, ldr, f, plan->d_c, 0, &ntiles, st);
  if (rc != SOLON_OK) return rc;
  return solon_project_reduce(plan, ntiles, st);
}

// ------------------------------------------------------------------------------------------------
// Single-wavefront solve.  Lane i stands for point i of the group when evaluating polynomials and for
// column i of the system when applying Householder reflections.
#define LDA 66
struct solve_smem {
  double A[64][LDA];  // system matrix, right-hand side in column nc
  double x[64];       // solution
  double cn[64];      // initial column norms
  double y[64];       // normalised projections of the finite points
  double wv[64];      // their evaluation points
  double val[64];     // scratch values compared across lanes
  double lag[SOLON_MAX_M][SOLON_MAX_M + 1];
  double Q[64][SOLON_MAX_M + 1];  // orthonormal polynomials of degree < m over the group's points (row = point)
  double med[2];
  int piv[64];
  int by_rank[64];    // by_rank[k] = point with the k-th smallest |D(w_i)|
  uint32_t cnt[65];   // cnt[c] = number of candidate sets of the widened search whose last point has position < c
};

// Value of `v` in lane `src` (src must be wave-uniform): two scalar broadcasts, no LDS.
__device__ __forceinline__ double lane_bcast(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}

// Least squares min ||A x - b|| by Householder QR without pivoting; b is column nc of S.A.  A column whose
// remaining part is (numerically) zero is dependent on earlier ones: its unknown is set to zero, which picks
// one of the system's solutions (any solution locates the same nodes, Lemma l9 case (ii)).
__device__ void wave_least_squares(solve_smem& S, int nr, int nc, int lane) {
  if (lane <= nc) {
    double sq = 0.0;
#pragma unroll 4
    for (int i = 0; i < nr; ++i) sq = fma(S.A[i][lane], S.A[i][lane], sq);
    S.cn[lane] = sqrt(sq);
  }
  __syncthreads();
  int row = 0;
  for (int k = 0; k < nc; ++k) {  // every lane follows the same control flow (all conditions are wave-uniform)
    bool dependent = row >= nr;
    double akk = 0.0, tail = 0.0, nrm = 0.0;
    if (!dependent) {
      const double below = (lane > row && lane < nr) ? S.A[lane][k] : 0.0;  // lane = row: the column's part below the pivot
      tail = wave_sum_all(below * below);
      akk = S.A[row][k];
      nrm = sqrt(fma(akk, akk, tail));
      dependent = !(nrm > SOLON_RANK_TOL * S.cn[k]);
    }
    if (dependent) {
      if (lane == 0) S.piv[k] = -1;
      continue;
    }
    const double alpha = akk >= 0.0 ? -nrm : nrm;
    const double v0 = akk - alpha;
    const double vtv = fma(v0, v0, tail);
    if (lane > k && lane <= nc) {
      double dot = v0 * S.A[row][lane];
#pragma unroll 4
      for (int i = row + 1; i < nr; ++i) dot = fma(S.A[i][k], S.A[i][lane], dot);
      const double cf = 2.0 * dot / vtv;
      S.A[row][lane] -= cf * v0;
#pragma unroll 4
      for (int i = row + 1; i < nr; ++i) S.A[i][lane] = fma(-cf, S.A[i][k], S.A[i][lane]);
    }
    __syncthreads();
    if (lane == 0) {
      S.A[row][k] = alpha;
      S.piv[k] = row;
    }
    __syncthreads();
    ++row;
  }
  // Back-substitution, column-oriented: lane j keeps the right-hand side of its column's pivot row; once x_k is known
  // every earlier column's lane takes its multiple of x_k off in parallel.
  const int myrow = lane < nc ? S.piv[lane] : -1;
  double y = myrow >= 0 ? S.A[myrow][nc] : 0.0;
  for (int k = nc - 1; k >= 0; --k) {
    const int r = __builtin_amdgcn_readlane(myrow, k);
    double xk = 0.0;
    if (r >= 0) {
      xk = lane_bcast(y, k) / S.A[r][k];
      if (lane < k && myrow >= 0) y = fma(-S.A[myrow][k], xk, y);
    }
    if (lane == k) S.x[k] = xk;
  }
  __syncthreads();
}

// |D(w_i)| for locator degrees up to SOLON_LANE_TEST_MAX without forming the system matrix: the same least-squares
// problem as wave_least_squares solves (numerator columns first, then the locator's, rows equilibrated), with lane =
// point.  The numerator's column space - polynomials of degree < m + se times the row scaling - gets an orthonormal
// basis from the three-term recurrence over the points, one degree at a time; the se + 1 columns y T_k(w) of the
// locator and the right-hand side are made orthogonal to each basis vector as it appears; what is left of them is a
// least-squares problem in the se locator coefficients alone, solved by Gram-Schmidt on those columns.  Two rounds
// of wavefront sums per degree (the se + 3 sums of a round share their latency) instead of a Householder sweep per
// column through LDS.  Only the first `rows` rows of 16 lanes hold points.
template <int SE>  // SE = locator degree
__device__ double locator_abs_values(double wl, double yl, bool pt, int m, int rows) {
  const double eq = pt ? 1.0 / fmax(1.0, fabs(yl)) : 0.0;  // row scaling; lanes without a point weigh nothing
  double c[SE + 1], cn0[SE + 1];
  {
    double t0 = 1.0, t1 = wl;
#pragma unroll
    for (int k = 0; k <= SE; ++k) {
      c[k] = eq * yl * t0;
      const double t2 = 2.0 * wl * t1 - t0;
      t0 = t1;
      t1 = t2;
    }
  }
  // One round of wavefront sums per degree: the next basis polynomial enters it UNNORMALISED (t, with |t|^2 among the
  // sums) and every other sum of the round is scaled afterwards, so that no sum has to wait for a norm.
  double p_cur = 0.0, t = eq;  // t: the polynomial of the current degree before normalisation
  {
    double v[SE + 2];
#pragma unroll
    for (int k = 0; k <= SE; ++k) v[k] = c[k] * c[k];
    v[SE + 1] = 0.0;
    wave_sums<SE + 2>(v, rows);
#pragma unroll
    for (int k = 0; k <= SE; ++k) cn0[k] = sqrt(v[k]);
  }
  const int nn = m + SE;
  for (int j = 0; j < nn; ++j) {
    const double xt = wl * t;
    double v[SE + 4];
#pragma unroll
    for (int k = 0; k <= SE; ++k) v[k] = c[k] * t;
    v[SE + 1] = t * t;
    v[SE + 2] = xt * t;
    v[SE + 3] = xt * p_cur;
    wave_sums<SE + 4>(v, rows);
    const double n2 = v[SE + 1];
    if (!(n2 > 1e-300)) break;  // fewer distinct weighted points than coefficients: nothing further to remove
    const double inv = 1.0 / sqrt(n2);
    const double p_new = t * inv;  // orthonormal polynomial of degree j
#pragma unroll
    for (int k = 0; k <= SE; ++k) c[k] = fma(-v[k] * inv, p_new, c[k]);
    // x p_new = (next) + alpha p_new + beta p_cur with alpha = <x p_new, p_new>, beta = <x p_new, p_cur>
    t = wl * p_new - (v[SE + 2] * inv * inv) * p_new - (v[SE + 3] * inv) * p_cur;
    p_cur = p_new;
  }
  // Gram-Schmidt on what is left of the locator columns (norm and dot products of a column in one round); a column
  // that has (numerically) nothing left is dependent on the earlier ones and gets coefficient zero, which picks one of
  // the system's solutions (Lemma l9, case ii)
  double r[SE][SE + 1];
  bool dep[SE];
#pragma unroll
  for (int k = 0; k < SE; ++k) {
    double v[SE + 1];
#pragma unroll
    for (int j = 0; j <= SE; ++j) v[j] = j >= k ? c[k] * c[j] : 0.0;
    wave_sums<SE + 1>(v, rows);
    const double nk = sqrt(v[k]);
    dep[k] = !(nk > SOLON_RANK_TOL * cn0[k]);
    const double ink = dep[k] ? 0.0 : 1.0 / nk;
    const double qk = c[k] * ink;
    r[k][k] = nk;
#pragma unroll
    for (int j = k + 1; j <= SE; ++j) {
      r[k][j] = v[j] * ink;
      c[j] = fma(-r[k][j], qk, c[j]);
    }
  }
  // sum_k x_k c_k ~ c_SE; the locator's coefficients are d_k = -x_k (the columns enter the system with a minus sign)
  double x[SE];
#pragma unroll
  for (int k = SE - 1; k >= 0; --k) {
    double t = r[k][SE];
#pragma unroll
    for (int j = k + 1; j < SE; ++j) t = fma(-r[k][j], x[j], t);
    x[k] = dep[k] ? 0.0 : t / r[k][k];
  }
  double dv = 0.0, t0 = 1.0, t1 = wl;
#pragma unroll
  for (int k = 0; k <= SE; ++k) {
    dv = fma(k < SE ? -x[k < SE ? k : 0] : 1.0, t0, dv);
    const double t2 = 2.0 * wl * t1 - t0;
    t0 = t1;
    t1 = t2;
  }
  return fabs(dv);
}

// Number of lanes (among `active`, all below `n`) whose value precedes this lane's in the total order (value, lane).
// The values go through LDS (`slot`, 64 doubles): every lane reads them back one by one, all lanes the same address.
__device__ int wave_rank(double* slot, double v, bool active, int n, int lane) {
  const unsigned long long mask = __ballot(active);
  __syncthreads();
  slot[lane] = v;
  __syncthreads();
  int rank = 0;
  for (int j = 0; j < n; ++j) {
    const double o = slot[j];
    if ((mask >> j) & 1ull) rank += (o < v || (o == v && j < lane)) ? 1 : 0;
  }
  __syncthreads();
  return rank;
}

// Lane holding the largest `key` (never negative) among the lanes with `valid` set, the lowest such lane on ties (-1 if
// there is none), among the first `rows` rows of 16 lanes.  The key's bit pattern - which orders non-negative doubles
// like integers - has its seven lowest bits replaced by 127 - lane, so one unsigned 64-bit maximum finds both.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void dpp_max_u64(unsigned long long& k) {
  const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp((int)(unsigned)k, (int)(unsigned)k, CTRL, ROW_MASK, 0xF, false);
  const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp((int)(unsigned)(k >> 32), (int)(unsigned)(k >> 32), CTRL, ROW_MASK, 0xF, false);
  const unsigned long long o = ((unsigned long long)hi << 32) | lo;
  k = o > k ? o : k;
}
__device__ int wave_argmax(double key, bool valid, int lane, int rows) {
  unsigned long long k = valid ? (((unsigned long long)__double_as_longlong(key) & ~127ull) | (unsigned long long)(127 - lane)) : 0ull;
  dpp_max_u64<0xB1, 0xF>(k);   // quad_perm [1,0,3,2]
  dpp_max_u64<0x4E, 0xF>(k);   // quad_perm [2,3,0,1]
  dpp_max_u64<0x141, 0xF>(k);  // row_half_mirror
  dpp_max_u64<0x140, 0xF>(k);  // row_mirror
  if (rows > 1) dpp_max_u64<0x142, 0xA>(k);  // row_bcast:15 into rows 1 and 3
  if (rows > 2) dpp_max_u64<0x143, 0xC>(k);  // row_bcast:31 into rows 2 and 3
  const int low = __builtin_amdgcn_readlane((int)(unsigned)k, __builtin_amdgcn_readfirstlane(rows * 16 - 1));
  return (low & 127) >= 64 ? 127 - (low & 127) : -1;
}

// Sum over the wavefront, identical bits in every lane.
__device__ __forceinline__ double wave_sum(double v) { return wave_sum_all(v); }

// Value at this lane's point x of the least-squares polynomial of degree m-1 through the points (x, y) of the lanes
// with `use` set.  Orthonormal polynomials of the discrete inner product over those points are generated by their
// three-term recurrence (lane = point, a handful of wave sums per degree); no matrix is formed.
__device__ double wave_polyfit(double x, double y, bool use, int m) {
  const double wgt = use ? 1.0 : 0.0;
  const double cnt = wave_sum(wgt);
  if (!(cnt > 0.0)) return 0.0;
  double p_prev = 0.0, p_cur = 1.0 / sqrt(cnt), fit = 0.0;
  for (int k = 0; k < m; ++k) {
    fit = fma(wave_sum(wgt * y * p_cur), p_cur, fit);
    if (k + 1 == m) break;
    const double xp = x * p_cur;
    const double alpha = wave_sum(wgt * xp * p_cur);
    const double beta = wave_sum(wgt * xp * p_prev);
    const double q = xp - alpha * p_cur - beta * p_prev;
    const double nrm = sqrt(wave_sum(wgt * q * q));
    if (!(nrm > 1e-150)) break;  // fewer distinct points than coefficients: the remaining terms stay zero
    p_prev = p_cur;
    p_cur = q / nrm;
  }
  return fit;
}

// ------------------------------------------------------------------------------------------------
// Candidate sets.  "Is S the corrupted set?" means: does the least-squares polynomial of degree m-1 through the points
// outside S pass within tau of all of them.  With Q an orthonormal basis of the polynomials over ALL points of the
// group, r = y - Q Q^T y the residual of the fit through all points and M = I - Q Q^T, leaving S out of the fit is the
// same as giving every point of S a free parameter delta: M_SS delta = r_S, and the residuals of the other points
// are r_k - sum_{j in S} M_kj delta_j.  That is a |S| x |S| Cholesky solve plus |S| multiply-adds per point, small
// enough for ONE LANE, so 64 candidate sets are judged at a time.  (The projections enter clamped to +-1e8 medians:
// a larger value can only belong to a corrupted point - the median is an honest magnitude - and inside S a point's
// value does not matter, while unclamped its 1e-16 relative rounding would swamp tau in r.)

// Binomial coefficients C(a, i), saturating at 2^30 (item numbers stay below SOLON_SEARCH_LIMIT).
struct binom_table {
  uint32_t c[65][34];
};
constexpr binom_table make_binom_table() {
  binom_table t{};
  for (int a = 0; a <= 64; ++a) {
    for (int i = 0; i < 34; ++i) {
      uint64_t v = i == 0 ? 1 : (a == 0 ? 0 : (uint64_t)t.c[a - 1][i - 1] + t.c[a - 1][i]);
      t.c[a][i] = v > (1u << 30) ? (1u << 30) : (uint32_t)v;
    }
  }
  return t;
}
static __device__ const binom_table g_binom = make_binom_table();

__device__ __forceinline__ unsigned long long lane_bcast_mask(unsigned long long v, int src) {
  const unsigned lo = (unsigned)__shfl((int)(unsigned)v, src, 64);
  const unsigned hi = (unsigned)__shfl((int)(unsigned)(v >> 32), src, 64);
  return ((unsigned long long)hi << 32) | lo;
}

// Orthonormal polynomials of degree < m over the points (three-term recurrence, lane = point): q[k] = value of the k-th one at
// this lane's point, fit = this lane's value of the projection of yc onto them.  One round of wavefront sums per degree.
template <int MM>  // MM >= m: number of basis polynomials the registers hold
__device__ __forceinline__ void lane_basis(double x, double yc, double wgt, int m, int rows, double (&q)[MM], double& fit) {
  double p_cur = 0.0, t = wgt;  // t: the polynomial of the current degree before normalisation
  fit = 0.0;
#pragma unroll
  for (int k = 0; k < MM; ++k) q[k] = 0.0;
#pragma unroll
  for (int k = 0; k < MM; ++k) {
    if (k < m) {  // wave-uniform; one round of sums per degree, scaled by the norm afterwards
      const double xt = x * t;
      double v[4] = {t * t, yc * t, xt * t, xt * p_cur};
      wave_sums<4>(v, rows);
      const double inv = v[0] > 1e-300 ? 1.0 / sqrt(v[0]) : 0.0;  // fewer distinct points than coefficients cannot happen (n >= m + s)
      const double p_new = t * inv;
      q[k] = p_new;
      fit = fma(v[1] * inv, p_new, fit);
      t = x * p_new - (v[2] * inv * inv) * p_new - (v[3] * inv) * p_cur;
      p_cur = p_new;
    }
  }
}

// Orthonormal basis Q, residual r = y - Q Q^T y into S.val, and M = I - Q Q^T into S.A (lane = row).  `n` points, lanes
// 0 .. n-1.  The basis depends on the points alone, so a plan keeps it in a table (`qrow`: this lane's row of it, or null when
// there is no table or some point of the group dropped out as non-finite); with it the m dependent rounds of sums shrink to
// ceil(m / 4) independent ones for the projection of y.
template <int MM>
__device__ void lane_test_setup(solve_smem& S, double x, double y, int n, int m, int lane, const double* qrow, bool have_table) {
  const bool pt = lane < n;
  const int rows = n <= 16 ? 1 : n <= 32 ? 2 : 4;
  const double yc = fmin(fmax(y, -SOLON_Y_CLAMP), SOLON_Y_CLAMP);
  double q[MM], fit;
  if (have_table) {
#pragma unroll
    for (int k = 0; k < MM; ++k) q[k] = (pt && k < m) ? qrow[k] : 0.0;
    fit = 0.0;
#pragma unroll
    for (int k0 = 0; k0 < MM; k0 += 4) {
      if (k0 < m) {  // wave-uniform
        double v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = k0 + e < MM ? yc * q[k0 + e] : 0.0;
        wave_sums<4>(v, rows);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (k0 + e < MM) fit = fma(v[e], q[k0 + e], fit);
      }
    }
  } else {
    lane_basis<MM>(x, yc, pt ? 1.0 : 0.0, m, rows, q, fit);
  }
  __syncthreads();  // S.A, S.val are free again
#pragma unroll
  for (int k = 0; k < MM; ++k) S.Q[lane][k] = q[k];
  S.val[lane] = pt ? yc - fit : 0.0;
  __syncthreads();
  for (int j = 0; j < n; ++j) {
    double acc = (j == lane) ? 1.0 : 0.0;
#pragma unroll
    for (int k = 0; k < MM; ++k) acc = fma(-q[k], S.Q[j][k], acc);  // q[k] = 0 beyond m
    S.A[lane][j] = acc;
  }
  __syncthreads();
}

// The table of lane_test_setup for every group of a plan: qtab[position in grp_nodes][k], one wavefront per group.
__global__ __launch_bounds__(64) void basis_table_kernel(const int32_t* __restrict__ grp_off, const int32_t* __restrict__ grp_nodes,
                                                         const float* __restrict__ w, int m, double yc0, double* __restrict__ qtab) {
  const int g = blockIdx.x, lane = threadIdx.x;
  const int n0 = grp_off[g], n = grp_off[g + 1] - n0;
  if (n > 64) return;  // wave-uniform
  const bool pt = lane < n;
  const double x = pt ? (double)w[grp_nodes[n0 + lane]] : 0.0;
  const int rows = n <= 16 ? 1 : n <= 32 ? 2 : 4;
  double q[SOLON_MAX_M], fit;
  // the same instantiation as the solve wavefront takes for this m (yc0 = 0 arrives as an argument, so nothing is folded away)
  if (m <= 4) {
    double q4[4];
    lane_basis<4>(x, yc0, pt ? 1.0 : 0.0, m, rows, q4, fit);
#pragma unroll
    for (int k = 0; k < SOLON_MAX_M; ++k) q[k] = k < 4 ? q4[k < 4 ? k : 0] : 0.0;
  } else if (m <= 8) {
    double q8[8];
    lane_basis<8>(x, yc0, pt ? 1.0 : 0.0, m, rows, q8, fit);
#pragma unroll
    for (int k = 0; k < SOLON_MAX_M; ++k) q[k] = k < 8 ? q8[k < 8 ? k : 0] : 0.0;
  } else if (m <= 12) {
    double q12[12];
    lane_basis<12>(x, yc0, pt ? 1.0 : 0.0, m, rows, q12, fit);
#pragma unroll
    for (int k = 0; k < SOLON_MAX_M; ++k) q[k] = k < 12 ? q12[k < 12 ? k : 0] : 0.0;
  } else {
    lane_basis<SOLON_MAX_M>(x, yc0, pt ? 1.0 : 0.0, m, rows, q, fit);
  }
  if (pt) {
#pragma unroll
    for (int k = 0; k < SOLON_MAX_M; ++k) qtab[(int64_t)(n0 + lane) * SOLON_MAX_M + k] = q[k];
  }
}

// One lane's verdict on one candidate set `mask` (bits = points) of at most E points.
template <int E>
__device__ bool lane_test(const solve_smem& S, unsigned long long mask, int n) {
  int el[E];
  bool have[E];
  double b[E], inv[E], L[E * (E + 1) / 2];
  unsigned long long mm = mask;
#pragma unroll
  for (int a = 0; a < E; ++a) {
    have[a] = mm != 0;
    el[a] = have[a] ? __ffsll((long long)mm) - 1 : 0;
    mm &= mm - 1;
    b[a] = have[a] ? S.val[el[a]] : 0.0;
  }
  // M_SS, padded with the identity where the set has fewer than E points
#pragma unroll
  for (int a = 0; a < E; ++a) {
#pragma unroll
    for (int c = 0; c <= a; ++c) {
      const double g = S.A[el[a]][el[c]];
      L[a * (a + 1) / 2 + c] = have[a] ? g : (a == c ? 1.0 : 0.0);
    }
  }
  bool ok = true;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    double d = L[j * (j + 1) / 2 + j];
#pragma unroll
    for (int k = 0; k < j; ++k) d = fma(-L[j * (j + 1) / 2 + k], L[j * (j + 1) / 2 + k], d);
    const bool good = d > SOLON_CHOL_MIN;  // false for NaN too
    ok = ok && good;
    const double dd = good ? d : 1.0;
    double rs = __builtin_amdgcn_rsq(dd);  // hardware estimate, then two Newton steps: full double precision
    rs = rs * fma(-0.5 * dd * rs, rs, 1.5);
    rs = rs * fma(-0.5 * dd * rs, rs, 1.5);
    inv[j] = rs;
#pragma unroll
    for (int i = j + 1; i < E; ++i) {
      double t = L[i * (i + 1) / 2 + j];
#pragma unroll
      for (int k = 0; k < j; ++k) t = fma(-L[i * (i + 1) / 2 + k], L[j * (j + 1) / 2 + k], t);
      L[i * (i + 1) / 2 + j] = t * inv[j];
    }
  }
  double dl[E];
#pragma unroll
  for (int a = 0; a < E; ++a) {  // L z = r_S
    double t = b[a];
#pragma unroll
    for (int c = 0; c < a; ++c) t = fma(-L[a * (a + 1) / 2 + c], dl[c], t);
    dl[a] = t * inv[a];
  }
#pragma unroll
  for (int a = E - 1; a >= 0; --a) {  // L^T delta = z
    double t = dl[a];
#pragma unroll
    for (int c = a + 1; c < E; ++c) t = fma(-L[c * (c + 1) / 2 + a], dl[c], t);
    dl[a] = t * inv[a];
  }
#pragma unroll 4
  for (int k = 0; k < n; ++k) {
    double res = S.val[k];
#pragma unroll
    for (int a = 0; a < E; ++a) res = fma(-S.A[el[a]][k], dl[a], res);  // delta is zero in the padding
    const bool inside = (mask >> k) & 1ull;
    ok = ok && (inside || fabs(res) <= SOLON_TAU);
  }
  return ok;
}

// The same verdict by the whole wavefront (any set size): fit through the points outside `mask`, lane = point.
__device__ bool wave_test(double x, double y, int n, int m, unsigned long long mask, int lane) {
  const bool keep = lane < n && !((mask >> lane) & 1ull);
  const double fitted = wave_polyfit(x, y, keep, m);
  return __ballot(keep && !(fabs(fitted - y) <= SOLON_TAU)) == 0;
}

struct test_ctx {
  double x, y;  // this lane's point (compacted position = lane)
  int n, m, se, lane;
  const double* qrow;  // this lane's row of the plan's basis table, when have_table
  bool have_table;     // wave-uniform: the table exists and every point of the group is finite
};

// Verdicts on the candidate sets of the lanes with `active` set: bit l = lane l's set explains the group.  Locator
// degrees above SOLON_LANE_TEST_MAX take the sets one after the other through the whole wavefront and stop at the
// first that passes (the callers only use the lowest set bit).
__device__ unsigned long long test_batch(const solve_smem& S, const test_ctx& c, unsigned long long mask, bool active) {
  if (c.se <= SOLON_LANE_TEST_MAX) {
    bool ok = false;
    switch (c.se) {
      case 0: case 1: ok = lane_test<1>(S, mask, c.n); break;
      case 2: ok = lane_test<2>(S, mask, c.n); break;
      case 3: ok = lane_test<3>(S, mask, c.n); break;
      case 4: ok = lane_test<4>(S, mask, c.n); break;
      case 5: ok = lane_test<5>(S, mask, c.n); break;
      case 6: ok = lane_test<6>(S, mask, c.n); break;
      case 7: ok = lane_test<7>(S, mask, c.n); break;
      default: ok = lane_test<8>(S, mask, c.n); break;
    }
    return __ballot(active && ok);
  }
  unsigned long long todo = __ballot(active);
  while (todo) {
    const int l = __ffsll((long long)todo) - 1;
    todo &= todo - 1;
    if (wave_test(c.x, c.y, c.n, c.m, lane_bcast_mask(mask, l), c.lane)) return 1ull << l;
  }
  return 0;
}

// Candidate set number t of the widened search: sets are ordered by the position c of their last point in the
// |D| order, then by size e = 1 .. se, then colexicographically in the other e-1 points (positions below c - 1
// in the |D| order), so every subset of the c leading points comes before any that needs a later point.
__device__ unsigned long long widened_set(const solve_smem& S, uint32_t t, int n, int se) {
  int c = 1;
  while (c < n && t >= S.cnt[c]) ++c;
  uint32_t idx = t - S.cnt[c - 1];
  int e = 1;
  for (; e < se; ++e) {
    const uint32_t ne = g_binom.c[c - 1][e - 1];
    if (idx < ne) break;
    idx -= ne;
  }
  unsigned long long mk = 1ull << S.by_rank[c - 1];
  int a = c - 2;
  for (int i = e - 1; i >= 1; --i) {  // combinatorial number system: the largest a with C(a, i) <= idx, then the rest
    while (g_binom.c[a][i] > idx) --a;
    mk |= 1ull << S.by_rank[a];
    idx -= g_binom.c[a][i];
    --a;
  }
  return mk;
}

// The located set of one group as a mask over its (finite) points, or found = false.  `drank` is this point's
// position in the order of increasing |D(w_i)|.
__device__ unsigned long long search_located_set(solve_smem& S, const test_ctx& c, int drank, uint32_t limit, bool* found_out) {
  const int lane = c.lane, n = c.n, se = c.se;
  const bool pt = lane < n;
  if (pt) S.by_rank[drank] = lane;
  __syncthreads();
  if (se <= SOLON_LANE_TEST_MAX) {
    if (c.m <= 4) lane_test_setup<4>(S, c.x, c.y, n, c.m, lane, c.qrow, c.have_table);
    else if (c.m <= 8) lane_test_setup<8>(S, c.x, c.y, n, c.m, lane, c.qrow, c.have_table);
    else if (c.m <= 12) lane_test_setup<12>(S, c.x, c.y, n, c.m, lane, c.qrow, c.have_table);
    else lane_test_setup<SOLON_MAX_M>(S, c.x, c.y, n, c.m, lane, c.qrow, c.have_table);
  }
  // 1. the leading roots of the locator: lane e <= se leaves out the e first points of the |D| order.  The lanes after
  // them (one candidate set per lane) already try each of those sets with one of its points but the last put back -
  // without the last one it is the next smaller leading set - so that step 3 can usually be skipped.
  const bool per_lane = se <= SOLON_LANE_TEST_MAX;
  int e_of = lane <= se ? lane : -1, j_of = -1;
  if (per_lane && lane > se) {
    int idx = lane - (se + 1);
    for (int e = 2; e <= se; ++e) {
      if (idx < e - 1) {
        e_of = e;
        j_of = idx;
        break;
      }
      idx -= e - 1;
    }
  }
  unsigned long long mask = 0;
  for (int k = 0; k < se; ++k)
    if (k < e_of && k != j_of) mask |= 1ull << S.by_rank[k];
  unsigned long long pass = test_batch(S, c, mask, e_of >= 0);
  const unsigned long long lead = pass & ((2ull << se) - 1ull);
  bool found = lead != 0;
  bool reduce = true;  // is step 3 still to be done
  unsigned long long located = 0;
  if (found) {
    const int e = __ffsll((long long)lead) - 1;
    located = lane_bcast_mask(mask, e);
    if (per_lane) {  // lanes se + 1 + (e - 2)(e - 1) / 2 ... hold this set's put-backs
      const int first = se + 1 + (e - 2) * (e - 1) / 2;
      reduce = e >= 2 && ((pass >> first) & ((1ull << (e - 1)) - 1ull)) != 0;
    }
  }
  // 2. every subset of at most se points
  if (!found && se > 0) {
    if (lane >= 1 && lane <= n) {
      uint32_t cnt = 0;
      for (int e = 1; e <= se; ++e) cnt = min(cnt + g_binom.c[lane - 1][e - 1], 1u << 30);
      S.cnt[lane] = cnt;
    }
    if (lane == 0) S.cnt[0] = 0;
    __syncthreads();
    if (lane == 0)
      for (int k = 1; k <= n; ++k) S.cnt[k] = min(S.cnt[k] + S.cnt[k - 1], 1u << 30);
    __syncthreads();
    const uint32_t total = min(S.cnt[n], limit);
    for (uint32_t base = 0; base < total && !found; base += 64) {
      const uint32_t t = base + lane;
      const bool active = t < total;
      mask = active ? widened_set(S, t, n, se) : 0;
      pass = test_batch(S, c, mask, active);
      if (pass) {
        found = true;
        reduce = true;
        located = lane_bcast_mask(mask, __ffsll((long long)pass) - 1);
      }
    }
  }
  // 3. smallest set: put back every point the others stay consistent with (lowest point first, one at a time)
  while (found && reduce && located) {
    const int e = __popcll(located);
    mask = located;
    for (int k = 0; k < lane && k < e; ++k) mask &= mask - 1;  // drop the `lane` lowest points ...
    const unsigned long long mine = mask & (~mask + 1);          // ... the next one is this lane's
    mask = located & ~mine;
    pass = test_batch(S, c, mask, lane < e);
    if (!pass) break;
    located = lane_bcast_mask(mask, __ffsll((long long)pass) - 1);
  }
  *found_out = found;
  return located;
}

// mode: SOLVE_TABLES = psi's tables for the located set already in vmask; SOLVE_LOCATE = phi, then psi's tables;
// SOLVE_SPECULATE = phi on a projection of a sample of the columns, as a guess of the located set for the fused
// locate + decode pass: never fails (a group it cannot explain is taken as clean) and leaves vmask and status alone.
struct solve_args {
  int s, m, mode;
  int blind;                  // SOLVE_SPECULATE: skip phi and guess that every node is honest (times the repeated recombination)
  const int32_t* guess_rows;  // SOLVE_LOCATE: rows a speculative recombination used, or null
  int32_t* redo;              // set to 1 when some group's rows differ from guess_rows; SOLVE_SPECULATE clears it
  int32_t* order;             // SOLVE_SPECULATE: every group's nodes, the chosen rows first
  const int32_t* grp_off;
  const int32_t* grp_nodes;
  const float* w;
  const double* rho;
  const double* qtab;         // [n_active][SOLON_MAX_M] orthonormal basis of every group's points (basis_table_kernel), or null
  int32_t* vmask;
  int32_t* status;
  int32_t* dec_rows;
  float* dec_coef;
};

__global__ __launch_bounds__(64) void solve_kernel(solve_args a) {
  __shared__ solve_smem S;
  const int g = blockIdx.x, lane = threadIdx.x;
  const int n0 = a.grp_off[g], n = a.grp_off[g + 1] - n0;
  const int m = a.m, s = a.s;
  const bool in_group = lane < n;
  const int node = in_group ? a.grp_nodes[n0 + lane] : -1;
  const double wi = in_group ? (double)a.w[node] : 0.0;
  int st = SOLON_OK;
  bool located = false;
  if (a.mode == SOLVE_SPECULATE && g == 0 && lane == 0) *a.redo = 0;

  if (a.mode == SOLVE_SPECULATE && a.blind) {
    // nothing located: psi's tables below are those of a clean group
  } else if (a.mode != SOLVE_TABLES) {
    const double rho = in_group ? a.rho[node] : 0.0;
    const bool finite = in_group && isfinite(rho);
    const unsigned long long fin_mask = __ballot(finite);
    const int nfin = __popcll(fin_mask);
    const int nnonfin = n - nfin;
    located = in_group && !finite;  // a non-finite projection names its sender at once
    if (nnonfin > s) {
      st = SOLON_E_DECODE;
    } else if (nfin > 0) {
      // scale: median |rho| over the finite entries (honest nodes are a strict majority); max if that is zero
      const double ar = fabs(rho);
      const int rk = wave_rank(S.x, ar, finite, n, lane);
      if (finite && rk == (nfin - 1) / 2) S.med[0] = ar;
      if (finite && rk == nfin / 2) S.med[1] = ar;
      __syncthreads();
      double scale = 0.5 * (S.med[0] + S.med[1]);
      if (scale == 0.0) {
        const int top = nfin - 1;
        __syncthreads();
        if (finite && rk == top) S.med[0] = ar;
        __syncthreads();
        scale = S.med[0];
      }
      __syncthreads();
      if (scale > 0.0) {
        // compact the finite points: position = number of finite lanes below this one
        const int pos = __popcll(fin_mask & ((1ull << lane) - 1ull));
        const double yi = finite ? rho / scale : 0.0;
        if (finite) {
          S.y[pos] = yi;
          S.wv[pos] = wi;
        }
        __syncthreads();
        const int se = s - nnonfin;  // locator degree left for the finite points
        const bool pt = lane < nfin;
        const double yl = pt ? S.y[lane] : 0.0, wl = pt ? S.wv[lane] : 0.0;
        int drank = 64;  // position of this point in the order of increasing |D(w_i)| (locator roots first)
        if (se > 0) {
          const int nn = m + se;      // numerator unknowns (Chebyshev coefficients 0 .. m+se-1)
          const int nc = nn + se;     // + locator unknowns (coefficients 0 .. se-1; T_se has coefficient one)
          double dv = 0.0;
          if (se <= SOLON_LANE_TEST_MAX) {
            const int rows = nfin <= 16 ? 1 : nfin <= 32 ? 2 : 4;
            switch (se) {
              case 1: dv = locator_abs_values<1>(wl, yl, pt, m, rows); break;
              case 2: dv = locator_abs_values<2>(wl, yl, pt, m, rows); break;
              case 3: dv = locator_abs_values<3>(wl, yl, pt, m, rows); break;
              case 4: dv = locator_abs_values<4>(wl, yl, pt, m, rows); break;
              case 5: dv = locator_abs_values<5>(wl, yl, pt, m, rows); break;
              case 6: dv = locator_abs_values<6>(wl, yl, pt, m, rows); break;
              case 7: dv = locator_abs_values<7>(wl, yl, pt, m, rows); break;
              default: dv = locator_abs_values<8>(wl, yl, pt, m, rows); break;
            }
          } else {
            if (pt) {
              const double eq = 1.0 / fmax(1.0, fabs(yl));
              double t0 = 1.0, t1 = wl;
              for (int k = 0; k < nn; ++k) {  // se < nn
                if (k < nn) S.A[lane][k] = t0 * eq;
                if (k < se) S.A[lane][nn + k] = -yl * t0 * eq;
                if (k == se) S.A[lane][nc] = yl * t0 * eq;
                const double t2 = 2.0 * wl * t1 - t0;
                t0 = t1;
                t1 = t2;
              }
            }
            __syncthreads();
            wave_least_squares(S, nfin, nc, lane);
            // |D(w_i)|: every corrupted point is a root of every solution's locator polynomial
            if (pt) {
              double t0 = 1.0, t1 = wl;
              for (int k = 0; k <= se; ++k) {
                dv = fma(k < se ? S.x[nn + k] : 1.0, t0, dv);
                const double t2 = 2.0 * wl * t1 - t0;
                t0 = t1;
                t1 = t2;
              }
              dv = fabs(dv);
            }
          }
          drank = wave_rank(S.x, dv, pt, nfin, lane);
        }
        // V: the smallest set of points without which the rest is consistent (leading roots first, then wider)
        test_ctx tc;
        tc.x = wl; tc.y = yl; tc.n = nfin; tc.m = m; tc.se = se; tc.lane = lane;
        tc.have_table = a.qtab != nullptr && nnonfin == 0;  // all points finite: compacted position = position in the group
        tc.qrow = tc.have_table && pt ? a.qtab + (int64_t)(n0 + lane) * SOLON_MAX_M : nullptr;
        if (se == 0 && pt) drank = lane;
        bool consistent = false;
        const unsigned long long flag_mask = search_located_set(S, tc, drank, a.mode == SOLVE_SPECULATE ? SOLON_SPEC_SEARCH_LIMIT : SOLON_SEARCH_LIMIT, &consistent);
        if (!consistent) st = SOLON_E_DECODE;
        if (finite && ((flag_mask >> pos) & 1ull)) located = true;
      }
    }
    if (a.mode == SOLVE_SPECULATE) {
      if (st != SOLON_OK) {  // the sample cannot be explained: guess that the group is clean
        st = SOLON_OK;
        located = false;
      }
    } else if (in_group) {
      a.vmask[node] = located ? 1 : 0;
    }
  } else {
    located = in_group && a.vmask[node] != 0;
  }

  // ---- psi set-up: m honest nodes in Leja order (each next point maximises the product of distances to the
  // ones already taken), which keeps the m x m Vandermonde well conditioned; then its inverse, column t of
  // which holds the monomial coefficients of the Lagrange basis polynomial of the t-th chosen point.
  const bool honest = in_group && !located;
  const int nh = __popcll(__ballot(honest));
  if (st == SOLON_OK && nh < m) st = SOLON_E_DECODE;
  if (st == SOLON_OK) {
    bool taken = false;
    double prod = fabs(wi);  // first pick: largest |w|
    const int rows_g = n <= 16 ? 1 : n <= 32 ? 2 : 4;
    for (int t = 0; t < m; ++t) {
      const int sel = wave_argmax(prod, honest && !taken, lane, rows_g);  // largest product, lowest lane on ties; nh >= m: never -1
      if (lane == sel) taken = true;
      const double dist = fabs(wi - lane_bcast(wi, sel));
      prod = (t == 0) ? dist : prod * dist;
    }
    const unsigned long long taken_mask = __ballot(taken);
    const int tpos = __popcll(taken_mask & ((1ull << lane) - 1ull));  // ascending node order
    if (taken) {
      S.val[tpos] = wi;
      a.dec_rows[g * m + tpos] = node;
    }
    if (a.mode == SOLVE_SPECULATE && in_group) {  // node order for the fused pass: chosen rows first, then the others
      const unsigned long long rest = __ballot(in_group && !taken);
      a.order[n0 + (taken ? tpos : m + __popcll(rest & ((1ull << lane) - 1ull)))] = node;
    }
    if (a.mode == SOLVE_LOCATE && a.guess_rows) {  // same rows in the same order give the same table
      const bool differs = taken && a.guess_rows[g * m + tpos] != node;
      if (__ballot(differs) && lane == 0) *a.redo = 1;
    }
    __syncthreads();
    if (taken) {  // this lane's Lagrange basis polynomial: prod over the other chosen points of (w - w_u) / (w_t - w_u)
      double poly[SOLON_MAX_M];
#pragma unroll
      for (int l = 0; l < SOLON_MAX_M; ++l) poly[l] = l == 0 ? 1.0 : 0.0;
      double den = 1.0;
      for (int u = 0; u < m; ++u) {
        const double wu = S.val[u];
        if (u != tpos) {  // multiply by (w - w_u); coefficients above the current degree are zero and stay zero
#pragma unroll
          for (int l = SOLON_MAX_M - 1; l >= 1; --l) poly[l] = fma(-wu, poly[l], poly[l - 1]);
          poly[0] = -wu * poly[0];
          den *= (wi - wu);
        }
      }
      const double inv_den = 1.0 / den;
#pragma unroll
      for (int l = 0; l < SOLON_MAX_M; ++l) S.lag[tpos][l] = poly[l] * inv_den;
    }
    __syncthreads();
    double rowsum = 0.0;
    if (lane < m) {
      for (int t = 0; t < m; ++t) {
        const double c = S.lag[t][lane];
        rowsum += fabs(c);
        a.dec_coef[(g * m + t) * m + lane] = (float)c;  // T[g][l][t], stored with l fastest
      }
    }
    const unsigned long long bad = __ballot(lane < m && !(rowsum <= SOLON_INV_NORM_MAX));
    if (bad) st = SOLON_E_NUMERIC;
  }
  if (a.mode == SOLVE_LOCATE && a.guess_rows && st != SOLON_OK && lane == 0) *a.redo = 1;
  if (lane == 0 && a.mode != SOLVE_SPECULATE) a.status[g] = st;
}

int solon_launch_solve_on(const solon_plan* plan, const solon_dev& D, int mode, hipStream_t st) {
  solve_args a;
  a.s = plan->s; a.m = plan->m; a.mode = mode;
  a.blind = mode == SOLVE_SPECULATE && solon_tuning("fuse_blind_guess", 0) != 0;
  a.grp_off = D.grp_off; a.grp_nodes = D.grp_nodes; a.w = D.w; a.rho = D.rho;
  a.qtab = solon_tuning("solve_basis_table", 1) != 0 ? D.qtab : nullptr;
  a.vmask = D.vmask; a.status = D.status; a.redo = D.redo;
  a.guess_rows = nullptr;
  a.order = D.spec_order;
  a.dec_rows = D.dec_rows; a.dec_coef = D.dec_coef;
  if (mode == SOLVE_SPECULATE) {
    a.dec_rows = D.spec_rows; a.dec_coef = D.spec_coef;
  } else if (mode == SOLVE_LOCATE_CHECK) {
    a.mode = SOLVE_LOCATE; a.guess_rows = D.spec_rows;
  }
  hipLaunchKernelGGL(solve_kernel, dim3(plan->q), dim3(64), 0, st, a);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

int solon_launch_basis_table(const solon_plan* plan, const solon_dev& D, hipStream_t st) {
  if (!D.qtab || plan->q < 1) return SOLON_OK;
  hipLaunchKernelGGL(basis_table_kernel, dim3(plan->q), dim3(64), 0, st, D.grp_off, D.grp_nodes, D.w, plan->m, 0.0, D.qtab);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

int solon_launch_solve(solon_plan* plan, int mode, hipStream_t st) { return solon_launch_solve_on(plan, plan->dev, mode, st); }

int solon_collect_status(solon_plan* plan, hipStream_t st, int32_t* vmask_host /*P or null*/, double* rho_host /*P or null*/) {
  // staging layout: [double rho[P]] [int32 vmask[P]] [int32 status[q]]
  char* base = (char*)plan->pinned;
  double* h_rho = (double*)base;
  int32_t* h_vmask = (int32_t*)(base + sizeof(double) * plan->P);
  int32_t* h_status = h_vmask + plan->P;
  if (rho_host) SOLON_HIP(hipMemcpyAsync(h_rho, plan->dev.rho, sizeof(double) * plan->P, hipMemcpyDeviceToHost, st));
  if (vmask_host) SOLON_HIP(hipMemcpyAsync(h_vmask, plan->dev.vmask, sizeof(int32_t) * plan->P, hipMemcpyDeviceToHost, st));
  SOLON_HIP(hipMemcpyAsync(h_status, plan->dev.status, sizeof(int32_t) * plan->q, hipMemcpyDeviceToHost, st));
  SOLON_HIP(hipStreamSynchronize(st));
  if (rho_host) std::copy(h_rho, h_rho + plan->P, rho_host);
  if (vmask_host) std::copy(h_vmask, h_vmask + plan->P, vmask_host);
  int worst = SOLON_OK;
  for (int g = 0; g < plan->q; ++g) {
    if (h_status[g] != SOLON_OK && worst == SOLON_OK) {
      worst = h_status[g];
      if (worst == SOLON_E_DECODE) solon_set_error("group %d cannot be explained by <= s = %d corrupted nodes", g, plan->s);
      else solon_set_error("group %d: the m x m Vandermonde of the chosen honest nodes is too ill-conditioned", g);
    }
  }
  return worst;
}

extern "C" int solon_locate(solon_plan* plan, const float* R, int64_t ldr, const float* f, int32_t* byz_idx, int32_t* n_byz,
                            double* rho_out, void* hip_stream) {
  if (!plan || !R || !f) {
    solon_set_error("solon_locate: null argument");
    return SOLON_E_INVAL;
  }
  if (ldr < plan->d_c) {
    solon_set_error("solon_locate: ldr %lld < d_c %lld", (long long)ldr, (long long)plan->d_c);
    return SOLON_E_INVAL;
  }
  if (!plan->ws) {
    solon_set_error("solon_locate: the plan has no device workspace (no GPU at creation)");
    return SOLON_E_HIP;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  int rc = solon_launch_project(plan, R, ldr, f, st);
  if (rc != SOLON_OK) return rc;
  rc = solon_launch_solve(plan, SOLVE_LOCATE, st);
  if (rc != SOLON_OK) return rc;
  if (!byz_idx && !n_byz && !rho_out) return SOLON_OK;
  std::vector<int32_t> vm(plan->P);
  rc = solon_collect_status(plan, st, vm.data(), rho_out);
  if (rc == SOLON_E_HIP) return rc;
  int cnt = 0;
  for (int j = 0; j < plan->P; ++j) {
    if (plan->group_of_node[j] >= 0 && vm[j]) {
      if (byz_idx && cnt < plan->q * plan->s) byz_idx[cnt] = j;
      ++cnt;
    }
  }
  if (n_byz) *n_byz = cnt;
  return rc;
}

extern "C" int solon_decode_status(solon_plan* plan, void* hip_stream) {
  if (!plan) {
    solon_set_error("solon_decode_status: null plan");
    return SOLON_E_INVAL;
  }
  if (!plan->ws) {
    solon_set_error("solon_decode_status: the plan has no device workspace");
    return SOLON_E_HIP;
  }
  return solon_collect_status(plan, (hipStream_t)hip_stream, nullptr, nullptr);
}
