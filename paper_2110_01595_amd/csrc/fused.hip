// phi and psi in one pass over R (paper Sec. 3.4 and Algorithm 1; the step after the path, "decode", needs only m
// honest rows per group, all of which the projection rho = f R reads anyway).
//
// solon_locate followed by solon_decode reads R 1 + q m / P times.  Here the rows for psi are GUESSED first, the
// single pass over R then produces both the exact projections of all P rows and the recombination of the guessed
// rows, and the error-locator solve on the exact projections decides - as in solon_locate - which nodes are
// corrupt.  If none of the guessed rows is among them the recombination already is the result; otherwise (a device-side
// flag, no host round trip) the ordinary recombination kernels run after all.  The guess comes from the locator
// itself, run on the projection of a small leading sample of the columns: a node whose corruption shows in the
// sample is avoided, so the second pass is needed only against an adversary that corrupts nothing but columns
// outside the sample.  The located set and the status never depend on the guess.
//
// The pass is a persistent grid; each time round a thread takes FUSE_U float4 column units through all groups: fp64
// partial projections of every row (reduced over each wavefront by lane permutations, over the block through LDS,
// one partial per block, round and row, summed in fixed order afterwards) and the fp32 recombination of the
// guessed rows, kept in registers and stored at the end of the round.  Writes are 4 % of the traffic here, and waiting
// for the whole chip at the alignment points, as the encoder does, was measured to buy nothing for this pass: the spin
// limit defaults to zero, which leaves a block-wide pause between a block's reads and its stores and nothing more.
#include <algorithm>
#include <vector>

#include "grid_phase.h"
#include "solon_internal.h"
#include "wave_ops.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define FUSE_U 2      // float4 column units per thread and phase
#define FUSE_BLOCK 1024
#define FUSE_SAMPLE (1 << 17)  // columns of the sample projection behind the guess

struct fuse_args {
  const float* R;
  int64_t ldr;
  const float* f;
  int64_t nunits;  // float4 column units: columns [0, 4 nunits), all of whose chunks lie below d
  int P, q;
  const int32_t* grp_off;
  const int32_t* order;  // every group's nodes, the guessed rows first
  const float* coef;    // their table, [q][m][m]
  double* partials;     // [pass * gridDim.x + block][P]
  float* u;
  uint32_t* sync;
  int spin_limit;
};

// rows of R loaded back to back: as many as leave four waves per SIMD resident without spills
constexpr int fuse_rows(int m) { return m == 4 ? 6 : 8; }

// Dynamic LDS: one fp64 slot per (wavefront, node).  A wavefront parks the sums of its own columns there row by row,
// so the loop over the groups needs no block-wide synchronisation (wavefronts that run in lockstep leave HBM idle while they
// all compute); the block adds the wavefronts' slots in fixed order once per tile.
// The three small tables come in as separate restrict-qualified read-only arguments so that the compiler may fetch
// them through the scalar cache (a vector load of a wave-uniform index costs a full memory round trip before the
// batch's row loads can even be issued).
template <int M>
__global__ __launch_bounds__(FUSE_BLOCK, 4) void project_recombine_kernel(fuse_args a, const int32_t* __restrict__ grp_off,
                                                                           const int32_t* __restrict__ order,
                                                                           const float* __restrict__ coef) {
  constexpr int FUSE_ROWS = fuse_rows(M);
  constexpr int NW = FUSE_BLOCK / 64;
  extern __shared__ double sm[];  // [NW][P]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double* mine = sm + wave * a.P;
  // Pass ph of the grid covers the units [ph, ph + 1) * span * FUSE_U; for a fixed i the whole grid reads one contiguous
  // span of every row (measured: 2.23 ms at P = 100, d = 124 M, against 2.37 ms with one contiguous tile per block)
  const int64_t span = (int64_t)gridDim.x * FUSE_BLOCK;
  const int64_t gtid = (int64_t)blockIdx.x * FUSE_BLOCK + tid;
  const int npass = (int)((a.nunits + span * FUSE_U - 1) / (span * FUSE_U));
  uint32_t nbar = 0;
  for (int ph = 0; ph < npass; ++ph) {
    const int64_t tl = (int64_t)ph * gridDim.x + blockIdx.x;
    uint32_t off[FUSE_U];  // first column of the unit (the launcher keeps 4 nunits below 2^32); past the end: the last
    bool valid[FUSE_U];    // unit again, with f = 0 (adds exact zeros)
    f32x4 fv[FUSE_U];
    float out[FUSE_U][4 * M];
#pragma unroll
    for (int i = 0; i < FUSE_U; ++i) {
      const int64_t unit = (int64_t)ph * span * FUSE_U + i * span + gtid;
      valid[i] = unit < a.nunits;
      off[i] = (uint32_t)(4 * (valid[i] ? unit : a.nunits - 1));
      fv[i] = *reinterpret_cast<const f32x4*>(a.f + off[i]);
      if (!valid[i]) fv[i] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
      for (int e = 0; e < 4 * M; ++e) out[i][e] = 0.0f;
    }
    for (int g = 0; g < a.q; ++g) {
      const int n0 = grp_off[g], n1 = grp_off[g + 1];
      float cf[M][M];  // the guessed rows' table, held in scalar registers (wave-uniform)
#pragma unroll
      for (int t = 0; t < M; ++t)
#pragma unroll
        for (int l = 0; l < M; ++l)
          cf[t][l] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(coef[(g * M + t) * M + l])));
      const int nbatch = (n1 - n0 + FUSE_ROWS - 1) / FUSE_ROWS;
      const int per_batch = (n1 - n0 + nbatch - 1) / nbatch;  // batches of equal size, at most FUSE_ROWS rows, at least M
      for (int b0 = n0; b0 < n1; b0 += per_batch) {
        const int nb = min(per_batch, n1 - b0);
        double acc[FUSE_ROWS];
        int node[FUSE_ROWS];
#pragma unroll
        for (int r = 0; r < FUSE_ROWS; ++r) {
          acc[r] = 0.0;
          node[r] = __builtin_amdgcn_readfirstlane(order[b0 + min(r, nb - 1)]);  // wave-uniform; a short batch re-reads its last row
        }
#pragma unroll
        for (int i = 0; i < FUSE_U; ++i) {
          f32x4 rv[FUSE_ROWS];
#pragma unroll
          for (int r = 0; r < FUSE_ROWS; ++r)
            rv[r] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.R + (int64_t)node[r] * a.ldr + off[i]));
          const double f0 = fv[i].x, f1 = fv[i].y, f2 = fv[i].z, f3 = fv[i].w;
#pragma unroll
          for (int r = 0; r < FUSE_ROWS; ++r) {  // projection, fp64
            acc[r] = fma(f0, (double)rv[r].x, acc[r]);
            acc[r] = fma(f1, (double)rv[r].y, acc[r]);
            acc[r] = fma(f2, (double)rv[r].z, acc[r]);
            acc[r] = fma(f3, (double)rv[r].w, acc[r]);
          }
          if (b0 == n0) {  // the group's first batch starts with the M guessed rows: their recombination
#pragma unroll
            for (int t = 0; t < M; ++t) {
              const float v[4] = {rv[t].x, rv[t].y, rv[t].z, rv[t].w};
#pragma unroll
              for (int l = 0; l < M; ++l)
#pragma unroll
                for (int c = 0; c < 4; ++c) out[i][c * M + l] = fmaf(cf[t][l], v[c], out[i][c * M + l]);
            }
          }
          __builtin_amdgcn_sched_barrier(0);  // one unit's rows in registers at a time: hoisting the next unit's loads spills
        }
#pragma unroll
        for (int r = 0; r < FUSE_ROWS; ++r) {  // this wavefront's share of rho
          const double v = wave_sum_lane63(acc[r]);
          if (lane == 63 && r < nb) mine[node[r]] = v;
        }
      }
    }
    __syncthreads();
    double* tile = a.partials + tl * a.P;
    for (int n = tid; n < a.P; n += FUSE_BLOCK) {  // the wavefronts in order
      double v = sm[n];
#pragma unroll
      for (int w = 1; w < NW; ++w) v += sm[w * a.P + n];
      tile[n] = v;
    }
    solon_phase_align(a.sync, ++nbar, a.spin_limit);
#pragma unroll
    for (int i = 0; i < FUSE_U; ++i) {
      if (valid[i]) {
        float* dst = a.u + (int64_t)off[i] * M;
#pragma unroll
        for (int e = 0; e < 4 * M; e += 4)
          *reinterpret_cast<f32x4*>(dst + e) = (f32x4){out[i][e], out[i][e + 1], out[i][e + 2], out[i][e + 3]};
      }
    }
    solon_phase_align(a.sync, ++nbar, a.spin_limit);
  }
  solon_phase_exit(a.sync);
}

template <int M>
static int fused_pass(solon_plan* plan, const fuse_args& a0, int grid, hipStream_t st) {
  fuse_args a = a0;
  const size_t lds = sizeof(double) * (FUSE_BLOCK / 64) * plan->P;
  hipLaunchKernelGGL((project_recombine_kernel<M>), dim3((unsigned)grid), dim3(FUSE_BLOCK), lds, st, a, a.grp_off, a.order, a.coef);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

// Size of the persistent grid of the fused pass for this plan and these buffers, or 0 when the pass does not apply
// (m not in {1, 2, 4}, unaligned buffers, idle nodes, input too small to pay for it, partial-sum table or LDS too small).
static int fused_grid(const solon_plan* plan, const float* R, int64_t ldr, const float* f, const float* u, int64_t nunits) {
  const int want = solon_tuning("fuse", -1);
  if (want == 0 || nunits < 1 || nunits >= ((int64_t)1 << 30)) return 0;
  if (plan->m != 1 && plan->m != 2 && plan->m != 4) return 0;
  if (plan->n_active != plan->P) return 0;  // the pass projects the rows group by group: idle nodes would be left out
  if (sizeof(double) * (FUSE_BLOCK / 64) * plan->P > 48 * 1024) return 0;  // one LDS slot per wavefront and node
  if ((uintptr_t)R % 16 != 0 || ldr % 4 != 0 || (uintptr_t)f % 16 != 0 || (uintptr_t)u % 16 != 0) return 0;
  const void* k = plan->m == 1 ? (const void*)project_recombine_kernel<1>
                : plan->m == 2 ? (const void*)project_recombine_kernel<2> : (const void*)project_recombine_kernel<4>;
  int grid = solon_resident_grid(k, FUSE_BLOCK);
  const int cap = solon_tuning("fuse_grid", 0);  // tests: a few blocks that go round many times
  if (cap > 0) grid = std::min(grid, cap);
  if (grid < 1) return 0;
  const int64_t per_pass = (int64_t)grid * FUSE_BLOCK * FUSE_U;
  const int64_t npass = (nunits + per_pass - 1) / per_pass;
  if (want < 0 && npass < 8) return 0;  // measured: on small inputs the two separate passes are faster
  if (npass * grid + 64 > SOLON_PROJ_MAX_TILES) return 0;
  return grid;
}

extern "C" int solon_locate_decode(solon_plan* plan, const float* R, int64_t ldr, const float* f, float* u, int32_t* byz_idx,
                                   int32_t* n_byz, double* rho_out, void* hip_stream) {
  if (!plan || !R || !f || !u) {
    solon_set_error("solon_locate_decode: null argument");
    return SOLON_E_INVAL;
  }
  if (ldr < plan->d_c) {
    solon_set_error("solon_locate_decode: ldr %lld < d_c %lld", (long long)ldr, (long long)plan->d_c);
    return SOLON_E_INVAL;
  }
  if (!plan->ws) {
    solon_set_error("solon_locate_decode: the plan has no device workspace (no GPU at creation)");
    return SOLON_E_HIP;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  const int m = plan->m, P = plan->P;
  const int64_t nunits = (plan->d / m) / 4;  // float4 column units whose chunks all lie below d
  const int grid = fused_grid(plan, R, ldr, f, u, nunits);
  int rc;
  if (grid == 0) {  // the two passes of solon_locate + solon_decode
    rc = solon_launch_project(plan, R, ldr, f, st);
    if (rc != SOLON_OK) return rc;
    rc = solon_launch_solve(plan, SOLVE_LOCATE, st);
    if (rc != SOLON_OK) return rc;
    rc = solon_launch_recombine(plan, R, ldr, u, nullptr, st);
    if (rc != SOLON_OK) return rc;
  } else {
    // 1. the guess: phi on the projection of the leading sample columns
    int ntiles = 0;
    const int64_t sample = std::min<int64_t>(plan->d_c, std::max(4, solon_tuning("fuse_sample", FUSE_SAMPLE)));
    rc = solon_project_partials(plan, R, ldr, f, sample, 0, &ntiles, st);
    if (rc != SOLON_OK) return rc;
    rc = solon_project_reduce(plan, ntiles, st);
    if (rc != SOLON_OK) return rc;
    rc = solon_launch_solve(plan, SOLVE_SPECULATE, st);
    if (rc != SOLON_OK) return rc;
    // 2. one pass over R: exact projections of all rows, recombination of the guessed rows
    fuse_args a;
    a.R = R; a.ldr = ldr; a.f = f; a.nunits = nunits; a.P = P; a.q = plan->q;
    a.grp_off = plan->dev.grp_off; a.order = plan->dev.spec_order; a.coef = plan->dev.spec_coef;
    a.partials = plan->dev.partials; a.u = u; a.sync = plan->dev.grid_sync;
    a.spin_limit = solon_tuning("fuse_spin_limit", 0);
    rc = m == 1 ? fused_pass<1>(plan, a, grid, st) : m == 2 ? fused_pass<2>(plan, a, grid, st) : fused_pass<4>(plan, a, grid, st);
    if (rc != SOLON_OK) return rc;
    const int64_t per_pass = (int64_t)grid * FUSE_BLOCK * FUSE_U;
    int tiles = (int)((nunits + per_pass - 1) / per_pass) * grid;
    const int64_t done = 4 * nunits;  // columns covered by the pass
    if (done < plan->d_c) {           // at most four whole columns and one partial chunk are left
      int tail_tiles = 0;
      rc = solon_project_partials(plan, R + done, ldr, f + done, plan->d_c - done, tiles, &tail_tiles, st);
      if (rc != SOLON_OK) return rc;
      tiles += tail_tiles;
    }
    rc = solon_project_reduce(plan, tiles, st);
    if (rc != SOLON_OK) return rc;
    // 3. phi on the exact projections; raises the redo flag if a guessed row turns out corrupt
    rc = solon_launch_solve(plan, SOLVE_LOCATE_CHECK, st);
    if (rc != SOLON_OK) return rc;
    // 4. the ordinary recombination, which returns at once unless the flag is up; the few trailing columns always
    rc = solon_launch_recombine(plan, R, ldr, u, plan->dev.redo, st);
    if (rc != SOLON_OK) return rc;
    if (done < plan->d_c) {
      rc = solon_launch_recombine_from(plan, R, ldr, u, done, st);
      if (rc != SOLON_OK) return rc;
    }
  }
  if (!byz_idx && !n_byz && !rho_out) return SOLON_OK;
  std::vector<int32_t> vm(P);
  rc = solon_collect_status(plan, st, vm.data(), rho_out);
  if (rc == SOLON_E_HIP) return rc;
  int cnt = 0;
  for (int j = 0; j < P; ++j) {
    if (plan->group_of_node[j] >= 0 && vm[j]) {
      if (byz_idx && cnt < plan->q * plan->s) byz_idx[cnt] = j;
      ++cnt;
    }
  }
  if (n_byz) *n_byz = cnt;
  return rc;
}
