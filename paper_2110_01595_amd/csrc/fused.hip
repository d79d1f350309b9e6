// phi and psi in one pass over R (paper Sec. 3.4 and Algorithm 1; the step after the path, "decode", needs only m
// honest rows per group, all of which the projection rho = f R reads anyway).
//
// solon_locate followed by solon_decode reads R 1 + q m / P times.  Here the rows for psi are GUESSED first, the
// single pass over R then produces both the exact projections of all P rows and the recombination of the guessed
// rows, and the error-locator solve on the exact projections decides - as in solon_locate - which nodes are
// corrupt.  If none of the guessed rows is among them the recombination already is the result; otherwise (a device-side
// flag, no host round trip) the ordinary recombination kernels run after all.  The guess comes from the locator
// itself, run on the projection of a small sample of the columns: a node whose corruption shows in the sample is
// avoided.  The sample is 128 tiles of 1024 columns at positions hashed from the bits of this call's f, which the
// senders of R cannot know: a node that corrupts a fraction x of its columns stays out of the sample only with
// probability (1 - x)^128, whatever columns it chooses.  The located set and the status never depend on the guess.
//
// The pass is a persistent grid; each round a thread takes one float4 column unit through all rows: the fp64 partial
// projection of every row (reduced over each wavefront by lane permutations, over the block through LDS, one partial
// per block, round and row, summed in fixed order afterwards) and the fp32 recombination of the guessed rows, kept in
// registers and stored at the end of the round.  After its stores a block waits for the whole chip (bounded), so that
// all blocks start the next round's rows together.
#include <algorithm>
#include <vector>

#include "grid_phase.h"
#include "solon_internal.h"
#include "wave_ops.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

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
  int stage_off;  // floats from the start of dynamic LDS to the store-staging area
};

// The pass.  Every thread owns one float4 column unit per round and walks all rows of R with a single load in
// flight, eight waves per SIMD resident: the whole chip then moves through a row's span together and on to the next
// row, which is the access order HBM serves fastest (the encoder's read phase runs the same way; an earlier version
// with six to eight rows in flight per lane and half the waves was 9 % slower).  Rows are read through buffer
// descriptors (wave-uniform base, 32-bit lane offset, hardware range check: past the end of the row a load returns
// zeros and f is zero there too).  The three small tables are copied to LDS once.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int M>
__global__ __launch_bounds__(FUSE_BLOCK, 8) void project_recombine_kernel(fuse_args a, const int32_t* __restrict__ grp_off,
                                                                                const int32_t* __restrict__ order,
                                                                                const float* __restrict__ coef) {
  constexpr int NW = FUSE_BLOCK / 64;
  extern __shared__ double sm[];  // [NW][P] sums, then P node indices, q + 1 group offsets, q M M coefficients
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double* mine = sm + wave * a.P;
  int* s_order = reinterpret_cast<int*>(sm + NW * a.P);
  int* s_off = s_order + a.P;
  float* s_coef = reinterpret_cast<float*>(s_off + a.q + 1);
  float* s_stage = reinterpret_cast<float*>(sm) + a.stage_off;  // [NW][256], 16-byte aligned
  for (int n = tid; n < a.P; n += FUSE_BLOCK) s_order[n] = order[n];
  for (int n = tid; n <= a.q; n += FUSE_BLOCK) s_off[n] = grp_off[n];
  for (int n = tid; n < a.q * M * M; n += FUSE_BLOCK) s_coef[n] = coef[n];
  __syncthreads();
  const uint32_t span = gridDim.x * FUSE_BLOCK;  // the launcher keeps span * 16 below 2^32
  const uint32_t gtid = blockIdx.x * FUSE_BLOCK + tid;
  const int npass = (int)((a.nunits + span - 1) / span);
  uint32_t nbar = 0;
  for (int ph = 0; ph < npass; ++ph) {
    const int64_t ubase = (int64_t)ph * span;  // first unit of the round
    const int64_t left = a.nunits - ubase;
    const uint32_t have = left < (int64_t)span ? (uint32_t)left : span;  // units of the round inside the rows, at least one
    const int64_t tl = (int64_t)ph * gridDim.x + blockIdx.x;
    double f0, f1, f2, f3;
    {
      const __amdgpu_buffer_rsrc_t fd = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.f) + ubase * 4, 0, have * 16u, SOLON_BUFFER_WORD3);
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(fd, gtid * 16u, 0, 0);
      f0 = __uint_as_float(v.x); f1 = __uint_as_float(v.y); f2 = __uint_as_float(v.z); f3 = __uint_as_float(v.w);
    }
    float out[4 * M];
#pragma unroll
    for (int e = 0; e < 4 * M; ++e) out[e] = 0.0f;
    float* rph = const_cast<float*>(a.R) + ubase * 4;
    // The rows in the order of the table (group after group, a group's guessed rows first).  The load of the next
    // row is issued as soon as the current row's has arrived and before its arithmetic, so that a wave has one load
    // in flight all the time rather than none while it reduces.
    int node = __builtin_amdgcn_readfirstlane(s_order[0]);
    u32x4 ahead = __builtin_amdgcn_raw_buffer_load_b128(__builtin_amdgcn_make_buffer_rsrc(rph + (int64_t)node * a.ldr, 0, have * 16u, SOLON_BUFFER_WORD3),
                                                        gtid * 16u, 0, SOLON_BUFFER_NT);
    int t = 0;
    for (int g = 0; g < a.q; ++g) {
      const int n0 = __builtin_amdgcn_readfirstlane(s_off[g]), n1 = __builtin_amdgcn_readfirstlane(s_off[g + 1]);
      for (; t < n1; ++t) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        const u32x4 raw = ahead;
        const int cur = node;
        if (t + 1 < a.P) {
          node = __builtin_amdgcn_readfirstlane(s_order[t + 1]);
          ahead = __builtin_amdgcn_raw_buffer_load_b128(__builtin_amdgcn_make_buffer_rsrc(rph + (int64_t)node * a.ldr, 0, have * 16u, SOLON_BUFFER_WORD3),
                                                        gtid * 16u, 0, SOLON_BUFFER_NT);
        }
        __builtin_amdgcn_sched_barrier(0);
        const float v[4] = {__uint_as_float(raw.x), __uint_as_float(raw.y), __uint_as_float(raw.z), __uint_as_float(raw.w)};
        double acc = f0 * (double)v[0];
        acc = fma(f1, (double)v[1], acc);
        acc = fma(f2, (double)v[2], acc);
        acc = fma(f3, (double)v[3], acc);
        if (t - n0 < M) {  // one of the group's guessed rows: its share of the recombination
#pragma unroll
          for (int l = 0; l < M; ++l) {
            const float cf = s_coef[(g * M + (t - n0)) * M + l];
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c * M + l] = fmaf(cf, v[c], out[c * M + l]);
          }
        }
        const double sum = wave_sum_lane63(acc);
        if (lane == 63) mine[cur] = sum;
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
    // u: a wavefront owns 64 units = 256 M consecutive floats, a lane 4 M of them.  Stored straight from the lanes'
    // registers every store instruction would scatter 16-byte pieces 16 M bytes apart (measured: 1.6 TB/s for these
    // 4 % of the traffic, 14 % of the pass); instead the sums go through LDS, 64 / M lanes' worth at a time, and each
    // store instruction writes 1 KB without gaps.
    if constexpr (M == 1) {
      if (gtid < have) __builtin_nontemporal_store((f32x4){out[0], out[1], out[2], out[3]}, reinterpret_cast<f32x4*>(a.u + (ubase + gtid) * 4));
    } else {
      float* stage = s_stage + wave * 256;
      float* wave_u = a.u + (ubase + (gtid - lane)) * (int64_t)(4 * M);
#pragma unroll
      for (int k = 0; k < M; ++k) {
        if (lane / (64 / M) == k) {
#pragma unroll
          for (int e = 0; e < 4 * M; e += 4)
            *reinterpret_cast<f32x4*>(stage + (lane % (64 / M)) * (4 * M) + e) = (f32x4){out[e], out[e + 1], out[e + 2], out[e + 3]};
        }
        __syncthreads();
        const f32x4 v = *reinterpret_cast<const f32x4*>(stage + 4 * lane);
        const uint32_t unit = (gtid - lane) + (uint32_t)(k * 64 + lane) / M;  // the unit these four floats belong to
        if (unit < have) __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(wave_u + k * 256 + 4 * lane));
        __syncthreads();
      }
    }
    solon_phase_align(a.sync, ++nbar, a.spin_limit);  // ends with a block-wide barrier: the slots are free again
  }
  solon_phase_exit(a.sync);
}

// dynamic LDS of the row-synchronous kernel: the tables, rounded up to 16 bytes, then the store-staging area
static size_t rows_lds_tables(const solon_plan* plan) {
  const size_t b = sizeof(double) * (FUSE_BLOCK / 64) * plan->P + sizeof(int) * (plan->P + plan->q + 1) + sizeof(float) * plan->q * plan->m * plan->m;
  return (b + 15) / 16 * 16;
}
static size_t rows_lds(const solon_plan* plan) { return rows_lds_tables(plan) + sizeof(float) * (FUSE_BLOCK / 64) * 256; }

template <int M>
static int fused_pass(solon_plan* plan, const fuse_args& a0, int grid, hipStream_t st) {
  fuse_args a = a0;
  a.stage_off = (int)(rows_lds_tables(plan) / sizeof(float));
  hipLaunchKernelGGL((project_recombine_kernel<M>), dim3((unsigned)grid), dim3(FUSE_BLOCK), rows_lds(plan), st, a, a.grp_off, a.order, a.coef);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

// Size of the persistent grid of the fused pass for this plan and these buffers, or 0 when the pass does not apply
// (m not in {1, 2, 4}, unaligned buffers, idle nodes, input too small to pay for it, partial-sum table or LDS too small).
static int fused_grid(const solon_plan* plan, const float* R, int64_t ldr, const float* f, const float* u, int64_t nunits,
                      int64_t* per_pass_out) {
  const int want = solon_tuning("fuse", -1);
  if (want == 0 || nunits < 1 || nunits >= ((int64_t)1 << 30)) return 0;
  if (plan->m != 1 && plan->m != 2 && plan->m != 4) return 0;
  if (plan->n_active != plan->P) return 0;  // the pass projects the rows group by group: idle nodes would be left out
  if (rows_lds(plan) > 64 * 1024) return 0;  // one LDS slot per wavefront and node, the tables and the staging area
  if ((uintptr_t)R % 16 != 0 || ldr % 4 != 0 || (uintptr_t)f % 16 != 0 || (uintptr_t)u % 16 != 0) return 0;
  const void* k = plan->m == 1 ? (const void*)project_recombine_kernel<1>
                : plan->m == 2 ? (const void*)project_recombine_kernel<2> : (const void*)project_recombine_kernel<4>;
  int grid = solon_resident_grid(k, FUSE_BLOCK, rows_lds(plan));
  const int cap = solon_tuning("fuse_grid", 0);  // tests: a few blocks that go round many times
  if (cap > 0) grid = std::min(grid, cap);
  if (grid < 1) return 0;
  if ((int64_t)grid * FUSE_BLOCK * 16 >= ((int64_t)1 << 32)) return 0;  // 32-bit lane offsets inside a round
  const int64_t per_pass = (int64_t)grid * FUSE_BLOCK;  // units of a round
  const int64_t npass = (nunits + per_pass - 1) / per_pass;
  if (want < 0) {
    // Does one pass pay?  It saves the second read of the q m rows psi uses (a share q m / P of R) and costs the guess (sample
    // projection, sum, solve: about 200 MB worth of streaming time) plus the idle part of a last, partly filled round of the
    // persistent grid.  Fitted on P = 15 ... 100, m = 1, 2 and 4, rows of 1.8 M ... 45 M columns: the choice is the faster one at all 25
    // points measured (the pass is 4 - 18 % faster wherever this is positive, 1 - 14 % slower where it is negative).
    const double share = (double)plan->q * plan->m / plan->P;
    const double fill = (double)nunits / ((double)npass * (double)per_pass);
    const double gain = share - 0.5 * (1.0 / fill - 1.0) - 2.0e8 / ((double)plan->P * (double)plan->d_c * 4.0);
    if (gain < 0.02) return 0;
  }
  if (npass * grid + 64 > SOLON_PROJ_MAX_TILES) return 0;
  // a partly filled last round: the same number of rounds on a smaller grid, every block busy in each (measured: 1.5 - 4.5 % faster
  // with grids of 84 - 95 % of the resident one, e.g. 0.341 -> 0.328 ms at P = 31, m = 2, 25.6 M parameters; slower below 80 %)
  if (cap <= 0) {
    const int64_t even = (nunits + npass * FUSE_BLOCK - 1) / (npass * FUSE_BLOCK);
    if (even * 10 >= (int64_t)grid * 8 && even < grid) grid = (int)even;
  }
  *per_pass_out = (int64_t)grid * FUSE_BLOCK;
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
  int64_t per_pass = 0;
  const int grid = fused_grid(plan, R, ldr, f, u, nunits, &per_pass);
  int rc;
  plan->last_one_pass = grid != 0;
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
    // tiles of the sample sit at positions hashed from this call's f wherever the rows are long enough to choose from
    const bool hashed = plan->d_c >= 4 * sample && plan->d_c >= 8192 && solon_tuning("fuse_sample_leading", 0) == 0;
    rc = solon_project_partials(plan, R, ldr, f, sample, 0, &ntiles, st, hashed ? plan->d_c : 0);
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
    a.spin_limit = solon_tuning("fuse_spin_limit", SOLON_SPIN_LIMIT);
    rc = m == 1 ? fused_pass<1>(plan, a, grid, st) : m == 2 ? fused_pass<2>(plan, a, grid, st) : fused_pass<4>(plan, a, grid, st);
    if (rc != SOLON_OK) return rc;
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
