// psi for every group and the sum over groups (paper Algorithm 1, Lemma 2, Thm. 3):
//   u[p m + l] = sum_g sum_t T[g][l][t] * R[U_g[t]][p]
// with U_g the m honest nodes chosen for group g and T[g] the inverse of their m x m Vandermonde,
// both left in the plan's workspace by the locator wavefront.  Reads q m rows of R once, writes u once.
// Every kernel can instead apply the step that follows the path in training (paper Sec. 3.1, "Distributed learning":
// w <- w - gamma / |S| * sum of the gradients): with `update` set, `u` points at the parameters and each coordinate is
// read, reduced by step * (its recombined value) and written back, so the aggregate never makes a round trip through HBM.
#include "grid_phase.h"
#include "solon_internal.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int CH> struct chunk_vec;
template <> struct chunk_vec<1> { typedef float type; };
template <> struct chunk_vec<2> { typedef f32x2 type; };
template <> struct chunk_vec<4> { typedef f32x4 type; };

// A thread owns CH consecutive chunks (CH * M output coordinates).  VEC: rows of R and u are aligned so that
// CH-wide loads and 16-byte stores are legal.
template <int M, int CH, bool VEC>
__global__ __launch_bounds__(256) void recombine_kernel(const float* __restrict__ R, int64_t ldr, int q, const int32_t* __restrict__ rows,
                                                         const float* __restrict__ coef, float* __restrict__ u, int64_t d,
                                                         int64_t d_c, int64_t p_begin, const int32_t* __restrict__ run_flag, float step,
                                                         int update) {
  if (run_flag && *run_flag == 0) return;  // a speculative recombination already produced u
  const int64_t nunits = (d_c + CH - 1) / CH;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t unit = p_begin / CH + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; unit < nunits; unit += stride) {
    const int64_t p = unit * CH;
    const bool full = (p + CH <= d_c) && ((p + CH) * M <= d);
    float out[CH * M];
#pragma unroll
    for (int i = 0; i < CH * M; ++i) out[i] = 0.0f;
    for (int g = 0; g < q; ++g) {
#pragma unroll
      for (int t = 0; t < M; ++t) {
        const float* src = R + (int64_t)rows[g * M + t] * ldr + p;
        float v[CH];
        if (VEC && full) {
          typedef typename chunk_vec<CH>::type vt;
          const vt x = __builtin_nontemporal_load(reinterpret_cast<const vt*>(src));
          if constexpr (CH == 1) { v[0] = x; }
          else if constexpr (CH == 2) { v[0] = x.x; v[1] = x.y; }
          else { v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; }
        } else {
#pragma unroll
          for (int c = 0; c < CH; ++c) v[c] = (p + c < d_c) ? src[c] : 0.0f;
        }
#pragma unroll
        for (int l = 0; l < M; ++l) {
          const float cf = coef[(g * M + t) * M + l];
#pragma unroll
          for (int c = 0; c < CH; ++c) out[c * M + l] = fmaf(cf, v[c], out[c * M + l]);
        }
      }
    }
    float* dst = u + p * M;
    if (VEC && full && (CH * M) % 4 == 0) {
#pragma unroll
      for (int i = 0; i < CH * M; i += 4) {
        f32x4 x = {out[i], out[i + 1], out[i + 2], out[i + 3]};
        if (update) x = *reinterpret_cast<const f32x4*>(dst + i) - step * x;
        __builtin_nontemporal_store(x, reinterpret_cast<f32x4*>(dst + i));
      }
    } else {
#pragma unroll
      for (int i = 0; i < CH * M; ++i)
        if (p * M + i < d) dst[i] = update ? dst[i] - step * out[i] : out[i];  // the last chunk may reach past d
    }
  }
}

// Phase-separated fast path for large inputs and m in {1, 2, 4} (see grid_phase.h): a persistent grid alternates
// a chip-wide read phase - every thread recombines U units of 4 / m chunks each from the q m chosen rows, in
// registers - and a write phase that stores the 4 U output coordinates as U coalesced 16-byte stores.  Same
// arithmetic and order of additions as recombine_kernel.
// units per thread that keep eight waves per SIMD resident without spills
constexpr int recombine_phase_units(int m) { return m == 4 ? 8 : m == 2 ? 6 : 8; }

template <int M>
__global__ __launch_bounds__(1024, 8) void recombine_phase_kernel(const float* __restrict__ R, int64_t ldr, int q,
                                                                   const int32_t* __restrict__ rows, const float* __restrict__ coef,
                                                                   float* __restrict__ u, int64_t nunits, uint32_t* sync, int spin_limit,
                                                                   const int32_t* __restrict__ run_flag, float step, int update) {
  if (run_flag && *run_flag == 0) return;  // every block leaves before the first alignment point: the counters stay zero
  constexpr int CH = 4 / M;
  constexpr int U = recombine_phase_units(M);
  typedef typename chunk_vec<CH>::type vt;
  // unit indices fit 32 bits (checked by the launcher), which keeps the U positions of a thread in U registers
  const uint32_t span = gridDim.x * blockDim.x;
  const uint32_t gtid = blockIdx.x * blockDim.x + threadIdx.x;
  const uint32_t per_phase = span * U;
  const uint32_t last = (uint32_t)nunits - 1u;
  const int nphase = (int)((nunits + per_phase - 1) / per_phase);
  uint32_t nbar = 0;
  for (int ph = 0; ph < nphase; ++ph) {
    const uint32_t u0 = (uint32_t)ph * per_phase + gtid;
    float out[U][4];
#pragma unroll
    for (int i = 0; i < U; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) out[i][e] = 0.0f;
    for (int g = 0; g < q; ++g) {
#pragma unroll
      for (int t = 0; t < M; ++t) {
        const float* src = R + (int64_t)rows[g * M + t] * ldr;
        float cf[M];
#pragma unroll
        for (int l = 0; l < M; ++l) cf[l] = coef[(g * M + t) * M + l];
        vt x[U];
#pragma unroll
        for (int i = 0; i < U; ++i) {
          uint32_t unit = u0 + (uint32_t)i * span;
          unit = unit < last ? unit : last;  // past the end: reload the last unit (in bounds, result unused)
          x[i] = __builtin_nontemporal_load(reinterpret_cast<const vt*>(src + (int64_t)unit * CH));
        }
#pragma unroll
        for (int i = 0; i < U; ++i) {
          float v[CH];
          if constexpr (CH == 1) { v[0] = x[i]; }
          else if constexpr (CH == 2) { v[0] = x[i].x; v[1] = x[i].y; }
          else { v[0] = x[i].x; v[1] = x[i].y; v[2] = x[i].z; v[3] = x[i].w; }
#pragma unroll
          for (int l = 0; l < M; ++l)
#pragma unroll
            for (int c = 0; c < CH; ++c) out[i][c * M + l] = fmaf(cf[l], v[c], out[i][c * M + l]);
        }
      }
    }
    solon_phase_align(sync, ++nbar, spin_limit);
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const uint32_t unit = u0 + (uint32_t)i * span;
      if (unit <= last) {
        f32x4 o = {out[i][0], out[i][1], out[i][2], out[i][3]};
        if (update) o = *reinterpret_cast<const f32x4*>(u + (int64_t)unit * 4) - step * o;
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(u + (int64_t)unit * 4));
      }
    }
    solon_phase_align(sync, ++nbar, spin_limit);
  }
  solon_phase_exit(sync);
}

// Tiled path for compression ratios other than 1, 2, 4.  A block owns 256 consecutive chunks: each thread
// recombines its chunk from coalesced 4-byte loads, the 256 m results pass through LDS and leave as coalesced
// 16-byte stores.
template <int M>
__global__ __launch_bounds__(256) void recombine_tile_kernel(const float* __restrict__ R, int64_t ldr, int q,
                                                              const int32_t* __restrict__ rows, const float* __restrict__ coef,
                                                              float* __restrict__ u, int64_t d, int64_t d_c,
                                                              const int32_t* __restrict__ run_flag, float step, int update) {
  if (run_flag && *run_flag == 0) return;
  __shared__ float tile_out[256 * M];
  const int tid = threadIdx.x;
  const int64_t tile = blockIdx.x;
  const int64_t p = tile * 256 + tid;
  const bool have = p < d_c;  // the last tile may be a partial one (d a multiple of four: no 16-byte store straddles the end)
  float out[M];
#pragma unroll
  for (int l = 0; l < M; ++l) out[l] = 0.0f;
  for (int g = 0; g < q; ++g) {
#pragma unroll
    for (int t = 0; t < M; ++t) {
      const float v = have ? __builtin_nontemporal_load(R + (int64_t)rows[g * M + t] * ldr + p) : 0.0f;
#pragma unroll
      for (int l = 0; l < M; ++l) out[l] = fmaf(coef[(g * M + t) * M + l], v, out[l]);
    }
  }
#pragma unroll
  for (int l = 0; l < M; ++l) tile_out[tid * M + l] = out[l];
  __syncthreads();
  float* dst = u + tile * (256 * M);
  for (int v = tid; v < 64 * M; v += 256) {
    if (tile * (256 * M) + 4 * v >= d) break;
    f32x4 x = *reinterpret_cast<const f32x4*>(&tile_out[4 * v]);
    if (update) x = *reinterpret_cast<const f32x4*>(dst + 4 * v) - step * x;
    __builtin_nontemporal_store(x, reinterpret_cast<f32x4*>(dst + 4 * v));
  }
}

template <int M, int CH = ((M % 4 == 0) ? 1 : (M % 2 == 0 ? 2 : 4))>  // CH * M is a multiple of four
static int recombine_dispatch(const solon_plan* plan, const float* R, int64_t ldr, float* u, const int32_t* run_flag, hipStream_t st, float step,
                              int update) {
  // CH-float loads from the rows of R and 16-byte stores of u
  const bool vec = ((uintptr_t)R % (4 * CH) == 0) && (ldr % CH == 0) && ((uintptr_t)u % 16 == 0);
  const int cap = solon_tuning("decode_blocks", 1 << 22);
  int64_t p_begin = 0;
  if constexpr (M != 1 && M != 2 && M != 4) {
    // tiles that lie entirely below d, and the partial last one when d is a multiple of four
    const int64_t ntiles = plan->d % 4 == 0 ? (plan->d + 256 * M - 1) / (256 * M) : plan->d / (256 * M);
    if (ntiles > 0 && (uintptr_t)u % 16 == 0 && solon_tuning("decode_force_generic", 0) == 0) {
      hipLaunchKernelGGL((recombine_tile_kernel<M>), dim3((unsigned)ntiles), dim3(256), 0, st, R, ldr, plan->q, plan->dev.dec_rows,
                         plan->dev.dec_coef, u, plan->d, plan->d_c, run_flag, step, update);
      SOLON_HIP(hipGetLastError());
      p_begin = std::min<int64_t>(ntiles * 256, plan->d_c);
    }
  }
  if constexpr (M == 1 || M == 2 || M == 4) {
    // units of four output coordinates that lie entirely below d; rows of R aligned for (4 / m)-float loads
    constexpr int PCH = 4 / M;
    const int64_t punits = plan->d / 4;
    const bool pvec = ((uintptr_t)R % (4 * PCH) == 0) && (ldr % PCH == 0) && ((uintptr_t)u % 16 == 0);
    const int want_phase = solon_tuning("decode_phase", -1);
    int phase_grid = 0;
    if (pvec && punits > 0 && punits < (int64_t)1 << 30 && want_phase != 0) {
      phase_grid = solon_resident_grid((const void*)recombine_phase_kernel<M>, 1024);
      const int grid_cap = solon_tuning("decode_phase_grid", 0);
      if (grid_cap > 0) phase_grid = std::min(phase_grid, grid_cap);
      // Measured against the flat kernel (P = 15 ... 100, d up to 124 M): m = 4 (24 - 28 rows read) gains 5 - 7 % from three
      // phases of work on and loses up to 15 % below; m = 1 (9 rows) gains 3 - 8 % from one and a half phases on; m = 2
      // (6 - 10 rows, 8-byte loads) loses 6 - 22 % at every size tried, up to six phases, and stays with the flat kernel.
      const int64_t per_phase = (int64_t)phase_grid * 1024 * recombine_phase_units(M);
      const int64_t min_half_phases = M == 1 ? 3 : M == 4 ? 6 : (int64_t)1 << 40;
      if (want_phase < 0 && 2 * punits < min_half_phases * per_phase) phase_grid = 0;
    }
    if (phase_grid > 0) {
      hipLaunchKernelGGL((recombine_phase_kernel<M>), dim3((unsigned)phase_grid), dim3(1024), 0, st, R, ldr, plan->q, plan->dev.dec_rows,
                         plan->dev.dec_coef, u, punits, plan->dev.grid_sync, solon_tuning("phase_spin_limit", SOLON_SPIN_LIMIT), run_flag, step, update);
      SOLON_HIP(hipGetLastError());
      p_begin = punits * PCH;  // a multiple of every CH used below
    }
  }
  if (p_begin >= plan->d_c) return SOLON_OK;
  const int64_t nunits = (plan->d_c - p_begin + CH - 1) / CH;
  int64_t blocks = std::min<int64_t>((nunits + 255) / 256, cap);
  blocks = std::max<int64_t>(blocks, 1);
  if (vec)
    hipLaunchKernelGGL((recombine_kernel<M, CH, true>), dim3((unsigned)blocks), dim3(256), 0, st, R, ldr, plan->q, plan->dev.dec_rows,
                       plan->dev.dec_coef, u, plan->d, plan->d_c, p_begin, run_flag, step, update);
  else
    hipLaunchKernelGGL((recombine_kernel<M, CH, false>), dim3((unsigned)blocks), dim3(256), 0, st, R, ldr, plan->q, plan->dev.dec_rows,
                       plan->dev.dec_coef, u, plan->d, plan->d_c, p_begin, run_flag, step, update);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

template <int M, int CH = ((M % 4 == 0) ? 1 : (M % 2 == 0 ? 2 : 4))>
static int recombine_from(const solon_plan* plan, const float* R, int64_t ldr, float* u, int64_t p_start, hipStream_t st) {
  if (p_start >= plan->d_c) return SOLON_OK;
  const bool vec = ((uintptr_t)R % (4 * CH) == 0) && (ldr % CH == 0) && ((uintptr_t)u % 16 == 0);
  const int64_t nunits = (plan->d_c - p_start + CH - 1) / CH;
  const int64_t blocks = std::max<int64_t>(1, (nunits + 255) / 256);
  if (vec)
    hipLaunchKernelGGL((recombine_kernel<M, CH, true>), dim3((unsigned)blocks), dim3(256), 0, st, R, ldr, plan->q, plan->dev.dec_rows,
                       plan->dev.dec_coef, u, plan->d, plan->d_c, p_start, (const int32_t*)nullptr, 0.0f, 0);
  else
    hipLaunchKernelGGL((recombine_kernel<M, CH, false>), dim3((unsigned)blocks), dim3(256), 0, st, R, ldr, plan->q, plan->dev.dec_rows,
                       plan->dev.dec_coef, u, plan->d, plan->d_c, p_start, (const int32_t*)nullptr, 0.0f, 0);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}

int solon_launch_recombine_from(const solon_plan* plan, const float* R, int64_t ldr, float* u, int64_t p_start, hipStream_t st) {
  switch (plan->m) {
#define SOLON_CASE(MV) case MV: return recombine_from<MV>(plan, R, ldr, u, p_start, st);
    SOLON_CASE(1) SOLON_CASE(2) SOLON_CASE(3) SOLON_CASE(4) SOLON_CASE(5) SOLON_CASE(6) SOLON_CASE(7) SOLON_CASE(8)
    SOLON_CASE(9) SOLON_CASE(10) SOLON_CASE(11) SOLON_CASE(12) SOLON_CASE(13) SOLON_CASE(14) SOLON_CASE(15) SOLON_CASE(16)
#undef SOLON_CASE
  }
  solon_set_error("solon_decode: no kernel for m = %d", plan->m);
  return SOLON_E_INVAL;
}

int solon_launch_recombine(const solon_plan* plan, const float* R, int64_t ldr, float* u, const int32_t* run_flag, hipStream_t st, float step,
                           int update) {
  if (plan->m == 4) {
    // chunks per thread of the flat kernel: two measured best on large inputs (C4 / C5: 0.68 vs 0.70 ms with one, 0.95 ms with
    // four; 616 MB of rows: 118 vs 123 us), one on small ones (205 MB: 34.5 vs 41.8 us; 240 MB: 47 vs 60; 313 MB: 55.5 vs 60.5)
    int ch = solon_tuning("decode_ch", 0);
    if (ch != 1 && ch != 2 && ch != 4) ch = (int64_t)plan->q * plan->m * plan->d_c * 4 >= ((int64_t)450 << 20) ? 2 : 1;
    if (ch == 4) return recombine_dispatch<4, 4>(plan, R, ldr, u, run_flag, st, step, update);
    if (ch == 2) return recombine_dispatch<4, 2>(plan, R, ldr, u, run_flag, st, step, update);
  }
  switch (plan->m) {
#define SOLON_CASE(MV) case MV: return recombine_dispatch<MV>(plan, R, ldr, u, run_flag, st, step, update);
    SOLON_CASE(1) SOLON_CASE(2) SOLON_CASE(3) SOLON_CASE(4) SOLON_CASE(5) SOLON_CASE(6) SOLON_CASE(7) SOLON_CASE(8)
    SOLON_CASE(9) SOLON_CASE(10) SOLON_CASE(11) SOLON_CASE(12) SOLON_CASE(13) SOLON_CASE(14) SOLON_CASE(15) SOLON_CASE(16)
#undef SOLON_CASE
  }
  solon_set_error("solon_decode: no kernel for m = %d", plan->m);
  return SOLON_E_INVAL;
}

// psi's tables for the located set: either the caller names it (host list) or the preceding locate left it on the device
static int prepare_decode(const char* who, solon_plan* plan, const float* R, int64_t ldr, const int32_t* byz_idx, int32_t n_byz, const float* out,
                          hipStream_t st) {
  if (!plan || !R || !out) {
    solon_set_error("%s: null argument", who);
    return SOLON_E_INVAL;
  }
  if (ldr < plan->d_c) {
    solon_set_error("%s: ldr %lld < d_c %lld", who, (long long)ldr, (long long)plan->d_c);
    return SOLON_E_INVAL;
  }
  if (!plan->ws) {
    solon_set_error("%s: the plan has no device workspace (no GPU at creation)", who);
    return SOLON_E_HIP;
  }
  if (!byz_idx && n_byz > 0) {
    solon_set_error("%s: n_byz > 0 with a null index list", who);
    return SOLON_E_INVAL;
  }
  if (!byz_idx && n_byz < 0) return SOLON_OK;  // the preceding solon_locate's result, still on the device
  if (n_byz < 0) {
    solon_set_error("%s: n_byz < 0 requires a null index list", who);
    return SOLON_E_INVAL;
  }
  // the caller names the located set: rebuild psi's tables for it on the device
  SOLON_HIP(hipStreamSynchronize(st));  // the staging buffer may still be in use by an earlier call on this stream
  int32_t* h_vmask = (int32_t*)plan->pinned;
  std::vector<int> per_group(plan->q, 0);
  for (int j = 0; j < plan->P; ++j) h_vmask[j] = 0;
  for (int i = 0; i < n_byz; ++i) {
    const int j = byz_idx[i];
    if (j < 0 || j >= plan->P) {
      solon_set_error("%s: located index %d outside [0, %d)", who, j, plan->P);
      return SOLON_E_INVAL;
    }
    if (!h_vmask[j] && plan->group_of_node[j] >= 0) per_group[plan->group_of_node[j]]++;
    h_vmask[j] = 1;
  }
  for (int g = 0; g < plan->q; ++g) {
    const int n = plan->grp_off[g + 1] - plan->grp_off[g];
    if (n - per_group[g] < plan->m) {
      solon_set_error("%s: group %d keeps fewer than m = %d nodes", who, g, plan->m);
      return SOLON_E_DECODE;
    }
  }
  SOLON_HIP(hipMemcpyAsync(plan->dev.vmask, h_vmask, sizeof(int32_t) * plan->P, hipMemcpyHostToDevice, st));
  return solon_launch_solve(plan, SOLVE_TABLES, st);
}

extern "C" int solon_decode(solon_plan* plan, const float* R, int64_t ldr, const int32_t* byz_idx, int32_t n_byz, float* u,
                            void* hip_stream) {
  hipStream_t st = (hipStream_t)hip_stream;
  const int rc = prepare_decode("solon_decode", plan, R, ldr, byz_idx, n_byz, u, st);
  if (rc != SOLON_OK) return rc;
  return solon_launch_recombine(plan, R, ldr, u, nullptr, st);
}

extern "C" int solon_decode_update(solon_plan* plan, const float* R, int64_t ldr, const int32_t* byz_idx, int32_t n_byz, float* params,
                                   float step, void* hip_stream) {
  hipStream_t st = (hipStream_t)hip_stream;
  const int rc = prepare_decode("solon_decode_update", plan, R, ldr, byz_idx, n_byz, params, st);
  if (rc != SOLON_OK) return rc;
  return solon_launch_recombine(plan, R, ldr, params, nullptr, st, step, 1);
}
