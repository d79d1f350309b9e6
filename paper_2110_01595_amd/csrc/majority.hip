// Repetition-code decoder for compression ratio m = 1 (the special case in which W_j = I_d, so every honest node
// of a group sends the group's gradient sum itself): per group and coordinate the value sent by the majority of
// the group's nodes, found with the Boyer-Moore streaming majority vote (the paper's appendix on the repetition
// code and its "Streaming Majority Vote" listing), then the sum over groups.  Nodes that differ from the majority
// anywhere are reported as Byzantine.  One pass over R, one pass over u; no projection, no locator system.
#include "grid_phase.h"
#include "solon_internal.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ void clear_flags_kernel(int32_t* vmask, int P, int32_t* status, int q) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < P) vmask[i] = 0;
  if (i < q) status[i] = SOLON_OK;
}

__device__ __forceinline__ void vote(float v, float& cand, int& count) {
  if (count == 0) {
    cand = v;
    count = 1;
  } else if (cand == v) {
    ++count;
  } else {
    --count;
  }
}

// A thread owns VEC consecutive coordinates (VEC = 4 with 16-byte loads when rows are aligned, else 1).
template <int VEC>
__global__ __launch_bounds__(256) void majority_kernel(const float* __restrict__ R, int64_t ldr, int q, const int32_t* __restrict__ grp_off,
                                                        const int32_t* __restrict__ grp_nodes, float* __restrict__ u, int64_t d,
                                                        int32_t* __restrict__ vmask, int32_t* __restrict__ status) {
  const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t c0 = unit * VEC;
  if (c0 >= d) return;
  float total[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) total[e] = 0.0f;
  for (int g = 0; g < q; ++g) {
    const int n0 = grp_off[g], n1 = grp_off[g + 1];
    float cand[VEC];
    int count[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { cand[e] = 0.0f; count[e] = 0; }
    for (int t = n0; t < n1; ++t) {  // first pass: streaming vote
      const float* src = R + (int64_t)grp_nodes[t] * ldr + c0;
      if (VEC == 4) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(src);
        vote(v.x, cand[0], count[0]); vote(v.y, cand[1], count[1]); vote(v.z, cand[2], count[2]); vote(v.w, cand[3], count[3]);
      } else {
        vote(src[0], cand[0], count[0]);
      }
    }
    int agree[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) agree[e] = 0;
    for (int t = n0; t < n1; ++t) {  // second pass (cache hits): confirm the majority, mark the dissenters
      const int j = grp_nodes[t];
      const float* src = R + (int64_t)j * ldr + c0;
      bool same = true;
      if (VEC == 4) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(src);
        const bool s0 = v.x == cand[0], s1 = v.y == cand[1], s2 = v.z == cand[2], s3 = v.w == cand[3];
        agree[0] += s0; agree[1] += s1; agree[2] += s2; agree[3] += s3;
        same = s0 && s1 && s2 && s3;
      } else {
        same = src[0] == cand[0];
        agree[0] += same;
      }
      if (!same) vmask[j] = 1;  // every writer stores the same value
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      if (2 * agree[e] <= n1 - n0) status[g] = SOLON_E_DECODE;  // no value is held by more than half of the group
      total[e] += cand[e];
    }
  }
  if (VEC == 4) {
    f32x4 o = {total[0], total[1], total[2], total[3]};
    __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(u + c0));
  } else {
    u[c0] = total[0];
  }
}

// Same result for groups of at most NMAX nodes and 16-byte aligned rows: the group's values stay in registers
// between the vote and the confirmation pass (all loads are issued up front), and the vote is branch-free.
template <int NMAX>
__global__ __launch_bounds__(256) void majority_reg_kernel(const float* __restrict__ R, int64_t ldr, int q, const int32_t* __restrict__ grp_off,
                                                            const int32_t* __restrict__ grp_nodes, float* __restrict__ u, int64_t d,
                                                            int32_t* __restrict__ vmask, int32_t* __restrict__ status) {
  const int64_t unit = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t c0 = unit * 4;
  if (c0 >= d) return;
  f32x4 total = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 1
  for (int g = 0; g < q; ++g) {
    const int n0 = grp_off[g], n = grp_off[g + 1] - n0;
    f32x4 v[NMAX];
#pragma unroll
    for (int t = 0; t < NMAX; ++t)
      if (t < n) v[t] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(R + (int64_t)grp_nodes[n0 + t] * ldr + c0));
    float cand[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    int count[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < NMAX; ++t) {
      if (t < n) {
        const float x[4] = {v[t].x, v[t].y, v[t].z, v[t].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool fresh = count[e] == 0, same = cand[e] == x[e];
          cand[e] = fresh ? x[e] : cand[e];
          count[e] = fresh ? 1 : (same ? count[e] + 1 : count[e] - 1);
        }
      }
    }
    int agree[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < NMAX; ++t) {
      if (t < n) {
        const bool s0 = v[t].x == cand[0], s1 = v[t].y == cand[1], s2 = v[t].z == cand[2], s3 = v[t].w == cand[3];
        agree[0] += s0; agree[1] += s1; agree[2] += s2; agree[3] += s3;
        if (!(s0 && s1 && s2 && s3)) vmask[grp_nodes[n0 + t]] = 1;  // every writer stores the same value
      }
    }
    if (2 * min(min(agree[0], agree[1]), min(agree[2], agree[3])) <= n) status[g] = SOLON_E_DECODE;
    total += (f32x4){cand[0], cand[1], cand[2], cand[3]};
  }
  __builtin_nontemporal_store(total, reinterpret_cast<f32x4*>(u + c0));
}


// Row-synchronous version for long rows and groups of at most NMAX nodes (16-byte aligned rows).  A persistent grid;
// each round a thread takes one float4 column unit through all groups, loading a group's rows one at a time (a single
// load in flight per wave, so that the whole chip reads one span of one row together, the access order HBM serves
// fastest) into registers, then votes and confirms as above; u is stored 16 bytes per lane without gaps, and the block
// waits for the whole chip (bounded) before the next round.  Rows are read through buffer descriptors (wave-uniform
// base, 32-bit lane offset, hardware range check: past the end of the rows every load returns zeros, which agree).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int NMAX>
__global__ __launch_bounds__(1024, 8) void majority_rows_kernel(const float* __restrict__ R, int64_t ldr, int q, int P,
                                                                 const int32_t* __restrict__ grp_off, const int32_t* __restrict__ grp_nodes,
                                                                 float* __restrict__ u, int64_t nunits, int32_t* __restrict__ vmask,
                                                                 int32_t* __restrict__ status, uint32_t* sync, int spin_limit) {
  extern __shared__ int s_tab[];  // P node indices, then q + 1 group offsets
  int* s_nodes = s_tab;
  int* s_off = s_tab + P;
  const int tid = threadIdx.x;
  for (int n = tid; n < grp_off[q]; n += 1024) s_nodes[n] = grp_nodes[n];
  for (int n = tid; n <= q; n += 1024) s_off[n] = grp_off[n];
  __syncthreads();
  const uint32_t span = gridDim.x * 1024u;  // the launcher keeps span * 16 below 2^32
  const uint32_t gtid = blockIdx.x * 1024u + tid;
  const int nround = (int)((nunits + span - 1) / span);
  uint32_t nbar = 0;
  for (int ph = 0; ph < nround; ++ph) {
    const int64_t ubase = (int64_t)ph * span;
    const int64_t left = nunits - ubase;
    const uint32_t have = left < (int64_t)span ? (uint32_t)left : span;  // units of the round inside the rows, at least one
    float* rph = const_cast<float*>(R) + ubase * 4;
    f32x4 total = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int g = 0; g < q; ++g) {
      const int n0 = __builtin_amdgcn_readfirstlane(s_off[g]), n = __builtin_amdgcn_readfirstlane(s_off[g + 1]) - n0;
      f32x4 v[NMAX];
#pragma unroll
      for (int t = 0; t < NMAX; ++t) {
        if (t < n) {
          const int node = __builtin_amdgcn_readfirstlane(s_nodes[n0 + t]);
          const __amdgpu_buffer_rsrc_t row = __builtin_amdgcn_make_buffer_rsrc(rph + (int64_t)node * ldr, 0, have * 16u, SOLON_BUFFER_WORD3);
          const u32x4 raw = __builtin_amdgcn_raw_buffer_load_b128(row, gtid * 16u, 0, SOLON_BUFFER_NT);
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          v[t] = (f32x4){__uint_as_float(raw.x), __uint_as_float(raw.y), __uint_as_float(raw.z), __uint_as_float(raw.w)};
        }
      }
      float cand[4] = {0.0f, 0.0f, 0.0f, 0.0f};
      int count[4] = {0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < NMAX; ++t) {
        if (t < n) {
          const float x[4] = {v[t].x, v[t].y, v[t].z, v[t].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const bool fresh = count[e] == 0, same = cand[e] == x[e];
            cand[e] = fresh ? x[e] : cand[e];
            count[e] = fresh ? 1 : (same ? count[e] + 1 : count[e] - 1);
          }
        }
      }
      int agree[4] = {0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < NMAX; ++t) {
        if (t < n) {
          const bool s0 = v[t].x == cand[0], s1 = v[t].y == cand[1], s2 = v[t].z == cand[2], s3 = v[t].w == cand[3];
          agree[0] += s0; agree[1] += s1; agree[2] += s2; agree[3] += s3;
          if (!(s0 && s1 && s2 && s3)) vmask[s_nodes[n0 + t]] = 1;  // every writer stores the same value
        }
      }
      if (2 * min(min(agree[0], agree[1]), min(agree[2], agree[3])) <= n) status[g] = SOLON_E_DECODE;
      total += (f32x4){cand[0], cand[1], cand[2], cand[3]};
    }
    if (gtid < have) __builtin_nontemporal_store(total, reinterpret_cast<f32x4*>(u + (ubase + gtid) * 4));
    solon_phase_align(sync, ++nbar, spin_limit);
  }
  solon_phase_exit(sync);
}

extern "C" int solon_decode_majority(solon_plan* plan, const float* R, int64_t ldr, float* u, int32_t* byz_idx, int32_t* n_byz,
                                     void* hip_stream) {
  if (!plan || !R || !u) {
    solon_set_error("solon_decode_majority: null argument");
    return SOLON_E_INVAL;
  }
  if (plan->m != 1) {
    solon_set_error("solon_decode_majority: the repetition-code decoder needs m = 1 (plan has m = %d)", plan->m);
    return SOLON_E_INVAL;
  }
  if (ldr < plan->d) {
    solon_set_error("solon_decode_majority: ldr %lld < d %lld", (long long)ldr, (long long)plan->d);
    return SOLON_E_INVAL;
  }
  if (!plan->ws) {
    solon_set_error("solon_decode_majority: the plan has no device workspace (no GPU at creation)");
    return SOLON_E_HIP;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  const int nflag = std::max(plan->P, plan->q);
  hipLaunchKernelGGL(clear_flags_kernel, dim3((nflag + 255) / 256), dim3(256), 0, st, plan->dev.vmask, plan->P, plan->dev.status, plan->q);
  SOLON_HIP(hipGetLastError());
  const bool vec = ((uintptr_t)R % 16 == 0) && (ldr % 4 == 0) && ((uintptr_t)u % 16 == 0) && (plan->d % 4 == 0);
  if (vec) {
    const int64_t units = plan->d / 4;
    const dim3 grid((unsigned)((units + 255) / 256));
    // long rows in groups of at most nine nodes: the persistent row-synchronous kernel
    int rows_grid = 0;
    const size_t rlds = sizeof(int) * (plan->P + plan->q + 1);
    const int want_rows = solon_tuning("majority_rows", -1);
    // (nine rows of four values are what fits eight waves per SIMD; a sixteen-row version at four waves per SIMD
    // ran 26 % slower than the flat kernel below)
    if (plan->max_group <= 9 && want_rows != 0 && rlds <= 64 * 1024) {
      rows_grid = solon_resident_grid((const void*)majority_rows_kernel<9>, 1024, rlds);
      const int grid_cap = solon_tuning("majority_rows_grid", 0);  // tests: a few blocks that go round many times
      if (grid_cap > 0) rows_grid = std::min(rows_grid, grid_cap);
      if ((int64_t)rows_grid * 1024 * 16 >= ((int64_t)1 << 32)) rows_grid = 0;
      // measured against the flat kernels below (groups of 3, 7 and 9 nodes, d = 0.3 M ... 50 M): 10 - 25 % faster from three
      // quarters of a round of work on in groups of 7 - 9 (slower by a third below that), within 3 % either way in groups of 3
      if (want_rows < 0 && 4 * units < 3 * (int64_t)rows_grid * 1024) rows_grid = 0;
    }
    if (rows_grid > 0)
      hipLaunchKernelGGL(majority_rows_kernel<9>, dim3((unsigned)rows_grid), dim3(1024), rlds, st, R, ldr, plan->q, plan->P, plan->dev.grp_off,
                         plan->dev.grp_nodes, u, units, plan->dev.vmask, plan->dev.status, plan->dev.grid_sync,
                         solon_tuning("phase_spin_limit", SOLON_SPIN_LIMIT));
    else if (plan->max_group <= 16)  // (an 8-node instance compiled to 234 registers per lane and ran slower than this one)
      hipLaunchKernelGGL(majority_reg_kernel<16>, grid, dim3(256), 0, st, R, ldr, plan->q, plan->dev.grp_off, plan->dev.grp_nodes, u,
                         plan->d, plan->dev.vmask, plan->dev.status);
    else
      hipLaunchKernelGGL(majority_kernel<4>, grid, dim3(256), 0, st, R, ldr, plan->q, plan->dev.grp_off, plan->dev.grp_nodes, u,
                         plan->d, plan->dev.vmask, plan->dev.status);
  } else {
    hipLaunchKernelGGL(majority_kernel<1>, dim3((unsigned)((plan->d + 255) / 256)), dim3(256), 0, st, R, ldr, plan->q, plan->dev.grp_off,
                       plan->dev.grp_nodes, u, plan->d, plan->dev.vmask, plan->dev.status);
  }
  SOLON_HIP(hipGetLastError());
  if (!byz_idx && !n_byz) return SOLON_OK;
  std::vector<int32_t> vm(plan->P);
  const int rc = solon_collect_status(plan, st, vm.data(), nullptr);
  if (rc == SOLON_E_HIP) return rc;
  int cnt = 0;
  for (int j = 0; j < plan->P; ++j) {
    if (plan->group_of_node[j] >= 0 && vm[j]) {
      if (byz_idx) byz_idx[cnt] = j;
      ++cnt;
    }
  }
  if (n_byz) *n_byz = cnt;
  return rc;
}
