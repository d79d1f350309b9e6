// Encoder of the linear block code (paper Sec. 3.4): for every group the sum of its gradients
// Y_j 1_P is formed once in registers, and each node j of the group writes
// z_j[p] = sum_l w_j^l * ybar[p m + l]  (row p of W_j = I_{d_c} (x) [1, w_j, .., w_j^{m-1}]).
// One pass over G, one pass over Z; HBM-bound, no matrix cores (inner dimension <= group size).
#include "grid_phase.h"
#include "solon_internal.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct enc_args {
  const void* G;
  int64_t ldg;
  float* Z;
  int64_t ldz;
  int64_t d, d_c;
  const int32_t* grp_off;
  const int32_t* grp_nodes;
  const int32_t* bat_off;
  const int32_t* grp_batches;
  const float* w;
};

// The small tables reach every kernel as read-only, non-aliased kernel arguments of their own (a pointer inside the
// argument struct cannot carry that promise): the compiler then fetches them with scalar loads, which do not share a
// counter with the vector loads and stores - a vector load of w_j would make every row's store wait for all stores
// before it.
#define ENC_TABLE_PARAMS                                                                                             \
  const int32_t *__restrict__ grp_off, const int32_t *__restrict__ grp_nodes, const int32_t *__restrict__ bat_off, \
      const int32_t *__restrict__ grp_batches, const float *__restrict__ w
#define ENC_TABLE_ARGS(a) (a).grp_off, (a).grp_nodes, (a).bat_off, (a).grp_batches, (a).w

__device__ __forceinline__ float elem_to_float(float v) { return v; }
__device__ __forceinline__ float elem_to_float(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }  // bf16 widens exactly

template <typename T> struct load_traits;
template <> struct load_traits<float> { static constexpr int LV = 4; };
template <> struct load_traits<uint16_t> { static constexpr int LV = 8; };

// 16-byte load of LV consecutive elements, accumulated into acc[0..LV)
template <bool NT>
__device__ __forceinline__ void load_add(const float* src, float* acc) {
  const f32x4* p = reinterpret_cast<const f32x4*>(src);
  f32x4 v = NT ? __builtin_nontemporal_load(p) : *p;
  acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
}
template <bool NT>
__device__ __forceinline__ void load_add(const uint16_t* src, float* acc) {
  const u32x4* p = reinterpret_cast<const u32x4*>(src);
  u32x4 v = NT ? __builtin_nontemporal_load(p) : *p;
  acc[0] += __uint_as_float(v.x << 16); acc[1] += __uint_as_float(v.x & 0xffff0000u);
  acc[2] += __uint_as_float(v.y << 16); acc[3] += __uint_as_float(v.y & 0xffff0000u);
  acc[4] += __uint_as_float(v.z << 16); acc[5] += __uint_as_float(v.z & 0xffff0000u);
  acc[6] += __uint_as_float(v.w << 16); acc[7] += __uint_as_float(v.w & 0xffff0000u);
}

// the same accumulation from 16 bytes already in registers (the tag selects the element type)
__device__ __forceinline__ void add_raw(const u32x4 v, float* acc, float) {
  acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y); acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
}
__device__ __forceinline__ void add_raw(const u32x4 v, float* acc, uint16_t) {
  acc[0] += __uint_as_float(v.x << 16); acc[1] += __uint_as_float(v.x & 0xffff0000u);
  acc[2] += __uint_as_float(v.y << 16); acc[3] += __uint_as_float(v.y & 0xffff0000u);
  acc[4] += __uint_as_float(v.z << 16); acc[5] += __uint_as_float(v.z & 0xffff0000u);
  acc[6] += __uint_as_float(v.w << 16); acc[7] += __uint_as_float(v.w & 0xffff0000u);
}

template <int NC, bool NT>
__device__ __forceinline__ void store_chunks(float* dst, const float* z) {
  if constexpr (NC % 4 == 0) {
#pragma unroll
    for (int i = 0; i < NC; i += 4) {
      f32x4 v = {z[i], z[i + 1], z[i + 2], z[i + 3]};
      if (NT) __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst + i)); else *reinterpret_cast<f32x4*>(dst + i) = v;
    }
  } else if constexpr (NC % 2 == 0) {
#pragma unroll
    for (int i = 0; i < NC; i += 2) {
      f32x2 v = {z[i], z[i + 1]};
      if (NT) __builtin_nontemporal_store(v, reinterpret_cast<f32x2*>(dst + i)); else *reinterpret_cast<f32x2*>(dst + i) = v;
    }
  } else {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      if (NT) __builtin_nontemporal_store(z[i], dst + i); else dst[i] = z[i];
    }
  }
}

// Fast path.  A thread owns UE consecutive coordinates (UE a multiple of m and of the 16-byte load width),
// i.e. NC = UE / m whole chunks; blockIdx.y is the group.  Requires 16-byte aligned rows of G and rows of Z
// aligned to the NC floats (at most four) a thread stores at once.
template <int M, int UE, typename T, bool NT>
__global__ __launch_bounds__(256) void encode_vec_kernel(enc_args a, int64_t nunits, ENC_TABLE_PARAMS) {
  constexpr int LV = load_traits<T>::LV;
  constexpr int NL = UE / LV;
  constexpr int NC = UE / M;
  const int g = blockIdx.y;
  const int b0 = bat_off[g], b1 = bat_off[g + 1];
  const int n0 = grp_off[g], n1 = grp_off[g + 1];
  const T* G = static_cast<const T*>(a.G);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < nunits; u += stride) {
    float acc[UE];
#pragma unroll
    for (int i = 0; i < UE; ++i) acc[i] = 0.0f;
    const T* base = G + u * UE;
#pragma unroll 4
    for (int k = b0; k < b1; ++k) {  // group sum, in batch order
      const T* src = base + (int64_t)grp_batches[k] * a.ldg;
#pragma unroll
      for (int v = 0; v < NL; ++v) load_add<NT>(src + v * LV, acc + v * LV);
    }
    float* zbase = a.Z + u * NC;
    for (int t = n0; t < n1; ++t) {  // one message element per node of the group and chunk
      const int j = grp_nodes[t];
      const float wj = w[j];
      float z[NC];
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        float h = acc[c * M + M - 1];
#pragma unroll
        for (int l = M - 2; l >= 0; --l) h = fmaf(h, wj, acc[c * M + l]);  // Horner in w_j
        z[c] = h;
      }
      store_chunks<NC, NT>(zbase + (int64_t)j * a.ldz, z);
    }
  }
}

// Phase-separated fast path for large inputs.  A persistent grid (as many blocks as are resident at once) walks
// the groups; for each it alternates a chip-wide read phase - every thread sums U units of all the group's
// gradient rows into registers - and a write phase - the Horner evaluations of all the group's nodes for those
// units - with an alignment point between them, so that HBM sees long runs of reads and long runs of writes
// instead of their mixture.  For a fixed i the grid covers one contiguous span of every row.  Same arithmetic,
// same order of additions as encode_vec_kernel.
// units a thread of the phase-separated kernel keeps in registers: as many as leave eight waves per SIMD resident
// (40 partial sums; with 48 the kernel would need more than 64 registers)
template <typename T> struct phase_units;
template <> struct phase_units<float> { static constexpr int U = 10; };
template <> struct phase_units<uint16_t> { static constexpr int U = 5; };

// block-tiles per block and phase of the tiled phase-separated kernel: as many as keep the sums within `budget`
// registers.  32 gives the faster code; 40 is used where it saves a phase per group.
constexpr int tile_phase_tiles(int sums_per_tile, int budget) { return budget / sums_per_tile > 0 ? budget / sums_per_tile : 1; }

template <int M, typename T>
__global__ __launch_bounds__(1024, 8) void encode_phase_kernel(enc_args a, int64_t nunits, int q, uint32_t* sync, int spin_limit, uint32_t pace8, ENC_TABLE_PARAMS) {
  constexpr int LV = load_traits<T>::LV;
  constexpr int NC = LV / M;
  constexpr int U = phase_units<T>::U;
  // In a phase, thread t of the grid owns units t, t + span, .., t + (U-1) span counted from the phase's first unit.
  // The rows of G are read through buffer descriptors: position i of a row gets one of its own - wave-uniform base
  // (row, phase, i), bytes left in the row from there (at most one span) - and the lane offset is the same 32-bit
  // t * 16 for all of them, so no 64-bit lane addresses are kept, and the hardware range check makes the ragged last
  // phase branch-free: a load past the end of the row returns zeros (never used).
  __shared__ int s_node[SOLON_MAX_GROUP], s_batch[SOLON_MAX_GROUP];
  __shared__ float s_w[SOLON_MAX_GROUP];
  const uint32_t span = gridDim.x * blockDim.x;  // the host checks span * 16 < 2^32
  const uint32_t gtid = blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_phase = (int64_t)span * U;
  const int nphase = (int)((nunits + per_phase - 1) / per_phase);
  constexpr uint32_t ZB = NC * sizeof(float);  // bytes of Z per unit
  uint32_t nbar = 0;
  for (int g = 0; g < q; ++g) {
    const int b0 = bat_off[g], b1 = bat_off[g + 1];
    const int n0 = grp_off[g], n1 = grp_off[g + 1];
    // the group's tables go to LDS once: fetched from memory in the middle of a phase, each would cost a wave a
    // round trip through the busy memory system per row (two in a chain for w_j).  The previous group's last
    // alignment point separates these writes from its reads, the first one below separates them from the reads here.
    if ((int)threadIdx.x < n1 - n0) {
      const int j = grp_nodes[n0 + threadIdx.x];
      s_node[threadIdx.x] = j;
      s_w[threadIdx.x] = w[j];
    }
    const bool staged = b1 - b0 <= SOLON_MAX_GROUP;  // a group may own any number of batches, the table holds this many
    if (staged && (int)threadIdx.x < b1 - b0) s_batch[threadIdx.x] = grp_batches[b0 + threadIdx.x];
    __syncthreads();
    for (int ph = 0; ph < nphase; ++ph) {
      const int64_t ubase = (int64_t)ph * per_phase;  // first unit of the phase
      uint32_t have[U];                               // units of position i that lie inside the row
#pragma unroll
      for (int i = 0; i < U; ++i) {
        const int64_t left = nunits - ubase - (int64_t)i * span;
        have[i] = left <= 0 ? 0u : left < (int64_t)span ? (uint32_t)left : span;
      }
      char* gph = const_cast<char*>(static_cast<const char*>(a.G)) + ubase * 16;
      float acc[U][LV];
#pragma unroll
      for (int i = 0; i < U; ++i)
#pragma unroll
        for (int e = 0; e < LV; ++e) acc[i][e] = 0.0f;
      for (int k = 0; k < b1 - b0; ++k) {  // group sum, in batch order
        const int batch = staged ? __builtin_amdgcn_readfirstlane(s_batch[k]) : grp_batches[b0 + k];
        char* src = gph + (int64_t)batch * a.ldg * (int64_t)sizeof(T);
        // one load in flight per wave: with all U of a row in flight the kernel measured 2 to 7 % slower, the chip then
        // reads from U spans of the row at once instead of moving through them in step
#pragma unroll
        for (int i = 0; i < U; ++i) {
          if (have[i] != 0) {  // wave-uniform: an empty position of the ragged last phase costs no round trip
            const __amdgpu_buffer_rsrc_t piece = __builtin_amdgcn_make_buffer_rsrc(src + (int64_t)i * span * 16, 0, have[i] * 16u, SOLON_BUFFER_WORD3);
            add_raw(__builtin_amdgcn_raw_buffer_load_b128(piece, gtid * 16u, 0, SOLON_BUFFER_NT), acc[i], T());
          }
        }
      }
      solon_phase_align(sync, ++nbar, spin_limit);
      const unsigned long long t0 = pace8 ? wall_clock64() : 0ull;
      uint32_t step = 0;
      char* zph = reinterpret_cast<char*>(a.Z + ubase * NC);
      for (int t = 0; t < n1 - n0; ++t) {
        const int j = __builtin_amdgcn_readfirstlane(s_node[t]);
        const float wj = s_w[t];
        char* zrow = zph + (int64_t)j * a.ldz * (int64_t)sizeof(float);
#pragma unroll
        for (int i = 0; i < U; ++i) {
          // step (t, i) of all waves covers one contiguous window of row j; in the ragged last phase a position none
          // of whose units lies inside the row takes no slot of the schedule
          if (pace8 && have[i]) solon_pace(t0, step++, pace8);
          float z[NC];
#pragma unroll
          for (int c = 0; c < NC; ++c) {
            float h = acc[i][c * M + M - 1];
#pragma unroll
            for (int l = M - 2; l >= 0; --l) h = fmaf(h, wj, acc[i][c * M + l]);  // Horner in w_j
            z[c] = h;
          }
          // plain global stores: the same stores through a buffer descriptor measured 2.7 % slower on the whole kernel
          if (gtid < have[i]) store_chunks<NC, true>(reinterpret_cast<float*>(zrow + (int64_t)i * span * ZB + (size_t)gtid * ZB), z);
          // one store in flight per wave: a wave whose store HBM has not taken yet does not add the next one to the
          // queues, whatever the schedule says (without this wait a pace a few percent too fast costs 5 %)
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
      }
      solon_phase_align(sync, ++nbar, spin_limit);
    }
  }
  solon_phase_exit(sync);
}

// Phase-separated version of the tiled path (compression ratios that do not divide the load width), for large
// inputs.  A persistent grid of 1024-thread blocks; a block-tile is 1024 consecutive chunks (1024 m coordinates) of
// one group.  Read phase: every thread sums its share of UT block-tiles position-wise over the group's rows into
// registers (coalesced 16-byte loads).  Write phase: tile by tile the sums pass through LDS, each thread picks up
// the m coefficients of its own chunk and writes one message element per node.  Same order of additions as
// encode_tile_kernel.
template <int M, typename T, int BUDGET>
__global__ __launch_bounds__(1024, 8) void encode_tile_phase_kernel(enc_args a, int64_t ntiles, int q, uint32_t* sync, int spin_limit, ENC_TABLE_PARAMS) {
  constexpr int LV = load_traits<T>::LV;
  constexpr int NVEC = 1024 * M / LV;           // 16-byte vectors per row and block-tile (1024 m is a multiple of LV)
  constexpr int NI = (NVEC + 1023) / 1024;      // vectors per thread and block-tile
  constexpr int UT = tile_phase_tiles(NI * LV, BUDGET);  // block-tiles per block and phase
  extern __shared__ float ybar[];               // [1024 * M]
  const int tid = threadIdx.x;
  const int64_t per_phase = (int64_t)gridDim.x * UT;
  const int nphase = (int)((ntiles + per_phase - 1) / per_phase);
  uint32_t nbar = 0;
  for (int g = 0; g < q; ++g) {
    const int b0 = bat_off[g], b1 = bat_off[g + 1];
    const int n0 = grp_off[g], n1 = grp_off[g + 1];
    for (int ph = 0; ph < nphase; ++ph) {
      // tile j of this block in this phase: consecutive blocks take consecutive tiles
      const int64_t t0 = (int64_t)ph * per_phase + blockIdx.x;
      float acc[UT][NI][LV];
#pragma unroll
      for (int j = 0; j < UT; ++j)
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
          for (int e = 0; e < LV; ++e) acc[j][i][e] = 0.0f;
      for (int k = b0; k < b1; ++k) {  // group sum, in batch order
        const T* row = static_cast<const T*>(a.G) + (int64_t)grp_batches[k] * a.ldg;
#pragma unroll
        for (int j = 0; j < UT; ++j) {
          const int64_t tile = t0 + (int64_t)j * gridDim.x;
          if (tile < ntiles) {  // block-uniform: a slot past the end of the ragged last phase costs nothing
            const T* src = row + tile * (1024 * M);
#pragma unroll
            for (int i = 0; i < NI; ++i) {
              int v = tid + 1024 * i;
              if (NVEC % 1024 != 0) v = v < NVEC ? v : NVEC - 1;  // the tile's last vector again (unused)
              load_add<true>(src + v * LV, acc[j][i]);
              // one load in flight per wave, so that the chip moves through the row together (measured at m = 10: 6 to
              // 10 % faster than with a tile's loads queued at once; no difference at m = 6 and 8)
              asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
          }
        }
      }
      solon_phase_align(sync, ++nbar, spin_limit);
#pragma unroll
      for (int j = 0; j < UT; ++j) {
        const int64_t tile = t0 + (int64_t)j * gridDim.x;
        if (tile < ntiles) {  // block-uniform
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            const int v = tid + 1024 * i;
            if (NVEC % 1024 == 0 || v < NVEC) {
#pragma unroll
              for (int e = 0; e < LV; e += 4)
                *reinterpret_cast<f32x4*>(&ybar[v * LV + e]) = (f32x4){acc[j][i][e], acc[j][i][e + 1], acc[j][i][e + 2], acc[j][i][e + 3]};
            }
          }
        }
        __syncthreads();
        if (tile < ntiles) {
          float y[M];
#pragma unroll
          for (int l = 0; l < M; ++l) y[l] = ybar[tid * M + l];
          float* zbase = a.Z + tile * 1024 + tid;
          for (int t = n0; t < n1; ++t) {
            const int jn = grp_nodes[t];
            const float wj = w[jn];
            float h = y[M - 1];
#pragma unroll
            for (int l = M - 2; l >= 0; --l) h = fmaf(h, wj, y[l]);  // Horner in w_j
            __builtin_nontemporal_store(h, zbase + (int64_t)jn * a.ldz);
          }
        }
        __syncthreads();
      }
      solon_phase_align(sync, ++nbar, spin_limit);
    }
  }
  solon_phase_exit(sync);
}

// General path: any alignment, any d; a thread owns one chunk p in [p0, p1).
template <int M, typename T>
__global__ __launch_bounds__(256) void encode_chunk_kernel(enc_args a, int64_t p0, int64_t p1, ENC_TABLE_PARAMS) {
  const int g = blockIdx.y;
  const int b0 = bat_off[g], b1 = bat_off[g + 1];
  const int n0 = grp_off[g], n1 = grp_off[g + 1];
  const T* G = static_cast<const T*>(a.G);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = p0 + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < p1; p += stride) {
    float y[M];
#pragma unroll
    for (int l = 0; l < M; ++l) y[l] = 0.0f;
    // coordinates past d count as zero.  The rows' loads are independent of one another: four rows' worth are issued
    // before the first is used (this kernel usually serves a ragged tail of a few hundred chunks, where nothing but the
    // latency of these loads takes time)
    const int nl = (int)((a.d - p * M) < M ? (a.d - p * M) : M);  // coefficients of this chunk that lie inside the row
#pragma unroll 4
    for (int k = b0; k < b1; ++k) {
      const T* src = G + (int64_t)grp_batches[k] * a.ldg + p * M;
      float v[M];
#pragma unroll
      for (int l = 0; l < M; ++l) v[l] = l < nl ? elem_to_float(src[l]) : 0.0f;
#pragma unroll
      for (int l = 0; l < M; ++l) y[l] += v[l];
    }
    for (int t = n0; t < n1; ++t) {
      const int j = grp_nodes[t];
      const float wj = w[j];
      float h = y[M - 1];
#pragma unroll
      for (int l = M - 2; l >= 0; --l) h = fmaf(h, wj, y[l]);
      a.Z[(int64_t)j * a.ldz + p] = h;
    }
  }
}

// Tiled path for compression ratios that do not divide the 16-byte load width.  A block owns 256 consecutive
// chunks of one group (256 m coordinates): the group sum is accumulated position-wise with coalesced 16-byte
// loads (that part does not depend on m), parked in LDS, and then each thread picks up the m coefficients of its
// own chunk and writes one message element per node (coalesced 4-byte stores).  The last tile may be a partial one as
// long as the row ends on a vector boundary: vectors past the row's end count as zero, chunks past d_c are not written.
// RU = rows of the group sum whose loads are in flight together: 2 for a grid that fills the chip; 8 for the launch of a
// few tiles behind the phase-separated kernel, which is a chain of latencies: that variant loads without branches and keeps
// the group's tables in LDS (one partial tile of a group of 20 rows: 13.5 -> 10.9 us; on a full grid the same code is 8 - 12 %
// slower than the plain one).  The additions keep their order either way.
template <int M, typename T, bool NT, int RU = 2>
__global__ __launch_bounds__(256) void encode_tile_kernel(enc_args a, int64_t tile0, ENC_TABLE_PARAMS) {
  constexpr int LV = load_traits<T>::LV;
  constexpr int NVEC = 256 * M / LV;          // 16-byte vectors per row and tile
  constexpr int NI = (NVEC + 255) / 256;      // vectors per thread
  __shared__ float ybar[256 * M];
  __shared__ int s_node[SOLON_MAX_GROUP];
  __shared__ float s_w[SOLON_MAX_GROUP];
  const int g = blockIdx.y, tid = threadIdx.x;
  const int b0 = bat_off[g], b1 = bat_off[g + 1];
  const int n0 = grp_off[g], n1 = grp_off[g + 1];
  // small launches: the group's node list and points go to LDS first (read from memory inside the store loop they are two
  // chained round trips per node, which a few blocks cannot hide)
  const bool staged = RU > 2 && n1 - n0 <= SOLON_MAX_GROUP;
  if (staged && tid < n1 - n0) {
    const int j = grp_nodes[n0 + tid];
    s_node[tid] = j;
    s_w[tid] = w[j];
  }
  const int64_t tile = tile0 + blockIdx.x;
  const T* base = static_cast<const T*>(a.G) + tile * (256 * M);
  float acc[NI][LV];
  bool inside[NI];  // this thread's vectors that lie inside the tile and inside the row
  const int64_t row_vecs = a.d / LV - tile * NVEC;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int v = tid + 256 * i;
    inside[i] = (NVEC % 256 == 0 || v < NVEC) && v < row_vecs;
#pragma unroll
    for (int e = 0; e < LV; ++e) acc[i][e] = 0.0f;
  }
  if constexpr (RU > 2) {
    // small launches: every thread loads in every round - a vector outside the tile or the row is replaced by the tile's first
    // one (always inside the row) and not added - so that no branch stands between the loads of successive rows
    int off[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) off[i] = inside[i] ? (tid + 256 * i) * LV : 0;
#pragma unroll RU
    for (int k = b0; k < b1; ++k) {  // group sum, in batch order
      const T* src = base + (int64_t)grp_batches[k] * a.ldg;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        float v[LV];
#pragma unroll
        for (int e = 0; e < LV; ++e) v[e] = 0.0f;
        load_add<NT>(src + off[i], v);  // 0 + x = x exactly
#pragma unroll
        for (int e = 0; e < LV; ++e) acc[i][e] += inside[i] ? v[e] : 0.0f;
      }
    }
  } else {
#pragma unroll 2
    for (int k = b0; k < b1; ++k) {  // group sum, in batch order
      const T* src = base + (int64_t)grp_batches[k] * a.ldg;
#pragma unroll
      for (int i = 0; i < NI; ++i)
        if (inside[i]) load_add<NT>(src + (tid + 256 * i) * LV, acc[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int v = tid + 256 * i;
    if (NVEC % 256 == 0 || v < NVEC) {
#pragma unroll
      for (int e = 0; e < LV; e += 4)
        *reinterpret_cast<f32x4*>(&ybar[v * LV + e]) = (f32x4){acc[i][e], acc[i][e + 1], acc[i][e + 2], acc[i][e + 3]};
    }
  }
  __syncthreads();
  float y[M];
#pragma unroll
  for (int l = 0; l < M; ++l) y[l] = ybar[tid * M + l];
  float* zbase = a.Z + tile * 256 + tid;
  if (tile * 256 + tid >= a.d_c) return;  // partial last tile
  for (int t = n0; t < n1; ++t) {
    const int j = staged ? s_node[t - n0] : grp_nodes[t];
    const float wj = staged ? s_w[t - n0] : w[j];
    float h = y[M - 1];
#pragma unroll
    for (int l = M - 2; l >= 0; --l) h = fmaf(h, wj, y[l]);  // Horner in w_j
    if (NT) __builtin_nontemporal_store(h, zbase + (int64_t)j * a.ldz); else zbase[(int64_t)j * a.ldz] = h;
  }
}

// The same tiling for rows of G that are not 16-byte aligned (an odd d with unpadded rows, say): the group sum is
// accumulated element by element - position tid + 256 i of the tile, coalesced 4- or 2-byte loads - so it needs no
// alignment beyond the element's own, and any m.  Same order of additions.
template <int M, typename T>
__global__ __launch_bounds__(256) void encode_tile_elem_kernel(enc_args a, ENC_TABLE_PARAMS) {
  __shared__ float ybar[256 * M];
  const int g = blockIdx.y, tid = threadIdx.x;
  const int b0 = bat_off[g], b1 = bat_off[g + 1];
  const int n0 = grp_off[g], n1 = grp_off[g + 1];
  const int64_t tile = blockIdx.x;
  const T* base = static_cast<const T*>(a.G) + tile * (256 * M) + tid;
  float acc[M];
#pragma unroll
  for (int i = 0; i < M; ++i) acc[i] = 0.0f;
#pragma unroll 2
  for (int k = b0; k < b1; ++k) {  // group sum, in batch order
    const T* src = base + (int64_t)grp_batches[k] * a.ldg;
#pragma unroll
    for (int i = 0; i < M; ++i) acc[i] += elem_to_float(__builtin_nontemporal_load(src + 256 * i));
  }
#pragma unroll
  for (int i = 0; i < M; ++i) ybar[tid + 256 * i] = acc[i];
  __syncthreads();
  float y[M];
#pragma unroll
  for (int l = 0; l < M; ++l) y[l] = ybar[tid * M + l];
  float* zbase = a.Z + tile * 256 + tid;
  for (int t = n0; t < n1; ++t) {
    const int j = grp_nodes[t];
    const float wj = w[j];
    float h = y[M - 1];
#pragma unroll
    for (int l = M - 2; l >= 0; --l) h = fmaf(h, wj, y[l]);  // Horner in w_j
    __builtin_nontemporal_store(h, zbase + (int64_t)j * a.ldz);
  }
}

template <int M, typename T>
static int encode_dispatch(const solon_plan* plan, const enc_args& a, bool aligned, hipStream_t st) {
  constexpr int LV = load_traits<T>::LV;
  const int threads = 256;
  const int q = plan->q;
  const int cap = solon_tuning("encode_blocks", 1 << 22);  // blocks per group; below the work size the kernel strides
  const bool nt = solon_tuning("encode_nt", 1) != 0;
  int64_t done_chunks = 0;
  if (aligned && solon_tuning("encode_force_generic", 0) == 0) {
    if constexpr (LV % M == 0) {  // m divides the load width: one 16-byte load per row and thread
      const int64_t nunits = plan->d / LV;
      // phase-separated persistent grid when the rows are long enough to pay for the alignment points
      int phase_grid = 0;
      const int want_phase = solon_tuning("encode_phase", -1);
      if (nunits > 0 && want_phase != 0) {
        phase_grid = solon_resident_grid((const void*)encode_phase_kernel<M, T>, 1024);
        const int grid_cap = solon_tuning("encode_phase_grid", 0);  // tests: a few blocks make many phases of a small input
        if (grid_cap > 0) phase_grid = std::min(phase_grid, grid_cap);
        if (want_phase < 0 && phase_grid > 0) {
          // Measured (P = 15 ... 100, fp32 and bf16, rows of 15 ... 170 MB): what decides is how many row-phases of work a group
          // holds - a thread takes U units of a row per phase, the chip `cap` bytes - not the bytes as such: from about four
          // (fp32: 336 MB per group, bf16: 168 MB) the phase-separated kernel is 3 - 15 % faster than the flat one, below
          // about three it is 5 - 7 % slower; and two phases per group of which the second is 7 % filled lose 5 % (22 % filled: 9 % faster).
          const int64_t cap = (int64_t)phase_grid * 1024 * phase_units<T>::U;       // units of a row per phase
          const int64_t rows = plan->B / plan->q;
          const int64_t nph = (nunits + cap - 1) / cap;
          const bool ragged_pair = nph == 2 && 8 * (nunits - cap) < cap;
          if (nunits * rows < 4 * cap || 7 * nunits < 2 * cap || ragged_pair) phase_grid = 0;
        }
        if ((int64_t)phase_grid * 1024 * 16 >= ((int64_t)1 << 32)) phase_grid = 0;  // the kernel's 32-bit byte offsets inside a span
      }
      if (phase_grid > 0) {
        uint32_t pace8 = solon_store_pace8((int64_t)phase_grid * 1024 * (LV / M) * (int64_t)sizeof(float));
        // a single phase per group that is less than three quarters filled writes faster unpaced (measured at fills of 35 - 57 %:
        // 0.6 - 3.9 % faster without the schedule; full or several phases: 3 - 11 % faster with it)
        const int64_t phase_cap = (int64_t)phase_grid * 1024 * phase_units<T>::U;
        if (4 * nunits < 3 * phase_cap && solon_tuning("store_pace_always", 0) == 0) pace8 = 0;
        hipLaunchKernelGGL((encode_phase_kernel<M, T>), dim3((unsigned)phase_grid), dim3(1024), 0, st, a, nunits, q, plan->dev.grid_sync,
                           solon_tuning("phase_spin_limit", SOLON_SPIN_LIMIT), pace8, ENC_TABLE_ARGS(a));
        SOLON_HIP(hipGetLastError());
        done_chunks = nunits * (LV / M);
      } else if (nunits > 0) {
        int64_t bx = std::min<int64_t>((nunits + threads - 1) / threads, std::max(1, cap));
        dim3 grid((unsigned)bx, (unsigned)q);
        if (nt) hipLaunchKernelGGL((encode_vec_kernel<M, LV, T, true>), grid, dim3(threads), 0, st, a, nunits, ENC_TABLE_ARGS(a));
        else hipLaunchKernelGGL((encode_vec_kernel<M, LV, T, false>), grid, dim3(threads), 0, st, a, nunits, ENC_TABLE_ARGS(a));
        SOLON_HIP(hipGetLastError());
        done_chunks = nunits * (LV / M);
      }
    } else {
      const int64_t ptiles = plan->d / (1024 * M);  // block-tiles of 1024 chunks that lie entirely below d
      const int want_phase = solon_tuning("encode_phase", -1);
      int phase_grid = 0;
      constexpr int SUMS = (1024 * M / LV + 1023) / 1024 * LV;  // partial sums per thread and block-tile
      constexpr int UT32 = tile_phase_tiles(SUMS, 32), UT40 = tile_phase_tiles(SUMS, 40);
      const size_t lds = sizeof(float) * 1024 * M;
      bool wide = false;            // the 40-register version
      int64_t phase_tiles = ptiles;  // block-tiles given to the phase-separated kernel
      if (ptiles > 0 && want_phase != 0) {
        const void* k32 = (const void*)encode_tile_phase_kernel<M, T, 32>;
        const void* k40 = (const void*)encode_tile_phase_kernel<M, T, 40>;
        if (lds <= 64 * 1024 || (hipFuncSetAttribute(k32, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                                 hipFuncSetAttribute(k40, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess))
          phase_grid = std::min(solon_resident_grid(k32, 1024, lds), solon_resident_grid(k40, 1024, lds));
        else
          (void)hipGetLastError();
        const int grid_cap = solon_tuning("encode_phase_grid", 0);
        if (grid_cap > 0) phase_grid = std::min(phase_grid, grid_cap);
        const int resident = phase_grid;
        if (phase_grid > 0) {
          // a last position that only a few blocks would work on (the others idle through it) goes to the flat kernel
          if (ptiles >= phase_grid && (ptiles % phase_grid) * 8 < ptiles) phase_tiles = ptiles - ptiles % phase_grid;
          // a last position that is less than 80 % filled: the same number of positions on a smaller grid, every block busy in
          // each (measured at P = 100: 716 block-tiles (last position 40 % filled) on 358 blocks 6.08 TB/s, on 512 blocks 5.81;
          // 66 - 78 % filled: 2.5 - 3.5 % faster balanced; 84 % filled: the same; 89 % filled is better left alone: 969 tiles on
          // 512 blocks 6.58 TB/s, on 485 blocks 6.38)
          if (grid_cap <= 0 && phase_tiles % phase_grid != 0 && (phase_tiles % phase_grid) * 10 < (int64_t)phase_grid * 8) {
            const int64_t positions = (phase_tiles + phase_grid - 1) / phase_grid;
            phase_grid = (int)((phase_tiles + positions - 1) / positions);
          }
          const int64_t n32 = (phase_tiles + (int64_t)phase_grid * UT32 - 1) / ((int64_t)phase_grid * UT32);
          const int64_t n40 = (phase_tiles + (int64_t)phase_grid * UT40 - 1) / ((int64_t)phase_grid * UT40);
          wide = UT40 > UT32 && n40 < n32;
          // same rule for the length of the rows as above; in addition the last phase of a group must not be a nearly
          // empty one (measured at 1.07 phases per group: 24 % slower than the flat kernel)
          const int64_t per_phase = (int64_t)phase_grid * (wide ? UT40 : UT32);
          if (want_phase < 0) {
            const int64_t rest = phase_tiles % per_phase;
            // Measured (P = 30 ... 100, m = 3, 6, 10, fp32 and bf16, rows of 11 ... 150 MB): the phase-separated kernel is 1 - 15 %
            // faster than the flat one from about 1.5 block-tiles per resident block on and 2 - 25 % slower below, whatever the
            // bytes (512 resident blocks, fp32: m = 10: 969 block-tiles + 10 %, 716 - 2 %, 615 - 10 %; m = 8: 895 and 793 + 4 %; m = 6: 1025
            // + 9 %, 813 + 2 %, 651 - 15 %).
            if (ptiles * 2 < (int64_t)resident * 3) phase_grid = 0;
            else if (phase_tiles > per_phase && phase_tiles < 2 * per_phase && rest != 0 && 2 * rest < per_phase) phase_grid = 0;
          }
        }
      }
      if (phase_grid > 0) {
        if (wide)
          hipLaunchKernelGGL((encode_tile_phase_kernel<M, T, 40>), dim3((unsigned)phase_grid), dim3(1024), lds, st, a, phase_tiles, q,
                             plan->dev.grid_sync, solon_tuning("phase_spin_limit", SOLON_SPIN_LIMIT), ENC_TABLE_ARGS(a));
        else
          hipLaunchKernelGGL((encode_tile_phase_kernel<M, T, 32>), dim3((unsigned)phase_grid), dim3(1024), lds, st, a, phase_tiles, q,
                             plan->dev.grid_sync, solon_tuning("phase_spin_limit", SOLON_SPIN_LIMIT), ENC_TABLE_ARGS(a));
        SOLON_HIP(hipGetLastError());
        done_chunks = phase_tiles * 1024;
      }
      const int64_t tile0 = phase_grid > 0 ? 4 * phase_tiles : 0;  // flat tiles of 256 chunks from here on
      // a row that ends on a vector boundary: its partial last tile goes along (no separate launch for the ragged tail)
      const int64_t ntiles = (plan->d % LV == 0 ? (plan->d + 256 * M - 1) / (256 * M) : plan->d / (256 * M)) - tile0;
      if (ntiles > 0) {
        dim3 grid((unsigned)ntiles, (unsigned)q);
        if (ntiles <= 8 && nt) hipLaunchKernelGGL((encode_tile_kernel<M, T, true, 8>), grid, dim3(threads), 0, st, a, tile0, ENC_TABLE_ARGS(a));
        else if (nt) hipLaunchKernelGGL((encode_tile_kernel<M, T, true>), grid, dim3(threads), 0, st, a, tile0, ENC_TABLE_ARGS(a));
        else hipLaunchKernelGGL((encode_tile_kernel<M, T, false>), grid, dim3(threads), 0, st, a, tile0, ENC_TABLE_ARGS(a));
        SOLON_HIP(hipGetLastError());
        done_chunks = std::min<int64_t>((tile0 + ntiles) * 256, plan->d_c);
      }
    }
  }
  if (!aligned && solon_tuning("encode_force_generic", 0) == 0) {  // rows of G without 16-byte alignment
    const int64_t ntiles = plan->d / (256 * M);
    if (ntiles > 0) {
      hipLaunchKernelGGL((encode_tile_elem_kernel<M, T>), dim3((unsigned)ntiles, (unsigned)q), dim3(threads), 0, st, a, ENC_TABLE_ARGS(a));
      SOLON_HIP(hipGetLastError());
      done_chunks = ntiles * 256;
    }
  }
  if (done_chunks < plan->d_c) {  // ragged tail (or everything, when the generic kernel is forced)
    const int64_t n = plan->d_c - done_chunks;
    int64_t bx = std::min<int64_t>((n + threads - 1) / threads, std::max(1, cap));
    hipLaunchKernelGGL((encode_chunk_kernel<M, T>), dim3((unsigned)bx, (unsigned)q), dim3(threads), 0, st, a, done_chunks,
                       plan->d_c, ENC_TABLE_ARGS(a));
    SOLON_HIP(hipGetLastError());
  }
  return SOLON_OK;
}

template <typename T>
static int encode_by_m(const solon_plan* plan, const enc_args& a, bool aligned, hipStream_t st) {
  switch (plan->m) {
#define SOLON_CASE(MV) case MV: return encode_dispatch<MV, T>(plan, a, aligned, st);
    SOLON_CASE(1) SOLON_CASE(2) SOLON_CASE(3) SOLON_CASE(4) SOLON_CASE(5) SOLON_CASE(6) SOLON_CASE(7) SOLON_CASE(8)
    SOLON_CASE(9) SOLON_CASE(10) SOLON_CASE(11) SOLON_CASE(12) SOLON_CASE(13) SOLON_CASE(14) SOLON_CASE(15) SOLON_CASE(16)
#undef SOLON_CASE
  }
  solon_set_error("solon_encode: no kernel for m = %d", plan->m);
  return SOLON_E_INVAL;
}

int solon_launch_encode(const solon_plan* plan, const void* G, int64_t ldg, float* Z, int64_t ldz, hipStream_t st) {
  enc_args a;
  a.G = G; a.ldg = ldg; a.Z = Z; a.ldz = ldz; a.d = plan->d; a.d_c = plan->d_c;
  a.grp_off = plan->dev.grp_off; a.grp_nodes = plan->dev.grp_nodes;
  a.bat_off = plan->dev.bat_off; a.grp_batches = plan->dev.grp_batches; a.w = plan->dev.w;
  const size_t esz = plan->dtype == SOLON_BF16 ? 2 : 4;
  // 16-byte loads need aligned rows of G; a thread of the fast kernels stores max(1, LV / m) floats per node
  // at once (LV = elements per 16-byte load), so rows of Z need that alignment only
  const int lv = plan->dtype == SOLON_BF16 ? 8 : 4;
  const int zw = (lv % plan->m == 0) ? std::min(4, lv / plan->m) : 1;
  const bool aligned = ((uintptr_t)G % 16 == 0) && ((size_t)ldg * esz % 16 == 0) && ((uintptr_t)Z % (4 * zw) == 0) && (ldz % zw == 0);
  if (plan->dtype == SOLON_BF16) return encode_by_m<uint16_t>(plan, a, aligned, st);
  return encode_by_m<float>(plan, a, aligned, st);
}

extern "C" int solon_encode(const solon_plan* plan, const void* G, int64_t ldg, float* Z, int64_t ldz, void* hip_stream) {
  if (!plan || !G || !Z) {
    solon_set_error("solon_encode: null argument");
    return SOLON_E_INVAL;
  }
  if (ldg < plan->d || ldz < plan->d_c) {
    solon_set_error("solon_encode: row stride smaller than the row length (ldg %lld < d %lld or ldz %lld < d_c %lld)",
                    (long long)ldg, (long long)plan->d, (long long)ldz, (long long)plan->d_c);
    return SOLON_E_INVAL;
  }
  if (!plan->ws) {
    solon_set_error("solon_encode: the plan has no device workspace (no GPU at creation)");
    return SOLON_E_HIP;
  }
  return solon_launch_encode(plan, G, ldg, Z, ldz, (hipStream_t)hip_stream);
}
