// The projection vector of phi drawn on the device (paper Sec. 3.4: f is generated inside phi, i.i.d. normal with mean
// one).  Counter-based, so that any part of f can be produced anywhere, in any order, from (seed, column) alone:
// Philox-4x32 with ten rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC 2011) turns
// the counter (column / 4, 0, 0, 0) under the key (seed low word, seed high word) into four 32-bit words; each pair of
// words (x, y) gives two normals by the Box-Muller transform with u1 = (x + 1/2) 2^-32, u2 = (y + 1/2) 2^-32.  The
// transform is evaluated in double precision and rounded to float once, so that a host implementation of the same
// recipe reproduces the values (up to the rare double-rounding tie).
#include <math.h>

#include "solon_internal.h"

struct philox4 {
  uint32_t x[4];
};

__device__ __forceinline__ philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return philox4{{c0, c1, c2, c3}};
}

__device__ __forceinline__ void box_muller(uint32_t x, uint32_t y, float& a, float& b) {
  const double u1 = ((double)x + 0.5) * 0x1p-32, u2 = ((double)y + 0.5) * 0x1p-32;
  const double r = sqrt(-2.0 * log(u1));
  double sn, cs;
  sincos(6.283185307179586476925286766559 * u2, &sn, &cs);
  a = (float)(1.0 + r * cs);
  b = (float)(1.0 + r * sn);
}

__global__ __launch_bounds__(256) void draw_projection_kernel(uint32_t k0, uint32_t k1, int64_t d_c, float* __restrict__ f) {
  const int64_t nquads = (d_c + 3) / 4;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nquads; q += stride) {
    const philox4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), 0u, 0u, k0, k1);
    float v[4];
    box_muller(r.x[0], r.x[1], v[0], v[1]);
    box_muller(r.x[2], r.x[3], v[2], v[3]);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (4 * q + e < d_c) f[4 * q + e] = v[e];
  }
}

extern "C" int solon_draw_projection(uint64_t seed, int64_t d_c, float* f, void* hip_stream) {
  if (!f || d_c < 1) {
    solon_set_error("solon_draw_projection: null output or d_c < 1");
    return SOLON_E_INVAL;
  }
  const int64_t nquads = (d_c + 3) / 4;
  const int64_t blocks = std::min<int64_t>((nquads + 255) / 256, 1 << 16);
  hipLaunchKernelGGL(draw_projection_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream, (uint32_t)seed, (uint32_t)(seed >> 32), d_c, f);
  SOLON_HIP(hipGetLastError());
  return SOLON_OK;
}
