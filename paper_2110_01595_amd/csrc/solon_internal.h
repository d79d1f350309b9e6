// Internal declarations shared by the translation units of libsolon (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "solon.h"

#define SOLON_MAX_M 16          // largest compression ratio with a compiled kernel
#define SOLON_PROJ_ROWS 32      // most rows of R one projection block accumulates at once
#define SOLON_PROJ_MAX_TILES 8192
#define SOLON_SYNC_WORDS 512     // 8 counters 128 bytes apart, one grid-wide counter, one exit counter

// Device-side tables of a plan; every pointer points into the plan's single workspace allocation.
struct solon_dev {
  int32_t* grp_off;      // [q + 1] offsets into grp_nodes
  int32_t* grp_nodes;    // [n_active] node indices, grouped, ascending inside a group
  int32_t* bat_off;      // [q + 1] offsets into grp_batches
  int32_t* grp_batches;  // [B] gradient indices, grouped
  float* w;              // [P] evaluation point of every node
  double* partials;      // [SOLON_PROJ_MAX_TILES][P] per-block partial projections
  double* rho;           // [P]
  int32_t* vmask;        // [P] 1 = located
  int32_t* status;       // [q] per-group status of the last locate / decode set-up
  int32_t* dec_rows;     // [q * m] rows of R chosen for psi
  float* dec_coef;       // [q][m][m] psi's coefficients T[g][l][t], stored as [g][t][l]
  uint32_t* grid_sync;   // [SOLON_SYNC_WORDS] arrival counters of the phase-separated kernels; zero between launches
};

struct solon_plan {
  int P, B, s, m, r, q, dtype, max_group, n_active;
  int64_t d, d_c;
  std::vector<int32_t> group_of_node, group_of_batch;
  std::vector<int32_t> grp_off, grp_nodes, bat_off, grp_batches;
  std::vector<float> w;
  // device side
  void* ws;            // one hipMalloc block, nullptr when no GPU was available
  size_t ws_bytes;
  solon_dev dev;
  void* pinned;        // hipHostMalloc staging for small host <-> device transfers
  size_t pinned_bytes;
  int proj_tiles;      // tiles used by the last projection launch
};

void solon_set_error(const char* fmt, ...);
int solon_hip_fail(hipError_t e, const char* what);

#define SOLON_HIP(call)                                        \
  do {                                                         \
    hipError_t e__ = (call);                                   \
    if (e__ != hipSuccess) return solon_hip_fail(e__, #call);  \
  } while (0)

int solon_tuning(const char* key, int fallback);
// Number of blocks of `threads` threads of `kernel` that the current device keeps resident at once (0 on error);
// cached per kernel.
int solon_resident_grid(const void* kernel, int threads);

// launchers (defined next to their kernels)
int solon_launch_encode(const solon_plan* plan, const void* G, int64_t ldg, float* Z, int64_t ldz, hipStream_t st);
int solon_launch_project(solon_plan* plan, const float* R, int64_t ldr, const float* f, hipStream_t st);
int solon_launch_solve(solon_plan* plan, bool run_locator, hipStream_t st);
// waits for the stream, copies status (and optionally the located mask and rho) to the host, returns the worst group status
int solon_collect_status(solon_plan* plan, hipStream_t st, int32_t* vmask_host, double* rho_host);
int solon_launch_recombine(const solon_plan* plan, const float* R, int64_t ldr, float* u, hipStream_t st);
