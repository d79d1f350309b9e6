// Internal declarations shared by the translation units of libsolon (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "solon.h"

#define SOLON_MAX_M 16          // largest compression ratio with a compiled kernel
#define SOLON_PROJ_ROWS 32      // most rows of R one projection block accumulates at once
#define SOLON_PROJ_MAX_TILES 16384
// raw buffer descriptors (wave-uniform base and length, 32-bit lane offsets, hardware range check): word 3 on gfx9
// (32-bit data format, no swizzle) and the non-temporal bit of a buffer instruction's cache policy
#define SOLON_BUFFER_WORD3 0x00020000
#define SOLON_BUFFER_NT 2
#define SOLON_SYNC_WORDS 512     // 8 counters 128 bytes apart, one grid-wide counter (top bit: adrift), one exit counter

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
  int32_t* spec_rows;    // [q * m] rows guessed for psi by the fused locate + decode pass
  float* spec_coef;      // [q][m][m] their coefficient table
  int32_t* spec_order;   // [n_active] every group's nodes with the guessed rows first (both parts ascending)
  int32_t* redo;         // [1] 1 = the guess was wrong, the recombination has to run again
  double* qtab;          // [n_active][SOLON_MAX_M] orthonormal polynomials over every group's points (the consistency test's basis), or null
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
  int last_one_pass;   // 1 if the last solon_locate_decode ran the one-pass kernel, 0 if it fell back to the two passes
};

void solon_set_error(const char* fmt, ...);
int solon_hip_fail(hipError_t e, const char* what);

#define SOLON_HIP(call)                                        \
  do {                                                         \
    hipError_t e__ = (call);                                   \
    if (e__ != hipSuccess) return solon_hip_fail(e__, #call);  \
  } while (0)

int solon_tuning(const char* key, int fallback);
// Number of blocks of `threads` threads (with `dynamic_lds` bytes of dynamic LDS) of `kernel` that the current device keeps
// resident at once (0 on error, or if the kernel spills to scratch memory);
// cached per kernel.
int solon_resident_grid(const void* kernel, int threads, size_t dynamic_lds = 0);
// interval between store steps of a paced write phase whose steps cover `step_bytes` each chip-wide, in eighths of a
// tick of the device's constant-rate clock (0: pacing off or clock rate unknown); knob "store_pace_gbps"
uint32_t solon_store_pace8(int64_t step_bytes);

// launchers (defined next to their kernels)
int solon_launch_encode(const solon_plan* plan, const void* G, int64_t ldg, float* Z, int64_t ldz, hipStream_t st);
int solon_launch_project(solon_plan* plan, const float* R, int64_t ldr, const float* f, hipStream_t st);
// the two halves of solon_launch_project: per-tile partial projections of columns [0, ncols) of R and f, written to tiles
// tile_base, tile_base + 1, ... of the plan's table (*ntiles receives how many); and the fixed-order sum of the first
// ntiles tiles into rho
// With sample_of > 0 the launch projects a SAMPLE of about ncols columns of rows that are sample_of columns long: tiles of
// 1024 columns at positions hashed from the bits of f (needs sample_of >= 2048; positions are whole tiles inside the row).
int solon_project_partials(solon_plan* plan, const float* R, int64_t ldr, const float* f, int64_t ncols, int tile_base, int* ntiles, hipStream_t st,
                           int64_t sample_of = 0);
int solon_project_reduce(solon_plan* plan, int ntiles, hipStream_t st);
// modes of the per-group solve wavefront: psi's tables for the located set already on the device; phi, then psi's
// tables; phi on a projection of a sample of the columns as a guess for the fused locate + decode pass (never fails,
// writes the guess tables only); phi that also raises the redo flag when its rows differ from the guess
enum { SOLVE_TABLES = 0, SOLVE_LOCATE = 1, SOLVE_SPECULATE = 2, SOLVE_LOCATE_CHECK = 3 };
int solon_launch_solve(solon_plan* plan, int mode, hipStream_t st);
// fills D.qtab from the group tables already on the device (once, when a plan is created)
int solon_launch_basis_table(const solon_plan* plan, const solon_dev& D, hipStream_t st);
// the same three steps on a table of device buffers other than the plan's own workspace (`max_tiles` = rows of D.partials)
int solon_project_partials_on(const solon_plan* plan, const solon_dev& D, int max_tiles, const float* R, int64_t ldr, const float* f,
                              int64_t ncols, int tile_base, int* ntiles, hipStream_t st, int64_t sample_of = 0);
int solon_project_reduce_on(const solon_plan* plan, const solon_dev& D, int ntiles, hipStream_t st);
int solon_launch_solve_on(const solon_plan* plan, const solon_dev& D, int mode, hipStream_t st);
// waits for the stream, copies status (and optionally the located mask and rho) to the host, returns the worst group status
int solon_collect_status(solon_plan* plan, hipStream_t st, int32_t* vmask_host, double* rho_host);
// run_flag: device int32 or null; when it points at 0 the kernels return at once (u already holds the result)
// update != 0: u points at the parameters, which are reduced in place by step * (the recombined aggregate)
int solon_launch_recombine(const solon_plan* plan, const float* R, int64_t ldr, float* u, const int32_t* run_flag, hipStream_t st, float step = 0.0f,
                           int update = 0);
// chunks p_start .. d_c - 1 only (p_start a multiple of four), with the general kernel
int solon_launch_recombine_from(const solon_plan* plan, const float* R, int64_t ldr, float* u, int64_t p_start, hipStream_t st);
// asks for the device address of the library's static scratch array on the current device (kept per device)
int solon_static_prepare(void);
