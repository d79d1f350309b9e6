// solon_locate_static: phi for callers that cannot allocate (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc).  The same projection and solve kernels as solon_locate, but every buffer they need
// beyond the caller's inputs and outputs - group tables, per-tile partial projections, psi's tables - lives in one
// file-scope device array instead of a plan's workspace, so the call works on any plan, touches none of its device
// memory and allocates nothing.  Each GPU holds its own copy of the array from the moment the library is loaded until
// the process ends; all calls on one GPU share it, so calls that overlap there race.
#include <mutex>

#include "solon_internal.h"

#define SOLON_STATIC_MAX_P 128        // nodes
#define SOLON_STATIC_MAX_TILES 1024   // per-tile partial projections kept at once
#define SOLON_STATIC_MAX_DEVICES 64

namespace {

constexpr size_t up256(size_t x) { return (x + 255) / 256 * 256; }
// layout of the array (every part 256-byte aligned)
constexpr size_t O_GRP_OFF = 0;                                                                            // int32[P + 1]
constexpr size_t O_GRP_NODES = O_GRP_OFF + up256(sizeof(int32_t) * (SOLON_STATIC_MAX_P + 1));              // int32[P]
constexpr size_t O_W = O_GRP_NODES + up256(sizeof(int32_t) * SOLON_STATIC_MAX_P);                          // float[P]
constexpr size_t O_RHO = O_W + up256(sizeof(float) * SOLON_STATIC_MAX_P);                                  // double[P]
constexpr size_t O_ROWS = O_RHO + up256(sizeof(double) * SOLON_STATIC_MAX_P);                              // int32[q m <= P]
constexpr size_t O_COEF = O_ROWS + up256(sizeof(int32_t) * SOLON_STATIC_MAX_P);                            // float[q m m <= P m]
constexpr size_t O_REDO = O_COEF + up256(sizeof(float) * SOLON_STATIC_MAX_P * SOLON_MAX_M);                // int32
constexpr size_t O_PARTIALS = O_REDO + 256;                                                                // double[tiles][P]
constexpr size_t SCRATCH_BYTES = O_PARTIALS + sizeof(double) * SOLON_STATIC_MAX_TILES * SOLON_STATIC_MAX_P;  // about 1.03 MiB

}  // namespace

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

// In host code `scratch` is only a handle of the symbol; its device address differs from GPU to GPU and is asked for
// once per device.
static int scratch_address(char** out) {
  static std::mutex mu;
  static char* base[SOLON_STATIC_MAX_DEVICES] = {};
  int dev = -1;
  SOLON_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= SOLON_STATIC_MAX_DEVICES) {
    solon_set_error("solon_locate_static: device index %d outside [0, %d)", dev, SOLON_STATIC_MAX_DEVICES);
    return SOLON_E_HIP;
  }
  std::lock_guard<std::mutex> lk(mu);
  if (!base[dev]) {
    void* p = nullptr;
    SOLON_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) {
      solon_set_error("solon_locate_static: the static scratch array has no device address");
      return SOLON_E_HIP;
    }
    base[dev] = (char*)p;
  }
  *out = base[dev];
  return SOLON_OK;
}

int solon_static_prepare(void) {  // called when a plan is created on a device, so that the first real call may be captured
  char* base = nullptr;
  return scratch_address(&base);
}

// The plan's small host tables travel as kernel arguments and are written into the array by one block: no copy from
// host memory is queued, nothing has to be pinned.  Also clears the caller's located[] (idle nodes are never written
// by the solve).
struct static_tables {
  int32_t P, q, n_active;
  uint8_t grp_off[SOLON_STATIC_MAX_P + 4];
  uint8_t grp_nodes[SOLON_STATIC_MAX_P];
  float w[SOLON_STATIC_MAX_P];
};

__global__ __launch_bounds__(SOLON_STATIC_MAX_P + 64) void static_tables_kernel(static_tables t, int32_t* grp_off, int32_t* grp_nodes, float* w,
                                                                                 int32_t* located) {
  const int i = threadIdx.x;
  if (i <= t.q) grp_off[i] = t.grp_off[i];
  if (i < t.n_active) grp_nodes[i] = t.grp_nodes[i];
  if (i < t.P) {
    w[i] = t.w[i];
    located[i] = 0;
  }
}

extern "C" int solon_locate_static(const solon_plan* plan, const float* R, int64_t ldr, const float* f, int32_t* located, int32_t* status,
                                   double* rho, void* hip_stream) {
  if (!plan || !R || !f || !located || !status) {
    solon_set_error("solon_locate_static: null argument");
    return SOLON_E_INVAL;
  }
  if (ldr < plan->d_c) {
    solon_set_error("solon_locate_static: ldr %lld < d_c %lld", (long long)ldr, (long long)plan->d_c);
    return SOLON_E_INVAL;
  }
  if (plan->P > SOLON_STATIC_MAX_P) {
    solon_set_error("solon_locate_static: P = %d exceeds the %d nodes the static scratch array holds", plan->P, SOLON_STATIC_MAX_P);
    return SOLON_E_INVAL;
  }
  char* base = nullptr;
  int rc = scratch_address(&base);
  if (rc != SOLON_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  solon_dev D = {};
  D.grp_off = (int32_t*)(base + O_GRP_OFF);
  D.grp_nodes = (int32_t*)(base + O_GRP_NODES);
  D.w = (float*)(base + O_W);
  D.partials = (double*)(base + O_PARTIALS);
  D.rho = rho ? rho : (double*)(base + O_RHO);
  D.vmask = located;
  D.status = status;
  D.dec_rows = (int32_t*)(base + O_ROWS);
  D.dec_coef = (float*)(base + O_COEF);
  D.redo = (int32_t*)(base + O_REDO);
  static_tables t = {};
  t.P = plan->P; t.q = plan->q; t.n_active = plan->n_active;
  for (int g = 0; g <= plan->q; ++g) t.grp_off[g] = (uint8_t)plan->grp_off[g];      // q <= P <= 128, offsets <= 128
  for (int i = 0; i < plan->n_active; ++i) t.grp_nodes[i] = (uint8_t)plan->grp_nodes[i];
  for (int j = 0; j < plan->P; ++j) t.w[j] = plan->w[j];
  hipLaunchKernelGGL(static_tables_kernel, dim3(1), dim3(SOLON_STATIC_MAX_P + 64), 0, st, t, D.grp_off, D.grp_nodes, D.w, located);
  SOLON_HIP(hipGetLastError());
  int ntiles = 0;
  rc = solon_project_partials_on(plan, D, SOLON_STATIC_MAX_TILES, R, ldr, f, plan->d_c, 0, &ntiles, st);
  if (rc != SOLON_OK) return rc;
  rc = solon_project_reduce_on(plan, D, ntiles, st);
  if (rc != SOLON_OK) return rc;
  return solon_launch_solve_on(plan, D, SOLVE_LOCATE, st);
}
