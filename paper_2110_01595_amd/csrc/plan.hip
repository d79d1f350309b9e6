// Plan creation: allocation matrix A (as group tables), evaluation points, parameter checks of
// Thm. 2 and its corollary, and the plan-owned device workspace.  Host code only.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>

#include "solon_internal.h"

static thread_local char g_err[512] = "";

void solon_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int solon_hip_fail(hipError_t e, const char* what) {
  solon_set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return SOLON_E_HIP;
}

extern "C" const char* solon_last_error(void) { return g_err; }

// ---------------------------------------------------------------- launch-shape knobs
static std::mutex g_tune_mu;
static std::map<std::string, int> g_tune;

extern "C" int solon_tune(const char* key, int value) {
  if (!key) return SOLON_E_INVAL;
  std::lock_guard<std::mutex> lk(g_tune_mu);
  g_tune[key] = value;
  return SOLON_OK;
}

int solon_tuning(const char* key, int fallback) {
  std::lock_guard<std::mutex> lk(g_tune_mu);
  auto it = g_tune.find(key);
  return it == g_tune.end() ? fallback : it->second;
}

// ---------------------------------------------------------------- persistent-grid size
int solon_resident_grid(const void* kernel, int threads, size_t dynamic_lds) {
  static std::mutex mu;
  static std::map<std::pair<const void*, size_t>, int> cache;
  std::lock_guard<std::mutex> lk(mu);
  const auto key = std::make_pair(kernel, dynamic_lds);
  auto it = cache.find(key);
  if (it != cache.end()) return it->second;
  int dev = 0, cus = 0, per_cu = 0;
  hipFuncAttributes attr;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dynamic_lds) != hipSuccess ||
      hipFuncGetAttributes(&attr, kernel) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  // a kernel that spills to scratch memory may get fewer resident waves than the occupancy query promises, and a
  // persistent grid that is not resident all at once only waits out its spin limits: such a build uses the flat kernels
  const int grid = attr.localSizeBytes > 0 ? 0 : cus * per_cu;
  cache[key] = grid;
  return grid;
}

// ---------------------------------------------------------------- store pacing
uint32_t solon_store_pace8(int64_t step_bytes) {
  // the rate at which MI355X absorbs ordered writes.  Measured on the encoder at the 124 M-parameter bf16 shape: 7 %
  // faster at 7.8 TB/s than without pacing, 6 % at 7.4 (the pace then throttles), 4 % at 8.0 and 3 % at 8.2 (the stores
  // are then held back by their own completion rather than the schedule, as without pacing); the default keeps a little
  // distance from that knee
  const int gbps = solon_tuning("store_pace_gbps", 7700);
  if (gbps <= 0 || step_bytes <= 0) return 0;
  static std::mutex mu;
  static std::map<int, int> rate;  // constant-rate clock of each device, kHz
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  {
    std::lock_guard<std::mutex> lk(mu);
    auto it = rate.find(dev);
    if (it == rate.end()) {
      if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) {
        (void)hipGetLastError();
        khz = 0;
      }
      rate[dev] = khz;
    } else {
      khz = it->second;
    }
  }
  if (khz <= 0) return 0;
  const double ticks = (double)step_bytes / ((double)gbps * 1e9) * ((double)khz * 1e3);
  const double p8 = ticks * 8.0 + 0.5;
  return p8 < 1.0 ? 0u : p8 > 1e6 ? 1000000u : (uint32_t)p8;  // steps shorter than an eighth of a tick or longer than 1 ms: no pacing / capped
}

// ---------------------------------------------------------------- evaluation points
extern "C" int solon_default_points(int r_g, float* out) {
  if (r_g < 1 || !out) {
    solon_set_error("solon_default_points: r_g < 1 or null output");
    return SOLON_E_INVAL;
  }
  const int K = 2 * ((r_g + 1) / 2);
  int n = 0;
  for (int i = 1; i <= K; ++i) {
    if ((r_g & 1) && (i - 1) == K / 2) continue;  // odd group: leave out the first node below zero
    out[n++] = (float)cos((2.0 * i - 1.0) * M_PI / (2.0 * K));
  }
  return SOLON_OK;
}

// ---------------------------------------------------------------- plan
static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

extern "C" int solon_plan_create(solon_plan** out, int P, int B, int s, int m, int64_t d, int grad_dtype,
                                 const int32_t* group_of_node, const int32_t* group_of_batch, const float* w) {
  if (!out) {
    solon_set_error("solon_plan_create: null output pointer");
    return SOLON_E_INVAL;
  }
  *out = nullptr;
  if (P < 1 || B < 1 || s < 0 || m < 1 || d < 1) {
    solon_set_error("solon_plan_create: need P >= 1, B >= 1, s >= 0, m >= 1, d >= 1");
    return SOLON_E_INVAL;
  }
  if (grad_dtype != SOLON_F32 && grad_dtype != SOLON_BF16) {
    solon_set_error("solon_plan_create: unknown gradient dtype %d", grad_dtype);
    return SOLON_E_INVAL;
  }
  if (m > SOLON_MAX_M) {
    solon_set_error("solon_plan_create: m = %d exceeds the largest compiled compression ratio %d", m, SOLON_MAX_M);
    return SOLON_E_INVAL;
  }
  const int r = 2 * s + m;
  if (r >= SOLON_MAX_GROUP) {  // the locator wavefront keeps one system column (plus the right-hand side) per lane
    solon_set_error("solon_plan_create: 2 s + m = %d must stay below %d", r, SOLON_MAX_GROUP);
    return SOLON_E_INVAL;
  }
  if (2 * s > P - m) {  // corollary of Thm. 2
    solon_set_error("solon_plan_create: s = %d exceeds (P - m) / 2 with P = %d, m = %d", s, P, m);
    return SOLON_E_BOUND;
  }
  std::vector<int32_t> gon(P), gob(B);
  if (group_of_node) {
    std::copy(group_of_node, group_of_node + P, gon.begin());
  } else {
    const int q = P / r;  // >= 1 because r <= P
    const int base = P / q, extra = P % q;
    int j = 0;
    for (int g = 0; g < q; ++g)
      for (int i = 0; i < base + (g < extra ? 1 : 0); ++i) gon[j++] = g;
  }
  int q = 0;
  for (int j = 0; j < P; ++j) {
    if (gon[j] < -1) {
      solon_set_error("solon_plan_create: group_of_node[%d] = %d", j, gon[j]);
      return SOLON_E_INVAL;
    }
    q = std::max(q, gon[j] + 1);
  }
  if (q < 1) {
    solon_set_error("solon_plan_create: no node belongs to a group");
    return SOLON_E_INVAL;
  }
  if (group_of_batch) {
    std::copy(group_of_batch, group_of_batch + B, gob.begin());
  } else {
    if (B != P) {
      solon_set_error("solon_plan_create: group_of_batch is required when B != P");
      return SOLON_E_INVAL;
    }
    for (int k = 0; k < B; ++k) {
      if (gon[k] < 0) {
        solon_set_error("solon_plan_create: group_of_batch is required when a node is idle");
        return SOLON_E_INVAL;
      }
      gob[k] = gon[k];
    }
  }
  for (int k = 0; k < B; ++k)
    if (gob[k] < 0 || gob[k] >= q) {
      solon_set_error("solon_plan_create: group_of_batch[%d] = %d outside [0, %d)", k, gob[k], q);
      return SOLON_E_INVAL;
    }

  solon_plan* p = new solon_plan();
  p->P = P; p->B = B; p->s = s; p->m = m; p->r = r; p->q = q; p->dtype = grad_dtype;
  p->d = d; p->d_c = (d + m - 1) / m;
  p->group_of_node = gon; p->group_of_batch = gob;
  p->ws = nullptr; p->ws_bytes = 0; p->pinned = nullptr; p->pinned_bytes = 0; p->last_one_pass = 0;
  p->grp_off.assign(q + 1, 0);
  p->bat_off.assign(q + 1, 0);
  for (int j = 0; j < P; ++j) if (gon[j] >= 0) p->grp_off[gon[j] + 1]++;
  for (int k = 0; k < B; ++k) p->bat_off[gob[k] + 1]++;
  p->max_group = 0;
  for (int g = 0; g < q; ++g) {
    const int n = p->grp_off[g + 1];
    if (n < r) {  // Thm. 2: every gradient must be replicated on at least 2 s + m nodes
      solon_set_error("solon_plan_create: group %d has %d nodes, fewer than 2 s + m = %d", g, n, r);
      delete p;
      return SOLON_E_BOUND;
    }
    if (n > SOLON_MAX_GROUP) {
      solon_set_error("solon_plan_create: group %d has %d nodes, more than %d", g, n, SOLON_MAX_GROUP);
      delete p;
      return SOLON_E_INVAL;
    }
    p->max_group = std::max(p->max_group, n);
    p->grp_off[g + 1] += p->grp_off[g];
    p->bat_off[g + 1] += p->bat_off[g];
  }
  p->n_active = p->grp_off[q];
  p->grp_nodes.resize(p->n_active);
  p->grp_batches.resize(B);
  {
    std::vector<int32_t> cur(p->grp_off.begin(), p->grp_off.end() - 1);
    for (int j = 0; j < P; ++j) if (gon[j] >= 0) p->grp_nodes[cur[gon[j]]++] = j;
    std::vector<int32_t> curb(p->bat_off.begin(), p->bat_off.end() - 1);
    for (int k = 0; k < B; ++k) p->grp_batches[curb[gob[k]]++] = k;
  }
  p->w.assign(P, 1.0f);
  if (w) {
    std::copy(w, w + P, p->w.begin());
  } else {
    std::vector<float> pts(SOLON_MAX_GROUP);
    for (int g = 0; g < q; ++g) {
      const int n = p->grp_off[g + 1] - p->grp_off[g];
      solon_default_points(n, pts.data());
      for (int i = 0; i < n; ++i) p->w[p->grp_nodes[p->grp_off[g] + i]] = pts[i];
    }
  }
  for (int g = 0; g < q; ++g) {  // "distinct nonzero scalars": distinctness is only needed inside a group
    for (int a = p->grp_off[g]; a < p->grp_off[g + 1]; ++a) {
      const float wa = p->w[p->grp_nodes[a]];
      bool bad = !(wa != 0.0f) || !std::isfinite(wa);
      for (int b = p->grp_off[g]; b < a && !bad; ++b) bad = (p->w[p->grp_nodes[b]] == wa);
      if (bad) {
        solon_set_error("solon_plan_create: evaluation point of node %d is zero, non-finite or repeated in its group",
                        p->grp_nodes[a]);
        delete p;
        return SOLON_E_POINTS;
      }
    }
  }

  // ---- device workspace (skipped when no device is present: host queries keep working)
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    *out = p;
    return SOLON_OK;
  }
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t o_grp_off = take(sizeof(int32_t) * (q + 1));
  const size_t o_grp_nodes = take(sizeof(int32_t) * std::max(1, p->n_active));
  const size_t o_bat_off = take(sizeof(int32_t) * (q + 1));
  const size_t o_grp_batches = take(sizeof(int32_t) * B);
  const size_t o_w = take(sizeof(float) * P);
  const size_t o_partials = take(sizeof(double) * (size_t)SOLON_PROJ_MAX_TILES * P);
  const size_t o_rho = take(sizeof(double) * P);
  const size_t o_vmask = take(sizeof(int32_t) * P);
  const size_t o_status = take(sizeof(int32_t) * q);
  const size_t o_rows = take(sizeof(int32_t) * q * m);
  const size_t o_coef = take(sizeof(float) * q * m * m);
  const size_t o_sync = take(sizeof(uint32_t) * SOLON_SYNC_WORDS);
  const size_t o_srows = take(sizeof(int32_t) * q * m);
  const size_t o_scoef = take(sizeof(float) * q * m * m);
  const size_t o_redo = take(sizeof(int32_t));
  const size_t o_sorder = take(sizeof(int32_t) * std::max(1, p->n_active));
  const size_t o_qtab = take(sizeof(double) * SOLON_MAX_M * std::max(1, p->n_active));
  p->ws_bytes = off;
  hipError_t e = hipMalloc(&p->ws, p->ws_bytes);
  if (e != hipSuccess) {
    delete p;
    return solon_hip_fail(e, "hipMalloc(workspace)");
  }
  char* base = (char*)p->ws;
  p->dev.grp_off = (int32_t*)(base + o_grp_off);
  p->dev.grp_nodes = (int32_t*)(base + o_grp_nodes);
  p->dev.bat_off = (int32_t*)(base + o_bat_off);
  p->dev.grp_batches = (int32_t*)(base + o_grp_batches);
  p->dev.w = (float*)(base + o_w);
  p->dev.partials = (double*)(base + o_partials);
  p->dev.rho = (double*)(base + o_rho);
  p->dev.vmask = (int32_t*)(base + o_vmask);
  p->dev.status = (int32_t*)(base + o_status);
  p->dev.dec_rows = (int32_t*)(base + o_rows);
  p->dev.dec_coef = (float*)(base + o_coef);
  p->dev.grid_sync = (uint32_t*)(base + o_sync);
  p->dev.spec_rows = (int32_t*)(base + o_srows);
  p->dev.spec_coef = (float*)(base + o_scoef);
  p->dev.redo = (int32_t*)(base + o_redo);
  p->dev.spec_order = (int32_t*)(base + o_sorder);
  p->dev.qtab = (double*)(base + o_qtab);
  p->pinned_bytes = align_up(sizeof(double) * P + sizeof(int32_t) * (P + q), 256);
  e = hipHostMalloc(&p->pinned, p->pinned_bytes, hipHostMallocDefault);
  if (e != hipSuccess) {
    (void)hipFree(p->ws);
    delete p;
    return solon_hip_fail(e, "hipHostMalloc(staging)");
  }
  bool ok = hipMemset(p->ws, 0, p->ws_bytes) == hipSuccess &&
            hipMemcpy(p->dev.grp_off, p->grp_off.data(), sizeof(int32_t) * (q + 1), hipMemcpyHostToDevice) == hipSuccess &&
            hipMemcpy(p->dev.grp_nodes, p->grp_nodes.data(), sizeof(int32_t) * p->n_active, hipMemcpyHostToDevice) == hipSuccess &&
            hipMemcpy(p->dev.bat_off, p->bat_off.data(), sizeof(int32_t) * (q + 1), hipMemcpyHostToDevice) == hipSuccess &&
            hipMemcpy(p->dev.grp_batches, p->grp_batches.data(), sizeof(int32_t) * B, hipMemcpyHostToDevice) == hipSuccess &&
            hipMemcpy(p->dev.w, p->w.data(), sizeof(float) * P, hipMemcpyHostToDevice) == hipSuccess;
  if (!ok) {
    hipError_t le = hipGetLastError();
    (void)hipFree(p->ws);
    (void)hipHostFree(p->pinned);
    delete p;
    return solon_hip_fail(le, "workspace initialisation");
  }
  if (solon_launch_basis_table(p, p->dev, nullptr) != SOLON_OK || hipDeviceSynchronize() != hipSuccess) {
    hipError_t le = hipGetLastError();
    (void)hipFree(p->ws);
    (void)hipHostFree(p->pinned);
    delete p;
    return solon_hip_fail(le, "basis tables");
  }
  (void)solon_static_prepare();  // set-up of solon_locate_static on this device; a failure is reported by that call itself
  *out = p;
  return SOLON_OK;
}

extern "C" void solon_plan_destroy(solon_plan* plan) {
  if (!plan) return;
  if (plan->ws) (void)hipFree(plan->ws);
  if (plan->pinned) (void)hipHostFree(plan->pinned);
  delete plan;
}

extern "C" int solon_plan_query(const solon_plan* plan, int what, int64_t* value) {
  if (value && what == SOLON_Q_LIMIT_GROUP) {
    *value = SOLON_MAX_GROUP;
    return SOLON_OK;
  }
  if (value && what == SOLON_Q_LIMIT_M) {
    *value = SOLON_MAX_M;
    return SOLON_OK;
  }
  if (!plan || !value) {
    solon_set_error("solon_plan_query: null argument");
    return SOLON_E_INVAL;
  }
  switch (what) {
    case SOLON_Q_LAST_ONE_PASS: *value = plan->last_one_pass; break;
    case SOLON_Q_LAST_REDO: {
      int32_t flag = 0;
      if (plan->ws) {
        SOLON_HIP(hipDeviceSynchronize());
        SOLON_HIP(hipMemcpy(&flag, plan->dev.redo, sizeof(flag), hipMemcpyDeviceToHost));
      }
      *value = flag;
      break;
    }
    case SOLON_Q_GROUPS: *value = plan->q; break;
    case SOLON_Q_REDUNDANCY: *value = plan->r; break;
    case SOLON_Q_MESSAGE_LEN: *value = plan->d_c; break;
    case SOLON_Q_MAX_GROUP: *value = plan->max_group; break;
    case SOLON_Q_WORKSPACE: *value = (int64_t)plan->ws_bytes; break;
    case SOLON_Q_HAS_DEVICE: *value = plan->ws ? 1 : 0; break;
    default:
      solon_set_error("solon_plan_query: unknown item %d", what);
      return SOLON_E_INVAL;
  }
  return SOLON_OK;
}

extern "C" int solon_plan_groups(const solon_plan* plan, int32_t* group_of_node) {
  if (!plan || !group_of_node) {
    solon_set_error("solon_plan_groups: null argument");
    return SOLON_E_INVAL;
  }
  std::copy(plan->group_of_node.begin(), plan->group_of_node.end(), group_of_node);
  return SOLON_OK;
}

extern "C" int solon_plan_points(const solon_plan* plan, float* w) {
  if (!plan || !w) {
    solon_set_error("solon_plan_points: null argument");
    return SOLON_E_INVAL;
  }
  std::copy(plan->w.begin(), plan->w.end(), w);
  return SOLON_OK;
}
