// C ABI of the superkernel library: plan upload, the one-launch superkernel and
// the one-launch-per-operator baseline (Sections 4.1, 5.1 and 5.3 of the paper).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "kernels.hip.h"
#include "sk_internal.h"

static_assert(sizeof(sk_tile) == 32, "tile records are 32 bytes");

namespace {

thread_local std::string g_last_error;

sk_status set_error(sk_status st, const std::string &msg) {
  g_last_error = msg;
  return st;
}

sk_status hip_error(const char *what, hipError_t e) {
  return set_error(SK_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// The device side of one tile table: one allocation holding
//   work records (tile + its operator's descriptor) | queue counters | tiles left per operator |
//   completion stamps | split-K offsets | split-K arrival counters | split-K workspace
struct DeviceTables {
  void *blob = nullptr;
  sk::TileWork *work = nullptr;
  uint32_t *counters = nullptr;
  uint32_t *remaining = nullptr;
  uint64_t *stamps = nullptr;
  uint32_t *ws_off = nullptr;   // per output rectangle
  uint32_t *arrive = nullptr;   // per output rectangle
  sk::f32x4 *ws = nullptr;      // split-K partial sums (not initialised: written before it is read)
};

struct sk_plan {
  sk::HostPlan host;
  bool resident = false;
  int device = -1;
  int grid = 0;      // persistent workgroups of sk_launch
  int64_t grid_cap = 0;  // most workgroups any launch of this plan may use
  int only_dtype = -1;   // the element type all operators share, or -1 if they differ
  double ticks_per_ms = 0.0;
  DeviceTables dev;
  // the one-launch-per-operator baseline: every operator tiled as if it were alone;
  // planned and uploaded by the first sk_launch_sequential
  bool seq_ready = false;
  sk::HostPlan seq_host;
  DeviceTables seq_dev;
};

namespace {

// Uploads the tables of `hp` to the current device.
sk_status upload_tables(const sk::HostPlan &hp, DeviceTables &dt) {
  const size_t nt = hp.tiles.size(), np = hp.dev.size(), nrect = hp.ws_off.size();
  const size_t off_work = 0;
  const size_t off_cnt = align_up(off_work + nt * sizeof(sk::TileWork), 256);
  const size_t off_rem = align_up(off_cnt + 2 * sizeof(uint32_t), 256);
  const size_t off_stamps = align_up(off_rem + np * sizeof(uint32_t), 256);
  const size_t off_wsoff = align_up(off_stamps + (np + 1) * sizeof(uint64_t), 256);
  const size_t off_arrive = align_up(off_wsoff + nrect * sizeof(uint32_t), 256);
  const size_t upload = align_up(off_arrive + nrect * sizeof(uint32_t), 256);  // everything before the workspace
  const size_t total = upload + (size_t)hp.ws_f32x4 * 16;
  std::string stage;
  try {
    stage.assign(upload, '\0');
  } catch (const std::bad_alloc &) {
    return set_error(SK_ERR_ALLOC, "host staging allocation failed");
  }
  if (nrect) std::memcpy(&stage[off_wsoff], hp.ws_off.data(), nrect * sizeof(uint32_t));
  for (size_t i = 0; i < nt; ++i) {
    sk::TileWork w;
    std::memset(&w, 0, sizeof(w));
    w.tile = hp.tiles[i];
    w.prob = hp.dev[w.tile.problem];
    std::memcpy(&stage[off_work + i * sizeof(w)], &w, sizeof(w));
  }
  for (size_t i = 0; i < np; ++i) {
    const uint32_t c = (uint32_t)hp.count[i];
    std::memcpy(&stage[off_rem + i * sizeof(uint32_t)], &c, sizeof(c));
  }
  hipError_t e = hipMalloc(&dt.blob, total);
  if (e != hipSuccess) {
    dt.blob = nullptr;
    return set_error(SK_ERR_ALLOC, std::string("hipMalloc: ") + hipGetErrorString(e));
  }
  e = hipMemcpy(dt.blob, stage.data(), upload, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(dt.blob);
    dt.blob = nullptr;
    return hip_error("hipMemcpy", e);
  }
  char *b = (char *)dt.blob;
  dt.work = (sk::TileWork *)(b + off_work);
  dt.counters = (uint32_t *)(b + off_cnt);
  dt.remaining = (uint32_t *)(b + off_rem);
  dt.stamps = (uint64_t *)(b + off_stamps);
  dt.ws_off = (uint32_t *)(b + off_wsoff);
  dt.arrive = (uint32_t *)(b + off_arrive);
  dt.ws = (sk::f32x4 *)(b + upload);
  return SK_OK;
}

}  // namespace

extern "C" {

sk_status sk_plan_create(const sk_problem *problems, int32_t n, const sk_plan_params *params, sk_plan **out) {
  if (!out) return set_error(SK_ERR_INVALID_ARG, "out is null");
  sk_plan *plan = new (std::nothrow) sk_plan();
  if (!plan) return set_error(SK_ERR_ALLOC, "host allocation failed");
  std::string err;
  sk_status st;
  try {
    st = sk::plan_host(problems, n, params, plan->host, err);
  } catch (const std::bad_alloc &) {
    delete plan;
    return set_error(SK_ERR_ALLOC, "host allocation failed while planning");
  }
  if (st != SK_OK) {
    delete plan;
    return set_error(st, err);
  }
  const sk_plan_params &prm = plan->host.params;
  if (!plan->host.problems.empty()) {
    plan->only_dtype = plan->host.problems[0].dtype;
    for (const sk_problem &p : plan->host.problems)
      if (p.dtype != plan->only_dtype) plan->only_dtype = -1;
  }
  if (!prm.host_only) {
    hipError_t e = hipGetDevice(&plan->device);
    if (e != hipSuccess) {
      delete plan;
      return hip_error("hipGetDevice", e);
    }
    int cus = 0, clock_khz = 0;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, plan->device);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, plan->device);
    if (e != hipSuccess) {
      delete plan;
      return hip_error("hipDeviceGetAttribute", e);
    }
    plan->ticks_per_ms = (double)clock_khz;
    const int64_t limit = prm.grid_limit > 0 ? prm.grid_limit : 2 * (int64_t)cus;
    const int64_t ntiles = (int64_t)plan->host.tiles.size();
    plan->grid_cap = limit;
    plan->grid = (int)(ntiles < limit ? ntiles : limit);
    st = upload_tables(plan->host, plan->dev);
    if (st != SK_OK) {
      delete plan;
      return st;
    }
    plan->resident = true;
  }
  *out = plan;
  return SK_OK;
}

sk_status sk_plan_destroy(sk_plan *plan) {
  if (!plan) return SK_OK;
  sk_status st = SK_OK;
  for (DeviceTables *dt : {&plan->dev, &plan->seq_dev}) {
    if (dt->blob) {
      hipError_t e = hipFree(dt->blob);
      if (e != hipSuccess) st = hip_error("hipFree", e);
    }
  }
  delete plan;
  return st;
}

static sk_status launch_range(sk_plan *plan, const DeviceTables &dt, hipStream_t stream, uint32_t begin, uint32_t end,
                              int grid, bool dynamic, bool write_start) {
  if (end <= begin || grid <= 0) return SK_OK;
  sk::KernelArgs a;
  a.counters = dt.counters;
  a.remaining = plan->host.params.stamps ? dt.remaining : nullptr;
  a.stamps = plan->host.params.stamps ? plan->dev.stamps : nullptr;  // one set of stamps, whichever table ran last
  a.n_problems = (uint32_t)plan->host.dev.size();
  a.tile_begin = begin;
  a.tile_end = end;
  a.dynamic = dynamic ? 1u : 0u;
  a.write_start = write_start ? 1u : 0u;
  a.ws = dt.ws;
  a.ws_off = dt.ws_off;
  a.arrive = dt.arrive;
  const dim3 g((unsigned)grid), b(sk::WG_THREADS);
  switch (plan->only_dtype) {
    case SK_F32:
      hipLaunchKernelGGL(sk::sk_superkernel<SK_F32>, g, b, 0, stream, dt.work, a);
      break;
    case SK_BF16:
      hipLaunchKernelGGL(sk::sk_superkernel<SK_BF16>, g, b, 0, stream, dt.work, a);
      break;
    case SK_F16:
      hipLaunchKernelGGL(sk::sk_superkernel<SK_F16>, g, b, 0, stream, dt.work, a);
      break;
    default:
      hipLaunchKernelGGL(sk::sk_superkernel<-1>, g, b, 0, stream, dt.work, a);
      break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_error("kernel launch", e);
  return SK_OK;
}

static sk_status check_launchable(sk_plan *plan) {
  if (!plan) return set_error(SK_ERR_INVALID_ARG, "plan is null");
  if (!plan->resident) return set_error(SK_ERR_STATE, "plan was created host-only; it has no device tables");
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_error("hipGetDevice", e);
  if (dev != plan->device) return set_error(SK_ERR_STATE, "plan belongs to another device than the current one");
  return SK_OK;
}

sk_status sk_launch(sk_plan *plan, void *hip_stream) {
  sk_status st = check_launchable(plan);
  if (st != SK_OK) return st;
  return launch_range(plan, plan->dev, (hipStream_t)hip_stream, 0u, (uint32_t)plan->host.tiles.size(), plan->grid, true,
                      true);
}

sk_status sk_launch_sequential(sk_plan *plan, void *hip_stream) {
  sk_status st = check_launchable(plan);
  if (st != SK_OK) return st;
  if (!plan->seq_ready) {
    std::string err;
    try {
      st = sk::plan_host_each_alone(plan->host, plan->seq_host, err);
    } catch (const std::bad_alloc &) {
      return set_error(SK_ERR_ALLOC, "host allocation failed while planning");
    }
    if (st != SK_OK) return set_error(st, err);
    st = upload_tables(plan->seq_host, plan->seq_dev);
    if (st != SK_OK) return st;
    plan->seq_ready = true;
  }
  const size_t n = plan->seq_host.dev.size();
  for (size_t i = 0; i < n; ++i) {
    const int64_t first = plan->seq_host.first[i], count = plan->seq_host.count[i];
    const int grid = (int)(count < plan->grid_cap ? count : plan->grid_cap);
    st = launch_range(plan, plan->seq_dev, (hipStream_t)hip_stream, (uint32_t)first, (uint32_t)(first + count), grid,
                      false, i == 0);
    if (st != SK_OK) return st;
  }
  return SK_OK;
}

int64_t sk_plan_num_tiles(const sk_plan *plan) { return plan ? (int64_t)plan->host.tiles.size() : -1; }
int32_t sk_plan_num_problems(const sk_plan *plan) { return plan ? (int32_t)plan->host.dev.size() : -1; }
int32_t sk_plan_grid(const sk_plan *plan) { return plan ? plan->grid : -1; }

sk_status sk_plan_get_tiles(const sk_plan *plan, void *dst, int64_t dst_bytes) {
  if (!plan) return set_error(SK_ERR_INVALID_ARG, "plan is null");
  const int64_t need = (int64_t)(plan->host.tiles.size() * sizeof(sk_tile));
  if (need == 0) return SK_OK;
  if (!dst || dst_bytes < need) return set_error(SK_ERR_INVALID_ARG, "destination too small for the tile table");
  std::memcpy(dst, plan->host.tiles.data(), (size_t)need);
  return SK_OK;
}

sk_status sk_plan_get_order(const sk_plan *plan, int32_t *order) {
  if (!plan) return set_error(SK_ERR_INVALID_ARG, "plan is null");
  if (plan->host.order.empty()) return SK_OK;
  if (!order) return set_error(SK_ERR_INVALID_ARG, "order is null");
  std::memcpy(order, plan->host.order.data(), plan->host.order.size() * sizeof(int32_t));
  return SK_OK;
}

sk_status sk_plan_get_ranges(const sk_plan *plan, int64_t *first_tile, int64_t *tile_count) {
  if (!plan) return set_error(SK_ERR_INVALID_ARG, "plan is null");
  const size_t n = plan->host.first.size();
  if (n == 0) return SK_OK;
  if (!first_tile || !tile_count) return set_error(SK_ERR_INVALID_ARG, "output array is null");
  std::memcpy(first_tile, plan->host.first.data(), n * sizeof(int64_t));
  std::memcpy(tile_count, plan->host.count.data(), n * sizeof(int64_t));
  return SK_OK;
}

sk_status sk_plan_get_stamps(sk_plan *plan, uint64_t *done_ticks, uint64_t *start_tick, double *ticks_per_ms) {
  if (!plan) return set_error(SK_ERR_INVALID_ARG, "plan is null");
  if (!plan->resident || !plan->host.params.stamps)
    return set_error(SK_ERR_STATE, "plan was not created with stamps enabled on a device");
  const size_t n = plan->host.dev.size();
  if (done_ticks && n) {
    hipError_t e = hipMemcpy(done_ticks, plan->dev.stamps, n * sizeof(uint64_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_error("hipMemcpy", e);
  }
  if (start_tick) {
    hipError_t e = hipMemcpy(start_tick, plan->dev.stamps + n, sizeof(uint64_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_error("hipMemcpy", e);
  }
  if (ticks_per_ms) *ticks_per_ms = plan->ticks_per_ms;
  return SK_OK;
}

const char *sk_strerror(sk_status status) {
  switch (status) {
    case SK_OK: return "success";
    case SK_ERR_INVALID_ARG: return "invalid argument";
    case SK_ERR_UNSUPPORTED: return "unsupported operator, dtype or size";
    case SK_ERR_OVERLAP: return "output ranges overlap";
    case SK_ERR_ALLOC: return "allocation failed";
    case SK_ERR_HIP: return "HIP runtime error";
    case SK_ERR_STATE: return "plan is not in a state that allows this call";
  }
  return "unknown status";
}

const char *sk_last_error(void) { return g_last_error.c_str(); }

}  // extern "C"
