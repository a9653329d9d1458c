// C ABI of the superkernel library: plan upload, the one-launch superkernel and
// the one-launch-per-operator baseline (Sections 4.1, 5.1 and 5.3 of the paper).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.hip.h"
#include "sk_internal.h"

static_assert(sizeof(sk_tile) == 32, "tile records are 32 bytes");

namespace {

thread_local std::string g_last_error;

sk_status set_error(sk_status st, const std::string &msg) {
  g_last_error = msg;
  return st;
}

}  // namespace

sk_status sk::set_last_error(sk_status st, const std::string &msg) { return set_error(st, msg); }

namespace {

sk_status hip_error(const char *what, hipError_t e) {
  return set_error(SK_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Table memory is recycled.  A runtime that coalesces whatever is ready (Section 5) creates and
// destroys a plan per launch, and a hipMalloc of a size not seen before costs several hundred
// microseconds, more than planning and uploading a small table together.  Freed tables go to a
// bounded per-process list; a new table takes the smallest listed block of its device that
// holds it without wasting more than half.
class TablePool {
 public:
  // Block sizes: four steps per power of two, at least 64 KiB.
  static size_t block_size(size_t need) {
    size_t p = 64 * 1024;
    while (p < need) p <<= 1;
    if (p == 64 * 1024) return p;
    const size_t q = p / 8;  // p/2 < need <= p: steps of p/8 above p/2
    return align_up(need, q);
  }
  hipError_t acquire(int device, size_t need, void **ptr, size_t *cap) {
    {
      std::lock_guard<std::mutex> g(mu_);
      int best = -1;
      for (size_t i = 0; i < free_.size(); ++i)
        if (free_[i].device == device && free_[i].cap >= need && free_[i].cap / 2 <= need &&
            (best < 0 || free_[i].cap < free_[(size_t)best].cap))
          best = (int)i;
      if (best >= 0) {
        *ptr = free_[(size_t)best].ptr;
        *cap = free_[(size_t)best].cap;
        held_ -= *cap;
        free_.erase(free_.begin() + best);
        return hipSuccess;
      }
    }
    *cap = block_size(need);
    return hipMalloc(ptr, *cap);
  }
  // The caller has made sure no kernel still uses the block.
  hipError_t release(int device, void *ptr, size_t cap) {
    std::vector<Entry> drop;
    {
      std::lock_guard<std::mutex> g(mu_);
      if (cap > MAX_HELD) {
        drop.push_back({device, ptr, cap});
      } else {
        free_.push_back({device, ptr, cap});
        held_ += cap;
        while (held_ > MAX_HELD || free_.size() > MAX_BLOCKS) {  // oldest first
          drop.push_back(free_.front());
          held_ -= free_.front().cap;
          free_.erase(free_.begin());
        }
      }
    }
    hipError_t st = hipSuccess;
    for (const Entry &e : drop) {
      hipError_t r = hipFree(e.ptr);
      if (r != hipSuccess) st = r;
    }
    return st;
  }
  hipError_t trim() {
    std::vector<Entry> drop;
    {
      std::lock_guard<std::mutex> g(mu_);
      drop.swap(free_);
      held_ = 0;
    }
    hipError_t st = hipSuccess;
    for (const Entry &e : drop) {
      hipError_t r = hipFree(e.ptr);
      if (r != hipSuccess) st = r;
    }
    return st;
  }

 private:
  struct Entry {
    int device;
    void *ptr;
    size_t cap;
  };
  static constexpr size_t MAX_HELD = (size_t)512 << 20;
  static constexpr size_t MAX_BLOCKS = 32;
  std::mutex mu_;
  std::vector<Entry> free_;
  size_t held_ = 0;
};

// Host staging for the upload of a table: pinned memory, kept per thread and grown on demand
// (a copy from pageable memory goes through a staging buffer of the runtime's first).  Falls back
// to pageable memory when pinned memory cannot be had.
class HostStage {
 public:
  // `bytes` of staging memory (contents undefined), valid until the next call on this thread
  char *acquire(size_t bytes) {
    if (bytes > cap_) {
      if (ptr_) (void)hipHostFree(ptr_);
      ptr_ = nullptr;
      cap_ = 0;
      const size_t want = align_up(bytes + bytes / 2, (size_t)1 << 20);
      void *p = nullptr;
      if (hipHostMalloc(&p, want, hipHostMallocPortable) == hipSuccess) {
        ptr_ = (char *)p;
        cap_ = want;
      } else {
        (void)hipGetLastError();
        try {
          fallback_.assign(bytes, '\0');
        } catch (const std::bad_alloc &) {
          return nullptr;
        }
        return &fallback_[0];
      }
    }
    return ptr_;
  }

 private:
  char *ptr_ = nullptr;  // never freed at thread exit: the runtime may already be gone
  size_t cap_ = 0;
  std::string fallback_;
};
thread_local HostStage t_stage;

TablePool &table_pool() {
  static TablePool *pool = new TablePool();  // never destroyed: the runtime may already be gone at exit
  return *pool;
}

}  // namespace

// Scratch of sk_launch_static: the table block (work records, queue counters, split-K arrival counters and
// workspace) that sk_plan_create otherwise allocates, as a fixed array in the library's code object.  Each
// GPU the library runs on holds its own copy, at its own address, until the process ends.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SK_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` and the compute-unit count, per device; looked up on the first
// sk_launch_static of a device, with that device current.  (In host code the array's name is not a
// device address: everything below uses the looked-up pointer.)
struct StaticScratch {
  static constexpr int MAX_DEVICES = 64;
  std::mutex mu;
  void *ptr[MAX_DEVICES] = {};
  int cus[MAX_DEVICES] = {};
  sk_status get(int device, void **out, int *cu_count) {
    if (device < 0 || device >= MAX_DEVICES) return set_error(SK_ERR_UNSUPPORTED, "device index beyond 63");
    std::lock_guard<std::mutex> g(mu);
    if (!ptr[device]) {
      void *p = nullptr;
      hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p) return hip_error("hipGetSymbolAddress", e);
      int n = 0;
      e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device);
      if (e != hipSuccess) return hip_error("hipDeviceGetAttribute", e);
      cus[device] = n;
      ptr[device] = p;
    }
    *out = ptr[device];
    *cu_count = cus[device];
    return SK_OK;
  }
};
StaticScratch &static_scratch() {
  static StaticScratch *s = new StaticScratch();
  return *s;
}

}  // namespace

// The device side of one tile table: one allocation holding
//   work records (tile + its operator's descriptor) | the LDS tiles' records once more, die by die, and the
//   lists' offsets | queue counters | tiles left per operator | completion stamps | split-K offsets |
//   split-K arrival counters | split-K workspace
struct DeviceTables {
  void *blob = nullptr;
  size_t blob_bytes = 0;  // size of the pooled block behind `blob`
  sk::TileWork *work = nullptr;
  sk::TileWork *xwork = nullptr;  // null: the plan has no per-die lists
  uint32_t *xoff = nullptr;       // [9]
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
  bool any_alignment = false;  // some operator cannot be read in aligned 16-byte pieces
  // Every tile is short (at most 64 KB of operands): sk_launch gives workgroup b the tiles b, b + grid, ...
  // instead of running the queue.  A queue claim is an atomic round trip before the next record can be
  // fetched, and such tiles are over before it returns: three thousand tiny operators take 29 instead of
  // 47 us this way, and with tiles this short the fixed assignment cannot leave anyone idle for long.
  bool fixed_assignment = false;
  double ticks_per_ms = 0.0;
  DeviceTables dev;
  // the one-launch-per-operator baseline: every operator tiled as if it were alone;
  // planned and uploaded by the first sk_launch_sequential
  bool seq_ready = false;
  sk::HostPlan seq_host;
  DeviceTables seq_dev;
  // sk_launch_static: host image of the uploaded part of the tables (built by sk_plan_create for host-only
  // plans, pageable memory) and where its parts lie
  std::vector<char> image;
  // which launch a new one must not overlap, and what sk_plan_destroy has to wait for
  hipEvent_t last_use = nullptr;  // recorded behind the latest launch made outside a stream capture
  sk::LaunchLedger ledger;
};

namespace {

// Where the parts of a table set lie inside its one block of device memory.
struct TableLayout {
  size_t off_work, off_xwork, off_xoff, off_cnt, off_rem, off_stamps, off_wsoff, off_arrive;
  size_t upload;  // bytes the host fills in (everything before the workspace)
  size_t total;   // upload + split-K workspace
};

TableLayout layout_of(const sk::HostPlan &hp) {
  const size_t nt = hp.tiles.size(), np = hp.dev.size(), nrect = hp.ws_off.size();
  TableLayout l;
  l.off_work = 0;
  l.off_xwork = align_up(l.off_work + nt * sizeof(sk::TileWork), 256);
  l.off_xoff = align_up(l.off_xwork + hp.xorder.size() * sizeof(sk::TileWork), 256);
  l.off_cnt = align_up(l.off_xoff + 9 * sizeof(uint32_t), 256);
  l.off_rem = align_up(l.off_cnt + sk::QUEUE_COUNTERS * sizeof(uint32_t), 256);
  l.off_stamps = align_up(l.off_rem + np * sizeof(uint32_t), 256);
  l.off_wsoff = align_up(l.off_stamps + (np + 1) * sizeof(uint64_t), 256);
  l.off_arrive = align_up(l.off_wsoff + nrect * sizeof(uint32_t), 256);
  l.upload = align_up(l.off_arrive + nrect * sizeof(uint32_t), 256);
  l.total = l.upload + (size_t)hp.ws_f32x4 * 16;
  return l;
}

// The host image of the uploaded part: work records, zeroed counters and stamps, countdowns, offsets.
void fill_image(const sk::HostPlan &hp, const TableLayout &l, char *stage) {
  const size_t nt = hp.tiles.size(), np = hp.dev.size(), nrect = hp.ws_off.size();
  // the work records are written in full below; everything behind them starts at zero
  std::memset(stage + nt * sizeof(sk::TileWork), 0, l.upload - nt * sizeof(sk::TileWork));
  if (nrect) std::memcpy(&stage[l.off_wsoff], hp.ws_off.data(), nrect * sizeof(uint32_t));
  for (size_t i = 0; i < nt; ++i) {
    sk::TileWork w;
    std::memset(&w, 0, sizeof(w));
    w.tile = hp.tiles[i];
    w.prob = hp.dev[w.tile.problem];
    std::memcpy(&stage[l.off_work + i * sizeof(w)], &w, sizeof(w));
  }
  for (size_t i = 0; i < hp.xorder.size(); ++i)
    std::memcpy(&stage[l.off_xwork + i * sizeof(sk::TileWork)], &stage[l.off_work + hp.xorder[i] * sizeof(sk::TileWork)],
                sizeof(sk::TileWork));
  std::memcpy(&stage[l.off_xoff], hp.xoff, sizeof(hp.xoff));
  for (size_t i = 0; i < np; ++i) {
    const uint32_t c = (uint32_t)hp.count[i];
    std::memcpy(&stage[l.off_rem + i * sizeof(uint32_t)], &c, sizeof(c));
  }
}

void bind_tables(DeviceTables &dt, void *base, const TableLayout &l) {
  char *b = (char *)base;
  dt.work = (sk::TileWork *)(b + l.off_work);
  dt.xwork = l.off_xoff > l.off_xwork ? (sk::TileWork *)(b + l.off_xwork) : nullptr;
  dt.xoff = (uint32_t *)(b + l.off_xoff);
  dt.counters = (uint32_t *)(b + l.off_cnt);
  dt.remaining = (uint32_t *)(b + l.off_rem);
  dt.stamps = (uint64_t *)(b + l.off_stamps);
  dt.ws_off = (uint32_t *)(b + l.off_wsoff);
  dt.arrive = (uint32_t *)(b + l.off_arrive);
  dt.ws = (sk::f32x4 *)(b + l.upload);
}

// Uploads the tables of `hp` to the current device (`device`).
sk_status upload_tables(const sk::HostPlan &hp, int device, DeviceTables &dt) {
  const TableLayout l = layout_of(hp);
  char *stage = t_stage.acquire(l.upload);
  if (!stage) return set_error(SK_ERR_ALLOC, "host staging allocation failed");
  fill_image(hp, l, stage);
  hipError_t e = table_pool().acquire(device, l.total, &dt.blob, &dt.blob_bytes);
  if (e != hipSuccess) {
    dt.blob = nullptr;
    return set_error(SK_ERR_ALLOC, std::string("hipMalloc: ") + hipGetErrorString(e));
  }
  e = hipMemcpy(dt.blob, stage, l.upload, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)table_pool().release(device, dt.blob, dt.blob_bytes);
    dt.blob = nullptr;
    return hip_error("hipMemcpy", e);
  }
  bind_tables(dt, dt.blob, l);
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
    const int32_t vec = sk::FLAG_VEC_A | sk::FLAG_VEC_B;
    for (const sk::DevProblem &d : plan->host.dev)
      if ((d.flags & vec) != vec) plan->any_alignment = true;
  }
  plan->fixed_assignment = !plan->host.tiles.empty();
  for (const sk_tile &t : plan->host.tiles) {
    const int es = sk::elem_size(plan->host.problems[t.problem].dtype);
    if (((int64_t)t.m_len + t.n_len) * (int64_t)t.k_len * es > 65536) {
      plan->fixed_assignment = false;
      break;
    }
  }
  if (prm.host_only && !plan->host.tiles.empty()) {
    const TableLayout l = layout_of(plan->host);
    if (l.total <= STATIC_SCRATCH_BYTES) {  // (larger plans cannot use sk_launch_static anyway)
      try {
        plan->image.resize(l.upload);
      } catch (const std::bad_alloc &) {
        delete plan;
        return set_error(SK_ERR_ALLOC, "host allocation failed");
      }
      fill_image(plan->host, l, plan->image.data());
    }
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
    st = upload_tables(plan->host, plan->device, plan->dev);
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
  if (plan->dev.blob || plan->seq_dev.blob) {
    // the tables go back to the pool, where the next plan may overwrite them at once:
    // wait for every launch that may still read them
    hipError_t e = hipSuccess;
    int cur = -1;
    const sk::LaunchLedger::Wait wait = plan->ledger.before_destroy();
    if (wait == sk::LaunchLedger::DEVICE) {
      e = hipGetDevice(&cur);
      if (e == hipSuccess && cur != plan->device) e = hipSetDevice(plan->device);
      if (e == hipSuccess) e = hipDeviceSynchronize();
      if (cur >= 0 && cur != plan->device) (void)hipSetDevice(cur);
    } else if (wait == sk::LaunchLedger::EVENT) {
      e = hipEventSynchronize(plan->last_use);
    }
    if (e != hipSuccess) st = hip_error("waiting for the plan's launches", e);
    for (DeviceTables *dt : {&plan->dev, &plan->seq_dev}) {
      if (!dt->blob) continue;
      // after a failed wait the block is neither reused nor freed under a running kernel
      if (st == SK_OK) {
        e = table_pool().release(plan->device, dt->blob, dt->blob_bytes);
        if (e != hipSuccess) st = hip_error("hipFree", e);
      }
    }
  }
  if (plan->last_use) (void)hipEventDestroy(plan->last_use);
  delete plan;
  return st;
}

#ifdef SK_DIAG_CLOCKS
// Diagnostic build only (not in include/superkernel.h): copies the phase stamps of the current device to `dst`
// (host memory, at most `bytes`), resp. zeroes them (return a hipError_t); the shape of the stamp array.
int sk_diag_read(void *dst, uint64_t bytes) {
  return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(sk::g_diag), bytes <= sizeof(sk::g_diag) ? bytes : sizeof(sk::g_diag));
}
// How many workgroups are stamped, and how many tiles of each.
void sk_diag_shape(int *workgroups, int *tiles) {
  *workgroups = sk::SK_DIAG_WGS;
  *tiles = sk::SK_DIAG_TILES;
}
int sk_diag_clear(void) {
  void *p = nullptr;
  hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(sk::g_diag));
  if (e != hipSuccess) return (int)e;
  return (int)hipMemset(p, 0, sizeof(sk::g_diag));
}
#endif

sk_status sk_release_cached_memory(void) {
  hipError_t e = table_pool().trim();
  if (e != hipSuccess) return hip_error("hipFree", e);
  return SK_OK;
}

static sk_status launch_range(sk_plan *plan, const DeviceTables &dt, hipStream_t stream, uint32_t begin, uint32_t end,
                              int grid, bool dynamic, bool write_start, bool whole_table = false) {
  if (end <= begin || grid <= 0) return SK_OK;
  sk::KernelArgs a;
  // the per-die lists cover the LDS tiles of the whole table, and only the queue hands them out
  const bool lists = whole_table && dynamic && dt.xwork != nullptr;
  a.xwork = lists ? dt.xwork : nullptr;
  a.xoff = lists ? dt.xoff : nullptr;
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
  void (*kernel)(const sk::TileWork *, sk::KernelArgs) = nullptr;
  if (plan->any_alignment) {
    switch (plan->only_dtype) {
      case SK_F32: kernel = sk::sk_superkernel<SK_F32, true>; break;
      case SK_BF16: kernel = sk::sk_superkernel<SK_BF16, true>; break;
      case SK_F16: kernel = sk::sk_superkernel<SK_F16, true>; break;
      default: kernel = sk::sk_superkernel<-1, true>; break;
    }
  } else {
    switch (plan->only_dtype) {
      case SK_F32: kernel = sk::sk_superkernel<SK_F32, false>; break;
      case SK_BF16: kernel = sk::sk_superkernel<SK_BF16, false>; break;
      case SK_F16: kernel = sk::sk_superkernel<SK_F16, false>; break;
      default: kernel = sk::sk_superkernel<-1, false>; break;
    }
  }
  hipLaunchKernelGGL(kernel, g, b, 0, stream, dt.work, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_error("kernel launch", e);
  return SK_OK;
}

// Admission of a launch (see sk::LaunchLedger): SK_ERR_BUSY when the plan's previous launch went to another
// stream and has not completed.  Best effort: launches recorded into graphs are not tracked.
static sk_status admit_launch(sk_plan *plan, hipStream_t stream, bool *capturing) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  *capturing = hipStreamIsCapturing(stream, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone;
  if (plan->ledger.before_launch((uintptr_t)stream, *capturing) == sk::LaunchLedger::QUERY_EVENT) {
    const hipError_t q = hipEventQuery(plan->last_use);
    if (q == hipErrorNotReady) {
      (void)hipGetLastError();
      return set_error(SK_ERR_BUSY, "the plan's previous launch is still running on another stream");
    }
    if (q != hipSuccess) return hip_error("hipEventQuery", q);
  }
  return SK_OK;
}

// Records the event that the next launch on another stream and sk_plan_destroy look at.
static void note_launch(sk_plan *plan, hipStream_t stream, bool capturing) {
  bool recorded = false;
  if (!capturing) {
    if (!plan->last_use && hipEventCreateWithFlags(&plan->last_use, hipEventDisableTiming) != hipSuccess)
      plan->last_use = nullptr;
    recorded = plan->last_use && hipEventRecord(plan->last_use, stream) == hipSuccess;
  }
  plan->ledger.after_launch((uintptr_t)stream, capturing, recorded);
}

// Ahead of a stamped launch: the start stamp is a running minimum over the workgroups' first clocks.
static sk_status arm_start_stamp(sk_plan *plan, hipStream_t stream) {
  if (!plan->host.params.stamps) return SK_OK;
  hipLaunchKernelGGL(sk::sk_arm_start_stamp, dim3(1), dim3(1), 0, stream, plan->dev.stamps + plan->host.dev.size());
  const hipError_t e = hipGetLastError();
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
  if (plan->host.tiles.empty()) return SK_OK;
  const hipStream_t stream = (hipStream_t)hip_stream;
  bool capturing = false;
  st = admit_launch(plan, stream, &capturing);
  if (st != SK_OK) return st;
  st = arm_start_stamp(plan, stream);
  if (st != SK_OK) return st;
  st = launch_range(plan, plan->dev, stream, 0u, (uint32_t)plan->host.tiles.size(), plan->grid,
                    !plan->fixed_assignment, true, true);
  note_launch(plan, stream, capturing);
  return st;
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
    st = upload_tables(plan->seq_host, plan->device, plan->seq_dev);
    if (st != SK_OK) return st;
    plan->seq_ready = true;
  }
  const size_t n = plan->seq_host.dev.size();
  if (n == 0) return SK_OK;
  const hipStream_t stream = (hipStream_t)hip_stream;
  bool capturing = false;
  st = admit_launch(plan, stream, &capturing);
  if (st != SK_OK) return st;
  st = arm_start_stamp(plan, stream);
  if (st != SK_OK) return st;
  for (size_t i = 0; i < n && st == SK_OK; ++i) {
    const int64_t first = plan->seq_host.first[i], count = plan->seq_host.count[i];
    const int grid = (int)(count < plan->grid_cap ? count : plan->grid_cap);
    st = launch_range(plan, plan->seq_dev, stream, (uint32_t)first, (uint32_t)(first + count), grid, false, i == 0);
  }
  note_launch(plan, stream, capturing);  // also after a failure: some launches may be out
  return st;
}

sk_status sk_launch_static(sk_plan *plan, void *hip_stream) {
  if (!plan) return set_error(SK_ERR_INVALID_ARG, "plan is null");
  if (!plan->host.params.host_only)
    return set_error(SK_ERR_STATE, "sk_launch_static takes a plan created with host_only = 1; use sk_launch for this one");
  if (plan->host.params.stamps)
    return set_error(SK_ERR_STATE, "completion stamps are not available through sk_launch_static");
  if (plan->host.tiles.empty()) return SK_OK;
  const TableLayout l = layout_of(plan->host);
  if (l.total > STATIC_SCRATCH_BYTES)
    return set_error(SK_ERR_UNSUPPORTED, "plan needs " + std::to_string(l.total) + " bytes of tables and workspace, the static scratch holds " +
                                             std::to_string(STATIC_SCRATCH_BYTES));
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_error("hipGetDevice", e);
  void *base = nullptr;
  int cus = 0;
  sk_status st = static_scratch().get(dev, &base, &cus);
  if (st != SK_OK) return st;
  const hipStream_t stream = (hipStream_t)hip_stream;
  // Records, zeroed queue and arrival counters, workspace offsets: everything the kernel expects to find.
  // (The split-K workspace behind them is written before it is read and needs no clearing.)
  e = hipMemcpyAsync(base, plan->image.data(), l.upload, hipMemcpyHostToDevice, stream);
  if (e != hipSuccess) return hip_error("hipMemcpyAsync", e);
  DeviceTables dt;
  bind_tables(dt, base, l);
  const int64_t limit = plan->host.params.grid_limit > 0 ? plan->host.params.grid_limit : 2 * (int64_t)cus;
  const int64_t ntiles = (int64_t)plan->host.tiles.size();
  plan->grid_cap = limit;
  plan->grid = (int)(ntiles < limit ? ntiles : limit);
  return launch_range(plan, dt, stream, 0u, (uint32_t)ntiles, plan->grid, !plan->fixed_assignment, false, true);
}

int64_t sk_plan_num_tiles(const sk_plan *plan) { return plan ? (int64_t)plan->host.tiles.size() : -1; }
int32_t sk_plan_num_problems(const sk_plan *plan) { return plan ? (int32_t)plan->host.dev.size() : -1; }
int32_t sk_plan_grid(const sk_plan *plan) { return plan ? plan->grid : -1; }

sk_status sk_plan_get_xcd_lists(const sk_plan *plan, uint32_t *offsets, uint32_t *tiles, int64_t cap) {
  if (!plan || !offsets) return set_error(SK_ERR_INVALID_ARG, "plan or offsets is null");
  std::memcpy(offsets, plan->host.xoff, sizeof(plan->host.xoff));
  if (tiles) {
    if (cap < (int64_t)plan->host.xorder.size()) return set_error(SK_ERR_INVALID_ARG, "destination too small for the lists");
    if (!plan->host.xorder.empty()) std::memcpy(tiles, plan->host.xorder.data(), plan->host.xorder.size() * sizeof(uint32_t));
  }
  return SK_OK;
}

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
  if (done_ticks || start_tick) {
    // one copy for both: the start stamp follows the n completion stamps
    std::vector<uint64_t> host;
    try {
      host.resize(n + 1);
    } catch (const std::bad_alloc &) {
      return set_error(SK_ERR_ALLOC, "host allocation failed");
    }
    hipError_t e = hipMemcpy(host.data(), plan->dev.stamps, (n + 1) * sizeof(uint64_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_error("hipMemcpy", e);
    if (done_ticks && n) std::memcpy(done_ticks, host.data(), n * sizeof(uint64_t));
    if (start_tick) *start_tick = host[n];
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
    case SK_ERR_BUSY: return "the plan's previous launch is still running on another stream";
    case SK_ERR_STATE: return "plan is not in a state that allows this call";
  }
  return "unknown status";
}

const char *sk_last_error(void) { return g_last_error.c_str(); }

}  // extern "C"
