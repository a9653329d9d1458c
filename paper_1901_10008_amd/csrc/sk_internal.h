// Internal declarations shared by the host planner and the HIP launch code.
// Not part of the public ABI (include/superkernel.h is).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "superkernel.h"

namespace sk {

enum : int32_t {
  FLAG_VEC_A = 1,  // activation rows can be read in aligned 16-byte pieces
  FLAG_VEC_B = 2,  // weight rows can be read in aligned 16-byte pieces
  FLAG_VEC_C = 4,  // four consecutive outputs of a row can be stored as one vector
};

enum : uint16_t {
  CLS_SKINNY_FIRST = 0,  // 0..8: 3*log2(rm) + log2(wk), rm = 1, 2, 4 blocks of 16 activation rows
  CLS_TILE_128x128 = 9,
  CLS_TILE_128x64 = 10,  // operators with at most 64 output columns
};

// Device-side description of one operator in its canonical GEMM view
//   C[Mg,Ng] = A'[Mg,Kg] . Bs[Ng,Kg]^T
// where A' is either a plain row-major matrix (gather == 0) or the implicit
// patch matrix of an image (gather == 1; Section 5.3: a convolution is
// executed through the GEMM that backs it), NHWC or, with nchw set, NCHW.
struct DevProblem {
  const void *A;
  const void *B;
  void *C;
  int64_t lda, ldb, ldc;  // row strides in elements (lda unused when gather)
  int32_t Mg, Ng, Kg;
  int32_t dtype;
  int32_t gather;
  int32_t H, W, Cin, Ho, Wo, R, S, pad_h, pad_w;
  int32_t flags;
  int32_t tile_first, tile_count;
  int32_t stride;  // of a convolution, both directions (>= 1)
  int32_t nchw;    // convolution on channel-major arrays: X[Nb,Cin,H,W], W[Cout,Cin,R,S], Y[Nb,Cout,Ho,Wo]
  int32_t pad0;
  // Division by a convolution's Ho*Wo, Wo, Cin and S as multiply and shift (see FastDiv): the tile set-up
  // divides row and reduction indices by them for every row a thread stages.
  uint32_t div_hw[2], div_wo[2], div_cin[2], div_s[2];
};
static_assert(sizeof(DevProblem) % 8 == 0, "DevProblem must stay 8-byte sized");

// n / d for 0 <= n < 2^31 as (n * mul) >> shift with mul = floor(2^(31+l) / d) + 1, l = ceil(log2 d), shift = 31 + l:
// mul * d = 2^(31+l) + e with 0 < e <= d <= 2^l, so the quotient is off by less than n / (d * 2^31) < 1 / d.
struct FastDiv {
  uint32_t mul, shift;
};
inline FastDiv fast_div_of(uint32_t d) {
  if (d == 0) return FastDiv{0u, 0u};
  uint32_t l = 0;
  while (((uint64_t)1 << l) < d) ++l;
  const uint64_t mul = (((uint64_t)1 << (31 + l)) / d) + 1;  // < 2^32 + 1; equals 2^32 only for d = 1 ... see below
  // d = 1: l = 0, mul = 2^31 + 1, shift 31: (n * (2^31 + 1)) >> 31 = n for n < 2^31
  return FastDiv{(uint32_t)mul, 31u + l};
}

// What the device reads per tile: the record of the tile table with a copy of its operator's
// descriptor beside it, so that one fetch (and one prefetch) brings everything a workgroup
// needs to start the tile.
struct TileWork {
  sk_tile tile;
  DevProblem prob;
};
static_assert(sizeof(TileWork) == 192, "TileWork layout");

struct HostPlan {
  std::vector<sk_problem> problems;
  std::vector<DevProblem> dev;
  std::vector<sk_tile> tiles;
  std::vector<int32_t> order;
  std::vector<int64_t> first, count;
  std::vector<uint32_t> ws_off;  // per output rectangle: offset of its split-K partials, in 16-byte units
  int64_t ws_f32x4 = 0;          // size of the split-K workspace, in 16-byte units
  // The LDS tiles of the table once more, as eight lists (one per accelerator die): xorder[xoff[x] .. xoff[x+1])
  // are the table indices of the tiles die x takes, in the order it takes them.  Empty when xcd_part is 0.
  std::vector<uint32_t> xorder;
  uint32_t xoff[9] = {};
  sk_plan_params params;
  int64_t target_tile_bytes = 0;
};

// Pure host planning (no HIP call).  Returns SK_OK or an error with `err` set.
sk_status plan_host(const sk_problem *problems, int32_t n, const sk_plan_params *params,
                    HostPlan &out, std::string &err);

// The tile tables of the one-launch-per-operator baseline: every operator of `whole` planned
// by plan_host as if it were submitted alone, concatenated in submission order.
sk_status plan_host_each_alone(const HostPlan &whole, HostPlan &out, std::string &err);

inline int elem_size(int32_t dtype) { return dtype == SK_F32 ? 4 : 2; }

// Sets the calling thread's sk_last_error() text and passes the status through (superkernel.hip).
sk_status set_last_error(sk_status st, const std::string &msg);

// ---- the arrival queue's decisions, free of HIP calls so that they can be exercised on the host ----

// One submitted operator as the batch selection sees it.
struct QueuedOp {
  double deadline_ms;  // absolute: submit time + budget (+inf if none)
  int64_t bytes;       // operand bytes, for the duration estimate
  const void *C;       // its output buffer
};

// Operand bytes of an operator (activations + weights + output, each once), 0 for a malformed one.
int64_t operand_bytes(const sk_problem &p);

// Estimated duration of a launch over `bytes` of operands.
double estimate_launch_ms(int64_t bytes, double bytes_per_ms, double floor_ms);

// Which of `ops` (any order) go into the next launch, as indices in the order they are to be planned:
// earliest deadline first, ties by index; an operator whose output buffer is in `busy` (sorted) or was
// taken by an earlier pick waits; SK_QUEUE_OOO closes the batch before the operator that would take
// the estimate (times `corr`) past cap_ms, unless the batch is still empty; SK_QUEUE_SEQUENTIAL takes
// the first submitted operator only (index 0), whatever its deadline.
std::vector<size_t> select_batch(const std::vector<QueuedOp> &ops, const std::vector<const void *> &busy, int policy,
                                 double cap_ms, double corr, double bytes_per_ms, double floor_ms);

// Bookkeeping of one plan's launches, free of HIP calls so that it can be exercised on the host.
// A plan has one tile queue, one set of split-reduction counters and one workspace: a launch may only
// start when the one before it has finished or precedes it on the same stream.  The ledger says when
// the caller has to ask the event behind the latest launch, and what sk_plan_destroy must wait for.
struct LaunchLedger {
  enum Ask { GO, QUERY_EVENT };            // QUERY_EVENT: launch only if the event has completed, else SK_ERR_BUSY
  enum Wait { NOTHING, EVENT, DEVICE };
  bool has_event = false;                  // an event sits behind the latest launch made outside a stream capture
  uintptr_t last_stream = 0;
  bool device_wide = false;                // launches the event does not cover (captured into a graph, or the
                                           // event could not be recorded): only a device-wide wait covers them
  Ask before_launch(uintptr_t stream, bool capturing) const;
  // event_recorded: the caller recorded the plan's event behind the launch (never under capture)
  void after_launch(uintptr_t stream, bool capturing, bool event_recorded);
  Wait before_destroy() const;
};

}  // namespace sk
