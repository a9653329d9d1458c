// The arrival queue of the C ABI (sk_queue_*): operators that arrive over time, coalesced into
// superkernel launches under one of three policies (Section 5, items (a) and (b), and Section 5.2 of the
// paper: tighter latency budgets first, operators that do not fit held back for a later launch).
//
// Everything here is host code on top of the library's own plan and launch calls and HIP events; the
// decisions themselves (which operators go into the next launch) are sk::select_batch in planner.cpp.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <deque>
#include <limits>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "sk_internal.h"

namespace {

using Clock = std::chrono::steady_clock;

struct Pending {
  sk_problem op;
  uint64_t ticket;
  double t_submit_ms;
  double budget_ms;  // +inf if none
  int64_t bytes;
};

struct Launch {
  sk_plan *plan = nullptr;  // owned unless `cached`
  bool cached = false;      // a single-operator plan of the time-multiplexing policy, kept for reuse
  hipEvent_t done = nullptr;
  std::vector<Pending> ops;  // in the order they were given to the planner
  double estimate_ms = 0.0;
  int32_t number = 0;
};

}  // namespace

struct sk_queue {
  sk_queue_params prm;
  hipStream_t stream = nullptr;
  Clock::time_point t0;
  std::vector<Pending> pending;  // arrival order
  std::deque<Launch> inflight;
  std::vector<sk_completion> ready;  // completions not yet handed out
  std::vector<hipEvent_t> spare_events;
  std::unordered_map<std::string, sk_plan *> solo;  // SK_QUEUE_SEQUENTIAL: one plan per distinct operator
  uint64_t next_ticket = 1;
  int32_t launches = 0;
  sk_queue_stats stats{};
  double corr = 1.0;     // running ratio of measured to estimated launch durations
  double prep_ms = 0.1;  // running cost of planning and launching a batch
  double t_free_ms = 0.0;  // when the device is expected to run dry
  double t_first_submit_ms = -1.0, t_last_done_ms = 0.0;

  double now_ms() const { return std::chrono::duration<double, std::milli>(Clock::now() - t0).count(); }
  int depth() const { return prm.depth > 0 ? prm.depth : (prm.policy == SK_QUEUE_SEQUENTIAL ? 16 : 2); }
};

namespace {

sk_status hip_fail(const char *what, hipError_t e) {
  return sk::set_last_error(SK_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

sk_status get_event(sk_queue *q, hipEvent_t *ev) {
  if (!q->spare_events.empty()) {
    *ev = q->spare_events.back();
    q->spare_events.pop_back();
    return SK_OK;
  }
  const hipError_t e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
  if (e != hipSuccess) return hip_fail("hipEventCreate", e);
  return SK_OK;
}

void complete(sk_queue *q, const Pending &p, double t_end_ms, int32_t launch, bool failed) {
  sk_completion c;
  c.ticket = p.ticket;
  c.budget_ms = p.budget_ms;
  c.launch = launch;
  if (failed) {
    c.latency_ms = -1.0;
    c.met = -1;
  } else {
    c.latency_ms = t_end_ms - p.t_submit_ms;
    c.met = c.latency_ms <= p.budget_ms ? 1 : 0;
    q->stats.met += c.met;
  }
  q->stats.completed += 1;
  q->ready.push_back(c);
}

// The front launch has completed on the device: hand out its operators' completions.
sk_status retire_front(sk_queue *q) {
  Launch l = std::move(q->inflight.front());
  q->inflight.pop_front();
  const double t_done = q->now_ms();
  q->t_last_done_ms = t_done;
  sk_status st = SK_OK;
  if (l.cached) {
    for (const Pending &p : l.ops) complete(q, p, t_done, l.number, false);
  } else {
    const size_t n = l.ops.size();
    std::vector<uint64_t> done(n);
    uint64_t start = 0;
    double rate = 0.0;
    st = sk_plan_get_stamps(l.plan, done.data(), &start, &rate);
    if (st == SK_OK && rate > 0.0) {
      uint64_t last = 0;
      for (uint64_t d : done) last = std::max(last, d);
      // anchored at the end: the host saw the launch complete at t_done
      for (size_t i = 0; i < n; ++i) complete(q, l.ops[i], t_done - (double)(last - done[i]) / rate, l.number, false);
      const double took = (double)(last - start) / rate;
      q->stats.device_busy_ms += took;
      if (l.estimate_ms > 0.0) q->corr = 0.8 * q->corr + 0.2 * std::min(4.0, std::max(0.25, took / l.estimate_ms));
    } else {
      for (const Pending &p : l.ops) complete(q, p, t_done, l.number, false);
    }
    const sk_status sd = sk_plan_destroy(l.plan);
    if (st == SK_OK) st = sd;
  }
  q->spare_events.push_back(l.done);
  q->t_free_ms = q->inflight.empty() ? t_done : std::max(t_done, q->t_free_ms);
  return st;
}

std::string key_of(const sk_problem &p) {
  sk_problem k = p;
  k.deadline_ms = 0.0;
  return std::string((const char *)&k, sizeof(k));
}

// Plans and launches the next batch if one is due.  *launched says whether it did.
sk_status launch_next(sk_queue *q, bool *launched) {
  *launched = false;
  if (q->pending.empty() || (int)q->inflight.size() >= q->depth()) return SK_OK;
  const double t = q->now_ms();
  const bool seq = q->prm.policy == SK_QUEUE_SEQUENTIAL;
  // The next launch is planned while the device still works on the one before it: early enough that it is
  // queued when that one ends (planning cost plus a margin for what the duration estimate is off by), not
  // earlier, because whatever arrives after planning waits for the launch after.
  if (!seq && !q->inflight.empty()) {
    const double margin = 0.03 + 0.15 * q->inflight.back().estimate_ms * q->corr;
    if (t < q->t_free_ms - q->prep_ms - margin) return SK_OK;
  }

  std::vector<sk::QueuedOp> view(q->pending.size());
  for (size_t i = 0; i < view.size(); ++i)
    view[i] = sk::QueuedOp{q->pending[i].t_submit_ms + q->pending[i].budget_ms, q->pending[i].bytes, q->pending[i].op.C};
  std::vector<const void *> busy;
  for (const Launch &l : q->inflight)
    for (const Pending &p : l.ops) busy.push_back(p.op.C);
  std::sort(busy.begin(), busy.end());
  const std::vector<size_t> pick = sk::select_batch(view, busy, q->prm.policy, q->prm.cap_ms, q->corr, q->prm.bytes_per_ms,
                                                    q->prm.launch_floor_ms);
  if (pick.empty()) return SK_OK;

  Launch l;
  l.number = ++q->launches;
  int64_t total = 0;
  std::vector<sk_problem> probs;
  probs.reserve(pick.size());
  for (size_t i : pick) {
    Pending p = q->pending[i];
    // what is left of the budget, from now (the planner orders by it; nothing is dropped when it is missed)
    p.op.deadline_ms = std::isfinite(p.budget_ms) ? std::max(1e-3, p.t_submit_ms + p.budget_ms - t) : 0.0;
    probs.push_back(p.op);
    total += p.bytes;
    l.ops.push_back(p);
  }
  {  // drop the picked operators from the pending list, keeping arrival order
    std::vector<char> gone(q->pending.size(), 0);
    for (size_t i : pick) gone[i] = 1;
    size_t w = 0;
    for (size_t i = 0; i < q->pending.size(); ++i)
      if (!gone[i]) q->pending[w++] = q->pending[i];
    q->pending.resize(w);
  }
  sk_status st = get_event(q, &l.done);
  if (st == SK_OK) {
    if (seq) {
      const std::string key = key_of(probs[0]);
      auto it = q->solo.find(key);
      if (it == q->solo.end()) {
        sk_plan *plan = nullptr;
        st = sk_plan_create(probs.data(), 1, nullptr, &plan);
        if (st == SK_OK) it = q->solo.emplace(key, plan).first;
      }
      if (st == SK_OK) {
        l.plan = it->second;
        l.cached = true;
      }
    } else {
      sk_plan_params prm;
      sk_plan_params_default(&prm);
      prm.stamps = 1;
      st = sk_plan_create(probs.data(), (int32_t)probs.size(), &prm, &l.plan);
    }
  }
  if (st == SK_OK) st = sk_launch(l.plan, q->stream);
  if (st == SK_OK) {
    const hipError_t e = hipEventRecord(l.done, q->stream);
    if (e != hipSuccess) st = hip_fail("hipEventRecord", e);
  }
  if (st != SK_OK) {
    // the batch is lost: its operators complete as failed, the caller sees the status
    const std::string why = sk_last_error();
    for (const Pending &p : l.ops) complete(q, p, 0.0, l.number, true);
    if (l.plan && !l.cached) (void)sk_plan_destroy(l.plan);
    if (l.done) q->spare_events.push_back(l.done);
    return sk::set_last_error(st, why);
  }
  l.estimate_ms = sk::estimate_launch_ms(total, q->prm.bytes_per_ms, q->prm.launch_floor_ms);
  q->stats.launches += 1;
  const double t_end = q->now_ms();
  if (!seq) {
    q->prep_ms = 0.8 * q->prep_ms + 0.2 * (t_end - t);
    q->t_free_ms = std::max(q->t_free_ms, t_end) + l.estimate_ms * q->corr;
  }
  q->inflight.push_back(std::move(l));
  *launched = true;
  return SK_OK;
}

// Retires what has finished, launches what is due; repeats while either makes progress.
sk_status pump(sk_queue *q) {
  sk_status first = SK_OK;
  for (;;) {
    bool progress = false;
    while (!q->inflight.empty()) {
      const hipError_t e = hipEventQuery(q->inflight.front().done);
      if (e == hipErrorNotReady) {
        (void)hipGetLastError();
        break;
      }
      if (e != hipSuccess) return hip_fail("hipEventQuery", e);
      const sk_status st = retire_front(q);
      if (st != SK_OK && first == SK_OK) first = st;
      progress = true;
    }
    bool launched = false;
    const sk_status st = launch_next(q, &launched);
    if (st != SK_OK && first == SK_OK) first = st;
    if (launched || st != SK_OK) progress = true;
    if (!progress) break;
  }
  return first;
}

}  // namespace

extern "C" {

void sk_queue_params_default(sk_queue_params *p) {
  if (!p) return;
  std::memset(p, 0, sizeof(*p));
  p->policy = SK_QUEUE_OOO;
  p->depth = 0;
  p->cap_ms = 0.5;
  p->bytes_per_ms = 5.5e9;
  p->launch_floor_ms = 0.02;
}

sk_status sk_queue_create(const sk_queue_params *params, void *hip_stream, sk_queue **out) {
  if (!out) return sk::set_last_error(SK_ERR_INVALID_ARG, "out is null");
  sk_queue_params prm;
  if (params)
    prm = *params;
  else
    sk_queue_params_default(&prm);
  if (prm.policy < SK_QUEUE_SEQUENTIAL || prm.policy > SK_QUEUE_OOO || prm.depth < 0 || prm.depth > 64 ||
      !(prm.cap_ms > 0.0) || !(prm.bytes_per_ms > 0.0) || !(prm.launch_floor_ms >= 0.0))
    return sk::set_last_error(SK_ERR_INVALID_ARG, "sk_queue_params field out of range");
  sk_queue *q = new (std::nothrow) sk_queue();
  if (!q) return sk::set_last_error(SK_ERR_ALLOC, "host allocation failed");
  q->prm = prm;
  q->stream = (hipStream_t)hip_stream;
  q->t0 = Clock::now();
  *out = q;
  return SK_OK;
}

sk_status sk_queue_submit(sk_queue *q, const sk_problem *ops, const double *budget_ms, int32_t n, uint64_t *tickets) {
  if (!q) return sk::set_last_error(SK_ERR_INVALID_ARG, "queue is null");
  if (n < 0 || (n > 0 && !ops)) return sk::set_last_error(SK_ERR_INVALID_ARG, "ops is null or n < 0");
  try {
    const double t = q->now_ms();
    if (n > 0 && q->t_first_submit_ms < 0.0) q->t_first_submit_ms = t;
    for (int32_t i = 0; i < n; ++i) {
      Pending p;
      p.op = ops[i];
      p.ticket = q->next_ticket++;
      p.t_submit_ms = t;
      const double b = budget_ms ? budget_ms[i] : std::numeric_limits<double>::infinity();
      p.budget_ms = (b > 0.0 && !std::isnan(b)) ? b : std::numeric_limits<double>::infinity();
      p.bytes = sk::operand_bytes(p.op);
      if (tickets) tickets[i] = p.ticket;
      q->pending.push_back(p);
      q->stats.submitted += 1;
    }
    return pump(q);
  } catch (const std::bad_alloc &) {
    return sk::set_last_error(SK_ERR_ALLOC, "host allocation failed");
  }
}

sk_status sk_queue_poll(sk_queue *q, int32_t wait, sk_completion *out, int32_t cap, int32_t *n_out) {
  if (!q) return sk::set_last_error(SK_ERR_INVALID_ARG, "queue is null");
  if (cap < 0 || (cap > 0 && !out) || !n_out) return sk::set_last_error(SK_ERR_INVALID_ARG, "bad output arguments");
  *n_out = 0;
  sk_status st = SK_OK;
  try {
    st = pump(q);
    while (wait && q->ready.empty() && st == SK_OK && (!q->inflight.empty() || !q->pending.empty())) {
      if (!q->inflight.empty()) {
        // nothing to hand out yet: sleep on the oldest launch, unless the next batch falls due first
        const bool more = !q->pending.empty() && (int)q->inflight.size() < q->depth();
        if (more && q->prm.policy != SK_QUEUE_SEQUENTIAL) {
          // (busy-wait: the gap is a fraction of a millisecond)
          st = pump(q);
          continue;
        }
        const hipError_t e = hipEventSynchronize(q->inflight.front().done);
        if (e != hipSuccess) return hip_fail("hipEventSynchronize", e);
      }
      st = pump(q);
    }
  } catch (const std::bad_alloc &) {
    return sk::set_last_error(SK_ERR_ALLOC, "host allocation failed");
  }
  const int32_t n = (int32_t)std::min<size_t>((size_t)cap, q->ready.size());
  if (n > 0) {
    std::memcpy(out, q->ready.data(), (size_t)n * sizeof(sk_completion));
    q->ready.erase(q->ready.begin(), q->ready.begin() + n);
  }
  *n_out = n;
  return st;
}

sk_status sk_queue_get_stats(const sk_queue *q, sk_queue_stats *stats) {
  if (!q || !stats) return sk::set_last_error(SK_ERR_INVALID_ARG, "null argument");
  *stats = q->stats;
  stats->span_ms = q->t_first_submit_ms < 0.0 ? 0.0 : std::max(0.0, q->t_last_done_ms - q->t_first_submit_ms);
  return SK_OK;
}

sk_status sk_queue_destroy(sk_queue *q) {
  if (!q) return SK_OK;
  sk_status st = SK_OK;
  for (Launch &l : q->inflight) {
    if (l.done) {
      const hipError_t e = hipEventSynchronize(l.done);
      if (e != hipSuccess && st == SK_OK) st = hip_fail("hipEventSynchronize", e);
      (void)hipEventDestroy(l.done);
    }
    if (l.plan && !l.cached) {
      const sk_status sd = sk_plan_destroy(l.plan);
      if (st == SK_OK) st = sd;
    }
  }
  for (auto &kv : q->solo) {
    const sk_status sd = sk_plan_destroy(kv.second);
    if (st == SK_OK) st = sd;
  }
  for (hipEvent_t e : q->spare_events) (void)hipEventDestroy(e);
  delete q;
  return st;
}

}  // extern "C"
