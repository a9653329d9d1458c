// Host-only driver for the planner under AddressSanitizer / UndefinedBehaviorSanitizer:
// seeded random operator lists (odd sizes, strides, all element types, every parameter
// combination the planner accepts, and lists it must reject), planned whole and operator by
// operator.  Checks only what must hold for any input: status codes, table sizes, that every
// record stays inside its operator.  Byte-exact comparison with the reference planner is the
// Python tests' job.
#include <cstdint>
#include <algorithm>
#include <cstdio>
#include <limits>
#include <random>
#include <string>
#include <vector>

#include "sk_internal.h"

static int fail(const char *what, int seed) {
  std::fprintf(stderr, "planner_driver: %s (seed %d)\n", what, seed);
  return 1;
}

int main() {
  for (int seed = 0; seed < 300; ++seed) {
    std::mt19937 g(seed);
    auto pick = [&](std::initializer_list<int> v) { return *(v.begin() + g() % v.size()); };
    const int n = (int)(g() % 40);
    std::vector<sk_problem> ps((size_t)n);
    uintptr_t addr = 0x10000000;
    bool expect_ok = true;
    for (int i = 0; i < n; ++i) {
      sk_problem &p = ps[(size_t)i];
      p = sk_problem{};
      p.dtype = pick({SK_F32, SK_BF16, SK_F16});
      const int es = p.dtype == SK_F32 ? 4 : 2;
      int64_t na, nb, nc;
      if (g() % 5 < 3) {
        p.op = SK_GEMM;
        p.M = pick({1, 2, 7, 16, 17, 33, 64, 65, 129, 300, 1000});
        p.N = pick({1, 5, 31, 32, 33, 127, 128, 129, 500, 4097});
        p.K = pick({1, 3, 8, 63, 64, 65, 256, 1000, 4096, 9000});
        p.lda = g() % 3 ? 0 : p.K + (int)(g() % 9);
        p.ldb = g() % 3 ? 0 : p.K + (int)(g() % 9);
        p.ldc = g() % 3 ? 0 : p.N + (int)(g() % 9);
        na = (int64_t)p.M * (p.lda ? p.lda : p.K);
        nb = (int64_t)p.N * (p.ldb ? p.ldb : p.K);
        nc = (int64_t)p.M * (p.ldc ? p.ldc : p.N);
      } else {
        p.op = SK_CONV2D_NHWC;
        p.Nb = 1 + (int)(g() % 2);
        p.H = 1 + (int)(g() % 40);
        p.Wd = 1 + (int)(g() % 40);
        p.Cin = pick({1, 3, 8, 64, 200});
        p.Cout = pick({1, 7, 64, 130});
        p.R = pick({1, 3, 5, 7});
        p.S = pick({1, 3});
        p.pad_h = (int)(g() % 4);
        p.pad_w = (int)(g() % 2);
        p.stride = (int)(g() % 4);
        if (p.H + 2 * p.pad_h < p.R || p.Wd + 2 * p.pad_w < p.S) expect_ok = false;
        na = (int64_t)p.Nb * p.H * p.Wd * p.Cin;
        nb = (int64_t)p.Cout * p.R * p.S * p.Cin;
        nc = (int64_t)p.Nb * (p.H + 2 * p.pad_h + 1) * (p.Wd + 2 * p.pad_w + 1) * p.Cout;
      }
      p.A = (const void *)addr;
      addr += (uintptr_t)(na * es + 511) / 256 * 256;
      p.B = (const void *)addr;
      addr += (uintptr_t)(nb * es + 511) / 256 * 256;
      p.C = (void *)(addr + (g() % 4 == 0 ? 2 : 0));  // sometimes misaligned
      addr += (uintptr_t)(nc * es + 767) / 256 * 256;
      const double ds[] = {0.0, -1.0, 0.5, 0.5, 3.0, 1e300, std::numeric_limits<double>::infinity(),
                           std::numeric_limits<double>::quiet_NaN()};
      p.deadline_ms = ds[g() % 8];
    }
    sk_plan_params prm;
    sk_plan_params_default(&prm);
    prm.host_only = 1;
    prm.edf = (int)(g() % 2);
    prm.skinny_max_m = pick({0, 8, 16, 32, 64});
    prm.tile_bytes_min = pick({1024, 4096, 32768, 1 << 18});
    prm.tile_bytes_max = prm.tile_bytes_min * pick({1, 2, 16, 64});
    prm.balance_div = pick({1, 7, 64, 512, 2048});
    prm.max_groups = pick({1, 3, 4, 64, 256});
    prm.tail_div = pick({0, 1, 16, 384, 5000});
    sk::HostPlan hp;
    std::string err;
    const sk_status st = sk::plan_host(n ? ps.data() : nullptr, n, &prm, hp, err);
    if (!expect_ok) {
      if (st == SK_OK) return fail("a filter larger than its padded image was accepted", seed);
      continue;
    }
    if (st != SK_OK) {
      std::fprintf(stderr, "%s\n", err.c_str());
      return fail("plan_host failed on a valid list", seed);
    }
    if ((int)hp.dev.size() != n || (int)hp.order.size() != n) return fail("table sizes", seed);
    int64_t sum = 0;
    for (int i = 0; i < n; ++i) sum += hp.count[(size_t)i];
    if (sum != (int64_t)hp.tiles.size()) return fail("tile counts do not add up", seed);
    for (const sk_tile &t : hp.tiles) {
      if ((int)t.problem >= n) return fail("record names a missing operator", seed);
      const sk::DevProblem &d = hp.dev[t.problem];
      if (t.m_len < 1 || t.n_len < 1 || t.k_len < 1 || (int64_t)t.m0 + t.m_len > d.Mg ||
          (int64_t)t.n0 + t.n_len > d.Ng || (int64_t)t.k0 + t.k_len > d.Kg || t.ks_idx >= t.S ||
          t.out_tile_id >= hp.ws_off.size())
        return fail("record leaves its operator", seed);
    }
    sk::HostPlan alone;
    if (sk::plan_host_each_alone(hp, alone, err) != SK_OK) return fail("plan_host_each_alone", seed);
    if (alone.dev.size() != hp.dev.size()) return fail("baseline tables", seed);
  }
  // lists the planner must reject
  {
    sk::HostPlan hp;
    std::string err;
    sk_problem p{};
    p.op = SK_GEMM;
    p.dtype = SK_BF16;
    p.M = 4;
    p.N = 64;
    p.K = 64;
    p.A = (const void *)0x1000;
    p.B = (const void *)0x2000;
    p.C = (void *)0x3000;
    sk_problem two[2] = {p, p};  // same output twice
    if (sk::plan_host(two, 2, nullptr, hp, err) != SK_ERR_OVERLAP) return fail("overlap not detected", -1);
    p.M = 0;
    if (sk::plan_host(&p, 1, nullptr, hp, err) != SK_ERR_INVALID_ARG) return fail("M = 0 accepted", -1);
    if (sk::plan_host(nullptr, 3, nullptr, hp, err) != SK_ERR_INVALID_ARG) return fail("null list accepted", -1);
  }
  // the launch ledger: which launches are admitted at once, which only after the plan's event has
  // completed, and what destroying the plan waits for
  {
    using L = sk::LaunchLedger;
    L l;
    const uintptr_t s1 = 0x100, s2 = 0x200;
    if (l.before_destroy() != L::NOTHING) return fail("a plan never launched waits for something", -2);
    if (l.before_launch(s1, false) != L::GO) return fail("first launch not admitted", -2);
    l.after_launch(s1, false, true);
    if (l.before_launch(s1, false) != L::GO) return fail("same stream must be admitted: the stream orders it", -2);
    if (l.before_launch(s2, false) != L::QUERY_EVENT) return fail("another stream must ask the event", -2);
    if (l.before_launch(0, false) != L::QUERY_EVENT) return fail("the default stream is another stream", -2);
    if (l.before_destroy() != L::EVENT) return fail("destroy must wait for the event", -2);
    l.after_launch(s2, false, true);  // admitted after the event completed: now the latest launch is on s2
    if (l.before_launch(s2, false) != L::GO || l.before_launch(s1, false) != L::QUERY_EVENT)
      return fail("the ledger did not move to the new stream", -2);
    if (l.before_destroy() != L::EVENT) return fail("one event covers launches admitted one after the other", -2);
    if (l.before_launch(s1, true) != L::GO) return fail("a captured launch cannot ask anything", -2);
    l.after_launch(s1, true, false);
    if (l.before_destroy() != L::DEVICE) return fail("graph replays need the device-wide wait", -2);
    if (l.before_launch(s1, false) != L::QUERY_EVENT) return fail("eager launches are still checked after a capture", -2);
    L m;
    m.after_launch(s1, false, false);  // the event could not be recorded
    if (m.before_destroy() != L::DEVICE) return fail("a launch without an event needs the device-wide wait", -2);
    if (m.before_launch(s2, false) != L::GO) return fail("nothing to ask without an event", -2);
    L d;                               // first launch on the default stream (handle 0)
    d.after_launch(0, false, true);
    if (d.before_launch(0, false) != L::GO || d.before_launch(s1, false) != L::QUERY_EVENT)
      return fail("default stream as the plan's stream", -2);
  }
  // the arrival queue's batch selection
  {
    const double inf = std::numeric_limits<double>::infinity();
    char buf[8];
    const void *c0 = buf, *c1 = buf + 1, *c2 = buf + 2, *c3 = buf + 3;
    // arrival order: deadlines 5, 1, inf, 1 (tie with index 1), 0.5 on the buffer of index 0
    std::vector<sk::QueuedOp> ops = {{5.0, 1000, c0}, {1.0, 1000, c1}, {inf, 1000, c2}, {1.0, 4000, c3}, {0.5, 1000, c0}};
    std::vector<const void *> none, busy = {c1};
    std::sort(busy.begin(), busy.end());
    auto same = [](const std::vector<size_t> &a, std::initializer_list<size_t> b) { return a == std::vector<size_t>(b); };
    // everything that is free, earliest deadline first, ties by arrival; the later operator of a shared buffer waits
    if (!same(sk::select_batch(ops, none, SK_QUEUE_COALESCE, 0.5, 1.0, 1000.0, 0.0), {4, 1, 3, 2}))
      return fail("coalesce order", -3);
    if (!same(sk::select_batch(ops, busy, SK_QUEUE_COALESCE, 0.5, 1.0, 1000.0, 0.0), {4, 3, 2}))
      return fail("an operator whose output is in flight must wait", -3);
    // 1000 bytes per ms: the cap of 2.5 ms closes the batch before the 4000-byte operator; the operators behind
    // it in deadline order wait as well
    if (!same(sk::select_batch(ops, none, SK_QUEUE_OOO, 2.5, 1.0, 1000.0, 0.0), {4, 1})) return fail("cap", -3);
    // ... a correction factor of 2 already before the second operator
    if (!same(sk::select_batch(ops, none, SK_QUEUE_OOO, 2.5, 2.0, 1000.0, 0.0), {4})) return fail("corrected cap", -3);
    // a first operator is always taken, however long
    if (!same(sk::select_batch(ops, none, SK_QUEUE_OOO, 0.001, 1.0, 1000.0, 0.0), {4})) return fail("first operator", -3);
    // the floor counts: three operators of 1 ms each are estimated at the floor of 10 ms
    if (!same(sk::select_batch(ops, none, SK_QUEUE_OOO, 10.0, 1.0, 1000.0, 10.0), {4, 1, 3, 2})) return fail("floor", -3);
    if (!same(sk::select_batch(ops, busy, SK_QUEUE_SEQUENTIAL, 0.5, 1.0, 1000.0, 0.0), {0})) return fail("arrival order", -3);
    if (!sk::select_batch({}, none, SK_QUEUE_OOO, 0.5, 1.0, 1000.0, 0.0).empty()) return fail("empty queue", -3);
    if (sk::estimate_launch_ms(5000, 1000.0, 0.02) != 5.0 || sk::estimate_launch_ms(10, 1000.0, 0.02) != 0.02)
      return fail("estimate", -3);
    sk_problem g{};
    g.op = SK_GEMM;
    g.dtype = SK_BF16;
    g.M = 3;
    g.N = 5;
    g.K = 7;
    if (sk::operand_bytes(g) != 2 * (3 * 7 + 5 * 7 + 3 * 5)) return fail("GEMM bytes", -3);
    sk_problem cv{};
    cv.op = SK_CONV2D_NHWC;
    cv.dtype = SK_F32;
    cv.Nb = 2; cv.H = 9; cv.Wd = 8; cv.Cin = 3; cv.Cout = 4; cv.R = 3; cv.S = 3; cv.pad_h = 1; cv.pad_w = 1; cv.stride = 2;
    // Ho = (9 + 2 - 3) / 2 + 1 = 5, Wo = (8 + 2 - 3) / 2 + 1 = 4
    if (sk::operand_bytes(cv) != 4 * (2 * 9 * 8 * 3 + 4 * 3 * 3 * 3 + 2 * 5 * 4 * 4)) return fail("convolution bytes", -3);
    cv.R = 20;
    if (sk::operand_bytes(cv) != 0) return fail("malformed operator", -3);
  }
  std::puts("planner_driver: ok");
  return 0;
}
