// Host planner: operators -> canonical GEMM view -> tile classes -> earliest-
// deadline-first operator order -> flat tile table.
//
// This is the paper's runtime packing step (Section 5.3: many small kernels are
// repacked into one large execution block) together with its latency-aware
// reordering (Section 5, item (a): tighter latency budgets first).  The paper
// gives no algorithm for either; the rule implemented here is a pure integer
// function of the operator list and sk_plan_params, so that it can be checked
// byte for byte against an independent reference planner.
//
// No HIP call is made in this file.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>
#include <unordered_set>

#include "sk_internal.h"

namespace sk {

namespace {

struct Canon {
  int64_t Mg, Ng, Kg;
  int32_t Ho, Wo;
};

std::string at(int32_t i) { return "problem " + std::to_string(i) + ": "; }

// Canonical GEMM view (rows = output pixels, columns = output channels,
// reduction = filter taps x input channels for a convolution).
sk_status canonicalise(const sk_problem &p, int32_t i, Canon &c, std::string &err) {
  if (p.dtype != SK_F32 && p.dtype != SK_BF16 && p.dtype != SK_F16) {
    err = at(i) + "unknown dtype " + std::to_string(p.dtype);
    return SK_ERR_UNSUPPORTED;
  }
  if (!p.A || !p.B || !p.C) {
    err = at(i) + "null operand pointer";
    return SK_ERR_INVALID_ARG;
  }
  if (p.op == SK_GEMM) {
    if (p.M < 1 || p.N < 1 || p.K < 1) {
      err = at(i) + "GEMM dimensions must be >= 1";
      return SK_ERR_INVALID_ARG;
    }
    if (p.lda < 0 || p.ldb < 0 || p.ldc < 0 || (p.lda && p.lda < p.K) || (p.ldb && p.ldb < p.K) ||
        (p.ldc && p.ldc < p.N)) {
      err = at(i) + "row stride smaller than a row";
      return SK_ERR_INVALID_ARG;
    }
    c = Canon{p.M, p.N, p.K, 0, 0};
  } else if (p.op == SK_CONV2D_NHWC || p.op == SK_CONV2D_NCHW) {
    if (p.Nb < 1 || p.H < 1 || p.Wd < 1 || p.Cin < 1 || p.Cout < 1 || p.R < 1 || p.S < 1 || p.pad_h < 0 ||
        p.pad_w < 0) {
      err = at(i) + "convolution dimensions must be >= 1 and padding >= 0";
      return SK_ERR_INVALID_ARG;
    }
    if (p.stride < 0 || p.stride > 1 << 10) {
      err = at(i) + "stride must be 0 (meaning 1) or 1..1024";
      return SK_ERR_INVALID_ARG;
    }
    const int64_t st = p.stride ? p.stride : 1;
    const int64_t span_h = (int64_t)p.H + 2 * (int64_t)p.pad_h - p.R;
    const int64_t span_w = (int64_t)p.Wd + 2 * (int64_t)p.pad_w - p.S;
    const int64_t Ho = span_h < 0 ? 0 : span_h / st + 1;
    const int64_t Wo = span_w < 0 ? 0 : span_w / st + 1;
    if (Ho < 1 || Wo < 1) {
      err = at(i) + "filter larger than the padded image";
      return SK_ERR_INVALID_ARG;
    }
    if (Ho > 1 << 20 || Wo > 1 << 20) {
      err = at(i) + "image too large";
      return SK_ERR_UNSUPPORTED;
    }
    c = Canon{(int64_t)p.Nb * Ho * Wo, p.Cout, (int64_t)p.R * p.S * p.Cin, (int32_t)Ho, (int32_t)Wo};
  } else {
    err = at(i) + "unknown operator " + std::to_string(p.op);
    return SK_ERR_UNSUPPORTED;
  }
  const int64_t lim = std::numeric_limits<int32_t>::max() / 2;
  if (c.Mg > lim || c.Ng > lim || c.Kg > lim) {
    err = at(i) + "canonical dimension does not fit 31 bits";
    return SK_ERR_UNSUPPORTED;
  }
  return SK_OK;
}

double deadline_key(double d) {
  if (!(d > 0.0) || std::isinf(d)) return std::numeric_limits<double>::infinity();
  return d;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

// Operand bytes the tiles of an operator load ("stream bytes"): what the tile targets are measured in.
// A skinny operator reads its weights once.  An operator in the LDS-tile classes reads, per 128 x BN output
// tile, the 128 + BN operand rows of that tile over the whole reduction: its weight array alone would
// understate its share of a launch by the number of row blocks.
static int64_t stream_bytes(int64_t Mg, int64_t Ng, int64_t Kg, int64_t es, const sk_plan_params &prm) {
  if (Mg <= prm.skinny_max_m) return Ng * Kg * es;
  const int64_t bn = Ng <= 64 ? 64 : 128;
  return ((Mg + 127) / 128) * ((Ng + bn - 1) / bn) * (128 + bn) * Kg * es;
}

// Which accelerator die (XCD: 32 compute units behind one 4 MB L2) runs which LDS tile.  The tiles of an
// operator in the LDS-tile classes share operands: the tiles of one row block read the same 128 activation
// rows, those of one column block the same weight rows.  Handed out in table order they land on all eight
// dies, and every die fetches every panel from memory for itself.  So the output rectangles of such an
// operator are cut into `p` two-dimensional parts (p = 1, 2, 4 or 8: the fewest with at most xcd_part
// rectangles each; the pm x pn grid of parts that fetches the fewest operand rows in total), each part goes to
// one die (the dies with the fewest entries so far, lowest index first), and within a part the rectangles
// follow a Z-order curve in blocks of 8 x 8, so that the handful of tiles a die runs at any one time share panels as well.
// The reduction slices of a rectangle stay together.  The lists name tiles of the table; the table itself,
// and with it the order in which the launch takes LDS tiles up, does not change.
// xcd_part = -1: the planner decides.  The lists pay where the matrix cores, not memory, bound the launch and no
// skinny tile is in it (measured: plans of LDS tiles only gain 0 to 10 % when the sum over operators of
// flops / peak exceeds that of operand bytes / bandwidth, lose 2 to 5 % otherwise, and every plan that mixes in
// skinny tiles loses).  Peaks as the ratio of the datasheet figures (2500 TFLOP/s for 16-bit types, 157.3 for
// fp32, 8 TB/s), so that no device property enters: flops * 2 * (1573 | 25000) against bytes * 983125.
// Then a part is an eighth of all output rectangles of the plan: whole operators per die where there are
// many, an operator's eighths where there is one.
static int64_t resolve_xcd_part(const HostPlan &out, const std::vector<Canon> &canon) {
  if (out.params.xcd_part >= 0) return out.params.xcd_part;
  unsigned __int128 t_flops = 0, t_bytes = 0;
  int64_t rects = 0;
  for (size_t i = 0; i < out.problems.size(); ++i) {
    if (out.count[i] == 0) continue;
    const sk_tile &t0 = out.tiles[(size_t)out.first[i]];
    if (t0.cls != CLS_TILE_128x128 && t0.cls != CLS_TILE_128x64) return 0;  // a skinny operator
    const int64_t bn = t0.cls == CLS_TILE_128x64 ? 64 : 128;
    rects += ((canon[i].Mg + 127) / 128) * ((canon[i].Ng + bn - 1) / bn);
    const unsigned __int128 flops = (unsigned __int128)2 * (uint64_t)canon[i].Mg * (uint64_t)canon[i].Ng * (uint64_t)canon[i].Kg;
    t_flops += flops * 2u * (out.problems[i].dtype == SK_F32 ? 25000u : 1573u);
    t_bytes += (unsigned __int128)(uint64_t)operand_bytes(out.problems[i]) * 983125u;
  }
  if (rects == 0 || t_flops <= t_bytes) return 0;
  return (rects + 7) / 8;
}

static void build_xcd_lists(HostPlan &out, const std::vector<Canon> &canon) {
  out.xorder.clear();
  std::fill(std::begin(out.xoff), std::end(out.xoff), 0u);
  const int64_t part = resolve_xcd_part(out, canon);
  if (part <= 0) return;
  std::vector<uint32_t> lists[8];
  for (const int32_t i : out.order) {
    if (out.count[i] == 0) continue;
    const sk_tile &t0 = out.tiles[(size_t)out.first[i]];
    if (t0.cls != CLS_TILE_128x128 && t0.cls != CLS_TILE_128x64) continue;
    const int64_t bn = t0.cls == CLS_TILE_128x64 ? 64 : 128;
    const int64_t MB = (canon[i].Mg + 127) / 128, NB = (canon[i].Ng + bn - 1) / bn, S = t0.S;
    int64_t p = 1;
    while (p < 8 && MB * NB > p * part) p *= 2;
    // pn parts along the columns: every row block is then fetched by pn dies, every column block by pm
    int64_t pm = 1, pn = 1, best = -1;
    for (int64_t cn = 1; cn <= p; cn *= 2) {
      const int64_t cm = p / cn;
      if (cm > MB || cn > NB) continue;
      const int64_t rows = cn * MB * 128 + cm * NB * bn;
      if (best < 0 || rows < best) best = rows, pm = cm, pn = cn;
    }
    if (best < 0) {  // no such grid (three column blocks and one row block cut in four, say): cut the rows only
      pm = std::min<int64_t>(p, MB);
      pn = 1;
    }
    bool used[8] = {};
    for (int64_t a = 0; a < pm; ++a) {
      for (int64_t b = 0; b < pn; ++b) {
        int die = -1;
        for (int x = 0; x < 8; ++x)
          if (!used[x] && (die < 0 || lists[x].size() < lists[die].size())) die = x;
        used[die] = true;
        const int64_t m_lo = a * MB / pm, m_hi = (a + 1) * MB / pm, n_lo = b * NB / pn, n_hi = (b + 1) * NB / pn;
        // blocks of 8 x 8 rectangles row by row, a Z-order curve inside each block
        for (int64_t bm = m_lo; bm < m_hi; bm += 8) {
          for (int64_t bnn = n_lo; bnn < n_hi; bnn += 8) {
            for (int code = 0; code < 64; ++code) {
              // even bits of the code: column offset, odd bits: row offset
              const int64_t dn = (code & 1) | ((code >> 1) & 2) | ((code >> 2) & 4);
              const int64_t dm = ((code >> 1) & 1) | ((code >> 2) & 2) | ((code >> 3) & 4);
              if (bm + dm >= m_hi || bnn + dn >= n_hi) continue;
              const int64_t rect = (bm + dm) * NB + (bnn + dn);
              for (int64_t ks = 0; ks < S; ++ks) lists[die].push_back((uint32_t)(out.first[i] + rect * S + ks));
            }
          }
        }
      }
    }
  }
  for (int x = 0; x < 8; ++x) {
    out.xoff[x] = (uint32_t)out.xorder.size();
    out.xorder.insert(out.xorder.end(), lists[x].begin(), lists[x].end());
  }
  out.xoff[8] = (uint32_t)out.xorder.size();
}

sk_status plan_host(const sk_problem *problems, int32_t n, const sk_plan_params *params, HostPlan &out,
                    std::string &err) {
  if (n < 0 || (n > 0 && !problems)) {
    err = "problems is null or n < 0";
    return SK_ERR_INVALID_ARG;
  }
  sk_plan_params prm;
  if (params)
    prm = *params;
  else
    sk_plan_params_default(&prm);
  if (prm.skinny_max_m < 0 || prm.skinny_max_m > 64 || prm.tile_bytes_min < 1 ||
      prm.tile_bytes_max < prm.tile_bytes_min || prm.balance_div < 1 || prm.max_groups < 1 ||
      prm.max_groups > 256 || prm.grid_limit < 0 || prm.tail_div < 0 || prm.xcd_part < -1) {
    err = "sk_plan_params field out of range";
    return SK_ERR_INVALID_ARG;
  }
  out = HostPlan{};
  out.params = prm;
  out.problems.assign(problems, problems + n);
  out.dev.resize(n);
  out.first.assign(n, 0);
  out.count.assign(n, 0);

  // ---- canonical view, operand strides, vector-access flags ----
  std::vector<Canon> canon(n);
  int64_t total_w = 0;
  for (int32_t i = 0; i < n; ++i) {
    const sk_problem &p = out.problems[i];
    sk_status st = canonicalise(p, i, canon[i], err);
    if (st != SK_OK) return st;
    const Canon &c = canon[i];
    const int es = elem_size(p.dtype);
    const int ce = 16 / es;  // elements per 16-byte piece
    DevProblem d;
    std::memset(&d, 0, sizeof(d));
    d.A = p.A;
    d.B = p.B;
    d.C = p.C;
    d.Mg = (int32_t)c.Mg;
    d.Ng = (int32_t)c.Ng;
    d.Kg = (int32_t)c.Kg;
    d.dtype = p.dtype;
    if (p.op == SK_GEMM) {
      d.lda = p.lda ? p.lda : p.K;
      d.ldb = p.ldb ? p.ldb : p.K;
      d.ldc = p.ldc ? p.ldc : p.N;
      d.gather = 0;
    } else {
      d.ldb = c.Kg;
      d.ldc = p.Cout;
      d.H = p.H;
      d.W = p.Wd;
      d.Cin = p.Cin;
      d.Ho = c.Ho;
      d.Wo = c.Wo;
      d.R = p.R;
      d.S = p.S;
      d.pad_h = p.pad_h;
      d.pad_w = p.pad_w;
      d.stride = p.stride ? p.stride : 1;
      // a 1x1 filter without padding or stride reads the image as a plain [pixels, Cin] matrix
      d.gather = !(p.R == 1 && p.S == 1 && p.pad_h == 0 && p.pad_w == 0 && d.stride == 1);
      d.lda = p.Cin;
      const FastDiv f_hw = fast_div_of((uint32_t)(c.Ho * c.Wo)), f_wo = fast_div_of((uint32_t)c.Wo);
      const FastDiv f_cin = fast_div_of((uint32_t)p.Cin), f_s = fast_div_of((uint32_t)p.S);
      d.div_hw[0] = f_hw.mul, d.div_hw[1] = f_hw.shift;
      d.div_wo[0] = f_wo.mul, d.div_wo[1] = f_wo.shift;
      d.div_cin[0] = f_cin.mul, d.div_cin[1] = f_cin.shift;
      d.div_s[0] = f_s.mul, d.div_s[1] = f_s.shift;
      if (p.op == SK_CONV2D_NCHW) {
        d.nchw = 1;
        d.gather = 1;  // neither a patch row nor an output row is contiguous in this storage order
      }
    }
    int32_t flags = 0;
    if (d.nchw) {
      // element-wise paths: no 16-byte pieces of the image along the reduction or along an output row
      // (the weights, one contiguous row per output channel in either order, may still be read in pieces)
    } else if (d.gather) {
      if (aligned16(p.A) && p.Cin % ce == 0) flags |= FLAG_VEC_A;
    } else {
      if (aligned16(p.A) && d.lda % ce == 0 && c.Kg % ce == 0) flags |= FLAG_VEC_A;
    }
    if (aligned16(p.B) && d.ldb % ce == 0 && c.Kg % ce == 0) flags |= FLAG_VEC_B;
    if (!d.nchw && (reinterpret_cast<uintptr_t>(p.C) % (4 * es)) == 0 && d.ldc % 4 == 0) flags |= FLAG_VEC_C;
    d.flags = flags;
    out.dev[i] = d;
    total_w += stream_bytes(c.Mg, c.Ng, c.Kg, es, prm);
  }

  // ---- output ranges must be pairwise disjoint ----
  {
    struct Range {
      uintptr_t lo, hi;
      int32_t idx;
    };
    std::vector<Range> r(n);
    for (int32_t i = 0; i < n; ++i) {
      const DevProblem &d = out.dev[i];
      const uintptr_t lo = reinterpret_cast<uintptr_t>(d.C);
      const uint64_t elems = (uint64_t)(d.Mg - 1) * (uint64_t)d.ldc + (uint64_t)d.Ng;
      r[i] = Range{lo, lo + elems * (uint64_t)elem_size(d.dtype), i};
    }
    std::sort(r.begin(), r.end(), [](const Range &a, const Range &b) { return a.lo < b.lo; });
    for (int32_t i = 1; i < n; ++i) {
      if (r[i].lo < r[i - 1].hi) {
        err = "output ranges of problems " + std::to_string(r[i - 1].idx) + " and " + std::to_string(r[i].idx) +
              " overlap";
        return SK_ERR_OVERLAP;
      }
    }
  }

  // ---- target operand bytes per tile ----
  int64_t T = total_w / prm.balance_div;
  T = std::max<int64_t>(prm.tile_bytes_min, std::min<int64_t>(prm.tile_bytes_max, T));
  if (n == 0) T = prm.tile_bytes_min;
  out.target_tile_bytes = T;

  // ---- operator order: earliest deadline first, ties by index ----
  out.order.resize(n);
  std::iota(out.order.begin(), out.order.end(), 0);
  if (prm.edf) {
    std::stable_sort(out.order.begin(), out.order.end(), [&](int32_t a, int32_t b) {
      return deadline_key(out.problems[a].deadline_ms) < deadline_key(out.problems[b].deadline_ms);
    });
  }

  // ---- stream bytes from each position of the order to its end ----
  std::vector<int64_t> remaining(n + 1, 0);
  for (int32_t pos = n - 1; pos >= 0; --pos) {
    const int32_t i = out.order[pos];
    remaining[pos] = remaining[pos + 1] + stream_bytes(canon[i].Mg, canon[i].Ng, canon[i].Kg, elem_size(out.problems[i].dtype), prm);
  }

  // ---- flat table ----
  const int64_t T_all = T;
  uint32_t out_id = 0;
  for (int32_t pos = 0; pos < n; ++pos) {
    const int32_t i = out.order[pos];
    const Canon &c = canon[i];
    const int es = elem_size(out.problems[i].dtype);
    // towards the end of the table the target shrinks with what is left to do
    T = T_all;
    // towards the end of the table the target shrinks with the bytes that remain, but not below eight
    // times the lower clamp (tiles of a few dozen KB are all fixed cost, and a reduction cut to match
    // them ends in dozens of slices)
    if (prm.tail_div > 0)
      T = std::min<int64_t>(T_all, std::max<int64_t>(8 * prm.tile_bytes_min, remaining[pos] / prm.tail_div));
    uint16_t cls;
    int64_t BM, BN;
    int64_t S = 1, slice_len = c.Kg;  // reduction slices per output rectangle and their length
    if (c.Mg <= prm.skinny_max_m) {
      const int rm_code = c.Mg <= 16 ? 0 : (c.Mg <= 32 ? 1 : 2);  // 1, 2 or 4 blocks of 16 activation rows
      const int64_t gb = 32 * c.Kg * es;                          // bytes of one 32-row weight group
      int64_t G;
      if (4 * gb <= T) {
        G = std::min<int64_t>(prm.max_groups, 4 * std::max<int64_t>(1, T / (4 * gb)));
      } else {
        // four groups already exceed the target: cut the reduction into slices of whole chunks
        G = 4;
        const int64_t chunk = (16384 / (16 << rm_code)) / es;  // reduction elements per activation chunk
        const int64_t nchunks = (c.Kg + chunk - 1) / chunk;
        int64_t want = std::min<int64_t>(std::min<int64_t>(nchunks, (4 * gb + T - 1) / T), 255);
        const int64_t per = (nchunks + want - 1) / want;
        S = (nchunks + per - 1) / per;
        slice_len = per * chunk;
      }
      cls = (uint16_t)(3 * rm_code);
      BM = c.Mg;
      BN = 32 * G;
    } else {
      // 128 output columns per tile, or 64 for an operator that has no more than that
      cls = c.Ng <= 64 ? CLS_TILE_128x64 : CLS_TILE_128x128;
      BM = 128;
      BN = c.Ng <= 64 ? 64 : 128;
      // operand bytes of one tile over the whole reduction; far beyond the target: cut the reduction
      const int64_t tb = (BM + BN) * c.Kg * es;
      if (tb > 2 * T) {
        const int64_t chunk = 256;  // reduction elements: whole stages of every element type
        const int64_t nchunks = (c.Kg + chunk - 1) / chunk;
        // a slice hands over 64 KB of partial sums: never shorter than 1024 reduction elements
        int64_t want = std::min<int64_t>(std::min<int64_t>(nchunks, (tb + T - 1) / T), 255);
        want = std::min<int64_t>(want, std::max<int64_t>(1, c.Kg / 1024));
        const int64_t per = (nchunks + want - 1) / want;
        S = (nchunks + per - 1) / per;
        slice_len = per * chunk;
      }
    }
    out.first[i] = (int64_t)out.tiles.size();
    for (int64_t m0 = 0; m0 < c.Mg; m0 += BM) {
      for (int64_t n0 = 0; n0 < c.Ng; n0 += BN) {
        for (int64_t ks = 0; ks < S; ++ks) {
          sk_tile t;
          t.problem = (uint32_t)i;
          t.cls = cls;
          t.ks_idx = (uint8_t)ks;
          t.S = (uint8_t)S;
          t.m0 = (uint32_t)m0;
          t.n0 = (uint32_t)n0;
          t.m_len = (uint16_t)std::min<int64_t>(BM, c.Mg - m0);
          t.n_len = (uint16_t)std::min<int64_t>(BN, c.Ng - n0);
          t.k0 = (uint32_t)(ks * slice_len);
          t.k_len = (uint32_t)std::min<int64_t>(slice_len, c.Kg - ks * slice_len);
          t.out_tile_id = out_id;
          out.tiles.push_back(t);
        }
        if (S > 1) {
          // partial sums of this rectangle: S slices x 4 waves x (2 * rm) accumulators x 64 lanes, 16 bytes each
          // (LDS tiles: S slices x 256 threads x 16 accumulator quads, 8 for the 64-column tile)
          out.ws_off.push_back((uint32_t)out.ws_f32x4);
          out.ws_f32x4 += cls == CLS_TILE_128x128  ? S * 4096
                          : cls == CLS_TILE_128x64 ? S * 2048
                                                   : S * 4 * 2 * ((int64_t)1 << (cls / 3)) * 64;
        } else {
          out.ws_off.push_back(0u);
        }
        ++out_id;
        if (out.tiles.size() > (size_t)1 << 30 || out.ws_f32x4 > ((int64_t)1 << 31)) {
          err = "tile table or split-K workspace too large";
          return SK_ERR_UNSUPPORTED;
        }
      }
    }
    out.count[i] = (int64_t)out.tiles.size() - out.first[i];
    out.dev[i].tile_first = (int32_t)out.first[i];
    out.dev[i].tile_count = (int32_t)out.count[i];
  }
  build_xcd_lists(out, canon);
  return SK_OK;
}

sk_status plan_host_each_alone(const HostPlan &whole, HostPlan &out, std::string &err) {
  const int32_t n = (int32_t)whole.problems.size();
  out = HostPlan{};
  out.params = whole.params;
  out.problems = whole.problems;
  out.dev = whole.dev;
  out.order.resize(n);
  std::iota(out.order.begin(), out.order.end(), 0);
  out.first.assign(n, 0);
  out.count.assign(n, 0);
  out.target_tile_bytes = 0;
  sk_plan_params prm = whole.params;
  prm.host_only = 1;
  uint32_t rect_base = 0;
  for (int32_t i = 0; i < n; ++i) {
    HostPlan one;
    const sk_status st = plan_host(&whole.problems[i], 1, &prm, one, err);
    if (st != SK_OK) return st;
    out.first[i] = (int64_t)out.tiles.size();
    out.count[i] = (int64_t)one.tiles.size();
    for (sk_tile t : one.tiles) {
      t.problem = (uint32_t)i;
      t.out_tile_id += rect_base;
      out.tiles.push_back(t);
    }
    for (uint32_t w : one.ws_off) out.ws_off.push_back(w + (uint32_t)out.ws_f32x4);
    rect_base += (uint32_t)one.ws_off.size();
    out.ws_f32x4 += one.ws_f32x4;
    out.dev[i].tile_first = (int32_t)out.first[i];
    out.dev[i].tile_count = (int32_t)out.count[i];
    if (out.tiles.size() > (size_t)1 << 30 || out.ws_f32x4 > ((int64_t)1 << 31)) {
      err = "tile table or split-K workspace too large";
      return SK_ERR_UNSUPPORTED;
    }
  }
  return SK_OK;
}

// A launch on the stream of the previous launch is ordered behind it by the stream.  On another stream it
// may only go ahead when the previous launch has completed (the caller asks the event).  Inside a stream
// capture nothing can be asked: the launch is recorded, and the graph's replays are the caller's to order.
LaunchLedger::Ask LaunchLedger::before_launch(uintptr_t stream, bool capturing) const {
  if (capturing || !has_event || stream == last_stream) return GO;
  return QUERY_EVENT;
}

void LaunchLedger::after_launch(uintptr_t stream, bool capturing, bool event_recorded) {
  if (capturing || !event_recorded) {
    device_wide = true;  // replays of a graph, or a launch without an event behind it
    return;
  }
  // every earlier eager launch either shares this stream or had completed before this one was admitted:
  // the event behind this launch covers them all
  has_event = true;
  last_stream = stream;
}

LaunchLedger::Wait LaunchLedger::before_destroy() const {
  if (device_wide) return DEVICE;
  return has_event ? EVENT : NOTHING;
}

int64_t operand_bytes(const sk_problem &p) {
  const int64_t es = elem_size(p.dtype);
  if (p.op == SK_GEMM) {
    if (p.M < 1 || p.N < 1 || p.K < 1) return 0;
    return es * ((int64_t)p.M * p.K + (int64_t)p.N * p.K + (int64_t)p.M * p.N);
  }
  if (p.op != SK_CONV2D_NHWC && p.op != SK_CONV2D_NCHW) return 0;
  const int64_t st = p.stride > 0 ? p.stride : 1;
  const int64_t span_h = (int64_t)p.H + 2 * (int64_t)p.pad_h - p.R, span_w = (int64_t)p.Wd + 2 * (int64_t)p.pad_w - p.S;
  if (p.Nb < 1 || p.Cin < 1 || p.Cout < 1 || p.R < 1 || p.S < 1 || span_h < 0 || span_w < 0) return 0;
  const int64_t Ho = span_h / st + 1, Wo = span_w / st + 1;
  return es * ((int64_t)p.Nb * p.H * p.Wd * p.Cin + (int64_t)p.Cout * p.R * p.S * p.Cin + (int64_t)p.Nb * Ho * Wo * p.Cout);
}

double estimate_launch_ms(int64_t bytes, double bytes_per_ms, double floor_ms) {
  const double t = (double)bytes / bytes_per_ms;
  return t > floor_ms ? t : floor_ms;
}

std::vector<size_t> select_batch(const std::vector<QueuedOp> &ops, const std::vector<const void *> &busy, int policy,
                                 double cap_ms, double corr, double bytes_per_ms, double floor_ms) {
  std::vector<size_t> picked;
  if (ops.empty()) return picked;
  if (policy == SK_QUEUE_SEQUENTIAL) {
    // arrival order; one stream keeps launches into one buffer ordered, so a busy output does not hold it back
    picked.push_back(0);
    return picked;
  }
  std::vector<size_t> order(ops.size());
  std::iota(order.begin(), order.end(), (size_t)0);
  std::stable_sort(order.begin(), order.end(),
                   [&](size_t a, size_t b) { return ops[a].deadline_ms < ops[b].deadline_ms; });
  std::unordered_set<const void *> taken;  // outputs of this batch
  int64_t total = 0;
  for (size_t i : order) {
    const void *c = ops[i].C;
    if (std::binary_search(busy.begin(), busy.end(), c) || taken.count(c)) continue;
    if (policy == SK_QUEUE_OOO && !picked.empty() &&
        estimate_launch_ms(total + ops[i].bytes, bytes_per_ms, floor_ms) * corr > cap_ms)
      break;
    picked.push_back(i);
    taken.insert(c);
    total += ops[i].bytes;
  }
  return picked;
}

}  // namespace sk

extern "C" void sk_plan_params_default(sk_plan_params *p) {
  if (!p) return;
  std::memset(p, 0, sizeof(*p));
  p->edf = 1;
  p->stamps = 0;
  p->host_only = 0;
  p->skinny_max_m = 64;
  p->tile_bytes_max = 2048 * 1024;
  p->tile_bytes_min = 32 * 1024;
  p->balance_div = 512;
  p->max_groups = 256;
  p->grid_limit = 0;
  p->tail_div = 384;
  p->xcd_part = -1;
  p->reserved = 0;
}
