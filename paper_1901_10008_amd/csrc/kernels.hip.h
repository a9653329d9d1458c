// Device code of the superkernel (gfx950 / CDNA4 only).
//
// One persistent kernel walks the flat tile table (Section 5.3 of the paper:
// many small kernels repacked into one large execution block).  Every tile
// belongs to one operator in its canonical GEMM view
//     C[Mg,Ng] = A'[Mg,Kg] . Bs[Ng,Kg]^T          (fp32 accumulate)
// with both operands K-contiguous, so a 16-byte piece of a row is at the same
// time one 128-bit load and one MFMA operand (8 halves or 4 floats of K).
//
// Two families of tile code:
//   * skinny (Mg <= 32): weights go HBM -> registers -> MFMA directly; the
//     weight rows are the MFMA's row operand and the few activation rows its
//     column operand, so a lane ends up with four consecutive output columns.
//     The four waves of a workgroup either take different 32-row weight groups
//     or split the reduction (wk = 2, 4) and combine through LDS in fixed order.
//   * LDS tiles (64x128, 128x128): classic staged GEMM, global -> registers ->
//     LDS -> 32x32 MFMA; the activation operand may be gathered on the fly from
//     an NHWC image (implicit GEMM for convolutions).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sk_internal.h"

namespace sk {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Operand pointers reach the kernel through descriptors in memory, so the compiler cannot
// see that they are global addresses; say so explicitly (global_load instead of flat_load).
#define SK_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const T SK_GLOBAL *as_global(const void *p) {
  return (const T SK_GLOBAL *)(uintptr_t)p;
}
template <class T>
__device__ __forceinline__ T SK_GLOBAL *as_global_mut(void *p) {
  return (T SK_GLOBAL *)(uintptr_t)p;
}

constexpr int WG_THREADS = 256;
constexpr int LDS_ROW = 144;                  // 128 bytes of K + 16 bytes of padding (bank spread)
constexpr int LDS_TILE_BYTES = 256 * LDS_ROW;  // 128 activation rows + 128 weight rows

struct KernelArgs {
  uint32_t *counters;   // [0] tiles handed out beyond the first grid-full, [1] finished workgroups
  uint32_t *remaining;  // per operator: tiles not yet retired (null = no stamps)
  uint64_t *stamps;     // [n] completion ticks, [n] = start tick
  uint32_t n_problems;
  uint32_t tile_begin, tile_end;
  uint32_t dynamic;      // 1: tiles come from the atomic counter; 0: static stride over the range
  uint32_t write_start;  // 1: workgroup 0 records the start tick
};

// ---------------------------------------------------------------------------
// element helpers
// ---------------------------------------------------------------------------
template <int DT>
struct Elem;
template <>
struct Elem<SK_F32> {
  static constexpr int ES = 4;
};
template <>
struct Elem<SK_BF16> {
  static constexpr int ES = 2;
};
template <>
struct Elem<SK_F16> {
  static constexpr int ES = 2;
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                    // nearest, ties to even
}
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  _Float16 h = (_Float16)f;  // v_cvt_f16_f32: nearest, ties to even
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}

template <int DT>
__device__ __forceinline__ uint32_t cvt_bits(float f) {
  if constexpr (DT == SK_BF16) return f32_to_bf16_bits(f);
  if constexpr (DT == SK_F16) return f32_to_f16_bits(f);
  return __builtin_bit_cast(uint32_t, f);
}

// Store four consecutive outputs of one row (columns n .. n+3, clipped to n_end).
template <int DT>
__device__ __forceinline__ void store4(void *C, int64_t row_off, int n, int n_end, f32x4 v, bool vec_ok) {
  constexpr int ES = Elem<DT>::ES;
  char SK_GLOBAL *p = as_global_mut<char>(C) + (row_off + n) * ES;
  if (vec_ok && n + 3 < n_end) {
    if constexpr (ES == 4) {
      *(f32x4 SK_GLOBAL *)p = v;
    } else {
      u32x2 o;
      o.x = cvt_bits<DT>(v.x) | (cvt_bits<DT>(v.y) << 16);
      o.y = cvt_bits<DT>(v.z) | (cvt_bits<DT>(v.w) << 16);
      *(u32x2 SK_GLOBAL *)p = o;
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (n + i < n_end) {
        if constexpr (ES == 4)
          ((float SK_GLOBAL *)p)[i] = v[i];
        else
          ((uint16_t SK_GLOBAL *)p)[i] = (uint16_t)cvt_bits<DT>(v[i]);
      }
    }
  }
}

// One 16-byte piece (elements k .. k+CE-1 of a row) read element by element
// with a bound on k: the path for unaligned operands and ragged K.
template <int ES>
__device__ __forceinline__ u32x4 load_piece_scalar(const void *base, int64_t off, int k, int Kg) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if constexpr (ES == 4) {
    const uint32_t SK_GLOBAL *p = as_global<uint32_t>(base) + off;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (k + e < Kg) v[e] = p[e];
  } else {
    const uint16_t SK_GLOBAL *p = as_global<uint16_t>(base) + off;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (k + e < Kg) v[e >> 1] |= (uint32_t)p[e] << (16 * (e & 1));
  }
  return v;
}

template <int ES, bool NT>
__device__ __forceinline__ u32x4 load_piece_vec(const void *base, int64_t off) {
  const u32x4 SK_GLOBAL *p = (const u32x4 SK_GLOBAL *)(as_global<char>(base) + off * ES);
  if constexpr (NT)
    return __builtin_nontemporal_load(p);
  else
    return *p;
}

// Weight piece: row n of Bs[Ng,Kg], elements k .. k+CE-1 (zero beyond Kg).
template <int ES, bool NT>
__device__ __forceinline__ u32x4 fetch_B(const DevProblem &P, int64_t row_off, int k) {
  if (P.flags & FLAG_VEC_B) {
    if (k >= P.Kg) return u32x4{0u, 0u, 0u, 0u};
    return load_piece_vec<ES, NT>(P.B, row_off + k);
  }
  return load_piece_scalar<ES>(P.B, row_off + k, k, P.Kg);
}

// Where row m of the activation operand starts.
struct RowA {
  int64_t base;  // plain: m*lda.  gather: offset of pixel (b, ho-pad_h, wo-pad_w, 0); may be negative
  int hb, wb;    // gather: ho-pad_h, wo-pad_w
};

__device__ __forceinline__ RowA row_of(const DevProblem &P, int m) {
  RowA r;
  if (!P.gather) {
    r.base = (int64_t)m * P.lda;
    r.hb = 0;
    r.wb = 0;
  } else {
    const int hw = P.Ho * P.Wo;
    const int b = m / hw;
    const int rem = m - b * hw;
    const int ho = rem / P.Wo;
    const int wo = rem - ho * P.Wo;
    r.hb = ho - P.pad_h;
    r.wb = wo - P.pad_w;
    r.base = (((int64_t)b * P.H + r.hb) * P.W + r.wb) * P.Cin;
  }
  return r;
}

// Element k of the implicit patch row: k = (r*S + s)*Cin + c  ->  pixel (hb+r, wb+s), channel c.
__device__ __forceinline__ bool patch_offset(const DevProblem &P, const RowA &row, int k, int64_t &off) {
  const int tap = k / P.Cin;
  const int c = k - tap * P.Cin;
  const int r = tap / P.S;
  const int s = tap - r * P.S;
  const int h = row.hb + r, w = row.wb + s;
  off = row.base + ((int64_t)r * P.W + s) * P.Cin + c;
  return (unsigned)h < (unsigned)P.H && (unsigned)w < (unsigned)P.W;
}

// Activation piece: elements k .. k+CE-1 of row `row` of A' (zero beyond Kg and in the padding).
template <int ES>
__device__ __forceinline__ u32x4 fetch_A(const DevProblem &P, const RowA &row, int k) {
  constexpr int CE = 16 / ES;
  if (P.flags & FLAG_VEC_A) {
    if (k >= P.Kg) return u32x4{0u, 0u, 0u, 0u};
    if (!P.gather) return load_piece_vec<ES, false>(P.A, row.base + k);
    int64_t off;
    if (!patch_offset(P, row, k, off)) return u32x4{0u, 0u, 0u, 0u};
    return load_piece_vec<ES, false>(P.A, off);
  }
  if (!P.gather) return load_piece_scalar<ES>(P.A, row.base + k, k, P.Kg);
  u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < CE; ++e) {
    int64_t off;
    if (k + e < P.Kg && patch_offset(P, row, k + e, off)) {
      if constexpr (ES == 4)
        v[e] = as_global<uint32_t>(P.A)[off];
      else
        v[e >> 1] |= (uint32_t)as_global<uint16_t>(P.A)[off] << (16 * (e & 1));
    }
  }
  return v;
}

// ---------------------------------------------------------------------------
// MFMA wrappers: one 16-byte piece per lane and operand.
// 16x16: lane l gives row/column l%16 and K-slot l/16.  32x32: l%32 and l/32.
// The two operands use the same lane -> K-slot map, so which K elements a
// slot really holds does not matter as long as both operands agree.
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void mma16(const u32x4 &a, const u32x4 &b, f32x4 &c) {
  if constexpr (DT == SK_BF16) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0,
                                                0);
  } else if constexpr (DT == SK_F16) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  } else {
    // (whole-vector casts: a bit cast applied to a single vector element reads element 0)
    const f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[j], bf[j], c, 0, 0, 0);
  }
}

template <int DT>
__device__ __forceinline__ void mma32(const u32x4 &a, const u32x4 &b, f32x16 &c) {
  if constexpr (DT == SK_BF16) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0,
                                                0);
  } else if constexpr (DT == SK_F16) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  } else {
    const f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(af[j], bf[j], c, 0, 0, 0);
  }
}

// ---------------------------------------------------------------------------
// skinny tiles
// ---------------------------------------------------------------------------
// A tile is all Mg (<= 16*RM) rows against n_len weight rows, processed in
// groups of 32 weight rows.  Within a reduction block of 8 pieces (128 bytes
// per row) lane slot q = lane/16 owns pieces 2q and 2q+1, so the four slots
// of a row read one full 128-byte line between them.
template <int DT, int RM>
__device__ __forceinline__ void run_skinny(const DevProblem &P, const sk_tile &T, int wk_log2, unsigned char *lds) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;  // reduction elements per block

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r16 = lane & 15, q = lane >> 4;
  const int wk = 1 << wk_log2;
  const int kpart = wave & (wk - 1);
  const int rowlane = wave >> wk_log2;
  const int nrowlanes = 4 >> wk_log2;

  const int n_end = (int)T.n0 + (int)T.n_len;
  const int ngroups = ((int)T.n_len + 31) >> 5;
  const int iters = (ngroups + nrowlanes - 1) / nrowlanes;

  // reduction range of this wave, in whole blocks
  const int kblocks = ((int)T.k_len + KB - 1) / KB;
  const int per = (kblocks + wk - 1) >> wk_log2;
  const int k_lo = (int)T.k0 + kpart * per * KB;
  int k_hi = k_lo + per * KB;
  const int k_stop = (int)T.k0 + (int)T.k_len;
  if (k_hi > k_stop) k_hi = k_stop;

  // activation rows of this lane
  RowA rowa[RM];
  bool m_ok[RM];
#pragma unroll
  for (int mb = 0; mb < RM; ++mb) {
    const int m = mb * 16 + r16;
    m_ok[mb] = m < P.Mg;
    rowa[mb] = row_of(P, m_ok[mb] ? m : 0);
  }
  const bool fast = (P.flags & FLAG_VEC_A) && (P.flags & FLAG_VEC_B) && !P.gather;
  const bool vec_c = (P.flags & FLAG_VEC_C) != 0;

  for (int it = 0; it < iters; ++it) {
    const int g = it * nrowlanes + rowlane;
    const bool active = g < ngroups;
    const int n_base = (int)T.n0 + g * 32;

    f32x4 acc[2][RM];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int mb = 0; mb < RM; ++mb) acc[rb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    if (active) {
      int64_t wrow[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        int n = n_base + rb * 16 + r16;
        if (n >= n_end) n = n_end - 1;  // rows past the edge repeat the last row; never stored
        wrow[rb] = (int64_t)n * P.ldb;
      }
      int k = k_lo;
      if (fast) {
        // whole blocks, aligned operands, plain row-major activations: no predicates at all.
        // Activation rows past Mg repeat row 0; their output columns are never stored.
        const char SK_GLOBAL *wp0 = as_global<char>(P.B) + (wrow[0] + q * 2 * CE) * ES;
        const char SK_GLOBAL *wp1 = as_global<char>(P.B) + (wrow[1] + q * 2 * CE) * ES;
        const char SK_GLOBAL *ap[RM];
#pragma unroll
        for (int mb = 0; mb < RM; ++mb) ap[mb] = as_global<char>(P.A) + (rowa[mb].base + q * 2 * CE) * ES;
        constexpr int U = 2;  // blocks per trip: all loads of a trip are issued before its first MFMA
        const int k_full = k_lo + ((k_hi - k_lo) / (U * KB)) * (U * KB);
        for (; k < k_full; k += U * KB) {
          u32x4 w[U][4], av[U][RM][2];
#pragma unroll
          for (int u = 0; u < U; ++u) {
            const int64_t ko = (int64_t)(k + u * KB) * ES;
            w[u][0] = __builtin_nontemporal_load((const u32x4 SK_GLOBAL *)(wp0 + ko));
            w[u][1] = __builtin_nontemporal_load((const u32x4 SK_GLOBAL *)(wp0 + ko + 16));
            w[u][2] = __builtin_nontemporal_load((const u32x4 SK_GLOBAL *)(wp1 + ko));
            w[u][3] = __builtin_nontemporal_load((const u32x4 SK_GLOBAL *)(wp1 + ko + 16));
#pragma unroll
            for (int mb = 0; mb < RM; ++mb) {
              av[u][mb][0] = *(const u32x4 SK_GLOBAL *)(ap[mb] + ko);
              av[u][mb][1] = *(const u32x4 SK_GLOBAL *)(ap[mb] + ko + 16);
            }
          }
#pragma unroll
          for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mb = 0; mb < RM; ++mb) {
              mma16<DT>(w[u][0], av[u][mb][0], acc[0][mb]);
              mma16<DT>(w[u][1], av[u][mb][1], acc[0][mb]);
              mma16<DT>(w[u][2], av[u][mb][0], acc[1][mb]);
              mma16<DT>(w[u][3], av[u][mb][1], acc[1][mb]);
            }
        }
      }
      // general blocks: ragged K, unaligned operands, gathered activations
      for (; k < k_hi; k += KB) {
        const int kk = k + q * 2 * CE;
        u32x4 w[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          w[rb][0] = fetch_B<ES, true>(P, wrow[rb], kk);
          w[rb][1] = fetch_B<ES, true>(P, wrow[rb], kk + CE);
        }
#pragma unroll
        for (int mb = 0; mb < RM; ++mb) {
          u32x4 a0 = {0u, 0u, 0u, 0u}, a1 = {0u, 0u, 0u, 0u};
          if (m_ok[mb]) {
            a0 = fetch_A<ES>(P, rowa[mb], kk);
            a1 = fetch_A<ES>(P, rowa[mb], kk + CE);
          }
          mma16<DT>(w[0][0], a0, acc[0][mb]);
          mma16<DT>(w[0][1], a1, acc[0][mb]);
          mma16<DT>(w[1][0], a0, acc[1][mb]);
          mma16<DT>(w[1][1], a1, acc[1][mb]);
        }
      }
    }

    if (wk > 1) {
      // combine the reduction parts in fixed order: ((p0 + p1) + p2) + p3
      f32x4 *part = (f32x4 *)lds;  // [wave][2*RM][64 lanes]
      if (kpart != 0) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int mb = 0; mb < RM; ++mb) part[(wave * 2 * RM + rb * RM + mb) * 64 + lane] = acc[rb][mb];
      }
      __syncthreads();
      if (kpart == 0) {
        for (int p = 1; p < wk; ++p) {
#pragma unroll
          for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int mb = 0; mb < RM; ++mb) {
              const f32x4 o = part[((wave + p) * 2 * RM + rb * RM + mb) * 64 + lane];
              acc[rb][mb] += o;
            }
        }
      }
    }

    if (active && kpart == 0) {
      // lane holds, per (rb, mb): row m = mb*16 + lane%16, columns n_base + rb*16 + (lane/16)*4 + 0..3
#pragma unroll
      for (int mb = 0; mb < RM; ++mb) {
        const int m = mb * 16 + r16;
        if (m < P.Mg) {
          const int64_t row_off = (int64_t)m * P.ldc;
#pragma unroll
          for (int rb = 0; rb < 2; ++rb) {
            const int n = n_base + rb * 16 + q * 4;
            if (n < n_end) store4<DT>(P.C, row_off, n, n_end, acc[rb][mb], vec_c);
          }
        }
      }
    }
    if (wk > 1) __syncthreads();  // partials are reused by the next group
  }
}

// ---------------------------------------------------------------------------
// LDS-staged tiles: BM x BN outputs per workgroup, 128 bytes of K per stage
// ---------------------------------------------------------------------------
template <int DT, int BM, int BN, int WAVES_M, int WAVES_N>
__device__ __forceinline__ void run_tile(const DevProblem &P, const sk_tile &T, unsigned char *lds) {
  constexpr int ES = Elem<DT>::ES;
  constexpr int CE = 16 / ES;
  constexpr int KB = 8 * CE;                  // reduction elements per stage
  constexpr int FM = BM / (32 * WAVES_M);     // 32x32 blocks per wave along m
  constexpr int FN = BN / (32 * WAVES_N);     // ... along n
  constexpr int A_ITERS = BM / 32;            // 16-byte pieces per thread per stage, activations
  constexpr int B_ITERS = BN / 32;            // ... weights
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert((BM + BN) * LDS_ROW <= LDS_TILE_BYTES, "tile does not fit the LDS buffer");

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int l32 = lane & 31, half = lane >> 5;

  unsigned char *ldsA = lds;
  unsigned char *ldsB = lds + BM * LDS_ROW;

  const int m0 = (int)T.m0, n0 = (int)T.n0;
  const int m_end = m0 + (int)T.m_len, n_end = n0 + (int)T.n_len;

  // staging map: thread -> piece c of rows (tid/8) + 32*i
  const int c8 = tid & 7;
  const int srow = tid >> 3;
  RowA rowa[A_ITERS];
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    int m = m0 + srow + 32 * i;
    if (m >= m_end) m = m_end - 1;  // rows past the edge repeat the last row; never stored
    rowa[i] = row_of(P, m);
  }
  int64_t wrow[B_ITERS];
#pragma unroll
  for (int i = 0; i < B_ITERS; ++i) {
    int n = n0 + srow + 32 * i;
    if (n >= n_end) n = n_end - 1;
    wrow[i] = (int64_t)n * P.ldb;
  }

  f32x16 acc[FN][FM];
#pragma unroll
  for (int fn = 0; fn < FN; ++fn)
#pragma unroll
    for (int fm = 0; fm < FM; ++fm)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fn][fm][i] = 0.f;

  const int k_begin = (int)T.k0, k_stop = (int)T.k0 + (int)T.k_len;
  u32x4 ra[A_ITERS], rb[B_ITERS];

  auto gload = [&](int kbase) {
    const int k = kbase + c8 * CE;
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) ra[i] = (k < k_stop) ? fetch_A<ES>(P, rowa[i], k) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) rb[i] = (k < k_stop) ? fetch_B<ES, false>(P, wrow[i], k) : u32x4{0u, 0u, 0u, 0u};
  };
  auto lstore = [&]() {
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) *(u32x4 *)(ldsA + (srow + 32 * i) * LDS_ROW + c8 * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) *(u32x4 *)(ldsB + (srow + 32 * i) * LDS_ROW + c8 * 16) = rb[i];
  };

  gload(k_begin);
  for (int kb = k_begin; kb < k_stop; kb += KB) {
    lstore();
    __syncthreads();
    if (kb + KB < k_stop) gload(kb + KB);  // in flight while this stage is multiplied
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int piece = (2 * kk + half) * 16;
      u32x4 fa[FM], fb[FN];
#pragma unroll
      for (int fm = 0; fm < FM; ++fm)
        fa[fm] = *(const u32x4 *)(ldsA + ((wm * FM + fm) * 32 + l32) * LDS_ROW + piece);
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
        fb[fn] = *(const u32x4 *)(ldsB + ((wn * FN + fn) * 32 + l32) * LDS_ROW + piece);
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) mma32<DT>(fb[fn], fa[fm], acc[fn][fm]);
    }
    __syncthreads();
  }

  // lane holds, per (fn, fm): row m = l32, columns 8*(i/4) + 4*half + (i%4)
  const bool vec_c = (P.flags & FLAG_VEC_C) != 0;
#pragma unroll
  for (int fm = 0; fm < FM; ++fm) {
    const int m = m0 + (wm * FM + fm) * 32 + l32;
    if (m < m_end) {
      const int64_t row_off = (int64_t)m * P.ldc;
#pragma unroll
      for (int fn = 0; fn < FN; ++fn) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int n = n0 + (wn * FN + fn) * 32 + 8 * j + 4 * half;
          if (n < n_end) {
            f32x4 v = {acc[fn][fm][4 * j], acc[fn][fm][4 * j + 1], acc[fn][fm][4 * j + 2], acc[fn][fm][4 * j + 3]};
            store4<DT>(P.C, row_off, n, n_end, v, vec_c);
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// dispatch and the persistent shell
// ---------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void run_class(const DevProblem &P, const sk_tile &T, unsigned char *lds) {
  const int cls = T.cls;
  if (cls < 3) {
    run_skinny<DT, 1>(P, T, cls, lds);
  } else if (cls < 6) {
    run_skinny<DT, 2>(P, T, cls - 3, lds);
  } else if (cls == CLS_TILE_64x128) {
    run_tile<DT, 64, 128, 1, 4>(P, T, lds);
  } else {
    run_tile<DT, 128, 128, 2, 2>(P, T, lds);
  }
}

__global__ void __launch_bounds__(WG_THREADS)
    sk_superkernel(const sk_tile *__restrict__ tiles, const DevProblem *__restrict__ probs, KernelArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_TILE_BYTES];
  __shared__ uint32_t s_next[2];

  const int tid = threadIdx.x;
  if (a.write_start && a.stamps && blockIdx.x == 0 && tid == 0) a.stamps[a.n_problems] = wall_clock64();

  uint32_t t = a.tile_begin + blockIdx.x;
  int par = 0;
  while (t < a.tile_end) {
    t = __builtin_amdgcn_readfirstlane(t);
    // ask for the next tile now; the answer is only needed after this one
    uint32_t nxt = 0;
    if (a.dynamic && tid == 0) nxt = a.tile_begin + gridDim.x + atomicAdd(&a.counters[0], 1u);

    const sk_tile T = tiles[t];
    const DevProblem &P = probs[T.problem];
    switch (P.dtype) {
      case SK_BF16: run_class<SK_BF16>(P, T, lds); break;
      case SK_F16: run_class<SK_F16>(P, T, lds); break;
      default: run_class<SK_F32>(P, T, lds); break;
    }

    if (a.remaining) __threadfence();
    if (a.dynamic && tid == 0) s_next[par] = nxt;
    __syncthreads();
    if (a.remaining && tid == 0) {
      // the workgroup that retires an operator's last tile stamps it and re-arms the count
      const uint32_t left = atomicSub(&a.remaining[T.problem], 1u);
      if (left == 1u) {
        a.stamps[T.problem] = wall_clock64();
        a.remaining[T.problem] = (uint32_t)P.tile_count;
      }
    }
    t = a.dynamic ? s_next[par] : t + gridDim.x;
    par ^= 1;
  }

  // the last workgroup to leave re-arms the queue for the next launch
  if (a.dynamic && tid == 0) {
    const uint32_t done = atomicAdd(&a.counters[1], 1u);
    if (done == gridDim.x - 1) {
      a.counters[0] = 0u;
      a.counters[1] = 0u;
      __threadfence();
    }
  }
}

}  // namespace sk
