// Compression of one tile by one wavefront (Section 3.2, Fig. 3(c) compression workflow):
// load -> statistics -> outlier mask -> zero the outliers -> group scale (Eq. 2 / Eq. 3)
// -> quantise, pack, store -> ordered append of the outliers to the (index, value) stream.
//
// The kernel is bound by vector-ALU issue as much as by HBM (about 20 lane-operations per
// element are affordable at 70 % of peak bandwidth), so the common case - a row of 512
// elements without any outlier - is kept to the operations that can not be avoided, and
// everything that only matters when outliers are present sits behind wavefront-uniform
// branches.
#pragma once

#include <type_traits>

#include "adacc_common.hpp"

namespace adacc {

// ------------------------------------------------------------------ small helpers
__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

__device__ __forceinline__ float widen_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float widen_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
// element e (0..7) of an octet held in 4 dwords
#define ADACC_ELEM_F32(oct, e) (((e)&1) ? widen_hi((oct)[(e) >> 1]) : widen_lo((oct)[(e) >> 1]))
#define ADACC_ELEM_MAG(oct, e) ((((e)&1) ? ((oct)[(e) >> 1] >> 16) : (oct)[(e) >> 1]) & 0x7FFFu)

// compile-time loop: body(std::integral_constant<int, J>) for J = 0..N-1.  Used where a
// data-dependent inner loop would otherwise keep the compiler from unrolling, which would
// turn the per-row register arrays into scratch memory.
template <int N, int J = 0, class F>
__device__ __forceinline__ void static_for(F&& body) {
  if constexpr (J < N) {
    body(std::integral_constant<int, J>());
    static_for<N, J + 1>(body);
  }
}

struct OpAdd { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpMin { __device__ __forceinline__ float operator()(float a, float b) const { return fminf(a, b); } };
struct OpUMax { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };
struct OpIMax { __device__ __forceinline__ int32_t operator()(int32_t a, int32_t b) const { return a > b ? a : b; } };
struct OpIMin { __device__ __forceinline__ int32_t operator()(int32_t a, int32_t b) const { return a < b ? a : b; } };

// Order-preserving map between finite floats and signed integers (and back: it is its own
// inverse).  Cross-lane max / min run on these integers: the integer instructions take the
// DPP lane permute as an operand, while a float max would first have to quiet a possible NaN.
__device__ __forceinline__ int32_t float_key(float f) {
  const int32_t u = (int32_t)__float_as_uint(f);
  return u ^ ((u >> 31) & 0x7FFFFFFF);
}
__device__ __forceinline__ float key_float(int32_t k) {
  return __uint_as_float((uint32_t)(k ^ ((k >> 31) & 0x7FFFFFFF)));
}

// value of the partner lane of one xor-butterfly step.  Steps 1..8 are DPP lane permutes
// (they fuse into the arithmetic instruction); 16 and 32 go through the LDS crossbar.
// row_half_mirror / row_mirror stand in for xor 4 / xor 8: after the lower steps every
// value is uniform within its 4 resp. 8 lanes, so reversing the order is the same exchange.
template <int CTRL, class T>
__device__ __forceinline__ T dpp_move(T v) {
  const int i = __builtin_bit_cast(int, v);
  return __builtin_bit_cast(T, __builtin_amdgcn_update_dpp(i, i, CTRL, 0xF, 0xF, true));
}
template <class T>
__device__ __forceinline__ T swap16(T v) {  // lane ^ 16
  return __builtin_bit_cast(T, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
}

// all-reduce over `lanes` adjacent lanes (power of two) by xor butterfly, masks 1, 2, 4, ...
// For sums the association is the balanced binary tree over lane order, which is what makes
// the variance a function of the input bits alone.
template <class T, class Op>
__device__ __forceinline__ T lanes_reduce(T v, int lanes, Op op) {
  if (lanes > 1) v = op(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
  if (lanes > 2) v = op(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
  if (lanes > 4) v = op(v, dpp_move<0x141>(v));  // row_half_mirror
  if (lanes > 8) v = op(v, dpp_move<0x140>(v));  // row_mirror
  if (lanes > 16) v = op(v, swap16(v));
  if (lanes > 32) v = op(v, __shfl_xor(v, 32));
  return v;
}

// s[j] for the first row of every group of R rows <- op over the group's rows (tree order)
template <int E, class T, class Op>
__device__ __forceinline__ void rows_combine(T (&s)[E], int R, Op op) {
#pragma unroll
  for (int r = 1; r < E; r <<= 1) {
    if (r < R) {
#pragma unroll
      for (int j = 0; j < E; j += 2 * r) s[j] = op(s[j], s[j + r]);
    }
  }
}
// copy the group's value from its first row to its other rows
template <int E, class T>
__device__ __forceinline__ void rows_broadcast(T (&s)[E], int R) {
#pragma unroll
  for (int r = E / 2; r >= 1; r >>= 1) {
    if (r < R) {
#pragma unroll
      for (int j = 0; j < E; j += 2 * r) s[j + r] = s[j];
    }
  }
}

// Reduce per-row, per-lane partials over groups of 2^lg elements.  lg <= 9: the group is
// 2^(lg-3) adjacent lanes of one row.  lg > 9: the group is 2^(lg-9) whole rows; rows are
// first reduced over all 64 lanes, then combined pairwise, so that sums follow the
// canonical tree (512-element blocks first, then blocks two by two).
template <int E, class T, class Op>
__device__ __forceinline__ void groups_reduce(T (&s)[E], uint32_t lg, Op op) {
  if (lg <= 9) {
    const int lanes = 1 << (lg - 3);
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = lanes_reduce(s[j], lanes, op);
  } else {
    const int R = 1 << (lg - 9);
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = lanes_reduce(s[j], kWave, op);
    rows_combine<E>(s, R, op);
    rows_broadcast<E>(s, R);
  }
}
// same for an order-free operation: combine the rows in the lane first, one butterfly per group
template <int E, class T, class Op>
__device__ __forceinline__ void groups_reduce_any_order(T (&s)[E], uint32_t lg, Op op) {
  if (lg <= 9) {
    const int lanes = 1 << (lg - 3);
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = lanes_reduce(s[j], lanes, op);
  } else {
    const int R = 1 << (lg - 9);
    rows_combine<E>(s, R, op);
#pragma unroll
    for (int j = 0; j < E; ++j)
      if ((j & (R - 1)) == 0) s[j] = lanes_reduce(s[j], kWave, op);
    rows_broadcast<E>(s, R);
  }
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) v += __shfl_xor(v, m);
  return v;
}

// number of set bits of a wavefront mask in the lanes below this one
__device__ __forceinline__ uint32_t lanes_below(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// ------------------------------------------------------------------ chained scan across tiles
struct ScanCtx {
  uint64_t* state;
  uint32_t tag;         // epoch << 2
  uint32_t spin_limit;  // polls before a wavefront gives up
};

__device__ __forceinline__ uint64_t ld_state(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_state(uint64_t* p, uint32_t hi, uint32_t lo) {
  __hip_atomic_store(p, ((uint64_t)hi << 32) | lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Single-pass scan of outlier counts with decoupled look-back.  The scan unit is a "run": the
// kTilesPerUnit consecutive tiles that one wavefront compresses one after the other.  A run
// publishes its total when it is done (flag "aggregate"), looks back over its predecessors -
// 128 of them per memory round trip, two per lane - adding their totals until it meets a run
// that already knows its inclusive prefix, then publishes its own prefix.  Runs are numbered
// in launch order (workgroup index, wavefront index) and a run only ever waits for
// lower-numbered ones, which the hardware has dispatched earlier.  The poll bound is a second
// line of defence: when it trips, the run publishes "abort", which every later run inherits
// at once, so the kernel always drains and reports the failure in the status words.
__device__ __forceinline__ void scan_publish(const ScanCtx& sc, uint32_t unit, uint32_t flag, uint32_t value) {
  if (lane_id() == 0) st_state(&sc.state[unit], sc.tag | flag, value);
}

// Sum of the totals of runs first..unit-1.
__device__ __forceinline__ uint32_t scan_lookback(const ScanCtx& sc, uint32_t unit, uint32_t first, bool& aborted) {
  const int lane = lane_id();
  aborted = false;
  if (unit == first) return 0;
  uint32_t excl = 0;
  int64_t top = (int64_t)unit - 1;
  while (true) {
    const int64_t pa = top - lane, pb = top - kWave - lane;  // nearer and farther window
    const bool in_a = pa >= (int64_t)first, in_b = pb >= (int64_t)first;
    uint32_t fa = kFlagPrefix, va = 0, fb = kFlagPrefix, vb = 0;  // before the first run: prefix 0
    uint32_t polls = 0;
    uint64_t need_a, need_b;
    bool found;
    while (true) {
      uint64_t wa = 0, wb = 0;
      if (in_a) wa = ld_state(&sc.state[pa]);
      if (in_b) wb = ld_state(&sc.state[pb]);
      if (in_a) {
        const uint32_t hi = (uint32_t)(wa >> 32);
        fa = ((hi & ~3u) == sc.tag) ? (hi & 3u) : (uint32_t)kFlagEmpty;
        va = (uint32_t)wa;
      }
      if (in_b) {
        const uint32_t hi = (uint32_t)(wb >> 32);
        fb = ((hi & ~3u) == sc.tag) ? (hi & 3u) : (uint32_t)kFlagEmpty;
        vb = (uint32_t)wb;
      }
      const uint64_t pm_a = __builtin_amdgcn_ballot_w64(fa >= kFlagPrefix);
      const uint64_t pm_b = __builtin_amdgcn_ballot_w64(fb >= kFlagPrefix);
      if (pm_a) {         // the walk ends in the nearer window
        const int last = __builtin_ctzll(pm_a);
        need_a = (last == kWave - 1) ? ~0ull : ((2ull << last) - 1ull);
        need_b = 0ull;
        found = true;
      } else if (pm_b) {  // all of the nearer window, part of the farther one
        const int last = __builtin_ctzll(pm_b);
        need_a = ~0ull;
        need_b = (last == kWave - 1) ? ~0ull : ((2ull << last) - 1ull);
        found = true;
      } else {
        need_a = need_b = ~0ull;
        found = false;
      }
      const uint64_t empty = (__builtin_amdgcn_ballot_w64(fa == kFlagEmpty) & need_a) |
                             (__builtin_amdgcn_ballot_w64(fb == kFlagEmpty) & need_b);
      if (empty == 0ull) break;
      if (++polls > sc.spin_limit) { aborted = true; break; }
      __builtin_amdgcn_s_sleep(2);
    }
    if (aborted) break;
    if ((__builtin_amdgcn_ballot_w64(fa == kFlagAbort) & need_a) | (__builtin_amdgcn_ballot_w64(fb == kFlagAbort) & need_b)) {
      aborted = true;
      break;
    }
    const uint32_t mine = (((need_a >> lane) & 1ull) ? va : 0u) + (((need_b >> lane) & 1ull) ? vb : 0u);
    excl += wave_sum_u32(mine);
    if (found) break;
    top -= 2 * kWave;
  }
  return excl;
}

// ------------------------------------------------------------------ packing of rounded codes
// t holds integers in [-2^(b-1), 2^(b-1)-1] as floats.  Adding 1.5 * 2^23 puts the integer, in
// two's complement, into the low mantissa bits; the bytes / nibbles are then gathered.
__device__ __forceinline__ uint32_t code_bits(float t) { return __float_as_uint(t + 12582912.0f); }

__device__ __forceinline__ uint32_t pack_bytes4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);  // [a.0, b.0, 0, 0]
  const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
  return ab | (cd << 16);
}
__device__ __forceinline__ uint32_t pack_nibbles8(const uint32_t (&c)[kOct]) {
  uint32_t w = 0u;
#pragma unroll
  for (int e = 0; e < kOct; ++e) w |= (c[e] & 0xFu) << (4 * e);
  return w;
}

// ------------------------------------------------------------------ outlier test of the rows of a tile
struct RowCtx {
  uint64_t numel, lane_base;
  float param;             // ABS: tau
  uint32_t topk_lane_pos;  // TOPK: position of the lane's first element in its group's row
  int topk_rows;           // TOPK: rows per group
};

// For every row j: which elements are outliers (mask[j], bit e = element e), the inlier view
// y[j][*] (outliers, Inf and NaN as zero), the lane's max |y| (symmetric quantisation), the
// number of outliers of the row in lower lanes, and the row's outlier count.  A row without
// outliers - the common case - costs a compare, a select and half a max per element beyond
// the widening; the mask and the positions are only worked out behind a wavefront-uniform branch.
// CHECK_NONFINITE: additionally test every element for Inf / NaN (statistics were poisoned).
template <int MODE, bool ASYM, bool CHECK_NONFINITE, int E>
__device__ __forceinline__ void outlier_rows(const RowCtx& rc, const uint32_t (&raw)[E][4], const float (&limit)[E],
                                             const uint32_t (&kth)[E], float (&y)[E][kOct], float (&amax)[E],
                                             uint32_t (&mask)[E], uint32_t (&lane_excl)[E], uint32_t (&row_cnt)[E]) {
  constexpr float kInf = __builtin_inff();
#pragma unroll
  for (int j = 0; j < E; ++j) {
    float x[kOct];
    bool o[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      x[e] = ADACC_ELEM_F32(raw[j], e);
      if constexpr (MODE == kModeNone) {
        o[e] = !(fabsf(x[e]) < kInf);            // Inf / NaN: nothing is kept aside, the value counts as zero
      } else if constexpr (MODE == kModeAbs) {
        o[e] = !(fabsf(x[e]) <= rc.param);       // |x| > tau, and also Inf / NaN
      } else if constexpr (MODE == kModeStd) {
        o[e] = x[e] * x[e] > limit[j];
      } else {
        const bool valid = (rc.lane_base + (uint64_t)j * kRow) < rc.numel;
        const uint32_t row_pos = ((uint32_t)(j & (rc.topk_rows - 1)) << 9) | rc.topk_lane_pos;
        const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
        o[e] = (key >= kth[j]) && valid;         // rows past the end hold zeros, which TOPK would rank too
      }
      if constexpr (CHECK_NONFINITE) o[e] = o[e] || (ADACC_ELEM_MAG(raw[j], e) >= 0x7F80u);
    }
    // y and the lane's max |y| are computed without a branch (a select and half a max3 per
    // element); only the bookkeeping of rows that do have outliers is conditional
    float am = 0.0f;
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      y[j][e] = o[e] ? 0.0f : x[e];
      if constexpr (!ASYM) am = fmaxf(am, fabsf(y[j][e]));
    }
    amax[j] = am;
    uint64_t b[kOct];
    uint64_t any = 0ull;
#pragma unroll
    for (int e = 0; e < kOct; ++e) { b[e] = __builtin_amdgcn_ballot_w64(o[e]); any |= b[e]; }
    if (any != 0ull) {
      uint32_t m = 0u, below = 0u, cnt = 0u;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        m |= o[e] ? (1u << e) : 0u;
        below += lanes_below(b[e]);
        cnt += (uint32_t)__popcll(b[e]);
      }
      mask[j] = m;
      lane_excl[j] = below;
      row_cnt[j] = cnt;
    } else {
      mask[j] = 0u;
      lane_excl[j] = 0u;
      row_cnt[j] = 0u;
    }
  }
}

// ------------------------------------------------------------------ one tile
// ---- a1: load (16 bytes per lane per row; rows past the end of the tensor read as zero)
template <int E>
__device__ __forceinline__ void load_tile(const TensorDesc& d, uint32_t tile, uint32_t (&raw)[E][4]) {
  const uint64_t lane_base = (uint64_t)tile * (uint64_t)(E * kRow) + (uint64_t)lane_id() * kOct;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint64_t e0 = lane_base + (uint64_t)j * kRow;
    if (e0 < d.numel) {
      const uint4 v = *reinterpret_cast<const uint4*>(d.src + e0);
      raw[j][0] = v.x; raw[j][1] = v.y; raw[j][2] = v.z; raw[j][3] = v.w;
    } else {
      raw[j][0] = raw[j][1] = raw[j][2] = raw[j][3] = 0u;
    }
  }
}

// What a tile leaves behind for the outlier stream.
template <int E>
struct TileOutliers {
  uint32_t mask[E];       // bit e of mask[j]: element e of this lane's octet in row j is an outlier
  uint32_t lane_excl[E];  // outliers of row j in lower lanes
  uint32_t row_off[E];    // outliers of the tile in rows before j (uniform)
  uint32_t row_cnt[E];    // outliers of row j (uniform)
  uint32_t total;         // outliers of the tile (uniform)
};

// ---- a2 .. a8 for one tile: everything except the placement of the outliers in the stream.
template <int MODE, int BITS, bool ASYM, int E>
__device__ __forceinline__ void encode_tile(const TensorDesc& d, uint32_t tile, const uint32_t (&raw)[E][4],
                                            TileOutliers<E>& out) {
  constexpr int Q = 1 << (BITS - 1);
  const int lane = lane_id();
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const uint64_t lane_base = tile_base + (uint64_t)lane * kOct;

  // ---- a2: statistics of the statistics groups
  float limit[E];    // STD: k^2 * var of the row's group
  uint32_t kth[E];   // TOPK: the k-th largest key of the row's group
  bool poisoned = false;  // uniform: some group's statistics met Inf / NaN (or more than k of them)
  uint32_t topk_lane_pos = 0u;
  int topk_rows = 1;
  if constexpr (MODE == kModeStd) {
    float s1[E], s2[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      float x[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) x[e] = ADACC_ELEM_F32(raw[j], e);
      s1[j] = ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
      // squares of bf16 values are exact in binary32
      s2[j] = ((x[0] * x[0] + x[1] * x[1]) + (x[2] * x[2] + x[3] * x[3])) +
              ((x[4] * x[4] + x[5] * x[5]) + (x[6] * x[6] + x[7] * x[7]));
    }
    groups_reduce<E>(s1, d.lgs, OpAdd());
    groups_reduce<E>(s2, d.lgs, OpAdd());
    const float inv_gs = __uint_as_float((127u - d.lgs) << 23);  // 2^-lgs, exact
    const float k2 = d.param;
    bool nan_seen = false;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float mean = s1[j] * inv_gs;
      float var = __fmaf_rn(-mean, mean, s2[j] * inv_gs);
      var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
      limit[j] = k2 * var;
      nan_seen |= (limit[j] != limit[j]);
    }
    // an Inf or NaN anywhere in a group makes its limit NaN; only then is the per-element
    // test for non-finite values needed
    poisoned = __builtin_amdgcn_ballot_w64(nan_seen) != 0ull;
  } else if constexpr (MODE == kModeTopk) {
    // key = magnitude bits above, reversed position in the group below: the k largest keys
    // are the k largest magnitudes with ties going to the lower index; keys are unique.
    const uint32_t lgs = d.lgs;
    topk_rows = (lgs > 9) ? (1 << (lgs - 9)) : 1;
    topk_lane_pos = (lgs > 9) ? ((uint32_t)lane << 3) : (((uint32_t)lane & ((1u << (lgs - 3)) - 1u)) << 3);
#pragma unroll
    for (int j = 0; j < E; ++j) kth[j] = 0xFFFFFFFFu;
    for (uint32_t r = 0; r < d.topk; ++r) {
      uint32_t best[E];
#pragma unroll
      for (int j = 0; j < E; ++j) {
        const uint32_t row_pos = ((uint32_t)(j & (topk_rows - 1)) << 9) | topk_lane_pos;
        uint32_t m = 0u;
#pragma unroll
        for (int e = 0; e < kOct; ++e) {
          const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
          const uint32_t cand = (key < kth[j]) ? key : 0u;
          m = (cand > m) ? cand : m;
        }
        best[j] = m;
      }
      groups_reduce_any_order<E>(best, lgs, OpUMax());
#pragma unroll
      for (int j = 0; j < E; ++j) kth[j] = best[j];
    }
    // if even the k-th largest is Inf / NaN there may be more of them than k: check every element
    bool many = false;
#pragma unroll
    for (int j = 0; j < E; ++j) many |= (kth[j] >> 16) >= 0x7F80u;
    poisoned = __builtin_amdgcn_ballot_w64(many) != 0ull;
  }

  // ---- a3 + a5: outlier test and inlier view y, row by row
  float y[E][kOct];
  float amax[E];        // symmetric: max |y| over the lane's octet
  uint32_t (&mask)[E] = out.mask;
  uint32_t (&lane_excl)[E] = out.lane_excl;
  uint32_t (&row_cnt)[E] = out.row_cnt;
  const RowCtx rc{d.numel, lane_base, d.param, topk_lane_pos, topk_rows};
  if constexpr (MODE == kModeStd || MODE == kModeTopk) {
    // the variant that also tests every element for Inf / NaN is a separate copy of the loop, so
    // that the common one carries no trace of it
    if (poisoned) outlier_rows<MODE, ASYM, true, E>(rc, raw, limit, kth, y, amax, mask, lane_excl, row_cnt);
    else outlier_rows<MODE, ASYM, false, E>(rc, raw, limit, kth, y, amax, mask, lane_excl, row_cnt);
  } else {
    outlier_rows<MODE, ASYM, false, E>(rc, raw, limit, kth, y, amax, mask, lane_excl, row_cnt);
  }

  out.total = 0u;
#pragma unroll
  for (int j = 0; j < E; ++j) { out.row_off[j] = out.total; out.total += row_cnt[j]; }

  // ---- a6: per-group scale (and offset)
  float inv[E], off[E], scl[E];
  if constexpr (!ASYM) {
    uint32_t a[E];  // max |y| as bit patterns: for non-negative floats the integer order is the float order
#pragma unroll
    for (int j = 0; j < E; ++j) a[j] = __float_as_uint(amax[j]);
    groups_reduce_any_order<E>(a, d.lgq, OpUMax());
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float am = __uint_as_float(a[j]);
      scl[j] = am / d.divisor;                                                 // Eq. 2: S = max|X| / D
      inv[j] = (am != 0.0f) ? fminf(d.divisor / am, 3.402823466e+38f) : 0.0f;  // one division per group
      off[j] = 0.0f;
    }
  } else {
    int32_t hi[E], lo[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      float mx = y[j][0], mn = y[j][0];
#pragma unroll
      for (int e = 1; e < kOct; ++e) { mx = fmaxf(mx, y[j][e]); mn = fminf(mn, y[j][e]); }
      hi[j] = float_key(mx); lo[j] = float_key(mn);
    }
    groups_reduce_any_order<E>(hi, d.lgq, OpIMax());
    groups_reduce_any_order<E>(lo, d.lgq, OpIMin());
#pragma unroll
    for (int j = 0; j < E; ++j) {
      // a zero extreme is +0 whatever signs the zeros had
      const float h = key_float(hi[j]) + 0.0f, l = key_float(lo[j]) + 0.0f;
      const float o = (h + l) * 0.5f;                   // Eq. 3: O = (max+min)/2
      const float r = h - l;
      off[j] = o;
      scl[j] = r / d.divisor;                           // Eq. 3: S = (max-min) / D2
      inv[j] = (r != 0.0f) ? fminf(d.divisor / r, 3.402823466e+38f) : 0.0f;
    }
  }

  // ---- a7 + a8: quantise, pack, store codes and scales
  const uint32_t q_lanes_mask = (d.lgq <= 9) ? ((1u << (d.lgq - 3)) - 1u) : 63u;
  const uint32_t q_rows_mask = (d.lgq <= 9) ? 0u : ((1u << (d.lgq - 9)) - 1u);
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint64_t e0 = lane_base + (uint64_t)j * kRow;
    if (e0 >= d.numel) continue;
    uint32_t c[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      float t = ASYM ? (y[j][e] - off[j]) * inv[j] : y[j][e] * inv[j];
      // clip first, then round: the bounds are integers, so this equals round-then-clip
      // ("values greater than 7 are capped at 7"); a NaN lands on the lower bound
      t = fminf(fmaxf(t, (float)(-Q)), (float)(Q - 1));
      c[e] = code_bits(t);  // the addition rounds to nearest, ties to even
    }
    if constexpr (BITS == 8) {
      uint2 w;
      w.x = pack_bytes4(c[0], c[1], c[2], c[3]);
      w.y = pack_bytes4(c[4], c[5], c[6], c[7]);
      *reinterpret_cast<uint2*>(d.codes + e0) = w;
    } else {
      *reinterpret_cast<uint32_t*>(d.codes + (e0 >> 1)) = pack_nibbles8(c);
    }
    if (((uint32_t)lane & q_lanes_mask) == 0u && ((uint32_t)j & q_rows_mask) == 0u) {
      const uint64_t g = e0 >> d.lgq;
      d.scales[g] = scl[j];
      if constexpr (ASYM) d.zp[g] = off[j];
    }
  }

}

// ---- a4: append a tile's outliers, in ascending index order, to `idx_out` / `val_out` starting
// at position pos0 (entries at or past `limit` are dropped).  The destination is either the
// stream in global memory or the wavefront's staging area in LDS.
template <int E, class IdxPtr, class ValPtr>
__device__ __forceinline__ void emit_outliers(const uint32_t (&raw)[E][4], const TileOutliers<E>& out, uint32_t tile,
                                              IdxPtr idx_out, ValPtr val_out, uint32_t pos0, uint32_t limit) {
  const uint32_t lane_first = tile * (uint32_t)(E * kRow) + (uint32_t)lane_id() * kOct;
  static_for<E>([&](auto J) {
    constexpr int j = decltype(J)::value;
    if (out.row_cnt[j] != 0u) {
      uint32_t bits = out.mask[j];
      uint32_t pos = pos0 + out.row_off[j] + out.lane_excl[j];
      const uint32_t i0 = lane_first + (uint32_t)(j * kRow);
      while (bits) {
        const int e = __builtin_ctz(bits);
        bits &= bits - 1u;
        // element e of the octet by shifting (an indexed read would push the octets to scratch)
        const uint64_t half = (e < 4) ? (((uint64_t)raw[j][1] << 32) | raw[j][0]) : (((uint64_t)raw[j][3] << 32) | raw[j][2]);
        if (pos < limit) {
          idx_out[pos] = (int32_t)(i0 + (uint32_t)e);
          val_out[pos] = (uint16_t)(half >> (16 * (e & 3)));
        }
        ++pos;
      }
    }
  });
}

// ------------------------------------------------------------------ one run of tiles (outlier modes)
constexpr int kStageCap = 256;  // outliers a wavefront can hold back in LDS while its offset is unknown
struct WaveStage {
  int32_t idx[kStageCap];
  uint16_t val[kStageCap];
};

// One wavefront compresses the tiles [unit*T, unit*T + T) of a tensor one after the other.  The
// outliers of the run are collected in LDS; when the run is done its total is published, the
// offset of the run in the stream is resolved by look-back, and the staged outliers are
// copied out in one coalesced sweep.  A run whose outliers do not fit the staging area
// resolves its offset early (it only has to wait for lower-numbered runs) and from then on
// appends straight to the stream.
template <int MODE, int BITS, bool ASYM, int E>
__device__ __forceinline__ void compress_run(const TensorDesc& d, uint32_t unit, const ScanCtx& sc, WaveStage* stage) {
  static_assert(MODE != kModeNone, "runs exist for the scan only");
  const int lane = lane_id();
  const uint32_t T = d.tiles_per_unit;
  const uint32_t t0 = unit * T;
  const uint32_t t1 = (t0 + T < d.n_tiles) ? t0 + T : d.n_tiles;
  const uint32_t gunit = d.first_unit + unit;

  bool base_known = false, aborted = false;
  uint32_t excl = 0u;       // outliers of the tensor before this run
  uint32_t run_total = 0u;  // outliers of the run so far
  uint32_t staged = 0u;     // of which are waiting in LDS
  uint32_t tile_off = 0u;   // lane k: outliers of the run before its k-th tile

  uint32_t raw[E][4];
  load_tile<E>(d, t0, raw);
  for (uint32_t t = t0; t < t1; ++t) {
    uint32_t nxt[E][4];
    if (t + 1 < t1) load_tile<E>(d, t + 1, nxt);  // in flight while this tile is encoded

    TileOutliers<E> out;
    encode_tile<MODE, BITS, ASYM, E>(d, t, raw, out);
    if ((uint32_t)lane == t - t0) tile_off = run_total;

    if (out.total != 0u) {
      if (!base_known && staged + out.total > (uint32_t)kStageCap) {
        // no room: find the run's offset now and empty the staging area
        excl = scan_lookback(sc, gunit, d.first_unit, aborted);
        base_known = true;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (!aborted) {
          for (uint32_t i = (uint32_t)lane; i < staged; i += kWave) {
            const uint32_t p = excl + i;
            if (p < d.cap) { d.idx[p] = stage->idx[i]; d.val[p] = stage->val[i]; }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        staged = 0u;
      }
      if (base_known) {
        if (!aborted) emit_outliers<E>(raw, out, t, d.idx, d.val, excl + run_total, d.cap);
      } else {
        emit_outliers<E>(raw, out, t, stage->idx, stage->val, staged, (uint32_t)kStageCap);
        staged += out.total;
      }
      run_total += out.total;
    }
    if (t + 1 < t1) {
#pragma unroll
      for (int j = 0; j < E; ++j) {
        raw[j][0] = nxt[j][0]; raw[j][1] = nxt[j][1]; raw[j][2] = nxt[j][2]; raw[j][3] = nxt[j][3];
      }
    }
  }

  // the run is complete: make its total visible, resolve its offset, publish the prefix
  if (!base_known) {
    scan_publish(sc, gunit, unit == 0u ? kFlagPrefix : kFlagAggregate, run_total);
    excl = scan_lookback(sc, gunit, d.first_unit, aborted);
  }
  if (unit != 0u || base_known) scan_publish(sc, gunit, aborted ? kFlagAbort : kFlagPrefix, excl + run_total);

  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  if (!aborted) {
    for (uint32_t i = (uint32_t)lane; i < staged; i += kWave) {
      const uint32_t p = excl + i;
      if (p < d.cap) { d.idx[p] = stage->idx[i]; d.val[p] = stage->val[i]; }
    }
    if ((uint32_t)lane < t1 - t0) d.tile_ptr[t0 + (uint32_t)lane] = excl + tile_off;
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the staging area is reused by the next run
  if (lane == 0) {
    if (t1 == d.n_tiles) {
      const uint32_t n_out = excl + run_total;
      d.tile_ptr[d.n_tiles] = n_out;
      d.status[0] = n_out;
      d.status[1] = (n_out > d.cap) ? 1u : 0u;
      d.status[3] = 0u;
      if (!aborted) d.status[2] = 0u;
    }
    if (aborted) d.status[2] = 1u;
  }
}

// ------------------------------------------------------------------ one tile without outliers (NONE)
template <int BITS, bool ASYM, int E>
__device__ __forceinline__ void compress_tile_plain(const TensorDesc& d, uint32_t tile) {
  uint32_t raw[E][4];
  load_tile<E>(d, tile, raw);
  TileOutliers<E> out;
  encode_tile<kModeNone, BITS, ASYM, E>(d, tile, raw, out);
  if (tile == 0 && lane_id() == 0) {
    d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
}

}  // namespace adacc
