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

// Tells the compiler that the values may have changed, so that anything derived from them (the
// squares, the keys) is formed again where it is next needed instead of being kept in
// registers across a whole phase: a multiply is one instruction, a live register costs
// occupancy.  No instruction is emitted.
template <int E>
__device__ __forceinline__ void forget_derived(float (&x)[E][kOct]) {
#pragma unroll
  for (int j = 0; j < E; ++j) {
#pragma unroll
    for (int e = 0; e < kOct; ++e) asm volatile("" : "+v"(x[j][e]));
  }
}

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

// all-reduce over LANES adjacent lanes (power of two) by xor butterfly, masks 1, 2, 4, ...
// For sums the association is the balanced binary tree over lane order, which is what makes
// the variance a function of the input bits alone.
template <int LANES, class T, class Op>
__device__ __forceinline__ T lanes_reduce(T v, Op op) {
  if constexpr (LANES > 1) v = op(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
  if constexpr (LANES > 2) v = op(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
  if constexpr (LANES > 4) v = op(v, dpp_move<0x141>(v));  // row_half_mirror
  if constexpr (LANES > 8) v = op(v, dpp_move<0x140>(v));  // row_mirror
  if constexpr (LANES > 16) v = op(v, swap16(v));
  if constexpr (LANES > 32) v = op(v, __shfl_xor(v, 32));
  return v;
}

// s[j] for the first row of every group of R rows <- op over the group's rows (tree order)
template <int E, int R, class T, class Op>
__device__ __forceinline__ void rows_combine(T (&s)[E], Op op) {
#pragma unroll
  for (int r = 1; r < R; r <<= 1) {
#pragma unroll
    for (int j = 0; j < E; j += 2 * r) s[j] = op(s[j], s[j + r]);
  }
}
// copy the group's value from its first row to its other rows
template <int E, int R, class T>
__device__ __forceinline__ void rows_broadcast(T (&s)[E]) {
#pragma unroll
  for (int r = R / 2; r >= 1; r >>= 1) {
#pragma unroll
    for (int j = 0; j < E; j += 2 * r) s[j + r] = s[j];
  }
}

template <int E, int LANES, class T, class Op>
__device__ __forceinline__ void each_row_reduce(T (&s)[E], Op op) {
#pragma unroll
  for (int j = 0; j < E; ++j) s[j] = lanes_reduce<LANES>(s[j], op);
}
// ORDERED: reduce every row over all 64 lanes first, then combine rows pairwise (sums: the
// canonical tree, 512-element blocks first, then blocks two by two).  Otherwise the rows are
// combined in the lane first and only one butterfly per group is needed.
template <int E, int R, bool ORDERED, class T, class Op>
__device__ __forceinline__ void row_groups_reduce(T (&s)[E], Op op) {
  if constexpr (R <= E) {
    if constexpr (ORDERED) {
      each_row_reduce<E, kWave>(s, op);
      rows_combine<E, R>(s, op);
    } else {
      rows_combine<E, R>(s, op);
#pragma unroll
      for (int j = 0; j < E; j += R) s[j] = lanes_reduce<kWave>(s[j], op);
    }
    rows_broadcast<E, R>(s);
  }
}

// Reduce per-row, per-lane partials over groups of 2^lg elements.  lg <= 9: the group is
// 2^(lg-3) adjacent lanes of one row.  lg > 9: the group is 2^(lg-9) whole rows.  The group
// size is a run-time value of the method; one switch selects straight-line code for it, so
// that the butterflies themselves carry no branches.
template <int E, bool ORDERED, class T, class Op>
__device__ __forceinline__ void groups_reduce_impl(T (&s)[E], uint32_t lg, Op op) {
  switch (lg) {
    case 3: break;
    case 4: each_row_reduce<E, 2>(s, op); break;
    case 5: each_row_reduce<E, 4>(s, op); break;
    case 6: each_row_reduce<E, 8>(s, op); break;
    case 7: each_row_reduce<E, 16>(s, op); break;
    case 8: each_row_reduce<E, 32>(s, op); break;
    case 9: each_row_reduce<E, 64>(s, op); break;
    case 10: row_groups_reduce<E, 2, ORDERED>(s, op); break;
    case 11: row_groups_reduce<E, 4, ORDERED>(s, op); break;
    default: row_groups_reduce<E, 8, ORDERED>(s, op); break;
  }
}
template <int E, class T, class Op>
__device__ __forceinline__ void groups_reduce(T (&s)[E], uint32_t lg, Op op) {
  groups_reduce_impl<E, true>(s, lg, op);
}
template <int E, class T, class Op>
__device__ __forceinline__ void groups_reduce_any_order(T (&s)[E], uint32_t lg, Op op) {
  groups_reduce_impl<E, false>(s, lg, op);
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

// ------------------------------------------------------------------ offsets of the runs in the outlier stream
// The scan unit is a "run": the consecutive tiles that one wavefront compresses one after the
// other.  All runs of a launch end at about the same time, so a chain in which every run waits
// for its predecessor's prefix would add one memory round trip per link to the end of the
// kernel.  Instead the totals are summed in two levels, without any chain:
//   state1[u]  total of run u                          (published by run u when it is done)
//   state2[b]  total of block b = runs [64b, 64b+64)   (published by the block's last run,
//              which waits for the 63 others of its block)
// and the offset of run u is the sum of state2 over the blocks before its own plus the sum of
// state1 over the runs before it in its own block: two polls, each one load per lane.
// Runs are numbered in launch order (workgroup index, wavefront index) and a run only ever
// waits for lower-numbered ones, which the hardware has dispatched earlier.  The poll bound is
// a second line of defence: when it trips, the run publishes "abort", which every run that
// polls it inherits, so the kernel always drains and reports the failure in the status words.
struct ScanCtx {
  uint64_t* state1;
  uint64_t* state2;
  uint32_t tag;         // epoch << 2
  uint32_t spin_limit;  // polls before a wavefront gives up
};

__device__ __forceinline__ uint64_t ld_state(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_state(uint64_t* p, uint32_t hi, uint32_t lo) {
  __hip_atomic_store(p, ((uint64_t)hi << 32) | lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void scan_publish(uint64_t* state, uint32_t i, uint32_t tag_flag, uint32_t value) {
  if (lane_id() == 0) st_state(&state[i], tag_flag, value);
}

// Waits until the words state[lo..hi) of this launch are all published and returns the sum of
// their values (0 for an empty range).
__device__ __forceinline__ uint32_t scan_poll_sum(const ScanCtx& sc, const uint64_t* state, uint32_t lo, uint32_t hi,
                                                  bool& aborted) {
  const uint32_t lane = (uint32_t)lane_id();
  uint32_t sum = 0u;
  for (uint32_t i0 = lo; i0 < hi && !aborted; i0 += kWave) {  // uniform
    const uint32_t i = i0 + lane;
    const bool in = i < hi;
    uint32_t flag = kFlagAggregate, value = 0u, polls = 0u;
    while (true) {
      if (in) {
        const uint64_t w = ld_state(&state[i]);
        const uint32_t h = (uint32_t)(w >> 32);
        flag = ((h & ~3u) == sc.tag) ? (h & 3u) : (uint32_t)kFlagEmpty;
        value = (uint32_t)w;
      }
      if (__builtin_amdgcn_ballot_w64(flag == kFlagEmpty) == 0ull) break;
      if (++polls > sc.spin_limit) { aborted = true; break; }
      __builtin_amdgcn_s_sleep(2);
    }
    if (__builtin_amdgcn_ballot_w64(flag == kFlagAbort) != 0ull) aborted = true;
    sum += value;
  }
  return aborted ? 0u : wave_sum_u32(sum);
}

// ------------------------------------------------------------------ rounding and packing of codes
// code = clip(nearest integer of y * inv).  One fused multiply-add with 1.5 * 2^23 rounds the
// exact product to the nearest integer (ties to even) and leaves it, in two's complement, in
// the low mantissa bits; the clip is a median with the two bounds shifted the same way
// ("values greater than 7 are capped at 7"); a NaN lands on the lower bound.
constexpr float kMagic = 12582912.0f;
template <int Q>
__device__ __forceinline__ uint32_t code_bits(float y, float inv) {
  const float r = __fmaf_rn(y, inv, kMagic);
  return __float_as_uint(fminf(fmaxf(r, kMagic - (float)Q), kMagic + (float)(Q - 1)));
}

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

// For every row j: which elements are outliers (mask[j], bit e = element e), the lane's extreme
// values of the inlier view y (outliers, Inf and NaN count as zero), the number of outliers of
// the row in lower lanes, and the row's outlier count.  A row without outliers - the common
// case - costs a compare and half a max per element beyond the widening; the mask, the
// positions and the exact extremes are only worked out behind a wavefront-uniform branch.
// y itself is not kept: the quantisation step forms it again from x and the mask.
// In NONE mode the "outliers" are the Inf / NaN elements: they are zeroed but reported nowhere.
// CHECK_NONFINITE: additionally test every element for Inf / NaN (statistics were poisoned).
// ext0 / ext1: symmetric: ext0 = max |y|.  asymmetric: ext0 = max y, ext1 = min y.
template <int MODE, bool ASYM, bool CHECK_NONFINITE, int E>
__device__ __forceinline__ void outlier_rows(const RowCtx& rc, const float (&xs)[E][kOct], const float (&limit)[E],
                                             const uint32_t (&kth)[E], float (&ext0)[E], float (&ext1)[E],
                                             uint32_t (&mask)[E], uint32_t (&lane_excl)[E], uint32_t (&row_cnt)[E]) {
  constexpr float kInf = __builtin_inff();
#pragma unroll
  for (int j = 0; j < E; ++j) {
    float x[kOct];
    bool o[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      x[e] = xs[j][e];
      if constexpr (MODE == kModeNone) {
        o[e] = !(fabsf(x[e]) < kInf);            // Inf / NaN: nothing is kept aside, the value counts as zero
      } else if constexpr (MODE == kModeAbs) {
        o[e] = !(fabsf(x[e]) <= rc.param);       // |x| > tau, and also Inf / NaN
      } else if constexpr (MODE == kModeStd) {
        o[e] = x[e] * x[e] > limit[j];
      } else {
        const bool valid = (rc.lane_base + (uint64_t)j * kRow) < rc.numel;
        const uint32_t row_pos = ((uint32_t)(j & (rc.topk_rows - 1)) << 9) | rc.topk_lane_pos;
        const uint32_t key = (__float_as_uint(x[e]) & 0x7FFF0000u) | (0xFFFFu - (row_pos | (uint32_t)e));
        o[e] = (key >= kth[j]) && valid;         // rows past the end hold zeros, which TOPK would rank too
      }
      if constexpr (CHECK_NONFINITE) o[e] = o[e] || ((__float_as_uint(x[e]) & 0x7FFFFFFFu) >= 0x7F800000u);
    }
    uint64_t b[kOct];
    uint64_t any = 0ull;
#pragma unroll
    for (int e = 0; e < kOct; ++e) { b[e] = __builtin_amdgcn_ballot_w64(o[e]); any |= b[e]; }
    if (any != 0ull) {
      uint32_t m = 0u, below = 0u, cnt = 0u;
      float y0 = o[0] ? 0.0f : x[0];
      float mx = ASYM ? y0 : fabsf(y0), mn = y0;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        m |= o[e] ? (1u << e) : 0u;
        below += lanes_below(b[e]);
        cnt += (uint32_t)__popcll(b[e]);
        const float ye = o[e] ? 0.0f : x[e];
        if constexpr (ASYM) { mx = fmaxf(mx, ye); mn = fminf(mn, ye); }
        else mx = fmaxf(mx, fabsf(ye));
      }
      mask[j] = m;
      lane_excl[j] = below;
      row_cnt[j] = cnt;
      ext0[j] = mx;
      ext1[j] = mn;
    } else {
      // no outlier in the row, hence every element is finite and y = x
      float mx = ASYM ? x[0] : fabsf(x[0]), mn = x[0];
#pragma unroll
      for (int e = 1; e < kOct; ++e) {
        if constexpr (ASYM) { mx = fmaxf(mx, x[e]); mn = fminf(mn, x[e]); }
        else mx = fmaxf(mx, fabsf(x[e]));
      }
      mask[j] = 0u;
      lane_excl[j] = 0u;
      row_cnt[j] = 0u;
      ext0[j] = mx;
      ext1[j] = mn;
    }
  }
}

// ------------------------------------------------------------------ one tile
// ---- a1: load (16 bytes per lane per row; rows past the end of the tensor read as zero).
// The loads are issued unconditionally (octets past the end re-read the tensor's last octet
// and are blanked afterwards): a load under a branch would make the number of loads in flight
// unknown to the compiler's wait-count bookkeeping, which then waits for the prefetched tile
// together with the current one.
template <int E>
__device__ __forceinline__ void load_tile(const TensorDesc& d, uint32_t tile, uint32_t (&raw)[E][4]) {
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const uint64_t lane_base = tile_base + (uint64_t)lane_id() * kOct;
  const uint64_t last = d.numel - kOct;  // numel is a positive multiple of 8
#pragma unroll
  for (int j = 0; j < E; ++j) {
    uint64_t e0 = lane_base + (uint64_t)j * kRow;
    e0 = e0 < last ? e0 : last;
    const uint4 v = *reinterpret_cast<const uint4*>(d.src + e0);
    raw[j][0] = v.x; raw[j][1] = v.y; raw[j][2] = v.z; raw[j][3] = v.w;
  }
}
// blank the octets of a tile that lie past the end of the tensor (uniform test: only a tensor's last tile)
template <int E>
__device__ __forceinline__ void blank_tail(const TensorDesc& d, uint32_t tile, uint32_t (&raw)[E][4]) {
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  if (tile_base + (uint64_t)(E * kRow) <= d.numel) return;
  const uint64_t lane_base = tile_base + (uint64_t)lane_id() * kOct;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if (lane_base + (uint64_t)j * kRow >= d.numel) raw[j][0] = raw[j][1] = raw[j][2] = raw[j][3] = 0u;
  }
}

// bf16 -> binary32 (exact): the 16 bits become the upper half of the word
template <int E>
__device__ __forceinline__ void widen_tile(const uint32_t (&raw)[E][4], float (&x)[E][kOct]) {
#pragma unroll
  for (int j = 0; j < E; ++j) {
#pragma unroll
    for (int e = 0; e < kOct; ++e) x[j][e] = ADACC_ELEM_F32(raw[j], e);
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
__device__ __forceinline__ void encode_tile(const TensorDesc& d, uint32_t tile, float (&x)[E][kOct],
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
      const float (&r)[kOct] = x[j];
      s1[j] = ((r[0] + r[1]) + (r[2] + r[3])) + ((r[4] + r[5]) + (r[6] + r[7]));
      // squares of bf16 values are exact in binary32
      s2[j] = ((r[0] * r[0] + r[1] * r[1]) + (r[2] * r[2] + r[3] * r[3])) +
              ((r[4] * r[4] + r[5] * r[5]) + (r[6] * r[6] + r[7] * r[7]));
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
          const uint32_t key = (__float_as_uint(x[j][e]) & 0x7FFF0000u) | (0xFFFFu - (row_pos | (uint32_t)e));
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

  // ---- a3 + a5: outlier test row by row; extremes of the inlier view per lane
  forget_derived<E>(x);
  float ext0[E], ext1[E];
  uint32_t (&mask)[E] = out.mask;
  uint32_t (&lane_excl)[E] = out.lane_excl;
  uint32_t (&row_cnt)[E] = out.row_cnt;
  const RowCtx rc{d.numel, lane_base, d.param, topk_lane_pos, topk_rows};
  if constexpr (MODE == kModeStd || MODE == kModeTopk) {
    // the variant that also tests every element for Inf / NaN is a separate copy of the loop, so
    // that the common one carries no trace of it
    if (poisoned) outlier_rows<MODE, ASYM, true, E>(rc, x, limit, kth, ext0, ext1, mask, lane_excl, row_cnt);
    else outlier_rows<MODE, ASYM, false, E>(rc, x, limit, kth, ext0, ext1, mask, lane_excl, row_cnt);
  } else {
    outlier_rows<MODE, ASYM, false, E>(rc, x, limit, kth, ext0, ext1, mask, lane_excl, row_cnt);
  }
  out.total = 0u;
#pragma unroll
  for (int j = 0; j < E; ++j) { out.row_off[j] = out.total; out.total += row_cnt[j]; }

  // ---- a6: per-group scale (and offset).  Cross-lane max / min run on integer images of the floats.
  float inv[E], off[E], scl[E];
  if constexpr (!ASYM) {
    uint32_t a[E];  // max |y| as bit patterns: for non-negative floats the integer order is the float order
#pragma unroll
    for (int j = 0; j < E; ++j) a[j] = __float_as_uint(ext0[j]);
    groups_reduce_any_order<E>(a, d.lgq, OpUMax());
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float am = __uint_as_float(a[j]);
      // Eq. 2: S = max|X| / D.  For a power-of-two D the division is a multiplication by 1/D, same bits
      scl[j] = d.inv_divisor != 0.0f ? am * d.inv_divisor : am / d.divisor;
      inv[j] = (am != 0.0f) ? fminf(d.divisor / am, 3.402823466e+38f) : 0.0f;  // one division per group
      off[j] = 0.0f;
    }
  } else {
    int32_t hi[E], lo[E];
#pragma unroll
    for (int j = 0; j < E; ++j) { hi[j] = float_key(ext0[j]); lo[j] = float_key(ext1[j]); }
    groups_reduce_any_order<E>(hi, d.lgq, OpIMax());
    groups_reduce_any_order<E>(lo, d.lgq, OpIMin());
#pragma unroll
    for (int j = 0; j < E; ++j) {
      // a zero extreme is +0 whatever signs the zeros had
      const float h = key_float(hi[j]) + 0.0f, l = key_float(lo[j]) + 0.0f;
      const float o = (h + l) * 0.5f;                   // Eq. 3: O = (max+min)/2
      const float r = h - l;
      off[j] = o;
      scl[j] = d.inv_divisor != 0.0f ? r * d.inv_divisor : r / d.divisor;  // Eq. 3: S = (max-min) / D2
      inv[j] = (r != 0.0f) ? fminf(d.divisor / r, 3.402823466e+38f) : 0.0f;
    }
  }

  // ---- a7 + a8: quantise, pack, store codes and scales
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint64_t e0 = lane_base + (uint64_t)j * kRow;
    // the inlier view: x, or zero where the mask says so
    float y[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) y[e] = x[j][e];
    if (row_cnt[j] != 0u) {  // uniform
#pragma unroll
      for (int e = 0; e < kOct; ++e) y[e] = ((mask[j] >> e) & 1u) ? 0.0f : y[e];
    }
    uint32_t c[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) c[e] = code_bits<Q>(ASYM ? y[e] - off[j] : y[e], inv[j]);
    // Every lane stores, always: a store under a branch would make the number of stores in flight
    // unknown to the compiler's wait-count bookkeeping, and the wait for the prefetched tile would
    // then also wait for these stores.  Octets past the end of the tensor go to a scrap area in the
    // unused part of the blob's status block; all lanes of a group store their (identical) scale.
    const bool valid = e0 < d.numel;
    unsigned char* scrap = reinterpret_cast<unsigned char*>(d.status) + 64;
    if constexpr (BITS == 8) {
      uint2 w;
      w.x = pack_bytes4(c[0], c[1], c[2], c[3]);
      w.y = pack_bytes4(c[4], c[5], c[6], c[7]);
      *reinterpret_cast<uint2*>(valid ? d.codes + e0 : scrap) = w;
    } else {
      *reinterpret_cast<uint32_t*>(valid ? d.codes + (e0 >> 1) : scrap) = pack_nibbles8(c);
    }
    const uint64_t g = e0 >> d.lgq;
    *(valid ? d.scales + g : reinterpret_cast<float*>(scrap + 16)) = scl[j];
    if constexpr (ASYM) *(valid ? d.zp + g : reinterpret_cast<float*>(scrap + 32)) = off[j];
  }
}

// ---- a4: append a tile's outliers, in ascending index order, to `idx_out` / `val_out` starting
// at position pos0 (entries at or past `limit` are dropped).  The destination is either the
// stream in global memory or the wavefront's staging area in LDS.  Only rows that have
// outliers are visited; the original bf16 pattern is the upper half of the widened value.
template <int E, class IdxPtr, class ValPtr>
__device__ __forceinline__ void emit_outliers(const float (&x)[E][kOct], const TileOutliers<E>& out, uint32_t tile,
                                              IdxPtr idx_out, ValPtr val_out, uint32_t pos0, uint32_t limit) {
  const uint32_t lane_first = tile * (uint32_t)(E * kRow) + (uint32_t)lane_id() * kOct;
  static_for<E>([&](auto J) {
    constexpr int j = decltype(J)::value;
    if (out.row_cnt[j] != 0u) {  // uniform
      const uint32_t bits = out.mask[j];
      uint32_t pos = pos0 + out.row_off[j] + out.lane_excl[j];
      const uint32_t i0 = lane_first + (uint32_t)(j * kRow);
      static_for<kOct>([&](auto Ec) {
        constexpr int e = decltype(Ec)::value;
        if ((bits >> e) & 1u) {
          if (pos < limit) {
            idx_out[pos] = (int32_t)(i0 + (uint32_t)e);
            val_out[pos] = (uint16_t)(__float_as_uint(x[j][e]) >> 16);
          }
          ++pos;
        }
      });
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
  const uint32_t gunit = d.first_unit + unit;                // index into state1
  const uint32_t block = unit / kWave;                       // block of 64 runs, local to the tensor
  const uint32_t gblock0 = d.first_block;                    // index of the tensor's block 0 in state2
  const uint32_t gunit_block0 = d.first_unit + block * kWave;  // first run of this run's block in state1

  bool base_known = false, aborted = false;
  uint32_t in_block = 0u;   // outliers of the runs before this one in its block
  uint32_t excl = 0u;       // outliers of the tensor before this run
  uint32_t run_total = 0u;  // outliers of the run so far
  uint32_t staged = 0u;     // of which are waiting in LDS
  uint32_t tile_off = 0u;   // lane k: outliers of the run before its k-th tile

#ifndef ADACC_PREFETCH
#define ADACC_PREFETCH 1
#endif
  uint32_t raw[E][4];
#if ADACC_PREFETCH
  load_tile<E>(d, t0, raw);
  // Let the first tile arrive before the loop is entered.  Inside the loop the current tile is then
  // complete on every path, and the only wait left is the one for the prefetched tile at the end of
  // an iteration, which the compiler can count exactly (vmcnt(0), other counters untouched).
  __builtin_amdgcn_s_waitcnt(0x0F70);
#endif
  for (uint32_t t = t0; t < t1; ++t) {
#if ADACC_PREFETCH
    // the next tile is in flight while this one is encoded (the run's last tile fetches itself again)
    uint32_t nxt[E][4];
    load_tile<E>(d, (t + 1 < t1) ? t + 1 : t, nxt);
#else
    load_tile<E>(d, t, raw);
#endif

    blank_tail<E>(d, t, raw);
    float x[E][kOct];
    widen_tile<E>(raw, x);
    TileOutliers<E> out;
    encode_tile<MODE, BITS, ASYM, E>(d, t, x, out);
    if ((uint32_t)lane == t - t0) tile_off = run_total;

    if (out.total != 0u) {
      if (!base_known && staged + out.total > (uint32_t)kStageCap) {
        // no room: find the run's offset now (this waits for every earlier run) and empty the staging area
        in_block = scan_poll_sum(sc, sc.state1, gunit_block0, gunit, aborted);
        excl = in_block + scan_poll_sum(sc, sc.state2, gblock0, gblock0 + block, aborted);
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
        if (!aborted) emit_outliers<E>(x, out, t, d.idx, d.val, excl + run_total, d.cap);
        // rare path with a data-dependent number of stores: drain it, so that the common path's
        // wait counts stay exact
        __builtin_amdgcn_s_waitcnt(0);
      } else {
        emit_outliers<E>(x, out, t, stage->idx, stage->val, staged, (uint32_t)kStageCap);
        staged += out.total;
      }
      run_total += out.total;
    }
#if ADACC_PREFETCH
#pragma unroll
    for (int j = 0; j < E; ++j) {
      raw[j][0] = nxt[j][0]; raw[j][1] = nxt[j][1]; raw[j][2] = nxt[j][2]; raw[j][3] = nxt[j][3];
    }
#endif
  }

  // the run is complete: make its total visible, then find its offset in the stream
  scan_publish(sc.state1, gunit, sc.tag | (aborted ? kFlagAbort : kFlagAggregate), run_total);
  if (!base_known) {
    in_block = scan_poll_sum(sc, sc.state1, gunit_block0, gunit, aborted);
    excl = in_block;
    if (!aborted) excl += scan_poll_sum(sc, sc.state2, gblock0, gblock0 + block, aborted);
  }
  if ((unit % kWave) == kWave - 1)  // last run of a full block: close the block
    scan_publish(sc.state2, gblock0 + block, sc.tag | (aborted ? kFlagAbort : kFlagAggregate), in_block + run_total);
  if (aborted) scan_publish(sc.state1, gunit, sc.tag | kFlagAbort, 0u);

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
  blank_tail<E>(d, tile, raw);
  float x[E][kOct];
  widen_tile<E>(raw, x);
  TileOutliers<E> out;
  encode_tile<kModeNone, BITS, ASYM, E>(d, tile, x, out);
  if (tile == 0 && lane_id() == 0) {
    d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
}

}  // namespace adacc
