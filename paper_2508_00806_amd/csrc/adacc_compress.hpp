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
#include "adacc_dtype.hpp"

namespace adacc {
namespace ADACC_DT_NS {

// ------------------------------------------------------------------ small helpers
__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

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

// maximum over the whole wavefront, returned in a scalar register: four butterfly steps inside
// the rows of 16 lanes, two row broadcasts (lane 15 of rows 0 and 2 into rows 1 and 3, then
// lane 31 into rows 2 and 3), and lane 63 holds the result
__device__ __forceinline__ uint32_t wave_max_u32_scalar(uint32_t v) {
  v = lanes_reduce<16>(v, OpUMax());
  // rows that receive nothing read 0, the identity of the maximum, so each step is one instruction
  int t = __builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  v = OpUMax()(v, (uint32_t)t);
  t = __builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);      // row_bcast:31
  v = OpUMax()(v, (uint32_t)t);
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// number of set bits of a wavefront mask in the lanes below this one
__device__ __forceinline__ uint32_t lanes_below(uint64_t m) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// ------------------------------------------------------------------ rounding and packing of codes
// code = clip(nearest integer of the binary32 product y * inv) (Eq. 2 / Eq. 3).  The product is
// rounded to binary32 by the multiplication (never fused with what follows: the library is built
// with contraction off); adding 1.5 * 2^23 then rounds it to the nearest integer (ties to even)
// and leaves that integer, in two's complement, in the low mantissa bits; the clip is a median
// with the two bounds shifted the same way ("values greater than 7 are capped at 7"); a NaN
// lands on the lower bound.
// Symmetric codes need the upper bound only: |y| <= max and inv = RN(D / max) (or less, when that was cut
// to the largest finite value) give |y * inv| <= D * (1 + 2^-24), which rounds to at most D <= Q in
// magnitude, -Q is a code, and neither factor can be a NaN or infinite.  (Asymmetric codes keep both
// bounds: a group of huge values can make O infinite and the product a NaN.)
constexpr float kMagic = 12582912.0f;
template <int Q, bool BOTH_BOUNDS = true>
__device__ __forceinline__ uint32_t code_bits(float y, float inv) {
  const float p = __fmul_rn(y, inv);
  const float r = __fadd_rn(p, kMagic);
  if constexpr (BOTH_BOUNDS) return __float_as_uint(fminf(fmaxf(r, kMagic - (float)Q), kMagic + (float)(Q - 1)));
  else return __float_as_uint(fminf(r, kMagic + (float)(Q - 1)));
}

__device__ __forceinline__ uint32_t pack_bytes4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  const uint32_t ab = __builtin_amdgcn_perm(b, a, 0x0c0c0400u);  // [a.0, b.0, 0, 0]
  const uint32_t cd = __builtin_amdgcn_perm(d, c, 0x0c0c0400u);
  return ab | (cd << 16);
}
// 8 codes -> 8 nibbles, element e in nibble e: the even and the odd elements are gathered
// byte-wise first, then one shift and one bit-select interleave them.
__device__ __forceinline__ uint32_t pack_nibbles8(const uint32_t (&c)[kOct]) {
  const uint32_t even = pack_bytes4(c[0], c[2], c[4], c[6]);
  const uint32_t odd = pack_bytes4(c[1], c[3], c[5], c[7]);
  return (even & 0x0F0F0F0Fu) | ((odd << 4) & 0xF0F0F0F0u);
}

// ------------------------------------------------------------------ tile geometry, loads and stores
// A tile is addressed as a wavefront-uniform base (kept in scalar registers) plus a 32-bit
// lane offset, so that address arithmetic costs no vector instructions.
// STRIP: the E rows of 512 elements are not adjacent in memory but `stride` elements apart (rows of a
// matrix: a strip of 512 columns); such a tile is always complete, and base, stride are multiples of 512.
template <int E, bool STRIP = false>
struct TileGeo {
  uint64_t base;      // uniform: index of the tile's first element
  uint32_t rem;       // uniform: elements of the tensor from `base` on, at most E*512 (a multiple of 8, > 0)
  uint32_t lane_off;  // lane * 8
  bool full;          // uniform: rem == E*512
  uint32_t stride;    // uniform, STRIP only: elements from one row to the next
  __device__ __forceinline__ uint32_t row_offset(int j) const {
    if constexpr (STRIP) return (uint32_t)j * stride;
    else return (uint32_t)(j * kRow);
  }
};
// COMPLETE: the caller knows that every tile of the tensor is complete (the tile is a statistics
// group, and group sizes divide the tensor), so nothing about short tiles is computed or tested.
template <int E, bool COMPLETE = false>
__device__ __forceinline__ TileGeo<E> tile_geo(const TensorDesc& d, uint32_t tile) {
  TileGeo<E> g;
  g.base = (uint64_t)tile * (uint64_t)(E * kRow);
  g.lane_off = (uint32_t)lane_id() * kOct;
  g.stride = (uint32_t)kRow;
  if constexpr (COMPLETE) {
    g.rem = (uint32_t)(E * kRow);
    g.full = true;
  } else {
    const uint64_t left = d.numel - g.base;
    g.rem = left < (uint64_t)(E * kRow) ? (uint32_t)left : (uint32_t)(E * kRow);
    g.full = g.rem == (uint32_t)(E * kRow);
  }
  return g;
}

// ---- a1: load (16 bytes per lane per row).  The loads are issued unconditionally (octets past
// the end of the tensor re-read its last octet and are blanked afterwards): a load under a
// branch would make the number of loads in flight unknown to the compiler's wait-count
// bookkeeping, which then waits for the prefetched tile together with the current one.
template <int E, bool COMPLETE = false>
__device__ __forceinline__ void load_tile(const TensorDesc& d, uint32_t tile, uint32_t (&raw)[E][4]) {
  const TileGeo<E> g = tile_geo<E, COMPLETE>(d, tile);
  const uint16_t* sp = d.src + g.base;
  const uint32_t last = g.rem - kOct;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    uint32_t off = g.lane_off + (uint32_t)(j * kRow);
    if constexpr (!COMPLETE) off = off < last ? off : last;
    const uint4 v = ADACC_LOAD16(sp + off);
    raw[j][0] = v.x; raw[j][1] = v.y; raw[j][2] = v.z; raw[j][3] = v.w;
  }
}
// blank the octets of a tile that lie past the end of the tensor (only a tensor's last tile can have any)
template <int E>
__device__ __forceinline__ void blank_tail(const TileGeo<E>& g, uint32_t (&raw)[E][4]) {
  if (g.full) return;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if (g.lane_off + (uint32_t)(j * kRow) >= g.rem) raw[j][0] = raw[j][1] = raw[j][2] = raw[j][3] = 0u;
  }
}

// Makes the compiler forget everything it derived from the raw octets (their values do not
// change).  Between two phases that both widen the octets this keeps the 8 widened values per
// row from staying in registers all the way: forming them again costs one instruction each,
// keeping them costs a quarter of the wavefronts a SIMD can hold.
template <int E>
__device__ __forceinline__ void forget_derived(const uint32_t (&raw)[E][4]) {
  uint32_t(&r)[E][4] = const_cast<uint32_t(&)[E][4]>(raw);
#pragma unroll
  for (int j = 0; j < E; ++j) {
    asm volatile("" : "+v"(r[j][0]), "+v"(r[j][1]), "+v"(r[j][2]), "+v"(r[j][3]));
  }
}

// 16-bit format -> binary32 (exact)
__device__ __forceinline__ void widen_row(const uint32_t (&oct)[4], float (&x)[kOct]) {
#pragma unroll
  for (int e = 0; e < kOct; ++e) x[e] = ADACC_ELEM_F32(oct, e);
}

// ---- a8: store the codes of one octet and the scale (offset) of its group.  Every lane stores,
// always: a store under a branch would make the number of stores in flight unknown to the
// compiler's wait-count bookkeeping, and the wait for the prefetched tile would then also wait
// for these stores.  In a tensor's last tile, octets past the end go to a scrap area in the
// unused part of the blob's status block; all lanes of a group store their (identical) scale.
template <int BITS, bool ASYM, int E, bool STRIP>
__device__ __forceinline__ void store_row(const TensorDesc& d, const TileGeo<E, STRIP>& g, int j,
                                          const uint32_t (&c)[kOct], float scl, float off) {
  // The lane's offset is formed here, per row, from a copy the compiler knows nothing about: else it
  // prepares the offsets (and the group numbers) of all rows ahead of the first row, for every
  // group size the caller can be asked for, and keeps them in registers.
  uint32_t lane_off = g.lane_off;
  asm volatile("" : "+v"(lane_off));
  const uint32_t eo = lane_off + g.row_offset(j);  // element offset from the tile's first element
  unsigned char* cp = d.codes + g.base * BITS / 8;       // uniform
  float* sp = d.scales + (g.base >> d.lgq);                // uniform
  const uint32_t gl = eo >> d.lgq;
  uint2 w8;
  uint32_t w4 = 0u;
  if constexpr (BITS == 8) {
    w8.x = pack_bytes4(c[0], c[1], c[2], c[3]);
    w8.y = pack_bytes4(c[4], c[5], c[6], c[7]);
  } else {
    w4 = pack_nibbles8(c);
  }
  if (g.full) {
    if constexpr (BITS == 8) ADACC_STORE8(cp + eo, w8);
    else ADACC_STORE4(cp + (eo >> 1), w4);
    sp[gl] = scl;
    if constexpr (ASYM) (d.zp + (g.base >> d.lgq))[gl] = off;
  } else {
    const bool valid = eo < g.rem;
    unsigned char* scrap = reinterpret_cast<unsigned char*>(d.status) + 64;
    if constexpr (BITS == 8) ADACC_STORE8(valid ? cp + eo : scrap, w8);
    else ADACC_STORE4(valid ? cp + (eo >> 1) : scrap, w4);
    *(valid ? sp + gl : reinterpret_cast<float*>(scrap + 16)) = scl;
    if constexpr (ASYM) *(valid ? d.zp + (g.base >> d.lgq) + gl : reinterpret_cast<float*>(scrap + 32)) = off;
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
  uint32_t sparse;        // bit j: no lane holds more than one outlier of row j (uniform)
};

// ------------------------------------------------------------------ per-row pieces shared by both tile encoders
constexpr float kFltMax = 3.402823466e+38f;

// STD: limit = k^2 * var from the group's sums (population variance about the mean).
__device__ __forceinline__ float std_limit(float s1, float s2, float inv_gs, float k2) {
  const float mean = s1 * inv_gs;
  float var = __fmaf_rn(-mean, mean, s2 * inv_gs);
  var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
  return k2 * var;
}

// Bookkeeping of one row from the ballots of its 8 outlier tests: per-lane mask, number of the
// row's outliers in lower lanes, row count.  Only rows that have outliers do the work, and the
// usual such row - a few outliers, no two in one lane - does it mostly in scalar registers:
// the ballots live there, and a lane reads its own bit back as a select condition.
__device__ __forceinline__ void row_bookkeeping(const uint64_t (&b)[kOct], uint32_t& mask, uint32_t& lane_excl,
                                                uint32_t& row_cnt, bool& any_out, bool& sparse) {
  uint64_t any = 0ull;
#pragma unroll
  for (int e = 0; e < kOct; ++e) any |= b[e];
  any_out = any != 0ull;
  sparse = true;
  if (any_out) {
    uint32_t cnt = 0u;
#pragma unroll
    for (int e = 0; e < kOct; ++e) cnt += (uint32_t)__popcll(b[e]);
    row_cnt = cnt;
    sparse = cnt == (uint32_t)__popcll(any);
    uint32_t m = 0u;
    if (sparse) {
      lane_excl = lanes_below(any);
#pragma unroll
      for (int e = 0; e < kOct; ++e) m = __builtin_amdgcn_inverse_ballot_w64(b[e]) ? (1u << e) : m;  // at most one bit per lane
    } else {
      uint32_t below = 0u;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        m |= __builtin_amdgcn_inverse_ballot_w64(b[e]) ? (1u << e) : 0u;
        below += lanes_below(b[e]);
      }
      lane_excl = below;
    }
    mask = m;
  } else {
    mask = 0u; lane_excl = 0u; row_cnt = 0u;
  }
}
// extremes of the inlier view of one octet: symmetric ext0 = max |y|; asymmetric ext0 = max y, ext1 = min y
template <bool ASYM>
__device__ __forceinline__ void row_extremes(const float (&y)[kOct], float& ext0, float& ext1) {
  float mx = ASYM ? y[0] : fabsf(y[0]), mn = y[0];
#pragma unroll
  for (int e = 1; e < kOct; ++e) {
    if constexpr (ASYM) { mx = fmaxf(mx, y[e]); mn = fminf(mn, y[e]); }
    else mx = fmaxf(mx, fabsf(y[e]));
  }
  ext0 = mx; ext1 = mn;
}

// ---- a6: scale, reciprocal and offset of a group from its reduced extremes (Eq. 2 / Eq. 3)
template <bool ASYM>
__device__ __forceinline__ void group_scale(const TensorDesc& d, uint32_t r0, int32_t k0, int32_t k1, float& scl,
                                            float& inv, float& off) {
  if constexpr (!ASYM) {
    const float am = __uint_as_float(r0);
    // Eq. 2: S = max|X| / D.  For a power-of-two D the division is a multiplication by 1/D, same bits
    scl = d.inv_divisor != 0.0f ? am * d.inv_divisor : am / d.divisor;
    inv = (am != 0.0f) ? fminf(d.divisor / am, kFltMax) : 0.0f;  // one division per group
    off = 0.0f;
  } else {
    // a zero extreme is +0 whatever signs the zeros had
    const float h = key_float(k0) + 0.0f, l = key_float(k1) + 0.0f;
    off = (h + l) * 0.5f;  // Eq. 3: O = (max+min)/2
    const float r = h - l;
    scl = d.inv_divisor != 0.0f ? r * d.inv_divisor : r / d.divisor;  // Eq. 3: S = (max-min) / D2
    inv = (r != 0.0f) ? fminf(d.divisor / r, kFltMax) : 0.0f;
  }
}

template <int MODE>
__device__ __forceinline__ bool outlier_test(float x, float param_or_limit) {
  if constexpr (MODE == kModeNone) return !(fabsf(x) < __builtin_inff());  // Inf / NaN: zeroed, reported nowhere
  else if constexpr (MODE == kModeAbs) return !(fabsf(x) <= param_or_limit);  // |x| > tau, and also Inf / NaN
  else return x * x > param_or_limit;                                         // STD
}
__device__ __forceinline__ bool is_nonfinite(float x) { return (__float_as_uint(x) & 0x7FFFFFFFu) >= 0x7F800000u; }

// ---- a4: where the outliers of a tile go.  Entry `pos` of the stream of the blob (two arrays) ...
struct StreamSink {
  int32_t* idx;
  uint16_t* val;
  __device__ __forceinline__ void operator()(uint32_t pos, uint32_t index, uint32_t bits) const {
    idx[pos] = (int32_t)index;
    val[pos] = (uint16_t)bits;
  }
};
// ... or of a tile's slot in the workspace (one 8-byte record per entry: index, value) ...
struct SlotSink {
  uint2* rec;
  __device__ __forceinline__ void operator()(uint32_t pos, uint32_t index, uint32_t bits) const {
    rec[pos] = make_uint2(index, bits);
  }
};
// ... or nowhere (tiles without outliers)
struct NullSink {
  __device__ __forceinline__ void operator()(uint32_t, uint32_t, uint32_t) const {}
};

// The outliers of one row, in ascending index order, to positions pos_row, pos_row + 1, ... of the
// sink (entries at or past `limit` are dropped).  mask: this lane's outliers among its 8 elements;
// lane_excl: the row's outliers in lower lanes; sparse (uniform): no lane holds more than one;
// i0: flat index of the lane's first element of the row.
template <class Sink>
__device__ __forceinline__ void emit_row(const uint32_t (&oct)[4], uint32_t mask, uint32_t lane_excl, bool sparse,
                                         uint32_t i0, const Sink& sink, uint32_t pos_row, uint32_t limit) {
  uint32_t pos = pos_row + lane_excl;
  if (sparse) {
    if (mask != 0u && pos < limit) {
      const uint32_t e = (uint32_t)__builtin_ctz(mask);
      const uint64_t lo = ((uint64_t)oct[1] << 32) | oct[0], hi = ((uint64_t)oct[3] << 32) | oct[2];
      const uint64_t half = (e & 4u) ? hi : lo;
      sink(pos, i0 + e, (uint32_t)(half >> ((e & 3u) * 16u)) & 0xFFFFu);
    }
  } else {
    static_for<kOct>([&](auto Ec) {
      constexpr int e = decltype(Ec)::value;
      if ((mask >> e) & 1u) {
        if (pos < limit) sink(pos, i0 + (uint32_t)e, (e & 1) ? (oct[e >> 1] >> 16) : (oct[e >> 1] & 0xFFFFu));
        ++pos;
      }
    });
  }
}

// the outliers of a whole tile whose bookkeeping was kept (general encoder); only rows that have any are visited
template <int E, class Sink>
__device__ __forceinline__ void emit_outliers(const uint32_t (&raw)[E][4], const TileOutliers<E>& out, uint32_t tile,
                                              const Sink& sink, uint32_t pos0, uint32_t limit) {
  const uint32_t lane_first = tile * (uint32_t)(E * kRow) + (uint32_t)lane_id() * kOct;
  static_for<E>([&](auto J) {
    constexpr int j = decltype(J)::value;
    if (out.row_cnt[j] != 0u)  // uniform
      emit_row(raw[j], out.mask[j], out.lane_excl[j], ((out.sparse >> j) & 1u) != 0u, lane_first + (uint32_t)(j * kRow),
               sink, pos0 + out.row_off[j], limit);
  });
}

// ------------------------------------------------------------------ rows without outliers
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t,
                            __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, a), __builtin_bit_cast(u16x2_t, b)));
}

// zero the elements of an octet that `mask` names (bit e: element e)
__device__ __forceinline__ void clear_elements(uint32_t (&oct)[4], uint32_t mask) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe((int)mask, 2 * k, 1);  // 0 or all ones
    const uint32_t hi = (uint32_t)__builtin_amdgcn_sbfe((int)mask, 2 * k + 1, 1);
    oct[k] &= ~((lo & 0x0000FFFFu) | (hi & 0xFFFF0000u));
  }
}

// largest magnitude (15 low bits of the patterns) among the 8 elements of an octet
__device__ __forceinline__ uint32_t octet_magnitude(const uint32_t (&oct)[4]) {
  constexpr uint32_t kMag2 = 0x7FFF7FFFu;
  const uint32_t m = pk_max_u16(pk_max_u16(oct[0] & kMag2, oct[1] & kMag2), pk_max_u16(oct[2] & kMag2, oct[3] & kMag2));
  const uint32_t hi = m >> 16, lo = m & 0xFFFFu;
  return hi > lo ? hi : lo;
}

// a6, symmetric, for a row free of outliers and of values that are not finite: S and D / max from
// the group's largest magnitude (`am_bits`: its binary32 bits; it has at most 11 significant bits).
// For the paper's divisor, a power of two, D / max needs no division sequence: the hardware
// reciprocal is within one unit in the last place, and for an operand of 11 significant bits one
// Newton step then gives the correctly rounded 1 / max (verified for every significand and every
// such starting value); the factor D is exact.  Outside 2^-100 .. 2^100 (where the reciprocal, or
// D / max, leaves the normal range) and for other divisors the division is carried out.
__device__ __forceinline__ void scale_sym_clean(const TensorDesc& d, uint32_t am_bits, float& scl, float& inv) {
  const float am = __uint_as_float(am_bits);
  const bool mid = am_bits - 0x0D800000u <= 0x71800000u - 0x0D800000u;  // 2^-100 <= max <= 2^100
  const bool hard = !mid && am_bits != 0u;
  if ((d.pow2_divisor != 0u) & (__builtin_amdgcn_ballot_w64(hard) == 0ull)) {  // uniform
    scl = am * d.inv_divisor;
    float r = __builtin_amdgcn_rcpf(am);
    const float e = __fmaf_rn(-am, r, 1.0f);
    r = __fmaf_rn(r, e, r);
    inv = am_bits != 0u ? r * d.divisor : 0.0f;
  } else {
    float off;
    group_scale<false>(d, am_bits, 0, 0, scl, inv, off);
  }
}

// a6 .. a8 for one row of a tile from which outliers and values that are not finite are gone
// (they are zero in `oct`).  top: symmetric, the lane's largest magnitude of the row as binary32 bits.
template <int BITS, bool ASYM, int E, int LANES, bool STRIP>
__device__ __forceinline__ void encode_clean_row(const TensorDesc& d, const TileGeo<E, STRIP>& g, int j,
                                                 const uint32_t (&oct)[4], uint32_t top) {
  constexpr int Q = 1 << (BITS - 1);
  float x[kOct];
  widen_row(oct, x);
  float scl, inv, off = 0.0f;
  if constexpr (!ASYM) {
    scale_sym_clean(d, lanes_reduce<LANES>(top, OpUMax()), scl, inv);
  } else {
    float ext0, ext1;
    row_extremes<true>(x, ext0, ext1);
    const int32_t k0 = lanes_reduce<LANES>(float_key(ext0), OpIMax());
    const int32_t k1 = lanes_reduce<LANES>(float_key(ext1), OpIMin());
    group_scale<true>(d, 0u, k0, k1, scl, inv, off);
  }
  uint32_t c[kOct];
#pragma unroll
  for (int e = 0; e < kOct; ++e) c[e] = code_bits<Q, ASYM>(ASYM ? x[e] - off : x[e], inv);
  store_row<BITS, ASYM, E>(d, g, j, c, scl, off);
}

// ------------------------------------------------------------------ TOPK over groups inside a row
// The k largest of every group of LANES lanes (8 * LANES elements of one row) by (magnitude, lower index),
// as the 8 ballots of the row: k rounds of a maximum over keys (magnitude in the high bits, the reversed
// position in the group below it, plus one so that no live key is zero); the winner's key is unique in its
// group, its owner sets it to zero.  Every value that is not finite is an outlier besides.
template <int LANES>
__device__ __forceinline__ void topk_row_ballots(const TensorDesc& d, const uint32_t (&oct)[4], uint64_t (&b)[kOct]) {
  const uint32_t last = (uint32_t)(LANES * kOct) - 1u - ((uint32_t)lane_id() & (uint32_t)(LANES - 1)) * kOct;  // reversed position of element 0
  uint32_t key[kOct];
  bool nonfinite[kOct];
#pragma unroll
  for (int e = 0; e < kOct; ++e) {
    const uint32_t word = oct[e >> 1];
    const uint32_t mag = (e & 1) ? (word >> 16) & 0x7FFFu : word & 0x7FFFu;
    nonfinite[e] = mag >= kNonfiniteMag;
    key[e] = ((mag << 9) | (last - (uint32_t)e)) + 1u;
  }
  for (uint32_t r = 0; r < d.topk; ++r) {  // uniform
    uint32_t best = key[0];
#pragma unroll
    for (int e = 1; e < kOct; ++e) best = key[e] > best ? key[e] : best;
    const uint32_t win = lanes_reduce<LANES>(best, OpUMax());
#pragma unroll
    for (int e = 0; e < kOct; ++e) key[e] = key[e] == win ? 0u : key[e];
  }
#pragma unroll
  for (int e = 0; e < kOct; ++e) b[e] = __builtin_amdgcn_ballot_w64(key[e] == 0u || nonfinite[e]);
}

// ------------------------------------------------------------------ tile encoder for groups inside a row
// Used when every group (statistics and quantisation) lies inside one 512-element row and both
// kinds have the same size: each row is taken from the raw octets to its stored codes in one
// go, so nothing but the raw octets lives across rows.  LANES = lanes per group.
template <int MODE, int BITS, bool ASYM, int E, int LANES, bool STORE, class Sink, bool STRIP>
__device__ __forceinline__ uint32_t encode_rows(const TensorDesc& d, const TileGeo<E, STRIP>& g,
                                                const uint32_t (&raw)[E][4], uint32_t tile, const Sink& sink,
                                                uint32_t pos0, uint32_t limit) {
  static_assert(!STRIP || MODE == kModeNone, "element indices of outliers are formed for adjacent rows only");
  constexpr int Q = 1 << (BITS - 1);
  const float inv_gs = __uint_as_float((127u - d.lgs) << 23);  // 2^-lgs, exact
  const uint32_t lane_first = tile * (uint32_t)(E * kRow) + (uint32_t)lane_id() * kOct;
  uint32_t total = 0u;  // uniform: outliers of the rows so far
#pragma unroll
  for (int j = 0; j < E; ++j) {
    __builtin_amdgcn_sched_barrier(0);  // one row after the other
    float x[kOct];
    widen_row(raw[j], x);
    // First a test per lane that is cheap and errs on the safe side: can this lane's octet hold an
    // outlier (or, without outliers, a value that is not finite)?  If no lane says yes - nearly
    // every row - the row is quantised as it is.  am_bits: the lane's largest |x| (symmetric).
    float q[kOct];
    float limit_sq = 0.0f;
    uint32_t am_bits = 0u;
    bool suspect;
    uint64_t b[kOct];
    if constexpr (MODE == kModeTopk) {
      suspect = true;  // every group has outliers: its k largest
      topk_row_ballots<LANES>(d, raw[j], b);
      if (!g.full) {  // uniform; the tensor's last tile: groups past its end (blanked) have no outliers
        const uint64_t valid = __builtin_amdgcn_ballot_w64(g.lane_off + g.row_offset(j) < g.rem);
#pragma unroll
        for (int e = 0; e < kOct; ++e) b[e] &= valid;
      }
    } else if constexpr (MODE == kModeStd) {
#pragma unroll
      for (int e = 0; e < kOct; ++e) q[e] = x[e] * x[e];  // exact: two 8-bit significands
      float s1 = ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
      float s2 = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
      s1 = lanes_reduce<LANES>(s1, OpAdd());
      s2 = lanes_reduce<LANES>(s2, OpAdd());
      limit_sq = std_limit(s1, s2, inv_gs, d.param);
      const float qm = fmaxf(fmaxf(fmaxf(q[0], q[1]), fmaxf(q[2], q[3])), fmaxf(fmaxf(q[4], q[5]), fmaxf(q[6], q[7])));
      // an Inf or NaN anywhere in a group makes its limit NaN
      suspect = !(qm <= limit_sq);
      if constexpr (!ASYM) {
        const float am = fmaxf(fmaxf(fmaxf(fabsf(x[0]), fabsf(x[1])), fmaxf(fabsf(x[2]), fabsf(x[3]))),
                               fmaxf(fmaxf(fabsf(x[4]), fabsf(x[5])), fmaxf(fabsf(x[6]), fabsf(x[7]))));
        am_bits = __float_as_uint(am);
      }
    } else {
      am_bits = mag_bits32(octet_magnitude(raw[j]));  // Inf / NaN show as a value of 0x7F800000 or more
      if constexpr (MODE == kModeAbs) suspect = am_bits > __float_as_uint(d.param);  // tau >= 0, finite
      else suspect = am_bits >= 0x7F800000u;
    }
    if constexpr (MODE != kModeTopk) {
      if (__builtin_amdgcn_ballot_w64(suspect) == 0ull) {  // uniform
        if constexpr (STORE) encode_clean_row<BITS, ASYM, E, LANES>(d, g, j, raw[j], am_bits);
        continue;
      }
    }
    // the 8 outlier tests of the row as wavefront ballots (scalar registers)
    if constexpr (MODE == kModeTopk) {
      // formed above
    } else if constexpr (MODE == kModeStd) {
#pragma unroll
      for (int e = 0; e < kOct; ++e) b[e] = __builtin_amdgcn_ballot_w64(q[e] > limit_sq);
      if (__builtin_amdgcn_ballot_w64(limit_sq != limit_sq) != 0ull) {  // then every element is tested for Inf / NaN
#pragma unroll
        for (int e = 0; e < kOct; ++e) b[e] |= __builtin_amdgcn_ballot_w64(is_nonfinite(x[e]));
      }
    } else {
#pragma unroll
      for (int e = 0; e < kOct; ++e) b[e] = __builtin_amdgcn_ballot_w64(outlier_test<MODE>(x[e], d.param));
    }
    uint32_t mask, lane_excl, row_cnt;
    bool any, sparse;
    row_bookkeeping(b, mask, lane_excl, row_cnt, any, sparse);
    if constexpr (STORE) {
      float y[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) y[e] = __builtin_amdgcn_inverse_ballot_w64(b[e]) ? 0.0f : x[e];
      float ext0, ext1;
      row_extremes<ASYM>(y, ext0, ext1);
      float scl, inv, off;
      if constexpr (!ASYM) {
        const uint32_t r0 = lanes_reduce<LANES>(__float_as_uint(ext0), OpUMax());
        group_scale<false>(d, r0, 0, 0, scl, inv, off);
      } else {
        const int32_t k0 = lanes_reduce<LANES>(float_key(ext0), OpIMax());
        const int32_t k1 = lanes_reduce<LANES>(float_key(ext1), OpIMin());
        group_scale<true>(d, 0u, k0, k1, scl, inv, off);
      }
      uint32_t c[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) c[e] = code_bits<Q, ASYM>(ASYM ? y[e] - off : y[e], inv);
      store_row<BITS, ASYM, E>(d, g, j, c, scl, off);
    }
    if constexpr (MODE != kModeNone) {
      if (any) {  // uniform: the row's outliers leave at once, nothing about them is kept
        emit_row(raw[j], mask, lane_excl, sparse, lane_first + (uint32_t)(j * kRow), sink, pos0 + total, limit);
        total += row_cnt;
      }
    }
  }
  return total;
}

template <int MODE, int BITS, bool ASYM, int E, bool STORE, class Sink, bool STRIP>
__device__ __forceinline__ uint32_t encode_tile_rowwise(const TensorDesc& d, const TileGeo<E, STRIP>& g,
                                                        const uint32_t (&raw)[E][4], uint32_t tile, const Sink& sink,
                                                        uint32_t pos0, uint32_t limit) {
  switch (d.lgq) {  // one switch per tile selects straight-line code for the group size
    case 3: return encode_rows<MODE, BITS, ASYM, E, 1, STORE>(d, g, raw, tile, sink, pos0, limit);
    case 4: return encode_rows<MODE, BITS, ASYM, E, 2, STORE>(d, g, raw, tile, sink, pos0, limit);
    case 5: return encode_rows<MODE, BITS, ASYM, E, 4, STORE>(d, g, raw, tile, sink, pos0, limit);
    case 6: return encode_rows<MODE, BITS, ASYM, E, 8, STORE>(d, g, raw, tile, sink, pos0, limit);
    case 7: return encode_rows<MODE, BITS, ASYM, E, 16, STORE>(d, g, raw, tile, sink, pos0, limit);
    case 8: return encode_rows<MODE, BITS, ASYM, E, 32, STORE>(d, g, raw, tile, sink, pos0, limit);
    default: return encode_rows<MODE, BITS, ASYM, E, 64, STORE>(d, g, raw, tile, sink, pos0, limit);
  }
}

// ------------------------------------------------------------------ TOPK selection
// Magnitudes are the 15 low bits of the patterns.  Two ways to find a group's k largest:
//
// By lane maxima (groups of whole rows, small k): every lane takes the largest magnitude among
// its own elements of the group, and the k-th largest of these lane maxima, w, is found by k
// max-reductions over the lanes.  At least k elements are >= w.  If exactly k are, they are the
// k largest of the group whatever their order, and the selection is the plain test |x| >= w.
// Otherwise (two of the largest in one lane, or a tie at the boundary) the caller falls back to
// the rounds below.
//
// By rounds (any group, any k): k max-reductions over keys (magnitude above, inverted position
// below, so ties go to the lower index), each restricted to the keys below the previous winner.
// largest magnitude (15 low bits of the patterns) among the lane's 8 elements of every row:
// two 16-bit lanes at a time.  An Inf or NaN shows as a value >= kNonfiniteMag.
template <int E>
__device__ __forceinline__ void row_magnitudes(const uint32_t (&raw)[E][4], uint32_t (&rowmag)[E]) {
#pragma unroll
  for (int j = 0; j < E; ++j) {
    constexpr uint32_t kMag2 = 0x7FFF7FFFu;
    const uint32_t m =
        pk_max_u16(pk_max_u16(raw[j][0] & kMag2, raw[j][1] & kMag2), pk_max_u16(raw[j][2] & kMag2, raw[j][3] & kMag2));
    const uint32_t hi = m >> 16, lo = m & 0xFFFFu;
    rowmag[j] = hi > lo ? hi : lo;
  }
}

// One group per tile, in straight-line code: t16 <- the k-th largest of the candidates the lanes offer, as
// a 15-bit magnitude.  Returns (uniform) false when the tile holds an Inf or NaN.
// Every lane offers its two largest row maxima: the threshold then fails to cut off exactly k
// elements only when a lane holds three of the k largest, or two of them in one octet, or on a tie.
template <int E>
__device__ __forceinline__ bool topk_whole_threshold(const TensorDesc& d, const uint32_t (&rowmag)[E], uint32_t& t16) {
  const uint32_t lane = (uint32_t)lane_id();
  uint32_t m1 = rowmag[0], m2 = 0u;
#pragma unroll
  for (int j = 1; j < E; ++j) {
    const uint32_t lo = m1 < rowmag[j] ? m1 : rowmag[j];
    m2 = m2 > lo ? m2 : lo;
    m1 = m1 > rowmag[j] ? m1 : rowmag[j];
  }
  const bool finite = __builtin_amdgcn_ballot_w64(m1 >= kNonfiniteMag) == 0ull;
  uint32_t cur = (m1 << 6) | lane;  // unique per lane: equal maxima are taken one after the other
  uint32_t nxt = (m2 << 6) | lane;
  uint32_t win = 0u;                // uniform
  for (uint32_t r = 0; r < d.topk; ++r) {
    win = wave_max_u32_scalar(cur);
    const bool won = cur == win;
    cur = won ? nxt : cur;
    nxt = won ? 0u : nxt;
  }
  t16 = win >> 6;
  return finite;
}

// thr[j] <- the k-th largest lane maximum of row j's group, as the bits of a binary32 value.
// Returns (uniform) false when the tile holds an Inf or NaN.
template <int E>
__device__ __forceinline__ bool topk_lane_maxima(const TensorDesc& d, const uint32_t (&rowmag)[E], uint32_t (&thr)[E]) {
  const uint32_t lane = (uint32_t)lane_id();
  const int R = 1 << (d.lgs - 9);  // rows per group (the caller guarantees lgs >= 9)
  uint32_t m[E];
#pragma unroll
  for (int j = 0; j < E; ++j) m[j] = rowmag[j];
  // rows of a group -> its first row
#pragma unroll
  for (int r = 1; r < E; r <<= 1) {
    if (r < R) {
#pragma unroll
      for (int j = 0; j < E; j += 2 * r) m[j] = m[j] > m[j + r] ? m[j] : m[j + r];
    }
  }
  uint32_t cur[E], win[E];  // win[] is uniform
  bool nonfinite = false;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if ((j & (R - 1)) == 0) nonfinite |= m[j] >= kNonfiniteMag;
    cur[j] = (m[j] << 6) | lane;
    win[j] = 0u;
  }
  for (uint32_t r = 0; r < d.topk; ++r) {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      if ((j & (R - 1)) != 0) continue;  // uniform: a group's state lives in its first row
      win[j] = wave_max_u32_scalar(cur[j]);
      cur[j] = (cur[j] == win[j]) ? 0u : cur[j];
    }
  }
#pragma unroll
  for (int r = E / 2; r >= 1; r >>= 1) {
    if (r < R) {
#pragma unroll
      for (int j = 0; j < E; j += 2 * r) win[j + r] = win[j];
    }
  }
#pragma unroll
  for (int j = 0; j < E; ++j) thr[j] = mag_bits32(win[j] >> 6);
  return __builtin_amdgcn_ballot_w64(nonfinite) == 0ull;
}

// Rounds: thr[j] <- the k-th largest key of row j's group.  Returns (uniform) whether some group's
// k-th largest is Inf / NaN: then there may be more than k outliers.
template <int E>
__device__ __forceinline__ bool topk_select_rounds(const TensorDesc& d, const uint32_t (&raw)[E][4], uint32_t (&kth)[E],
                                                   uint32_t lane_pos, int R) {
#pragma unroll
  for (int j = 0; j < E; ++j) kth[j] = 0xFFFFFFFFu;
  for (uint32_t r = 0; r < d.topk; ++r) {
    forget_derived<E>(raw);  // the keys are formed again in every round: holding them would cost 8 registers per row
    asm volatile("" : "+v"(lane_pos));  // and so are the position codes
    uint32_t best[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint32_t row_pos = ((uint32_t)(j & (R - 1)) << 9) | lane_pos;
      uint32_t m = 0u;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
        const uint32_t cand = (key < kth[j]) ? key : 0u;
        m = (cand > m) ? cand : m;
      }
      best[j] = m;
    }
    groups_reduce_any_order<E>(best, d.lgs, OpUMax());
#pragma unroll
    for (int j = 0; j < E; ++j) kth[j] = best[j];
  }
  bool many = false;
#pragma unroll
  for (int j = 0; j < E; ++j) many |= (kth[j] >> 16) >= kNonfiniteMag;
  return __builtin_amdgcn_ballot_w64(many) != 0ull;
}

// ------------------------------------------------------------------ general tile encoder
// Groups of any supported size (up to the whole tile).  Works in phases over all rows; between
// the phases only the raw octets and a few values per row stay in registers, the widened
// values are formed again where needed (one instruction each).
// a3 + a5 for all rows of a tile: the outlier tests (as wavefront ballots, which live in scalar
// registers, so the run-time choices between tests are uniform branches that cost no vector
// registers), the bookkeeping of the rows that have outliers, and the per-lane extremes of the
// inlier view.  `by_magnitude` (TOPK): thr[j] holds the bits of a binary32 magnitude threshold,
// else the smallest selected key.  `poisoned`: every element is also tested for Inf / NaN.
template <int MODE, bool ASYM, int E>
__device__ __forceinline__ void outlier_phase(const TensorDesc& d, const TileGeo<E>& g, const uint32_t (&raw)[E][4],
                                              const float (&limit)[E], const uint32_t (&thr)[E], bool by_magnitude,
                                              bool poisoned, uint32_t lane_pos, int R,
                                              const uint32_t (&rowmag)[E], float (&ext0)[E], float (&ext1)[E],
                                              TileOutliers<E>& out, int row0 = 0) {
  out.sparse = 0u;
  forget_derived<E>(raw);  // nothing formed from the octets so far is worth its registers
  // uniform, as an integer so that it stays in a scalar register: rows may be skipped on the strength
  // of their largest magnitude (not when keys decide, nor when Inf / NaN are about)
  const uint32_t can_skip = ((MODE != kModeTopk || by_magnitude) && !poisoned) ? 1u : 0u;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    if constexpr (!ASYM) {
      // Symmetric: one test of the lane's largest magnitude of the row tells whether the row can
      // hold an outlier at all; if not, that magnitude is also the lane's share of max |y|, and
      // neither the widened values nor the 8 tests are needed.
      const uint32_t top = mag_bits32(rowmag[j]);  // bits of the largest |x|
      bool maybe;
      if constexpr (MODE == kModeTopk) maybe = top >= thr[j];
      else if constexpr (MODE == kModeAbs) maybe = top > __float_as_uint(d.param);  // tau >= 0; Inf / NaN are above every tau
      else if constexpr (MODE == kModeStd) maybe = __uint_as_float(top) * __uint_as_float(top) > limit[j];
      else maybe = top >= 0x7F800000u;
      if ((__builtin_amdgcn_ballot_w64(maybe) == 0ull) & (can_skip != 0u)) {
        out.mask[j] = 0u; out.lane_excl[j] = 0u; out.row_cnt[j] = 0u;
        out.sparse |= 1u << j;
        ext0[j] = __uint_as_float(top);
        ext1[j] = 0.0f;
        continue;
      }
    }
    float x[kOct];
    widen_row(raw[j], x);
    uint64_t b[kOct];
    if constexpr (MODE == kModeTopk) {
      if (__builtin_expect(by_magnitude, 1)) {
        // rows past the end of the tensor are all selected here, which the caller's count check rejects
        const float t = __uint_as_float(thr[j]);
#pragma unroll
        for (int e = 0; e < kOct; ++e) b[e] = __builtin_amdgcn_ballot_w64(fabsf(x[e]) >= t);
      } else {
        const bool valid = g.lane_off + (uint32_t)(j * kRow) < g.rem;  // blanked octets would be ranked too
        const uint32_t row_pos = ((uint32_t)((row0 + j) & (R - 1)) << 9) | lane_pos;
#pragma unroll
        for (int e = 0; e < kOct; ++e) {
          const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
          b[e] = __builtin_amdgcn_ballot_w64((key >= thr[j]) && valid);
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < kOct; ++e)
        b[e] = __builtin_amdgcn_ballot_w64(outlier_test<MODE>(x[e], MODE == kModeStd ? limit[j] : d.param));
    }
    if (poisoned) {
#pragma unroll
      for (int e = 0; e < kOct; ++e) b[e] |= __builtin_amdgcn_ballot_w64(is_nonfinite(x[e]));
    }
    bool any, sparse;
    row_bookkeeping(b, out.mask[j], out.lane_excl[j], out.row_cnt[j], any, sparse);
    out.sparse |= sparse ? (1u << j) : 0u;
    if (any) {
      float y[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) y[e] = __builtin_amdgcn_inverse_ballot_w64(b[e]) ? 0.0f : x[e];
      row_extremes<ASYM>(y, ext0[j], ext1[j]);
    } else {
      row_extremes<ASYM>(x, ext0[j], ext1[j]);
    }
  }
}

// ---- a6 .. a8 for a tile (or a piece of one) whose outliers are known: scales from the per-lane
// extremes of the inlier view, then quantise, pack, store.
template <int BITS, bool ASYM, int E>
__device__ __forceinline__ void finish_tile(const TensorDesc& d, const TileGeo<E>& g, const uint32_t (&raw)[E][4],
                                            const float (&ext0)[E], const float (&ext1)[E],
                                            const TileOutliers<E>& out) {
  constexpr int Q = 1 << (BITS - 1);
  // ---- a6: per-group scale (and offset).  Cross-lane max / min run on integer images of the floats.
  // Every lane of a group would compute the same scale; with at least 4 lanes per group and 4 rows,
  // lane l of every quad takes row l instead, so that one division serves the whole tile, and the
  // results go back to the rows by a broadcast inside the quad.
  float inv[E], off[E], scl[E];
  const bool transposed = (E == 4) && d.lgq >= 5u;
  const bool row1 = __builtin_amdgcn_inverse_ballot_w64(0x2222222222222222ull);
  const bool row2 = __builtin_amdgcn_inverse_ballot_w64(0x4444444444444444ull);
  const bool row3 = __builtin_amdgcn_inverse_ballot_w64(0x8888888888888888ull);
  if constexpr (!ASYM) {
    uint32_t a[E];  // max |y| as bit patterns: for non-negative floats the integer order is the float order
#pragma unroll
    for (int j = 0; j < E; ++j) a[j] = __float_as_uint(ext0[j]);
    groups_reduce_any_order<E>(a, d.lgq, OpUMax());
    if (transposed) {
      uint32_t am = row1 ? a[1 % E] : a[0];
      am = row2 ? a[2 % E] : am;
      am = row3 ? a[3 % E] : am;
      float s, i, o;
      group_scale<false>(d, am, 0, 0, s, i, o);
      scl[0] = dpp_move<0x00>(s); scl[1 % E] = dpp_move<0x55>(s); scl[2 % E] = dpp_move<0xAA>(s); scl[3 % E] = dpp_move<0xFF>(s);
      inv[0] = dpp_move<0x00>(i); inv[1 % E] = dpp_move<0x55>(i); inv[2 % E] = dpp_move<0xAA>(i); inv[3 % E] = dpp_move<0xFF>(i);
#pragma unroll
      for (int j = 0; j < E; ++j) off[j] = 0.0f;
    } else {
#pragma unroll
      for (int j = 0; j < E; ++j) group_scale<false>(d, a[j], 0, 0, scl[j], inv[j], off[j]);
    }
  } else {
    int32_t hi[E], lo[E];
#pragma unroll
    for (int j = 0; j < E; ++j) { hi[j] = float_key(ext0[j]); lo[j] = float_key(ext1[j]); }
    groups_reduce_any_order<E>(hi, d.lgq, OpIMax());
    groups_reduce_any_order<E>(lo, d.lgq, OpIMin());
    if (transposed) {
      int32_t h = row1 ? hi[1 % E] : hi[0], l = row1 ? lo[1 % E] : lo[0];
      h = row2 ? hi[2 % E] : h; l = row2 ? lo[2 % E] : l;
      h = row3 ? hi[3 % E] : h; l = row3 ? lo[3 % E] : l;
      float s, i, o;
      group_scale<true>(d, 0u, h, l, s, i, o);
      scl[0] = dpp_move<0x00>(s); scl[1 % E] = dpp_move<0x55>(s); scl[2 % E] = dpp_move<0xAA>(s); scl[3 % E] = dpp_move<0xFF>(s);
      inv[0] = dpp_move<0x00>(i); inv[1 % E] = dpp_move<0x55>(i); inv[2 % E] = dpp_move<0xAA>(i); inv[3 % E] = dpp_move<0xFF>(i);
      off[0] = dpp_move<0x00>(o); off[1 % E] = dpp_move<0x55>(o); off[2 % E] = dpp_move<0xAA>(o); off[3 % E] = dpp_move<0xFF>(o);
    } else {
#pragma unroll
      for (int j = 0; j < E; ++j) group_scale<true>(d, 0u, hi[j], lo[j], scl[j], inv[j], off[j]);
    }
  }

  // ---- a7 + a8: quantise, pack, store codes and scales
#pragma unroll
  for (int j = 0; j < E; ++j) {
    float y[kOct];
    widen_row(raw[j], y);
    if (out.row_cnt[j] != 0u) {  // uniform: the inlier view is zero where the mask says so
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        const uint32_t keep = (uint32_t)(((int32_t)(~out.mask[j] << (31 - e))) >> 31);  // all ones unless bit e is set
        y[e] = __uint_as_float(__float_as_uint(y[e]) & keep);
      }
    }
    uint32_t c[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) c[e] = code_bits<Q, ASYM>(ASYM ? y[e] - off[j] : y[e], inv[j]);
    store_row<BITS, ASYM, E>(d, g, j, c, scl[j], off[j]);
  }
}

template <int MODE, int BITS, bool ASYM, int E, bool STORE>
__device__ __forceinline__ void encode_tile_general(const TensorDesc& d, const TileGeo<E>& g,
                                                    const uint32_t (&raw)[E][4], TileOutliers<E>& out) {
  // ---- a2: statistics of the statistics groups
  float limit[E];   // STD: k^2 * var of the row's group
  uint32_t thr[E];  // TOPK: selection threshold of the row's group
  bool poisoned = false;  // uniform: Inf / NaN met in some group's statistics
  uint32_t lane_pos = 0u;
  int R = 1;
  uint32_t rowmag[E];  // symmetric only: the lane's largest magnitude of every row
  if constexpr (!ASYM) {
    row_magnitudes<E>(raw, rowmag);
  } else {
#pragma unroll
    for (int j = 0; j < E; ++j) rowmag[j] = 0u;
  }
  if constexpr (MODE == kModeStd) {
    float s1[E], s2[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      float x[kOct];
      widen_row(raw[j], x);
      s1[j] = ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
      // squares of 16-bit values (at most 11 significant bits) are exact in binary32
      s2[j] = ((x[0] * x[0] + x[1] * x[1]) + (x[2] * x[2] + x[3] * x[3])) +
              ((x[4] * x[4] + x[5] * x[5]) + (x[6] * x[6] + x[7] * x[7]));
    }
    groups_reduce<E>(s1, d.lgs, OpAdd());
    groups_reduce<E>(s2, d.lgs, OpAdd());
    const float inv_gs = __uint_as_float((127u - d.lgs) << 23);  // 2^-lgs, exact
    bool nan_seen = false;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      limit[j] = std_limit(s1[j], s2[j], inv_gs, d.param);
      nan_seen |= (limit[j] != limit[j]);
    }
    poisoned = __builtin_amdgcn_ballot_w64(nan_seen) != 0ull;
  } else if constexpr (MODE == kModeTopk) {
    const uint32_t lane = (uint32_t)lane_id();
    R = (d.lgs > 9) ? (1 << (d.lgs - 9)) : 1;
    lane_pos = (d.lgs > 9) ? (lane << 3) : ((lane & ((1u << (d.lgs - 3)) - 1u)) << 3);
  }

  // ---- a3 + a5: outlier test row by row; extremes of the inlier view per lane
  float ext0[E], ext1[E];
  if constexpr (MODE == kModeTopk) {
    // First the selection by lane maxima where it applies; if it does not stand, once more by rounds.
    // One copy of the code in a loop (rather than two in a row) keeps the registers of the rare second
    // pass from adding to those of the first.
    bool try_maxima = d.lgs >= 9u && d.topk <= 8u;
#pragma nounroll
    while (true) {
      bool by_magnitude = false;
      if (try_maxima) {
        if constexpr (ASYM) row_magnitudes<E>(raw, rowmag);
        by_magnitude = topk_lane_maxima<E>(d, rowmag, thr);
      }
      if (!by_magnitude) {
        // nothing on this rare path may be prepared outside the loop over tiles (32 position codes
        // would otherwise sit in registers for the whole run)
        asm volatile("" : "+v"(lane_pos));
        poisoned = topk_select_rounds<E>(d, raw, thr, lane_pos, R);
      }
      outlier_phase<MODE, ASYM, E>(d, g, raw, limit, thr, by_magnitude, poisoned, lane_pos, R, rowmag, ext0, ext1, out);
      if (!by_magnitude) break;
      // the selection stands if every group has exactly k elements at or above its threshold
      bool exact = true;
      uint32_t in_group = 0u;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        in_group += out.row_cnt[j];
        if ((j & (R - 1)) == R - 1) { exact = exact && (in_group == d.topk); in_group = 0u; }
      }
      if (exact) break;
      try_maxima = false;
    }
  } else {
    outlier_phase<MODE, ASYM, E>(d, g, raw, limit, thr, false, poisoned, lane_pos, R, rowmag, ext0, ext1, out);
  }
  out.total = 0u;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    out.row_off[j] = out.total;
    if constexpr (MODE != kModeNone) out.total += out.row_cnt[j];
  }

  if constexpr (STORE) finish_tile<BITS, ASYM, E>(d, g, raw, ext0, ext1, out);
}

// Rounds over a tile that is one statistics group: the k-th largest key, uniform.  Returns whether
// it belongs to an Inf / NaN (then there may be more than k outliers).
template <int E>
__device__ __forceinline__ bool topk_select_rounds_whole(const TensorDesc& d, const uint32_t (&raw)[E][4], uint32_t& kth_out,
                                                         uint32_t lane_pos) {
  uint32_t kth = 0xFFFFFFFFu;
  for (uint32_t r = 0; r < d.topk; ++r) {
    forget_derived<E>(raw);  // the keys are formed again in every round ...
    asm volatile("" : "+v"(lane_pos));  // ... and so are the position codes: 8 per row would sit in registers otherwise
    uint32_t m = 0u;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint32_t row_pos = ((uint32_t)j << 9) | lane_pos;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
        const uint32_t cand = (key < kth) ? key : 0u;
        m = (cand > m) ? cand : m;
      }
    }
    kth = wave_max_u32_scalar(m);
  }
  kth_out = kth;
  return (kth >> 16) >= kNonfiniteMag;
}

// ------------------------------------------------------------------ TOPK over a whole tile, quantisation groups inside a row
// The tile is one statistics group (so it is complete: group sizes divide the tensor) and every
// quantisation group lies inside a 512-element row.  The paper's order, literally: the outliers
// are found, handed to the sink, and set to zero in the registers that hold the tile; what is left
// is quantised row by row with no thought of outliers.  Nothing but the raw octets and the lane's
// largest magnitude per row lives across rows.  LANES = lanes per quantisation group.

// Extraction by keys (any tile): the k largest keys (magnitude above, inverted position below), and
// every value that is not finite when those are more than k.  Returns the number of outliers.
template <int E, class Sink>
__device__ __forceinline__ uint32_t topk_extract_by_keys(const TensorDesc& d, uint32_t (&raw)[E][4], uint32_t tile,
                                                        const Sink& sink, uint32_t pos0, uint32_t limit) {
  uint32_t lane_pos = (uint32_t)lane_id() << 3;
  uint32_t kth;
  const bool poisoned = topk_select_rounds_whole<E>(d, raw, kth, lane_pos);
  const uint32_t lane_first = tile * (uint32_t)(E * kRow) + (uint32_t)lane_id() * kOct;
  uint32_t total = 0u;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    __builtin_amdgcn_sched_barrier(0);  // row after row, and the position codes of a row formed when its turn comes
    asm volatile("" : "+v"(lane_pos));
    const uint32_t row_pos = ((uint32_t)j << 9) | lane_pos;
    uint64_t b[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      const uint32_t mag = ADACC_ELEM_MAG(raw[j], e);
      const uint32_t key = (mag << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
      b[e] = __builtin_amdgcn_ballot_w64(key >= kth || (poisoned && mag >= kNonfiniteMag));
    }
    uint32_t mask, lane_excl, row_cnt;
    bool any, sparse;
    row_bookkeeping(b, mask, lane_excl, row_cnt, any, sparse);
    if (any) {
      emit_row(raw[j], mask, lane_excl, sparse, lane_first + (uint32_t)(j * kRow), sink, pos0 + total, limit);
      total += row_cnt;
      clear_elements(raw[j], mask);
    }
  }
  return total;
}

// The elements of one octet (that of lane `owner`, a uniform number) whose magnitude reaches t16 leave for
// the sink, in index order from entry `pos` on, and are cleared in the owner's registers.  The octet is
// broadcast through scalar registers and lanes 0..7 take one element each.  Returns their number (uniform).
template <class Sink>
__device__ __forceinline__ uint32_t extract_octet(uint32_t (&oct)[4], uint32_t owner, uint32_t t16, uint32_t first_index,
                                                  const Sink& sink, uint32_t pos, uint32_t limit) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t w0 = (uint32_t)__builtin_amdgcn_readlane((int)oct[0], (int)owner);
  const uint32_t w1 = (uint32_t)__builtin_amdgcn_readlane((int)oct[1], (int)owner);
  const uint32_t w2 = (uint32_t)__builtin_amdgcn_readlane((int)oct[2], (int)owner);
  const uint32_t w3 = (uint32_t)__builtin_amdgcn_readlane((int)oct[3], (int)owner);
  const uint32_t e = lane & 7u;
  const uint32_t lo = (e & 4u) ? w2 : w0;
  const uint32_t hi = (e & 4u) ? w3 : w1;
  const uint32_t word = (e & 2u) ? hi : lo;
  const uint32_t pat = (e & 1u) ? word >> 16 : word & 0xFFFFu;
  const bool hit = lane < 8u && (pat & 0x7FFFu) >= t16;
  const uint32_t m8 = (uint32_t)__builtin_amdgcn_ballot_w64(hit);  // bit e: element e
  if (hit) {
    const uint32_t p = pos + __builtin_amdgcn_mbcnt_lo(m8, 0u);
    if (p < limit) sink(p, first_index + e, pat);
  }
  if (lane == owner) clear_elements(oct, m8);
  return (uint32_t)__builtin_popcount(m8);
}

// The extraction: finds the k largest, hands them to the sink, clears them in `raw`.  rowmag: the
// lane's largest magnitude per row of what is left.  Returns the number of outliers (uniform).
template <int E, bool STORE, class Sink>
__device__ __forceinline__ uint32_t topk_extract(const TensorDesc& d, uint32_t (&raw)[E][4], uint32_t (&rowmag)[E],
                                                 uint32_t tile, const Sink& sink, uint32_t pos0, uint32_t limit) {
  row_magnitudes<E>(raw, rowmag);
  const uint32_t tile_first = tile * (uint32_t)(E * kRow);
  uint32_t total = 0u;  // uniform: outliers found
  bool done = false;    // uniform
  if (d.topk <= 8u) {
    uint32_t t16;
    if (topk_whole_threshold<E>(d, rowmag, t16)) {  // false if the tile holds an Inf or a NaN
      // Selection |x| >= t: it is the answer if exactly k elements pass.  Only octets whose largest magnitude
      // reaches t can hold any; there are at most k of them if the selection is to stand, so they are
      // taken one at a time (a constant tile, where every octet passes, goes straight to the keys).
      uint64_t cand[E];
      uint32_t octets = 0u;
#pragma unroll
      for (int j = 0; j < E; ++j) {
        cand[j] = __builtin_amdgcn_ballot_w64(rowmag[j] >= t16);
        octets += (uint32_t)__builtin_popcountll(cand[j]);
      }
      if (octets <= d.topk) {
        // The outliers leave and are cleared as they are found; if in the end they were not k (two of
        // the largest in one octet, a tie at the k-th place) the tile is read again and done by keys.
#pragma unroll
        for (int j = 0; j < E; ++j) {
          uint64_t todo = cand[j];
          if (todo == 0ull) continue;  // uniform
          do {
            const uint32_t owner = (uint32_t)__builtin_ctzll(todo);
            todo &= todo - 1ull;
            total += extract_octet(raw[j], owner, t16, tile_first + (uint32_t)(j * kRow) + owner * kOct, sink, pos0 + total, limit);
          } while (todo != 0ull);
          rowmag[j] = octet_magnitude(raw[j]);
        }
        done = total == d.topk;
      }
    }
  }
  if (!done) {
    if (total != 0u) {
      // some outliers have left and are cleared already: start over from the source, once the
      // stores of the first attempt are complete (the second attempt writes the same entries)
      __builtin_amdgcn_s_waitcnt(0x0F70);
      load_tile<E, true>(d, tile, raw);
    }
    total = topk_extract_by_keys<E>(d, raw, tile, sink, pos0, limit);
    if constexpr (STORE) row_magnitudes<E>(raw, rowmag);
  }
  return total;
}

template <int BITS, bool ASYM, int E, int LANES>
__device__ __forceinline__ void encode_clean_rows(const TensorDesc& d, const TileGeo<E>& g, const uint32_t (&raw)[E][4],
                                                  const uint32_t (&rowmag)[E]) {
#pragma unroll
  for (int j = 0; j < E; ++j) {
    // one row after the other: the compiler shall not start on the next rows to hide this row's
    // latencies (other wavefronts do that), it would pay for it with the registers of a wavefront
    __builtin_amdgcn_sched_barrier(0);
    encode_clean_row<BITS, ASYM, E, LANES>(d, g, j, raw[j], mag_bits32(rowmag[j]));
  }
}

template <int BITS, bool ASYM, int E, bool STORE, class Sink>
__device__ __forceinline__ uint32_t encode_tile_topk_whole(const TensorDesc& d, const TileGeo<E>& g,
                                                           uint32_t (&raw)[E][4], uint32_t tile, const Sink& sink,
                                                           uint32_t pos0, uint32_t limit) {
  uint32_t rowmag[E];
  const uint32_t total = topk_extract<E, STORE>(d, raw, rowmag, tile, sink, pos0, limit);
  if constexpr (STORE) {
    switch (d.lgq) {  // one switch per tile selects straight-line code for the group size
      case 3: encode_clean_rows<BITS, ASYM, E, 1>(d, g, raw, rowmag); break;
      case 4: encode_clean_rows<BITS, ASYM, E, 2>(d, g, raw, rowmag); break;
      case 5: encode_clean_rows<BITS, ASYM, E, 4>(d, g, raw, rowmag); break;
      case 6: encode_clean_rows<BITS, ASYM, E, 8>(d, g, raw, rowmag); break;
      case 7: encode_clean_rows<BITS, ASYM, E, 16>(d, g, raw, rowmag); break;
      case 8: encode_clean_rows<BITS, ASYM, E, 32>(d, g, raw, rowmag); break;
      default: encode_clean_rows<BITS, ASYM, E, 64>(d, g, raw, rowmag); break;
    }
  }
  return total;
}

// ------------------------------------------------------------------ one tile, whatever the encoder
// Encodes the tile (a2 .. a8) and hands its outliers, in ascending index order, to `sink` from
// position pos0 on (entries at or past `limit` are dropped).  Returns the number of outliers of the
// tile (uniform).
// ROWWISE: all groups lie inside a row and statistics and quantisation groups coincide.
// WHOLE (TOPK): the statistics group is the whole tile and every quantisation group lies inside a row.
// STORE = false: only the outliers are found (nothing is quantised or stored).
template <int MODE, int BITS, bool ASYM, int E, bool ROWWISE, bool WHOLE, bool STORE, class Sink>
__device__ __forceinline__ uint32_t encode_tile(const TensorDesc& d, const TileGeo<E>& g, uint32_t (&raw)[E][4],
                                                uint32_t tile, const Sink& sink, uint32_t pos0, uint32_t limit) {
  static_assert(!WHOLE || (MODE == kModeTopk && !ROWWISE), "WHOLE is a TOPK encoder");
  if constexpr (ROWWISE) {
    return encode_tile_rowwise<MODE, BITS, ASYM, E, STORE>(d, g, raw, tile, sink, pos0, limit);
  } else if constexpr (WHOLE) {
    return encode_tile_topk_whole<BITS, ASYM, E, STORE>(d, g, raw, tile, sink, pos0, limit);
  } else {
    TileOutliers<E> out;
    encode_tile_general<MODE, BITS, ASYM, E, STORE>(d, g, raw, out);
    if constexpr (MODE != kModeNone) {
      if (out.total != 0u) emit_outliers<E>(raw, out, tile, sink, pos0, limit);
    }
    return out.total;
  }
}

// ------------------------------------------------------------------ one tile with outliers (ABS / STD / TOPK)
// Tiles are independent: a wavefront compresses one tile and never waits for another.  What the
// ordered outlier stream needs from all tiles together - the offset of every tile - is settled
// afterwards by place_block (below), from the per-tile counts written here.
//
// ABS / STD: the tile's outliers (ascending) go to the tile's own slot of kSlot records in the
// workspace; the placement kernel moves them to their final position.  A tile with more than
// kSlot outliers leaves the rest out; the placement kernel then selects that tile's outliers from
// the source once more.
// TOPK: every statistics group has exactly topk outliers unless it holds more than topk values that
// are not finite, so the offsets are known in advance: group g starts at topk * g.  The outliers
// are written to their final position at once, and a tile that finds another count raises the
// tensor's flag (the current epoch of the workspace); only then does the placement kernel do
// anything, and it then does everything again from the source.
template <int MODE, int BITS, bool ASYM, int E, bool ROWWISE, bool WHOLE = false>
__device__ __forceinline__ void compress_tile_outliers(const TensorDesc& d, uint32_t tile, uint32_t epoch) {
  static_assert(MODE != kModeNone, "tiles without outliers have compress_tile_plain");
  const bool last = tile + 1u == d.n_tiles;
  const bool lane0 = lane_id() == 0;
  uint32_t raw[E][4];
  if constexpr (MODE == kModeTopk) {
    const uint32_t per_tile = d.topk << (d.lgt - d.lgs);  // outliers of a complete, regular tile
    const uint32_t pos0 = per_tile * tile;
    uint32_t expected = per_tile;
    if (last) expected = d.topk * (uint32_t)((d.numel - (uint64_t)tile * (uint64_t)(E * kRow)) >> d.lgs);
    const uint32_t end = pos0 + expected;
    const StreamSink sink{d.idx, d.val};
    const uint32_t limit = end < d.cap ? end : d.cap;
    uint32_t total;
    if (WHOLE || !last) {  // only the last tile can be short: the copy for the others knows nothing of it
      load_tile<E, true>(d, tile, raw);
      total = encode_tile<MODE, BITS, ASYM, E, ROWWISE, WHOLE, true>(d, tile_geo<E, true>(d, tile), raw, tile, sink, pos0, limit);
    } else {
      load_tile<E, false>(d, tile, raw);
      const TileGeo<E> g = tile_geo<E, false>(d, tile);
      blank_tail<E>(g, raw);
      total = encode_tile<MODE, BITS, ASYM, E, ROWWISE, WHOLE, true>(d, g, raw, tile, sink, pos0, limit);
    }
    if (lane0) {
      d.tile_ptr[tile] = pos0;
      d.cnt[tile] = total;
      if (total != expected) *d.flag = epoch;
      if (last) {
        d.tile_ptr[d.n_tiles] = end;
        d.status[0] = end; d.status[1] = end > d.cap ? 1u : 0u; d.status[2] = 0u; d.status[3] = 0u;
      }
    }
  } else {
    const SlotSink sink{d.slot + (uint64_t)tile * (uint64_t)kSlot};
    uint32_t total;
    if (!last) {
      load_tile<E, true>(d, tile, raw);
      total = encode_tile<MODE, BITS, ASYM, E, ROWWISE, false, true>(d, tile_geo<E, true>(d, tile), raw, tile, sink, 0u, (uint32_t)kSlot);
    } else {
      load_tile<E, false>(d, tile, raw);
      const TileGeo<E> g = tile_geo<E, false>(d, tile);
      blank_tail<E>(g, raw);
      total = encode_tile<MODE, BITS, ASYM, E, ROWWISE, false, true>(d, g, raw, tile, sink, 0u, (uint32_t)kSlot);
    }
    if (lane0) d.cnt[tile] = total;
  }
}

// ------------------------------------------------------------------ placement of the outliers (a4)
// One workgroup of kPlaceThreads threads takes a block of kPlaceTiles consecutive tiles, one per
// thread.  It needs the number of outliers in all tiles before its block: for ABS / STD a kernel in
// between (place_sum_block) has added up the counts of every block, and the workgroup adds those
// sums; for short tensors, and for TOPK (where this kernel has work only if some group was
// irregular), it adds the counts themselves.  Nobody waits for anybody.  Then it scans the counts of
// its own tiles, writes their offsets, and moves the outliers of its tiles from the slots to their
// final positions, output position by output position (coalesced stores; the tile of a position is
// found by bisection over the block's offsets in LDS).  Tiles that hold more outliers than a slot
// takes (or all tiles, `reselect_all`) are selected again from the source, one wavefront per tile,
// and written straight to the stream.
struct PlaceShared {
  uint32_t excl[kPlaceTiles + 1];  // offsets of the block's tiles relative to the block, and the block total
  uint32_t part[kPlaceThreads / kWave];
};

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  struct OpUAdd { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; } };
  v = lanes_reduce<16>(v, OpUAdd());
  int t = __builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
  v += (uint32_t)t;
  t = __builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);      // row_bcast:31
  v += (uint32_t)t;
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// sum over the workgroup (kPlaceThreads threads), returned to every thread
__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t (&part)[kPlaceThreads / kWave]) {
  const uint32_t w = wave_sum_u32(v);
  const uint32_t wave = threadIdx.x / kWave;
  __syncthreads();  // earlier readers of part[] are done
  if (lane_id() == 0) part[wave] = w;
  __syncthreads();
  uint32_t s = 0u;
#pragma unroll
  for (int i = 0; i < kPlaceThreads / kWave; ++i) s += part[i];
  return s;
}

// sum of n 32-bit words (16-byte aligned) over the workgroup; four loads of 16 bytes per thread are
// in flight at a time
__device__ __forceinline__ uint32_t sum_words(const uint32_t* words, uint32_t n, uint32_t (&part)[kPlaceThreads / kWave]) {
  const uint4* w4 = reinterpret_cast<const uint4*>(words);
  const uint32_t n4 = n / 4u;
  uint32_t acc = 0u;
  for (uint32_t i0 = 0u; i0 < n4; i0 += 4u * (uint32_t)kPlaceThreads) {
    uint4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t i = i0 + (uint32_t)k * (uint32_t)kPlaceThreads + threadIdx.x;
      v[k] = i < n4 ? w4[i] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) acc += (v[k].x + v[k].y) + (v[k].z + v[k].w);
  }
  if (threadIdx.x < (n & 3u)) acc += words[4u * n4 + threadIdx.x];
  return block_sum_u32(acc, part);
}

// block_sum[block] = outliers in the block's tiles
__device__ __forceinline__ void place_sum_block(const TensorDesc& d, uint32_t block, uint32_t (&part)[kPlaceThreads / kWave]) {
  const uint32_t t = block * (uint32_t)kPlaceTiles + threadIdx.x;
  const uint32_t s = block_sum_u32(t < d.n_tiles ? d.cnt[t] : 0u, part);
  if (threadIdx.x == 0) d.block_sum[block] = s;
}

// select the outliers of one tile again and write them to the stream, into the tile's own `count`
// entries from position `pos` (an attempt of the selection that has to be given up must not reach
// into a neighbour's entries)
template <int MODE, int E, bool ROWWISE, bool WHOLE>
__device__ __forceinline__ void reselect_tile(const TensorDesc& d, uint32_t tile, uint32_t pos, uint32_t count) {
  uint32_t raw[E][4];
  load_tile<E, false>(d, tile, raw);
  const TileGeo<E> g = tile_geo<E, false>(d, tile);
  blank_tail<E>(g, raw);
  const uint32_t end = pos + count;
  encode_tile<MODE, 8, false, E, ROWWISE, WHOLE, false>(d, g, raw, tile, StreamSink{d.idx, d.val}, pos, end < d.cap ? end : d.cap);
}

// The offsets of a block's tiles from the counts: tile_ptr for the block's tiles, and in the block that holds the
// last tile the total and the overflow flag.  Leaves in sh.excl the offsets relative to the block (and the
// block's total behind them).  Returns the number of outliers before the block; n_here: tiles of the block.
// `from_sums`: the counts of the blocks are in d.block_sum (else the counts of the tiles are added up)
// mine: outliers of this thread's tile
__device__ __forceinline__ uint32_t place_offsets_block(const TensorDesc& d, uint32_t block, bool from_sums, PlaceShared& sh,
                                                        uint32_t& n_here, uint32_t& total, uint32_t& mine) {
  const uint32_t tid = threadIdx.x;
  const uint32_t first = block * (uint32_t)kPlaceTiles;
  // outliers of all tiles before this block
  const uint32_t base = from_sums ? sum_words(d.block_sum, block, sh.part) : sum_words(d.cnt, first, sh.part);
  // this thread's tile
  const uint32_t t = first + tid;
  const uint32_t c = t < d.n_tiles ? d.cnt[t] : 0u;
  mine = c;
  // exclusive scan over the workgroup: inside the wavefront by shuffles, across wavefronts through LDS
  uint32_t incl = c;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t up = (uint32_t)__shfl_up((int)incl, off);
    if (lane_id() >= off) incl += up;
  }
  const uint32_t wave = tid / kWave;
  __syncthreads();
  if (lane_id() == kWave - 1) sh.part[wave] = incl;
  __syncthreads();
  uint32_t wave_before = 0u;
  total = 0u;
#pragma unroll
  for (int i = 0; i < kPlaceThreads / kWave; ++i) {
    wave_before += (uint32_t)i < wave ? sh.part[i] : 0u;
    total += sh.part[i];
  }
  const uint32_t e0 = wave_before + incl - c;  // relative to the block
  sh.excl[tid] = e0;
  if (tid == 0) sh.excl[kPlaceTiles] = total;
  if (t < d.n_tiles) d.tile_ptr[t] = base + e0;
  n_here = d.n_tiles - first < (uint32_t)kPlaceTiles ? d.n_tiles - first : (uint32_t)kPlaceTiles;
  if (first + n_here == d.n_tiles && tid == 0) {  // the block that holds the last tile also closes the blob
    const uint32_t n_out = base + total;
    d.tile_ptr[d.n_tiles] = n_out;
    d.status[0] = n_out; d.status[1] = n_out > d.cap ? 1u : 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
  return base;
}

// The offsets of a block's tiles, and the outliers of its tiles from the slots to the stream: four positions per
// thread at a time, so that their loads overlap.  Tiles with more outliers than a slot takes are left out.
// Returns the number of outliers before the block; n_here: tiles of the block.  `move`: false = offsets only
__device__ __forceinline__ uint32_t place_moves_block(const TensorDesc& d, uint32_t block, bool from_sums, bool move,
                                                      PlaceShared& sh, uint32_t& n_here, uint32_t& mine) {
  const uint32_t tid = threadIdx.x;
  const uint32_t first = block * (uint32_t)kPlaceTiles;
  uint32_t total;
  const uint32_t base = place_offsets_block(d, block, from_sums, sh, n_here, total, mine);
  __syncthreads();
  if (move) {
    for (uint32_t p0 = 0u; p0 < total; p0 += 4u * (uint32_t)kPlaceThreads) {
      uint64_t src[4];
      uint32_t dst[4];
      bool ok[4];
      // last tile j with excl[j] <= p (tiles without outliers share their successor's offset): the four
      // bisections step together, so that a step is one round trip to LDS for all of them (a block has at
      // most 2^8 tiles)
      uint32_t lo[4], hi[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) { lo[k] = 0u; hi[k] = n_here; }
#pragma unroll
      for (int step = 0; step < 8; ++step) {
        uint32_t mid[4], at[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) { mid[k] = (lo[k] + hi[k]) >> 1; at[k] = sh.excl[mid[k]]; }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t p = p0 + (uint32_t)k * (uint32_t)kPlaceThreads + tid;
          if (hi[k] - lo[k] > 1u) {
            if (at[k] <= p) lo[k] = mid[k]; else hi[k] = mid[k];
          }
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t p = p0 + (uint32_t)k * (uint32_t)kPlaceThreads + tid;
        const uint32_t n_tile = sh.excl[lo[k] + 1u] - sh.excl[lo[k]];
        dst[k] = base + p;
        ok[k] = p < total && n_tile <= (uint32_t)kSlot && dst[k] < d.cap;
        src[k] = ok[k] ? (uint64_t)(first + lo[k]) * (uint64_t)kSlot + (p - sh.excl[lo[k]]) : 0ull;
      }
      uint2 rec[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) rec[k] = d.slot[src[k]];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (ok[k]) { d.idx[dst[k]] = (int32_t)rec[k].x; d.val[dst[k]] = (uint16_t)rec[k].y; }
      }
    }
  }
  return base;
}

template <int MODE, int E, bool ROWWISE, bool WHOLE>
__device__ __forceinline__ void place_block(const TensorDesc& d, uint32_t block, bool from_sums, bool reselect_all,
                                            PlaceShared& sh) {
  const uint32_t tid = threadIdx.x;
  const uint32_t first = block * (uint32_t)kPlaceTiles;
  uint32_t n_here, mine;
  const uint32_t base = place_moves_block(d, block, from_sums, !reselect_all, sh, n_here, mine);
  // tiles whose outliers are not (all) in a slot: once more from the source, a wavefront per tile
  if (__syncthreads_or(mine > (reselect_all ? 0u : (uint32_t)kSlot) ? 1 : 0) == 0) return;  // the usual case: none
  const uint32_t w = __builtin_amdgcn_readfirstlane(tid / kWave);
  for (uint32_t j = w; j < n_here; j += (uint32_t)(kPlaceThreads / kWave)) {
    const uint32_t n_tile = sh.excl[j + 1u] - sh.excl[j];
    if (n_tile > (reselect_all ? 0u : (uint32_t)kSlot))
      reselect_tile<MODE, E, ROWWISE, WHOLE>(d, first + j, base + sh.excl[j], n_tile);
  }
}

// ------------------------------------------------------------------ one tile without outliers (NONE)
template <int BITS, bool ASYM, int E, bool ROWWISE>
__device__ __forceinline__ void compress_tile_plain(const TensorDesc& d, uint32_t tile) {
  uint32_t raw[E][4];
  if (tile + 1u < d.n_tiles) {  // only the last tile can be short: the copy for the others knows nothing of it
    load_tile<E, true>(d, tile, raw);
    encode_tile<kModeNone, BITS, ASYM, E, ROWWISE, false, true>(d, tile_geo<E, true>(d, tile), raw, tile, NullSink{}, 0u, 0u);
  } else {
    load_tile<E, false>(d, tile, raw);
    const TileGeo<E> g = tile_geo<E, false>(d, tile);
    blank_tail<E>(g, raw);
    encode_tile<kModeNone, BITS, ASYM, E, ROWWISE, false, true>(d, g, raw, tile, NullSink{}, 0u, 0u);
  }
  if (tile == 0 && lane_id() == 0) {
    d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
