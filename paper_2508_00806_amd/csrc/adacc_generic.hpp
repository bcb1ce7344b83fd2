// Compression and decompression for methods outside the fast kernels' shapes (Section 3.2 asks for groups
// of the activation and treats a tensor of any shape as a flat array; nothing there makes the groups powers
// of two): quantisation groups of any multiple of 8 elements, statistics groups of any multiple of the
// quantisation group up to 16384 elements (a whole 11008-wide row as one STD / TOPK group).  The fast
// kernels reduce over power-of-two numbers of lanes inside one wavefront's tile and cannot take these.
//
// Here a workgroup of four wavefronts takes a "segment": as many whole statistics groups as fit 4096
// elements (one group, if it is larger), held in LDS as 16-bit patterns, and works through it with plain
// loops - by the same definitions as everywhere: canonical pairwise sums (pad to a power of two, add
// neighbours level by level), mean and variance over the group's own count, the k largest by (magnitude,
// lower index), D / max by one IEEE division per group, the same rounding of the codes.  A segment that is
// one statistics group is worked on by the whole workgroup; in a segment of several groups every wavefront
// takes groups of its own.  It is a fallback, several times slower than the tile kernels, not a hot path.
//
// With outliers a compression is two launches of the same kernel around the placement kernels: the first
// only counts the outliers of every segment (cnt[segment]), the placement kernels turn the counts into
// offsets (tile_ptr, the total, the overflow flag), the second writes the outliers at their offsets and
// everything else.  The segment is the blob's tile (adacc_layout.tile_elems).
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_dtype.hpp"

namespace adacc {
namespace ADACC_DT_NS {

constexpr uint32_t kSegThreads = (uint32_t)kThreads;
constexpr uint32_t kSegWaves = kSegThreads / (uint32_t)kWave;
// bytes of LDS before the segment's arrays: the words the wavefronts meet in
constexpr uint32_t kSegHeadBytes = 4u * 16u;

// The LDS of a workgroup, sized by the host for the method's segment length:
// [meet: 16 words][raw: tile_elems 16-bit patterns][byte: tile_elems bytes]
struct SegmentShared {
  uint32_t* meet;
  uint16_t* raw;   // the patterns of the segment; an element that is kept aside or not finite is set to zero
  uint8_t* byte;   // first: 1 = outlier; later: the element's code
};
__device__ __forceinline__ SegmentShared segment_shared(unsigned char* lds, uint32_t tile_elems) {
  SegmentShared sh;
  sh.meet = reinterpret_cast<uint32_t*>(lds);
  sh.raw = reinterpret_cast<uint16_t*>(lds + kSegHeadBytes);
  sh.byte = lds + kSegHeadBytes + 2u * tile_elems;
  return sh;
}

__device__ __forceinline__ bool pattern_nonfinite(uint32_t pattern) { return (pattern & 0x7FFFu) >= kNonfiniteMag; }

// Who works on a group: the whole workgroup (WG) or one wavefront.  size / id: the members and this
// thread's number among them; sync: all members have finished their LDS accesses (a wavefront's own
// accesses are taken in order, so for a wavefront nothing is waited for); max_u32 / tree_sum: over all
// members, the result in every member.  tree_sum adds in the order of the balanced tree over the members.
template <bool WG>
struct Team {
  uint32_t* meet;  // WG: LDS words where the wavefronts meet
  __device__ __forceinline__ static uint32_t size() { return WG ? kSegThreads : (uint32_t)kWave; }
  __device__ __forceinline__ static uint32_t id() { return WG ? threadIdx.x : (uint32_t)lane_id(); }
  __device__ __forceinline__ static void sync() {
    if constexpr (WG) __syncthreads();
    else __builtin_amdgcn_wave_barrier();
  }
  __device__ __forceinline__ uint32_t max_u32(uint32_t v) const {
    v = wave_max_u32_scalar(v);
    if constexpr (WG) {
      __syncthreads();  // the previous use of meet is over
      if (lane_id() == 0) meet[threadIdx.x / kWave] = v;
      __syncthreads();
      v = meet[0];
#pragma unroll
      for (uint32_t w = 1; w < kSegWaves; ++w) v = meet[w] > v ? meet[w] : v;
    }
    return v;
  }
  __device__ __forceinline__ float tree_sum(float v) const {
    v = lanes_reduce<kWave>(v, OpAdd());
    if constexpr (WG) {
      static_assert(kSegWaves == 4, "the wavefronts' sums are added as a tree of four");
      __syncthreads();
      if (lane_id() == 0) meet[threadIdx.x / kWave] = __float_as_uint(v);
      __syncthreads();
      v = (__uint_as_float(meet[0]) + __uint_as_float(meet[1])) + (__uint_as_float(meet[2]) + __uint_as_float(meet[3]));
    }
    return v;
  }
};

// Canonical pairwise sums over the team of raw[i] and of raw[i]^2, i < cnt: the leaves are padded with zeros
// to a power of two p, member t owns the p / size leaves from t * (p / size) on (one leaf for p <= size) and
// adds them as a binary tree by carries (partial sums of 1, 2, 4, .. units wait in s[]), the members' sums then
// meet as a tree: together the balanced tree over the padded array.  A member with 8 leaves or more takes
// them an octet at a time (one 16-byte read; the tree over the 8 written out) and carries the octets' sums.
__device__ __forceinline__ void carry_in(float (&s)[7], uint32_t i, float v) {
  bool placed = false;
#pragma unroll
  for (int l = 0; l < 6; ++l) {
    if (!placed) {
      if ((i >> l) & 1u) v = s[l] + v;  // the earlier units on the left
      else { s[l] = v; placed = true; }
    }
  }
  if (!placed) s[6] = v;
}
template <bool WG>
__device__ __forceinline__ void segment_pairwise(const Team<WG>& team, const uint16_t* raw, uint32_t cnt, float& sum,
                                                 float& sum_sq) {
  uint32_t p = 1u;
  while (p < cnt) p <<= 1;
  const uint32_t per = p > team.size() ? p / team.size() : 1u;  // a power of two, at most 64 (2048 / 64, 16384 / 256)
  const uint32_t first = team.id() * per;
  float s1[7], s2[7];
#pragma unroll
  for (int l = 0; l < 7; ++l) s1[l] = s2[l] = 0.0f;
  uint32_t units = per;  // what the carries count: leaves, or octets of leaves
  if (per >= (uint32_t)kOct) {
    units = per / (uint32_t)kOct;
    const bool aligned = (reinterpret_cast<uintptr_t>(raw) & 15u) == 0;  // uniform: the group starts on a 16-byte boundary of the LDS
    for (uint32_t o = 0; o < units; ++o) {  // uniform
      const uint32_t i0 = first + o * (uint32_t)kOct;
      float v[kOct];
      if (aligned && i0 + (uint32_t)kOct <= cnt) {
        const uint4 w = *reinterpret_cast<const uint4*>(raw + i0);
        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[2 * k] = widen_lo(ww[k]); v[2 * k + 1] = widen_hi(ww[k]); }
      } else {
#pragma unroll
        for (int e = 0; e < kOct; ++e) v[e] = i0 + (uint32_t)e < cnt ? widen_lo(raw[i0 + e]) : 0.0f;
      }
      carry_in(s1, o, ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
#pragma unroll
      for (int e = 0; e < kOct; ++e) v[e] = v[e] * v[e];
      carry_in(s2, o, ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
    }
  } else {
    for (uint32_t i = 0; i < per; ++i) {  // uniform
      const float v = first + i < cnt ? widen_lo(raw[first + i]) : 0.0f;
      carry_in(s1, i, v);
      carry_in(s2, i, v * v);
    }
  }
  // after all units = 2^m the last carry chain has run up to level m and the sum sits in s[m]
  float mine1 = s1[0], mine2 = s2[0];
#pragma unroll
  for (int l = 1; l < 7; ++l) {
    mine1 = units == (1u << l) ? s1[l] : mine1;
    mine2 = units == (1u << l) ? s2[l] : mine2;
  }
  sum = team.tree_sum(mine1);
  sum_sq = team.tree_sum(mine2);
}

// a2 / a3 for one statistics group (ABS: the whole segment): byte[i] = 1 for the outliers among raw[0 .. cnt)
// TOPK: the kernel is the one for TOPK methods (its keys take 64 registers, the other modes do without)
template <bool WG, bool TOPK>
__device__ __forceinline__ void segment_select(const TensorDesc& d, const Team<WG>& team, const uint16_t* raw,
                                               uint8_t* byte, uint32_t cnt) {
  const uint32_t me = team.id(), step = team.size();
  if constexpr (!TOPK) {
    if (d.mode == kModeAbs) {
      for (uint32_t i = me; i < cnt; i += step)
        byte[i] = (fabsf(widen_lo(raw[i])) > d.param || pattern_nonfinite(raw[i])) ? 1 : 0;
    } else {  // STD
      float s1, s2;
      segment_pairwise<WG>(team, raw, cnt, s1, s2);
      const float n = (float)cnt;
      const float mean = __fdiv_rn(s1, n);
      float var = __fmaf_rn(-mean, mean, __fdiv_rn(s2, n));
      var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
      const float limit = d.param * var;  // param = k * k
      for (uint32_t i = me; i < cnt; i += step) {
        const float v = widen_lo(raw[i]);
        byte[i] = (v * v > limit || pattern_nonfinite(raw[i])) ? 1 : 0;
      }
    }
  } else {  // TOPK: the k largest magnitudes, ties to the lower index
    // Every member holds the keys of its own elements (at most 16384 / 256 resp. 2048 / 64 of them) in
    // registers: magnitude above the reversed index, never zero.  A round is one maximum over everything;
    // the winner's key is unique, its owner sets it to zero.  Zero keys are the outliers.
    constexpr int kCap = WG ? 64 : 32;
    uint32_t key[kCap];
#pragma unroll
    for (int j = 0; j < kCap; ++j) {
      const uint32_t i = me + (uint32_t)j * step;
      key[j] = i < cnt ? (((uint32_t)(raw[i] & 0x7FFFu) << 16) | (0xFFFFu - i)) : 0u;
    }
    const uint32_t rounds = d.topk < cnt ? d.topk : cnt;
    for (uint32_t round = 0; round < rounds; ++round) {
      uint32_t best = 0u;
#pragma unroll
      for (int j = 0; j < kCap; ++j) best = key[j] > best ? key[j] : best;
      const uint32_t win = team.max_u32(best);  // not zero: fewer than cnt elements are taken so far
#pragma unroll
      for (int j = 0; j < kCap; ++j) key[j] = key[j] == win ? 0u : key[j];
    }
#pragma unroll
    for (int j = 0; j < kCap; ++j) {
      const uint32_t i = me + (uint32_t)j * step;
      // a value that cannot be quantised at all is always kept exactly
      if (i < cnt) byte[i] = (key[j] == 0u || pattern_nonfinite(raw[i])) ? 1 : 0;
    }
  }
  team.sync();
}

// The outliers of raw[0 .. cnt) (byte[i] == 1), in index order: their number (uniform), and, when `emit`,
// entry pos, pos + 1, .. of the stream for them (indices first_index + i).  The whole workgroup.
__device__ __forceinline__ uint32_t segment_outliers(const TensorDesc& d, SegmentShared& sh, uint32_t cnt, bool emit,
                                                     uint32_t pos, uint64_t first_index) {
  const uint32_t tid = threadIdx.x;
  const uint32_t per = (cnt + kSegThreads - 1u) / kSegThreads;
  const uint32_t i0 = tid * per < cnt ? tid * per : cnt;
  const uint32_t i1 = i0 + per < cnt ? i0 + per : cnt;
  uint32_t mine = 0u;
  for (uint32_t i = i0; i < i1; ++i) mine += sh.byte[i];
  // threads before this one: inside the wavefront by a scan over the lanes, the wavefronts through LDS
  const uint32_t lane = (uint32_t)lane_id(), wave = tid / (uint32_t)kWave;
  uint32_t incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t t = (uint32_t)__shfl_up((int)incl, o, kWave);
    if (lane >= (uint32_t)o) incl += t;
  }
  if (lane == (uint32_t)kWave - 1u) sh.meet[8u + wave] = incl;
  __syncthreads();
  uint32_t before = incl - mine, total = 0u;
#pragma unroll
  for (uint32_t w = 0; w < kSegWaves; ++w) {
    const uint32_t c = sh.meet[8u + w];
    before += w < wave ? c : 0u;
    total += c;
  }
  if (emit) {
    uint32_t p = pos + before;
    for (uint32_t i = i0; i < i1; ++i) {
      if (sh.byte[i] == 0) continue;
      if (p < d.cap) {
        d.idx[p] = (int32_t)(first_index + i);
        d.val[p] = sh.raw[i];
      }
      ++p;
    }
  }
  __syncthreads();
  return total;
}

// a5: from here on the outliers, and every value that is not finite, count as zero
__device__ __forceinline__ void segment_clear(const TensorDesc& d, SegmentShared& sh, uint32_t cnt) {
  for (uint32_t i = threadIdx.x; i < cnt; i += kSegThreads)
    if ((d.mode != kModeNone && sh.byte[i] != 0) || pattern_nonfinite(sh.raw[i])) sh.raw[i] = 0;
  __syncthreads();
}

// a6 .. a8 for one quantisation group raw[g0 .. g0 + n) by a team: scale (offset) and the codes into byte[]
template <int Q, bool ASYM, bool WG>
__device__ __forceinline__ void quantise_group(const TensorDesc& d, const Team<WG>& team, SegmentShared& sh, uint32_t g0,
                                               uint32_t n, uint64_t group) {
  const uint32_t me = team.id(), step = team.size();
  float scl, inv, off;
  if constexpr (!ASYM) {
    uint32_t am = 0u;
    for (uint32_t i = me; i < n; i += step) {
      const uint32_t bits = __float_as_uint(fabsf(widen_lo(sh.raw[g0 + i])));
      am = bits > am ? bits : am;
    }
    group_scale<false>(d, team.max_u32(am), 0, 0, scl, inv, off);
  } else {
    int32_t hi = float_key(widen_lo(sh.raw[g0])), lo = hi;
    for (uint32_t i = me; i < n; i += step) {
      const int32_t k = float_key(widen_lo(sh.raw[g0 + i]));
      hi = k > hi ? k : hi;
      lo = k < lo ? k : lo;
    }
    // signed keys through the unsigned maximum: flip the sign bit (and, for the minimum, the rest)
    const int32_t k0 = (int32_t)(team.max_u32((uint32_t)hi ^ 0x80000000u) ^ 0x80000000u);
    const int32_t k1 = (int32_t)(~team.max_u32(~((uint32_t)lo ^ 0x80000000u)) ^ 0x80000000u);
    group_scale<true>(d, 0u, k0, k1, scl, inv, off);
  }
  for (uint32_t i = me; i < n; i += step) {
    const float y = widen_lo(sh.raw[g0 + i]);
    sh.byte[g0 + i] = (uint8_t)code_bits<Q>(ASYM ? y - off : y, inv);
  }
  if (me == 0u) {
    d.scales[group] = scl;
    if constexpr (ASYM) d.zp[group] = off;
  }
}

// a6 .. a8 for raw[0 .. cnt), cut into groups of gq from its start (the last one may be short); first_elem:
// the tensor index of raw[0], a multiple of gq and of 8.  Small groups are taken one per thread, larger ones
// one per wavefront, those beyond 1024 elements (at most four to a segment) by the whole workgroup in turn.
template <int Q, bool ASYM>
__device__ __forceinline__ void segment_quantise(const TensorDesc& d, SegmentShared& sh, uint32_t cnt, uint64_t first_elem) {
  const uint32_t tid = threadIdx.x;
  const uint32_t gq = d.gq;
  const uint64_t first_group = first_elem / gq;
  const uint32_t n_groups = (cnt + gq - 1u) / gq;
  if (gq <= 64u) {
    for (uint32_t g = tid; g < n_groups; g += kSegThreads) {
      const uint32_t g0 = g * gq;
      const uint32_t n = cnt - g0 < gq ? cnt - g0 : gq;
      float scl, inv, off;
      if constexpr (!ASYM) {
        uint32_t am = 0u;
        for (uint32_t i = 0; i < n; ++i) {
          const uint32_t bits = __float_as_uint(fabsf(widen_lo(sh.raw[g0 + i])));
          am = bits > am ? bits : am;
        }
        group_scale<false>(d, am, 0, 0, scl, inv, off);
      } else {
        int32_t hi = float_key(widen_lo(sh.raw[g0])), lo = hi;
        for (uint32_t i = 1; i < n; ++i) {
          const int32_t k = float_key(widen_lo(sh.raw[g0 + i]));
          hi = k > hi ? k : hi;
          lo = k < lo ? k : lo;
        }
        group_scale<true>(d, 0u, hi, lo, scl, inv, off);
      }
      for (uint32_t i = 0; i < n; ++i) {
        const float y = widen_lo(sh.raw[g0 + i]);
        sh.byte[g0 + i] = (uint8_t)code_bits<Q>(ASYM ? y - off : y, inv);
      }
      d.scales[first_group + g] = scl;
      if constexpr (ASYM) d.zp[first_group + g] = off;
    }
  } else if (gq <= 1024u) {
    const Team<false> team{nullptr};
    for (uint32_t g = tid / (uint32_t)kWave; g < n_groups; g += kSegWaves) {  // uniform in the wavefront
      const uint32_t g0 = g * gq;
      quantise_group<Q, ASYM, false>(d, team, sh, g0, cnt - g0 < gq ? cnt - g0 : gq, first_group + g);
    }
  } else {
    const Team<true> team{sh.meet};
    for (uint32_t g = 0; g < n_groups; ++g) {  // uniform
      const uint32_t g0 = g * gq;
      quantise_group<Q, ASYM, true>(d, team, sh, g0, cnt - g0 < gq ? cnt - g0 : gq, first_group + g);
    }
  }
  __syncthreads();
  // the codes leave an octet at a time (8 resp. 4 bytes; the segment starts on a multiple of 8 elements), what
  // is left of a tensor's ragged end one by one
  const uint32_t octs = cnt / (uint32_t)kOct;
  if constexpr (Q == 128) {
    uint8_t* out = d.codes + first_elem;
    for (uint32_t o = tid; o < octs; o += kSegThreads)
      *reinterpret_cast<uint2*>(out + o * kOct) = *reinterpret_cast<const uint2*>(sh.byte + o * kOct);
    for (uint32_t i = octs * kOct + tid; i < cnt; i += kSegThreads) out[i] = sh.byte[i];
  } else {
    uint8_t* out = d.codes + (first_elem >> 1);
    for (uint32_t o = tid; o < octs; o += kSegThreads) {
      const uint2 c = *reinterpret_cast<const uint2*>(sh.byte + o * kOct);
      const uint32_t e = (c.x & 0x0F0F0F0Fu) | ((c.x >> 4) & 0x00F000F0u);   // bytes 0 and 2: the nibble pairs of elements 0..3
      const uint32_t f = (c.y & 0x0F0F0F0Fu) | ((c.y >> 4) & 0x00F000F0u);
      // pair (2j, 2j+1) -> one byte: low nibble the even element
      const uint32_t lo = (e & 0xFFu) | ((e >> 8) & 0xFF00u);
      const uint32_t hi = (f & 0xFFu) | ((f >> 8) & 0xFF00u);
      *reinterpret_cast<uint32_t*>(out + o * 4u) = lo | (hi << 16);
    }
    for (uint32_t b = octs * 4u + tid; b < (cnt + 1u) / 2u; b += kSegThreads) {
      const uint32_t lo = sh.byte[2u * b] & 0xFu;
      const uint32_t hi = 2u * b + 1u < cnt ? (sh.byte[2u * b + 1u] & 0xFu) : 0u;  // an odd end: the high nibble is 0
      out[b] = (uint8_t)(lo | (hi << 4));
    }
  }
}

__device__ __forceinline__ void segment_quantise_any(const TensorDesc& d, SegmentShared& sh, uint32_t cnt, uint64_t first_elem) {
  if (d.bits == 8u) {
    if (d.asym) segment_quantise<128, true>(d, sh, cnt, first_elem); else segment_quantise<128, false>(d, sh, cnt, first_elem);
  } else {
    if (d.asym) segment_quantise<8, true>(d, sh, cnt, first_elem); else segment_quantise<8, false>(d, sh, cnt, first_elem);
  }
}

// One segment (d.tile_elems elements, the last one of the tensor may be short).  COUNT: only the number of
// its outliers, into d.cnt.
template <bool COUNT, bool TOPK>
__device__ __forceinline__ void compress_segment(const TensorDesc& d, SegmentShared& sh, uint32_t seg) {
  const uint32_t tid = threadIdx.x;
  const uint64_t first_elem = (uint64_t)seg * d.tile_elems;
  const uint64_t left = d.numel - first_elem;
  const uint32_t cnt = left < (uint64_t)d.tile_elems ? (uint32_t)left : d.tile_elems;
  // whole octets with one 16-byte load (the segment starts on a multiple of 8 elements), the rest one by one
  const uint32_t octs = cnt / kOct;
  for (uint32_t o = tid; o < octs; o += kSegThreads)
    *reinterpret_cast<uint4*>(sh.raw + o * kOct) = *reinterpret_cast<const uint4*>(d.src + first_elem + o * kOct);
  for (uint32_t i = octs * kOct + tid; i < cnt; i += kSegThreads) sh.raw[i] = d.src[first_elem + i];
  __syncthreads();
  if (d.mode != kModeNone) {
    if (d.mode == kModeAbs || d.gs >= d.tile_elems) {  // ABS needs no statistics; or the segment is one group
      const Team<true> team{sh.meet};
      segment_select<true, TOPK>(d, team, sh.raw, sh.byte, cnt);
    } else {  // several groups: each wavefront takes groups of its own
      const Team<false> team{nullptr};
      for (uint32_t g0 = (tid / (uint32_t)kWave) * d.gs; g0 < cnt; g0 += kSegWaves * d.gs)
        segment_select<false, TOPK>(d, team, sh.raw + g0, sh.byte + g0, cnt - g0 < d.gs ? cnt - g0 : d.gs);
      __syncthreads();
    }
    if constexpr (COUNT) {
      const uint32_t total = segment_outliers(d, sh, cnt, false, 0u, 0ull);
      if (tid == 0u) d.cnt[seg] = total;
      return;
    } else {
      segment_outliers(d, sh, cnt, true, d.tile_ptr[seg], first_elem);
    }
  } else if (seg == 0u && tid == 0u) {
    d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
  segment_clear(d, sh, cnt);
  segment_quantise_any(d, sh, cnt, first_elem);
}

// a9 / a10 for one segment
__device__ __forceinline__ void decompress_segment(const TensorDesc& d, uint32_t seg) {
  const uint32_t tid = threadIdx.x;
  const uint64_t first_elem = (uint64_t)seg * d.tile_elems;
  const uint64_t left = d.numel - first_elem;
  const uint32_t cnt = left < (uint64_t)d.tile_elems ? (uint32_t)left : d.tile_elems;
  const uint64_t first_group = first_elem / d.gq;
  // an octet at a time: it lies inside one quantisation group (groups are multiples of 8, the segment starts
  // on a group), so one scale serves it; what is left of a tensor's ragged end goes one by one
  const uint32_t octs = cnt / (uint32_t)kOct;
  for (uint32_t o = tid; o < octs; o += kSegThreads) {
    const uint64_t e0 = first_elem + (uint64_t)o * kOct;
    int code[kOct];
    if (d.bits == 8u) {
      const uint2 w = *reinterpret_cast<const uint2*>(d.codes + e0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        code[e] = (int)(int8_t)((w.x >> (8 * e)) & 0xFFu);
        code[4 + e] = (int)(int8_t)((w.y >> (8 * e)) & 0xFFu);
      }
    } else {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(d.codes + (e0 >> 1));
#pragma unroll
      for (int e = 0; e < kOct; ++e) code[e] = ((int)(w << (28 - 4 * e))) >> 28;  // sign-extended nibble
    }
    const uint64_t grp = first_group + (o * (uint32_t)kOct) / d.gq;
    const float s = d.scales[grp];
    const float z = d.asym ? d.zp[grp] : 0.0f;
    float v[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) v[e] = d.asym ? __fmaf_rn((float)code[e], s, z) : (float)code[e] * s;
    if (d.dst_f32) {
      float* p = reinterpret_cast<float*>(d.dst) + e0;
      *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(d.dst) + e0) =
          make_uint4(narrow_pair(v[0], v[1]), narrow_pair(v[2], v[3]), narrow_pair(v[4], v[5]), narrow_pair(v[6], v[7]));
    }
  }
  for (uint32_t i = octs * kOct + tid; i < cnt; i += kSegThreads) {
    int code;
    if (d.bits == 8u) code = (int)(int8_t)d.codes[first_elem + i];
    else code = ((int)((uint32_t)d.codes[(first_elem + i) >> 1] << (28u - 4u * (i & 1u)))) >> 28;  // first_elem is even
    const uint64_t grp = first_group + i / d.gq;
    const float s = d.scales[grp];
    const float v = d.asym ? __fmaf_rn((float)code, s, d.zp[grp]) : (float)code * s;
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[first_elem + i] = v;
    else reinterpret_cast<uint16_t*>(d.dst)[first_elem + i] = (uint16_t)narrow_pair(v, 0.0f);
  }
  if (d.mode == kModeNone) return;
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's stores above are complete ...
  __syncthreads();                       // ... and so are those of the other wavefronts of the segment
  uint32_t p0 = d.tile_ptr[seg], p1 = d.tile_ptr[seg + 1u];
  p0 = p0 < d.cap ? p0 : d.cap;
  p1 = p1 < d.cap ? p1 : d.cap;
  for (uint32_t p = p0 + tid; p < p1; p += kSegThreads) {
    const uint64_t i = (uint32_t)d.idx[p];
    if (i < first_elem || i >= first_elem + cnt) continue;  // a damaged stream must not write outside the segment
    const uint32_t pat = d.val[p];
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[i] = widen_lo(pat);
    else reinterpret_cast<uint16_t*>(d.dst)[i] = (uint16_t)pat;
  }
}

template <bool COUNT, bool TOPK>
__global__ __launch_bounds__(kSegThreads) void compress_generic_kernel(TensorDesc d) {
  extern __shared__ __attribute__((aligned(16))) unsigned char segment_lds[];
  SegmentShared sh = segment_shared(segment_lds, d.tile_elems);
  compress_segment<COUNT, TOPK>(d, sh, blockIdx.x);
}
__global__ __launch_bounds__(kSegThreads) void decompress_generic_kernel(TensorDesc d) { decompress_segment(d, blockIdx.x); }

}  // namespace ADACC_DT_NS
}  // namespace adacc
