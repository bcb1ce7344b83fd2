// Compression and decompression for methods outside the fast kernels' shapes (Section 3.2 asks for groups
// of the activation and treats a tensor of any shape as a flat array; nothing there makes the groups powers
// of two): quantisation groups of any multiple of 8 elements, statistics groups of any multiple of the
// quantisation group up to 16384 elements (a whole 11008-wide row as one STD / TOPK group).  The fast
// kernels reduce over power-of-two numbers of lanes inside one wavefront's tile and cannot take these.
//
// Here a wavefront takes a "segment": as many whole statistics groups as fit 4096 elements (one group, if it
// is larger), held in LDS as 16-bit patterns, and works through it with plain loops - by the same
// definitions as everywhere: canonical pairwise sums (pad to a power of two, add neighbours level by level),
// mean and variance over the group's own count, the k largest by (magnitude, lower index), D / max by one
// IEEE division per group, the same rounding of the codes.  It is a fallback, 5 to 60 times slower than the
// tile kernels (the statistics over a whole 11008-element row being the slow end), not a hot path.
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

// The LDS of a workgroup (one wavefront), sized by the host for the method's segment length:
// [lane_cnt: 64 words][raw: tile_elems 16-bit patterns][byte: tile_elems bytes]
struct SegmentShared {
  uint32_t* lane_cnt;
  uint16_t* raw;   // the patterns of the segment; an element that is kept aside or not finite is set to zero
  uint8_t* byte;   // first: 1 = outlier; later: the element's code
};
__device__ __forceinline__ SegmentShared segment_shared(unsigned char* lds, uint32_t tile_elems) {
  SegmentShared sh;
  sh.lane_cnt = reinterpret_cast<uint32_t*>(lds);
  sh.raw = reinterpret_cast<uint16_t*>(lds + 4u * (uint32_t)kWave);
  sh.byte = lds + 4u * (uint32_t)kWave + 2u * tile_elems;
  return sh;
}

__device__ __forceinline__ bool pattern_nonfinite(uint32_t pattern) { return (pattern & 0x7FFFu) >= kNonfiniteMag; }

// Canonical pairwise sum over the wavefront of f(raw[i]), i < cnt (f = the value, or its square): the leaves
// are padded with zeros to a power of two p, lane l owns the p / 64 leaves from l * (p / 64) on (one leaf for
// p <= 64) and adds them as a binary tree by carries (partial sums of 1, 2, 4, .. leaves wait in s[]), the
// lanes' sums then meet by the xor butterfly: together the balanced tree over the padded array.
template <bool SQUARE>
__device__ __forceinline__ float segment_pairwise(const uint16_t* raw, uint32_t cnt) {
  uint32_t p = 1u;
  while (p < cnt) p <<= 1;
  const uint32_t per_lane = p > (uint32_t)kWave ? p / (uint32_t)kWave : 1u;  // a power of two, at most 256
  const uint32_t first = (uint32_t)lane_id() * per_lane;
  float s[9];
#pragma unroll
  for (int l = 0; l < 9; ++l) s[l] = 0.0f;
  for (uint32_t i = 0; i < per_lane; ++i) {  // uniform
    float v = 0.0f;
    if (first + i < cnt) {
      v = widen_lo(raw[first + i]);
      if constexpr (SQUARE) v = v * v;
    }
    bool placed = false;
#pragma unroll
    for (int l = 0; l < 8; ++l) {
      if (!placed) {
        if ((i >> l) & 1u) v = s[l] + v;  // the earlier leaves on the left
        else { s[l] = v; placed = true; }
      }
    }
    if (!placed) s[8] = v;
  }
  // after all per_lane = 2^m leaves the last carry chain has run up to level m and the sum sits in s[m]
  float mine = s[0];
#pragma unroll
  for (int l = 1; l < 9; ++l) mine = per_lane == (1u << l) ? s[l] : mine;
  return lanes_reduce<kWave>(mine, OpAdd());
}

// a2 / a3 for one statistics group: byte[i] = 1 for the outliers among raw[0 .. cnt)
__device__ __forceinline__ void segment_select(const TensorDesc& d, const uint16_t* raw, uint8_t* byte, uint32_t cnt) {
  const uint32_t lane = (uint32_t)lane_id();
  for (uint32_t i = lane; i < cnt; i += kWave) byte[i] = 0;
  __syncthreads();
  if (d.mode == kModeAbs) {
    for (uint32_t i = lane; i < cnt; i += kWave) byte[i] = fabsf(widen_lo(raw[i])) > d.param ? 1 : 0;
  } else if (d.mode == kModeStd) {
    const float s1 = segment_pairwise<false>(raw, cnt);
    const float s2 = segment_pairwise<true>(raw, cnt);
    const float n = (float)cnt;
    const float mean = __fdiv_rn(s1, n);
    float var = __fmaf_rn(-mean, mean, __fdiv_rn(s2, n));
    var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
    const float limit = d.param * var;  // param = k * k
    for (uint32_t i = lane; i < cnt; i += kWave) {
      const float v = widen_lo(raw[i]);
      byte[i] = v * v > limit ? 1 : 0;
    }
  } else if (d.mode == kModeTopk) {  // the k largest magnitudes, ties to the lower index
    const uint32_t rounds = d.topk < cnt ? d.topk : cnt;
    for (uint32_t round = 0; round < rounds; ++round) {
      uint32_t best = 0u;
      for (uint32_t i = lane; i < cnt; i += kWave) {
        const uint32_t key = ((uint32_t)(raw[i] & 0x7FFFu) << 16) | (0xFFFFu - i);
        best = (byte[i] == 0 && key > best) ? key : best;
      }
      const uint32_t win = wave_max_u32_scalar(best);  // not zero: fewer than cnt elements are taken so far
      const uint32_t i = 0xFFFFu - (win & 0xFFFFu);
      if (i < cnt && (i & ((uint32_t)kWave - 1u)) == lane) byte[i] = 1;
      __syncthreads();
    }
  }
  __syncthreads();
  if (d.mode != kModeNone) {  // a value that cannot be quantised at all is always kept exactly
    for (uint32_t i = lane; i < cnt; i += kWave)
      if (pattern_nonfinite(raw[i])) byte[i] = 1;
  }
  __syncthreads();
}

// The outliers of raw[0 .. cnt) (byte[i] == 1), in index order: their number (uniform), and, when `emit`,
// entry pos, pos + 1, .. of the stream for them (indices first_index + i).
__device__ __forceinline__ uint32_t segment_outliers(const TensorDesc& d, SegmentShared& sh, uint32_t cnt, bool emit,
                                                     uint32_t pos, uint64_t first_index) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t per_lane = (cnt + (uint32_t)kWave - 1u) / (uint32_t)kWave;
  const uint32_t i0 = lane * per_lane < cnt ? lane * per_lane : cnt;
  const uint32_t i1 = i0 + per_lane < cnt ? i0 + per_lane : cnt;
  uint32_t mine = 0u;
  for (uint32_t i = i0; i < i1; ++i) mine += sh.byte[i];
  sh.lane_cnt[lane] = mine;
  __syncthreads();
  uint32_t before = 0u, total = 0u;
  for (uint32_t l = 0; l < (uint32_t)kWave; ++l) {
    const uint32_t c = sh.lane_cnt[l];
    before += l < lane ? c : 0u;
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
  for (uint32_t i = (uint32_t)lane_id(); i < cnt; i += kWave)
    if ((d.mode != kModeNone && sh.byte[i] != 0) || pattern_nonfinite(sh.raw[i])) sh.raw[i] = 0;
  __syncthreads();
}

// a6 .. a8 for raw[0 .. cnt), cut into groups of gq from its start (the last one may be short); first_elem:
// the tensor index of raw[0], a multiple of gq and of 8.  Small groups are taken one per lane, large ones
// one after the other by the whole wavefront.
template <int Q, bool ASYM>
__device__ __forceinline__ void segment_quantise(const TensorDesc& d, SegmentShared& sh, uint32_t cnt, uint64_t first_elem) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t gq = d.gq;
  const uint64_t first_group = first_elem / gq;
  const uint32_t n_groups = (cnt + gq - 1u) / gq;
  if (gq <= 128u) {
    for (uint32_t g = lane; g < n_groups; g += kWave) {
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
  } else {
    for (uint32_t g = 0; g < n_groups; ++g) {
      const uint32_t g0 = g * gq;
      const uint32_t n = cnt - g0 < gq ? cnt - g0 : gq;
      float scl, inv, off;
      if constexpr (!ASYM) {
        uint32_t am = 0u;
        for (uint32_t i = lane; i < n; i += kWave) {
          const uint32_t bits = __float_as_uint(fabsf(widen_lo(sh.raw[g0 + i])));
          am = bits > am ? bits : am;
        }
        group_scale<false>(d, wave_max_u32_scalar(am), 0, 0, scl, inv, off);
      } else {
        int32_t hi = float_key(widen_lo(sh.raw[g0])), lo = hi;
        for (uint32_t i = lane; i < n; i += kWave) {
          const int32_t k = float_key(widen_lo(sh.raw[g0 + i]));
          hi = k > hi ? k : hi;
          lo = k < lo ? k : lo;
        }
        // signed keys through the unsigned maximum: flip the sign bit (and, for the minimum, the rest)
        const int32_t k0 = (int32_t)(wave_max_u32_scalar((uint32_t)hi ^ 0x80000000u) ^ 0x80000000u);
        const int32_t k1 = (int32_t)(~wave_max_u32_scalar(~((uint32_t)lo ^ 0x80000000u)) ^ 0x80000000u);
        group_scale<true>(d, 0u, k0, k1, scl, inv, off);
      }
      for (uint32_t i = lane; i < n; i += kWave) {
        const float y = widen_lo(sh.raw[g0 + i]);
        sh.byte[g0 + i] = (uint8_t)code_bits<Q>(ASYM ? y - off : y, inv);
      }
      if (lane == 0u) {
        d.scales[first_group + g] = scl;
        if constexpr (ASYM) d.zp[first_group + g] = off;
      }
    }
  }
  __syncthreads();
  if constexpr (Q == 128) {
    uint8_t* out = d.codes + first_elem;
    for (uint32_t i = lane; i < cnt; i += kWave) out[i] = sh.byte[i];
  } else {
    uint8_t* out = d.codes + (first_elem >> 1);
    for (uint32_t b = lane; b < (cnt + 1u) / 2u; b += kWave) {
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
template <bool COUNT>
__device__ __forceinline__ void compress_segment(const TensorDesc& d, SegmentShared& sh, uint32_t seg) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint64_t first_elem = (uint64_t)seg * d.tile_elems;
  const uint64_t left = d.numel - first_elem;
  const uint32_t cnt = left < (uint64_t)d.tile_elems ? (uint32_t)left : d.tile_elems;
  for (uint32_t i = lane; i < cnt; i += kWave) sh.raw[i] = d.src[first_elem + i];
  __syncthreads();
  if (d.mode != kModeNone) {
    const uint32_t gs = (d.mode == kModeAbs) ? cnt : d.gs;  // ABS needs no statistics: one go
    for (uint32_t g0 = 0; g0 < cnt; g0 += gs)
      segment_select(d, sh.raw + g0, sh.byte + g0, cnt - g0 < gs ? cnt - g0 : gs);
    if constexpr (COUNT) {
      const uint32_t total = segment_outliers(d, sh, cnt, false, 0u, 0ull);
      if (lane == 0u) d.cnt[seg] = total;
      return;
    } else {
      segment_outliers(d, sh, cnt, true, d.tile_ptr[seg], first_elem);
    }
  } else if (seg == 0u && lane == 0u) {
    d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
  segment_clear(d, sh, cnt);
  segment_quantise_any(d, sh, cnt, first_elem);
}

// a9 / a10 for one segment
__device__ __forceinline__ void decompress_segment(const TensorDesc& d, uint32_t seg) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint64_t first_elem = (uint64_t)seg * d.tile_elems;
  const uint64_t left = d.numel - first_elem;
  const uint32_t cnt = left < (uint64_t)d.tile_elems ? (uint32_t)left : d.tile_elems;
  const uint64_t first_group = first_elem / d.gq;
  for (uint32_t i = lane; i < cnt; i += kWave) {
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
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the stores above are complete
  __syncthreads();
  uint32_t p0 = d.tile_ptr[seg], p1 = d.tile_ptr[seg + 1u];
  p0 = p0 < d.cap ? p0 : d.cap;
  p1 = p1 < d.cap ? p1 : d.cap;
  for (uint32_t p = p0 + lane; p < p1; p += kWave) {
    const uint64_t i = (uint32_t)d.idx[p];
    if (i < first_elem || i >= first_elem + cnt) continue;  // a damaged stream must not write outside the segment
    const uint32_t pat = d.val[p];
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[i] = widen_lo(pat);
    else reinterpret_cast<uint16_t*>(d.dst)[i] = (uint16_t)pat;
  }
}

template <bool COUNT>
__global__ __launch_bounds__(kWave) void compress_generic_kernel(TensorDesc d) {
  extern __shared__ __attribute__((aligned(16))) unsigned char segment_lds[];
  SegmentShared sh = segment_shared(segment_lds, d.tile_elems);
  compress_segment<COUNT>(d, sh, blockIdx.x);
}
__global__ __launch_bounds__(kWave) void decompress_generic_kernel(TensorDesc d) { decompress_segment(d, blockIdx.x); }

}  // namespace ADACC_DT_NS
}  // namespace adacc
