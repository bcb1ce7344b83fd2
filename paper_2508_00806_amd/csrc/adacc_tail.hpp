// The end of a tensor whose length the group sizes do not divide (Section 3.2: a tensor of any shape is
// taken as one flat array and cut into groups from its start).  The kernels of adacc_compress.hpp and
// adacc_decompress.hpp take the part of the tensor made of whole groups of the larger kind
// (TensorDesc::numel elements, a multiple of that group size); what is left, fewer than 4096 elements,
// is the "tail": at most one short statistics group, cut into quantisation groups the last of which
// may be short.  It is treated like any other group over the elements it has (own scale; mean and
// variance over its own count; at most as many largest values as it holds).
//
// One wavefront does the whole tail, in plain loops over LDS arrays: this is the rare end of a tensor,
// not a hot path.  Compression runs after the placement kernel of the main part (stream order), appends
// the tail's outliers to the stream and completes the tile offsets and the status words.
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_dtype.hpp"

namespace adacc {
namespace ADACC_DT_NS {

constexpr uint32_t kTailMax = 4096;  // a tail is shorter than the largest group

struct TailShared {
  uint16_t raw[kTailMax];   // the patterns of the tail
  uint8_t out[kTailMax];    // 1: kept aside as an outlier
  uint8_t code[kTailMax];   // the code of every element, two's complement in the low bits
  float a[kTailMax];        // levels of the pairwise sums (ping)
  float b[kTailMax / 2];    // (pong)
  uint32_t lane_cnt[kWave];
};

__device__ __forceinline__ float tail_value(uint32_t pattern) { return widen_lo(pattern); }
__device__ __forceinline__ bool tail_nonfinite(uint32_t pattern) { return (pattern & 0x7FFFu) >= kNonfiniteMag; }

// Canonical pairwise sum of sh.a[0 .. p), p a power of two: neighbours are added until one value is
// left (the order of the statistics of whole groups, and of the definition they follow).
__device__ __forceinline__ float tail_pairwise(TailShared& sh, uint32_t p) {
  float* src = sh.a;
  float* dst = sh.b;
  for (uint32_t len = p; len > 1u; len >>= 1) {
    const uint32_t half = len >> 1;
    __syncthreads();
    for (uint32_t j = (uint32_t)lane_id(); j < half; j += kWave) dst[j] = src[2u * j] + src[2u * j + 1u];
    float* t = src; src = dst; dst = t;
  }
  __syncthreads();
  return src[0];
}

// a2 / a3 for the tail: sh.out[i] for its r elements
__device__ __forceinline__ void tail_select(const TensorDesc& d, TailShared& sh, uint32_t r) {
  const uint32_t lane = (uint32_t)lane_id();
  for (uint32_t i = lane; i < r; i += kWave) sh.out[i] = 0;
  if (d.mode == kModeNone) { __syncthreads(); return; }
  uint32_t p = 1u;
  while (p < r) p <<= 1;
  if (d.mode == kModeAbs) {
    for (uint32_t i = lane; i < r; i += kWave) sh.out[i] = fabsf(tail_value(sh.raw[i])) > d.param ? 1 : 0;
  } else if (d.mode == kModeStd) {
    for (uint32_t i = lane; i < p; i += kWave) sh.a[i] = i < r ? tail_value(sh.raw[i]) : 0.0f;
    const float s1 = tail_pairwise(sh, p);
    __syncthreads();
    for (uint32_t i = lane; i < p; i += kWave) {
      const float v = i < r ? tail_value(sh.raw[i]) : 0.0f;
      sh.a[i] = v * v;
    }
    const float s2 = tail_pairwise(sh, p);
    const float n = (float)r;
    const float mean = __fdiv_rn(s1, n);
    float var = __fmaf_rn(-mean, mean, __fdiv_rn(s2, n));
    var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
    const float limit = d.param * var;  // param = k * k
    for (uint32_t i = lane; i < r; i += kWave) {
      const float v = tail_value(sh.raw[i]);
      sh.out[i] = v * v > limit ? 1 : 0;
    }
  } else {  // the k largest magnitudes, ties to the lower index
    __syncthreads();
    const uint32_t rounds = d.topk < r ? d.topk : r;
    for (uint32_t round = 0; round < rounds; ++round) {
      uint32_t best = 0u;
      for (uint32_t i = lane; i < r; i += kWave) {
        const uint32_t key = ((uint32_t)(sh.raw[i] & 0x7FFFu) << 16) | (0xFFFFu - i);
        best = (sh.out[i] == 0 && key > best) ? key : best;
      }
      const uint32_t win = wave_max_u32_scalar(best);  // not zero: fewer than r elements are taken so far
      const uint32_t i = 0xFFFFu - (win & 0xFFFFu);
      if (i < r && (i & (kWave - 1u)) == lane) sh.out[i] = 1;
      __syncthreads();
    }
  }
  __syncthreads();
  // a value that cannot be quantised at all is always kept exactly
  for (uint32_t i = lane; i < r; i += kWave)
    if (tail_nonfinite(sh.raw[i])) sh.out[i] = 1;
  __syncthreads();
}

template <int Q, bool ASYM>
__device__ __forceinline__ void tail_quantise(const TensorDesc& d, TailShared& sh, uint32_t r) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t gq = 1u << d.lgq;
  const uint64_t first_group = d.numel >> d.lgq;
  for (uint32_t g0 = 0, g = 0; g0 < r; g0 += gq, ++g) {
    const uint32_t cnt = r - g0 < gq ? r - g0 : gq;
    // what is quantised: outliers and values that are not finite count as zero
    auto y_of = [&](uint32_t i) -> float {
      const uint32_t pat = sh.raw[g0 + i];
      return (sh.out[g0 + i] != 0 || tail_nonfinite(pat)) ? 0.0f : tail_value(pat);
    };
    float scl, inv, off;
    if constexpr (!ASYM) {
      uint32_t am = 0u;
      for (uint32_t i = lane; i < cnt; i += kWave) {
        const uint32_t bits = __float_as_uint(fabsf(y_of(i)));
        am = bits > am ? bits : am;
      }
      group_scale<false>(d, wave_max_u32_scalar(am), 0, 0, scl, inv, off);
    } else {
      const float y0 = y_of(0u);
      int32_t hi = float_key(y0), lo = hi;
      for (uint32_t i = lane; i < cnt; i += kWave) {
        const int32_t k = float_key(y_of(i));
        hi = k > hi ? k : hi;
        lo = k < lo ? k : lo;
      }
      // signed keys through the unsigned maximum: flip the sign bit (and, for the minimum, the rest)
      const int32_t k0 = (int32_t)(wave_max_u32_scalar((uint32_t)hi ^ 0x80000000u) ^ 0x80000000u);
      const int32_t k1 = (int32_t)(~wave_max_u32_scalar(~((uint32_t)lo ^ 0x80000000u)) ^ 0x80000000u);
      group_scale<true>(d, 0u, k0, k1, scl, inv, off);
    }
    for (uint32_t i = lane; i < cnt; i += kWave) {
      const float y = y_of(i);
      sh.code[g0 + i] = (uint8_t)code_bits<Q>(ASYM ? y - off : y, inv);
    }
    if (lane == 0u) {
      d.scales[first_group + g] = scl;
      if constexpr (ASYM) d.zp[first_group + g] = off;
    }
  }
  __syncthreads();
  // a8: the codes of the tail follow those of the main part (which ends on a multiple of 8 elements)
  if constexpr (Q == 128) {
    uint8_t* out = d.codes + d.numel;
    for (uint32_t i = lane; i < r; i += kWave) out[i] = sh.code[i];
  } else {
    uint8_t* out = d.codes + (d.numel >> 1);
    for (uint32_t b = lane; b < (r + 1u) / 2u; b += kWave) {
      const uint32_t lo = sh.code[2u * b] & 0xFu;
      const uint32_t hi = 2u * b + 1u < r ? (sh.code[2u * b + 1u] & 0xFu) : 0u;  // an odd end: the high nibble is 0
      out[b] = (uint8_t)(lo | (hi << 4));
    }
  }
}

// The whole tail of one tensor, by one wavefront (a workgroup of 64 threads).
__device__ __forceinline__ void compress_tail(const TensorDesc& d, TailShared& sh) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t r = d.tail;
  for (uint32_t i = lane; i < r; i += kWave) sh.raw[i] = d.src[d.numel + i];
  __syncthreads();
  tail_select(d, sh, r);
  if (d.mode != kModeNone) {
    // a4: the tail's outliers, ascending, behind those of the main part
    const uint32_t per_lane = (r + kWave - 1u) / kWave;
    const uint32_t i0 = lane * per_lane;
    const uint32_t i1 = i0 + per_lane < r ? i0 + per_lane : r;
    uint32_t mine = 0u;
    for (uint32_t i = i0; i < i1; ++i) mine += sh.out[i];
    sh.lane_cnt[lane] = mine;
    __syncthreads();
    uint32_t before = 0u, total_tail = 0u;
    for (uint32_t l = 0; l < (uint32_t)kWave; ++l) {
      const uint32_t c = sh.lane_cnt[l];
      before += l < lane ? c : 0u;
      total_tail += c;
    }
    const uint32_t main_tiles = d.n_tiles;  // tile_ptr[main_tiles] holds the main part's count
    const uint32_t total_main = main_tiles != 0u ? d.tile_ptr[main_tiles] : 0u;
    uint32_t pos = total_main + before;
    for (uint32_t i = i0; i < i1; ++i) {
      if (sh.out[i] == 0) continue;
      if (pos < d.cap) {
        d.idx[pos] = (int32_t)(d.numel + i);
        d.val[pos] = sh.raw[i];
      }
      ++pos;
    }
    __syncthreads();  // every lane has read tile_ptr[main_tiles] before it may be overwritten
    if (lane == 0u) {
      const uint32_t total = total_main + total_tail;
      if (main_tiles == 0u) d.tile_ptr[0] = 0u;
      d.tile_ptr[d.n_tiles_all] = total;
      d.status[0] = total;
      d.status[1] = total > d.cap ? 1u : 0u;
      d.status[2] = 0u;
      d.status[3] = 0u;
    }
  } else if (d.n_tiles == 0u && lane == 0u) {  // no main part whose kernel would have written the status
    d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
  }
  if (d.bits == 8u) {
    if (d.asym) tail_quantise<128, true>(d, sh, r); else tail_quantise<128, false>(d, sh, r);
  } else {
    if (d.asym) tail_quantise<8, true>(d, sh, r); else tail_quantise<8, false>(d, sh, r);
  }
}

// a9 / a10 for the tail
__device__ __forceinline__ void decompress_tail(const TensorDesc& d) {
  const uint32_t lane = (uint32_t)lane_id();
  const uint32_t r = d.tail;
  const uint64_t first_group = d.numel >> d.lgq;
  for (uint32_t i = lane; i < r; i += kWave) {
    int code;
    if (d.bits == 8u) code = (int)(int8_t)d.codes[d.numel + i];
    else code = ((int)((uint32_t)d.codes[(d.numel >> 1) + (i >> 1)] << (28u - 4u * (i & 1u)))) >> 28;
    const uint64_t grp = first_group + (i >> d.lgq);
    const float s = d.scales[grp];
    const float v = d.asym ? __fmaf_rn((float)code, s, d.zp[grp]) : (float)code * s;
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[d.numel + i] = v;
    else reinterpret_cast<uint16_t*>(d.dst)[d.numel + i] = (uint16_t)narrow_pair(v, 0.0f);
  }
  if (d.mode == kModeNone) return;
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the stores above are complete
  __syncthreads();
  const uint32_t tile = (uint32_t)(d.numel >> d.lgt);
  uint32_t p0 = d.tile_ptr[tile], p1 = d.tile_ptr[d.n_tiles_all];
  p1 = p1 < d.cap ? p1 : d.cap;
  for (uint32_t p = p0 + lane; p < p1; p += kWave) {
    const uint64_t i = (uint32_t)d.idx[p];
    if (i < d.numel || i >= d.numel + r) continue;  // the main part's, or a damaged stream
    const uint32_t pat = d.val[p];
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[i] = widen_lo(pat);
    else reinterpret_cast<uint16_t*>(d.dst)[i] = (uint16_t)pat;
  }
}

__global__ __launch_bounds__(kWave) void compress_tail_kernel(TensorDesc d) {
  __shared__ TailShared sh;
  compress_tail(d, sh);
}
__global__ __launch_bounds__(kWave) void compress_tail_batch_kernel(const TensorDesc* __restrict__ table,
                                                                    const uint32_t* __restrict__ members) {
  __shared__ TailShared sh;
  const TensorDesc d = table[members[blockIdx.x]];
  compress_tail(d, sh);
}
__global__ __launch_bounds__(kWave) void decompress_tail_kernel(TensorDesc d) { decompress_tail(d); }
__global__ __launch_bounds__(kWave) void decompress_tail_batch_kernel(const TensorDesc* __restrict__ table,
                                                                      const uint32_t* __restrict__ members) {
  const TensorDesc d = table[members[blockIdx.x]];
  decompress_tail(d);
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
