// Decompression of one tile by one wavefront (Section 3.2: X^ = code * S, resp. code * S + O,
// then the outliers are written back; Fig. 3(c) decompression workflow).
#pragma once

#include "adacc_common.hpp"

namespace adacc {

// binary32 -> bf16, round to nearest even (dequantised values are always finite)
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// Decompression always works on pieces of E = 4 rows (2048 elements), whatever the tile of the
// blob: a piece of a 4096-element tile looks through the outliers of the whole tile and takes
// those that fall inside it.
//
// The outliers are written over the dequantised values in memory: the piece is stored first, the
// wavefront waits until those stores have reached the L2 (its store counter at zero), and then
// stores the outliers of the piece, 2 (or 4) bytes each, to their positions.  Both rounds of
// stores come from the same wavefront and the second is issued only after the first is complete,
// so the outliers are what stays.  (Staging the piece in LDS to patch it there cost a round trip
// through LDS for every piece of a TOPK tensor, a third of the kernel's time.)
template <int BITS, bool ASYM, int E, bool F32>
__device__ __forceinline__ void decompress_tile(const TensorDesc& d, uint32_t tile /* piece */, bool has_outliers) {
  static_assert(E == 4, "pieces of 2048 elements");
  const int lane = (int)__lane_id();
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const uint64_t lane_base = tile_base + (uint64_t)lane * kOct;

  // this tile's slice of the outlier stream; its first 64 entries are fetched before anything else
  uint32_t p0 = 0u, p1 = 0u;
  if (has_outliers) {
    p0 = d.tile_ptr[tile >> d.ptr_shift];
    p1 = d.tile_ptr[(tile >> d.ptr_shift) + 1];
    p0 = p0 < d.cap ? p0 : d.cap;
    p1 = p1 < d.cap ? p1 : d.cap;
    if (p1 < p0) p1 = p0;
  }
  const bool patch = p1 > p0;  // uniform over the wavefront
  uint32_t o_idx = 0u, o_val = 0u;
  if (patch && p0 + (uint32_t)lane < p1) {
    o_idx = (uint32_t)d.idx[p0 + (uint32_t)lane];
    o_val = d.val[p0 + (uint32_t)lane];
  }

  // ---- a9: unpack, dequantise, store
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint64_t e0 = lane_base + (uint64_t)j * kRow;
    if (e0 >= d.numel) continue;
    int c[kOct];
    if constexpr (BITS == 8) {
      const uint2 w = *reinterpret_cast<const uint2*>(d.codes + e0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        c[e] = (int)(int8_t)((w.x >> (8 * e)) & 0xFFu);
        c[4 + e] = (int)(int8_t)((w.y >> (8 * e)) & 0xFFu);
      }
    } else {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(d.codes + (e0 >> 1));
#pragma unroll
      for (int e = 0; e < kOct; ++e) c[e] = ((int)(w << (28 - 4 * e))) >> 28;  // sign-extended nibble
    }
    const uint64_t g = e0 >> d.lgq;
    const float s = d.scales[g];
    float o = 0.0f;
    if constexpr (ASYM) o = d.zp[g];
    float v[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) v[e] = ASYM ? __fmaf_rn((float)c[e], s, o) : (float)c[e] * s;

    if constexpr (F32) {
      float* p = reinterpret_cast<float*>(d.dst) + e0;
      ADACC_STORE16(p, make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
      ADACC_STORE16(p + 4, make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])));
    } else {
      uint4 w;
      w.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
      w.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
      w.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
      w.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
      ADACC_STORE16(reinterpret_cast<uint16_t*>(d.dst) + e0, w);
    }
  }

  // ---- a10: the outliers overwrite their positions
  if (patch) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the stores above are complete
    const uint64_t piece_end = tile_base + (uint64_t)(E * kRow) < d.numel ? tile_base + (uint64_t)(E * kRow) : d.numel;
    for (uint32_t cpos = p0 + (uint32_t)lane; cpos < p1; cpos += kWave) {
      if (cpos >= p0 + (uint32_t)kWave) {  // past the entries fetched at the start
        o_idx = (uint32_t)d.idx[cpos];
        o_val = d.val[cpos];
      }
      const uint64_t i = o_idx;
      if (i >= tile_base && i < piece_end) {  // a damaged stream must not write outside the piece
        if constexpr (F32) reinterpret_cast<uint32_t*>(d.dst)[i] = o_val << 16;
        else reinterpret_cast<uint16_t*>(d.dst)[i] = (uint16_t)o_val;
      }
    }
  }
}

}  // namespace adacc
