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

// LDS bytes one wavefront needs to stage a tile while outliers are patched in
template <int E, bool F32>
constexpr int decompress_lds_per_wave() { return E * kRow * (F32 ? 4 : 2); }

// Decompression always works on pieces of E = 4 rows (2048 elements), whatever the tile of the
// blob: a piece of a 4096-element tile looks through the outliers of the whole tile and takes
// those that fall inside it.  (Pieces of 8 rows would need twice the staging area in LDS and
// leave room for 5 instead of 8 workgroups per CU.)
template <int BITS, bool ASYM, int E, bool F32>
__device__ __forceinline__ void decompress_tile(const TensorDesc& d, uint32_t tile /* piece */, bool has_outliers,
                                                unsigned char* lds /* this wavefront's slice */) {
  static_assert(E == 4, "pieces of 2048 elements");
  const int lane = (int)__lane_id();
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const uint64_t lane_base = tile_base + (uint64_t)lane * kOct;

  // this tile's slice of the outlier stream
  uint32_t p0 = 0u, p1 = 0u;
  if (has_outliers) {
    p0 = d.tile_ptr[tile >> d.ptr_shift];
    p1 = d.tile_ptr[(tile >> d.ptr_shift) + 1];
    p0 = p0 < d.cap ? p0 : d.cap;
    p1 = p1 < d.cap ? p1 : d.cap;
    if (p1 < p0) p1 = p0;
  }
  const bool patch = p1 > p0;  // uniform over the wavefront

  // ---- a9: unpack and dequantise
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
      const float4 a = make_float4(v[0], v[1], v[2], v[3]);
      const float4 b = make_float4(v[4], v[5], v[6], v[7]);
      if (patch) {
        float4* p = reinterpret_cast<float4*>(lds + ((size_t)j * kRow + (size_t)lane * kOct) * 4);
        p[0] = a; p[1] = b;
      } else {
        float* p = reinterpret_cast<float*>(d.dst) + e0;
        ADACC_STORE16(p, make_uint4(__float_as_uint(a.x), __float_as_uint(a.y), __float_as_uint(a.z), __float_as_uint(a.w)));
        ADACC_STORE16(p + 4, make_uint4(__float_as_uint(b.x), __float_as_uint(b.y), __float_as_uint(b.z), __float_as_uint(b.w)));
      }
    } else {
      uint4 w;
      w.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
      w.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
      w.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
      w.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
      if (patch)
        *reinterpret_cast<uint4*>(lds + ((size_t)j * kRow + (size_t)lane * kOct) * 2) = w;
      else
        ADACC_STORE16(reinterpret_cast<uint16_t*>(d.dst) + e0, w);
    }
  }

  // ---- a10: outliers overwrite their positions, then the staged tile is stored
  if (patch) {
    // LDS operations of one wavefront execute in program order; the fences only keep the
    // compiler from reordering the differently typed accesses to the slice
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (uint32_t cpos = p0 + (uint32_t)lane; cpos < p1; cpos += kWave) {
      const int64_t local = (int64_t)(uint32_t)d.idx[cpos] - (int64_t)tile_base;
      const uint32_t bits = d.val[cpos];
      if (local >= 0 && local < (int64_t)(E * kRow)) {  // a damaged stream must not write outside the slice
        if constexpr (F32)
          *reinterpret_cast<uint32_t*>(lds + (size_t)local * 4) = bits << 16;
        else
          *reinterpret_cast<uint16_t*>(lds + (size_t)local * 2) = (uint16_t)bits;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint64_t e0 = lane_base + (uint64_t)j * kRow;
      if (e0 >= d.numel) continue;
      if constexpr (F32) {
        const float4* p = reinterpret_cast<const float4*>(lds + ((size_t)j * kRow + (size_t)lane * kOct) * 4);
        float* q = reinterpret_cast<float*>(d.dst) + e0;
        const float4 a = p[0], b = p[1];
        ADACC_STORE16(q, make_uint4(__float_as_uint(a.x), __float_as_uint(a.y), __float_as_uint(a.z), __float_as_uint(a.w)));
        ADACC_STORE16(q + 4, make_uint4(__float_as_uint(b.x), __float_as_uint(b.y), __float_as_uint(b.z), __float_as_uint(b.w)));
      } else {
        ADACC_STORE16(reinterpret_cast<uint16_t*>(d.dst) + e0,
                      *reinterpret_cast<const uint4*>(lds + ((size_t)j * kRow + (size_t)lane * kOct) * 2));
      }
    }
    __builtin_amdgcn_wave_barrier();  // the slice is reused by this wavefront's next tile
  }
}

}  // namespace adacc
