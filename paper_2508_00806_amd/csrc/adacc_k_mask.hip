// Dropout mask of attention layers (Section 3.2, list of layer-specific schemes): byte format to bit
// format and back, lossless.  Element i of the mask (zero = dropped, anything else = kept) is bit
// i % 8 of byte i / 8.  Both kernels are plain streams (1.125 bytes per element): a lane turns 32
// mask bytes (two 16-byte loads) into one 32-bit word, or the other way round; consecutive lanes
// take consecutive words, so a wavefront reads 2 KiB and writes 256 bytes in one piece.
#include "adacc_common.hpp"
#include "adacc_fn.hpp"

namespace adacc {

// 4 mask bytes -> 4 bits (byte k -> bit k)
__device__ __forceinline__ uint32_t bytes_to_nibble(uint32_t w) {
  const uint32_t nz = (((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | w) & 0x80808080u;  // bit 7 of a byte: the byte is not zero
  // bytes b0..b3 (0 or 1) times 2^3 + 2^10 + 2^17 + 2^24: every product bit comes from one term only, and
  // bits 24..27 are b0..b3
  return ((nz >> 7) * 0x01020408u) >> 24;
}
// 4 bits -> 4 bytes of 0 / 1
__device__ __forceinline__ uint32_t nibble_to_bytes(uint32_t nib) {
  return (nib * 0x00204081u) & 0x01010101u;  // bit k lands on bit 8k; the other products fall between and are masked
}

constexpr int kMaskAhead = 4;  // words per lane and round: 8 loads of 16 bytes in flight

__global__ __launch_bounds__(kThreads) void mask_pack_kernel(const uint8_t* __restrict__ mask, uint64_t n,
                                                             uint8_t* __restrict__ bits) {
  const uint64_t n_words = n / 32u;
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  const uint64_t me = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (uint64_t w0 = me; w0 < n_words; w0 += stride * kMaskAhead) {
    uint4 v[kMaskAhead][2];
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t w = w0 + (uint64_t)i * stride;
      const uint64_t wl = w < n_words ? w : w0;  // a word past the end re-reads this lane's first one
      v[i][0] = reinterpret_cast<const uint4*>(mask)[2 * wl];
      v[i][1] = reinterpret_cast<const uint4*>(mask)[2 * wl + 1];
    }
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t w = w0 + (uint64_t)i * stride;
      if (w >= n_words) continue;
      const uint32_t out = bytes_to_nibble(v[i][0].x) | (bytes_to_nibble(v[i][0].y) << 4) |
                           (bytes_to_nibble(v[i][0].z) << 8) | (bytes_to_nibble(v[i][0].w) << 12) |
                           (bytes_to_nibble(v[i][1].x) << 16) | (bytes_to_nibble(v[i][1].y) << 20) |
                           (bytes_to_nibble(v[i][1].z) << 24) | (bytes_to_nibble(v[i][1].w) << 28);
      reinterpret_cast<uint32_t*>(bits)[w] = out;
    }
  }
  // the last n % 32 elements, byte by byte
  if (me == 0) {
    const uint64_t done = n_words * 32u;
    for (uint64_t b = done / 8u; b < (n + 7u) / 8u; ++b) {
      uint32_t out = 0u;
      for (uint32_t e = 0; e < 8u; ++e)
        if (b * 8u + e < n && mask[b * 8u + e] != 0) out |= 1u << e;
      bits[b] = (uint8_t)out;
    }
  }
}

__global__ __launch_bounds__(kThreads) void mask_unpack_kernel(const uint8_t* __restrict__ bits, uint64_t n,
                                                               uint8_t* __restrict__ mask) {
  const uint64_t n_words = n / 32u;
  const uint64_t stride = (uint64_t)gridDim.x * kThreads;
  const uint64_t me = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (uint64_t w0 = me; w0 < n_words; w0 += stride * kMaskAhead) {
    uint32_t v[kMaskAhead];
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t w = w0 + (uint64_t)i * stride;
      v[i] = reinterpret_cast<const uint32_t*>(bits)[w < n_words ? w : w0];
    }
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t w = w0 + (uint64_t)i * stride;
      if (w >= n_words) continue;
      uint4 lo, hi;
      lo.x = nibble_to_bytes(v[i] & 0xFu);         lo.y = nibble_to_bytes((v[i] >> 4) & 0xFu);
      lo.z = nibble_to_bytes((v[i] >> 8) & 0xFu);  lo.w = nibble_to_bytes((v[i] >> 12) & 0xFu);
      hi.x = nibble_to_bytes((v[i] >> 16) & 0xFu); hi.y = nibble_to_bytes((v[i] >> 20) & 0xFu);
      hi.z = nibble_to_bytes((v[i] >> 24) & 0xFu); hi.w = nibble_to_bytes(v[i] >> 28);
      reinterpret_cast<uint4*>(mask)[2 * w] = lo;
      reinterpret_cast<uint4*>(mask)[2 * w + 1] = hi;
    }
  }
  if (me == 0) {
    for (uint64_t i = n_words * 32u; i < n; ++i) mask[i] = (uint8_t)((bits[i / 8u] >> (i % 8u)) & 1u);
  }
}

MaskFn mask_pack_fn() { return mask_pack_kernel; }
MaskFn mask_unpack_fn() { return mask_unpack_kernel; }

}  // namespace adacc
