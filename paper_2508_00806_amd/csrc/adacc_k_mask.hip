// Dropout mask of attention layers (Section 3.2, list of layer-specific schemes): byte format to bit
// format and back, lossless.  Element i of the mask (zero = dropped, anything else = kept) is bit
// i % 8 of byte i / 8.  Both kernels are plain streams (1.125 bytes per element).
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

constexpr int kMaskAhead = 8;  // 16-byte pieces per lane and round

// A lane turns 16 mask bytes (one 16-byte load) into 16 bits; consecutive lanes take consecutive
// pieces, so every load instruction of a wavefront covers 1 KiB without gaps and every store 128 bytes.
__global__ __launch_bounds__(kThreads) void mask_pack_kernel(const uint8_t* __restrict__ mask, uint64_t n,
                                                             uint8_t* __restrict__ bits) {
  const uint64_t n_pieces = n / 16u;
  // a workgroup takes kMaskAhead * 4 KiB of mask in one piece per round
  constexpr uint64_t stride = kThreads;
  const uint64_t me = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (uint64_t p0 = (uint64_t)blockIdx.x * (kThreads * kMaskAhead) + threadIdx.x; p0 < n_pieces;
       p0 += (uint64_t)gridDim.x * (kThreads * kMaskAhead)) {
    uint4 v[kMaskAhead];
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t p = p0 + (uint64_t)i * stride;
      v[i] = load_stream16(reinterpret_cast<const uint4*>(mask) + (p < n_pieces ? p : p0));  // a piece past the end re-reads the first one
    }
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t p = p0 + (uint64_t)i * stride;
      if (p >= n_pieces) continue;
      const uint32_t out = bytes_to_nibble(v[i].x) | (bytes_to_nibble(v[i].y) << 4) |
                           (bytes_to_nibble(v[i].z) << 8) | (bytes_to_nibble(v[i].w) << 12);
      reinterpret_cast<uint16_t*>(bits)[p] = (uint16_t)out;
    }
  }
  // the last n % 16 elements, byte by byte
  if (me == 0) {
    for (uint64_t b = n_pieces * 2u; b < (n + 7u) / 8u; ++b) {
      uint32_t out = 0u;
      for (uint32_t e = 0; e < 8u; ++e)
        if (b * 8u + e < n && mask[b * 8u + e] != 0) out |= 1u << e;
      bits[b] = (uint8_t)out;
    }
  }
}

__global__ __launch_bounds__(kThreads) void mask_unpack_kernel(const uint8_t* __restrict__ bits, uint64_t n,
                                                               uint8_t* __restrict__ mask) {
  const uint64_t n_pieces = n / 16u;
  // a workgroup takes kMaskAhead * 4 KiB of mask in one piece per round
  constexpr uint64_t stride = kThreads;
  const uint64_t me = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  for (uint64_t p0 = (uint64_t)blockIdx.x * (kThreads * kMaskAhead) + threadIdx.x; p0 < n_pieces;
       p0 += (uint64_t)gridDim.x * (kThreads * kMaskAhead)) {
    uint32_t v[kMaskAhead];
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t p = p0 + (uint64_t)i * stride;
      v[i] = reinterpret_cast<const uint16_t*>(bits)[p < n_pieces ? p : p0];
    }
#pragma unroll
    for (int i = 0; i < kMaskAhead; ++i) {
      const uint64_t p = p0 + (uint64_t)i * stride;
      if (p >= n_pieces) continue;
      uint4 w;
      w.x = nibble_to_bytes(v[i] & 0xFu);
      w.y = nibble_to_bytes((v[i] >> 4) & 0xFu);
      w.z = nibble_to_bytes((v[i] >> 8) & 0xFu);
      w.w = nibble_to_bytes((v[i] >> 12) & 0xFu);
      store_stream16(reinterpret_cast<uint4*>(mask) + p, w);
    }
  }
  if (me == 0) {
    for (uint64_t i = n_pieces * 16u; i < n; ++i) mask[i] = (uint8_t)((bits[i / 8u] >> (i % 8u)) & 1u);
  }
}

MaskFn mask_pack_fn() { return mask_pack_kernel; }
MaskFn mask_unpack_fn() { return mask_unpack_kernel; }

}  // namespace adacc
