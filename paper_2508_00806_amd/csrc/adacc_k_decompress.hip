// Instantiations of the decompression kernels (single tensor and batch).
#include "adacc_kernels.hpp"

namespace adacc {

template <int BITS, bool ASYM>
static DecompressFn pick(bool e8, bool f32) {
  if (e8) return f32 ? decompress_kernel<BITS, ASYM, 8, true> : decompress_kernel<BITS, ASYM, 8, false>;
  return f32 ? decompress_kernel<BITS, ASYM, 4, true> : decompress_kernel<BITS, ASYM, 4, false>;
}

DecompressFn decompress_fn(uint32_t bits, uint32_t asym, bool e8, bool f32) {
  if (bits == 4) return asym ? pick<4, true>(e8, f32) : pick<4, false>(e8, f32);
  return asym ? pick<8, true>(e8, f32) : pick<8, false>(e8, f32);
}

BatchDecompressFn decompress_batch_fn(bool f32, bool eight_rows) {
  if (eight_rows) return f32 ? decompress_batch_kernel<true, true> : decompress_batch_kernel<false, true>;
  return f32 ? decompress_batch_kernel<true, false> : decompress_batch_kernel<false, false>;
}

}  // namespace adacc
