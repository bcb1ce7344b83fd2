// Instantiations of the decompression kernels (single tensor and batch).
#include "adacc_kernels.hpp"

namespace adacc {
namespace ADACC_DT_NS {

DecompressFn decompress_fn(uint32_t bits, uint32_t asym, bool f32) {
  if (bits == 4) {
    if (asym) return f32 ? decompress_kernel<4, true, true> : decompress_kernel<4, true, false>;
    return f32 ? decompress_kernel<4, false, true> : decompress_kernel<4, false, false>;
  }
  if (asym) return f32 ? decompress_kernel<8, true, true> : decompress_kernel<8, true, false>;
  return f32 ? decompress_kernel<8, false, true> : decompress_kernel<8, false, false>;
}

BatchDecompressFn decompress_batch_fn(bool f32) {
  return f32 ? decompress_batch_kernel<true> : decompress_batch_kernel<false>;
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
