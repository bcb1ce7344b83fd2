// Instantiations of the single-tensor compression kernels, outlier mode std.
#include "adacc_kernels.hpp"

namespace adacc {
namespace ADACC_DT_NS {

template <int BITS, bool ASYM>
static CompressFn pick(bool e8, bool rowwise) {
  if (rowwise) return compress_kernel<kModeStd, BITS, ASYM, 4, true>;
  return e8 ? compress_kernel<kModeStd, BITS, ASYM, 8, false> : compress_kernel<kModeStd, BITS, ASYM, 4, false>;
}

CompressFn compress_fn_std(uint32_t bits, uint32_t asym, bool e8, bool rowwise) {
  if (bits == 4) return asym ? pick<4, true>(e8, rowwise) : pick<4, false>(e8, rowwise);
  return asym ? pick<8, true>(e8, rowwise) : pick<8, false>(e8, rowwise);
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
