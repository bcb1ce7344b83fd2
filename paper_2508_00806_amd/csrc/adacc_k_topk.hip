// Instantiations of the single-tensor compression kernels, outlier mode topk.
#include "adacc_kernels.hpp"

namespace adacc {
namespace ADACC_DT_NS {

template <int BITS, bool ASYM>
static CompressFn pick(bool e8, bool whole, bool rows) {
  if (rows) return compress_kernel<kModeTopk, BITS, ASYM, 4, true>;  // groups inside a row: tiles of 4 rows
  if (whole) return e8 ? compress_kernel<kModeTopk, BITS, ASYM, 8, false, true> : compress_kernel<kModeTopk, BITS, ASYM, 4, false, true>;
  return e8 ? compress_kernel<kModeTopk, BITS, ASYM, 8, false> : compress_kernel<kModeTopk, BITS, ASYM, 4, false>;
}

CompressFn compress_fn_topk(uint32_t bits, uint32_t asym, bool e8, bool whole, bool rows) {
  if (bits == 4) return asym ? pick<4, true>(e8, whole, rows) : pick<4, false>(e8, whole, rows);
  return asym ? pick<8, true>(e8, whole, rows) : pick<8, false>(e8, whole, rows);
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
