// Instantiations of the batch compression kernels for tiles of 4 rows.
#include "adacc_kernels.hpp"

namespace adacc {
namespace ADACC_DT_NS {

BatchCompressFn compress_batch_fn4(int kind) {
  if (kind == kBatchRows4) return compress_batch_kernel<kBatchRows4>;
  if (kind == kBatchTopk4) return compress_batch_kernel<kBatchTopk4>;
  return compress_batch_kernel<kBatchAny4>;
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
