// Instantiations of the batch compression kernels for tiles of 8 rows.
#include "adacc_kernels.hpp"

namespace adacc {
namespace ADACC_DT_NS {

BatchCompressFn compress_batch_fn8(int kind) {
  return kind == kBatchTopk8 ? compress_batch_kernel<kBatchTopk8> : compress_batch_kernel<kBatchAny8>;
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
