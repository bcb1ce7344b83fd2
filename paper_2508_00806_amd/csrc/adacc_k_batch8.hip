// Instantiation of the batch compression kernel for tiles of 8 rows.
#include "adacc_kernels.hpp"

namespace adacc {

BatchCompressFn compress_batch_fn8() { return compress_batch_kernel<true>; }

}  // namespace adacc
