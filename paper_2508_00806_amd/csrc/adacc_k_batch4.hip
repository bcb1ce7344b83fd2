// Instantiation of the batch compression kernel for tiles of 4 rows.
#include "adacc_kernels.hpp"

namespace adacc {

BatchCompressFn compress_batch_fn4() { return compress_batch_kernel<false>; }

}  // namespace adacc
