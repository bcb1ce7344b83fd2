// Kernels for the end of a tensor whose length the group sizes do not divide.
#include "adacc_tail.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

TailFn compress_tail_fn() { return compress_tail_kernel; }
TailBatchFn compress_tail_batch_fn() { return compress_tail_batch_kernel; }
TailFn decompress_tail_fn() { return decompress_tail_kernel; }
TailBatchFn decompress_tail_batch_fn() { return decompress_tail_batch_kernel; }

}  // namespace ADACC_DT_NS
}  // namespace adacc
