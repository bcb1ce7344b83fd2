// The fallback kernels for group sizes the tile kernels do not take.
#include "adacc_generic.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

TailFn compress_generic_fn(bool count_only) {
  return count_only ? compress_generic_kernel<true> : compress_generic_kernel<false>;
}
TailFn decompress_generic_fn() { return decompress_generic_kernel; }

}  // namespace ADACC_DT_NS
}  // namespace adacc
