// The fallback kernels for group sizes the tile kernels do not take.
#include "adacc_generic.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

TailFn compress_generic_fn(bool count_only, bool topk) {
  if (topk) return count_only ? compress_generic_kernel<true, true> : compress_generic_kernel<false, true>;
  return count_only ? compress_generic_kernel<true, false> : compress_generic_kernel<false, false>;
}
TailFn decompress_generic_fn() { return decompress_generic_kernel; }
uint32_t generic_threads() { return kSegThreads; }
uint32_t generic_lds_bytes(uint32_t tile_elems) { return kSegHeadBytes + 3u * tile_elems; }

}  // namespace ADACC_DT_NS
}  // namespace adacc
