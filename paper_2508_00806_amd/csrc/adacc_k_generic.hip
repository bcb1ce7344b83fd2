// The fallback kernels for group sizes the tile kernels do not take.
#include "adacc_generic.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

CompressFn compress_generic_fn(uint32_t tile_elems, bool fixup) {
  const uint32_t slices = ((tile_elems + 7u) / 8u + kSegThreads - 1u) / kSegThreads;  // octets per thread
  if (slices <= 2u) return fixup ? compress_generic_kernel<2, true> : compress_generic_kernel<2, false>;
  if (slices <= 4u) return fixup ? compress_generic_kernel<4, true> : compress_generic_kernel<4, false>;
  if (slices <= 6u) return fixup ? compress_generic_kernel<6, true> : compress_generic_kernel<6, false>;
  return fixup ? compress_generic_kernel<8, true> : compress_generic_kernel<8, false>;
}
TailFn decompress_generic_fn() { return decompress_generic_kernel; }
uint32_t generic_threads() { return kSegThreads; }
uint32_t generic_lds_bytes(uint32_t tile_elems, uint32_t gq, bool topk_groups) {
  const uint32_t slices = ((tile_elems + 7u) / 8u + kSegThreads - 1u) / kSegThreads;
  const uint32_t sl = slices <= 2u ? 2u : slices <= 4u ? 4u : slices <= 6u ? 6u : 8u;  // the kernel compress_generic_fn picks
  const uint32_t n_oct = sl * kSegThreads, n_grp = (tile_elems + gq - 1u) / gq;
  const uint32_t words = 8u * n_oct + 8u * n_grp;     // a, b, g0, g1
  const uint32_t patterns = topk_groups ? 24u * n_oct : 0u;  // 16-bit patterns and a byte per element
  return kSegHeadBytes + (words > patterns ? words : patterns);
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
