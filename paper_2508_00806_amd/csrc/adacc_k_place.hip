// The kernels that place the outliers in the stream (single tensor and batch): one workgroup per block
// of kPlaceTiles tiles of one tensor, whatever the method (the choice of the selection code for tiles
// that have to be looked at again is a uniform switch).
#include "adacc_kernels.hpp"

namespace adacc {

__device__ __forceinline__ void place_dispatch(const TensorDesc& d, uint32_t block, uint32_t epoch, PlaceShared& sh) {
  const bool e8 = (d.variant & 1u) != 0u;
  switch (d.variant >> 3) {
    case kModeAbs:
      if (d.rowwise) place_block<kModeAbs, 4, true, false>(d, block, false, sh);
      else if (e8) place_block<kModeAbs, 8, false, false>(d, block, false, sh);
      else place_block<kModeAbs, 4, false, false>(d, block, false, sh);
      break;
    case kModeStd:
      if (d.rowwise) place_block<kModeStd, 4, true, false>(d, block, false, sh);
      else if (e8) place_block<kModeStd, 8, false, false>(d, block, false, sh);
      else place_block<kModeStd, 4, false, false>(d, block, false, sh);
      break;
    case kModeTopk:
      // regular counts everywhere (the usual case): the compression kernel has placed everything already
      if (__hip_atomic_load(d.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) return;
      if (topk_whole(d)) {
        if (e8) place_block<kModeTopk, 8, false, true>(d, block, true, sh);
        else place_block<kModeTopk, 4, false, true>(d, block, true, sh);
      } else {
        if (e8) place_block<kModeTopk, 8, false, false>(d, block, true, sh);
        else place_block<kModeTopk, 4, false, false>(d, block, true, sh);
      }
      break;
    default: break;
  }
}

__global__ __launch_bounds__(kPlaceThreads) void place_kernel(TensorDesc d, uint32_t epoch) {
  __shared__ PlaceShared sh;
  place_dispatch(d, blockIdx.x, epoch, sh);
}

// Placement for a table of tensors: blocks of kPlaceTiles tiles are numbered across the tensors that
// keep outliers (first_block[]); tensors without outliers have no blocks.
__global__ __launch_bounds__(kPlaceThreads) void place_batch_kernel(const TensorDesc* table, const uint32_t* first_block,
                                                                    uint32_t n, uint32_t epoch) {
  __shared__ PlaceShared sh;
  // entries without blocks share their successor's first block; the bisection returns the last entry
  // that starts at or before this block, which is the one that owns it
  const TensorDesc d = table[find_entry(first_block, n, blockIdx.x)];
  place_dispatch(d, blockIdx.x - d.first_block, epoch, sh);
}

PlaceFn place_fn() { return place_kernel; }
PlaceBatchFn place_batch_fn() { return place_batch_kernel; }

}  // namespace adacc
