// The kernels that place the outliers in the stream (single tensor and batch): one workgroup per block
// of kPlaceTiles tiles of one tensor, whatever the method (the choice of the selection code for tiles
// that have to be looked at again is a uniform switch).
#include "adacc_kernels.hpp"

namespace adacc {
namespace ADACC_DT_NS {

__device__ __forceinline__ void place_dispatch(const TensorDesc& d, uint32_t block, uint32_t epoch, PlaceShared& sh) {
  const bool e8 = (d.variant & 1u) != 0u;
  const bool from_sums = d.n_blocks > kPlaceDirectBlocks;
  if (d.generic != 0u) {
    // The fallback kernels select a segment's outliers again themselves (a second launch), where the slot did
    // not hold them or a TOPK group was irregular: here the offsets, and what the slots hold.
    uint32_t n_here, mine;
    if (d.mode == kModeTopk) {
      if (__hip_atomic_load(d.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) return;
      place_moves_block(d, block, false, false, sh, n_here, mine);
    } else {
      place_moves_block(d, block, from_sums, true, sh, n_here, mine);
    }
    return;
  }
  switch (d.variant >> 3) {
    case kModeAbs:
      if (d.rowwise) place_block<kModeAbs, 4, true, false>(d, block, from_sums, false, sh);
      else if (e8) place_block<kModeAbs, 8, false, false>(d, block, from_sums, false, sh);
      else place_block<kModeAbs, 4, false, false>(d, block, from_sums, false, sh);
      break;
    case kModeStd:
      if (d.rowwise) place_block<kModeStd, 4, true, false>(d, block, from_sums, false, sh);
      else if (e8) place_block<kModeStd, 8, false, false>(d, block, from_sums, false, sh);
      else place_block<kModeStd, 4, false, false>(d, block, from_sums, false, sh);
      break;
    case kModeTopk:
      // regular counts everywhere (the usual case): the compression kernel has placed everything already
      if (__hip_atomic_load(d.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) return;
      if (topk_whole(d)) {
        if (e8) place_block<kModeTopk, 8, false, true>(d, block, false, true, sh);
        else place_block<kModeTopk, 4, false, true>(d, block, false, true, sh);
      } else {
        if (e8) place_block<kModeTopk, 8, false, false>(d, block, false, true, sh);
        else place_block<kModeTopk, 4, false, false>(d, block, false, true, sh);
      }
      break;
    default: break;
  }
}

// single tensor: blockIdx.x is the block of tiles
__global__ __launch_bounds__(kPlaceThreads) void place_sum_kernel(TensorDesc d) {
  __shared__ uint32_t part[kPlaceThreads / kWave];
  place_sum_block(d, blockIdx.x, part);
}

// The selection code for tiles that have to be looked at again (rare) would take 173 registers and leave room
// for two wavefronts per SIMD; the kernel is a chain of dependent memory round trips, so it is held to 128.
__global__ __launch_bounds__(kPlaceThreads, 4) void place_kernel(TensorDesc d, uint32_t epoch) {
  __shared__ PlaceShared sh;
  place_dispatch(d, blockIdx.x, epoch, sh);
}

// a group of tensors of a table: blockIdx.y picks the tensor, blockIdx.x its block of tiles
__global__ __launch_bounds__(kPlaceThreads) void place_sum_batch_kernel(const TensorDesc* table, const uint32_t* members) {
  __shared__ uint32_t part[kPlaceThreads / kWave];
  const TensorDesc d = table[members[blockIdx.y]];
  if (blockIdx.x < d.n_blocks) place_sum_block(d, blockIdx.x, part);
}

__global__ __launch_bounds__(kPlaceThreads, 4) void place_batch_kernel(const TensorDesc* table, const uint32_t* members,
                                                                    uint32_t epoch) {
  __shared__ PlaceShared sh;
  const TensorDesc d = table[members[blockIdx.y]];
  if (blockIdx.x < d.n_blocks) place_dispatch(d, blockIdx.x, epoch, sh);
}

PlaceSumFn place_sum_fn() { return place_sum_kernel; }
PlaceFn place_fn() { return place_kernel; }
PlaceSumBatchFn place_sum_batch_fn() { return place_sum_batch_kernel; }
PlaceBatchFn place_batch_fn() { return place_batch_kernel; }

}  // namespace ADACC_DT_NS
}  // namespace adacc
