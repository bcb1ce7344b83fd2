// Kernel templates of libadacc.  Included by the translation units that instantiate them
// (one per outlier mode, one for decompression, one per batch kernel), so that the library builds
// in parallel; the host code reaches the instantiations through the getters of adacc_fn.hpp.
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_decompress.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

// ---- single tensor, compress: tiles are independent, one tile per wavefront, workgroups in the
// hardware's own order (which walks through memory front to back).
// Wavefronts per SIMD the register allocation of a variant is held to (the compiler would otherwise
// spend registers on overlapping the rows of a tile, which pays less than another resident
// wavefront): encoders that take a tile row by row need little beyond the raw octets.
template <int E, bool ROWWISE, bool WHOLE>
constexpr int compress_min_waves() {
  if (ROWWISE) return 6;
  if (WHOLE) return E == 8 ? 7 : 8;
  return E == 8 ? 2 : 4;
}
template <int MODE, int BITS, bool ASYM, int E, bool ROWWISE, bool WHOLE = false>
__global__ __launch_bounds__(kThreads, (compress_min_waves<E, ROWWISE, WHOLE>())) void compress_kernel(TensorDesc d, uint32_t epoch) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  // one tile per wavefront and no loop: inside a loop over tiles the compiler would prepare, ahead of
  // the loop, the lane's addresses for every group size the encoders can be asked for
  const uint32_t t = blockIdx.x * kWavesPerWg + wave;
  if (t >= d.n_tiles) return;
  if constexpr (MODE == kModeNone) compress_tile_plain<BITS, ASYM, E, ROWWISE>(d, t);
  else compress_tile_outliers<MODE, BITS, ASYM, E, ROWWISE, WHOLE>(d, t, epoch);
}

// TOPK whose statistics group is the whole tile, with quantisation groups inside a row, has an encoder of its own
__device__ __forceinline__ bool topk_whole(const TensorDesc& d) { return d.lgs == d.lgt && d.lgq <= 9u; }

// d.n_tiles counts pieces of 2048 elements here
template <int BITS, bool ASYM, bool F32>
__global__ __launch_bounds__(kThreads) void decompress_kernel(TensorDesc d, uint32_t has_outliers) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  __shared__ __attribute__((aligned(16))) DecompressShared shared;
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg)
    decompress_tile<BITS, ASYM, 4, F32>(d, t, has_outliers != 0u, shared);
}

// ---- batch
// One launch for a group of tensors of a table: blockIdx.y picks the tensor (members[] holds the
// group's table entries), blockIdx.x its tiles, four per workgroup; workgroups past the end of a
// shorter tensor leave at once.  The host groups the tensors by kernel and by size (tile counts
// within a factor of two), so few workgroups are empty; within a launch the hardware goes through
// the tensors one after the other, front to back.
// A kernel holds as many wavefronts per SIMD as its heaviest variant allows, so the variants come
// in five kernels by weight:
//   kBatchRows4   tiles of 4 rows, all groups inside a row (TOPK: over the quantisation groups)   lightest
//   kBatchAny4    tiles of 4 rows, any other grouping
//   kBatchTopk4   tiles of 4 rows, TOPK over the whole tile, quantisation groups inside a row
//   kBatchAny8    tiles of 8 rows, general encoder                                   heaviest
//   kBatchTopk8   tiles of 8 rows, TOPK over the whole tile, quantisation groups inside a row

template <int MODE, int E, bool ROWWISE, bool WHOLE>
__device__ __forceinline__ void compress_dispatch(const TensorDesc& d, uint32_t tile, uint32_t epoch) {
  if constexpr (MODE == kModeNone) {
    switch (d.variant & 6u) {
      case 0: compress_tile_plain<4, false, E, ROWWISE>(d, tile); break;
      case 2: compress_tile_plain<4, true, E, ROWWISE>(d, tile); break;
      case 4: compress_tile_plain<8, false, E, ROWWISE>(d, tile); break;
      default: compress_tile_plain<8, true, E, ROWWISE>(d, tile); break;
    }
  } else {
    switch (d.variant & 6u) {
      case 0: compress_tile_outliers<MODE, 4, false, E, ROWWISE, WHOLE>(d, tile, epoch); break;
      case 2: compress_tile_outliers<MODE, 4, true, E, ROWWISE, WHOLE>(d, tile, epoch); break;
      case 4: compress_tile_outliers<MODE, 8, false, E, ROWWISE, WHOLE>(d, tile, epoch); break;
      default: compress_tile_outliers<MODE, 8, true, E, ROWWISE, WHOLE>(d, tile, epoch); break;
    }
  }
}

template <int KIND>
constexpr int batch_min_waves() {
  return KIND == kBatchRows4 ? 6 : KIND == kBatchTopk4 ? 8 : KIND == kBatchTopk8 ? 7 : KIND == kBatchAny4 ? 4 : 2;
}

template <int KIND>
__global__ __launch_bounds__(kThreads, (batch_min_waves<KIND>())) void compress_batch_kernel(const TensorDesc* table, const uint32_t* members,
                                                                  uint32_t epoch) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  // members == nullptr: the group's entries are table[0 .. gridDim.y) themselves (the host lays the table out in the
  // order of these launches): one round trip to memory less before the wavefront's first load
  const TensorDesc d = table[members ? members[blockIdx.y] : blockIdx.y];
  const uint32_t tile = blockIdx.x * kWavesPerWg + wave;
  if (tile >= d.n_tiles) return;
  constexpr int E = (KIND == kBatchAny8 || KIND == kBatchTopk8) ? 8 : 4;
  if constexpr (KIND == kBatchTopk4 || KIND == kBatchTopk8) {
    compress_dispatch<kModeTopk, E, false, true>(d, tile, epoch);
  } else {
    constexpr bool ROWWISE = KIND == kBatchRows4;
    switch (d.variant >> 3) {
      case kModeNone: compress_dispatch<kModeNone, E, ROWWISE, false>(d, tile, epoch); break;
      case kModeAbs: compress_dispatch<kModeAbs, E, ROWWISE, false>(d, tile, epoch); break;
      case kModeStd: compress_dispatch<kModeStd, E, ROWWISE, false>(d, tile, epoch); break;
      default: compress_dispatch<kModeTopk, E, ROWWISE, false>(d, tile, epoch); break;
    }
  }
}

// Batch decompression: the same grouping, over the 2048-element pieces of the tensors.
// members == nullptr: the group's entries are table[0 .. gridDim.y) themselves (the host lays the table out in
// the order of the launches), which saves the wavefront one of its two round trips to memory before its first load.
template <bool F32>
__global__ __launch_bounds__(kThreads) void decompress_batch_kernel(const TensorDesc* table, const uint32_t* members) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  const TensorDesc d = table[members ? members[blockIdx.y] : blockIdx.y];
  const uint32_t piece = blockIdx.x * kWavesPerWg + wave;
  if (piece >= d.n_tiles) return;
  const bool ho = (d.variant >> 3) != kModeNone;
  __shared__ __attribute__((aligned(16))) DecompressShared shared;
  switch (d.variant & 6u) {
    case 0: decompress_tile<4, false, 4, F32>(d, piece, ho, shared); break;
    case 2: decompress_tile<4, true, 4, F32>(d, piece, ho, shared); break;
    case 4: decompress_tile<8, false, 4, F32>(d, piece, ho, shared); break;
    default: decompress_tile<8, true, 4, F32>(d, piece, ho, shared); break;
  }
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
