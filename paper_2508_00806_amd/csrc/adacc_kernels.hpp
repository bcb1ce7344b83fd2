// Kernel templates of libadacc.  Included by the translation units that instantiate them
// (one per outlier mode, one for decompression, one per batch kernel), so that the library builds
// in parallel; the host code reaches the instantiations through the getters of adacc_fn.hpp.
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_decompress.hpp"
#include "adacc_fn.hpp"

namespace adacc {

// ---- single tensor, compress: tiles are independent, one tile per wavefront, workgroups in the
// hardware's own order (which walks through memory front to back).
// the symmetric whole-tile TOPK kernels for 8-row tiles fit 4 wavefronts per SIMD when asked to
#ifndef ADACC_WHOLE8_MIN_WAVES
#define ADACC_WHOLE8_MIN_WAVES 4
#endif
#ifndef ADACC_COMPRESS_MIN_WAVES
#define ADACC_COMPRESS_MIN_WAVES 1
#endif
template <int MODE, int BITS, bool ASYM, int E, bool ROWWISE, bool WHOLE = false>
__global__ __launch_bounds__(kThreads, (E == 8 && WHOLE && !ASYM) ? ADACC_WHOLE8_MIN_WAVES : ADACC_COMPRESS_MIN_WAVES) void compress_kernel(TensorDesc d, uint32_t epoch) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg) {
    if constexpr (MODE == kModeNone) compress_tile_plain<BITS, ASYM, E, ROWWISE>(d, t);
    else compress_tile_outliers<MODE, BITS, ASYM, E, ROWWISE, WHOLE>(d, t, epoch);
  }
}

// TOPK whose statistics group is the whole tile has an encoder of its own
__device__ __forceinline__ bool topk_whole(const TensorDesc& d) { return d.lgs == d.lgt && d.lgq <= 11u; }

// d.n_tiles counts pieces of 2048 elements here
template <int BITS, bool ASYM, bool F32>
__global__ __launch_bounds__(kThreads) void decompress_kernel(TensorDesc d, uint32_t has_outliers) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg)
    decompress_tile<BITS, ASYM, 4, F32>(d, t, has_outliers != 0u);
}

// ---- batch
// Variants with tiles of 8 rows need about twice the registers of those with 4; a kernel that
// held both would run everything at the occupancy of the heaviest.  So the batch comes as two
// kernels over the same table, and a wavefront whose tensor belongs to the other one leaves.
template <int MODE, bool EIGHT_ROWS>
__device__ __forceinline__ void compress_dispatch_mode(const TensorDesc& d, uint32_t tile, uint32_t epoch) {
  if constexpr (!EIGHT_ROWS) {
    if (d.rowwise) {  // groups inside a row
      switch (d.variant & 6u) {
        case 0: compress_tile_outliers<MODE, 4, false, 4, true>(d, tile, epoch); break;
        case 2: compress_tile_outliers<MODE, 4, true, 4, true>(d, tile, epoch); break;
        case 4: compress_tile_outliers<MODE, 8, false, 4, true>(d, tile, epoch); break;
        default: compress_tile_outliers<MODE, 8, true, 4, true>(d, tile, epoch); break;
      }
      return;
    }
    switch (d.variant & 6u) {
      case 0: compress_tile_outliers<MODE, 4, false, 4, false>(d, tile, epoch); break;
      case 2: compress_tile_outliers<MODE, 4, true, 4, false>(d, tile, epoch); break;
      case 4: compress_tile_outliers<MODE, 8, false, 4, false>(d, tile, epoch); break;
      default: compress_tile_outliers<MODE, 8, true, 4, false>(d, tile, epoch); break;
    }
  } else {
    switch (d.variant & 6u) {
      case 0: compress_tile_outliers<MODE, 4, false, 8, false>(d, tile, epoch); break;
      case 2: compress_tile_outliers<MODE, 4, true, 8, false>(d, tile, epoch); break;
      case 4: compress_tile_outliers<MODE, 8, false, 8, false>(d, tile, epoch); break;
      default: compress_tile_outliers<MODE, 8, true, 8, false>(d, tile, epoch); break;
    }
  }
}

// TOPK over the whole tile: the specialised encoder
template <bool EIGHT_ROWS>
__device__ __forceinline__ void compress_dispatch_topk_whole(const TensorDesc& d, uint32_t tile, uint32_t epoch) {
  constexpr int kRows = EIGHT_ROWS ? 8 : 4;
  switch (d.variant & 6u) {
    case 0: compress_tile_outliers<kModeTopk, 4, false, kRows, false, true>(d, tile, epoch); break;
    case 2: compress_tile_outliers<kModeTopk, 4, true, kRows, false, true>(d, tile, epoch); break;
    case 4: compress_tile_outliers<kModeTopk, 8, false, kRows, false, true>(d, tile, epoch); break;
    default: compress_tile_outliers<kModeTopk, 8, true, kRows, false, true>(d, tile, epoch); break;
  }
}

// One launch for a group of tensors of a table: blockIdx.y picks the tensor (members[] holds the
// group's table entries), blockIdx.x its tiles, four per workgroup; workgroups past the end of a
// shorter tensor leave at once.  The host groups the tensors by register class (tiles of 4 or of 8
// rows: variants with 8 rows need about twice the registers, and a kernel that held both would run
// everything at the occupancy of the heaviest) and by size (tile counts within a factor of two), so
// few workgroups are empty; within a launch the hardware goes through the tensors one after the
// other, front to back.
// The kernel for tiles of 8 rows is held to 3 wavefronts per SIMD: the variants that matter
// (TOPK over the whole tile) fit, the rarely used ones spill a few registers.
#ifndef ADACC_BATCH8_MIN_WAVES
#define ADACC_BATCH8_MIN_WAVES 3
#endif
template <bool EIGHT_ROWS>
__global__ __launch_bounds__(kThreads, EIGHT_ROWS ? ADACC_BATCH8_MIN_WAVES : 1) void compress_batch_kernel(const TensorDesc* table, const uint32_t* members,
                                                                  uint32_t epoch) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  const TensorDesc d = table[members[blockIdx.y]];
  const uint32_t tile = blockIdx.x * kWavesPerWg + wave;
  if (tile >= d.n_tiles) return;
  switch (d.variant >> 3) {
    case kModeNone:
      if constexpr (!EIGHT_ROWS) {
        if (d.rowwise) {
          switch (d.variant & 6u) {
            case 0: compress_tile_plain<4, false, 4, true>(d, tile); break;
            case 2: compress_tile_plain<4, true, 4, true>(d, tile); break;
            case 4: compress_tile_plain<8, false, 4, true>(d, tile); break;
            default: compress_tile_plain<8, true, 4, true>(d, tile); break;
          }
          break;
        }
        switch (d.variant & 6u) {
          case 0: compress_tile_plain<4, false, 4, false>(d, tile); break;
          case 2: compress_tile_plain<4, true, 4, false>(d, tile); break;
          case 4: compress_tile_plain<8, false, 4, false>(d, tile); break;
          default: compress_tile_plain<8, true, 4, false>(d, tile); break;
        }
      } else {
        switch (d.variant & 6u) {
          case 0: compress_tile_plain<4, false, 8, false>(d, tile); break;
          case 2: compress_tile_plain<4, true, 8, false>(d, tile); break;
          case 4: compress_tile_plain<8, false, 8, false>(d, tile); break;
          default: compress_tile_plain<8, true, 8, false>(d, tile); break;
        }
      }
      break;
    case kModeAbs: compress_dispatch_mode<kModeAbs, EIGHT_ROWS>(d, tile, epoch); break;
    case kModeStd: compress_dispatch_mode<kModeStd, EIGHT_ROWS>(d, tile, epoch); break;
    default:
      if (topk_whole(d)) compress_dispatch_topk_whole<EIGHT_ROWS>(d, tile, epoch);
      else compress_dispatch_mode<kModeTopk, EIGHT_ROWS>(d, tile, epoch);
      break;
  }
}

// Batch decompression: the same grouping, over the 2048-element pieces of the tensors.
template <bool F32>
__global__ __launch_bounds__(kThreads) void decompress_batch_kernel(const TensorDesc* table, const uint32_t* members) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  const TensorDesc d = table[members[blockIdx.y]];
  const uint32_t piece = blockIdx.x * kWavesPerWg + wave;
  if (piece >= d.n_tiles) return;
  const bool ho = (d.variant >> 3) != kModeNone;
  switch (d.variant & 6u) {
    case 0: decompress_tile<4, false, 4, F32>(d, piece, ho); break;
    case 2: decompress_tile<4, true, 4, F32>(d, piece, ho); break;
    case 4: decompress_tile<8, false, 4, F32>(d, piece, ho); break;
    default: decompress_tile<8, true, 4, F32>(d, piece, ho); break;
  }
}

}  // namespace adacc
