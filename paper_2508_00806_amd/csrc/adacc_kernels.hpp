// Kernel templates of libadacc.  Included by the translation units that instantiate them
// (one per outlier mode, one for decompression, one per batch kernel), so that the library builds
// in parallel; the host code reaches the instantiations through the getters of adacc_fn.hpp.
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_decompress.hpp"
#include "adacc_fn.hpp"

namespace adacc {

// ---- single tensor, compress.  With outliers: run = 4 * workgroup + wavefront, and the grid is
// exactly ceil(n_units / 4) workgroups, because the chained scan relies on runs being started
// in index order.  NONE: tiles are independent, grid-stride loop over tiles.
// the symmetric whole-tile TOPK kernels for 8-row tiles fit 4 wavefronts per SIMD when asked to
#ifndef ADACC_WHOLE8_MIN_WAVES
#define ADACC_WHOLE8_MIN_WAVES 4
#endif
#ifndef ADACC_COMPRESS_MIN_WAVES
#define ADACC_COMPRESS_MIN_WAVES 1
#endif
template <int MODE, int BITS, bool ASYM, int E, bool ROWWISE, bool WHOLE = false>
__global__ __launch_bounds__(kThreads, (E == 8 && WHOLE && !ASYM) ? ADACC_WHOLE8_MIN_WAVES : ADACC_COMPRESS_MIN_WAVES) void compress_kernel(TensorDesc d, uint64_t* state1,
                                                                                      uint64_t* state2, uint32_t tag,
                                                                                      uint32_t spin_limit) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  if constexpr (MODE == kModeNone) {
    for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg)
      compress_tile_plain<BITS, ASYM, E, ROWWISE>(d, t);
  } else {
    __shared__ WaveStage stage[kWavesPerWg];
    const ScanCtx sc{state1, state2, tag, spin_limit};
    const uint32_t u = blockIdx.x * kWavesPerWg + wave;
    if (u < d.n_units) compress_run<MODE, BITS, ASYM, E, ROWWISE, WHOLE>(d, u, sc, &stage[wave]);
  }
}

// d.n_tiles counts pieces of 2048 elements here
template <int BITS, bool ASYM, bool F32>
__global__ __launch_bounds__(kThreads) void decompress_kernel(TensorDesc d, uint32_t has_outliers) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWavesPerWg * decompress_lds_per_wave<4, F32>()];
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  unsigned char* slice = lds + wave * decompress_lds_per_wave<4, F32>();
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg)
    decompress_tile<BITS, ASYM, 4, F32>(d, t, has_outliers != 0u, slice);
}

// ---- batch: a launch-wide tile numbering over all tensors of the table
template <bool BY_UNIT>
__device__ __forceinline__ uint32_t find_tensor(const TensorDesc* table, uint32_t n, uint32_t g) {
  uint32_t lo = 0u, hi = n;  // first_tile / first_unit ascend; find the last entry that starts at or before g
  while (hi - lo > 1u) {
    const uint32_t mid = (lo + hi) >> 1;
    const uint32_t first = BY_UNIT ? table[mid].first_unit : table[mid].first_tile;
    if (first <= g) lo = mid; else hi = mid;
  }
  return lo;
}

// Variants with tiles of 8 rows need about twice the registers of those with 4; a kernel that
// held both would run everything at the occupancy of the heaviest.  So the batch comes as two
// kernels over the same table, and a wavefront whose tensor belongs to the other one leaves.
template <int MODE, bool EIGHT_ROWS>
__device__ __forceinline__ void compress_dispatch_mode(const TensorDesc& d, uint32_t unit, const ScanCtx& sc,
                                                       WaveStage* stage) {
  if constexpr (!EIGHT_ROWS) {
    if (d.rowwise) {  // groups inside a row
      switch (d.variant & 6u) {
        case 0: compress_run<MODE, 4, false, 4, true>(d, unit, sc, stage); break;
        case 2: compress_run<MODE, 4, true, 4, true>(d, unit, sc, stage); break;
        case 4: compress_run<MODE, 8, false, 4, true>(d, unit, sc, stage); break;
        default: compress_run<MODE, 8, true, 4, true>(d, unit, sc, stage); break;
      }
      return;
    }
    switch (d.variant & 6u) {
      case 0: compress_run<MODE, 4, false, 4, false>(d, unit, sc, stage); break;
      case 2: compress_run<MODE, 4, true, 4, false>(d, unit, sc, stage); break;
      case 4: compress_run<MODE, 8, false, 4, false>(d, unit, sc, stage); break;
      default: compress_run<MODE, 8, true, 4, false>(d, unit, sc, stage); break;
    }
  } else {
    switch (d.variant & 6u) {
      case 0: compress_run<MODE, 4, false, 8, false>(d, unit, sc, stage); break;
      case 2: compress_run<MODE, 4, true, 8, false>(d, unit, sc, stage); break;
      case 4: compress_run<MODE, 8, false, 8, false>(d, unit, sc, stage); break;
      default: compress_run<MODE, 8, true, 8, false>(d, unit, sc, stage); break;
    }
  }
}

// TOPK over the whole tile: the specialised encoder
template <bool EIGHT_ROWS>
__device__ __forceinline__ void compress_dispatch_topk_whole(const TensorDesc& d, uint32_t unit, const ScanCtx& sc,
                                                             WaveStage* stage) {
  constexpr int kRows = EIGHT_ROWS ? 8 : 4;
  switch (d.variant & 6u) {
    case 0: compress_run<kModeTopk, 4, false, kRows, false, true>(d, unit, sc, stage); break;
    case 2: compress_run<kModeTopk, 4, true, kRows, false, true>(d, unit, sc, stage); break;
    case 4: compress_run<kModeTopk, 8, false, kRows, false, true>(d, unit, sc, stage); break;
    default: compress_run<kModeTopk, 8, true, kRows, false, true>(d, unit, sc, stage); break;
  }
}

template <int BITS, bool ASYM, int E, bool ROWWISE>
__device__ __forceinline__ void compress_plain_run(const TensorDesc& d, uint32_t unit) {
  const uint32_t t0 = unit * d.tiles_per_unit;
  const uint32_t t1 = (t0 + d.tiles_per_unit < d.n_tiles) ? t0 + d.tiles_per_unit : d.n_tiles;
  for (uint32_t t = t0; t < t1; ++t) compress_tile_plain<BITS, ASYM, E, ROWWISE>(d, t);
}

// One launch (per register class) for a table of tensors: runs are numbered across the table; a
// wavefront finds its tensor by binary search and dispatches on that tensor's method.
// The kernel for tiles of 8 rows is held to 3 wavefronts per SIMD: the variants that matter
// (TOPK over the whole tile) fit, the rarely used ones spill a few registers.
#ifndef ADACC_BATCH8_MIN_WAVES
#define ADACC_BATCH8_MIN_WAVES 3
#endif
template <bool EIGHT_ROWS>
__global__ __launch_bounds__(kThreads, EIGHT_ROWS ? ADACC_BATCH8_MIN_WAVES : 1) void compress_batch_kernel(const TensorDesc* table, uint32_t n,
                                                                  uint32_t total_units, uint64_t* state1,
                                                                  uint64_t* state2, uint32_t tag,
                                                                  uint32_t spin_limit) {
  __shared__ WaveStage stage[kWavesPerWg];
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  const ScanCtx sc{state1, state2, tag, spin_limit};
  const uint32_t g = blockIdx.x * kWavesPerWg + wave;
  if (g >= total_units) return;
  const uint32_t ti = __builtin_amdgcn_readfirstlane(find_tensor<true>(table, n, g));
  const TensorDesc d = table[ti];
  if (((d.variant & 1u) != 0u) != EIGHT_ROWS) return;
  const uint32_t unit = g - d.first_unit;
  switch (d.variant >> 3) {
    case kModeNone:
      if constexpr (!EIGHT_ROWS) {
        if (d.rowwise) {
          switch (d.variant & 6u) {
            case 0: compress_plain_run<4, false, 4, true>(d, unit); break;
            case 2: compress_plain_run<4, true, 4, true>(d, unit); break;
            case 4: compress_plain_run<8, false, 4, true>(d, unit); break;
            default: compress_plain_run<8, true, 4, true>(d, unit); break;
          }
          break;
        }
        switch (d.variant & 6u) {
          case 0: compress_plain_run<4, false, 4, false>(d, unit); break;
          case 2: compress_plain_run<4, true, 4, false>(d, unit); break;
          case 4: compress_plain_run<8, false, 4, false>(d, unit); break;
          default: compress_plain_run<8, true, 4, false>(d, unit); break;
        }
      } else {
        switch (d.variant & 6u) {
          case 0: compress_plain_run<4, false, 8, false>(d, unit); break;
          case 2: compress_plain_run<4, true, 8, false>(d, unit); break;
          case 4: compress_plain_run<8, false, 8, false>(d, unit); break;
          default: compress_plain_run<8, true, 8, false>(d, unit); break;
        }
      }
      break;
    case kModeAbs: compress_dispatch_mode<kModeAbs, EIGHT_ROWS>(d, unit, sc, &stage[wave]); break;
    case kModeStd: compress_dispatch_mode<kModeStd, EIGHT_ROWS>(d, unit, sc, &stage[wave]); break;
    default:
      if (d.lgs == (EIGHT_ROWS ? 12u : 11u) && d.lgq <= 11u) compress_dispatch_topk_whole<EIGHT_ROWS>(d, unit, sc, &stage[wave]);
      else compress_dispatch_mode<kModeTopk, EIGHT_ROWS>(d, unit, sc, &stage[wave]);
      break;
  }
}

// Batch decompression: a launch-wide numbering of the 2048-element pieces of all tensors.
template <bool F32>
__global__ __launch_bounds__(kThreads) void decompress_batch_kernel(const TensorDesc* table, uint32_t n,
                                                                    uint32_t total_tiles) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kWavesPerWg * decompress_lds_per_wave<4, F32>()];
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // uniform, and the compiler shall know it
  unsigned char* slice = lds + wave * decompress_lds_per_wave<4, F32>();
  // A wavefront's pieces ascend, so the tensor of a piece is the one of the previous piece or a later
  // one: one binary search at the start, then a walk, and the descriptor is read again only when
  // the tensor changes.
  uint32_t g = blockIdx.x * kWavesPerWg + wave;
  if (g >= total_tiles) return;
  uint32_t ti = __builtin_amdgcn_readfirstlane(find_tensor<false>(table, n, g));
  TensorDesc d = table[ti];
  uint32_t next_first = (ti + 1u < n) ? table[ti + 1u].first_tile : 0xFFFFFFFFu;
  for (; g < total_tiles; g += gridDim.x * kWavesPerWg) {
    if (g >= next_first) {
      do {
        ++ti;
        next_first = (ti + 1u < n) ? table[ti + 1u].first_tile : 0xFFFFFFFFu;
      } while (g >= next_first);
      d = table[ti];
    }
    const uint32_t tile = g - d.first_tile;
    const bool ho = (d.variant >> 3) != kModeNone;
    switch (d.variant & 6u) {
      case 0: decompress_tile<4, false, 4, F32>(d, tile, ho, slice); break;
      case 2: decompress_tile<4, true, 4, F32>(d, tile, ho, slice); break;
      case 4: decompress_tile<8, false, 4, F32>(d, tile, ho, slice); break;
      default: decompress_tile<8, true, 4, F32>(d, tile, ho, slice); break;
    }
  }
}

}  // namespace adacc
