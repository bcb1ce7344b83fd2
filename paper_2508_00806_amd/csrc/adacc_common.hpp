// Shared device/host definitions of libadacc (gfx950 only).
//
// Work decomposition used by every kernel here:
//   - a lane owns one "octet": 8 consecutive bf16 elements = one 16-byte load;
//   - a wavefront (64 lanes) covers one "row" of 512 consecutive elements per load
//     instruction, fully coalesced (1 KiB);
//   - a tile is E rows (E = 4 or 8, i.e. 2048 or 4096 elements) and belongs to ONE
//     wavefront; every statistics / quantisation group lies inside one tile, so all
//     reductions are wavefront-local and no kernel here needs a workgroup barrier.
//   - a workgroup is just 4 independent wavefronts.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adacc {

constexpr int kWave = 64;
constexpr int kOct = 8;               // elements per lane per row
constexpr int kRow = kWave * kOct;    // 512 elements
constexpr int kWavesPerWg = 4;
constexpr int kThreads = kWave * kWavesPerWg;

// Streaming accesses: data that is read or written once and not again by the same launch.  The
// non-temporal hint keeps such lines from being retained by the caches on their way; on this part a
// pure read stream runs about a third faster with it.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void store_stream16(void* p, uint4 v) {
  u32x4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
}
__device__ __forceinline__ void store_stream8(void* p, uint2 v) {
  u32x2_t t = {v.x, v.y};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x2_t*>(p));
}
__device__ __forceinline__ void store_stream4(void* p, uint32_t v) {
  __builtin_nontemporal_store(v, reinterpret_cast<uint32_t*>(p));
}

// The tensor streams of the compression / decompression kernels go through these (ADACC_NO_STREAM_HINT
// builds the plain accesses, for comparison).  The codes a decompression reads stay plain loads: on a
// blob that was written shortly before they are served by the caches, and the hint made that slower.
#ifndef ADACC_NO_STREAM_HINT
#define ADACC_LOAD16(p) load_stream16(p)
#define ADACC_STORE16(p, v) store_stream16((p), (v))
#define ADACC_STORE8(p, v) store_stream8((p), (v))
#define ADACC_STORE4(p, v) store_stream4((p), (v))
#else
#define ADACC_LOAD16(p) (*reinterpret_cast<const uint4*>(p))
#define ADACC_STORE16(p, v) (*reinterpret_cast<uint4*>(p) = (v))
#define ADACC_STORE8(p, v) (*reinterpret_cast<uint2*>(p) = (v))
#define ADACC_STORE4(p, v) (*reinterpret_cast<uint32_t*>(p) = (v))
#endif

// The statistics pass of the two-pass schemes reads what the second pass reads again: for a tensor that the
// Infinity Cache can hold a good part of, it leaves the lines to the caches (plain loads); for a larger one
// nothing would survive until the second pass, and it streams like every other pass (STREAM).
constexpr uint64_t kStatsKeepBytes = 128ull << 20;
template <bool STREAM>
__device__ __forceinline__ uint4 load_stats16(const void* p) {
  if constexpr (STREAM) return load_stream16(p);
  else return *reinterpret_cast<const uint4*>(p);
}

enum : uint32_t { kModeNone = 0, kModeAbs = 1, kModeStd = 2, kModeTopk = 3 };

// One tensor as the kernels see it.  Passed by value for single-tensor launches
// and read from a device table for batch launches.
struct TensorDesc {
  const uint16_t* src;  // compress: bf16 input
  void* dst;            // decompress: output
  uint8_t* codes;
  float* scales;
  float* zp;
  uint32_t* tile_ptr;
  int32_t* idx;
  uint16_t* val;
  uint32_t* status;
  uint32_t* cnt;            // compress, workspace: outliers found in every tile
  uint32_t* block_sum;      // compress, workspace (ABS / STD): outliers in every block of kPlaceTiles tiles
  uint2* slot;              // compress, workspace (ABS / STD): kSlot records (index, value) per tile, the tile's
                            //   outliers until the placement kernel has moved them to the stream
  uint32_t* flag;           // compress, workspace (TOPK): set to the epoch by a tile whose count is not the regular one
  uint64_t numel;           // elements the tile kernels take: the whole groups of the larger kind
  uint32_t tail;            // elements after those (fewer than the larger group), done by the tail kernels
  uint32_t n_tiles;         // tiles of the first numel elements (decompress: pieces of 2048 of them)
  uint32_t n_tiles_all;     // tiles of the whole tensor, tail included: tile_ptr has one entry more
  uint32_t bits, asym, mode;  // the method, for kernels that do not get it as template arguments
  uint32_t gq, gs;          // group sizes as numbers (the fallback kernels take groups that are no powers of two)
  uint32_t tile_elems;      // elements per tile of the blob
  uint32_t generic;         // 1: the method goes through the fallback kernels
  uint32_t n_blocks;        // compress: blocks of kPlaceTiles tiles (placement kernels)
  uint32_t lgt;             // log2(elements per tile): 11 or 12
  uint32_t lgq;         // log2(quant group)
  uint32_t lgs;         // log2(stat group) (STD / TOPK)
  uint32_t cap;         // capacity of idx / val
  uint32_t topk;
  float param;          // ABS: tau.  STD: k*k
  float divisor;        // D of Eq. 2 resp. Eq. 3 (2^(b-1), 2^b, or one less)
  float inv_divisor;    // 1/D when D is a power of two (the paper's rule), else 0
  uint32_t pow2_divisor;  // 1 when D is a power of two
  uint32_t rowwise;     // compress: 1 = every group lies inside a row (row-at-a-time encoder)
  uint32_t variant;     // index into the instantiation table
  uint32_t dst_f32;     // decompress: 1 = binary32 output
  uint32_t ptr_shift;   // decompress: works on pieces of 2048 elements; piece u belongs to tile u >> ptr_shift
};

// Outlier channels (Section 3.2, Eq. 1): what those kernels need beside the TensorDesc of the quantised part.
constexpr uint32_t kChunkTokens = 64;  // tokens per binary32 partial sum of the channel statistics
constexpr uint32_t kPartialWaves = 16;  // wavefronts that share a chunk in the statistics pass (one workgroup)
constexpr uint32_t kPartialRows = kChunkTokens / kPartialWaves;  // tokens per wavefront there
struct ChannelDesc {
  uint8_t* mask;        // hidden/8 bytes: bit (h & 7) of byte h >> 3 is set for an outlier channel
  uint32_t* base;       // hidden/8 words: number of outlier channels below channel 8 * (h >> 3)
  int32_t* ch_idx;      // the outlier channels, ascending
  uint16_t* ch_val;     // [tokens][n_ch] bf16 bit patterns
  uint32_t* status;     // [0] n_ch, [1] 1 if n_ch > max_channels
  uint32_t hidden;
  uint32_t tokens;
  uint32_t max_channels;
  float z_thresh;
  float inv_hidden;     // 1 / hidden rounded towards zero twice: never above the true reciprocal
};

// Channel-wise symmetric quantisation (Section 3.2, the Query / Key / Value scheme): one scale per channel.
struct ChannelwiseDesc {
  const uint16_t* src;  // compress: bf16 input [tokens][hidden]
  void* dst;            // decompress: output
  uint8_t* codes;
  float* scales;        // [hidden], S_h of Eq. 2
  float* inv;           // workspace [hidden]: D / max_h
  uint16_t* partial;    // workspace [n_chunks][hidden]: chunk maxima of the finite magnitudes
  uint64_t numel;
  uint32_t tokens, hidden, n_chunks;
  float divisor, inv_divisor;  // D of Eq. 2 and, when D is a power of two, 1/D (else 0)
};

// Outliers of a tile that travel through the tile's slot in the workspace (ABS / STD); a tile with
// more is selected a second time by the placement kernel.
constexpr int kSlot = 32;
// The placement kernels: a workgroup of kPlaceThreads threads takes kPlaceTiles consecutive tiles, one per thread.
constexpr int kPlaceThreads = 256;
constexpr int kPlaceTiles = 256;
// Tensors of at most this many blocks do without the kernel that adds up the blocks' counts.
constexpr uint32_t kPlaceDirectBlocks = 8;
// The workspace's launch counter ("epoch", kept on the host in adacc_workspace) marks what a launch
// wrote: a word that holds an older epoch reads as not set, so nothing has to be cleared per call.
constexpr uint32_t kEpochMax = 0x3FFFFFFFu;

// the batch compression kernels, by the weight of the variants they hold (adacc_kernels.hpp)
enum : int { kBatchRows4 = 0, kBatchAny4 = 1, kBatchTopk4 = 2, kBatchAny8 = 3, kBatchTopk8 = 4, kBatchKinds = 5 };

// variant index: ((mode*2 + (bits==8)) * 2 + asym) * 2 + (E==8)
__host__ __device__ inline uint32_t variant_index(uint32_t mode, uint32_t bits, uint32_t asym, uint32_t e8) {
  return ((mode * 2 + (bits == 8 ? 1u : 0u)) * 2 + asym) * 2 + e8;
}

}  // namespace adacc
