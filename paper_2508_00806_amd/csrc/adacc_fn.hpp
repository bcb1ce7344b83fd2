// Host-side handles of the kernel instantiations: each getter lives in the translation unit
// that instantiates the kernels it returns.
#pragma once

#include "adacc_common.hpp"

namespace adacc {

typedef void (*CompressFn)(TensorDesc, uint32_t);
typedef void (*DecompressFn)(TensorDesc, uint32_t);
typedef void (*BatchCompressFn)(const TensorDesc*, const uint32_t*, uint32_t);
typedef void (*BatchDecompressFn)(const TensorDesc*, const uint32_t*);
typedef void (*PlaceSumFn)(TensorDesc);
typedef void (*PlaceFn)(TensorDesc, uint32_t);
typedef void (*PlaceSumBatchFn)(const TensorDesc*, const uint32_t*);
typedef void (*PlaceBatchFn)(const TensorDesc*, const uint32_t*, uint32_t);
typedef void (*TailFn)(TensorDesc);
typedef void (*TailBatchFn)(const TensorDesc*, const uint32_t*);

// Types of the channel and channel-wise kernels
typedef void (*ChannelPartialFn)(const uint16_t*, uint32_t, uint32_t, float*, uint32_t);
typedef void (*ChannelScoreFn)(const float*, uint32_t, uint32_t, double*);
typedef void (*ChannelSelectFn)(const double*, ChannelDesc);
typedef void (*ChannelFn)(TensorDesc, ChannelDesc);
typedef void (*ChannelwiseItemsFn)(ChannelwiseDesc, uint32_t);
typedef void (*ChannelwiseFn)(ChannelwiseDesc);

// The getters of the kernels that read or write the tensor itself exist once per 16-bit format, in
// adacc::bf16 and adacc::f16 (the same sources compiled twice).
//   e8: tiles of 8 rows; rowwise: every group inside a row; whole (TOPK): the statistics group is the tile;
//   rows (TOPK): statistics group = quantisation group, inside a row
//   kind: kBatch* of adacc_common.hpp
//   generic_threads, generic_lds_bytes: workgroup size and dynamic LDS of the fallback kernels (one segment per workgroup;
//     topk_groups: TOPK over several statistics groups of a segment); compress_generic_fn(fixup): the second launch
//   stream: the statistics pass reads with the streaming hint (tensors beyond kStatsKeepBytes)
//   channel_score_channels: channels per workgroup of the score kernel
//   channel_select_threads: size of the one workgroup of the select kernel
//   channel_partial_threads, channelwise_partial_threads: size of a workgroup of the statistics pass (one chunk of
//     64 tokens of a strip of 512 channels)
//   channelwise_fold_octets: octets of channels per workgroup of the fold kernel
//   channelwise_strip_rows, channel_strip_rows: tokens a wavefront of the strip kernels takes
//   channel_compress_strip_fn: for matrices whose rows are multiples of 512 channels, groups inside 512 channels
#define ADACC_DTYPE_GETTERS                                                            \
  CompressFn compress_fn_none(uint32_t bits, uint32_t asym, bool e8, bool rowwise);    \
  CompressFn compress_fn_abs(uint32_t bits, uint32_t asym, bool e8, bool rowwise);     \
  CompressFn compress_fn_std(uint32_t bits, uint32_t asym, bool e8, bool rowwise);     \
  CompressFn compress_fn_topk(uint32_t bits, uint32_t asym, bool e8, bool whole, bool rows); \
  DecompressFn decompress_fn(uint32_t bits, uint32_t asym, bool f32);                  \
  BatchCompressFn compress_batch_fn4(int kind);                                        \
  BatchCompressFn compress_batch_fn8(int kind);                                        \
  BatchDecompressFn decompress_batch_fn(bool f32);                                     \
  PlaceSumFn place_sum_fn();                                                           \
  PlaceFn place_fn();                                                                  \
  PlaceSumBatchFn place_sum_batch_fn();                                                \
  PlaceBatchFn place_batch_fn();                                                       \
  TailFn compress_tail_fn();                                                           \
  TailBatchFn compress_tail_batch_fn();                                                \
  TailFn decompress_tail_fn();                                                         \
  TailBatchFn decompress_tail_batch_fn();                                              \
  CompressFn compress_generic_fn(uint32_t tile_elems, bool fixup);                     \
  TailFn decompress_generic_fn();                                                      \
  uint32_t generic_threads();                                                          \
  uint32_t generic_lds_bytes(uint32_t tile_elems, uint32_t gq, bool topk_groups);      \
  ChannelPartialFn channel_partial_fn(bool stream);                                    \
  ChannelScoreFn channel_score_fn();                                                   \
  ChannelSelectFn channel_select_fn();                                                 \
  uint32_t channel_score_channels();                                                   \
  uint32_t channel_select_threads();                                                   \
  uint32_t channel_partial_threads();                                                  \
  uint32_t channel_strip_rows();                                                       \
  ChannelFn channel_compress_fn(uint32_t bits, uint32_t asym, bool rowwise);           \
  ChannelFn channel_compress_strip_fn(uint32_t bits, uint32_t asym);                   \
  ChannelFn channel_decompress_fn(uint32_t bits, uint32_t asym, bool f32);             \
  ChannelwiseItemsFn channelwise_partial_fn(bool stream);                              \
  ChannelwiseFn channelwise_fold_fn();                                                 \
  uint32_t channelwise_fold_octets();                                                  \
  uint32_t channelwise_strip_rows();                                                   \
  uint32_t channelwise_partial_threads();                                              \
  ChannelwiseFn channelwise_quantise_fn(uint32_t bits);                                \
  ChannelwiseFn channelwise_dequantise_fn(uint32_t bits, bool f32);
namespace bf16 {
ADACC_DTYPE_GETTERS
}
namespace f16 {
ADACC_DTYPE_GETTERS
}
// half: the tensor is binary16 (else bf16)
#define ADACC_PICK(half, call) ((half) ? ::adacc::f16::call : ::adacc::bf16::call)

// dropout mask, byte format <-> bit format (Section 3.2)
typedef void (*MaskFn)(const uint8_t*, uint64_t, uint8_t*);
MaskFn mask_pack_fn();
MaskFn mask_unpack_fn();

}  // namespace adacc
