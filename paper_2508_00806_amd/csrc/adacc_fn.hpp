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

// e8: tiles of 8 rows; rowwise: every group inside a row; whole (TOPK): the statistics group is the tile
CompressFn compress_fn_none(uint32_t bits, uint32_t asym, bool e8, bool rowwise);
CompressFn compress_fn_abs(uint32_t bits, uint32_t asym, bool e8, bool rowwise);
CompressFn compress_fn_std(uint32_t bits, uint32_t asym, bool e8, bool rowwise);
CompressFn compress_fn_topk(uint32_t bits, uint32_t asym, bool e8, bool whole);
DecompressFn decompress_fn(uint32_t bits, uint32_t asym, bool f32);
BatchCompressFn compress_batch_fn(int kind);  // kind: kBatch* of adacc_kernels.hpp
BatchDecompressFn decompress_batch_fn(bool f32);
PlaceSumFn place_sum_fn();
PlaceFn place_fn();
PlaceSumBatchFn place_sum_batch_fn();
PlaceBatchFn place_batch_fn();

// outlier channels (Section 3.2, Eq. 1)
typedef void (*ChannelPartialFn)(const uint16_t*, uint32_t, uint32_t, float*, uint32_t);
typedef void (*ChannelScoreFn)(const float*, uint32_t, uint32_t, double*);
typedef void (*ChannelSelectFn)(const double*, ChannelDesc);
typedef void (*ChannelFn)(TensorDesc, ChannelDesc);
ChannelPartialFn channel_partial_fn();
ChannelScoreFn channel_score_fn();
ChannelSelectFn channel_select_fn();
uint32_t channel_score_channels();  // channels per workgroup of the score kernel
ChannelFn channel_compress_fn(uint32_t bits, uint32_t asym, bool rowwise);
ChannelFn channel_decompress_fn(uint32_t bits, uint32_t asym, bool f32);

// channel-wise symmetric quantisation (Section 3.2, Query / Key / Value)
typedef void (*ChannelwiseItemsFn)(ChannelwiseDesc, uint32_t);
typedef void (*ChannelwiseFn)(ChannelwiseDesc);
ChannelwiseItemsFn channelwise_partial_fn();
ChannelwiseFn channelwise_fold_fn();
uint32_t channelwise_fold_octets();  // octets of channels per workgroup of the fold kernel
ChannelwiseFn channelwise_quantise_fn(uint32_t bits);
ChannelwiseFn channelwise_dequantise_fn(uint32_t bits, bool f32);

// dropout mask, byte format <-> bit format (Section 3.2)
typedef void (*MaskFn)(const uint8_t*, uint64_t, uint8_t*);
MaskFn mask_pack_fn();
MaskFn mask_unpack_fn();

}  // namespace adacc
