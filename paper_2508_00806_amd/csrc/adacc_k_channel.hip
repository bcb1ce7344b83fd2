// Instantiations of the kernels for outlier channels (Section 3.2, Eq. 1).
#include "adacc_channel.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

ChannelPartialFn channel_partial_fn(bool stream) { return stream ? channel_partial_kernel<true> : channel_partial_kernel<false>; }
ChannelScoreFn channel_score_fn() { return channel_score_kernel; }
ChannelSelectFn channel_select_fn() { return channel_select_kernel; }
uint32_t channel_strip_rows() { return kChannelStripRows; }
uint32_t channel_score_channels() { return (uint32_t)kScoreChannels; }
uint32_t channel_select_threads() { return (uint32_t)kSelectThreads; }
uint32_t channel_partial_threads() { return kPartialWaves * (uint32_t)kWave; }

template <int BITS, bool ASYM>
static ChannelFn pick_compress(bool rowwise) {
  return rowwise ? channel_compress_kernel<BITS, ASYM, true> : channel_compress_kernel<BITS, ASYM, false>;
}
ChannelFn channel_compress_strip_fn(uint32_t bits, uint32_t asym) {
  if (bits == 4) return asym ? channel_compress_strip_kernel<4, true> : channel_compress_strip_kernel<4, false>;
  return asym ? channel_compress_strip_kernel<8, true> : channel_compress_strip_kernel<8, false>;
}
ChannelFn channel_compress_fn(uint32_t bits, uint32_t asym, bool rowwise) {
  if (bits == 4) return asym ? pick_compress<4, true>(rowwise) : pick_compress<4, false>(rowwise);
  return asym ? pick_compress<8, true>(rowwise) : pick_compress<8, false>(rowwise);
}

template <int BITS, bool ASYM>
static ChannelFn pick_decompress(bool f32) {
  return f32 ? channel_decompress_kernel<BITS, ASYM, true> : channel_decompress_kernel<BITS, ASYM, false>;
}
ChannelFn channel_decompress_fn(uint32_t bits, uint32_t asym, bool f32) {
  if (bits == 4) return asym ? pick_decompress<4, true>(f32) : pick_decompress<4, false>(f32);
  return asym ? pick_decompress<8, true>(f32) : pick_decompress<8, false>(f32);
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
