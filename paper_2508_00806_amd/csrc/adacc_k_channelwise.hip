// Channel-wise symmetric quantisation (Section 3.2, list of layer-specific schemes: the scheme for the
// Query, Key and Value matrices).  The tensor is a row-major matrix [tokens][hidden]; every channel
// (column) is one group of Eq. 2: S_h = max over the tokens of |x| / D, code = clip(round(x / S_h)).
// Codes stay in the tensor's own order: nothing is transposed.
//
// Three kernels: maxima of |x| over chunks of 64 tokens, their fold into S_h and D / max, and the
// quantisation proper.  A maximum does not depend on the order it is taken in, so unlike the sums of
// the outlier-channel statistics nothing here has an order to keep.
#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_decompress.hpp"
#include "adacc_fn.hpp"

namespace adacc {
namespace ADACC_DT_NS {

// magnitudes (15 low bits) of two 16-bit values; one that is not finite counts as zero
__device__ __forceinline__ uint32_t finite_magnitudes2(uint32_t w) {
  const uint32_t mag = w & 0x7FFF7FFFu;
  constexpr uint32_t kLift = (0x8000u - kNonfiniteMag) * 0x00010001u;
  const uint32_t nf = ((mag + kLift) >> 15) & 0x00010001u;  // magnitude >= kNonfiniteMag: bit 15 after the add
  return mag & ~(nf * 0xFFFFu);
}

// ---- step 1: partial[chunk][hidden] = max of the finite magnitudes over the chunk's tokens.
// Same decomposition as the chunk sums of the outlier-channel statistics: a workgroup takes one chunk of
// a strip of 512 channels, a lane owns 8 adjacent channels, each wavefront a run of the chunk's tokens
// with all its loads in flight at once; the wavefronts' maxima meet in LDS.
template <bool STREAM>
__global__ __launch_bounds__(kPartialWaves * kWave) void channelwise_partial_kernel(ChannelwiseDesc c, uint32_t strips) {
  __shared__ uint32_t meet[kPartialWaves - 1][4][kWave];
  const uint32_t wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint32_t chunk = blockIdx.x / strips;
  const uint32_t oct = (blockIdx.x - chunk * strips) * kWave + lane;
  const bool live = oct < c.hidden / kOct;
  const uint32_t t0 = chunk * kChunkTokens + wave * kPartialRows;
  const uint32_t rows = t0 >= c.tokens ? 0u : (c.tokens - t0 < kPartialRows ? c.tokens - t0 : kPartialRows);
  const uint16_t* p = c.src + (size_t)t0 * c.hidden + (size_t)oct * kOct;
  uint4 v[kPartialRows];
#pragma unroll
  for (uint32_t i = 0; i < kPartialRows; ++i) {
    v[i] = make_uint4(0u, 0u, 0u, 0u);  // a token that is not there: magnitude zero
    if (live && i < rows) v[i] = load_stats16<STREAM>(p + (size_t)i * c.hidden);
  }
  uint32_t acc[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (uint32_t i = 0; i < kPartialRows; ++i) {
    acc[0] = pk_max_u16(acc[0], finite_magnitudes2(v[i].x));
    acc[1] = pk_max_u16(acc[1], finite_magnitudes2(v[i].y));
    acc[2] = pk_max_u16(acc[2], finite_magnitudes2(v[i].z));
    acc[3] = pk_max_u16(acc[3], finite_magnitudes2(v[i].w));
  }
  if (wave != 0) {
#pragma unroll
    for (int k = 0; k < 4; ++k) meet[wave - 1][k][lane] = acc[k];
  }
  __syncthreads();
  if (wave == 0 && live) {
#pragma unroll
    for (uint32_t w = 0; w + 1 < kPartialWaves; ++w) {
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[k] = pk_max_u16(acc[k], meet[w][k][lane]);
    }
    *reinterpret_cast<uint4*>(c.partial + (size_t)chunk * c.hidden + (size_t)oct * kOct) =
        make_uint4(acc[0], acc[1], acc[2], acc[3]);
  }
}

// ---- step 2: fold the chunk maxima; Eq. 2: S_h = max / D, and the reciprocal D / max the codes are
// formed with.  A workgroup takes 16 octets of channels; 16 of its threads share the chunks of an octet.
constexpr int kFoldOcts = 16;
constexpr int kFoldParts = kThreads / kFoldOcts;
__global__ __launch_bounds__(kThreads) void channelwise_fold_kernel(ChannelwiseDesc c) {
  __shared__ uint4 part[kFoldParts][kFoldOcts];
  const uint32_t o = threadIdx.x % kFoldOcts;
  const uint32_t k = threadIdx.x / kFoldOcts;
  const uint32_t oct = blockIdx.x * kFoldOcts + o;
  const bool live = oct < c.hidden / kOct;
  uint32_t acc[4] = {0u, 0u, 0u, 0u};
  if (live) {
    for (uint32_t ch0 = k; ch0 < c.n_chunks; ch0 += kFoldParts * 8u) {
      uint4 v[8];
#pragma unroll
      for (uint32_t i = 0; i < 8u; ++i) {
        const uint32_t ch = ch0 + i * kFoldParts;
        v[i] = make_uint4(0u, 0u, 0u, 0u);
        if (ch < c.n_chunks) v[i] = *reinterpret_cast<const uint4*>(c.partial + (size_t)ch * c.hidden + (size_t)oct * kOct);
      }
#pragma unroll
      for (uint32_t i = 0; i < 8u; ++i) {
        acc[0] = pk_max_u16(acc[0], v[i].x); acc[1] = pk_max_u16(acc[1], v[i].y);
        acc[2] = pk_max_u16(acc[2], v[i].z); acc[3] = pk_max_u16(acc[3], v[i].w);
      }
    }
  }
  part[k][o] = make_uint4(acc[0], acc[1], acc[2], acc[3]);
  __syncthreads();
  if (k == 0 && live) {
#pragma unroll
    for (int i = 1; i < kFoldParts; ++i) {
      const uint4 v = part[i][o];
      acc[0] = pk_max_u16(acc[0], v.x); acc[1] = pk_max_u16(acc[1], v.y);
      acc[2] = pk_max_u16(acc[2], v.z); acc[3] = pk_max_u16(acc[3], v.w);
    }
    float scl[kOct], inv[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      const float am = (e & 1) ? widen_hi(acc[e >> 1]) : widen_lo(acc[e >> 1]);  // the magnitude is the value's absolute
      scl[e] = c.inv_divisor != 0.0f ? am * c.inv_divisor : am / c.divisor;
      inv[e] = (am != 0.0f) ? fminf(c.divisor / am, kFltMax) : 0.0f;
    }
    float4* sp = reinterpret_cast<float4*>(c.scales + (size_t)oct * kOct);
    float4* ip = reinterpret_cast<float4*>(c.inv + (size_t)oct * kOct);
    sp[0] = make_float4(scl[0], scl[1], scl[2], scl[3]); sp[1] = make_float4(scl[4], scl[5], scl[6], scl[7]);
    ip[0] = make_float4(inv[0], inv[1], inv[2], inv[3]); ip[1] = make_float4(inv[4], inv[5], inv[6], inv[7]);
  }
}

// ---- steps 3 and X^: a wavefront takes a strip of 512 adjacent channels (8 per lane) over kStripRows
// consecutive tokens, so the 8 per-channel factors of a lane are loaded once and stay in registers (with
// tiles of 2048 consecutive elements a lane had to fetch 32 bytes of factors for every 16 bytes of input).
// Units are numbered strip by strip within a block of tokens, so the four wavefronts of a workgroup take
// four adjacent strips and the launch walks through memory front to back.
constexpr uint32_t kStripRows = 8;

struct Strip {
  uint32_t col;    // first channel of the lane
  size_t first;    // element offset of the lane's octet in the strip's first token
  uint32_t rows;   // tokens of the strip (the last block of tokens may be short)
  bool live;
};
__device__ __forceinline__ Strip strip_of(const ChannelwiseDesc& c) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const uint32_t strips = (c.hidden + (uint32_t)kRow - 1u) / (uint32_t)kRow;
  const uint32_t unit = blockIdx.x * kWavesPerWg + wave;
  const uint32_t block = unit / strips;
  const uint32_t row0 = block * kStripRows;
  Strip s;
  s.col = (unit - block * strips) * (uint32_t)kRow + (uint32_t)lane_id() * kOct;
  s.live = row0 < c.tokens && s.col < c.hidden;
  s.rows = s.live ? (c.tokens - row0 < kStripRows ? c.tokens - row0 : kStripRows) : 0u;
  s.first = (size_t)row0 * c.hidden + s.col;
  return s;
}

// ---- step 3: code = clip(round(x * (D / max_h))), packed, in the tensor's own order
template <int BITS>
__global__ __launch_bounds__(kThreads) void channelwise_quantise_kernel(ChannelwiseDesc c) {
  constexpr int Q = 1 << (BITS - 1);
  const Strip s = strip_of(c);
  if (!s.live) return;
  const float4 i0 = *reinterpret_cast<const float4*>(c.inv + s.col);
  const float4 i1 = *reinterpret_cast<const float4*>(c.inv + s.col + 4);
  const float iv[kOct] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
  for (uint32_t r = 0; r < s.rows; r += 4u) {
    uint4 raw[4];
#pragma unroll
    for (uint32_t i = 0; i < 4u; ++i) {  // four loads in flight; rows past the end re-read the last one
      const uint32_t row = r + i < s.rows ? r + i : s.rows - 1u;
      raw[i] = ADACC_LOAD16(c.src + s.first + (size_t)row * c.hidden);
    }
#pragma unroll
    for (uint32_t i = 0; i < 4u; ++i) {
      if (r + i >= s.rows) break;
      const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
      uint32_t code[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        float x = ADACC_ELEM_F32(w, e);
        if (is_nonfinite(x)) x = 0.0f;  // counts as zero
        code[e] = code_bits<Q>(x, iv[e]);
      }
      const size_t e0 = s.first + (size_t)(r + i) * c.hidden;
      if constexpr (BITS == 8) {
        uint2 o;
        o.x = pack_bytes4(code[0], code[1], code[2], code[3]);
        o.y = pack_bytes4(code[4], code[5], code[6], code[7]);
        ADACC_STORE8(c.codes + e0, o);
      } else {
        ADACC_STORE4(c.codes + (e0 >> 1), pack_nibbles8(code));
      }
    }
  }
}

// ---- decompression: X^ = code * S_h
template <int BITS, bool F32>
__global__ __launch_bounds__(kThreads) void channelwise_dequantise_kernel(ChannelwiseDesc c) {
  const Strip s = strip_of(c);
  if (!s.live) return;
  const float4 s0 = *reinterpret_cast<const float4*>(c.scales + s.col);
  const float4 s1 = *reinterpret_cast<const float4*>(c.scales + s.col + 4);
  const float sc[kOct] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
  for (uint32_t r = 0; r < s.rows; r += 4u) {
    uint32_t cw[4][2];
#pragma unroll
    for (uint32_t i = 0; i < 4u; ++i) {
      const uint32_t row = r + i < s.rows ? r + i : s.rows - 1u;
      const size_t e0 = s.first + (size_t)row * c.hidden;
      if constexpr (BITS == 8) {
        const uint2 w = *reinterpret_cast<const uint2*>(c.codes + e0);
        cw[i][0] = w.x; cw[i][1] = w.y;
      } else {
        cw[i][0] = *reinterpret_cast<const uint32_t*>(c.codes + (e0 >> 1));
        cw[i][1] = 0u;
      }
    }
#pragma unroll
    for (uint32_t i = 0; i < 4u; ++i) {
      if (r + i >= s.rows) break;
      const size_t e0 = s.first + (size_t)(r + i) * c.hidden;
      float v[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        int code;
        if constexpr (BITS == 8) code = (int)(int8_t)((cw[i][e >> 2] >> (8 * (e & 3))) & 0xFFu);
        else code = ((int)(cw[i][0] << (28 - 4 * e))) >> 28;
        v[e] = (float)code * sc[e];
      }
      if constexpr (F32) {
        float* p = reinterpret_cast<float*>(c.dst) + e0;
        ADACC_STORE16(p, make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
        ADACC_STORE16(p + 4, make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])));
      } else {
        uint4 w;
        w.x = narrow_pair(v[0], v[1]);
        w.y = narrow_pair(v[2], v[3]);
        w.z = narrow_pair(v[4], v[5]);
        w.w = narrow_pair(v[6], v[7]);
        ADACC_STORE16(reinterpret_cast<uint16_t*>(c.dst) + e0, w);
      }
    }
  }
}

uint32_t channelwise_strip_rows() { return kStripRows; }
uint32_t channelwise_partial_threads() { return kPartialWaves * (uint32_t)kWave; }
ChannelwiseItemsFn channelwise_partial_fn(bool stream) {
  return stream ? channelwise_partial_kernel<true> : channelwise_partial_kernel<false>;
}
ChannelwiseFn channelwise_fold_fn() { return channelwise_fold_kernel; }
uint32_t channelwise_fold_octets() { return (uint32_t)kFoldOcts; }
ChannelwiseFn channelwise_quantise_fn(uint32_t bits) {
  return bits == 4 ? channelwise_quantise_kernel<4> : channelwise_quantise_kernel<8>;
}
ChannelwiseFn channelwise_dequantise_fn(uint32_t bits, bool f32) {
  if (bits == 4) return f32 ? channelwise_dequantise_kernel<4, true> : channelwise_dequantise_kernel<4, false>;
  return f32 ? channelwise_dequantise_kernel<8, true> : channelwise_dequantise_kernel<8, false>;
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
