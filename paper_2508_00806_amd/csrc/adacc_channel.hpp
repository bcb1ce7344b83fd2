// Outlier CHANNELS (Section 3.2, Eq. 1): the activation is a row-major matrix of `tokens` rows and
// `hidden` channels; S_h = sum over the tokens of |x|, Z_h = (S_h - mu) / sigma over the channels,
// channels with Z_h above the threshold are kept whole, zeroed in the activation, and the rest is
// group-quantised (Eq. 2 / Eq. 3) by the same encoder as a tensor without outliers.
//
// The selection is an integer decision taken by floating-point sums, so the order of the sums is
// fixed: chunks of 64 tokens added one after the other in binary32; the chunk sums added one after
// the other in binary64; sums over channels in 256 interleaved binary64 accumulators folded by halves.
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_decompress.hpp"

namespace adacc {

constexpr int kSelectThreads = 256;     // accumulators of the sums over channels

// ---- step 1: binary32 sums of |x| over chunks of 64 tokens.  One lane owns 8 adjacent channels
// (one 16-byte load per token), consecutive lanes consecutive octets: fully coalesced rows.
// partial[chunk][hidden].
__global__ __launch_bounds__(kThreads) void channel_partial_kernel(const uint16_t* __restrict__ x, uint32_t tokens,
                                                                   uint32_t hidden, float* __restrict__ partial,
                                                                   uint32_t n_items) {
  const uint32_t octs = hidden / kOct;
  for (uint32_t item = blockIdx.x * kThreads + threadIdx.x; item < n_items; item += gridDim.x * kThreads) {
    const uint32_t chunk = item / octs;
    const uint32_t oct = item - chunk * octs;
    const uint32_t t0 = chunk * kChunkTokens;
    const uint32_t rows = tokens - t0 < kChunkTokens ? tokens - t0 : kChunkTokens;
    const uint16_t* p = x + (size_t)t0 * hidden + (size_t)oct * kOct;
    float acc[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) acc[e] = 0.0f;
    constexpr uint32_t kBatch = 16;  // loads in flight per lane
    uint32_t r = 0;
    for (; r + kBatch <= rows; r += kBatch) {
      uint4 v[kBatch];
#pragma unroll
      for (uint32_t i = 0; i < kBatch; ++i) v[i] = *reinterpret_cast<const uint4*>(p + (size_t)(r + i) * hidden);
#pragma unroll
      for (uint32_t i = 0; i < kBatch; ++i) {
        const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          acc[2 * k] = acc[2 * k] + fabsf(__uint_as_float(w[k] << 16));
          acc[2 * k + 1] = acc[2 * k + 1] + fabsf(__uint_as_float(w[k] & 0xFFFF0000u));
        }
      }
    }
    for (; r < rows; ++r) {
      const uint4 v = *reinterpret_cast<const uint4*>(p + (size_t)r * hidden);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] = acc[2 * k] + fabsf(__uint_as_float(w[k] << 16));
        acc[2 * k + 1] = acc[2 * k + 1] + fabsf(__uint_as_float(w[k] & 0xFFFF0000u));
      }
    }
    float4* q = reinterpret_cast<float4*>(partial + (size_t)chunk * hidden + (size_t)oct * kOct);
    q[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    q[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
}

// ---- step 2: S_h = binary64 sum of the chunk sums, in chunk order.  The additions of one channel
// form a chain, so the kernel is bound by latency, not by bytes: a workgroup takes 32 channels, all
// its threads fetch a block of 256 chunk sums per channel into LDS at once, then one lane per channel
// adds them up in order.
constexpr int kScoreChannels = 32;
constexpr int kScoreChunks = 256;
__global__ __launch_bounds__(kThreads) void channel_score_kernel(const float* __restrict__ partial, uint32_t n_chunks,
                                                                 uint32_t hidden, double* __restrict__ S) {
  __shared__ __attribute__((aligned(16))) float stage[kScoreChunks][kScoreChannels];
  const uint32_t h0 = blockIdx.x * kScoreChannels;
  const uint32_t quad = threadIdx.x % (kScoreChannels / 4);   // which 4 channels of the 32
  const uint32_t row = threadIdx.x / (kScoreChannels / 4);    // 0..31
  constexpr uint32_t kRowsPerPass = kThreads / (kScoreChannels / 4);
  const bool col_ok = h0 + quad * 4u < hidden;                // hidden is a multiple of 8
  double s = 0.0;
  for (uint32_t c0 = 0; c0 < n_chunks; c0 += kScoreChunks) {
    const uint32_t rows = n_chunks - c0 < (uint32_t)kScoreChunks ? n_chunks - c0 : (uint32_t)kScoreChunks;
    float4 v[kScoreChunks / kRowsPerPass];
#pragma unroll
    for (uint32_t i = 0; i < kScoreChunks / kRowsPerPass; ++i) {
      const uint32_t r = row + i * kRowsPerPass;
      v[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (col_ok && r < rows)
        v[i] = *reinterpret_cast<const float4*>(partial + (size_t)(c0 + r) * hidden + h0 + quad * 4u);
    }
#pragma unroll
    for (uint32_t i = 0; i < kScoreChunks / kRowsPerPass; ++i)
      *reinterpret_cast<float4*>(&stage[row + i * kRowsPerPass][quad * 4u]) = v[i];
    __syncthreads();
    if (threadIdx.x < (uint32_t)kScoreChannels) {
      uint32_t r = 0;
      for (; r + 8 <= rows; r += 8) {
        float w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = stage[r + i][threadIdx.x];
#pragma unroll
        for (int i = 0; i < 8; ++i) s = __dadd_rn(s, (double)w[i]);
      }
      for (; r < rows; ++r) s = __dadd_rn(s, (double)stage[r][threadIdx.x]);
    }
    __syncthreads();
  }
  if (threadIdx.x < (uint32_t)kScoreChannels && h0 + threadIdx.x < hidden) S[h0 + threadIdx.x] = s;
}

__device__ __forceinline__ bool finite_f64(double v) {
  return ((uint64_t)__double_as_longlong(v) & 0x7FF0000000000000ull) != 0x7FF0000000000000ull;
}

// 256 accumulators (thread j holds the sum over the channels h = j mod 256, ascending) folded by halves
__device__ __forceinline__ double fold_accumulators(double mine, double* a /* LDS, 256 */) {
  const int j = (int)threadIdx.x;
  __syncthreads();  // the previous use of `a` is over
  a[j] = mine;
  __syncthreads();
  for (int s = kSelectThreads / 2; s >= 1; s >>= 1) {
    if (j < s) a[j] = __dadd_rn(a[j], a[j + s]);
    __syncthreads();
  }
  return a[0];
}

// ---- step 3 (Eq. 1): mu, sigma, Z, the channel mask, the list of outlier channels.  One
// workgroup of 256 threads; the work is a few passes over `hidden` numbers.
__global__ __launch_bounds__(kSelectThreads) void channel_select_kernel(const double* __restrict__ S, ChannelDesc c) {
  __shared__ double a[kSelectThreads];
  __shared__ uint32_t cnt[kSelectThreads];
  const uint32_t j = threadIdx.x;
  const uint32_t hidden = c.hidden;

  double acc = 0.0;
  uint32_t n = 0;
  for (uint32_t h = j; h < hidden; h += kSelectThreads) {
    const double s = S[h];
    if (finite_f64(s)) { acc = __dadd_rn(acc, s); ++n; }
  }
  const double total = fold_accumulators(acc, a);
  cnt[j] = n;
  __syncthreads();
  for (int s = kSelectThreads / 2; s >= 1; s >>= 1) {
    if ((int)j < s) cnt[j] += cnt[j + s];
    __syncthreads();
  }
  const double finite = (double)cnt[0];
  const double mu = __ddiv_rn(total, finite);

  acc = 0.0;
  for (uint32_t h = j; h < hidden; h += kSelectThreads) {
    const double s = S[h];
    if (finite_f64(s)) {
      const double d = __dsub_rn(s, mu);
      acc = __fma_rn(d, d, acc);
    }
  }
  const double sigma = __dsqrt_rn(__ddiv_rn(fold_accumulators(acc, a), finite));
  const double zt = (double)c.z_thresh;

  // every thread takes a contiguous stretch of mask bytes, so that the channels stay in order
  const uint32_t n_bytes = hidden / 8u;
  const uint32_t per = (n_bytes + kSelectThreads - 1) / kSelectThreads;
  const uint32_t b0 = j * per < n_bytes ? j * per : n_bytes;
  const uint32_t b1 = b0 + per < n_bytes ? b0 + per : n_bytes;
  uint32_t mine = 0;
  for (uint32_t b = b0; b < b1; ++b) {
    uint32_t m = 0;
    for (uint32_t e = 0; e < 8u; ++e) {
      const double s = S[b * 8u + e];
      const double z = __ddiv_rn(__dsub_rn(s, mu), sigma);
      if (!finite_f64(s) || z > zt) m |= 1u << e;  // a NaN z selects nothing
    }
    c.mask[b] = (uint8_t)m;
    mine += (uint32_t)__popc(m);
  }
  // exclusive scan of the per-thread counts
  __syncthreads();
  cnt[j] = mine;
  __syncthreads();
  for (int s = 1; s < kSelectThreads; s <<= 1) {
    const uint32_t add = (int)j >= s ? cnt[j - s] : 0u;
    __syncthreads();
    cnt[j] += add;
    __syncthreads();
  }
  uint32_t running = cnt[j] - mine;
  const uint32_t n_ch = cnt[kSelectThreads - 1];
  for (uint32_t b = b0; b < b1; ++b) {
    uint32_t m = c.mask[b];  // written by this thread
    c.base[b] = running;
    while (m) {
      const uint32_t e = (uint32_t)__builtin_ctz(m);
      m &= m - 1u;
      if (running < c.max_channels) c.ch_idx[running] = (int32_t)(b * 8u + e);
      ++running;
    }
  }
  if (j == 0) {
    c.status[0] = n_ch;
    c.status[1] = n_ch > c.max_channels ? 1u : 0u;
    c.status[2] = 0u;
    c.status[3] = 0u;
  }
}

// element e (0..7) of an octet held as 4 words
__device__ __forceinline__ uint32_t octet_half(const uint32_t (&w)[4], uint32_t e) {
  const uint32_t lo = (e & 4u) ? w[2] : w[0];
  const uint32_t hi = (e & 4u) ? w[3] : w[1];
  const uint32_t word = (e & 2u) ? hi : lo;
  return (e & 1u) ? word >> 16 : word & 0xFFFFu;
}

// where the tile's rows lie in the matrix
struct ChannelGeo {
  uint32_t row0, col0;  // uniform: token and channel of the tile's first element
};
__device__ __forceinline__ ChannelGeo channel_geo(uint32_t tile, uint32_t hidden) {
  const uint32_t base = tile * (uint32_t)(4 * kRow);  // numel < 2^32 in this mode
  ChannelGeo g;
  g.row0 = base / hidden;
  g.col0 = base - g.row0 * hidden;
  return g;
}

// ---- step 4: the outlier channels of one tile are stored and zeroed, then the tile is encoded
// like one of a tensor without outliers.
template <int BITS, bool ASYM, bool ROWWISE, bool COMPLETE>
__device__ __forceinline__ void channel_compress_tile(const TensorDesc& d, const ChannelDesc& c, uint32_t n_ch,
                                                      uint32_t tile) {
  constexpr int E = 4;
  uint32_t raw[E][4];
  load_tile<E, COMPLETE>(d, tile, raw);
  const TileGeo<E> g = tile_geo<E, COMPLETE>(d, tile);
  if constexpr (!COMPLETE) blank_tail<E>(g, raw);
  if (n_ch != 0u) {
    const ChannelGeo cg = channel_geo(tile, c.hidden);
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint32_t in_tile = g.lane_off + (uint32_t)(j * kRow);
      if (!COMPLETE && in_tile >= g.rem) continue;
      const uint32_t off = cg.col0 + in_tile;
      const uint32_t q = off / c.hidden;
      const uint32_t col = off - q * c.hidden;
      uint32_t m = c.mask[col >> 3];
      if (m != 0u) {
        uint16_t* dst = c.ch_val + (size_t)(cg.row0 + q) * n_ch + c.base[col >> 3];
        // clear the outlier elements: two bits of the mask per word
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t two = (m >> (2 * k)) & 3u;
          const uint32_t keep = ((two & 1u) ? 0u : 0x0000FFFFu) | ((two & 2u) ? 0u : 0xFFFF0000u);
          // the value goes out before it is cleared
          if (two & 1u) dst[__popc(m & ((1u << (2 * k)) - 1u))] = (uint16_t)(raw[j][k] & 0xFFFFu);
          if (two & 2u) dst[__popc(m & ((1u << (2 * k + 1)) - 1u))] = (uint16_t)(raw[j][k] >> 16);
          raw[j][k] &= keep;
        }
      }
    }
  }
  TileOutliers<E> out;
  encode_tile<kModeNone, BITS, ASYM, E, ROWWISE>(d, g, raw, out);
}

template <int BITS, bool ASYM, bool ROWWISE>
__global__ __launch_bounds__(kThreads) void channel_compress_kernel(TensorDesc d, ChannelDesc c) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (c.status[1] != 0u) return;  // more outlier channels than the blob holds: nothing else is produced
  const uint32_t n_ch = __builtin_amdgcn_readfirstlane(c.status[0]);
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg) {
    if (t + 1u < d.n_tiles) channel_compress_tile<BITS, ASYM, ROWWISE, true>(d, c, n_ch, t);
    else channel_compress_tile<BITS, ASYM, ROWWISE, false>(d, c, n_ch, t);
  }
}

// ---- decompression: dequantise a piece of 2048 elements, put the outlier channels back, store.
template <int BITS, bool ASYM, bool F32>
__device__ __forceinline__ void channel_decompress_tile(const TensorDesc& d, const ChannelDesc& c, uint32_t n_ch,
                                                        uint32_t tile) {
  constexpr int E = 4;
  const uint32_t lane_off = (uint32_t)lane_id() * kOct;
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const ChannelGeo cg = channel_geo(tile, c.hidden);
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint32_t in_tile = lane_off + (uint32_t)(j * kRow);
    const uint64_t e0 = tile_base + in_tile;
    if (e0 >= d.numel) continue;
    int code[kOct];
    if constexpr (BITS == 8) {
      const uint2 w = *reinterpret_cast<const uint2*>(d.codes + e0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        code[e] = (int)(int8_t)((w.x >> (8 * e)) & 0xFFu);
        code[4 + e] = (int)(int8_t)((w.y >> (8 * e)) & 0xFFu);
      }
    } else {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(d.codes + (e0 >> 1));
#pragma unroll
      for (int e = 0; e < kOct; ++e) code[e] = ((int)(w << (28 - 4 * e))) >> 28;
    }
    const uint64_t grp = e0 >> d.lgq;
    const float s = d.scales[grp];
    float o = 0.0f;
    if constexpr (ASYM) o = d.zp[grp];
    float v[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) v[e] = ASYM ? __fmaf_rn((float)code[e], s, o) : (float)code[e] * s;

    if (n_ch != 0u) {
      const uint32_t off = cg.col0 + in_tile;
      const uint32_t q = off / c.hidden;
      const uint32_t col = off - q * c.hidden;
      const uint32_t m = c.mask[col >> 3];
      if (m != 0u) {
        const uint32_t first = c.base[col >> 3];
        const uint16_t* src = c.ch_val + (size_t)(cg.row0 + q) * n_ch + first;
#pragma unroll
        for (int e = 0; e < kOct; ++e)
          if (m & (1u << e)) {
            const uint32_t r = (uint32_t)__popc(m & ((1u << e) - 1u));
            if (first < n_ch && r < n_ch - first) v[e] = __uint_as_float((uint32_t)src[r] << 16);  // a damaged blob must not be read past its end
          }
      }
    }

    if constexpr (F32) {
      float4* p = reinterpret_cast<float4*>(reinterpret_cast<float*>(d.dst) + e0);
      p[0] = make_float4(v[0], v[1], v[2], v[3]);
      p[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      uint4 w;  // the bf16 image of a widened bf16 value is that value
      w.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
      w.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
      w.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
      w.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
      *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(d.dst) + e0) = w;
    }
  }
}

template <int BITS, bool ASYM, bool F32>
__global__ __launch_bounds__(kThreads) void channel_decompress_kernel(TensorDesc d, ChannelDesc c) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (c.status[1] != 0u) return;  // not a usable blob
  uint32_t n_ch = __builtin_amdgcn_readfirstlane(c.status[0]);
  if (n_ch > c.max_channels) n_ch = c.max_channels;  // a damaged blob must not make the reads leave it
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg)
    channel_decompress_tile<BITS, ASYM, F32>(d, c, n_ch, t);
}

}  // namespace adacc
