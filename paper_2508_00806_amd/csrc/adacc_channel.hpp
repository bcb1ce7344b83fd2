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
namespace ADACC_DT_NS {

constexpr int kSelectThreads = 1024;    // accumulators of the sums over channels

// ---- step 1: binary32 sums of |x| over chunks of 64 tokens, partial[chunk][hidden].  A workgroup
// takes one chunk of a strip of 512 channels: a lane owns 8 adjacent channels (one 16-byte load per
// token, rows fully coalesced), each wavefront a run of the chunk's tokens, all its loads in flight
// at once; the wavefronts' sums meet in LDS and are added in token order.  Short-lived workgroups in
// the hardware's order walk through the tensor as a window, which reads faster than a grid that is
// resident as a whole and covers the tensor all the time.
template <bool STREAM>
__global__ __launch_bounds__(kPartialWaves * kWave) void channel_partial_kernel(const uint16_t* __restrict__ x,
                                                                               uint32_t tokens, uint32_t hidden,
                                                                               float* __restrict__ partial,
                                                                               uint32_t strips) {
  __shared__ float meet[kPartialWaves - 1][kOct][kWave];
  const uint32_t wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const uint32_t chunk = blockIdx.x / strips;
  const uint32_t oct = (blockIdx.x - chunk * strips) * kWave + lane;
  const bool live = oct < hidden / kOct;
  const uint32_t t0 = chunk * kChunkTokens + wave * kPartialRows;
  const uint32_t rows = t0 >= tokens ? 0u : (tokens - t0 < kPartialRows ? tokens - t0 : kPartialRows);
  const uint16_t* p = x + (size_t)t0 * hidden + (size_t)oct * kOct;
  uint4 v[kPartialRows];
#pragma unroll
  for (uint32_t i = 0; i < kPartialRows; ++i) {
    v[i] = make_uint4(0u, 0u, 0u, 0u);  // a token that is not there adds +0
    if (live && i < rows) v[i] = load_stats16<STREAM>(p + (size_t)i * hidden);
  }
  float acc[kOct];
#pragma unroll
  for (int e = 0; e < kOct; ++e) acc[e] = 0.0f;
#pragma unroll
  for (uint32_t i = 0; i < kPartialRows; ++i) {
    const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      acc[2 * k] = acc[2 * k] + fabsf(widen_lo(w[k]));
      acc[2 * k + 1] = acc[2 * k + 1] + fabsf(widen_hi(w[k]));
    }
  }
  if (wave != 0) {
#pragma unroll
    for (int e = 0; e < kOct; ++e) meet[wave - 1][e][lane] = acc[e];
  }
  __syncthreads();
  if (wave == 0 && live) {
#pragma unroll
    for (uint32_t w = 0; w + 1 < kPartialWaves; ++w) {
#pragma unroll
      for (int e = 0; e < kOct; ++e) acc[e] = acc[e] + meet[w][e][lane];
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
  constexpr uint32_t kPasses = kScoreChunks / kRowsPerPass;
  float4 v[kPasses];
  auto fetch = [&](uint32_t c0) {
    const uint32_t rows = n_chunks - c0 < (uint32_t)kScoreChunks ? n_chunks - c0 : (uint32_t)kScoreChunks;
#pragma unroll
    for (uint32_t i = 0; i < kPasses; ++i) {
      const uint32_t r = row + i * kRowsPerPass;
      v[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      if (col_ok && r < rows)
        v[i] = *reinterpret_cast<const float4*>(partial + (size_t)(c0 + r) * hidden + h0 + quad * 4u);
    }
  };
  double s = 0.0;
  fetch(0u);
  for (uint32_t c0 = 0; c0 < n_chunks; c0 += kScoreChunks) {
    const uint32_t rows = n_chunks - c0 < (uint32_t)kScoreChunks ? n_chunks - c0 : (uint32_t)kScoreChunks;
#pragma unroll
    for (uint32_t i = 0; i < kPasses; ++i)
      *reinterpret_cast<float4*>(&stage[row + i * kRowsPerPass][quad * 4u]) = v[i];
    __syncthreads();
    if (c0 + kScoreChunks < n_chunks) fetch(c0 + kScoreChunks);  // in flight while this block is added up
    if (threadIdx.x < (uint32_t)kScoreChannels) {
      constexpr uint32_t kBatch = 32;  // LDS reads in flight ahead of the chain of additions
      uint32_t r = 0;
      for (; r + kBatch <= rows; r += kBatch) {
        float w[kBatch];
#pragma unroll
        for (uint32_t i = 0; i < kBatch; ++i) w[i] = stage[r + i][threadIdx.x];
#pragma unroll
        for (uint32_t i = 0; i < kBatch; ++i) s = __dadd_rn(s, (double)w[i]);
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

// One accumulator per thread (thread j holds the sum over the channels h = j mod 1024, ascending).  They meet
// in a fixed order: the xor butterfly inside a wavefront (both partners add the same two numbers, so every
// lane ends with the same bits), then the wavefronts' sums through LDS, added in wavefront order by every
// thread.  Two barriers instead of one per level of a tree over LDS.
constexpr int kSelectWaves = kSelectThreads / kWave;
__device__ __forceinline__ double meet_accumulators(double mine, double* a /* LDS, one per wavefront */) {
#pragma unroll
  for (int o = kWave / 2; o >= 1; o >>= 1) mine = __dadd_rn(mine, __shfl_xor(mine, o, kWave));
  __syncthreads();  // the previous use of `a` is over
  if (threadIdx.x % kWave == 0) a[threadIdx.x / kWave] = mine;
  __syncthreads();
  double total = a[0];
#pragma unroll
  for (int w = 1; w < kSelectWaves; ++w) total = __dadd_rn(total, a[w]);
  return total;
}
// the same for counts; `below`: the sum over the threads before this one
__device__ __forceinline__ uint32_t meet_counts(uint32_t mine, uint32_t* cnt /* LDS, one per wavefront */, uint32_t* below) {
  const uint32_t lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  uint32_t incl = mine;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t t = __shfl_up(incl, o, kWave);
    if (lane >= (uint32_t)o) incl += t;
  }
  __syncthreads();  // the previous use of `cnt` is over
  if (lane == kWave - 1) cnt[wave] = incl;
  __syncthreads();
  uint32_t total = 0u, before = 0u;
#pragma unroll
  for (int w = 0; w < kSelectWaves; ++w) {
    if ((uint32_t)w < wave) before += cnt[w];
    total += cnt[w];
  }
  *below = before + incl - mine;
  return total;
}

// ---- step 3 (Eq. 1): mu, sigma, Z, the channel mask, the list of outlier channels.  One
// workgroup of 1024 threads; the work is a few passes over `hidden` numbers (a division per channel).
__global__ __launch_bounds__(kSelectThreads) void channel_select_kernel(const double* __restrict__ S, ChannelDesc c) {
  __shared__ double a[kSelectWaves];
  __shared__ uint32_t cnt[kSelectWaves];
  const uint32_t j = threadIdx.x;
  const uint32_t hidden = c.hidden;

  double acc = 0.0;
  uint32_t n = 0;
  // sixteen loads in flight per thread (the whole of a thread's share up to 16384 channels: the kernel is a
  // chain of round trips to memory); a position past the end reads as +Inf and is skipped like any other sum
  // that is not finite
  constexpr uint32_t kAhead = 16;
  const double skip = __longlong_as_double(0x7FF0000000000000ll);
  for (uint32_t h = j; h < hidden; h += kAhead * kSelectThreads) {
    double v[kAhead];
#pragma unroll
    for (uint32_t i = 0; i < kAhead; ++i) v[i] = h + i * kSelectThreads < hidden ? S[h + i * kSelectThreads] : skip;
#pragma unroll
    for (uint32_t i = 0; i < kAhead; ++i)
      if (finite_f64(v[i])) { acc = __dadd_rn(acc, v[i]); ++n; }
  }
  const double total = meet_accumulators(acc, a);
  uint32_t unused;
  const double finite = (double)meet_counts(n, cnt, &unused);
  const double mu = __ddiv_rn(total, finite);

  acc = 0.0;
  for (uint32_t h = j; h < hidden; h += kAhead * kSelectThreads) {
    double v[kAhead];
#pragma unroll
    for (uint32_t i = 0; i < kAhead; ++i) v[i] = h + i * kSelectThreads < hidden ? S[h + i * kSelectThreads] : skip;
#pragma unroll
    for (uint32_t i = 0; i < kAhead; ++i)
      if (finite_f64(v[i])) {
        const double d = __dsub_rn(v[i], mu);
        acc = __fma_rn(d, d, acc);
      }
  }
  const double sigma = __dsqrt_rn(__ddiv_rn(meet_accumulators(acc, a), finite));
  const double zt = (double)c.z_thresh;

  // every thread takes a contiguous stretch of mask bytes, so that the channels stay in order
  const uint32_t n_bytes = hidden / 8u;
  const uint32_t per = (n_bytes + kSelectThreads - 1) / kSelectThreads;
  const uint32_t b0 = j * per < n_bytes ? j * per : n_bytes;
  const uint32_t b1 = b0 + per < n_bytes ? b0 + per : n_bytes;
  uint32_t mine = 0;
  uint64_t masks = 0ull;  // the thread's mask bytes (at most 8: hidden <= 65536), first byte lowest
  for (uint32_t b = b0; b < b1; ++b) {
    double v[8];
#pragma unroll
    for (uint32_t e = 0; e < 8u; ++e) v[e] = S[b * 8u + e];
    uint32_t m = 0;
#pragma unroll
    for (uint32_t e = 0; e < 8u; ++e) {
      const double z = __ddiv_rn(__dsub_rn(v[e], mu), sigma);
      if (!finite_f64(v[e]) || z > zt) m |= 1u << e;  // a NaN z selects nothing
    }
    c.mask[b] = (uint8_t)m;
    masks |= (uint64_t)m << (8u * (b - b0));
    mine += (uint32_t)__popc(m);
  }
  // where this thread's channels go in the list: the outlier channels of the threads before it
  uint32_t running;
  const uint32_t n_ch = meet_counts(mine, cnt, &running);
  for (uint32_t b = b0; b < b1; ++b) {
    uint32_t m = (uint32_t)(masks >> (8u * (b - b0))) & 0xFFu;
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

// off = q * hidden + col for off < hidden + 2048 <= 2^24 / 8: the quotient through a binary32 reciprocal
// that the host rounded down, so the estimate is the true quotient or one less.
__device__ __forceinline__ void split_offset(uint32_t off, uint32_t hidden, float inv_hidden, uint32_t& q,
                                             uint32_t& col) {
  q = (uint32_t)((float)off * inv_hidden);
  col = off - __umul24(q, hidden);
  if (col >= hidden) { col -= hidden; ++q; }
}

// The channel mask is consulted for every octet, the rank table for every octet with an outlier:
// each workgroup keeps copies in LDS (ranks as 16 bits: they stay below 65536).
struct ChannelLds {
  const uint16_t* base;
  const uint8_t* mask;
};
__device__ __forceinline__ ChannelLds stage_channels(const ChannelDesc& c, uint8_t* lds) {
  const uint32_t n = c.hidden / 8u;
  uint16_t* base = reinterpret_cast<uint16_t*>(lds);
  uint8_t* mask = lds + 2u * n;
  for (uint32_t i = threadIdx.x; i < n; i += kThreads) {
    mask[i] = c.mask[i];
    base[i] = (uint16_t)c.base[i];
  }
  __syncthreads();
  return ChannelLds{base, mask};
}

// ---- step 4: the outlier channels of one tile are stored and zeroed, then the tile is encoded
// like one of a tensor without outliers.
template <int BITS, bool ASYM, bool ROWWISE, bool COMPLETE>
__device__ __forceinline__ void channel_compress_tile(const TensorDesc& d, const ChannelDesc& c, uint32_t n_ch,
                                                      const ChannelLds& lds, uint32_t tile) {
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
      uint32_t q, col;
      split_offset(cg.col0 + in_tile, c.hidden, c.inv_hidden, q, col);
      const uint32_t m = lds.mask[col >> 3];
      if (m != 0u) {
        uint16_t* dst = c.ch_val + (size_t)(cg.row0 + q) * n_ch + lds.base[col >> 3];
        // the values go out first (one round per outlier channel of the octet: mostly one) ...
        uint32_t todo = m, r = 0u;
        while (todo != 0u) {
          const uint32_t e = (uint32_t)__builtin_ctz(todo);
          todo &= todo - 1u;
          dst[r++] = (uint16_t)octet_half(raw[j], e);
        }
        // ... then they are cleared: two bits of the mask per word, each spread over its half
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe((int)m, 2 * k, 1);      // 0 or all ones
          const uint32_t hi = (uint32_t)__builtin_amdgcn_sbfe((int)m, 2 * k + 1, 1);
          const uint32_t clear = (lo & 0x0000FFFFu) | (hi & 0xFFFF0000u);
          raw[j][k] &= ~clear;
        }
      }
    }
  }
  encode_tile<kModeNone, BITS, ASYM, E, ROWWISE, false, true>(d, g, raw, tile, NullSink{}, 0u, 0u);
}

template <int BITS, bool ASYM, bool ROWWISE>
__global__ __launch_bounds__(kThreads) void channel_compress_kernel(TensorDesc d, ChannelDesc c) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_bytes[];
  if (c.status[1] != 0u) return;  // more outlier channels than the blob holds: nothing else is produced
  const uint32_t n_ch = __builtin_amdgcn_readfirstlane(c.status[0]);
  ChannelLds lds{nullptr, nullptr};
  if (n_ch != 0u) lds = stage_channels(c, lds_bytes);
  for (uint32_t t = blockIdx.x * kWavesPerWg + wave; t < d.n_tiles; t += gridDim.x * kWavesPerWg) {
    if (t + 1u < d.n_tiles) channel_compress_tile<BITS, ASYM, ROWWISE, true>(d, c, n_ch, lds, t);
    else channel_compress_tile<BITS, ASYM, ROWWISE, false>(d, c, n_ch, lds, t);
  }
}

// ---- step 4 for matrices whose rows are whole multiples of 512 channels, groups inside 512 channels:
// a wavefront takes a strip of 512 adjacent channels (8 per lane) over kChannelStripRows consecutive
// tokens.  Which of a lane's 8 channels are outlier channels, and where their values go in a token's
// record, is the same for every token: looked up once, no table in LDS and no division per octet.  All
// loads of the strip are issued first; its rows are then encoded four at a time like a tile's.
constexpr uint32_t kChannelStripRows = 8;

template <int BITS, bool ASYM>
__global__ __launch_bounds__(kThreads) void channel_compress_strip_kernel(TensorDesc d, ChannelDesc c) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (c.status[1] != 0u) return;  // more outlier channels than the blob holds: nothing else is produced
  const uint32_t n_ch = __builtin_amdgcn_readfirstlane(c.status[0]);
  const uint32_t strips = c.hidden / (uint32_t)kRow;
  const uint32_t unit = blockIdx.x * kWavesPerWg + wave;
  const uint32_t block = unit / strips;
  const uint32_t row0 = block * kChannelStripRows;
  if (row0 >= c.tokens) return;  // uniform
  const uint32_t col0 = (unit - block * strips) * (uint32_t)kRow;
  const uint32_t rows = c.tokens - row0 < kChannelStripRows ? c.tokens - row0 : kChannelStripRows;
  const uint32_t lane_off = (uint32_t)lane_id() * kOct;

  uint32_t m = 0u, first = 0u;
  if (n_ch != 0u) {
    m = c.mask[(col0 + lane_off) >> 3];
    first = c.base[(col0 + lane_off) >> 3];
  }
  constexpr uint32_t kHalf = kChannelStripRows / 2;
  const uint64_t base = (uint64_t)row0 * c.hidden + col0;  // uniform
  const uint16_t* sp = d.src + base;
  uint32_t raw[2][kHalf][4];
#pragma unroll
  for (uint32_t i = 0; i < kChannelStripRows; ++i) {  // rows past the end re-read the last one
    const uint32_t row = i < rows ? i : rows - 1u;
    const uint4 v = ADACC_LOAD16(sp + (row * c.hidden + lane_off));
    raw[i / kHalf][i % kHalf][0] = v.x; raw[i / kHalf][i % kHalf][1] = v.y;
    raw[i / kHalf][i % kHalf][2] = v.z; raw[i / kHalf][i % kHalf][3] = v.w;
  }
  if (m != 0u) {  // the kept channels go out first, then they are cleared
    uint16_t* dst = c.ch_val + (size_t)row0 * n_ch + first;
    static_for<(int)kChannelStripRows>([&](auto Ic) {  // the data-dependent loop inside must not keep this one rolled
      constexpr uint32_t i = (uint32_t)decltype(Ic)::value;
      if (i < rows) {
        uint32_t todo = m, r = 0u;
        while (todo != 0u) {
          const uint32_t e = (uint32_t)__builtin_ctz(todo);
          todo &= todo - 1u;
          dst[(size_t)i * n_ch + r++] = (uint16_t)octet_half(raw[i / kHalf][i % kHalf], e);
        }
      }
      clear_elements(raw[i / kHalf][i % kHalf], m);
    });
  }
  static_for<2>([&](auto Hc) {
    constexpr uint32_t h = (uint32_t)decltype(Hc)::value;
    if (rows >= (h + 1u) * kHalf) {  // uniform: four whole rows
      TileGeo<(int)kHalf, true> g;
      g.base = base + (uint64_t)(h * kHalf) * c.hidden;
      g.rem = kHalf * (uint32_t)kRow;
      g.lane_off = lane_off;
      g.full = true;
      g.stride = c.hidden;
      encode_tile_rowwise<kModeNone, BITS, ASYM, (int)kHalf, true>(d, g, raw[h], 0u, NullSink{}, 0u, 0u);
    } else {
      static_for<(int)kHalf>([&](auto Ic) {  // the last tokens of the matrix, one row at a time
        constexpr uint32_t i = (uint32_t)decltype(Ic)::value;
        if (h * kHalf + i < rows) {
          TileGeo<1, true> g;
          g.base = base + (uint64_t)(h * kHalf + i) * c.hidden;
          g.rem = (uint32_t)kRow;
          g.lane_off = lane_off;
          g.full = true;
          g.stride = c.hidden;
          const uint32_t one[1][4] = {{raw[h][i][0], raw[h][i][1], raw[h][i][2], raw[h][i][3]}};
          encode_tile_rowwise<kModeNone, BITS, ASYM, 1, true>(d, g, one, 0u, NullSink{}, 0u, 0u);
        }
      });
    }
  });
}

// ---- decompression: dequantise, put the outlier channels back, store.
// A wavefront takes a strip of 512 adjacent channels (8 per lane) over kChannelStripRows consecutive tokens:
// which of a lane's 8 channels are outlier channels, and where their values start in a token's record, is
// the same for every token, so it is looked up once (no table in LDS, no division per octet).  The loads of
// four tokens (codes, scale, offset, the first kept value of the octet) are issued before their first store;
// a second outlier channel in the same octet is rare and fetched when it is needed.
template <int BITS, bool ASYM, bool F32>
__global__ __launch_bounds__(kThreads) void channel_decompress_kernel(TensorDesc d, ChannelDesc c) {
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  if (c.status[1] != 0u) return;  // not a usable blob
  uint32_t n_ch = __builtin_amdgcn_readfirstlane(c.status[0]);
  if (n_ch > c.max_channels) n_ch = c.max_channels;  // a damaged blob must not make the reads leave it
  const uint32_t strips = (c.hidden + (uint32_t)kRow - 1u) / (uint32_t)kRow;
  const uint32_t unit = blockIdx.x * kWavesPerWg + wave;
  const uint32_t block = unit / strips;
  const uint32_t row0 = block * kChannelStripRows;
  const uint32_t col = (unit - block * strips) * (uint32_t)kRow + (uint32_t)lane_id() * kOct;
  if (row0 >= c.tokens || col >= c.hidden) return;
  const uint32_t rows = c.tokens - row0 < kChannelStripRows ? c.tokens - row0 : kChannelStripRows;

  // the lane's 8 channels: which are outlier channels, and the rank of the first of them
  uint32_t m = 0u, first = 0u;
  if (n_ch != 0u) {
    m = c.mask[col >> 3];
    first = c.base[col >> 3];
    if (first >= n_ch) m = 0u;  // a damaged blob must not be read past its end
  }
  const uint32_t lowest = m & (0u - m);
  const uint32_t rest = m ^ lowest;

  for (uint32_t r = 0; r < rows; r += 4u) {
    uint32_t cw[4][2];
    float sc[4], zp[4];
    uint32_t pre[4];
    const uint16_t* src[4];
#pragma unroll
    for (uint32_t i = 0; i < 4u; ++i) {  // rows past the end re-read the last one
      const uint32_t row = row0 + (r + i < rows ? r + i : rows - 1u);
      const uint64_t e0 = (uint64_t)row * c.hidden + col;
      if constexpr (BITS == 8) {
        const uint2 w = *reinterpret_cast<const uint2*>(d.codes + e0);
        cw[i][0] = w.x; cw[i][1] = w.y;
      } else {
        cw[i][0] = *reinterpret_cast<const uint32_t*>(d.codes + (e0 >> 1));
        cw[i][1] = 0u;
      }
      const uint64_t grp = e0 >> d.lgq;
      sc[i] = d.scales[grp];
      zp[i] = 0.0f;
      if constexpr (ASYM) zp[i] = d.zp[grp];
      src[i] = c.ch_val + (size_t)row * n_ch + first;
      pre[i] = m != 0u ? (uint32_t)src[i][0] : 0u;
    }
#pragma unroll
    for (uint32_t i = 0; i < 4u; ++i) {
      if (r + i >= rows) break;
      const uint64_t e0 = (uint64_t)(row0 + r + i) * c.hidden + col;
      int code[kOct];
      if constexpr (BITS == 8) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          code[e] = (int)(int8_t)((cw[i][0] >> (8 * e)) & 0xFFu);
          code[4 + e] = (int)(int8_t)((cw[i][1] >> (8 * e)) & 0xFFu);
        }
      } else {
#pragma unroll
        for (int e = 0; e < kOct; ++e) code[e] = ((int)(cw[i][0] << (28 - 4 * e))) >> 28;
      }
      float v[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) v[e] = ASYM ? __fmaf_rn((float)code[e], sc[i], zp[i]) : (float)code[e] * sc[i];

      // the kept channels of this octet, as their stored 16-bit patterns (hold[e] valid where keep has bit e)
      uint32_t keep = lowest, hold[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) hold[e] = lowest == (1u << e) ? pre[i] : 0u;
      if (rest != 0u) {
#pragma unroll
        for (int e = 1; e < kOct; ++e)
          if (rest & (1u << e)) {
            const uint32_t rank = (uint32_t)__popc(m & ((1u << e) - 1u));
            if (rank < n_ch - first) { hold[e] = src[i][rank]; keep |= 1u << e; }
          }
      }

      if constexpr (F32) {
        if (keep != 0u) {
#pragma unroll
          for (int e = 0; e < kOct; ++e) v[e] = (keep & (1u << e)) ? widen_lo(hold[e]) : v[e];
        }
        float* p = reinterpret_cast<float*>(d.dst) + e0;
        ADACC_STORE16(p, make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])));
        ADACC_STORE16(p + 4, make_uint4(__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])));
      } else {
        uint32_t w[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] = narrow_pair(v[2 * k], v[2 * k + 1]);
        if (keep != 0u) {  // the kept values go in as they were stored, bit for bit (no conversion touches a NaN)
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            if (keep & (1u << (2 * k))) w[k] = (w[k] & 0xFFFF0000u) | hold[2 * k];
            if (keep & (2u << (2 * k))) w[k] = (w[k] & 0x0000FFFFu) | (hold[2 * k + 1] << 16);
          }
        }
        ADACC_STORE16(reinterpret_cast<uint16_t*>(d.dst) + e0, make_uint4(w[0], w[1], w[2], w[3]));
      }
    }
  }
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
