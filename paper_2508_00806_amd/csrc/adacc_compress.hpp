// Compression of one tile by one wavefront (Section 3.2, Fig. 3(c) compression workflow):
// load -> statistics -> outlier mask -> zero the outliers -> group scale (Eq. 2 / Eq. 3)
// -> quantise, pack, store -> ordered append of the outliers to the (index, value) stream.
#pragma once

#include <type_traits>

#include "adacc_common.hpp"

namespace adacc {

// ------------------------------------------------------------------ small helpers
__device__ __forceinline__ int lane_id() { return (int)__lane_id(); }

__device__ __forceinline__ float widen_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float widen_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
// element e (0..7) of an octet held in 4 dwords
#define ADACC_ELEM_F32(oct, e) (((e)&1) ? widen_hi((oct)[(e) >> 1]) : widen_lo((oct)[(e) >> 1]))
#define ADACC_ELEM_MAG(oct, e) ((((e)&1) ? ((oct)[(e) >> 1] >> 16) : (oct)[(e) >> 1]) & 0x7FFFu)

// compile-time loop: body(std::integral_constant<int, J>) for J = 0..N-1.  Used where a
// data-dependent inner loop would otherwise keep the compiler from unrolling, which would
// turn the per-row register arrays into scratch memory.
template <int N, int J = 0, class F>
__device__ __forceinline__ void static_for(F&& body) {
  if constexpr (J < N) {
    body(std::integral_constant<int, J>());
    static_for<N, J + 1>(body);
  }
}

struct OpAdd { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpMin { __device__ __forceinline__ float operator()(float a, float b) const { return fminf(a, b); } };
struct OpUMax { __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; } };

// xor butterfly over `lanes` adjacent lanes (power of two).  Every lane of a group ends
// with the same value, and for sums the association is the balanced binary tree over
// lane order, which is what makes the variance independent of the machine.
template <class T, class Op>
__device__ __forceinline__ T lanes_reduce(T v, int lanes, Op op) {
  for (int m = 1; m < lanes; m <<= 1) v = op(v, __shfl_xor(v, m));
  return v;
}

// s[j] for the first row of every group of R rows <- op over the group's rows (tree order)
template <int E, class T, class Op>
__device__ __forceinline__ void rows_combine(T (&s)[E], int R, Op op) {
#pragma unroll
  for (int r = 1; r < E; r <<= 1) {
    if (r < R) {
#pragma unroll
      for (int j = 0; j < E; j += 2 * r) s[j] = op(s[j], s[j + r]);
    }
  }
}
// copy the group's value from its first row to its other rows
template <int E, class T>
__device__ __forceinline__ void rows_broadcast(T (&s)[E], int R) {
#pragma unroll
  for (int r = E / 2; r >= 1; r >>= 1) {
    if (r < R) {
#pragma unroll
      for (int j = 0; j < E; j += 2 * r) s[j + r] = s[j];
    }
  }
}

// Reduce per-row, per-lane partials over groups of 2^lg elements.  lg <= 9: the group is
// 2^(lg-3) adjacent lanes of one row.  lg > 9: the group is 2^(lg-9) whole rows; rows are
// first reduced over all 64 lanes, then combined pairwise, so that sums follow the
// canonical tree (512-element blocks first, then blocks two by two).
template <int E, class T, class Op>
__device__ __forceinline__ void groups_reduce(T (&s)[E], uint32_t lg, Op op) {
  if (lg <= 9) {
    const int lanes = 1 << (lg - 3);
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = lanes_reduce(s[j], lanes, op);
  } else {
    const int R = 1 << (lg - 9);
#pragma unroll
    for (int j = 0; j < E; ++j) s[j] = lanes_reduce(s[j], kWave, op);
    rows_combine<E>(s, R, op);
    rows_broadcast<E>(s, R);
  }
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1) v += __shfl_xor(v, m);
  return v;
}

// ------------------------------------------------------------------ chained scan across tiles
struct ScanCtx {
  uint64_t* state;
  uint32_t tag;         // epoch << 2
  uint32_t spin_limit;  // polls before a wavefront gives up
};

__device__ __forceinline__ uint64_t ld_state(const uint64_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_state(uint64_t* p, uint32_t hi, uint32_t lo) {
  __hip_atomic_store(p, ((uint64_t)hi << 32) | lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Single-pass scan of the per-tile outlier counts with decoupled look-back, one tile per
// wavefront.  scan_publish makes the tile's own count visible as early as possible;
// scan_resolve walks back over 64 predecessors at a time, one per lane, adding their counts
// until it meets a tile that already knows its inclusive prefix, then publishes its own.
// Tiles are numbered in launch order (workgroup index, wavefront index), and a tile only ever
// waits for lower-numbered ones, which the hardware has dispatched earlier.  The poll bound is
// a second line of defence: when it trips, the tile publishes "abort", which every later tile
// inherits at once, so the kernel always drains and reports the failure in the status words.
__device__ __forceinline__ void scan_publish(const ScanCtx& sc, uint32_t gtile, uint32_t first, uint32_t count) {
  if (lane_id() == 0)
    st_state(&sc.state[gtile], sc.tag | (gtile == first ? kFlagPrefix : kFlagAggregate), count);
}

__device__ __forceinline__ uint32_t scan_resolve(const ScanCtx& sc, uint32_t gtile, uint32_t first,
                                                 uint32_t count, bool& aborted) {
  const int lane = lane_id();
  aborted = false;
  if (gtile == first) return 0;
  uint32_t excl = 0;
  int64_t top = (int64_t)gtile - 1;
  while (true) {
    const int64_t p = top - lane;
    const bool in_range = p >= (int64_t)first;
    uint32_t flag = kFlagPrefix, value = 0;
    uint32_t polls = 0;
    uint64_t pm, need;
    int last;
    while (true) {
      if (in_range) {
        const uint64_t w = ld_state(&sc.state[p]);
        const uint32_t hi = (uint32_t)(w >> 32);
        flag = ((hi & ~3u) == sc.tag) ? (hi & 3u) : (uint32_t)kFlagEmpty;
        value = (uint32_t)w;
      }
      pm = __ballot(flag >= kFlagPrefix);
      last = pm ? __builtin_ctzll(pm) : kWave - 1;  // nearest tile that ends the walk
      need = (last == kWave - 1) ? ~0ull : ((2ull << last) - 1ull);
      if ((__ballot(flag == kFlagEmpty) & need) == 0) break;
      if (++polls > sc.spin_limit) { aborted = true; break; }
      __builtin_amdgcn_s_sleep(1);
    }
    if (aborted) break;
    if (__ballot(flag == kFlagAbort) & need) { aborted = true; break; }
    excl += wave_sum_u32(lane <= last ? value : 0u);
    if (pm) break;
    top -= kWave;
  }
  if (lane == 0) st_state(&sc.state[gtile], sc.tag | (aborted ? kFlagAbort : kFlagPrefix), excl + count);
  return excl;
}

// ------------------------------------------------------------------ one tile
template <int MODE, int BITS, bool ASYM, int E>
__device__ __forceinline__ void compress_tile(const TensorDesc& d, uint32_t tile, const ScanCtx& sc) {
  constexpr int Q = 1 << (BITS - 1);
  const int lane = lane_id();
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const uint64_t lane_base = tile_base + (uint64_t)lane * kOct;

  // ---- a1: load (16 bytes per lane per row; rows past the end read as zero)
  uint32_t raw[E][4];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint64_t e0 = lane_base + (uint64_t)j * kRow;
    if (e0 < d.numel) {
      const uint4 v = *reinterpret_cast<const uint4*>(d.src + e0);
      raw[j][0] = v.x; raw[j][1] = v.y; raw[j][2] = v.z; raw[j][3] = v.w;
    } else {
      raw[j][0] = raw[j][1] = raw[j][2] = raw[j][3] = 0u;
    }
  }

  // ---- a2 + a3: statistics and outlier mask (bit e of mask[j] = element e of row j)
  uint32_t mask[E];
#pragma unroll
  for (int j = 0; j < E; ++j) mask[j] = 0u;

  if constexpr (MODE == kModeAbs) {
    const float tau = d.param;
#pragma unroll
    for (int j = 0; j < E; ++j) {
#pragma unroll
      for (int e = 0; e < kOct; ++e)
        mask[j] |= (fabsf(ADACC_ELEM_F32(raw[j], e)) > tau) ? (1u << e) : 0u;
    }
  } else if constexpr (MODE == kModeStd) {
    float s1[E], s2[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      float x[kOct];
#pragma unroll
      for (int e = 0; e < kOct; ++e) x[e] = ADACC_ELEM_F32(raw[j], e);
      s1[j] = ((x[0] + x[1]) + (x[2] + x[3])) + ((x[4] + x[5]) + (x[6] + x[7]));
      // squares of bf16 values are exact in binary32
      s2[j] = ((x[0] * x[0] + x[1] * x[1]) + (x[2] * x[2] + x[3] * x[3])) +
              ((x[4] * x[4] + x[5] * x[5]) + (x[6] * x[6] + x[7] * x[7]));
    }
    groups_reduce<E>(s1, d.lgs, OpAdd());
    groups_reduce<E>(s2, d.lgs, OpAdd());
    const float inv_gs = __uint_as_float((127u - d.lgs) << 23);  // 2^-lgs, exact
    const float k2 = d.param;
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float mean = s1[j] * inv_gs;
      float var = __fmaf_rn(-mean, mean, s2[j] * inv_gs);
      var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
      const float limit = k2 * var;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        const float xe = ADACC_ELEM_F32(raw[j], e);
        mask[j] |= (xe * xe > limit) ? (1u << e) : 0u;
      }
    }
  } else if constexpr (MODE == kModeTopk) {
    // key = magnitude bits above, reversed position in the group below: the k largest keys
    // are the k largest magnitudes with ties going to the lower index; keys are unique.
    const uint32_t lgs = d.lgs;
    const int R = (lgs > 9) ? (1 << (lgs - 9)) : 1;
    const uint32_t lane_pos = (lgs > 9) ? ((uint32_t)lane << 3) : (((uint32_t)lane & ((1u << (lgs - 3)) - 1u)) << 3);
    uint32_t kth[E];
#pragma unroll
    for (int j = 0; j < E; ++j) kth[j] = 0xFFFFFFFFu;
    for (uint32_t r = 0; r < d.topk; ++r) {
      uint32_t best[E];
#pragma unroll
      for (int j = 0; j < E; ++j) {
        const uint32_t row_pos = ((uint32_t)(j & (R - 1)) << 9) | lane_pos;
        uint32_t m = 0u;
#pragma unroll
        for (int e = 0; e < kOct; ++e) {
          const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
          const uint32_t cand = (key < kth[j]) ? key : 0u;
          m = (cand > m) ? cand : m;
        }
        best[j] = m;
      }
      if (lgs <= 9) {
        const int lanes = 1 << (lgs - 3);
#pragma unroll
        for (int j = 0; j < E; ++j) best[j] = lanes_reduce(best[j], lanes, OpUMax());
      } else {
        rows_combine<E>(best, R, OpUMax());
#pragma unroll
        for (int j = 0; j < E; ++j)
          if ((j & (R - 1)) == 0) best[j] = lanes_reduce(best[j], kWave, OpUMax());
        rows_broadcast<E>(best, R);
      }
#pragma unroll
      for (int j = 0; j < E; ++j) kth[j] = best[j];
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint32_t row_pos = ((uint32_t)(j & (R - 1)) << 9) | lane_pos;
#pragma unroll
      for (int e = 0; e < kOct; ++e) {
        const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (row_pos | (uint32_t)e));
        mask[j] |= (key >= kth[j]) ? (1u << e) : 0u;
      }
    }
  }

  // Inf / NaN can not be quantised: always an outlier (when outliers are kept), never in a scale
  uint32_t nonfinite[E];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    uint32_t nf = 0u;
#pragma unroll
    for (int e = 0; e < kOct; ++e) nf |= (ADACC_ELEM_MAG(raw[j], e) >= 0x7F80u) ? (1u << e) : 0u;
    nonfinite[j] = nf;
    if constexpr (MODE != kModeNone) mask[j] |= nf;
  }
  // rows past the end of the tensor hold zeros; they must never yield outliers (TOPK ranks zeros too)
#pragma unroll
  for (int j = 0; j < E; ++j)
    if (lane_base + (uint64_t)j * kRow >= d.numel) mask[j] = 0u;

  // ---- a4 (first half): count the outliers and publish the tile's count before the long
  // quantise / store phase, so that later tiles rarely have to wait for it
  constexpr int W = E / 2;
  uint32_t cnt[E], lane_excl[E], row_off[E];
  uint32_t total = 0u;
  if constexpr (MODE != kModeNone) {
    // inclusive scan over lanes of the per-row counts, two rows per 32-bit word
    uint32_t packed[W];
#pragma unroll
    for (int j = 0; j < E; ++j) cnt[j] = __popc(mask[j]);
#pragma unroll
    for (int w = 0; w < W; ++w) packed[w] = cnt[2 * w] | (cnt[2 * w + 1] << 16);
#pragma unroll
    for (int dlt = 1; dlt < kWave; dlt <<= 1) {
#pragma unroll
      for (int w = 0; w < W; ++w) {
        const uint32_t t = __shfl_up(packed[w], dlt);
        packed[w] += (lane >= dlt) ? t : 0u;
      }
    }
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint32_t incl = (packed[j >> 1] >> ((j & 1) * 16)) & 0xFFFFu;
      lane_excl[j] = incl - cnt[j];
      row_off[j] = total;
      total += __shfl(incl, kWave - 1);
    }
    scan_publish(sc, d.first_tile + tile, d.first_tile, total);
  }

  // ---- a5 + a6: inlier view and per-group scale (and offset)
  float y[E][kOct];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint32_t zero = mask[j] | nonfinite[j];
#pragma unroll
    for (int e = 0; e < kOct; ++e) y[j][e] = ((zero >> e) & 1u) ? 0.0f : ADACC_ELEM_F32(raw[j], e);
  }

  float inv[E], off[E], scl[E];
  if constexpr (!ASYM) {
    float a[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      float m = 0.0f;
#pragma unroll
      for (int e = 0; e < kOct; ++e) m = fmaxf(m, fabsf(y[j][e]));
      a[j] = m;
    }
    groups_reduce<E>(a, d.lgq, OpMax());
#pragma unroll
    for (int j = 0; j < E; ++j) {
      scl[j] = a[j] / d.divisor;                                           // Eq. 2: S = max|X| / D
      inv[j] = (a[j] != 0.0f) ? fminf(d.divisor / a[j], 3.402823466e+38f) : 0.0f;  // one division per group
      off[j] = 0.0f;
    }
  } else {
    float hi[E], lo[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      float mx = y[j][0], mn = y[j][0];
#pragma unroll
      for (int e = 1; e < kOct; ++e) { mx = fmaxf(mx, y[j][e]); mn = fminf(mn, y[j][e]); }
      hi[j] = mx; lo[j] = mn;
    }
    groups_reduce<E>(hi, d.lgq, OpMax());
    groups_reduce<E>(lo, d.lgq, OpMin());
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const float h = hi[j] + 0.0f, l = lo[j] + 0.0f;  // a zero extreme is +0 whatever signs the zeros had
      const float o = (h + l) * 0.5f;                   // Eq. 3: O = (max+min)/2
      const float r = h - l;
      off[j] = o;
      scl[j] = r / d.divisor;                           // Eq. 3: S = (max-min) / D2
      inv[j] = (r != 0.0f) ? fminf(d.divisor / r, 3.402823466e+38f) : 0.0f;
    }
  }

  // ---- a7 + a8: quantise, pack, store codes and scales
  const uint32_t q_lanes_mask = (d.lgq <= 9) ? ((1u << (d.lgq - 3)) - 1u) : 63u;
  const uint32_t q_rows_mask = (d.lgq <= 9) ? 0u : ((1u << (d.lgq - 9)) - 1u);
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint64_t e0 = lane_base + (uint64_t)j * kRow;
    if (e0 >= d.numel) continue;
    int c[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) {
      const float t = ASYM ? (y[j][e] - off[j]) * inv[j] : y[j][e] * inv[j];
      float r = __builtin_rintf(t);          // nearest, ties to even
      r = fmaxf(r, (float)(-Q));             // a NaN lands on the lower bound
      r = fminf(r, (float)(Q - 1));          // "values greater than 7 are capped at 7"
      c[e] = (int)r;
    }
    if constexpr (BITS == 8) {
      uint2 w;
      w.x = (uint32_t)(c[0] & 0xFF) | ((uint32_t)(c[1] & 0xFF) << 8) | ((uint32_t)(c[2] & 0xFF) << 16) | ((uint32_t)c[3] << 24);
      w.y = (uint32_t)(c[4] & 0xFF) | ((uint32_t)(c[5] & 0xFF) << 8) | ((uint32_t)(c[6] & 0xFF) << 16) | ((uint32_t)c[7] << 24);
      *reinterpret_cast<uint2*>(d.codes + e0) = w;
    } else {
      uint32_t w = 0u;
#pragma unroll
      for (int e = 0; e < kOct; ++e) w |= (uint32_t)(c[e] & 0xF) << (4 * e);
      *reinterpret_cast<uint32_t*>(d.codes + (e0 >> 1)) = w;
    }
    if (((uint32_t)lane & q_lanes_mask) == 0u && ((uint32_t)j & q_rows_mask) == 0u) {
      const uint64_t g = e0 >> d.lgq;
      d.scales[g] = scl[j];
      if constexpr (ASYM) d.zp[g] = off[j];
    }
  }

  // ---- a4 (second half): resolve the tile's offset in the stream and append its outliers
  if constexpr (MODE != kModeNone) {
    bool aborted;
    const uint32_t base = scan_resolve(sc, d.first_tile + tile, d.first_tile, total, aborted);

    if (lane == 0) {
      d.tile_ptr[tile] = base;
      if (tile == d.n_tiles - 1) {
        const uint32_t n_out = base + total;
        d.tile_ptr[d.n_tiles] = n_out;
        d.status[0] = n_out;
        d.status[1] = (n_out > d.cap) ? 1u : 0u;
        d.status[3] = 0u;
        if (!aborted) d.status[2] = 0u;
      }
      if (aborted) d.status[2] = 1u;
    }
    if (total != 0u && !aborted) {
      static_for<E>([&](auto J) {
        constexpr int j = decltype(J)::value;
        uint32_t bits = mask[j];
        uint32_t pos = base + row_off[j] + lane_excl[j];
        const uint32_t i0 = (uint32_t)(lane_base + (uint64_t)j * kRow);
        while (bits) {
          const int e = __builtin_ctz(bits);
          bits &= bits - 1u;
          // element e of the octet by shifting (an indexed read would push the octets to scratch)
          const uint64_t half = (e < 4) ? (((uint64_t)raw[j][1] << 32) | raw[j][0]) : (((uint64_t)raw[j][3] << 32) | raw[j][2]);
          if (pos < d.cap) {
            d.idx[pos] = (int32_t)(i0 + (uint32_t)e);
            d.val[pos] = (uint16_t)(half >> (16 * (e & 3)));
          }
          ++pos;
        }
      });
    }
  } else {
    if (tile == 0 && lane == 0) {
      d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
    }
  }
}

}  // namespace adacc
