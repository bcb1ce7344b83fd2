// Compression and decompression for methods outside the fast kernels' shapes (Section 3.2 asks for groups
// of the activation and treats a tensor of any shape as a flat array; nothing there makes the groups powers
// of two): quantisation groups of any multiple of 8 elements, statistics groups of any multiple of the
// quantisation group up to 16384 elements (a whole 11008-wide row as one STD / TOPK group).  The fast
// kernels reduce over power-of-two numbers of lanes inside one wavefront's tile and cannot take these.
//
// Here a workgroup of four wavefronts takes a "segment": as many whole statistics groups as fit 4096
// elements (one group, if it is larger).  Thread t holds the octets t, t + 256, t + 512, .. of the segment in
// registers (one 16-byte load each, a wavefront's load is 1 KiB of consecutive memory); what the groups need
// from all their octets - the pairwise sums of the STD rule, the largest magnitude or the extremes of a
// quantisation group - goes through one word per octet in LDS and is reduced there by as many adjacent lanes
// as the group has octets (rounded up to a power of two; a wavefront per group beyond 64 octets, the whole
// workgroup beyond 256).  The definitions are those of the fast kernels: canonical pairwise sums (pad to a power
// of two, add neighbours level by level), mean and variance over the group's own count, the k largest by
// (magnitude, lower index), the correctly rounded D / max, the same rounding of the codes.
//
// Outliers take the ways of the tile kernels.  ABS / STD: a segment's outliers go to its slot of kSlot
// records in the workspace and its count to cnt[]; the placement kernels turn the counts into offsets and move
// the slots' records to the stream; a segment with more outliers than a slot holds is selected once more, by a
// second launch of this kernel (FIXUP) in which every other workgroup leaves at once.  TOPK: the offsets are
// known in advance (k per group), the outliers go straight to the stream, and a segment that finds another
// count (values that are not finite) raises the tensor's flag; only then do the placement kernel and the
// second launch anything: offsets from the counts, and every segment's outliers written again.
// The segment is the blob's tile (adacc_layout.tile_elems).
#pragma once

#include "adacc_common.hpp"
#include "adacc_compress.hpp"
#include "adacc_dtype.hpp"

namespace adacc {
namespace ADACC_DT_NS {

constexpr uint32_t kSegThreads = (uint32_t)kThreads;
constexpr uint32_t kSegWaves = kSegThreads / (uint32_t)kWave;
// octets per thread at most: 16384 elements / 8 / 256 threads = 8
// (the kernels exist for 2, 4, 6 and 8 octets per thread - SL - so that short segments do not pay for the registers of long ones)
// bytes of LDS before the segment's arrays: the words the wavefronts meet in
constexpr uint32_t kSegHeadWords = 64u;
constexpr uint32_t kSegHeadBytes = 4u * kSegHeadWords;

// The LDS of a workgroup, sized by the host for the method's segment length (n_oct = 256 * SL octets, one for each
// octet the threads hold, so that nobody has to ask whether its octet exists before it writes; n_grp quantisation groups):
// [head: 64 words][a: n_oct words][b: n_oct words][g0: n_grp words][g1: n_grp words]
//   head[0]      TOPK over a segment-wide group: entries in use of the list of candidate octets (in b)
//   head[8..39]  outliers of every (octet slice, wavefront)
//   head[40..55] the wavefronts' results of a group that the whole workgroup reduces (two sets of eight, used in turn)
//   a, b         one word per octet: sums / sums of squares (STD), largest magnitude or extreme keys (quantisation)
//   g0, g1       one word per group: the STD limit (and the mean) of a statistics group; the largest magnitude or the
//                extreme keys of a quantisation group
// TOPK over several groups of a segment keeps the segment's 16-bit patterns (16 bytes per octet, from a on) and
// behind them a byte per element instead, before a .. g1 are used (generic_lds_bytes gives the larger size).
struct SegmentShared {
  uint32_t* head;
  uint32_t* a;
  uint32_t* b;
  uint32_t* g0;
  uint32_t* g1;
  uint8_t* byte;  // TOPK over several groups: 1 = among the k largest
};
template <int SL>
__device__ __forceinline__ SegmentShared segment_shared(unsigned char* lds, uint32_t tile_elems, uint32_t gq) {
  constexpr uint32_t n_oct = (uint32_t)SL * kSegThreads;
  const uint32_t n_grp = (tile_elems + gq - 1u) / gq;
  SegmentShared sh;
  sh.head = reinterpret_cast<uint32_t*>(lds);
  sh.a = sh.head + kSegHeadWords;
  sh.b = sh.a + n_oct;
  sh.g0 = sh.b + n_oct;
  sh.g1 = sh.g0 + n_grp;
  sh.byte = reinterpret_cast<uint8_t*>(sh.a) + 16u * n_oct;
  return sh;
}

// What a thread knows of the segment and of its own octets
struct SegmentGeo {
  uint64_t first_elem;  // tensor index of the segment's first element (a multiple of 8)
  uint32_t cnt;         // elements of the segment (the tensor's last one may be short)
  uint32_t octs;        // octets that hold any of them
  bool full;            // uniform: cnt is the method's segment length (then every octet below octs is whole)
};
// octet o = tid + 256 * j is the thread's octet j

// o / opg for octets o < 2048 and 1 <= opg <= 2048 without the division sequence: `r` is 1 / opg moved up by three
// units in the last place, so that the binary32 product lies at or above the quotient where the quotient is an
// integer, and (the excess is below o * 2^-21 / opg < 1 / opg) below the next integer everywhere else.
__device__ __forceinline__ float group_reciprocal(uint32_t opg) {
  return __uint_as_float(__float_as_uint(__frcp_rn((float)opg)) + 3u);
}
__device__ __forceinline__ uint32_t group_of(uint32_t o, float r) { return (uint32_t)((float)o * r); }
__device__ __forceinline__ uint32_t octet_valid(const SegmentGeo& g, uint32_t o) {  // elements of octet o that exist
  const uint32_t first = o * (uint32_t)kOct;
  return first >= g.cnt ? 0u : (g.cnt - first < (uint32_t)kOct ? g.cnt - first : (uint32_t)kOct);
}

// reduce over LANES = 2^lg adjacent lanes, lg a run-time (uniform) value
template <class T, class Op>
__device__ __forceinline__ T lanes_reduce_lg(T v, uint32_t lg, Op op) {
  switch (lg) {
    case 0: break;
    case 1: v = lanes_reduce<2>(v, op); break;
    case 2: v = lanes_reduce<4>(v, op); break;
    case 3: v = lanes_reduce<8>(v, op); break;
    case 4: v = lanes_reduce<16>(v, op); break;
    case 5: v = lanes_reduce<32>(v, op); break;
    default: v = lanes_reduce<64>(v, op); break;
  }
  return v;
}

// For every group of `opg` consecutive octets (the last group of the segment may have fewer; n_oct octets in
// all): the balanced binary tree `op` over the group's words w[], padded with `pad` to the next power of two;
// finish(group, result) is called by one thread per group.  Groups of up to 64 octets are taken by as many
// adjacent lanes as the padded group has octets, several groups to a wavefront; groups of up to 256 by a
// wavefront each; longer ones by the whole workgroup in turn, every thread folding the padded group's consecutive
// words that fall to it first, the wavefronts' results meeting in head[40..47] (two sets, used in turn).
// Called by all threads of the workgroup.  (For sums the padding adds +0.0 to partial sums, which changes no value.)
// TWO: the same for a second array w1 with its own operation at the same time (sums and sums of squares; maxima
// and minima): finish(group, result of w0, result of w1).
template <bool TWO, class T, class Op0, class Op1, class Finish>
__device__ __forceinline__ void groups_tree(SegmentShared& sh, const uint32_t* w0, const uint32_t* w1, uint32_t n_oct,
                                            uint32_t opg, T pad0, T pad1, Op0 op0, Op1 op1, Finish finish) {
  const uint32_t lane = (uint32_t)lane_id(), wave = threadIdx.x / (uint32_t)kWave;
  const uint32_t n_grp = (n_oct + opg - 1u) / opg;
  uint32_t lg = 0u;
  while ((1u << lg) < opg) ++lg;  // uniform
  if (lg <= 6u) {
    const uint32_t per_wave = (uint32_t)kWave >> lg;  // groups a wavefront takes at a time
    const uint32_t leaf = lane & ((1u << lg) - 1u);
    for (uint32_t g0 = wave * per_wave; g0 < n_grp; g0 += kSegWaves * per_wave) {  // uniform
      const uint32_t g = g0 + (lane >> lg);
      const uint32_t o = g * opg + leaf;
      const bool there = g < n_grp && leaf < opg && o < n_oct;
      T v0 = pad0, v1 = pad1;
      if (there) v0 = __builtin_bit_cast(T, w0[o]);
      if constexpr (TWO) { if (there) v1 = __builtin_bit_cast(T, w1[o]); }
      v0 = lanes_reduce_lg(v0, lg, op0);
      if constexpr (TWO) v1 = lanes_reduce_lg(v1, lg, op1);
      if (g < n_grp && leaf == 0u) finish(g, v0, v1);
    }
  } else if (lg <= 8u) {
    const uint32_t per = 1u << (lg - 6u);  // consecutive words per lane: 2 or 4
    for (uint32_t g = wave; g < n_grp; g += kSegWaves) {  // uniform
      const uint32_t left = n_oct - g * opg < opg ? n_oct - g * opg : opg;
      const uint32_t first = g * opg;
      // the lane's words as the tree over 4 with the pad for the rest (the identity: same value)
      T t[4], u[4];
#pragma unroll
      for (uint32_t i = 0; i < 4u; ++i) {
        const uint32_t o = lane * per + i;
        const bool there = i < per && o < left;
        t[i] = there ? __builtin_bit_cast(T, w0[first + o]) : pad0;
        if constexpr (TWO) u[i] = there ? __builtin_bit_cast(T, w1[first + o]) : pad1;
      }
      const T v0 = lanes_reduce<kWave>(op0(op0(t[0], t[1]), op0(t[2], t[3])), op0);
      T v1 = pad1;
      if constexpr (TWO) v1 = lanes_reduce<kWave>(op1(op1(u[0], u[1]), op1(u[2], u[3])), op1);
      if (lane == 0u) finish(g, v0, v1);
    }
  } else {
    static_assert(kSegWaves == 4, "the wavefronts' results are combined as a tree of four");
    const uint32_t per = 1u << (lg - 8u);  // words per thread: 2 .. 8
    for (uint32_t g = 0; g < n_grp; ++g) {  // uniform
      const uint32_t left = n_oct - g * opg < opg ? n_oct - g * opg : opg;
      const uint32_t first = g * opg;
      // the thread's `per` consecutive words as the tree over 8 with the pad for the rest (the identity: same value)
      T t[8], u[8];
#pragma unroll
      for (uint32_t i = 0; i < 8u; ++i) {
        const uint32_t o = threadIdx.x * per + i;
        const bool there = i < per && o < left;
        t[i] = there ? __builtin_bit_cast(T, w0[first + o]) : pad0;
        if constexpr (TWO) u[i] = there ? __builtin_bit_cast(T, w1[first + o]) : pad1;
      }
      T v0 = op0(op0(op0(t[0], t[1]), op0(t[2], t[3])), op0(op0(t[4], t[5]), op0(t[6], t[7])));
      v0 = lanes_reduce<kWave>(v0, op0);
      T v1 = pad1;
      if constexpr (TWO) {
        v1 = op1(op1(op1(u[0], u[1]), op1(u[2], u[3])), op1(op1(u[4], u[5]), op1(u[6], u[7])));
        v1 = lanes_reduce<kWave>(v1, op1);
      }
      uint32_t* meet = sh.head + 40u + (g & 1u) * 2u * kSegWaves;  // two sets of [w0: 4 words][w1: 4 words]
      if (lane == 0u) {
        meet[wave] = __builtin_bit_cast(uint32_t, v0);
        if constexpr (TWO) meet[kSegWaves + wave] = __builtin_bit_cast(uint32_t, v1);
      }
      __syncthreads();
      if (threadIdx.x == 0u) {
        const T r0 = op0(op0(__builtin_bit_cast(T, meet[0]), __builtin_bit_cast(T, meet[1])),
                         op0(__builtin_bit_cast(T, meet[2]), __builtin_bit_cast(T, meet[3])));
        T r1 = pad1;
        if constexpr (TWO)
          r1 = op1(op1(__builtin_bit_cast(T, meet[4]), __builtin_bit_cast(T, meet[5])),
                   op1(__builtin_bit_cast(T, meet[6]), __builtin_bit_cast(T, meet[7])));
        finish(g, r0, r1);
      }
    }
    __syncthreads();  // the words in head[] are free for the next call
  }
}

// ---- a1: the thread's octets.  Whole octets with one 16-byte load, the tensor's ragged end one by one;
// what does not exist reads as +0.  The loads of all slices are issued without a branch between them (an
// octet that does not exist reads the segment's first one again and is blanked afterwards): a load under
// a branch is waited for at the end of that branch, and the slices' memory round trips would add up.
template <int SL>
__device__ __forceinline__ void segment_load(const TensorDesc& d, const SegmentGeo& g, uint32_t (&raw)[SL][4]) {
  const uint16_t* sp = d.src + g.first_elem;
  const uint32_t whole = g.cnt / (uint32_t)kOct;  // uniform
  if (whole != 0u) {
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      const uint32_t o = threadIdx.x + (uint32_t)j * kSegThreads;
      const uint4 v = ADACC_LOAD16(sp + (o < whole ? o : 0u) * (uint32_t)kOct);
      raw[j][0] = v.x; raw[j][1] = v.y; raw[j][2] = v.z; raw[j][3] = v.w;
    }
  }
#pragma unroll
  for (int j = 0; j < SL; ++j) {
    const uint32_t o = threadIdx.x + (uint32_t)j * kSegThreads;
    if (whole == 0u || o >= whole) raw[j][0] = raw[j][1] = raw[j][2] = raw[j][3] = 0u;
  }
  if ((g.cnt & 7u) != 0u) {  // uniform: the tensor's last segment
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      const uint32_t o = threadIdx.x + (uint32_t)j * kSegThreads;
      if (o == whole) {
#pragma unroll
        for (int e = 0; e < kOct - 1; ++e) {
          if ((uint32_t)e < (g.cnt & 7u)) raw[j][e >> 1] |= (uint32_t)sp[o * (uint32_t)kOct + (uint32_t)e] << (16 * (e & 1));
        }
      }
    }
  }
}

// bit e: element e of the octet is not finite
__device__ __forceinline__ uint32_t octet_nonfinite(const uint32_t (&oct)[4]) {
  uint32_t m = 0u;
#pragma unroll
  for (int e = 0; e < kOct; ++e) m |= (ADACC_ELEM_MAG(oct, e) >= kNonfiniteMag ? 1u : 0u) << e;
  return m;
}

// ---- a2 / a3: mask[j] bit e = element e of the thread's octet j is an outlier by the method's rule
// omag[j]: the largest magnitude of octet j, as the 15 low bits of the pattern
template <int SL>
__device__ __forceinline__ void segment_select(const TensorDesc& d, const SegmentGeo& g, SegmentShared& sh,
                                               const uint32_t (&raw)[SL][4], const uint32_t (&omag)[SL],
                                               uint32_t (&mask)[SL]) {
  const uint32_t tid = threadIdx.x;
#pragma unroll
  for (int j = 0; j < SL; ++j) mask[j] = 0u;
  if (d.mode == kModeAbs) {
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      // no element passes where the octet's largest magnitude does not (an octet with a NaN is looked at)
      if (!(widen_lo(omag[j]) <= d.param)) {
#pragma unroll
        for (int e = 0; e < kOct; ++e) mask[j] |= (fabsf(ADACC_ELEM_F32(raw[j], e)) > d.param ? 1u : 0u) << e;
      }
    }
  } else if (d.mode == kModeStd) {
    // the three lowest levels of the pairwise sums inside the octet, the rest over the octets' words
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      const uint32_t o = tid + (uint32_t)j * kSegThreads;  // (an octet that does not exist holds zeros; its words are not read)
      float v[kOct];
      widen_row(raw[j], v);
      sh.a[o] = __float_as_uint(((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
#pragma unroll
      for (int e = 0; e < kOct; ++e) v[e] = v[e] * v[e];
      sh.b[o] = __float_as_uint(((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7])));
    }
    __syncthreads();
    const uint32_t opg = d.gs / (uint32_t)kOct;
    groups_tree<true, float>(sh, sh.a, sh.b, g.octs, opg, 0.0f, 0.0f, OpAdd(), OpAdd(), [&](uint32_t grp, float s1, float s2) {
      const uint32_t left = g.cnt - grp * d.gs;
      const float n = (float)(left < d.gs ? left : d.gs);
      const float m = __fdiv_rn(s1, n);
      float var = __fmaf_rn(-m, m, __fdiv_rn(s2, n));
      var = (var < 0.0f) ? 0.0f : var;  // a NaN stays a NaN: then nothing passes the test
      sh.g0[grp] = __float_as_uint(d.param * var);  // param = k * k
    });
    __syncthreads();
    const float r = group_reciprocal(opg);
    const uint32_t last_grp = (g.octs - 1u) / opg;  // uniform
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      const uint32_t o = tid + (uint32_t)j * kSegThreads;
      // (zeros - what does not exist - pass no limit: a limit is never negative)
      const uint32_t grp = group_of(o, r);
      const float limit = __uint_as_float(sh.g0[grp < last_grp ? grp : last_grp]);
      const float top = widen_lo(omag[j]);
      if (!(top * top <= limit)) {  // the square is monotonic: no element passes where the largest magnitude does not
#pragma unroll
        for (int e = 0; e < kOct; ++e) {
          const float v = ADACC_ELEM_F32(raw[j], e);
          mask[j] |= (v * v > limit ? 1u : 0u) << e;
        }
      }
    }
    __syncthreads();  // a, b, g0, g1 are free again
  } else if (d.mode == kModeTopk) {
    if (d.gs >= d.tile_elems) {
      // The segment is one group.  The k largest elements lie in the k octets with the largest octet maxima (an
      // element outside them is beaten by one element of each of them), and those octets are among the k best
      // octets of every wavefront.  So: (1) every wavefront picks its k best octets by k rounds of a maximum over
      // its own lanes - keys in registers, the winner's owner only zeroes one key -, (2) the four lists meet in LDS
      // and every wavefront finds the k best octets overall by k rounds over the 4 k keys; the owner of each
      // of them (3) writes the keys of its 8 elements to an entry of a list in LDS, and (4) every wavefront finds
      // the k-th largest of those 8 k element keys, the threshold: an element is an outlier if its key reaches
      // it.  Three barriers whatever k is, and no step where one thread works while the workgroup waits.
      // Keys: magnitude above the reversed octet number resp. element index; 0 = nothing.
      const uint32_t lane = (uint32_t)lane_id(), wave = tid / (uint32_t)kWave;
      const uint32_t rounds = d.topk < g.cnt ? d.topk : g.cnt;  // at most 32
      uint32_t okey[SL];
#pragma unroll
      for (int j = 0; j < SL; ++j) {
        const uint32_t o = tid + (uint32_t)j * kSegThreads;
        okey[j] = o < g.octs ? (omag[j] << 16) | (0xFFFFu - o) : 0u;  // (elements that do not exist are zeros: they do not raise omag)
      }
      {  // (1)
        uint32_t live[SL], cand = 0u;
#pragma unroll
        for (int j = 0; j < SL; ++j) live[j] = okey[j];
        for (uint32_t r = 0; r < rounds; ++r) {  // uniform
          uint32_t best = 0u;
#pragma unroll
          for (int j = 0; j < SL; ++j) best = live[j] > best ? live[j] : best;
          const uint32_t w = wave_max_u32_scalar(best);
#pragma unroll
          for (int j = 0; j < SL; ++j) live[j] = live[j] == w ? 0u : live[j];
          cand = lane == r ? w : cand;
        }
        if (lane < 32u) sh.a[wave * 32u + lane] = cand;
        sh.b[tid] = 0u;  // the list of (3): 8 keys for each of up to 32 octets
        if (tid == 0u) sh.head[0] = 0u;  // and the number of its entries in use
      }
      __syncthreads();
      uint32_t least = 0u;  // the smallest key among the k best octets overall (0: there are fewer octets, all are taken)
      {  // (2)
        if (rounds <= 16u) {  // uniform: the first 16 keys of the four lists, one per lane
          uint32_t c0 = sh.a[(lane >> 4) * 32u + (lane & 15u)];  // lane = 16 * wavefront + entry
          for (uint32_t r = 0; r < rounds; ++r) {
            least = wave_max_u32_scalar(c0);
            c0 = c0 == least ? 0u : c0;
          }
        } else {
          uint32_t c0 = sh.a[lane], c1 = sh.a[(uint32_t)kWave + lane];
          for (uint32_t r = 0; r < rounds; ++r) {
            least = wave_max_u32_scalar(c0 > c1 ? c0 : c1);
            c0 = c0 == least ? 0u : c0;
            c1 = c1 == least ? 0u : c1;
          }
        }
      }
      // (3): which entry of the list an octet gets does not matter, a counter in LDS hands them out
#pragma unroll
      for (int j = 0; j < SL; ++j) {
        if (okey[j] != 0u && okey[j] >= least) {  // at most k octets of the workgroup
          const uint32_t o = tid + (uint32_t)j * kSegThreads;
          const uint32_t nv = octet_valid(g, o);
          const uint32_t entry = atomicAdd(&sh.head[0], 1u) & 31u;  // (below 32 anyway: keys are unique)
#pragma unroll
          for (int e = 0; e < kOct; ++e)
            sh.b[entry * (uint32_t)kOct + (uint32_t)e] =
                (uint32_t)e < nv ? (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (o * (uint32_t)kOct + (uint32_t)e)) : 0u;
        }
      }
      __syncthreads();
      uint32_t limit = 0u;
      {  // (4)
        // (never 0: the octets of (2) hold at least `rounds` elements)
        if (rounds <= 8u) {  // uniform: at most 64 keys, one per lane
          uint32_t c = sh.b[lane];
          for (uint32_t r = 0; r < rounds; ++r) {
            limit = wave_max_u32_scalar(c);
            c = c == limit ? 0u : c;
          }
        } else {
          uint32_t c[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) c[k] = sh.b[(uint32_t)k * (uint32_t)kWave + lane];
          for (uint32_t r = 0; r < rounds; ++r) {
            const uint32_t m0 = c[0] > c[1] ? c[0] : c[1], m1 = c[2] > c[3] ? c[2] : c[3];
            limit = wave_max_u32_scalar(m0 > m1 ? m0 : m1);
#pragma unroll
            for (int k = 0; k < 4; ++k) c[k] = c[k] == limit ? 0u : c[k];
          }
        }
      }
#pragma unroll
      for (int j = 0; j < SL; ++j) {
        if (okey[j] != 0u && ((omag[j] << 16) | 0xFFFFu) >= limit) {  // few octets get here
          const uint32_t o = tid + (uint32_t)j * kSegThreads;
          const uint32_t nv = octet_valid(g, o);
#pragma unroll
          for (int e = 0; e < kOct; ++e) {
            const uint32_t key = (ADACC_ELEM_MAG(raw[j], e) << 16) | (0xFFFFu - (o * (uint32_t)kOct + (uint32_t)e));
            mask[j] |= ((uint32_t)e < nv && key >= limit ? 1u : 0u) << e;
          }
        }
      }
      __syncthreads();  // a, b are free again
    } else {
      // Several groups (of at most 2048 elements): the patterns go to LDS, a wavefront takes a group at a time
      // with the keys of its elements in registers (2, 8 or 32 per lane by the size of the groups), k rounds of a
      // maximum over the wavefront.
      uint16_t* pat = reinterpret_cast<uint16_t*>(sh.a);
#pragma unroll
      for (int j = 0; j < SL; ++j) {
        const uint32_t o = tid + (uint32_t)j * kSegThreads;
        if (o < g.octs)
          *reinterpret_cast<uint4*>(pat + o * (uint32_t)kOct) = make_uint4(raw[j][0], raw[j][1], raw[j][2], raw[j][3]);
      }
      __syncthreads();
      const uint32_t lane = (uint32_t)lane_id();
      // KC: keys per lane, 64 * KC elements at most in a group
      auto groups_of = [&](auto KCc) {
        constexpr int KC = decltype(KCc)::value;
        for (uint32_t e0 = (tid / (uint32_t)kWave) * d.gs; e0 < g.cnt; e0 += kSegWaves * d.gs) {  // uniform
          const uint32_t n = g.cnt - e0 < d.gs ? g.cnt - e0 : d.gs;
          uint32_t key[KC];
#pragma unroll
          for (int k = 0; k < KC; ++k) {
            const uint32_t i = lane + (uint32_t)k * (uint32_t)kWave;
            key[k] = i < n ? (((uint32_t)(pat[e0 + i] & 0x7FFFu) << 16) | (0xFFFFu - i)) : 0u;
          }
          const uint32_t rounds = d.topk < n ? d.topk : n;
          for (uint32_t r = 0; r < rounds; ++r) {
            uint32_t best = 0u;
#pragma unroll
            for (int k = 0; k < KC; ++k) best = key[k] > best ? key[k] : best;
            const uint32_t win = wave_max_u32_scalar(best);
#pragma unroll
            for (int k = 0; k < KC; ++k) key[k] = key[k] == win ? 0u : key[k];
          }
#pragma unroll
          for (int k = 0; k < KC; ++k) {
            const uint32_t i = lane + (uint32_t)k * (uint32_t)kWave;
            if (i < n) sh.byte[e0 + i] = key[k] == 0u ? 1 : 0;
          }
        }
      };
      if (d.gs <= 2u * (uint32_t)kWave) groups_of(std::integral_constant<int, 2>());       // uniform
      else if (d.gs <= 8u * (uint32_t)kWave) groups_of(std::integral_constant<int, 8>());
      else groups_of(std::integral_constant<int, 32>());
      __syncthreads();
#pragma unroll
      for (int j = 0; j < SL; ++j) {
        const uint32_t o = tid + (uint32_t)j * kSegThreads;
        if (o < g.octs) {
          const uint2 f = *reinterpret_cast<const uint2*>(sh.byte + o * (uint32_t)kOct);
          const uint32_t nv = octet_valid(g, o);
#pragma unroll
          for (int e = 0; e < kOct; ++e) {
            const uint32_t bit = ((e < 4 ? f.x : f.y) >> (8 * (e & 3))) & 1u;
            mask[j] |= ((uint32_t)e < nv ? bit : 0u) << e;
          }
        }
      }
      __syncthreads();  // a, b and the bytes are free again
    }
  }
}

// ---- a4: the outliers of the segment (mask[]), in index order, to entries pos0, pos0 + 1, .. of the sink
// (entries at or past `limit` are dropped).  Returns their number (uniform).
template <int SL, class Sink>
__device__ __forceinline__ uint32_t segment_emit(const SegmentGeo& g, SegmentShared& sh, const uint32_t (&raw)[SL][4],
                                                 const uint32_t (&mask)[SL], const Sink& sink, uint32_t pos0,
                                                 uint32_t limit) {
  const uint32_t tid = threadIdx.x, wave = tid / (uint32_t)kWave;
  uint32_t* counts = sh.head + 8u;  // [slice][wavefront]
  // outliers of each of this wavefront's octet slices (element order is slice, wavefront, lane)
#pragma unroll
  for (int j = 0; j < SL; ++j) {
    uint32_t c = 0u;
    if (__builtin_amdgcn_ballot_w64(mask[j] != 0u) != 0ull) c = wave_sum_u32(__builtin_popcount(mask[j]));
    if (lane_id() == 0) counts[(uint32_t)j * kSegWaves + wave] = c;
  }
  __syncthreads();
  uint32_t total = 0u, before[SL];
#pragma unroll
  for (int j = 0; j < SL; ++j) {
#pragma unroll
    for (uint32_t w = 0; w < kSegWaves; ++w) {
      if (w == wave) before[j] = total;  // uniform in the wavefront
      total += counts[(uint32_t)j * kSegWaves + w];
    }
  }
  if (total != 0u) {  // uniform
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      const uint64_t any = __builtin_amdgcn_ballot_w64(mask[j] != 0u);
      if (any == 0ull) continue;  // uniform
      const bool sparse = __builtin_amdgcn_ballot_w64((mask[j] & (mask[j] - 1u)) != 0u) == 0ull;
      uint32_t lane_excl;
      if (sparse) {
        lane_excl = lanes_below(any);
      } else {
        const uint32_t c = (uint32_t)__builtin_popcount(mask[j]);
        uint32_t incl = c;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
          const uint32_t up = (uint32_t)__shfl_up((int)incl, off, kWave);
          if (lane_id() >= off) incl += up;
        }
        lane_excl = incl - c;
      }
      const uint32_t o = tid + (uint32_t)j * kSegThreads;
      emit_row(raw[j], mask[j], lane_excl, sparse, (uint32_t)g.first_elem + o * (uint32_t)kOct, sink, pos0 + before[j], limit);
    }
  }
  __syncthreads();  // counts[] is free again
  return total;
}

// ---- a6 .. a8: scales (offsets) of the quantisation groups and the codes of the thread's octets, from which
// outliers and values that are not finite are gone

// a7 / a8 for the thread's octet j = octet o of the segment, in group grp (of the segment), whose extremes are
// known: gm (symmetric: the largest magnitude) or the keys hi, lo (asymmetric).  Everything but the stores also
// for an octet that does not exist.
template <int BITS, bool ASYM>
__device__ __forceinline__ void octet_quantise(const TensorDesc& d, const SegmentGeo& g, const uint32_t (&oct)[4], uint32_t o,
                                               uint32_t grp, uint32_t opg, uint64_t first_group, uint32_t gm, int32_t hi,
                                               int32_t lo) {
  constexpr int Q = 1 << (BITS - 1);
  float scl, inv, off = 0.0f;
  if constexpr (!ASYM) scale_sym_clean(d, mag_bits32(gm), scl, inv);
  else group_scale<true>(d, 0u, hi, lo, scl, inv, off);
  uint32_t c[kOct];
#pragma unroll
  for (int e = 0; e < kOct; ++e) {
    const float y = ADACC_ELEM_F32(oct, e);
    c[e] = code_bits<Q, ASYM>(ASYM ? y - off : y, inv);  // symmetric codes cannot pass the lower bound
  }
  uint2 w8 = make_uint2(0u, 0u);
  uint32_t w4 = 0u;
  if constexpr (BITS == 8) {
    w8.x = pack_bytes4(c[0], c[1], c[2], c[3]);
    w8.y = pack_bytes4(c[4], c[5], c[6], c[7]);
  } else {
    w4 = pack_nibbles8(c);
  }
  if (o < g.octs) {
    if (grp * opg == o) {  // the group's first octet
      d.scales[first_group + grp] = scl;
      if constexpr (ASYM) d.zp[first_group + grp] = off;
    }
    const uint64_t e0 = g.first_elem + (uint64_t)o * kOct;
    const uint32_t nv = g.full ? (uint32_t)kOct : octet_valid(g, o);
    if constexpr (BITS == 8) {
      if (nv == (uint32_t)kOct) {
        ADACC_STORE8(d.codes + e0, w8);
      } else {  // the tensor's ragged end, byte by byte
#pragma unroll
        for (int e = 0; e < kOct - 1; ++e)
          if ((uint32_t)e < nv) d.codes[e0 + e] = (uint8_t)((e < 4 ? w8.x : w8.y) >> (8 * (e & 3)));
      }
    } else {
      if (nv == (uint32_t)kOct) {
        ADACC_STORE4(d.codes + (e0 >> 1), w4);
      } else {  // an odd end: the high nibble of the last byte is 0
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          if ((uint32_t)(2 * b) < nv) {
            uint32_t v = (w4 >> (8 * b)) & 0xFFu;
            if ((uint32_t)(2 * b + 1) >= nv) v &= 0x0Fu;
            d.codes[(e0 >> 1) + b] = (uint8_t)v;
          }
        }
      }
    }
  }
}

// the extreme keys of an octet's elements that exist (element 0 of an octet that exists does)
__device__ __forceinline__ void octet_extreme_keys(const SegmentGeo& g, const uint32_t (&oct)[4], uint32_t o, int32_t& hi,
                                                   int32_t& lo) {
  hi = float_key(widen_lo(oct[0]));
  lo = hi;
  if (g.full) {  // uniform
#pragma unroll
    for (int e = 1; e < kOct; ++e) {
      const int32_t k = float_key(ADACC_ELEM_F32(oct, e));
      hi = k > hi ? k : hi;
      lo = k < lo ? k : lo;
    }
  } else {
    const uint32_t nv = octet_valid(g, o);
#pragma unroll
    for (int e = 1; e < kOct; ++e) {
      const int32_t k = float_key(ADACC_ELEM_F32(oct, e));
      hi = ((uint32_t)e < nv && k > hi) ? k : hi;
      lo = ((uint32_t)e < nv && k < lo) ? k : lo;
    }
  }
}

// omag[j]: the largest magnitude of octet j as it is now
template <int BITS, bool ASYM, int SL>
__device__ __forceinline__ void segment_quantise(const TensorDesc& d, const SegmentGeo& g, SegmentShared& sh,
                                                 const uint32_t (&raw)[SL][4], const uint32_t (&omag)[SL]) {
  const uint32_t tid = threadIdx.x;
  const uint32_t opg = d.gq / (uint32_t)kOct;
  const uint64_t first_group = g.first_elem / d.gq;
  if ((opg & (opg - 1u)) == 0u && opg <= (uint32_t)kWave) {  // uniform
    // A group of 1, 2, 4, .. 64 octets is as many adjacent lanes of one wavefront (the segment starts on a group,
    // and 256 octets are whole groups): the extremes meet by the xor butterfly, in registers.  An octet that does
    // not exist brings the identity.
    const uint32_t lg = (uint32_t)__builtin_ctz(opg);
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      const uint32_t o = tid + (uint32_t)j * kSegThreads;
      if constexpr (!ASYM) {
        const uint32_t gm = lanes_reduce_lg(omag[j], lg, OpUMax());  // (zeros cannot raise the maximum)
        octet_quantise<BITS, false>(d, g, raw[j], o, o >> lg, opg, first_group, gm, 0, 0);
      } else {
        int32_t hi, lo;
        octet_extreme_keys(g, raw[j], o, hi, lo);
        hi = o < g.octs ? hi : (int32_t)0x80000000;
        lo = o < g.octs ? lo : (int32_t)0x7FFFFFFF;
        hi = lanes_reduce_lg(hi, lg, OpIMax());
        lo = lanes_reduce_lg(lo, lg, OpIMin());
        octet_quantise<BITS, true>(d, g, raw[j], o, o >> lg, opg, first_group, 0u, hi, lo);
      }
    }
    return;
  }
  if (d.gq >= d.tile_elems) {  // uniform
    // The segment is one group: the extremes meet thread by thread, wavefront by wavefront (any order does).
    static_assert(kSegWaves == 4, "four words per extreme in head[]");
    const uint32_t lane = (uint32_t)lane_id(), wave = tid / (uint32_t)kWave;
    uint32_t gm = 0u;
    int32_t hi = (int32_t)0x80000000, lo = (int32_t)0x7FFFFFFF;
    if constexpr (!ASYM) {
#pragma unroll
      for (int j = 0; j < SL; ++j) gm = omag[j] > gm ? omag[j] : gm;
      gm = wave_max_u32_scalar(gm);
      if (lane == 0u) sh.head[40u + wave] = gm;
    } else {
#pragma unroll
      for (int j = 0; j < SL; ++j) {
        const uint32_t o = tid + (uint32_t)j * kSegThreads;
        int32_t h, l;
        octet_extreme_keys(g, raw[j], o, h, l);
        hi = (o < g.octs && h > hi) ? h : hi;
        lo = (o < g.octs && l < lo) ? l : lo;
      }
      hi = lanes_reduce<kWave>(hi, OpIMax());
      lo = lanes_reduce<kWave>(lo, OpIMin());
      if (lane == 0u) { sh.head[40u + wave] = (uint32_t)hi; sh.head[44u + wave] = (uint32_t)lo; }
    }
    __syncthreads();
#pragma unroll
    for (uint32_t w = 0; w < kSegWaves; ++w) {
      if constexpr (!ASYM) {
        gm = sh.head[40u + w] > gm ? sh.head[40u + w] : gm;
      } else {
        const int32_t h = (int32_t)sh.head[40u + w], l = (int32_t)sh.head[44u + w];
        hi = h > hi ? h : hi;
        lo = l < lo ? l : lo;
      }
    }
#pragma unroll
    for (int j = 0; j < SL; ++j)
      octet_quantise<BITS, ASYM>(d, g, raw[j], tid + (uint32_t)j * kSegThreads, 0u, opg, first_group, gm, hi, lo);
    return;
  }
  // Other groups: one word (two) per octet to LDS (an octet that does not exist writes a word that nobody reads) ..
#pragma unroll
  for (int j = 0; j < SL; ++j) {
    const uint32_t o = tid + (uint32_t)j * kSegThreads;
    if constexpr (!ASYM) {
      sh.a[o] = omag[j];  // elements that do not exist are zero and cannot raise the maximum
    } else {
      int32_t hi, lo;
      octet_extreme_keys(g, raw[j], o, hi, lo);
      sh.a[o] = (uint32_t)hi;
      sh.b[o] = (uint32_t)lo;
    }
  }
  __syncthreads();
  // .. the groups' extremes to g0 (g1); every thread then forms D / max (and the offset) for each of its octets
  // itself instead of a few lanes doing it for all
  if constexpr (!ASYM) {
    groups_tree<false, uint32_t>(sh, sh.a, sh.a, g.octs, opg, 0u, 0u, OpUMax(), OpUMax(),
                                 [&](uint32_t grp, uint32_t mag, uint32_t) { sh.g0[grp] = mag; });
  } else {
    groups_tree<true, int32_t>(sh, sh.a, sh.b, g.octs, opg, (int32_t)0x80000000, (int32_t)0x7FFFFFFF, OpIMax(), OpIMin(),
                               [&](uint32_t grp, int32_t hi, int32_t lo) { sh.g0[grp] = (uint32_t)hi; sh.g1[grp] = (uint32_t)lo; });
  }
  __syncthreads();
  const float recip = group_reciprocal(opg);
  const uint32_t last_grp = (g.octs - 1u) / opg;  // uniform
#pragma unroll
  for (int j = 0; j < SL; ++j) {
    const uint32_t o = tid + (uint32_t)j * kSegThreads;
    uint32_t grp = group_of(o, recip);  // (an octet that does not exist takes the last group's values)
    grp = grp < last_grp ? grp : last_grp;
    if constexpr (!ASYM) octet_quantise<BITS, false>(d, g, raw[j], o, grp, opg, first_group, sh.g0[grp], 0, 0);
    else octet_quantise<BITS, true>(d, g, raw[j], o, grp, opg, first_group, 0u, (int32_t)sh.g0[grp], (int32_t)sh.g1[grp]);
  }
}

// The kernel's first argument (the tensor's descriptor, about fifty words) read again from the kernel argument
// segment, behind a barrier for the compiler: what a phase needs of it is then loaded (scalar loads) where the
// phase begins.  Otherwise all of it is loaded ahead of everything and, more than the scalar registers hold, is
// parked in lanes of vector registers, from where every use costs a lane read.
__device__ __forceinline__ const TensorDesc& descriptor_again() {
  typedef const __attribute__((address_space(4))) TensorDesc* KernargDesc;
  KernargDesc p = (KernargDesc)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(p));
  return *(const TensorDesc*)p;
}

// One segment (d.tile_elems elements, the last one of the tensor may be short).
// FIXUP: the second launch - only the outliers, straight to the stream at the offsets the placement kernel
// has written, and only where the first launch could not place them.
// d: the kernel's first argument
template <int SL, bool FIXUP>
__device__ __forceinline__ void compress_segment(const TensorDesc& d, SegmentShared& sh, uint32_t seg, uint32_t epoch) {
  const uint32_t tid = threadIdx.x;
  const bool topk = d.mode == kModeTopk;
  if constexpr (FIXUP) {
    if (topk) {
      if (__hip_atomic_load(d.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != epoch) return;  // uniform
    } else if (d.cnt[seg] <= (uint32_t)kSlot) {
      return;  // uniform
    }
  }
  SegmentGeo g;
  g.first_elem = (uint64_t)seg * d.tile_elems;
  const uint64_t left = d.numel - g.first_elem;
  g.cnt = left < (uint64_t)d.tile_elems ? (uint32_t)left : d.tile_elems;
  g.octs = (g.cnt + (uint32_t)kOct - 1u) / (uint32_t)kOct;
  g.full = g.cnt == d.tile_elems && (d.tile_elems & 7u) == 0u;
  uint32_t raw[SL][4];
  segment_load(d, g, raw);
  uint32_t mask[SL], omag[SL];
#pragma unroll
  for (int j = 0; j < SL; ++j) omag[j] = octet_magnitude(raw[j]);
  if (d.mode != kModeNone) {
    segment_select(descriptor_again(), g, sh, raw, omag, mask);
#pragma unroll
    for (int j = 0; j < SL; ++j)  // what cannot be quantised at all is always kept exactly
      if (omag[j] >= kNonfiniteMag) mask[j] |= octet_nonfinite(raw[j]);
    if constexpr (FIXUP) {
      const uint32_t pos0 = d.tile_ptr[seg], end = d.tile_ptr[seg + 1u];
      segment_emit(g, sh, raw, mask, StreamSink{d.idx, d.val}, pos0, end < d.cap ? end : d.cap);
      return;
    } else if (topk) {
      const uint32_t gps = d.tile_elems / d.gs;  // groups of a whole segment
      const uint32_t pos0 = seg * gps * d.topk;
      const uint32_t whole = g.cnt / d.gs, rest = g.cnt - whole * d.gs;
      const uint32_t expected = whole * d.topk + (rest < d.topk ? rest : d.topk);
      const uint32_t end = pos0 + expected;
      const uint32_t total = segment_emit(g, sh, raw, mask, StreamSink{d.idx, d.val}, pos0, end < d.cap ? end : d.cap);
      if (tid == 0u) {
        d.tile_ptr[seg] = pos0;
        d.cnt[seg] = total;
        if (total != expected) *d.flag = epoch;
        if (seg + 1u == d.n_tiles) {
          d.tile_ptr[d.n_tiles] = end;
          d.status[0] = end; d.status[1] = end > d.cap ? 1u : 0u; d.status[2] = 0u; d.status[3] = 0u;
        }
      }
    } else {
      const uint32_t total = segment_emit(g, sh, raw, mask, SlotSink{d.slot + (uint64_t)seg * (uint64_t)kSlot}, 0u, (uint32_t)kSlot);
      if (tid == 0u) d.cnt[seg] = total;
    }
  } else {
#pragma unroll
    for (int j = 0; j < SL; ++j) mask[j] = omag[j] >= kNonfiniteMag ? octet_nonfinite(raw[j]) : 0u;
    if (seg == 0u && tid == 0u) {
      d.status[0] = 0u; d.status[1] = 0u; d.status[2] = 0u; d.status[3] = 0u;
    }
  }
  if constexpr (!FIXUP) {
    const TensorDesc& d = descriptor_again();
    // a5: from here on the outliers, and every value that is not finite, count as zero
#pragma unroll
    for (int j = 0; j < SL; ++j) {
      if (mask[j] != 0u) {
        clear_elements(raw[j], mask[j]);
        omag[j] = octet_magnitude(raw[j]);
      }
    }
    if (d.bits == 8u) {
      if (d.asym) segment_quantise<8, true, SL>(d, g, sh, raw, omag); else segment_quantise<8, false, SL>(d, g, sh, raw, omag);
    } else {
      if (d.asym) segment_quantise<4, true, SL>(d, g, sh, raw, omag); else segment_quantise<4, false, SL>(d, g, sh, raw, omag);
    }
  }
}

// a9 / a10 for one segment
__device__ __forceinline__ void decompress_segment(const TensorDesc& d, uint32_t seg) {
  const uint32_t tid = threadIdx.x;
  const uint64_t first_elem = (uint64_t)seg * d.tile_elems;
  const uint64_t left = d.numel - first_elem;
  const uint32_t cnt = left < (uint64_t)d.tile_elems ? (uint32_t)left : d.tile_elems;
  const uint64_t first_group = first_elem / d.gq;
  // an octet at a time: it lies inside one quantisation group (groups are multiples of 8, the segment starts
  // on a group), so one scale serves it; what is left of a tensor's ragged end goes one by one
  const uint32_t octs = cnt / (uint32_t)kOct;
  for (uint32_t o = tid; o < octs; o += kSegThreads) {
    const uint64_t e0 = first_elem + (uint64_t)o * kOct;
    int code[kOct];
    if (d.bits == 8u) {
      const uint2 w = *reinterpret_cast<const uint2*>(d.codes + e0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        code[e] = (int)(int8_t)((w.x >> (8 * e)) & 0xFFu);
        code[4 + e] = (int)(int8_t)((w.y >> (8 * e)) & 0xFFu);
      }
    } else {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(d.codes + (e0 >> 1));
#pragma unroll
      for (int e = 0; e < kOct; ++e) code[e] = ((int)(w << (28 - 4 * e))) >> 28;  // sign-extended nibble
    }
    const uint64_t grp = first_group + (o * (uint32_t)kOct) / d.gq;
    const float s = d.scales[grp];
    const float z = d.asym ? d.zp[grp] : 0.0f;
    float v[kOct];
#pragma unroll
    for (int e = 0; e < kOct; ++e) v[e] = d.asym ? __fmaf_rn((float)code[e], s, z) : (float)code[e] * s;
    if (d.dst_f32) {
      float* p = reinterpret_cast<float*>(d.dst) + e0;
      *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
      *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(d.dst) + e0) =
          make_uint4(narrow_pair(v[0], v[1]), narrow_pair(v[2], v[3]), narrow_pair(v[4], v[5]), narrow_pair(v[6], v[7]));
    }
  }
  for (uint32_t i = octs * kOct + tid; i < cnt; i += kSegThreads) {
    int code;
    if (d.bits == 8u) code = (int)(int8_t)d.codes[first_elem + i];
    else code = ((int)((uint32_t)d.codes[(first_elem + i) >> 1] << (28u - 4u * (i & 1u)))) >> 28;  // first_elem is even
    const uint64_t grp = first_group + i / d.gq;
    const float s = d.scales[grp];
    const float v = d.asym ? __fmaf_rn((float)code, s, d.zp[grp]) : (float)code * s;
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[first_elem + i] = v;
    else reinterpret_cast<uint16_t*>(d.dst)[first_elem + i] = (uint16_t)narrow_pair(v, 0.0f);
  }
  if (d.mode == kModeNone) return;
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's stores above are complete ...
  __syncthreads();                       // ... and so are those of the other wavefronts of the segment
  uint32_t p0 = d.tile_ptr[seg], p1 = d.tile_ptr[seg + 1u];
  p0 = p0 < d.cap ? p0 : d.cap;
  p1 = p1 < d.cap ? p1 : d.cap;
  for (uint32_t p = p0 + tid; p < p1; p += kSegThreads) {
    const uint64_t i = (uint32_t)d.idx[p];
    if (i < first_elem || i >= first_elem + cnt) continue;  // a damaged stream must not write outside the segment
    const uint32_t pat = d.val[p];
    if (d.dst_f32) reinterpret_cast<float*>(d.dst)[i] = widen_lo(pat);
    else reinterpret_cast<uint16_t*>(d.dst)[i] = (uint16_t)pat;
  }
}

// wavefronts per SIMD (= workgroups per CU) the registers are held to: the kernel is a chain of memory and LDS
// round trips with barriers between, which only other resident workgroups can fill
template <int SL>
constexpr int generic_min_waves() { return SL <= 2 ? 8 : SL <= 4 ? 6 : SL <= 6 ? 4 : 3; }
template <int SL, bool FIXUP>
__global__ __launch_bounds__(kSegThreads, (generic_min_waves<SL>())) void compress_generic_kernel(TensorDesc d, uint32_t epoch) {
  extern __shared__ __attribute__((aligned(16))) unsigned char segment_lds[];
  SegmentShared sh = segment_shared<SL>(segment_lds, d.tile_elems, d.gq);
  compress_segment<SL, FIXUP>(d, sh, blockIdx.x, epoch);
}
__global__ __launch_bounds__(kSegThreads) void decompress_generic_kernel(TensorDesc d) { decompress_segment(d, blockIdx.x); }

}  // namespace ADACC_DT_NS
}  // namespace adacc
