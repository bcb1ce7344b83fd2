// Decompression of one tile by one wavefront (Section 3.2: X^ = code * S, resp. code * S + O,
// then the outliers are written back; Fig. 3(c) decompression workflow).
#pragma once

#include "adacc_common.hpp"
#include "adacc_dtype.hpp"

namespace adacc {
namespace ADACC_DT_NS {

// Decompression always works on pieces of E = 4 rows (2048 elements), whatever the tile of the
// blob: a piece of a 4096-element tile looks through the outliers of the whole tile and takes
// those that fall inside it.
//
// A piece whose tile has up to 64 outliers, no two of them in the same octet, takes them into the output
// words in registers before they are stored: the lanes that hold the entries of the stream drop them into a
// mailbox of the wavefront in LDS (one word per octet of the piece, 1 KiB), every lane picks up the four
// words of its own octets.  Otherwise the outliers are written over the dequantised values in memory: the
// piece is stored first, the wavefront waits until those stores have reached the L2 (its store counter at
// zero), and then stores the outliers of the piece, 2 (or 4) bytes each, to their positions.  Both rounds of
// stores come from the same wavefront and the second is issued only after the first is complete,
// so the outliers are what stays.  (Staging the whole piece in LDS to patch it there cost a round trip
// through LDS for every piece of a TOPK tensor, a third of the kernel's time.)
// One row (512 elements, 8 per lane) of a piece: codes and scale (offset) of the lane's octet.
template <int BITS>
struct RowCodes {
  uint32_t w[BITS == 8 ? 2 : 1];
  float s, o;
};

template <int BITS, bool ASYM>
__device__ __forceinline__ void load_row_codes(const TensorDesc& d, uint64_t e0, RowCodes<BITS>& r) {
  if constexpr (BITS == 8) {
    const uint2 w = *reinterpret_cast<const uint2*>(d.codes + e0);
    r.w[0] = w.x; r.w[1] = w.y;
  } else {
    r.w[0] = *reinterpret_cast<const uint32_t*>(d.codes + (e0 >> 1));
  }
  const uint64_t g = e0 >> d.lgq;
  r.s = d.scales[g];
  r.o = 0.0f;
  if constexpr (ASYM) r.o = d.zp[g];
}

// What a lane finds in the mailbox for one of its octets: 0, or bit 31 set, the element (0..7) in bits 16..18
// and the outlier's 16-bit pattern in the low half.  Applied to the output words of that row before they are
// stored: WORDS = 4 (two 16-bit values per word) or 8 (binary32).
constexpr uint32_t kMailFull = 0x80000000u;
template <int WORDS>
__device__ __forceinline__ void patch_row_words(uint32_t (&w)[WORDS], uint32_t mail) {
  const bool mine = mail != 0u;
  const uint32_t e = (mail >> 16) & 7u;
  const uint32_t pat = mail & 0xFFFFu;
  if constexpr (WORDS == 8) {
    const uint32_t bits = __float_as_uint(widen_lo(pat));
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = (mine && e == (uint32_t)k) ? bits : w[k];
  } else {
    const uint32_t keep = (e & 1u) ? 0x0000FFFFu : 0xFFFF0000u;
    const uint32_t put = (e & 1u) ? pat << 16 : pat;
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = (mine && (e >> 1) == (uint32_t)k) ? ((w[k] & keep) | put) : w[k];
  }
}

// a9 for one row: unpack, dequantise, [patch a few outliers in,] store
template <int BITS, bool ASYM, bool F32, bool PATCH = false>
__device__ __forceinline__ void store_row_values(const TensorDesc& d, uint64_t e0, const RowCodes<BITS>& r, uint32_t mail = 0u) {
  int c[kOct];
  if constexpr (BITS == 8) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      c[e] = (int)(int8_t)((r.w[0] >> (8 * e)) & 0xFFu);
      c[4 + e] = (int)(int8_t)((r.w[1] >> (8 * e)) & 0xFFu);
    }
  } else {
#pragma unroll
    for (int e = 0; e < kOct; ++e) c[e] = ((int)(r.w[0] << (28 - 4 * e))) >> 28;  // sign-extended nibble
  }
  float v[kOct];
#pragma unroll
  for (int e = 0; e < kOct; ++e) v[e] = ASYM ? __fmaf_rn((float)c[e], r.s, r.o) : (float)c[e] * r.s;
  if constexpr (F32) {
    uint32_t w[8];
#pragma unroll
    for (int e = 0; e < kOct; ++e) w[e] = __float_as_uint(v[e]);
    if constexpr (PATCH) patch_row_words<8>(w, mail);
    float* p = reinterpret_cast<float*>(d.dst) + e0;
    ADACC_STORE16(p, make_uint4(w[0], w[1], w[2], w[3]));
    ADACC_STORE16(p + 4, make_uint4(w[4], w[5], w[6], w[7]));
  } else {
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = narrow_pair(v[2 * k], v[2 * k + 1]);
    if constexpr (PATCH) patch_row_words<4>(w, mail);
    ADACC_STORE16(reinterpret_cast<uint16_t*>(d.dst) + e0, make_uint4(w[0], w[1], w[2], w[3]));
  }
}

// What the kernels that call decompress_tile keep in LDS: a mailbox of one word per octet of a piece for
// every wavefront of the workgroup.
struct DecompressShared {
  uint32_t mailbox[kWavesPerWg][kWave][4];
};

template <int BITS, bool ASYM, int E, bool F32>
__device__ __forceinline__ void decompress_tile(const TensorDesc& d, uint32_t tile /* piece */, bool has_outliers,
                                                DecompressShared& shared) {
  static_assert(E == 4, "pieces of 2048 elements");
  const int lane = (int)__lane_id();
  const uint64_t tile_base = (uint64_t)tile * (uint64_t)(E * kRow);
  const uint64_t lane_base = tile_base + (uint64_t)lane * kOct;
  const bool complete = tile_base + (uint64_t)(E * kRow) <= d.numel;  // uniform; only a tensor's last piece can be short

  // All loads of the piece are issued before anything waits for one of them: a complete piece
  // (every piece but possibly the last) has no branch between them.
  RowCodes<BITS> rc[E];
  if (complete) {
#pragma unroll
    for (int j = 0; j < E; ++j) load_row_codes<BITS, ASYM>(d, lane_base + (uint64_t)j * kRow, rc[j]);
  } else {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint64_t e0 = lane_base + (uint64_t)j * kRow;
      if (e0 < d.numel) load_row_codes<BITS, ASYM>(d, e0, rc[j]);
    }
  }

  // This tile's slice of the outlier stream and its first 64 entries.  The entries can only be asked for when
  // the slice is known, a second round trip to memory behind the first - except for TOPK, where the slice of
  // tile T is [T * k * groups per tile, + k * groups per tile) unless some group held more than k values that
  // are not finite: there the entries of that slice are asked for at once, together with the tile's offsets,
  // and are used if the offsets turn out to be those.
  const bool guess = has_outliers && d.mode == kModeTopk;  // uniform
  uint32_t g0 = 0u, g1 = 0u, o_idx = 0u, o_val = 0u;
  if (guess) {
    const uint32_t per_tile = d.topk << (d.lgt - d.lgs);
    g0 = per_tile * (tile >> d.ptr_shift);
    g1 = g0 + per_tile;
    g0 = g0 < d.cap ? g0 : d.cap;
    g1 = g1 < d.cap ? g1 : d.cap;
    if (g0 + (uint32_t)lane < g1) {
      o_idx = (uint32_t)d.idx[g0 + (uint32_t)lane];
      o_val = d.val[g0 + (uint32_t)lane];
    }
  }
  uint32_t p0 = 0u, p1 = 0u;
  if (has_outliers) {
    p0 = d.tile_ptr[tile >> d.ptr_shift];
    p1 = d.tile_ptr[(tile >> d.ptr_shift) + 1];
    p0 = p0 < d.cap ? p0 : d.cap;
    p1 = p1 < d.cap ? p1 : d.cap;
    if (p1 < p0) p1 = p0;
  }
  const bool patch = p1 > p0;  // uniform over the wavefront
  if (patch && !(guess && p0 == g0 && p1 == g1)) {  // uniform
    o_idx = 0u; o_val = 0u;
    if (p0 + (uint32_t)lane < p1) {
      o_idx = (uint32_t)d.idx[p0 + (uint32_t)lane];
      o_val = d.val[p0 + (uint32_t)lane];
    }
  }

  // ---- a9: unpack, dequantise, store.  A complete piece whose tile has at most 64 outliers (TOPK tensors:
  // every piece), no two in one octet, takes them in on the way, in registers: nothing is written twice and
  // nothing waits for a store.  The stream is ascending, so two entries of one octet are neighbours in it.
  if (complete && patch && p1 - p0 <= (uint32_t)kWave) {
    const uint32_t rel = o_idx - (uint32_t)tile_base;  // a tensor that keeps outliers has fewer than 2^31 elements
    const bool valid = (uint32_t)lane < p1 - p0 && rel < (uint32_t)(E * kRow);  // also: not in a 4096-element tile's other half
    const uint32_t oct = rel >> 3;
    const uint32_t prev_oct = (uint32_t)__shfl_up((int)oct, 1, kWave);
    if (__builtin_amdgcn_ballot_w64(valid && lane != 0 && oct == prev_oct) == 0ull) {  // uniform
      uint32_t(*box)[E] = shared.mailbox[threadIdx.x / kWave];
      *reinterpret_cast<uint4*>(box[lane]) = make_uint4(0u, 0u, 0u, 0u);
      __builtin_amdgcn_wave_barrier();  // LDS takes a wavefront's accesses in order: nothing may be moved across
      if (valid) box[oct & 63u][oct >> 6] = kMailFull | ((rel & 7u) << 16) | (o_val & 0xFFFFu);
      __builtin_amdgcn_wave_barrier();
      const uint4 mail = *reinterpret_cast<const uint4*>(box[lane]);
      __builtin_amdgcn_wave_barrier();  // the next piece of this wavefront clears the mailbox only after this
      const uint32_t m[E] = {mail.x, mail.y, mail.z, mail.w};
#pragma unroll
      for (int j = 0; j < E; ++j)
        store_row_values<BITS, ASYM, F32, true>(d, lane_base + (uint64_t)j * kRow, rc[j], m[j]);
      return;
    }
  }
  if (complete) {
#pragma unroll
    for (int j = 0; j < E; ++j) store_row_values<BITS, ASYM, F32>(d, lane_base + (uint64_t)j * kRow, rc[j]);
  } else {
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint64_t e0 = lane_base + (uint64_t)j * kRow;
      if (e0 < d.numel) store_row_values<BITS, ASYM, F32>(d, e0, rc[j]);
    }
  }

  // ---- a10: the outliers overwrite their positions
  if (patch) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the stores above are complete
    const uint64_t piece_end = complete ? tile_base + (uint64_t)(E * kRow) : d.numel;
    for (uint32_t cpos = p0 + (uint32_t)lane; cpos < p1; cpos += kWave) {
      if (cpos >= p0 + (uint32_t)kWave) {  // past the entries fetched at the start
        o_idx = (uint32_t)d.idx[cpos];
        o_val = d.val[cpos];
      }
      const uint64_t i = o_idx;
      if (i >= tile_base && i < piece_end) {  // a damaged stream must not write outside the piece
        if constexpr (F32) reinterpret_cast<float*>(d.dst)[i] = widen_lo(o_val);
        else reinterpret_cast<uint16_t*>(d.dst)[i] = (uint16_t)o_val;
      }
    }
  }
}

}  // namespace ADACC_DT_NS
}  // namespace adacc
