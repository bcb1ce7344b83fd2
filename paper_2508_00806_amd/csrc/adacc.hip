// libadacc: kernels and C ABI (see include/adacc.h).  gfx950 only.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <algorithm>
#include <mutex>
#include <vector>

#include "adacc.h"
#include "adacc_common.hpp"
#include "adacc_fn.hpp"

namespace adacc {

// ===================================================================== kernels

// ---- utilities
// The table of a batch reaches the device as kernel arguments, a slice per launch: the runtime
// copies kernel arguments when the launch is enqueued, so the host buffer may go away at once
// and the host never waits for the stream (a copy from pageable memory would).
constexpr uint32_t kDescsPerUpload = 3968 / sizeof(TensorDesc);
struct DescSlice { TensorDesc d[kDescsPerUpload]; };
static_assert(sizeof(DescSlice) <= 3968, "kernel arguments are limited to 4 KiB");
static_assert(sizeof(TensorDesc) % 4 == 0, "copied as 32-bit words");
__global__ __launch_bounds__(kThreads) void table_upload_kernel(DescSlice slice, TensorDesc* dst, uint32_t count) {
  const uint32_t words = count * (uint32_t)(sizeof(TensorDesc) / 4);
  const uint32_t* src = reinterpret_cast<const uint32_t*>(&slice);
  uint32_t* out = reinterpret_cast<uint32_t*>(dst);
  for (uint32_t i = threadIdx.x; i < words; i += kThreads) out[i] = src[i];
}

// clears a workspace (a kernel rather than a memset node, so that callers may capture it in a graph)
__global__ __launch_bounds__(kThreads) void workspace_clear_kernel(uint4* p, uint64_t n16) {
  const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
    p[i] = make_uint4(0, 0, 0, 0);
}

// small arrays of 32-bit words (the first-tile / first-block arrays of a batch) travel the same way
constexpr uint32_t kWordsPerUpload = 960;
struct WordSlice { uint32_t w[kWordsPerUpload]; };
__global__ __launch_bounds__(kThreads) void words_upload_kernel(WordSlice slice, uint32_t* dst, uint32_t count) {
  for (uint32_t i = threadIdx.x; i < count; i += kThreads) dst[i] = slice.w[i];
}

// Streams of known size in the shape the tensor kernels use (one piece of 4 KiB per wavefront per
// operand, full grid in the hardware's order, non-temporal accesses): what a kernel that only moves
// bytes reaches on this part for a given mix of reads and writes.
//   MIX 0: read a          1: write dst          2: dst = a (copy)          3: dst = a ^ b (two reads, one write)
template <int MIX>
__global__ __launch_bounds__(kThreads) void hbm_stream_kernel(uint4* __restrict__ dst, const uint4* __restrict__ a,
                                                              const uint4* __restrict__ b, uint64_t n16,
                                                              uint32_t* sink) {
  const uint64_t piece = ((uint64_t)blockIdx.x * kWavesPerWg + threadIdx.x / kWave) * 256u + (threadIdx.x % kWave);
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  uint4 v[4], w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint64_t i = piece + (uint64_t)j * 64u;
    const uint64_t ic = i < n16 ? i : n16 - 1u;
    if constexpr (MIX != 1) v[j] = load_stream16(a + ic);
    if constexpr (MIX == 3) w[j] = load_stream16(b + ic);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint64_t i = piece + (uint64_t)j * 64u;
    if constexpr (MIX == 0) { acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w; }
    if constexpr (MIX == 1) { if (i < n16) store_stream16(dst + i, make_uint4((uint32_t)i, 1u, 2u, 3u)); }
    if constexpr (MIX == 2) { if (i < n16) store_stream16(dst + i, v[j]); }
    if constexpr (MIX == 3) { if (i < n16) store_stream16(dst + i, make_uint4(v[j].x ^ w[j].x, v[j].y ^ w[j].y, v[j].z ^ w[j].z, v[j].w ^ w[j].w)); }
  }
  if constexpr (MIX == 0) {
    // keeps the loads alive; practically never true, so nothing is written
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && sink) *sink = acc.x;
  }
}

// ===================================================================== host side

static thread_local char g_hip_err[256] = "no HIP error recorded";

static int hip_fail(hipError_t e, const char* what) {
  std::snprintf(g_hip_err, sizeof g_hip_err, "%s: %s", what, hipGetErrorString(e));
  return ADACC_EHIP;
}

static int env_int(const char* name, int dflt) {
  const char* s = std::getenv(name);
  if (!s || !*s) return dflt;
  const long v = std::strtol(s, nullptr, 10);
  return v > 0 ? (int)v : dflt;
}

// Run-time knobs for measurements, read from the environment once per process.
struct Knobs {
  int grid_rounds;      // ADACC_GRID_ROUNDS: limit grids of independent tiles to this many rounds of resident workgroups
  int wgs_per_cu;       // ADACC_WGS_PER_CU: overrides the occupancy query behind that limit
  int mask_wgs_per_cu;  // ADACC_MASK_WGS_PER_CU: grid of the mask kernels
};
static const Knobs& knobs() {
  static const Knobs k = {env_int("ADACC_GRID_ROUNDS", 0), env_int("ADACC_WGS_PER_CU", 0),
                          env_int("ADACC_MASK_WGS_PER_CU", 128)};
  return k;
}

static int device_cus(int* cus) {
  static int cached[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev >= 0 && dev < 64 && cached[dev] > 0) { *cus = cached[dev]; return ADACC_OK; }
  int n = 0;
  e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return hip_fail(e, "hipDeviceGetAttribute");
  if (dev >= 0 && dev < 64) cached[dev] = n;
  *cus = n;
  return ADACC_OK;
}

static bool is_pow2(uint64_t v) { return v && !(v & (v - 1)); }
static uint32_t ilog2(uint64_t v) { uint32_t l = 0; while ((1ull << l) < v) ++l; return l; }
static uint64_t align256(uint64_t v) { return (v + 255ull) & ~255ull; }

struct Plan {  // everything derived from (method, numel)
  bool noop;
  bool outliers;
  uint32_t tile_elems, lgq, lgs, variant;
  uint64_t numel_main;   // the whole groups of the larger kind: what the tile kernels take
  uint32_t tail;         // elements after those, done by the tail kernels
  uint32_t n_tiles;      // tiles of the main part
  uint32_t n_tiles_all;  // tiles of the whole tensor (what the layout reports)
  bool rowwise;  // every group lies inside a 512-element row and both kinds of group coincide
  bool half;     // the tensor is binary16 (else bf16)
  bool generic;  // group sizes the tile kernels do not take: the fallback kernels do the whole tensor
  float param, divisor;
};

constexpr uint32_t kGenericMaxGroup = 16384;  // the longest segment of the fallback kernels

static int make_plan(const adacc_method* m, uint64_t numel, Plan* p) {
  std::memset(p, 0, sizeof *p);
  if (m->kind == ADACC_KIND_NOOP) { p->noop = true; return ADACC_OK; }
  if (m->kind != ADACC_KIND_QUANT) return ADACC_EINVAL;
  if (m->bits != 4 && m->bits != 8) return ADACC_EINVAL;
  if (m->asym > 1 || m->scale_rule > 1 || m->outlier_mode > ADACC_OUTLIER_TOPK) return ADACC_EINVAL;
  if (m->dtype > ADACC_DTYPE_F16) return ADACC_EINVAL;
  p->half = m->dtype == ADACC_DTYPE_F16;
  if (m->quant_group < 8 || m->quant_group % 8 != 0 || m->quant_group > kGenericMaxGroup) return ADACC_EINVAL;
  uint32_t gs = m->quant_group;
  const bool stat = m->outlier_mode == ADACC_OUTLIER_STD || m->outlier_mode == ADACC_OUTLIER_TOPK;
  if (stat) {
    if (m->stat_group < m->quant_group || m->stat_group % m->quant_group != 0 || m->stat_group > kGenericMaxGroup)
      return ADACC_EINVAL;
    gs = m->stat_group;
  }
  // the tile kernels take powers of two up to 4096; everything else goes through the fallback kernels
  p->generic = !is_pow2(m->quant_group) || !is_pow2(gs) || gs > 4096;
  if (m->outlier_mode == ADACC_OUTLIER_TOPK && (m->topk < 1 || m->topk > 32 || m->topk > gs)) return ADACC_EINVAL;
  if (m->outlier_mode == ADACC_OUTLIER_ABS || m->outlier_mode == ADACC_OUTLIER_STD) {
    if (!(m->thresh >= 0.0f) || std::isinf(m->thresh)) return ADACC_EINVAL;
  }
  p->outliers = m->outlier_mode != ADACC_OUTLIER_NONE;
  if (p->outliers && numel >= (1ull << 31)) return ADACC_EINVAL;  // 32-bit signed flat indices
  if (numel >= (1ull << 42)) return ADACC_EINVAL;
  if (p->generic) {
    // a segment: as many whole groups of the larger kind as fit 4096 elements (one, if it is larger);
    // the last segment and its last groups may be short, so there is no tail
    p->tile_elems = gs >= 4096 ? gs : gs * (4096u / gs);
    p->numel_main = numel;
    p->tail = 0;
    const uint64_t segs = (numel + p->tile_elems - 1) / p->tile_elems;
    if (segs >= (1ull << 31)) return ADACC_EINVAL;
    p->n_tiles = p->n_tiles_all = (uint32_t)segs;
  } else {
    p->tile_elems = gs > 2048 ? 4096u : 2048u;
    p->numel_main = numel - numel % gs;
    p->tail = (uint32_t)(numel % gs);
    p->n_tiles = (uint32_t)((p->numel_main + p->tile_elems - 1) / p->tile_elems);
    p->n_tiles_all = (uint32_t)((numel + p->tile_elems - 1) / p->tile_elems);
    p->lgq = ilog2(m->quant_group);
    p->lgs = ilog2(gs);
  }
  p->variant = variant_index(m->outlier_mode, m->bits, m->asym, p->tile_elems == 4096 ? 1u : 0u);
  p->rowwise = !p->generic && m->outlier_mode != ADACC_OUTLIER_TOPK && m->quant_group <= 512 &&
               (m->outlier_mode != ADACC_OUTLIER_STD || m->stat_group == m->quant_group);
  const float q = (float)(1u << (m->bits - 1));
  if (m->asym) p->divisor = m->scale_rule == ADACC_SCALE_PAPER ? 2.0f * q : 2.0f * q - 1.0f;
  else p->divisor = m->scale_rule == ADACC_SCALE_PAPER ? q : q - 1.0f;
  if (m->outlier_mode == ADACC_OUTLIER_ABS) p->param = m->thresh;
  if (m->outlier_mode == ADACC_OUTLIER_STD) p->param = m->thresh * m->thresh;
  return ADACC_OK;
}

static void fill_layout(const adacc_method* m, uint64_t numel, const Plan& p, adacc_layout* L) {
  std::memset(L, 0, sizeof *L);
  if (p.noop) return;
  const uint64_t groups = (numel + m->quant_group - 1) / m->quant_group;  // the last one may be short
  uint64_t off = 0;
  L->codes_off = off;   off = align256(off + (numel * m->bits + 7) / 8);
  L->scales_off = off;  off = align256(off + 4 * groups);
  L->zp_off = off;      off = align256(off + (m->asym ? 4 * groups : 0));
  L->tile_ptr_off = off; off = align256(off + (p.outliers ? 4ull * ((uint64_t)p.n_tiles_all + 1) : 0));
  L->idx_off = off;     off = align256(off + (p.outliers ? 4ull * m->max_outliers : 0));
  L->val_off = off;     off = align256(off + (p.outliers ? 2ull * m->max_outliers : 0));
  L->status_off = off;  off = align256(off + 16);
  L->total_bytes = off;
  L->tile_elems = p.tile_elems;
  L->n_tiles = p.n_tiles_all;
}

// Workgroups of `kernel` that one CU holds at once (cached per kernel: the query is not free).
static int resident_wgs(const void* kernel, int* wgs_out) {
  struct Entry { const void* kernel; int wgs; };
  static thread_local Entry cache[64];
  static thread_local int used = 0;
  for (int i = 0; i < used; ++i)
    if (cache[i].kernel == kernel) { *wgs_out = cache[i].wgs; return ADACC_OK; }
  int wgs = 0;
  const hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&wgs, kernel, kThreads, 0);
  if (e != hipSuccess) return hip_fail(e, "hipOccupancyMaxActiveBlocksPerMultiprocessor");
  if (wgs < 1) wgs = 1;
  if (used < 64) cache[used++] = Entry{kernel, wgs};
  *wgs_out = wgs;
  return ADACC_OK;
}

// Wavefronts of `kernel` that the device can hold at once.
static int wave_capacity(const void* kernel, int cus, uint32_t* waves) {
  int wgs = 0;
  const int rc = resident_wgs(kernel, &wgs);
  if (rc != ADACC_OK) return rc;
  if (knobs().wgs_per_cu > 0) wgs = knobs().wgs_per_cu;
  *waves = (uint32_t)(cus * wgs * kWavesPerWg);
  return ADACC_OK;
}

// TOPK whose statistics group is the tile, with every quantisation group inside a 512-element row, has kernels of its own
static bool topk_whole_tile(const adacc_method* m, const Plan& p) {
  return m->outlier_mode == ADACC_OUTLIER_TOPK && m->stat_group == p.tile_elems && m->quant_group <= 512;
}
// TOPK over groups that are the quantisation groups and lie inside a 512-element row: the row-at-a-time encoder
static bool topk_in_rows(const adacc_method* m, const Plan& p) {
  return !p.generic && m->outlier_mode == ADACC_OUTLIER_TOPK && m->stat_group == m->quant_group && m->quant_group <= 512;
}
static int batch_kind(const adacc_method* m, const Plan& p) {
  const bool whole = topk_whole_tile(m, p);
  if (p.tile_elems == 4096) return whole ? kBatchTopk8 : kBatchAny8;
  return (p.rowwise || topk_in_rows(m, p)) ? kBatchRows4 : (whole ? kBatchTopk4 : kBatchAny4);
}

static uint32_t decompress_pieces(uint64_t numel) { return (uint32_t)((numel + 2047ull) / 2048ull); }

// Workspace of one tensor that keeps outliers: [cnt: one word per tile][flag][block_sum][slots],
// block sums and slots for ABS / STD only.  Offsets relative to the tensor's region.
struct WsPlan { uint64_t cnt_off, flag_off, block_sum_off, slot_off, bytes; };
static uint32_t place_blocks(const Plan& p) { return p.outliers ? (p.n_tiles + kPlaceTiles - 1) / kPlaceTiles : 0u; }
static WsPlan ws_plan(const adacc_method* m, const Plan& p) {
  WsPlan w;
  std::memset(&w, 0, sizeof w);
  if (p.noop || !p.outliers) return w;
  uint64_t off = 0;
  w.cnt_off = off;  off = align256(off + 4ull * p.n_tiles);
  w.flag_off = off; off += 256;
  if (m->outlier_mode != ADACC_OUTLIER_TOPK) {
    w.block_sum_off = off; off = align256(off + 4ull * place_blocks(p));
    w.slot_off = off; off = align256(off + 8ull * kSlot * p.n_tiles);
  }
  w.bytes = off;
  return w;
}
// does the placement of this tensor start from per-block sums (a kernel of its own computes them)?
static bool needs_block_sums(const adacc_method* m, const Plan& p) {
  return p.outliers && m->outlier_mode != ADACC_OUTLIER_TOPK && place_blocks(p) > kPlaceDirectBlocks;
}

static void fill_desc(const adacc_method* m, uint64_t numel, const Plan& p, const adacc_layout& L, const void* src,
                      void* blob, void* dst, int dst_dtype, void* ws_region, TensorDesc* d) {
  std::memset(d, 0, sizeof *d);
  unsigned char* b = static_cast<unsigned char*>(blob);
  d->src = static_cast<const uint16_t*>(src);
  d->dst = dst;
  d->codes = b + L.codes_off;
  d->scales = reinterpret_cast<float*>(b + L.scales_off);
  d->zp = reinterpret_cast<float*>(b + L.zp_off);
  d->tile_ptr = reinterpret_cast<uint32_t*>(b + L.tile_ptr_off);
  d->idx = reinterpret_cast<int32_t*>(b + L.idx_off);
  d->val = reinterpret_cast<uint16_t*>(b + L.val_off);
  d->status = reinterpret_cast<uint32_t*>(b + L.status_off);
  if (ws_region && p.outliers) {
    const WsPlan w = ws_plan(m, p);
    unsigned char* r = static_cast<unsigned char*>(ws_region);
    d->cnt = reinterpret_cast<uint32_t*>(r + w.cnt_off);
    d->flag = reinterpret_cast<uint32_t*>(r + w.flag_off);
    d->block_sum = reinterpret_cast<uint32_t*>(r + w.block_sum_off);
    d->slot = reinterpret_cast<uint2*>(r + w.slot_off);
  }
  (void)numel;
  d->numel = p.numel_main;
  d->tail = p.tail;
  d->n_tiles = p.n_tiles;
  d->n_tiles_all = p.n_tiles_all;
  d->bits = m->bits;
  d->asym = m->asym;
  d->mode = m->outlier_mode;
  d->gq = m->quant_group;
  d->gs = (m->outlier_mode == ADACC_OUTLIER_STD || m->outlier_mode == ADACC_OUTLIER_TOPK) ? m->stat_group : m->quant_group;
  d->tile_elems = p.tile_elems;
  d->generic = p.generic ? 1u : 0u;
  d->n_blocks = place_blocks(p);
  d->lgt = p.tile_elems == 4096 ? 12u : 11u;
  if (dst && !p.generic) {  // decompression counts pieces of 2048 elements
    d->n_tiles = decompress_pieces(p.numel_main);
    d->ptr_shift = p.tile_elems == 4096 ? 1u : 0u;
  }
  d->lgq = p.lgq;
  d->lgs = p.lgs;
  d->cap = m->max_outliers;
  d->topk = m->topk;
  d->param = p.param;
  d->divisor = p.divisor;
  {
    int ex = 0;
    d->inv_divisor = (std::frexp(p.divisor, &ex) == 0.5f) ? 1.0f / p.divisor : 0.0f;  // exact for a power of two
    d->pow2_divisor = d->inv_divisor != 0.0f ? 1u : 0u;
  }
  d->variant = p.variant;
  d->rowwise = p.rowwise ? 1u : 0u;
  d->dst_f32 = dst_dtype == ADACC_DST_F32 ? 1u : 0u;
}

static bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// Grid for kernels whose tiles are independent (grid-stride loop).  By default one workgroup per
// four tiles, i.e. every wavefront takes one tile: with streaming accesses the hardware's own
// order of workgroups, which walks through memory front to back, beat every grid of resident
// workgroups that loop (C4 decompression: 0.308 ms with one round of resident workgroups, 0.275 ms
// like this).  ADACC_GRID_ROUNDS=r limits the grid to r times the workgroups the device holds at
// once, for comparison.
// `resident_rounds` > 0: the kernel has a set-up cost per workgroup (the outlier-channel kernels stage
// tables in LDS), so its grid is limited to that many times the resident workgroups.
static int grid_for(uint32_t n_tiles, const void* kernel, uint32_t* grid, int resident_rounds = 0) {
  const uint64_t want = ((uint64_t)n_tiles + kWavesPerWg - 1) / kWavesPerWg;
  uint64_t cap = want;
  const int rounds = knobs().grid_rounds > 0 ? knobs().grid_rounds : resident_rounds;
  if (rounds > 0) {
    int cus = 0;
    int rc = device_cus(&cus);
    if (rc != ADACC_OK) return rc;
    uint32_t waves = 0;
    rc = wave_capacity(kernel, cus, &waves);
    if (rc != ADACC_OK) return rc;
    cap = (uint64_t)(waves / kWavesPerWg) * (uint64_t)rounds;
  }
  *grid = (uint32_t)(want < cap ? want : cap);
  if (*grid == 0) *grid = 1;
  return ADACC_OK;
}

static BatchCompressFn compress_batch_fn(bool half, int kind) {
  return kind >= kBatchAny8 ? ADACC_PICK(half, compress_batch_fn8(kind)) : ADACC_PICK(half, compress_batch_fn4(kind));
}

// `whole` (TOPK only): the statistics group is the whole tile; that case has kernels of its own.
// `rowwise`: for TOPK, statistics group = quantisation group inside a row (topk_in_rows)
static CompressFn compress_fn(const adacc_method* m, bool e8, bool rowwise, bool whole) {
  const bool half = m->dtype == ADACC_DTYPE_F16;
  switch (m->outlier_mode) {
    case ADACC_OUTLIER_NONE: return ADACC_PICK(half, compress_fn_none(m->bits, m->asym, e8, rowwise));
    case ADACC_OUTLIER_ABS: return ADACC_PICK(half, compress_fn_abs(m->bits, m->asym, e8, rowwise));
    case ADACC_OUTLIER_STD: return ADACC_PICK(half, compress_fn_std(m->bits, m->asym, e8, rowwise));
    default: return ADACC_PICK(half, compress_fn_topk(m->bits, m->asym, e8, whole, rowwise));
  }
}

static int clear_device(void* mem, uint64_t bytes, hipStream_t s);

// Next epoch of a workspace; clears the buffer first when the counter is about to wrap.
static int next_epoch(adacc_workspace* ws, hipStream_t s, uint32_t* epoch) {
  if (ws->epoch >= kEpochMax) {
    const int rc = clear_device(ws->device_mem, ws->bytes, s);
    if (rc != ADACC_OK) return rc;
    ws->epoch = 0;
  }
  ws->epoch += 1;
  *epoch = ws->epoch;
  return ADACC_OK;
}

static int launch_check(const char* what) {
  const hipError_t e = hipGetLastError();
  return e == hipSuccess ? ADACC_OK : hip_fail(e, what);
}

static int upload_table(const std::vector<TensorDesc>& table, TensorDesc* dst, hipStream_t s) {
  for (size_t i = 0; i < table.size(); i += kDescsPerUpload) {
    DescSlice slice;
    const uint32_t count = (uint32_t)std::min<size_t>(kDescsPerUpload, table.size() - i);
    std::memset(&slice, 0, sizeof slice);
    std::memcpy(slice.d, table.data() + i, count * sizeof(TensorDesc));
    hipLaunchKernelGGL(table_upload_kernel, dim3(1), dim3(kThreads), 0, s, slice, dst + i, count);
    const int rc = launch_check("table_upload_kernel");
    if (rc != ADACC_OK) return rc;
  }
  return ADACC_OK;
}

static int upload_words(const std::vector<uint32_t>& words, uint32_t* dst, hipStream_t s) {
  for (size_t i = 0; i < words.size(); i += kWordsPerUpload) {
    WordSlice slice;
    const uint32_t count = (uint32_t)std::min<size_t>(kWordsPerUpload, words.size() - i);
    std::memcpy(slice.w, words.data() + i, count * sizeof(uint32_t));
    hipLaunchKernelGGL(words_upload_kernel, dim3(1), dim3(kThreads), 0, s, slice, dst + i, count);
    const int rc = launch_check("words_upload_kernel");
    if (rc != ADACC_OK) return rc;
  }
  return ADACC_OK;
}

static int clear_device(void* mem, uint64_t bytes, hipStream_t s) {
  const uint64_t n16 = bytes / 16;
  uint32_t grid = (uint32_t)((n16 + kThreads - 1) / kThreads);
  if (grid > 4096) grid = 4096;
  if (grid == 0) return ADACC_OK;
  hipLaunchKernelGGL(workspace_clear_kernel, dim3(grid), dim3(kThreads), 0, s, static_cast<uint4*>(mem), n16);
  return launch_check("workspace_clear_kernel");
}

// batch workspace: [table: n descriptors][member lists of the launches: 4 n words][the tensors' regions]
struct BatchPlan {
  uint64_t members_off, regions_off, bytes;
};
static BatchPlan batch_plan(uint32_t n_active, uint64_t region_bytes) {
  BatchPlan b;
  const uint64_t n = n_active ? n_active : 1;
  b.members_off = align256(n * sizeof(TensorDesc));
  b.regions_off = b.members_off + align256(4ull * 4ull * n);
  b.bytes = b.regions_off + region_bytes;
  return b;
}

// A launch over a group of table entries: grid.y = the group's entries, grid.x covers the largest.
struct GroupLaunch {
  uint32_t first_member, n_members, max_units;
  int kind;  // what the caller makes of it (register class, kernel)
};
// Groups the entries for which units[i] > 0 by kind[i] and by size (unit counts within a factor of
// two of each other, at most 65535 entries per launch) and appends their member lists to `members`.
static void group_launches(const std::vector<uint32_t>& units, const std::vector<int>& kind,
                           std::vector<uint32_t>* members, std::vector<GroupLaunch>* launches) {
  for (int k = 0; k < 2 * kBatchKinds; ++k) {  // kinds of the second half: the same for binary16 tensors
    for (uint32_t bucket = 0; bucket <= 32; ++bucket) {
      GroupLaunch g = {(uint32_t)members->size(), 0u, 0u, k};
      for (uint32_t i = 0; i < units.size(); ++i) {
        if (units[i] == 0 || kind[i] != k || ilog2(units[i]) != bucket) continue;
        if (g.n_members == 65535u) {
          launches->push_back(g);
          g = GroupLaunch{(uint32_t)members->size(), 0u, 0u, k};
        }
        members->push_back(i);
        g.n_members += 1;
        g.max_units = std::max(g.max_units, units[i]);
      }
      if (g.n_members) launches->push_back(g);
    }
  }
}

// one wavefront per strip of 512 channels and `rows` tokens, four wavefronts per workgroup
static uint32_t strip_grid(uint64_t tokens, uint32_t hidden, uint32_t rows) {
  const uint64_t units = ((tokens + rows - 1) / rows) * ((hidden + 511u) / 512u);
  return (uint32_t)((units + kWavesPerWg - 1) / kWavesPerWg);  // tokens * hidden < 2^32: far below 2^31
}

// ---- outlier channels (Section 3.2, Eq. 1)
struct ChannelPlan {
  adacc_method quant;  // the quantisation of the rest: the same method without outliers
  Plan plan;
  adacc_layout quant_layout;
  uint64_t numel;
  uint32_t n_chunks;
};

static int make_channel_plan(const adacc_channel_method* m, uint64_t tokens, uint32_t hidden, ChannelPlan* cp) {
  std::memset(cp, 0, sizeof *cp);
  if (hidden < 8 || hidden > 65536 || hidden % 8 != 0) return ADACC_EINVAL;
  if (tokens > 0xFFFFFFFFull / hidden) return ADACC_EINVAL;  // tokens * hidden < 2^32
  if (m->quant_group > 2048) return ADACC_EINVAL;
  if (m->max_channels < 1 || m->max_channels > hidden) return ADACC_EINVAL;
  if (!std::isfinite(m->z_thresh)) return ADACC_EINVAL;
  cp->quant.kind = ADACC_KIND_QUANT;
  cp->quant.bits = m->bits;
  cp->quant.quant_group = m->quant_group;
  cp->quant.asym = m->asym;
  cp->quant.scale_rule = m->scale_rule;
  cp->quant.outlier_mode = ADACC_OUTLIER_NONE;
  cp->quant.dtype = m->dtype;
  cp->numel = tokens * hidden;
  const int rc = make_plan(&cp->quant, cp->numel, &cp->plan);
  if (rc != ADACC_OK) return rc;
  if (cp->plan.tail != 0 || cp->plan.generic) return ADACC_EINVAL;  // here: a power of two that divides the tensor
  fill_layout(&cp->quant, cp->numel, cp->plan, &cp->quant_layout);
  cp->n_chunks = (uint32_t)((tokens + kChunkTokens - 1) / kChunkTokens);
  return ADACC_OK;
}

static void fill_channel_layout(const adacc_channel_method* m, uint64_t tokens, uint32_t hidden, const ChannelPlan& cp,
                                adacc_channel_layout* L) {
  std::memset(L, 0, sizeof *L);
  L->codes_off = cp.quant_layout.codes_off;
  L->scales_off = cp.quant_layout.scales_off;
  L->zp_off = cp.quant_layout.zp_off;
  uint64_t off = cp.quant_layout.status_off;  // the sections of this mode start where the plain blob's status would be
  L->ch_mask_off = off;  off = align256(off + hidden / 8);
  L->ch_base_off = off;  off = align256(off + 4ull * (hidden / 8));
  L->ch_idx_off = off;   off = align256(off + 4ull * m->max_channels);
  L->ch_val_off = off;   off = align256(off + 2ull * tokens * m->max_channels);
  L->status_off = off;   off = align256(off + 16);
  L->total_bytes = off;
}

static uint32_t channel_mask_lds(uint32_t hidden) { return (3u * (hidden / 8) + 15u) & ~15u; }  // LDS copy of mask and ranks

static uint64_t channel_partial_bytes(uint32_t n_chunks, uint32_t hidden) { return align256(4ull * n_chunks * hidden); }

static void fill_channel_desc(const adacc_channel_method* m, uint64_t tokens, uint32_t hidden,
                              const adacc_channel_layout& L, void* blob, ChannelDesc* c) {
  unsigned char* b = static_cast<unsigned char*>(blob);
  c->mask = b + L.ch_mask_off;
  c->base = reinterpret_cast<uint32_t*>(b + L.ch_base_off);
  c->ch_idx = reinterpret_cast<int32_t*>(b + L.ch_idx_off);
  c->ch_val = reinterpret_cast<uint16_t*>(b + L.ch_val_off);
  c->status = reinterpret_cast<uint32_t*>(b + L.status_off);
  c->hidden = hidden;
  c->tokens = (uint32_t)tokens;
  c->max_channels = m->max_channels;
  c->z_thresh = m->z_thresh;
  c->inv_hidden = std::nextafter(std::nextafter(1.0f / (float)hidden, 0.0f), 0.0f);
}

}  // namespace adacc

using namespace adacc;

// ===================================================================== C ABI

extern "C" {

const char* adacc_version(void) { return "0.1"; }

const char* adacc_strerror(int code) {
  switch (code) {
    case ADACC_OK: return "ok";
    case ADACC_EINVAL: return "invalid method or size";
    case ADACC_ENULL: return "null pointer";
    case ADACC_ESIZE: return "blob or workspace too small";
    case ADACC_EALIGN: return "device pointer not aligned";
    case ADACC_EHIP: return g_hip_err;
    case ADACC_ELIMIT: return "size beyond the limit of this entry point";
    default: return "unknown error code";
  }
}

int adacc_layout_of(const adacc_method* method, uint64_t numel, adacc_layout* out) {
  if (!method || !out) return ADACC_ENULL;
  Plan p;
  const int rc = make_plan(method, numel, &p);
  if (rc != ADACC_OK) return rc;
  fill_layout(method, numel, p, out);
  return ADACC_OK;
}

uint64_t adacc_workspace_bytes(const adacc_method* method, uint64_t numel) {
  if (!method) return 0;
  Plan p;
  if (make_plan(method, numel, &p) != ADACC_OK) return 0;
  return ws_plan(method, p).bytes;
}

int adacc_workspace_init(adacc_workspace* ws, void* device_mem, uint64_t bytes, void* hip_stream) {
  if (!ws || !device_mem) return ADACC_ENULL;
  if (bytes < 256 || bytes % 16 != 0) return ADACC_ESIZE;
  if (misaligned(device_mem, 256)) return ADACC_EALIGN;
  const int rc = clear_device(device_mem, bytes, static_cast<hipStream_t>(hip_stream));
  if (rc != ADACC_OK) return rc;
  ws->device_mem = device_mem;
  ws->bytes = bytes;
  ws->epoch = 0;
  ws->reserved = 0;
  return ADACC_OK;
}

// The fallback kernels for one tensor: count, offsets, then everything (one launch without outliers).
static int launch_generic_compress(const adacc_method* method, const Plan& p, const TensorDesc& d, uint32_t epoch,
                                   hipStream_t s) {
  int rc = ADACC_OK;
  const bool topk = method->outlier_mode == ADACC_OUTLIER_TOPK;
  const uint32_t lds = ADACC_PICK(p.half, generic_lds_bytes(p.tile_elems, method->quant_group, topk && d.gs < p.tile_elems));
  const uint32_t threads = ADACC_PICK(p.half, generic_threads());
  hipLaunchKernelGGL(ADACC_PICK(p.half, compress_generic_fn(p.tile_elems, false)), dim3(p.n_tiles), dim3(threads), lds, s, d, epoch);
  rc = launch_check("compress_generic_kernel");
  if (rc != ADACC_OK || !p.outliers) return rc;
  if (needs_block_sums(method, p)) {
    hipLaunchKernelGGL(ADACC_PICK(p.half, place_sum_fn()), dim3(d.n_blocks), dim3(kPlaceThreads), 0, s, d);
    rc = launch_check("place_sum_kernel");
    if (rc != ADACC_OK) return rc;
  }
  hipLaunchKernelGGL(ADACC_PICK(p.half, place_fn()), dim3(d.n_blocks), dim3(kPlaceThreads), 0, s, d, epoch);
  rc = launch_check("place_kernel");
  if (rc != ADACC_OK) return rc;
  // segments whose outliers the first launch could not place (more than a slot holds; TOPK: some group with
  // another count than k): every other workgroup of this launch leaves at once
  hipLaunchKernelGGL(ADACC_PICK(p.half, compress_generic_fn(p.tile_elems, true)), dim3(p.n_tiles), dim3(threads), lds, s, d, epoch);
  return launch_check("compress_generic_kernel (outliers again)");
}

static int compress_one(const adacc_method* method, const void* src, uint64_t numel, void* blob, uint64_t blob_bytes,
                        adacc_workspace* ws, void* hip_stream) {
  if (!method) return ADACC_ENULL;
  Plan p;
  int rc = make_plan(method, numel, &p);
  if (rc != ADACC_OK) return rc;
  if (p.noop || numel == 0) return ADACC_OK;
  if (!src || !blob) return ADACC_ENULL;
  adacc_layout L;
  fill_layout(method, numel, p, &L);
  if (blob_bytes < L.total_bytes) return ADACC_ESIZE;
  if (misaligned(src, 16) || misaligned(blob, 256)) return ADACC_EALIGN;
  if (p.outliers) {
    if (!ws || !ws->device_mem) return ADACC_ENULL;
    if (ws->bytes < ws_plan(method, p).bytes) return ADACC_ESIZE;
    if (misaligned(ws->device_mem, 256)) return ADACC_EALIGN;
  }
  int cus = 0;
  rc = device_cus(&cus);  // also: fail here, before any state changes, when there is no device
  if (rc != ADACC_OK) return rc;
  TensorDesc d;
  fill_desc(method, numel, p, L, src, blob, nullptr, 0, p.outliers ? ws->device_mem : nullptr, &d);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (p.generic) {
    uint32_t epoch = 0;
    if (p.outliers) {
      rc = next_epoch(ws, s, &epoch);
      if (rc != ADACC_OK) return rc;
    }
    return launch_generic_compress(method, p, d, epoch, s);
  }
  CompressFn fn = compress_fn(method, p.tile_elems == 4096, p.rowwise || topk_in_rows(method, p), topk_whole_tile(method, p));
  const uint32_t grid = (p.n_tiles + kWavesPerWg - 1) / kWavesPerWg;  // one tile per wavefront
  uint32_t epoch = 0;
  if (p.outliers) {
    rc = next_epoch(ws, s, &epoch);
    if (rc != ADACC_OK) return rc;
  }
  if (p.n_tiles != 0) {
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), 0, s, d, epoch);
    rc = launch_check("compress_kernel");
    if (rc != ADACC_OK) return rc;
    if (p.outliers) {
      if (needs_block_sums(method, p)) {
        hipLaunchKernelGGL(ADACC_PICK(p.half, place_sum_fn()), dim3(d.n_blocks), dim3(kPlaceThreads), 0, s, d);
        rc = launch_check("place_sum_kernel");
        if (rc != ADACC_OK) return rc;
      }
      hipLaunchKernelGGL(ADACC_PICK(p.half, place_fn()), dim3(d.n_blocks), dim3(kPlaceThreads), 0, s, d, epoch);
      rc = launch_check("place_kernel");
      if (rc != ADACC_OK) return rc;
    }
  }
  if (p.tail != 0) {  // after the placement: the tail's outliers go behind those of the main part
    hipLaunchKernelGGL(ADACC_PICK(p.half, compress_tail_fn()), dim3(1), dim3(kWave), 0, s, d);
    rc = launch_check("compress_tail_kernel");
  }
  return rc;
}

int adacc_compress(const adacc_method* method, const void* src, uint64_t numel, void* blob, uint64_t blob_bytes,
                   adacc_workspace* ws, void* hip_stream) {
  return compress_one(method, src, numel, blob, blob_bytes, ws, hip_stream);
}

// ---- the same for callers that cannot allocate: the workspace is a device array of the library
constexpr uint64_t kNoallocScratchBytes = 24ull << 20;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];

int adacc_compress_noalloc(const adacc_method* method, const void* src, uint64_t numel, void* blob,
                           uint64_t blob_bytes, void* hip_stream) {
  if (!method) return ADACC_ENULL;
  Plan p;
  int rc = make_plan(method, numel, &p);
  if (rc != ADACC_OK) return rc;
  if (p.noop || numel == 0 || !p.outliers) return compress_one(method, src, numel, blob, blob_bytes, nullptr, hip_stream);
  if (ws_plan(method, p).bytes > kNoallocScratchBytes) return ADACC_ELIMIT;
  // Every device has its own copy of the array at its own address: looked up once per device, with
  // that device current, and kept together with the launch counter of the words in it.
  static adacc_workspace per_device[64];
  static std::mutex lock;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= 64) return ADACC_EINVAL;
  std::lock_guard<std::mutex> hold(lock);  // calls that share the array are serialised on the host; on the GPU they must not overlap
  adacc_workspace* ws = &per_device[dev];
  if (!ws->device_mem) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    // the flag word of a tensor must not hold a value that a later launch counter takes: cleared by a
    // kernel on the caller's stream before the first use
    rc = clear_device(ptr, kNoallocScratchBytes, static_cast<hipStream_t>(hip_stream));
    if (rc != ADACC_OK) return rc;
    ws->device_mem = ptr;
    ws->bytes = kNoallocScratchBytes;
    ws->epoch = 0;
  }
  return compress_one(method, src, numel, blob, blob_bytes, ws, hip_stream);
}

int adacc_decompress(const adacc_method* method, const void* blob, uint64_t blob_bytes, uint64_t numel, void* dst,
                     int dst_dtype, void* hip_stream) {
  if (!method) return ADACC_ENULL;
  if (dst_dtype != ADACC_DST_16 && dst_dtype != ADACC_DST_F32) return ADACC_EINVAL;
  Plan p;
  int rc = make_plan(method, numel, &p);
  if (rc != ADACC_OK) return rc;
  if (p.noop || numel == 0) return ADACC_OK;
  if (!blob || !dst) return ADACC_ENULL;
  adacc_layout L;
  fill_layout(method, numel, p, &L);
  if (blob_bytes < L.total_bytes) return ADACC_ESIZE;
  if (misaligned(dst, 16) || misaligned(blob, 256)) return ADACC_EALIGN;
  TensorDesc d;
  fill_desc(method, numel, p, L, nullptr, const_cast<void*>(blob), dst, dst_dtype, nullptr, &d);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (p.generic) {
    hipLaunchKernelGGL(ADACC_PICK(p.half, decompress_generic_fn()), dim3(p.n_tiles), dim3(ADACC_PICK(p.half, generic_threads())), 0, s, d);
    return launch_check("decompress_generic_kernel");
  }
  DecompressFn fn = ADACC_PICK(p.half, decompress_fn(method->bits, method->asym, dst_dtype == ADACC_DST_F32));
  if (d.n_tiles != 0) {
    uint32_t grid = 0;
    rc = grid_for(d.n_tiles, reinterpret_cast<const void*>(fn), &grid);
    if (rc != ADACC_OK) return rc;
    hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), 0, s, d, p.outliers ? 1u : 0u);
    rc = launch_check("decompress_kernel");
    if (rc != ADACC_OK) return rc;
  }
  if (p.tail != 0) {  // writes elements the kernel above does not touch
    hipLaunchKernelGGL(ADACC_PICK(p.half, decompress_tail_fn()), dim3(1), dim3(kWave), 0, s, d);
    rc = launch_check("decompress_tail_kernel");
  }
  return rc;
}

static int batch_prepare(uint32_t n, const adacc_method* methods, const uint64_t* numels, std::vector<Plan>* plans,
                         uint32_t* total_tiles, uint32_t* n_active, uint64_t* region_bytes) {
  plans->resize(n);
  uint64_t tiles = 0, regions = 0;
  uint32_t act = 0;
  for (uint32_t i = 0; i < n; ++i) {
    const int rc = make_plan(&methods[i], numels[i], &(*plans)[i]);
    if (rc != ADACC_OK) return rc;
    if ((*plans)[i].noop || numels[i] == 0) { (*plans)[i].noop = true; continue; }
    tiles += (*plans)[i].n_tiles;
    regions += ws_plan(&methods[i], (*plans)[i]).bytes;
    ++act;
  }
  if (tiles >= (1ull << 32)) return ADACC_EINVAL;
  *total_tiles = (uint32_t)tiles;
  *n_active = act;
  *region_bytes = regions;
  return ADACC_OK;
}

uint64_t adacc_batch_workspace_bytes(uint32_t n, const adacc_method* methods, const uint64_t* numels) {
  if (n && (!methods || !numels)) return 0;
  std::vector<Plan> plans;
  uint32_t total = 0, act = 0;
  uint64_t regions = 0;
  if (batch_prepare(n, methods, numels, &plans, &total, &act, &regions) != ADACC_OK) return 0;
  return batch_plan(act, regions).bytes;
}

// Descriptors of the active tensors of a batch.
static int batch_table(uint32_t n, const adacc_method* methods, const std::vector<Plan>& plans, const uint64_t* numels,
                       const void* const* srcs, void* const* blobs, const uint64_t* blob_bytes, void* const* dsts,
                       int dst_dtype, bool compress, unsigned char* regions, std::vector<TensorDesc>* descs,
                       std::vector<uint32_t>* origin) {
  uint64_t region_off = 0;
  for (uint32_t i = 0; i < n; ++i) {
    if (plans[i].noop) continue;
    if (!blobs[i]) return ADACC_ENULL;
    if (compress ? !srcs[i] : !dsts[i]) return ADACC_ENULL;
    adacc_layout L;
    fill_layout(&methods[i], numels[i], plans[i], &L);
    if (blob_bytes[i] < L.total_bytes) return ADACC_ESIZE;
    if (misaligned(blobs[i], 256)) return ADACC_EALIGN;
    if (compress ? misaligned(srcs[i], 16) : misaligned(dsts[i], 16)) return ADACC_EALIGN;
    TensorDesc d;
    fill_desc(&methods[i], numels[i], plans[i], L, compress ? srcs[i] : nullptr, blobs[i], compress ? nullptr : dsts[i],
              dst_dtype, compress ? regions + region_off : nullptr, &d);
    descs->push_back(d);
    origin->push_back(i);
    if (compress) region_off += ws_plan(&methods[i], plans[i]).bytes;
  }
  return ADACC_OK;
}

int adacc_compress_batch(uint32_t n, const adacc_method* methods, const void* const* srcs, const uint64_t* numels,
                         void* const* blobs, const uint64_t* blob_bytes, adacc_workspace* ws, void* hip_stream) {
  if (n == 0) return ADACC_OK;
  if (!methods || !srcs || !numels || !blobs || !blob_bytes) return ADACC_ENULL;
  std::vector<Plan> plans;
  uint32_t total = 0, act = 0;
  uint64_t region_bytes = 0;
  int rc = batch_prepare(n, methods, numels, &plans, &total, &act, &region_bytes);
  if (rc != ADACC_OK) return rc;
  if (act == 0) return ADACC_OK;
  if (!ws || !ws->device_mem) return ADACC_ENULL;
  const BatchPlan bp = batch_plan(act, region_bytes);
  if (ws->bytes < bp.bytes) return ADACC_ESIZE;
  if (misaligned(ws->device_mem, 256)) return ADACC_EALIGN;
  unsigned char* mem = static_cast<unsigned char*>(ws->device_mem);
  std::vector<TensorDesc> descs;
  std::vector<uint32_t> origin;
  rc = batch_table(n, methods, plans, numels, srcs, blobs, blob_bytes, nullptr, 0, true, mem + bp.regions_off, &descs,
                   &origin);
  if (rc != ADACC_OK) return rc;  // every argument is checked before the device is touched
  int cus = 0;
  rc = device_cus(&cus);
  if (rc != ADACC_OK) return rc;
  // the launches: tiles (by register class), block sums, placement
  const uint32_t nt = (uint32_t)descs.size();
  std::vector<uint32_t> units(nt), members;
  std::vector<int> kind(nt);
  std::vector<GroupLaunch> tiles, sums, places, tails;
  // (tensors that go through the fallback kernels are launched one by one, after the others)
  for (uint32_t i = 0; i < nt; ++i) {
    units[i] = descs[i].generic ? 0u : descs[i].n_tiles;
    kind[i] = batch_kind(&methods[origin[i]], plans[origin[i]]) + (plans[origin[i]].half ? kBatchKinds : 0);
  }
  group_launches(units, kind, &members, &tiles);
  // The table goes up in the order of the tile launches' member lists, so that the tile kernels find the entry
  // of blockIdx.y at table + first_member without looking a number up first; the other kernels keep their lists.
  const uint32_t n_listed = (uint32_t)members.size();
  std::vector<uint32_t> place(nt, 0xFFFFFFFFu);
  std::vector<TensorDesc> ordered;
  ordered.reserve(nt);
  for (uint32_t j = 0; j < n_listed; ++j) { place[members[j]] = j; ordered.push_back(descs[members[j]]); }
  for (uint32_t i = 0; i < nt; ++i)
    if (place[i] == 0xFFFFFFFFu) { place[i] = (uint32_t)ordered.size(); ordered.push_back(descs[i]); }
  for (uint32_t i = 0; i < nt; ++i) {
    units[i] = (!descs[i].generic && needs_block_sums(&methods[origin[i]], plans[origin[i]])) ? descs[i].n_blocks : 0u;
    kind[i] = plans[origin[i]].half ? kBatchKinds : 0;
  }
  group_launches(units, kind, &members, &sums);
  for (uint32_t i = 0; i < nt; ++i) units[i] = descs[i].generic ? 0u : descs[i].n_blocks;
  group_launches(units, kind, &members, &places);
  for (uint32_t i = 0; i < nt; ++i) units[i] = descs[i].tail != 0u ? 1u : 0u;
  group_launches(units, kind, &members, &tails);
  for (uint32_t j = n_listed; j < (uint32_t)members.size(); ++j) members[j] = place[members[j]];
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  uint32_t epoch = 0;
  rc = next_epoch(ws, s, &epoch);
  if (rc != ADACC_OK) return rc;
  TensorDesc* dt = reinterpret_cast<TensorDesc*>(mem);
  uint32_t* dm = reinterpret_cast<uint32_t*>(mem + bp.members_off);
  rc = upload_table(ordered, dt, s);
  if (rc == ADACC_OK && members.size() > n_listed) rc = upload_words(members, dm, s);
  if (rc != ADACC_OK) return rc;
  for (const GroupLaunch& g : tiles)
    hipLaunchKernelGGL(compress_batch_fn(g.kind >= kBatchKinds, g.kind % kBatchKinds),
                       dim3((g.max_units + kWavesPerWg - 1) / kWavesPerWg, g.n_members),
                       dim3(kThreads), 0, s, dt + g.first_member, static_cast<const uint32_t*>(nullptr), epoch);
  rc = launch_check("compress_batch_kernel");
  if (rc != ADACC_OK) return rc;
  for (const GroupLaunch& g : sums)
    hipLaunchKernelGGL(ADACC_PICK(g.kind >= kBatchKinds, place_sum_batch_fn()), dim3(g.max_units, g.n_members), dim3(kPlaceThreads), 0, s, dt,
                       dm + g.first_member);
  for (const GroupLaunch& g : places)
    hipLaunchKernelGGL(ADACC_PICK(g.kind >= kBatchKinds, place_batch_fn()), dim3(g.max_units, g.n_members), dim3(kPlaceThreads), 0, s, dt,
                       dm + g.first_member, epoch);
  rc = launch_check("place_batch_kernel");
  if (rc != ADACC_OK) return rc;
  for (const GroupLaunch& g : tails)  // one workgroup per tensor that has a tail, after the placement
    hipLaunchKernelGGL(ADACC_PICK(g.kind >= kBatchKinds, compress_tail_batch_fn()), dim3(g.n_members), dim3(kWave), 0, s, dt,
                       dm + g.first_member);
  rc = launch_check("compress_tail_batch_kernel");
  for (uint32_t i = 0; i < nt && rc == ADACC_OK; ++i)
    if (descs[i].generic) rc = launch_generic_compress(&methods[origin[i]], plans[origin[i]], descs[i], epoch, s);
  return rc;
}

int adacc_decompress_batch(uint32_t n, const adacc_method* methods, const void* const* blobs, const uint64_t* blob_bytes,
                           const uint64_t* numels, void* const* dsts, int dst_dtype, adacc_workspace* ws,
                           void* hip_stream) {
  if (n == 0) return ADACC_OK;
  if (!methods || !blobs || !numels || !dsts || !blob_bytes) return ADACC_ENULL;
  if (dst_dtype != ADACC_DST_16 && dst_dtype != ADACC_DST_F32) return ADACC_EINVAL;
  std::vector<Plan> plans;
  uint32_t total = 0, act = 0;
  uint64_t region_bytes = 0;
  int rc = batch_prepare(n, methods, numels, &plans, &total, &act, &region_bytes);
  if (rc != ADACC_OK) return rc;
  if (act == 0) return ADACC_OK;
  if (!ws || !ws->device_mem) return ADACC_ENULL;
  const BatchPlan bp = batch_plan(act, region_bytes);
  if (ws->bytes < bp.bytes) return ADACC_ESIZE;
  if (misaligned(ws->device_mem, 256)) return ADACC_EALIGN;
  std::vector<TensorDesc> descs;
  std::vector<uint32_t> origin;
  rc = batch_table(n, methods, plans, numels, nullptr, const_cast<void* const*>(blobs), blob_bytes, dsts, dst_dtype,
                   false, nullptr, &descs, &origin);
  if (rc != ADACC_OK) return rc;
  int cus = 0;
  rc = device_cus(&cus);
  if (rc != ADACC_OK) return rc;
  const uint32_t nt = (uint32_t)descs.size();
  std::vector<uint32_t> units(nt), members;
  std::vector<int> kind(nt, 0);
  std::vector<GroupLaunch> launches;
  for (uint32_t i = 0; i < nt; ++i) {
    units[i] = descs[i].generic ? 0u : descs[i].n_tiles;  // pieces of 2048 elements
    kind[i] = plans[origin[i]].half ? kBatchKinds : 0;
  }
  group_launches(units, kind, &members, &launches);
  // The table goes up in the order of the launches' member lists, so that the main kernels find the entry of
  // blockIdx.y at table + first_member without looking a number up first; the tail kernels keep their lists.
  const uint32_t n_listed = (uint32_t)members.size();
  std::vector<uint32_t> place(nt, 0xFFFFFFFFu);
  std::vector<TensorDesc> ordered;
  ordered.reserve(nt);
  for (uint32_t j = 0; j < n_listed; ++j) { place[members[j]] = j; ordered.push_back(descs[members[j]]); }
  for (uint32_t i = 0; i < nt; ++i)
    if (place[i] == 0xFFFFFFFFu) { place[i] = (uint32_t)ordered.size(); ordered.push_back(descs[i]); }
  std::vector<GroupLaunch> tails;
  for (uint32_t i = 0; i < nt; ++i) units[i] = descs[i].tail != 0u ? 1u : 0u;
  group_launches(units, kind, &members, &tails);
  for (uint32_t j = n_listed; j < (uint32_t)members.size(); ++j) members[j] = place[members[j]];
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  unsigned char* mem = static_cast<unsigned char*>(ws->device_mem);
  TensorDesc* dt = reinterpret_cast<TensorDesc*>(mem);
  uint32_t* dm = reinterpret_cast<uint32_t*>(mem + bp.members_off);
  rc = upload_table(ordered, dt, s);
  if (rc == ADACC_OK && members.size() > n_listed) rc = upload_words(members, dm, s);
  if (rc != ADACC_OK) return rc;
  for (const GroupLaunch& g : launches)
    hipLaunchKernelGGL(ADACC_PICK(g.kind >= kBatchKinds, decompress_batch_fn(dst_dtype == ADACC_DST_F32)),
                       dim3((g.max_units + kWavesPerWg - 1) / kWavesPerWg, g.n_members), dim3(kThreads), 0, s,
                       dt + g.first_member, static_cast<const uint32_t*>(nullptr));
  for (const GroupLaunch& g : tails)
    hipLaunchKernelGGL(ADACC_PICK(g.kind >= kBatchKinds, decompress_tail_batch_fn()), dim3(g.n_members), dim3(kWave), 0, s, dt,
                       dm + g.first_member);
  for (uint32_t i = 0; i < nt; ++i)
    if (descs[i].generic)
      hipLaunchKernelGGL(ADACC_PICK(plans[origin[i]].half, decompress_generic_fn()), dim3(descs[i].n_tiles),
                         dim3(ADACC_PICK(plans[origin[i]].half, generic_threads())), 0, s, descs[i]);
  return launch_check("decompress_batch_kernel");
}

int adacc_read_status(const void* blob, const adacc_layout* layout, void* hip_stream, uint32_t status_out[4]) {
  if (!blob || !layout || !status_out) return ADACC_ENULL;
  if (layout->total_bytes == 0) { status_out[0] = status_out[1] = status_out[2] = status_out[3] = 0; return ADACC_OK; }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipMemcpyAsync(status_out, static_cast<const unsigned char*>(blob) + layout->status_off, 16,
                                hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(status)");
  e = hipStreamSynchronize(s);
  return e == hipSuccess ? ADACC_OK : hip_fail(e, "hipStreamSynchronize");
}

int adacc_channel_layout_of(const adacc_channel_method* method, uint64_t tokens, uint32_t hidden,
                            adacc_channel_layout* out) {
  if (!method || !out) return ADACC_ENULL;
  ChannelPlan cp;
  const int rc = make_channel_plan(method, tokens, hidden, &cp);
  if (rc != ADACC_OK) return rc;
  fill_channel_layout(method, tokens, hidden, cp, out);
  return ADACC_OK;
}

uint64_t adacc_channel_workspace_bytes(uint64_t tokens, uint32_t hidden) {
  if (hidden < 8 || hidden > 65536 || hidden % 8 != 0 || tokens > 0xFFFFFFFFull / hidden) return 0;
  const uint32_t n_chunks = (uint32_t)((tokens + kChunkTokens - 1) / kChunkTokens);
  return channel_partial_bytes(n_chunks, hidden) + align256(8ull * hidden);
}

int adacc_channel_compress(const adacc_channel_method* method, const void* src, uint64_t tokens, uint32_t hidden,
                           void* blob, uint64_t blob_bytes, void* workspace, uint64_t workspace_bytes,
                           void* hip_stream) {
  if (!method) return ADACC_ENULL;
  ChannelPlan cp;
  int rc = make_channel_plan(method, tokens, hidden, &cp);
  if (rc != ADACC_OK) return rc;
  if (tokens == 0) return ADACC_OK;
  if (!src || !blob || !workspace) return ADACC_ENULL;
  adacc_channel_layout L;
  fill_channel_layout(method, tokens, hidden, cp, &L);
  if (blob_bytes < L.total_bytes) return ADACC_ESIZE;
  if (workspace_bytes < adacc_channel_workspace_bytes(tokens, hidden)) return ADACC_ESIZE;
  if (misaligned(src, 16) || misaligned(blob, 256) || misaligned(workspace, 256)) return ADACC_EALIGN;
  TensorDesc d;
  fill_desc(&cp.quant, cp.numel, cp.plan, cp.quant_layout, src, blob, nullptr, 0, nullptr, &d);
  ChannelDesc c;
  fill_channel_desc(method, tokens, hidden, L, blob, &c);
  float* partial = static_cast<float*>(workspace);
  double* S = reinterpret_cast<double*>(static_cast<unsigned char*>(workspace) + channel_partial_bytes(cp.n_chunks, hidden));
  const bool half = cp.plan.half;
  // strips of 512 channels where the matrix and the groups allow them, else tiles of 2048 consecutive elements
  const bool by_strips = cp.plan.rowwise && hidden % 512u == 0;
  ChannelFn fn = by_strips ? ADACC_PICK(half, channel_compress_strip_fn(method->bits, method->asym))
                           : ADACC_PICK(half, channel_compress_fn(method->bits, method->asym, cp.plan.rowwise));
  uint32_t grid = 0;
  if (by_strips) {
    grid = strip_grid(tokens, hidden, ADACC_PICK(half, channel_strip_rows()));
  } else {
    rc = grid_for(cp.plan.n_tiles, reinterpret_cast<const void*>(fn), &grid, 2);
    if (rc != ADACC_OK) return rc;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);

  const uint32_t strips = (hidden / 8 + kWave - 1) / kWave;  // a workgroup: one chunk of a strip of 512 channels
  hipLaunchKernelGGL(ADACC_PICK(half, channel_partial_fn(2ull * cp.numel > kStatsKeepBytes)), dim3(cp.n_chunks * strips),
                     dim3(ADACC_PICK(half, channel_partial_threads())), 0, s, static_cast<const uint16_t*>(src), (uint32_t)tokens,
                     hidden, partial, strips);
  rc = launch_check("channel_partial_kernel");
  if (rc != ADACC_OK) return rc;
  const uint32_t per_wg = ADACC_PICK(half, channel_score_channels());
  hipLaunchKernelGGL(ADACC_PICK(half, channel_score_fn()), dim3((hidden + per_wg - 1) / per_wg), dim3(kThreads), 0, s,
                     static_cast<const float*>(partial), cp.n_chunks, hidden, S);
  rc = launch_check("channel_score_kernel");
  if (rc != ADACC_OK) return rc;
  hipLaunchKernelGGL(ADACC_PICK(half, channel_select_fn()), dim3(1), dim3(ADACC_PICK(half, channel_select_threads())), 0, s, static_cast<const double*>(S), c);
  rc = launch_check("channel_select_kernel");
  if (rc != ADACC_OK) return rc;
  hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), by_strips ? 0u : channel_mask_lds(hidden), s, d, c);
  return launch_check("channel_compress_kernel");
}

int adacc_channel_decompress(const adacc_channel_method* method, const void* blob, uint64_t blob_bytes,
                             uint64_t tokens, uint32_t hidden, void* dst, int dst_dtype, void* hip_stream) {
  if (!method) return ADACC_ENULL;
  if (dst_dtype != ADACC_DST_16 && dst_dtype != ADACC_DST_F32) return ADACC_EINVAL;
  ChannelPlan cp;
  int rc = make_channel_plan(method, tokens, hidden, &cp);
  if (rc != ADACC_OK) return rc;
  if (tokens == 0) return ADACC_OK;
  if (!blob || !dst) return ADACC_ENULL;
  adacc_channel_layout L;
  fill_channel_layout(method, tokens, hidden, cp, &L);
  if (blob_bytes < L.total_bytes) return ADACC_ESIZE;
  if (misaligned(dst, 16) || misaligned(blob, 256)) return ADACC_EALIGN;
  TensorDesc d;
  fill_desc(&cp.quant, cp.numel, cp.plan, cp.quant_layout, nullptr, const_cast<void*>(blob), dst, dst_dtype, nullptr,
            &d);
  ChannelDesc c;
  fill_channel_desc(method, tokens, hidden, L, const_cast<void*>(blob), &c);
  ChannelFn fn = ADACC_PICK(cp.plan.half, channel_decompress_fn(method->bits, method->asym, dst_dtype == ADACC_DST_F32));
  const uint32_t grid = strip_grid(tokens, hidden, ADACC_PICK(cp.plan.half, channel_strip_rows()));
  hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), d, c);
  return launch_check("channel_decompress_kernel");
}

int adacc_channel_read_status(const void* blob, const adacc_channel_layout* layout, void* hip_stream,
                              uint32_t status_out[4]) {
  if (!blob || !layout || !status_out) return ADACC_ENULL;
  if (layout->total_bytes == 0) return ADACC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipError_t e = hipMemcpyAsync(status_out, static_cast<const unsigned char*>(blob) + layout->status_off, 16,
                                hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(status)");
  e = hipStreamSynchronize(s);
  return e == hipSuccess ? ADACC_OK : hip_fail(e, "hipStreamSynchronize");
}

// ---- channel-wise symmetric quantisation (Section 3.2, Query / Key / Value)
static bool channelwise_sizes_ok(uint32_t bits, uint64_t tokens, uint32_t hidden) {
  if (bits != 4 && bits != 8) return false;
  if (hidden < 8 || hidden > 65536 || hidden % 8 != 0) return false;
  return tokens <= 0xFFFFFFFFull / hidden;
}

static void channelwise_layout(uint32_t bits, uint64_t tokens, uint32_t hidden, adacc_channelwise_layout* L) {
  L->codes_off = 0;
  L->scales_off = align256(tokens * hidden * bits / 8);
  L->total_bytes = L->scales_off + align256(4ull * hidden);
}

static uint64_t channelwise_partial_bytes(uint64_t tokens, uint32_t hidden) {
  return align256(2ull * ((tokens + kChunkTokens - 1) / kChunkTokens) * hidden);
}

int adacc_channelwise_layout_of(uint32_t bits, uint64_t tokens, uint32_t hidden, adacc_channelwise_layout* out) {
  if (!out) return ADACC_ENULL;
  if (!channelwise_sizes_ok(bits, tokens, hidden)) return ADACC_EINVAL;
  channelwise_layout(bits, tokens, hidden, out);
  return ADACC_OK;
}

uint64_t adacc_channelwise_workspace_bytes(uint64_t tokens, uint32_t hidden) {
  if (!channelwise_sizes_ok(8, tokens, hidden)) return 0;
  return channelwise_partial_bytes(tokens, hidden) + align256(4ull * hidden);
}

static void channelwise_desc(uint32_t bits, uint32_t scale_rule, uint64_t tokens, uint32_t hidden,
                             const adacc_channelwise_layout& L, void* blob, ChannelwiseDesc* c) {
  std::memset(c, 0, sizeof *c);
  unsigned char* b = static_cast<unsigned char*>(blob);
  c->codes = b + L.codes_off;
  c->scales = reinterpret_cast<float*>(b + L.scales_off);
  c->numel = tokens * hidden;
  c->tokens = (uint32_t)tokens;
  c->hidden = hidden;
  c->n_chunks = (uint32_t)((tokens + kChunkTokens - 1) / kChunkTokens);
  const float q = (float)(1u << (bits - 1));
  c->divisor = scale_rule == ADACC_SCALE_PAPER ? q : q - 1.0f;
  c->inv_divisor = scale_rule == ADACC_SCALE_PAPER ? 1.0f / q : 0.0f;  // exact for a power of two
}

int adacc_channelwise_compress(uint32_t bits, uint32_t scale_rule, uint32_t dtype, const void* src, uint64_t tokens,
                               uint32_t hidden, void* blob, uint64_t blob_bytes, void* workspace,
                               uint64_t workspace_bytes, void* hip_stream) {
  if (!channelwise_sizes_ok(bits, tokens, hidden) || scale_rule > 1 || dtype > ADACC_DTYPE_F16) return ADACC_EINVAL;
  const bool half = dtype == ADACC_DTYPE_F16;
  if (tokens == 0) return ADACC_OK;
  if (!src || !blob || !workspace) return ADACC_ENULL;
  adacc_channelwise_layout L;
  channelwise_layout(bits, tokens, hidden, &L);
  if (blob_bytes < L.total_bytes) return ADACC_ESIZE;
  if (workspace_bytes < adacc_channelwise_workspace_bytes(tokens, hidden)) return ADACC_ESIZE;
  if (misaligned(src, 16) || misaligned(blob, 256) || misaligned(workspace, 256)) return ADACC_EALIGN;
  ChannelwiseDesc c;
  channelwise_desc(bits, scale_rule, tokens, hidden, L, blob, &c);
  c.src = static_cast<const uint16_t*>(src);
  c.partial = static_cast<uint16_t*>(workspace);
  c.inv = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + channelwise_partial_bytes(tokens, hidden));
  ChannelwiseFn quant = ADACC_PICK(half, channelwise_quantise_fn(bits));
  const uint32_t grid = strip_grid(tokens, hidden, ADACC_PICK(half, channelwise_strip_rows()));
  int rc = ADACC_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const uint32_t strips = (hidden / 8 + kWave - 1) / kWave;  // a workgroup: one chunk of a strip of 512 channels
  hipLaunchKernelGGL(ADACC_PICK(half, channelwise_partial_fn(2ull * c.numel > kStatsKeepBytes)), dim3(c.n_chunks * strips),
                     dim3(ADACC_PICK(half, channelwise_partial_threads())), 0, s, c, strips);
  rc = launch_check("channelwise_partial_kernel");
  if (rc != ADACC_OK) return rc;
  const uint32_t per_wg = ADACC_PICK(half, channelwise_fold_octets());
  hipLaunchKernelGGL(ADACC_PICK(half, channelwise_fold_fn()), dim3((hidden / 8 + per_wg - 1) / per_wg), dim3(kThreads), 0, s, c);
  rc = launch_check("channelwise_fold_kernel");
  if (rc != ADACC_OK) return rc;
  hipLaunchKernelGGL(quant, dim3(grid), dim3(kThreads), 0, s, c);
  return launch_check("channelwise_quantise_kernel");
}

int adacc_channelwise_decompress(uint32_t bits, uint32_t dtype, const void* blob, uint64_t blob_bytes, uint64_t tokens,
                                 uint32_t hidden, void* dst, int dst_dtype, void* hip_stream) {
  if (dst_dtype != ADACC_DST_16 && dst_dtype != ADACC_DST_F32) return ADACC_EINVAL;
  if (dtype > ADACC_DTYPE_F16) return ADACC_EINVAL;
  if (!channelwise_sizes_ok(bits, tokens, hidden)) return ADACC_EINVAL;
  if (tokens == 0) return ADACC_OK;
  if (!blob || !dst) return ADACC_ENULL;
  adacc_channelwise_layout L;
  channelwise_layout(bits, tokens, hidden, &L);
  if (blob_bytes < L.total_bytes) return ADACC_ESIZE;
  if (misaligned(dst, 16) || misaligned(blob, 256)) return ADACC_EALIGN;
  ChannelwiseDesc c;
  channelwise_desc(bits, 0, tokens, hidden, L, const_cast<void*>(blob), &c);
  c.dst = dst;
  ChannelwiseFn fn = ADACC_PICK(dtype == ADACC_DTYPE_F16, channelwise_dequantise_fn(bits, dst_dtype == ADACC_DST_F32));
  const uint32_t grid = strip_grid(tokens, hidden, ADACC_PICK(dtype == ADACC_DTYPE_F16, channelwise_strip_rows()));
  hipLaunchKernelGGL(fn, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream), c);
  return launch_check("channelwise_dequantise_kernel");
}

uint64_t adacc_mask_packed_bytes(uint64_t n) { return (n + 7u) / 8u; }

static int mask_launch(MaskFn fn, const void* in, uint64_t n, void* out, void* hip_stream, const char* what) {
  if (n == 0) return ADACC_OK;
  if (!in || !out) return ADACC_ENULL;
  if (misaligned(in, 16) || misaligned(out, 16)) return ADACC_EALIGN;
  int cus = 0;
  const int rc = device_cus(&cus);
  if (rc != ADACC_OK) return rc;
  const uint64_t pieces = n / 16u;  // one lane turns over 16 elements at a time, eight times per round
  uint64_t grid = (pieces + 8ull * kThreads - 1) / (8ull * kThreads);
  const uint64_t cap = (uint64_t)cus * (uint64_t)knobs().mask_wgs_per_cu;
  if (grid > cap) grid = cap;
  if (grid == 0) grid = 1;
  hipLaunchKernelGGL(fn, dim3((uint32_t)grid), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const uint8_t*>(in), n, static_cast<uint8_t*>(out));
  return launch_check(what);
}

int adacc_mask_pack(const void* mask, uint64_t n, void* bits, void* hip_stream) {
  return mask_launch(mask_pack_fn(), mask, n, bits, hip_stream, "mask_pack_kernel");
}

int adacc_mask_unpack(const void* bits, uint64_t n, void* mask, void* hip_stream) {
  return mask_launch(mask_unpack_fn(), bits, n, mask, hip_stream, "mask_unpack_kernel");
}

uint64_t adacc_compressed_bytes(const adacc_method* method, uint64_t numel, uint64_t n_outliers) {
  if (!method) return 0;
  Plan p;
  if (make_plan(method, numel, &p) != ADACC_OK) return 0;
  if (p.noop) return 2ull * numel;
  const uint64_t groups = (numel + method->quant_group - 1) / method->quant_group;
  uint64_t bytes = (numel * method->bits + 7) / 8 + 4ull * groups * (method->asym ? 2u : 1u);
  if (p.outliers) bytes += 6ull * n_outliers + 4ull * ((uint64_t)p.n_tiles_all + 1u);
  return bytes;
}

uint64_t adacc_channel_compressed_bytes(const adacc_channel_method* method, uint64_t tokens, uint32_t hidden,
                                        uint64_t n_channels) {
  if (!method) return 0;
  ChannelPlan cp;
  if (make_channel_plan(method, tokens, hidden, &cp) != ADACC_OK) return 0;
  const uint64_t numel = tokens * hidden;
  const uint64_t groups = numel / method->quant_group;
  return numel * method->bits / 8 + 4ull * groups * (method->asym ? 2u : 1u) + n_channels * (2ull * tokens + 4u);
}

int adacc_hbm_stream(int mix, void* dst, const void* src_a, const void* src_b, uint64_t bytes, void* hip_stream) {
  if (mix < ADACC_STREAM_READ || mix > ADACC_STREAM_READ2_WRITE) return ADACC_EINVAL;
  const bool wr = mix != ADACC_STREAM_READ, rd = mix != ADACC_STREAM_WRITE, rd2 = mix == ADACC_STREAM_READ2_WRITE;
  if ((wr && !dst) || (rd && !src_a) || (rd2 && !src_b)) return ADACC_ENULL;
  if (bytes % 16 != 0) return ADACC_EINVAL;
  if ((wr && misaligned(dst, 16)) || (rd && misaligned(src_a, 16)) || (rd2 && misaligned(src_b, 16))) return ADACC_EALIGN;
  if (bytes == 0) return ADACC_OK;
  const uint64_t n16 = bytes / 16;
  const uint64_t grid = (n16 + 1023u) / 1024u;  // a workgroup moves 4 x 4 KiB per operand
  if (grid >= (1ull << 31)) return ADACC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  uint4* d = static_cast<uint4*>(dst);
  const uint4* a = static_cast<const uint4*>(src_a);
  const uint4* b = static_cast<const uint4*>(src_b);
  switch (mix) {
    case ADACC_STREAM_READ: hipLaunchKernelGGL(hbm_stream_kernel<0>, dim3((uint32_t)grid), dim3(kThreads), 0, s, d, a, b, n16, static_cast<uint32_t*>(dst)); break;
    case ADACC_STREAM_WRITE: hipLaunchKernelGGL(hbm_stream_kernel<1>, dim3((uint32_t)grid), dim3(kThreads), 0, s, d, a, b, n16, nullptr); break;
    case ADACC_STREAM_COPY: hipLaunchKernelGGL(hbm_stream_kernel<2>, dim3((uint32_t)grid), dim3(kThreads), 0, s, d, a, b, n16, nullptr); break;
    default: hipLaunchKernelGGL(hbm_stream_kernel<3>, dim3((uint32_t)grid), dim3(kThreads), 0, s, d, a, b, n16, nullptr); break;
  }
  return launch_check("hbm_stream_kernel");
}

int adacc_hbm_copy(void* dst, const void* src, uint64_t bytes, void* hip_stream) {
  return adacc_hbm_stream(ADACC_STREAM_COPY, dst, src, nullptr, bytes, hip_stream);
}

}  // extern "C"
