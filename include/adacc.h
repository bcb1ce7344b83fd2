/*
 * adacc.h - C ABI of libadacc: outlier-separated quantising compression of saved
 * 16-bit (bf16 or binary16) activation tensors on AMD MI355X (gfx950), after Adacc (arXiv 2508.00806),
 * Section 3.2 "Layer-specific Compression".
 *
 * What the library computes (Section 3.2, Fig. 3(c), Eq. 2 and Eq. 3):
 *   compress   : choose the outliers of the tensor, keep them (value + index)
 *                uncompressed, treat them as zero, and quantise everything else
 *                group by group in its original memory order to b-bit codes with
 *                one binary32 scale S (and, asymmetric, one offset O) per group;
 *   decompress : code * S (+ O), then the outliers are written back.
 * The paper quantises FP16 to INT4 and picks whole outlier channels; this
 * library takes bf16 or FP16 (adacc_method.dtype), b in {4, 8}, and picks single elements by one of three
 * rules (absolute threshold, multiple of the group's standard deviation, k
 * largest magnitudes); the paper's own rule, whole channels by Z-score (Eq. 1),
 * is served by the adacc_channel_* calls.  All arithmetic has a fixed precision
 * and order, so a compressed tensor is a pure function of the input bits.
 *
 * Conventions
 *   - Every pointer named src/dst/blob/workspace is DEVICE memory owned by the
 *     caller; the library never allocates, frees or keeps device memory.
 *     adacc_method / adacc_layout / arrays of them and the pointer arrays of the
 *     batch calls are HOST memory, read before the call returns.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call except adacc_read_status only enqueues work and returns.
 *   - Return value: ADACC_OK (0) or a negative ADACC_E* code.  Errors that the
 *     host can detect are returned before anything is enqueued.
 *   - Tensors are flat, contiguous, row-major; numel counts elements.
 */
#ifndef ADACC_H
#define ADACC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- error codes ---- */
#define ADACC_OK 0
#define ADACC_EINVAL (-1) /* malformed method or sizes                                */
#define ADACC_ENULL (-2)  /* a required pointer is NULL                               */
#define ADACC_ESIZE (-3)  /* blob or workspace smaller than the layout requires       */
#define ADACC_EALIGN (-4) /* a device pointer is not 16-byte aligned                  */
#define ADACC_EHIP (-5)   /* a HIP runtime call failed (no device, launch failure)    */
#define ADACC_ELIMIT (-6) /* size beyond the stated limit of the entry point          */

/* ---- method descriptor ---- */
#define ADACC_KIND_NOOP 0  /* tensor is retained as it is: nothing is read or written */
#define ADACC_KIND_QUANT 1 /* outlier-separated group quantisation                    */

#define ADACC_OUTLIER_NONE 0 /* plain group quantisation (Section 3.2, per-token / QKV scheme) */
#define ADACC_OUTLIER_ABS 1  /* |x| > thresh                                          */
#define ADACC_OUTLIER_STD 2  /* x*x > thresh^2 * var(stat group), population variance about the mean */
#define ADACC_OUTLIER_TOPK 3 /* the topk largest |x| of every stat group, ties to the lower index */

#define ADACC_DTYPE_BF16 0 /* bfloat16                                                */
#define ADACC_DTYPE_F16 1  /* IEEE binary16, the format the paper compresses (Section 3.2) */

#define ADACC_SCALE_PAPER 0     /* Eq. 2: S = max|X| / 2^(b-1);  Eq. 3: S = (max-min) / 2^b */
#define ADACC_SCALE_FULLRANGE 1 /* S = max|X| / (2^(b-1)-1);     S = (max-min) / (2^b-1)    */

typedef struct adacc_method {
  uint32_t kind;         /* ADACC_KIND_*                                                     */
  uint32_t bits;         /* 4 or 8                                                           */
  uint32_t quant_group;  /* Gq, elements per scale: a multiple of 8 in [8, 16384]; the groups are cut from the
                            start of the flat tensor, the last one may be short.  Powers of two up to 4096
                            (with a stat_group of that kind) run in the fast kernels, everything else in
                            fallback kernels that are 2 to 4 times slower                       */
  uint32_t asym;         /* 0: symmetric (Eq. 2), 1: asymmetric (Eq. 3, adds one offset per group) */
  uint32_t scale_rule;   /* ADACC_SCALE_*                                                    */
  uint32_t outlier_mode; /* ADACC_OUTLIER_*                                                  */
  uint32_t stat_group;   /* Gs, STD/TOPK only: a multiple of Gq, <= 16384; the last group may be
                            short: mean and variance over its own count, at most as many largest values
                            as it has elements                                                   */
  float thresh;          /* ABS: tau >= 0.  STD: k >= 0 (the library forms k*k in binary32)  */
  uint32_t topk;         /* TOPK: 1..32 outliers per stat group                              */
  uint32_t max_outliers; /* capacity of the outlier stream of the blob (0 allowed for NONE)  */
  uint32_t dtype;        /* ADACC_DTYPE_*: the 16-bit format of the tensor, of the outlier values kept in
                            the blob and of the 16-bit output of decompression                */
} adacc_method;

/* ---- blob layout ----
 * A compressed tensor ("blob") is one caller-owned device buffer cut into
 * sections, each starting on a 256-byte boundary:
 *   codes    ceil(numel*bits/8) bytes.  b=8: one two's-complement byte per element.
 *            b=4: element 2j in the low nibble of byte j, 2j+1 in the high nibble (zero when
 *            numel is odd and 2j+1 is past the end).
 *   scales   ceil(numel/Gq) binary32, S of Eq. 2 / Eq. 3.
 *   zp       ceil(numel/Gq) binary32, O of Eq. 3 (asym only, else empty).
 *   tile_ptr (n_tiles+1) uint32: tile t (elements [t*tile_elems, (t+1)*tile_elems))
 *            owns outliers [tile_ptr[t], tile_ptr[t+1]) of the stream; tile_ptr[n_tiles]
 *            is the total count.  Empty for ADACC_OUTLIER_NONE.
 *   idx,val  max_outliers int32 flat indices, ascending, and the 16-bit patterns of the tensor at
 *            those indices (structure of arrays).  Entries past the count are unspecified.
 *   status   4 uint32: [0] number of outliers found, [1] 1 if it exceeds max_outliers
 *            (the stream then holds the first max_outliers; the blob is not usable), [2], [3] 0.
 *            The rest of the 256-byte status block is scrap space of the kernels.
 */
typedef struct adacc_layout {
  uint64_t codes_off, scales_off, zp_off, tile_ptr_off, idx_off, val_off, status_off;
  uint64_t total_bytes; /* size the blob must have                                       */
  uint32_t tile_elems;  /* elements per tile: 2048, or 4096 when Gq or Gs is 4096; for group sizes that go
                           through the fallback kernels, the largest multiple of the larger group up to
                           4096 (the group itself if it is larger)                        */
  uint32_t n_tiles;     /* ceil(numel / tile_elems)                                      */
} adacc_layout;

/* Host only, pure.  Validates the method for this numel and fills *out.
 * NOOP: all zero.  Errors: ENULL, EINVAL. */
int adacc_layout_of(const adacc_method *method, uint64_t numel, adacc_layout *out);

/* ---- workspace ----
 * Compression with outliers takes every tile on its own (no tile waits for another) and settles the
 * order of the outlier stream afterwards, in a second, small kernel.  Between the two, the number
 * of outliers of every tile (4 bytes per tile) and, for ADACC_OUTLIER_ABS / _STD, the outliers
 * themselves (a slot of 256 bytes per tile) wait in a caller-owned device buffer described by an
 * adacc_workspace.  The struct is HOST memory owned by the caller; the library keeps a launch
 * counter ("epoch") in it: a flag word written by an earlier launch carries an older epoch and
 * reads as not set, so the buffer is cleared only by adacc_workspace_init and when the 30-bit
 * epoch wraps, never per call.
 * Rules: initialise once with adacc_workspace_init; afterwards any number of calls may
 * reuse it, one at a time in stream order (calls that may overlap on the GPU, or host
 * threads that call concurrently, must use different workspaces). */
typedef struct adacc_workspace {
  void *device_mem; /* caller-owned device buffer, 256-byte aligned            */
  uint64_t bytes;   /* its size                                                */
  uint32_t epoch;   /* launches since the last clear; maintained by the library */
  uint32_t reserved;
} adacc_workspace;

/* Bytes of device memory a workspace needs for this tensor (0 for ADACC_OUTLIER_NONE / NOOP). */
uint64_t adacc_workspace_bytes(const adacc_method *method, uint64_t numel);
/* Fills *ws and enqueues the clearing of device_mem on hip_stream.
 * Errors: ENULL, ESIZE (bytes < 256 or not a multiple of 16), EALIGN, EHIP. */
int adacc_workspace_init(adacc_workspace *ws, void *device_mem, uint64_t bytes, void *hip_stream);

/* ---- single tensor ----
 * adacc_compress: Section 3.2 / Fig. 3(c) compression workflow.
 *   src   numel 16-bit values of method->dtype, 16-byte aligned, never modified (the zeroing of outliers happens in registers)
 *   blob  at least adacc_layout_of(...).total_bytes, 256-byte aligned
 *   ws    an initialised workspace of at least adacc_workspace_bytes(...); may be NULL for
 *         ADACC_OUTLIER_NONE
 * numel == 0 or NOOP: returns ADACC_OK without touching anything.
 * Errors: ENULL, EINVAL, ESIZE, EALIGN, EHIP. */
int adacc_compress(const adacc_method *method, const void *src, uint64_t numel, void *blob,
                   uint64_t blob_bytes, adacc_workspace *ws, void *hip_stream);

/* adacc_compress for callers that cannot allocate device memory at all (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same blob, but the
 * workspace is a device array inside the library (24 MiB per GPU the library runs on, held until
 * the process ends) instead of a caller's buffer.  The call allocates and frees nothing.
 * Limit: adacc_workspace_bytes(method, numel) <= 24 MiB, which holds for every method up to
 * ADACC_NOALLOC_MAX_NUMEL elements (and for ADACC_OUTLIER_TOPK / _NONE at any legal size); beyond
 * that the call returns ADACC_ELIMIT.  All calls on one GPU share that array: they may follow each
 * other on one stream, or be ordered otherwise, but two that overlap on the GPU race.  The first
 * call on a device also enqueues the clearing of the array on hip_stream.  Other errors as
 * adacc_compress. */
#define ADACC_NOALLOC_MAX_NUMEL (1ull << 27)
int adacc_compress_noalloc(const adacc_method *method, const void *src, uint64_t numel, void *blob,
                           uint64_t blob_bytes, void *hip_stream);

/* adacc_decompress: Section 3.2 dequantisation (X^ = code*S, resp. code*S+O) followed by
 * the write-back of the outliers (Fig. 3(c) decompression workflow).
 *   dst_dtype ADACC_DST_16:  the tensor's own 16-bit format, method->dtype (round-to-nearest-even of the
 *                            binary32 result, too large becomes infinite; outliers bit-exact)
 *             ADACC_DST_F32: binary32
 *   dst   numel elements of that type, 16-byte aligned */
#define ADACC_DST_16 0
#define ADACC_DST_BF16 ADACC_DST_16 /* the same, for a bf16 tensor */
#define ADACC_DST_F32 1
int adacc_decompress(const adacc_method *method, const void *blob, uint64_t blob_bytes, uint64_t numel,
                     void *dst, int dst_dtype, void *hip_stream);

/* ---- batch: one call for a table of tensors (the per-tensor policy of Section 3.3,
 * R_{i,t}: compress or retain); the tiles of the whole table are served by one kernel launch, or by
 * two when it mixes methods whose groups reach 4096 elements with smaller ones, followed by one
 * launch that places the outliers of all tensors ----
 * methods[i], srcs[i], numels[i], blobs[i], blob_bytes[i] describe tensor i; NOOP entries
 * are skipped.  The workspace holds what the single-tensor workspaces would hold plus a device copy
 * of the table (adacc_batch_workspace_bytes device bytes); same init/reuse rules as above.
 * adacc_decompress_batch restores every non-NOOP tensor i into dsts[i]. */
uint64_t adacc_batch_workspace_bytes(uint32_t n, const adacc_method *methods, const uint64_t *numels);
int adacc_compress_batch(uint32_t n, const adacc_method *methods, const void *const *srcs,
                         const uint64_t *numels, void *const *blobs, const uint64_t *blob_bytes,
                         adacc_workspace *ws, void *hip_stream);
int adacc_decompress_batch(uint32_t n, const adacc_method *methods, const void *const *blobs,
                           const uint64_t *blob_bytes, const uint64_t *numels, void *const *dsts,
                           int dst_dtype, adacc_workspace *ws, void *hip_stream);

/* Copies the 4 status words of a blob to host memory and waits for the stream:
 * the only call that synchronises.  (The outlier count is what the policy
 * evolution of Section 3.4 tracks.) */
int adacc_read_status(const void *blob, const adacc_layout *layout, void *hip_stream, uint32_t status_out[4]);

/* ---- outlier channels: the selection rule of Section 3.2, Eq. 1 ----
 * The tensor is a row-major matrix of `tokens` rows and `hidden` channels.  S_h is the sum of |x|
 * over the tokens of channel h, mu and sigma are mean and (population) standard deviation of S_h
 * over the channels, Z_h = (S_h - mu) / sigma.  Channels with Z_h > z_thresh (3 in the paper), and
 * channels whose sum is not finite (they take no part in mu and sigma), are kept whole and
 * uncompressed together with their indices, count as zero in the activation, and everything else
 * is group-quantised in memory order exactly as with ADACC_OUTLIER_NONE (Eq. 2 / Eq. 3).
 * The sums are floating-point sums in a fixed order (binary32 partial sums over runs of consecutive
 * tokens, binary64 from there on), so the blob is a pure function of the input bits; a channel whose
 * Z lies within the rounding error of those sums of z_thresh (a few 1e-6 times S_h / sigma) may fall
 * on either side of the exact rule.
 * Limits: hidden a multiple of 8 in [8, 65536]; tokens * hidden < 2^32; quant_group a power of two
 * in [8, 2048] dividing tokens * hidden; 1 <= max_channels <= hidden. */
typedef struct adacc_channel_method {
  uint32_t bits;         /* 4 or 8                                                    */
  uint32_t quant_group;  /* Gq                                                        */
  uint32_t asym;         /* 0: Eq. 2, 1: Eq. 3                                        */
  uint32_t scale_rule;   /* ADACC_SCALE_*                                             */
  float z_thresh;        /* threshold on Z (finite)                                   */
  uint32_t max_channels; /* outlier channels the blob has room for                    */
  uint32_t dtype;        /* ADACC_DTYPE_*, as in adacc_method                         */
} adacc_channel_method;

/* Blob sections (each on a 256-byte boundary):
 *   codes, scales, zp   as in adacc_layout
 *   ch_mask  hidden/8 bytes: bit (h & 7) of byte h >> 3 is set for an outlier channel
 *   ch_base  hidden/8 uint32: number of outlier channels below channel 8 * (h >> 3)
 *   ch_idx   max_channels int32: the outlier channels, ascending
 *   ch_val   room for tokens * max_channels 16-bit values; used as [tokens][n_ch]: ch_val[t * n_ch + r] is
 *            channel ch_idx[r] of token t, bit for bit
 *   status   4 uint32: [0] n_ch, the number of outlier channels found, [1] 1 if n_ch exceeds
 *            max_channels (then only ch_mask, ch_base, the first max_channels entries of ch_idx
 *            and status are produced and the blob cannot be decompressed), [2], [3] 0. */
typedef struct adacc_channel_layout {
  uint64_t codes_off, scales_off, zp_off, ch_mask_off, ch_base_off, ch_idx_off, ch_val_off, status_off;
  uint64_t total_bytes;
} adacc_channel_layout;

/* Host only, pure.  Errors: ENULL, EINVAL. */
int adacc_channel_layout_of(const adacc_channel_method *method, uint64_t tokens, uint32_t hidden,
                            adacc_channel_layout *out);
/* Device bytes adacc_channel_compress needs as scratch space (chunk sums and S_h); 0 if the
 * sizes are not valid.  Any 256-byte aligned device buffer of that size; no initialisation, may be
 * shared by calls that follow each other on one stream. */
uint64_t adacc_channel_workspace_bytes(uint64_t tokens, uint32_t hidden);
/* Enqueues the four kernels: chunk sums, channel sums, Eq. 1 selection, quantisation of the rest
 * with extraction of the outlier channels.  src: tokens*hidden 16-bit values, 16-byte aligned, not modified.
 * tokens == 0: ADACC_OK, nothing is touched.  Errors: ENULL, EINVAL, ESIZE, EALIGN, EHIP. */
int adacc_channel_compress(const adacc_channel_method *method, const void *src, uint64_t tokens, uint32_t hidden,
                           void *blob, uint64_t blob_bytes, void *workspace, uint64_t workspace_bytes,
                           void *hip_stream);
/* Dequantisation followed by the write-back of the outlier channels (Fig. 3(c) decompression
 * workflow).  dst as in adacc_decompress.  A blob whose status[1] is set leaves dst untouched. */
int adacc_channel_decompress(const adacc_channel_method *method, const void *blob, uint64_t blob_bytes,
                             uint64_t tokens, uint32_t hidden, void *dst, int dst_dtype, void *hip_stream);
/* As adacc_read_status, for a blob of this kind. */
int adacc_channel_read_status(const void *blob, const adacc_channel_layout *layout, void *hip_stream,
                              uint32_t status_out[4]);

/* ---- channel-wise symmetric quantisation: the scheme for the Query, Key and Value matrices
 * (Section 3.2, list of layer-specific schemes) ----
 * The tensor is a row-major matrix of `tokens` rows and `hidden` channels; every channel is one
 * group of Eq. 2: S_h = max over the tokens of |x| / D, code = clip(round(x / S_h)), with D as
 * scale_rule says.  The codes keep the tensor's own order (nothing is transposed); no outliers are
 * separated; a value that is not finite counts as zero.  bits: 4 or 8.
 * Blob: codes (tokens*hidden*bits/8 bytes, packed as in adacc_layout) and scales (hidden binary32),
 * each on a 256-byte boundary.  Workspace: any 256-byte aligned device buffer of
 * adacc_channelwise_workspace_bytes (chunk maxima and reciprocals), no initialisation.
 * Limits: hidden a multiple of 8 in [8, 65536]; tokens * hidden < 2^32.
 * tokens == 0: ADACC_OK, nothing is touched.  Errors: ENULL, EINVAL, ESIZE, EALIGN, EHIP. */
typedef struct adacc_channelwise_layout {
  uint64_t codes_off, scales_off, total_bytes;
} adacc_channelwise_layout;
int adacc_channelwise_layout_of(uint32_t bits, uint64_t tokens, uint32_t hidden, adacc_channelwise_layout *out);
uint64_t adacc_channelwise_workspace_bytes(uint64_t tokens, uint32_t hidden);
int adacc_channelwise_compress(uint32_t bits, uint32_t scale_rule, uint32_t dtype, const void *src, uint64_t tokens,
                               uint32_t hidden, void *blob, uint64_t blob_bytes, void *workspace,
                               uint64_t workspace_bytes, void *hip_stream);
/* X^ = code * S_h; dst and dst_dtype as in adacc_decompress, dtype (ADACC_DTYPE_*) names the 16-bit
 * format ADACC_DST_16 stands for. */
int adacc_channelwise_decompress(uint32_t bits, uint32_t dtype, const void *blob, uint64_t blob_bytes, uint64_t tokens,
                                 uint32_t hidden, void *dst, int dst_dtype, void *hip_stream);

/* ---- dropout mask of attention layers: byte format <-> bit format, lossless (Section 3.2,
 * list of layer-specific schemes) ----
 * mask: n bytes, zero = dropped, anything else = kept (a torch.bool tensor is such an array).
 * bits: adacc_mask_packed_bytes(n) = ceil(n/8) bytes; element i is bit i % 8 of byte i / 8; the
 * unused bits of the last byte are written as zero.  Unpacking writes bytes 0 and 1.
 * Both pointers are device memory, 16-byte aligned.  n == 0: ADACC_OK, nothing is touched.
 * Errors: ENULL, EALIGN, EHIP. */
uint64_t adacc_mask_packed_bytes(uint64_t n);
int adacc_mask_pack(const void *mask, uint64_t n, void *bits, void *hip_stream);
int adacc_mask_unpack(const void *bits, uint64_t n, void *mask, void *hip_stream);

/* ---- what the policy maker consumes (Section 3.3: CRate_i in the memory constraint; Section 3.4:
 * the rate is re-evaluated while training, as the number of outliers moves) ----
 * Host only, pure.  Bytes of the blob that carry information for a tensor compressed with `method`
 * that produced n_outliers outliers: codes + scales (+ offsets) + 6 bytes per outlier + the tile
 * offsets (4 bytes per tile and one more; none for ADACC_OUTLIER_NONE); padding between sections is
 * not counted.  CRate_i = this / (2 * numel).  NOOP: 2 * numel (the tensor is retained as it is).
 * Returns 0 for a malformed method. */
uint64_t adacc_compressed_bytes(const adacc_method *method, uint64_t numel, uint64_t n_outliers);
/* The same figure for a [tokens, hidden] tensor compressed by outlier channels (Section 3.2, Eq. 1) that
 * produced n_channels of them: codes + scales (+ offsets) of the whole tensor + per outlier channel its
 * index (4 bytes) and its tokens values (2 bytes each).  The channel bitmap and prefix table are derived from the
 * indices and are not counted.  Returns 0 for a malformed method or shape. */
uint64_t adacc_channel_compressed_bytes(const adacc_channel_method *method, uint64_t tokens, uint32_t hidden,
                                        uint64_t n_channels);

/* Streams of `bytes` (a multiple of 16) per operand in the access shape of the library's tensor
 * kernels (4 KiB pieces per wavefront, full grid, non-temporal accesses): the practical HBM
 * ceiling for a given mix of reads and writes, and the calibration kernels for hardware byte
 * counters.  READ reads src_a; WRITE writes dst; COPY is dst = src_a; READ2_WRITE is
 * dst = src_a ^ src_b (two bytes read per byte written, the mix of a decompression).  Operands a
 * mix does not use may be NULL.  adacc_hbm_copy is the COPY mix.
 * Errors: EINVAL, ENULL, EALIGN, EHIP. */
#define ADACC_STREAM_READ 0
#define ADACC_STREAM_WRITE 1
#define ADACC_STREAM_COPY 2
#define ADACC_STREAM_READ2_WRITE 3
int adacc_hbm_stream(int mix, void *dst, const void *src_a, const void *src_b, uint64_t bytes, void *hip_stream);
int adacc_hbm_copy(void *dst, const void *src, uint64_t bytes, void *hip_stream);

/* Text for an error code; for ADACC_EHIP, the last HIP error string seen by this thread. */
const char *adacc_strerror(int code);

/* Library version, "major.minor". */
const char *adacc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADACC_H */
