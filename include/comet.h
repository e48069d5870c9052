/*
 * libcomet -- error-bounded lossy compression of convolution activations for
 * memory-efficient CNN training (COMET), native HIP for gfx950 (MI355X).
 *
 * The codec is the paper's "modified cuSZ" (Sec. 3.4, Sec. 4.1): quantise the
 * fp32 activations against an absolute error bound eb, predict every point from
 * its neighbours (2-D Lorenzo over each H x W plane), turn the residual into an
 * integer quantisation code, Huffman-code the codes; on decompression undo the
 * steps and re-zero every value that lies within eb of zero.  The error-bounded
 * mode guarantees |x - xhat| <= eb for every element (Sec. 2.2).
 *
 * Conventions for every entry point
 *   - "dev" pointers are device memory on the current HIP device, owned by the
 *     caller; "host" pointers are ordinary host memory.  Nothing is allocated
 *     per call: all scratch lives in the comet_ctx.
 *   - Tensors are fp32, NCHW, contiguous.  N*C*H*W must be in [1, 2^31) and
 *     W <= 8192.
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*;
 *     NULL is the default stream).  A context must not be used by two calls
 *     that can overlap in time; use one context per stream.
 *   - Return value: COMET_OK or a negative COMET_ERR_* code.  Conditions that
 *     are only known on the device (container too small, malformed container)
 *     are latched in the context and reported by the next synchronising call
 *     (comet_compress with bytes_out != NULL, or comet_sync).
 *   - NaN / Inf / huge inputs are not errors: they are stored verbatim and come
 *     back bit-identical.
 */
#ifndef COMET_H
#define COMET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COMET_OK 0
#define COMET_ERR_INVALID (-1)     /* bad argument (null pointer, zero dimension, eb or nbins out of range, ...) */
#define COMET_ERR_CAPACITY (-2)    /* the container does not fit the caller's buffer */
#define COMET_ERR_FORMAT (-3)      /* not a valid container / does not match the shape passed */
#define COMET_ERR_HIP (-4)         /* a HIP runtime call failed; see comet_strerror */
#define COMET_ERR_NOMEM (-5)       /* workspace allocation failed / context too small for the request */
#define COMET_ERR_INTERNAL (-6)    /* a device-side safety net tripped (should not happen) */
#define COMET_ERR_CODEBOOK (-7)    /* comet_compress_with_codebook: the length table is no complete prefix code, or the
                                      tensor needs an escape and the table has no code word for the escape symbol */

#define COMET_HEADER_BYTES 128u
#define COMET_DEFAULT_CHUNK_SYMS 64u

typedef struct comet_ctx comet_ctx;                     /* opaque; owns the device workspace */
typedef struct { uint32_t n, c, h, w; } comet_shape;    /* NCHW */

/* Header of a container, as returned by comet_peek (host copy). */
typedef struct {
    comet_shape shape;
    uint32_t nbins, chunk_syms, n_chunks, n_active, max_len, n_outlier_records, n_value_records;
    float eb;
    uint64_t nnz;            /* number of non-zero input elements (R of Sec. 4.2 = nnz / elements) */
    uint64_t payload_words, total_bytes;
} comet_info;

/* Create a context able to handle tensors of up to max_elems elements and
 * max_nbins quantisation bins.  Allocates 2 bytes per element plus a few MB of
 * device workspace on the current device.  *ctx is set on success. */
int comet_create(comet_ctx **ctx, uint64_t max_elems, uint32_t max_nbins);
void comet_destroy(comet_ctx *ctx);

/* Symbols per Huffman chunk for subsequent comet_compress calls: 64 (default),
 * 128 or 256.  Stored in the container; the decompressor reads it there. */
int comet_set_chunk_syms(comet_ctx *ctx, uint32_t chunk_syms);

/* Zero-chunk containers for subsequent comet_compress calls (off by default).
 * Activations behind ReLU are sparse (the ratio R of Sec. 4.2): a run of zeros,
 * like any constant run, leaves residual 0 after prediction, i.e. the centre
 * code nbins/2.  With enable != 0 a chunk that holds nothing but that code
 * takes no payload words at all (its entry in the chunk table equals the next
 * one; a chunk with symbols otherwise has at least one bit), and the container
 * says version 2 in its header; everything else, code book included, is as in
 * version 1.  The decompressor reads the version and takes either. */
int comet_set_zero_chunks(comet_ctx *ctx, int enable);

/* Worst-case container size in bytes for a shape (every element an outlier and
 * stored verbatim); 0 if the arguments are invalid.  Realistic activations need
 * a small fraction of it; callers that pass less rely on COMET_ERR_CAPACITY,
 * the paper's "unexpectedly low compression ratio" case (Sec. 3.4). */
uint64_t comet_compress_bound(comet_shape shape, uint32_t nbins, uint32_t chunk_syms);

/* Compress one activation tensor right after its layer's forward pass
 * (Sec. 3.4): dev_in (fp32, read-only) -> container at dev_out (16-byte
 * aligned, `capacity` bytes).  eb: absolute error bound, finite, in
 * [2^-100, 2^100].  nbins: even, in [4, 65536]; residuals outside
 * (-nbins/2, nbins/2) are stored as outliers.
 * bytes_out != NULL: the call synchronises `stream`, stores the container size
 * and returns any device-side error of this call (COMET_ERR_CAPACITY leaves the
 * buffer contents undefined but never writes past capacity) or, if this call
 * raised none, the first one that earlier asynchronous calls on this context
 * have latched (*bytes_out is then still this call's valid size).
 * bytes_out == NULL: fully asynchronous; the size is in the container header
 * (comet_peek) and errors are reported by comet_sync. */
int comet_compress(comet_ctx *ctx, const float *dev_in, comet_shape shape, float eb, uint32_t nbins,
                   void *stream, void *dev_out, uint64_t capacity, uint64_t *bytes_out);

/* Compress with the code book of an earlier compression of the same layer.  COMET refreshes a
 * layer's statistics only every W iterations because they change slowly (Sec. 3.1); the same holds
 * for the layer's histogram, so the histogram and the Huffman construction (Sec. 4.1) can be skipped
 * between refreshes; with the code words known beforehand the tensor is read once, every part of it
 * quantised and encoded by the same wavefront.  dev_len: device pointer to u8[nbins] code lengths (the length section of an
 * earlier container of the same nbins starts COMET_HEADER_BYTES into it); it must stay valid and
 * unchanged until the call has completed and may lie inside another container, not inside dev_out.
 * The lengths must form a complete prefix code (or one symbol of length 1), none above 57.  A
 * quantisation code without a code word in the table is stored like a residual outside the
 * alphabet (escape symbol + outlier record); the container carries the table, so it decompresses
 * with comet_decompress to exactly the values comet_compress would give.  Everything else as
 * comet_compress.  Limits: nbins <= 8192 and planes of at most 512 columns (COMET_ERR_INVALID
 * otherwise).  A table that is no such code, that lacks a code word for the escape symbol when
 * the tensor needs one, or that spends more than 16 bits per symbol on some run of rows (about
 * 2048 elements or more: the encoded run does not fit its share of the workspace; such a table
 * expands the data) raises COMET_ERR_CODEBOOK (device-side: returned here if bytes_out is given,
 * else by comet_sync); the caller then compresses in full. */
int comet_compress_with_codebook(comet_ctx *ctx, const float *dev_in, comet_shape shape, float eb, uint32_t nbins,
                                 const uint8_t *dev_len, void *stream, void *dev_out, uint64_t capacity,
                                 uint64_t *bytes_out);

/* Decompress a container for the backward pass (Sec. 3.4): dev_in (`bytes`
 * bytes, 16-byte aligned) -> dev_out (fp32, shape.n*c*h*w elements).  `shape`
 * is the shape the caller compressed; it sizes the launch and is checked on
 * the device against the header.  Asynchronous; a malformed container is
 * reported by comet_sync (the output is then undefined, never out of bounds). */
int comet_decompress(comet_ctx *ctx, const void *dev_in, uint64_t bytes, comet_shape shape,
                     void *stream, float *dev_out);

/* Activations held in 16 bits (mixed-precision training; the paper trains in fp32 and this goes
 * beyond it).  The codec itself is the fp32 one of Sec. 4.1: comet_compress_16 widens every input
 * element to fp32 as it is loaded (exact for both types) and from there on is comet_compress, so
 * the container is byte for byte the one comet_compress writes for the widened tensor, and either
 * decompression reads it.  comet_decompress_16 rounds the fp32 result of comet_decompress to the
 * 16-bit type (nearest, ties to even; after the re-zero filter), so a value differs from the
 * input by at most eb plus half a unit in the last place of the 16-bit type; verbatim values come
 * back exactly.  dtype: COMET_F16 (IEEE binary16) or COMET_BF16 (bfloat16); the tensor is device
 * memory of the 16-bit type, owned by the caller (input of comet_compress_16: 16-byte aligned, as
 * for comet_compress; output of comet_decompress_16: any element-aligned address).  Limit: planes
 * of at most 512 columns (COMET_ERR_INVALID otherwise).  Errors, `bytes_out`, streams: as for the
 * fp32 calls. */
#define COMET_F16 1
#define COMET_BF16 2
int comet_compress_16(comet_ctx *ctx, const void *dev_in, int dtype, comet_shape shape, float eb, uint32_t nbins,
                      void *stream, void *dev_out, uint64_t capacity, uint64_t *bytes_out);
int comet_decompress_16(comet_ctx *ctx, const void *dev_in, uint64_t bytes, comet_shape shape, int dtype,
                        void *stream, void *dev_out);

/* comet_decompress for callers that cannot allocate device memory or hold a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  No comet_create is needed and
 * the call allocates nothing: its control block, decode tables and work buffer live in a static device
 * array inside the library (about 8.2 MiB, held by every GPU the library runs on until the process
 * ends), which limits the tensor to COMET_STATIC_MAX_ELEMS elements (COMET_ERR_NOMEM beyond).
 * dev_in, bytes, shape, stream, dev_out: as for comet_decompress.  dev_status: device memory, one
 * int32 owned by the caller, or NULL; when the call's kernels have run it holds COMET_OK, or
 * COMET_ERR_FORMAT if the container was refused (dev_out is then undefined, never out of bounds).
 * Asynchronous, kernels only.  All calls on one GPU share the one array: calls that can overlap in
 * time on the same GPU (two streams, two threads) race; issue them on one stream. */
#define COMET_STATIC_MAX_ELEMS (4u << 20)
int comet_decompress_static(const void *dev_in, uint64_t bytes, comet_shape shape, void *stream, float *dev_out,
                            int32_t *dev_status);

/* Wait for `stream` and return (then clear) the first device-side error latched
 * in the context since the last synchronising call. */
int comet_sync(comet_ctx *ctx, void *stream);

/* Read and validate a container's header (synchronises `stream`). */
int comet_peek(comet_ctx *ctx, const void *dev_in, uint64_t bytes, void *stream, comet_info *info);

/* Adaptive error bound (Sec. 3.2, 3.3): sigma = sigma_frac * momentum_abs_mean;
 * eb = sigma / (a * loss_grad_mean * sqrt(batch * nonzero_ratio)), evaluated in
 * fp64 on the host, rounded to fp32, clamped to [eb_min, eb_max].  The paper's
 * constants are a = 0.32 (Sec. 5.2) and sigma_frac = 0.01 (Sec. 3.2).
 * loss_grad_mean == 0 or nonzero_ratio == 0 returns eb_max. */
typedef struct { double momentum_abs_mean, loss_grad_mean, nonzero_ratio; uint32_t batch; } comet_layer_stats;
typedef struct { double a, sigma_frac; float eb_min, eb_max; } comet_adapt_cfg;
void comet_adapt_defaults(comet_adapt_cfg *cfg);   /* 0.32, 0.01, 2^-100, 2^100 */
int comet_adapt_eb(const comet_layer_stats *stats, const comet_adapt_cfg *cfg /* NULL = defaults */, float *eb_out /* host */);

/* Semi-online statistic for comet_layer_stats (Sec. 3.1: the average of the momentum, the average
 * gradient of the loss; taken as means of absolute values): mean of |dev_in[i]| over n fp32 values
 * on the device, accumulated in fp64 by a fixed tree (the same result on every call).  Synchronises
 * `stream`; *mean_out is host memory.  Non-finite inputs give a non-finite mean.  The fraction of
 * non-zero activations comes with every compression (comet_info.nnz). */
int comet_abs_mean(comet_ctx *ctx, const float *dev_in, uint64_t n, void *stream, double *mean_out);

/* Active factor W (Sec. 3.1), a host-side counter: statistics are collected and the error bounds
 * re-estimated every W iterations, W = 1000 by default; after a re-estimation, if the bound of any
 * layer changed by more than 2x (in either direction) since the previous one, W is halved (not below
 * 1), else it returns to its default. */
typedef struct { uint32_t w_default, w, since; } comet_controller;
int comet_controller_init(comet_controller *c, uint32_t w_default /* 0 = 1000 */);
/* One training iteration has passed; *collect = 1 in every W-th call. */
int comet_controller_tick(comet_controller *c, int *collect);
/* After a re-estimation: eb_old / eb_new are host arrays of the n_layers bounds before and after
 * (all finite and > 0, else COMET_ERR_INVALID). */
int comet_controller_update(comet_controller *c, const float *eb_old, const float *eb_new, uint32_t n_layers);

/* ---- stage-level entry points: each runs one step of the pipeline alone so
 * ---- that it can be compared with the reference implementation ------------ */

/* Sec. 4.1 steps 1-3 fused: prequantise, Lorenzo-predict, emit codes, count the
 * histogram and compact the outlier records.
 * dev_codes: u16[elements]; dev_hist: u32[nbins]; dev_records: u32[2*rec_capacity]
 * (key, payload) pairs in ascending key order, key = 2*index + type (type 0: the
 * payload is the int32 residual of an escaped code, type 1: the fp32 bit pattern
 * of an element stored verbatim); dev_counts: u64[3] = records, value records,
 * non-zero inputs. */
int comet_stage_quantize(comet_ctx *ctx, const float *dev_in, comet_shape shape, float eb, uint32_t nbins,
                         void *stream, uint16_t *dev_codes, uint32_t *dev_hist,
                         uint32_t *dev_records, uint64_t rec_capacity, uint64_t *dev_counts);

/* Huffman code lengths (two-queue construction, leaf before internal node on
 * equal weight, leaves ordered by (frequency, symbol)) and canonical codes.
 * dev_hist: u32[nbins]; dev_len: u8[nbins]; dev_code: u64[nbins] (may be NULL).
 * The context keeps the table for a following comet_stage_encode. */
int comet_stage_codebook(comet_ctx *ctx, const uint32_t *dev_hist, uint32_t nbins, void *stream,
                         uint8_t *dev_len, uint64_t *dev_code);

/* Chunked Huffman encode with the table of the last comet_stage_codebook on
 * this context.  dev_chunk_off: u32[ceil(n/chunk_syms)] word offset of every
 * chunk; dev_payload: u32[payload_capacity_words]; dev_payload_words: u64[1]. */
int comet_stage_encode(comet_ctx *ctx, const uint16_t *dev_codes, uint64_t n, uint32_t nbins, uint32_t chunk_syms,
                       void *stream, uint32_t *dev_chunk_off, uint32_t *dev_payload,
                       uint64_t payload_capacity_words, uint64_t *dev_payload_words);

/* Chunk-parallel Huffman decode from a length table. dev_codes_out: u16[n]. */
int comet_stage_decode(comet_ctx *ctx, const uint8_t *dev_len, uint32_t nbins,
                       const uint32_t *dev_chunk_off, const uint32_t *dev_payload, uint64_t payload_words,
                       uint64_t n, uint32_t chunk_syms, void *stream, uint16_t *dev_codes_out);

/* Lorenzo reconstruction (plane-wise 2-D prefix sums), dequantisation, verbatim
 * values and the re-zero filter of Sec. 3.4, from a code array and records. */
int comet_stage_reconstruct(comet_ctx *ctx, const uint16_t *dev_codes, const uint32_t *dev_records, uint64_t n_records,
                            comet_shape shape, uint32_t nbins, float eb, void *stream, float *dev_out);

/* ---- per-kernel timing, for benchmarks ---------------------------------------
 * When enabled, every kernel the context launches is bracketed by two HIP events
 * recorded on the call's stream.  comet_profile_read waits for those events and
 * returns, for kernel `kernel_id`, the number of launches since the last
 * comet_profile_reset and their summed duration in milliseconds.  Kernel ids:
 * 0 quantize (sweep), 1 codebook, 2 encode (pack pass), 3 decode tables,
 * 4 reconstruct (scans + store; for planes wider than 512 columns the fused
 * decode + reconstruct kernel), 5 Huffman decode, 6 gather of the outlier
 * records, 7 encode (count pass), 8 decompression in one kernel (Huffman decode, reconstruction and
 * store; containers with chunks of 64 symbols and planes of at most 512 columns).
 * At most 16384 launches are kept between resets; further ones are not timed. */
#define COMET_KERNEL_QUANTIZE 0
#define COMET_KERNEL_CODEBOOK 1
#define COMET_KERNEL_ENCODE 2
#define COMET_KERNEL_TABLES 3
#define COMET_KERNEL_RECONSTRUCT 4
#define COMET_KERNEL_DECODE 5
#define COMET_KERNEL_GATHER 6
#define COMET_KERNEL_ENCODE_COUNT 7
#define COMET_KERNEL_FUSED 8
#define COMET_KERNEL_COUNT 9
int comet_profile_enable(comet_ctx *ctx, int enable);
int comet_profile_reset(comet_ctx *ctx);
int comet_profile_read(comet_ctx *ctx, uint32_t kernel_id, uint32_t *launches /* host */, double *total_ms /* host */);

/* Text for a COMET_ERR_* code; for COMET_ERR_HIP the last HIP error string seen
 * by this thread.  Never NULL. */
const char *comet_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* COMET_H */
