/*
 * kvtc.h -- C ABI of the MI355X (gfx950) KV-cache transform coder.
 *
 * The library implements the data-parallel hot path of "KV Cache Transform
 * Coding for Compact Storage in LLM Inference" (KVTC):
 *
 *   encode (paper, Section "Method", mode "Compression"; Sections "Feature
 *           decorrelation", eq. 3, and "Quantization"):
 *       d = (x - mu) V_kept            per token, bf16 matrix-core product, fp32 sums
 *       per token and per group of subsequent PCA coordinates: min-max uniform
 *       quantisation at the group's calibrated width with a shared fp16 shift
 *       and fp16 scale; coordinates with zero width are never computed;
 *       codes are bit-packed into one fixed-size record per token.
 *   decode (same Section, mode "Decompression"; eq. 3 right-hand side):
 *       unpack, d_hat = shift + code * scale, x_hat = d_hat V_kept^T + mu.
 *
 * Calibration (PCA basis, mean, bit allocation) is done elsewhere and enters
 * as data through kvtc_plan_create.  The entropy stage (DEFLATE, Section
 * "Entropy coding") is not part of this library.
 *
 * Record format (the paper only says "packed into a single byte array"):
 * a record is a little-endian bit string of R = 4*ceil((32 G + sum n_g b_g)/32)
 * bytes: G header dwords (group g: fp16 shift in bits 0-15, fp16 scale in
 * bits 16-31), then every kept coordinate's code in PCA order, width b_g,
 * least significant bit first, no gaps; zero padding to 32 bits.  A tensor's
 * stream is its records back to back in token order.
 *
 * Numerics of the code decision (both sides of any comparison must use them):
 *   lo/hi = min/max of the group's fp32 coefficients; shift = largest fp16 <= lo;
 *   scale = smallest fp16 >= (hi - shift)/(2^b - 1) (fp32 subtract and divide);
 *   code = clamp(round_half_even((d - shift) * (1/scale)), 0, 2^b - 1), each
 *   operation one fp32 operation; scale == 0 gives code 0; shift and scale
 *   saturate at +-65504.  NaN inputs give unspecified codes and never fault.
 *
 * All pointers named *_dev are device pointers, all named *_host host
 * pointers.  `stream` arguments are a hipStream_t passed as void*.
 * Every function returns a kvtc_status; kvtc_last_error() gives a
 * thread-local message for the last non-OK status.  No function throws.
 * encode/decode calls never allocate and never synchronise; they are ordered
 * on the given stream.
 */
#ifndef KVTC_H
#define KVTC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvtc_plan kvtc_plan;     /* one per (layer, K or V, compression ratio); immutable */
typedef struct kvtc_batch kvtc_batch;   /* a set of plans addressable from one batched launch   */
typedef void* kvtc_stream;              /* a hipStream_t */

typedef enum {
    KVTC_OK = 0,
    KVTC_E_ARG = 1,          /* null pointer, negative size, bad alignment, inconsistent plan   */
    KVTC_E_UNSUPPORTED = 2,  /* valid request the kernels cannot serve (see kvtc_plan_create)   */
    KVTC_E_SMALL = 3,        /* output capacity / input size below n_tokens * record bytes      */
    KVTC_E_HIP = 4,          /* a HIP runtime call failed                                        */
    KVTC_E_NOMEM = 5         /* host or device allocation failed (plan/batch creation only)     */
} kvtc_status;

typedef enum { KVTC_BF16 = 0, KVTC_F32 = 1 } kvtc_dtype;

/* A kept group: n subsequent kept PCA coordinates sharing one shift/scale, each coded on `bits` bits. */
typedef struct { uint16_t n; uint8_t bits; uint8_t reserved; } kvtc_group;

/* One tensor of a batched call.  x_row0 is the row of the job's first token in the shared
 * feature array; the job's stream starts at offsets[job] in the shared stream buffer. */
typedef struct { int32_t plan; int32_t n_tokens; int64_t x_row0; } kvtc_job;

/*
 * Build a plan (paper, Section "Method", mode "Calibration", gives the inputs:
 * mean mu, basis V trimmed to the coordinates with non-zero width, and the
 * per-group widths and sizes).
 *   p            features per token; multiple of 64
 *   r            kept coordinates, 16 <= r <= 1024
 *   mu_host      [p] fp32
 *   v_kept_host  [p][r] row-major bf16 bit patterns (column j = j-th kept coordinate)
 *   groups_host  n_groups kept groups in PCA order; sum of n must equal r
 * The arrays are copied; they may be freed when the call returns.  The call
 * allocates device memory on the current device and synchronises `stream`.
 * Errors: KVTC_E_ARG for null/inconsistent input or bits outside 1..16;
 * KVTC_E_UNSUPPORTED if a group size is not a multiple of 16 (the kernels work
 * on 16-coordinate blocks; the group sizes 16, 64, 256, 1024 all qualify) or the
 * record is too large for the kernels' on-chip staging.
 */
kvtc_status kvtc_plan_create(kvtc_plan** out, int p, int r, const float* mu_host,
                             const uint16_t* v_kept_host, int n_groups,
                             const kvtc_group* groups_host, kvtc_stream stream);
void kvtc_plan_destroy(kvtc_plan* plan);                                  /* NULL is a no-op */
size_t kvtc_record_bytes(const kvtc_plan* plan);                          /* R; 0 for NULL    */
size_t kvtc_encoded_bytes(const kvtc_plan* plan, int64_t n_tokens);       /* n_tokens * R     */

/*
 * Encode one tensor (paper, "Compression": project, quantise, pack).
 *   x_dev     [n_tokens][ld_x] elements of `dtype`, row-major, p <= ld_x <= 2^21, 16-byte
 *             aligned base and row pitch (a larger pitch is KVTC_E_ARG).  fp32 inputs are
 *             rounded to bf16 (nearest even) on load.
 *   out_dev   receives n_tokens records; 16-byte aligned; out_cap >= n_tokens * R else
 *             KVTC_E_SMALL and nothing is written.
 * n_tokens == 0 is KVTC_OK and does nothing.
 */
kvtc_status kvtc_encode(const kvtc_plan* plan, const void* x_dev, kvtc_dtype dtype,
                        int64_t n_tokens, int64_t ld_x, void* out_dev, size_t out_cap,
                        kvtc_stream stream);

/*
 * Decode one tensor (paper, "Decompression": unpack, dequantise, back-project, add mu).
 *   in_dev    n_tokens records, 16-byte aligned; in_bytes >= n_tokens * R else KVTC_E_SMALL.
 *             The kernel fetches the stream in aligned 16-byte pieces, so when a tensor's
 *             records do not end on a 16-byte boundary it also reads the rest of that last
 *             16-byte block (never beyond it; the bytes are ignored).
 *   x_out_dev [n_tokens][ld_x] of `dtype`; results are rounded to nearest even for bf16.
 */
kvtc_status kvtc_decode(const kvtc_plan* plan, const void* in_dev, size_t in_bytes,
                        int64_t n_tokens, void* x_out_dev, kvtc_dtype dtype, int64_t ld_x,
                        kvtc_stream stream);

/*
 * Batched / ragged calls: many tensors (jobs), each with its own plan and length, in
 * one launch per direction and per kernel variant among the batch's plans (plans of
 * similar rank share a variant: usually one launch; encode adds one small launch per
 * variant for the jobs of at most 64 tokens, which run on narrower tiles).  A kvtc_batch makes the plans' descriptors addressable
 * from the device; it copies what it needs, but the plans must outlive it.
 * At most 1024 jobs per call (KVTC_E_UNSUPPORTED beyond).
 */
kvtc_status kvtc_batch_create(kvtc_batch** out, const kvtc_plan* const* plans, int n_plans,
                              kvtc_stream stream);
void kvtc_batch_destroy(kvtc_batch* batch);

/*
 * Stream offsets of a ragged batch, computed on the GPU:
 *   offsets_dev[j] = sum_{i<j} jobs_dev[i].n_tokens * R(plan of job i),  j = 0..n_jobs
 * (an exclusive prefix sum; offsets_dev[n_jobs] is the total stream size).
 * jobs_dev: device array of n_jobs kvtc_job.  Jobs with a plan index outside the
 * batch or n_tokens < 0 count as empty here and are reported by the encode/decode call.
 */
kvtc_status kvtc_offsets(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                         uint64_t* offsets_dev, kvtc_stream stream);

/*
 * Encode / decode every job.  x_base_dev is the shared feature array (rows of ld_x
 * elements); job j reads/writes rows x_row0 .. x_row0 + n_tokens - 1 and the stream
 * bytes offsets_dev[j] .. offsets_dev[j] + n_tokens * R - 1 of the shared stream buffer
 * (offsets from kvtc_offsets lay the jobs back to back; kvtc_offsets_append gives each job
 * a place inside a region of its own; offsets_dev[n_jobs] is not read).
 * The host cannot see device-resident sizes without synchronising, so capacity is
 * checked on the device: a job whose bytes would not lie inside [0, cap), or whose plan
 * index / token count is invalid, is skipped entirely and *status_dev is set to
 * 1 + (index of the lowest such job); it stays 0 when every job ran.  The caller
 * zeroes *status_dev beforehand and reads it after synchronising.  Jobs must not overlap
 * in the stream buffer (not checked).
 */
kvtc_status kvtc_encode_batch(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                              const void* x_base_dev, kvtc_dtype dtype, int64_t ld_x,
                              const uint64_t* offsets_dev, void* out_base_dev, size_t out_cap,
                              uint32_t* status_dev, kvtc_stream stream);
kvtc_status kvtc_decode_batch(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                              const void* in_base_dev, size_t in_bytes,
                              const uint64_t* offsets_dev, void* x_out_base_dev,
                              kvtc_dtype dtype, int64_t ld_x, uint32_t* status_dev,
                              kvtc_stream stream);

/*
 * kvtc_encode_batch for callers that cannot allocate device memory or keep a kvtc_batch: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  One call does what
 * kvtc_batch_create + kvtc_offsets + kvtc_encode_batch do (jobs laid back to back in the stream
 * buffer) and calls no allocating routine: the plan-descriptor table and the stream offsets live in a
 * fixed work area inside the library (about 17 KB per GPU, held until the process ends).
 *   plans             host array of n_plans handles, 1 <= n_plans <= 64 (KVTC_E_UNSUPPORTED beyond);
 *                     jobs_dev[j].plan indexes it
 *   offsets_out_dev   NULL, or a device array of n_jobs + 1 entries that receives the offsets
 *                     (the same values kvtc_offsets gives), e.g. for a later kvtc_decode_batch
 * Everything else, including *status_dev and the limit of 1024 jobs, is as in kvtc_encode_batch.
 * All calls on one GPU share the work area: calls on the same stream are ordered; calls that
 * overlap on one GPU (different streams, or different threads without ordering) race and must
 * not be made.  Nothing of an earlier call is read by a later one.
 */
kvtc_status kvtc_encode_batch_static(const kvtc_plan* const* plans, int n_plans, const kvtc_job* jobs_dev,
                                     int n_jobs, const void* x_base_dev, kvtc_dtype dtype, int64_t ld_x,
                                     void* out_base_dev, size_t out_cap, uint64_t* offsets_out_dev,
                                     uint32_t* status_dev, kvtc_stream stream);

/*
 * ---- Sink tokens, sliding window, incremental coding ------------------------------------
 * (paper, Section "Sliding Windows and Sink Tokens": the s oldest and the w most recent tokens
 * are not transform-coded; Section "Experimental setup": the coder runs every c new tokens,
 * which leaves the window between w - c and w; Appendix "Compression ratio with sliding
 * window": the sinks are kept in FP8 and the ratio that counts them.)
 */

/* How a context of ctx tokens divides.  Host only, no GPU call.  A token joins the window when it
 * arrives; whenever the window holds w tokens its c oldest are coded:
 *   n_sink = min(ctx, s), n_coded = c * max(0, floor((ctx - s - (w - c)) / c)), n_window = the rest.
 * KVTC_E_ARG unless ctx >= 0, s >= 0, 1 <= c <= w. */
typedef struct { int64_t n_sink, n_coded, n_window; } kvtc_split;
kvtc_status kvtc_window_split(int64_t ctx, int s, int w, int c, kvtc_split* out);

/* ctx / ((ctx - w - s) / cr + w + s / 2): compression ratio of a context of ctx tokens of which w stay
 * in 16 bits, s in FP8 and the rest is coded at ratio cr.  Host only. */
double kvtc_cr_with_window(double ctx, double w, double s, double cr);

/*
 * Sinks to and from FP8 (OCP E4M3, one byte per value, no scale factor: the paper says "FP8" only).
 * Round to nearest, ties to the even mantissa; magnitudes from 448 up (and infinities) give +-448;
 * NaN gives 0x7f.  fp32 inputs are first rounded to bf16 like the coder's inputs.
 *   x_dev     [n_tokens][ld_x] of `dtype`, base and pitch 16-byte aligned, ld_x >= p
 *   out_dev   [n_tokens][p] bytes; out_cap >= n_tokens * p else KVTC_E_SMALL
 * Unpacking is exact (every E4M3 value is a bf16 value).  Both are ordered on `stream`, allocate
 * nothing and do not synchronise; n_tokens == 0 is a no-op.
 */
kvtc_status kvtc_fp8_pack(const void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int p, int64_t ld_x,
                          void* out_dev, size_t out_cap, kvtc_stream stream);
kvtc_status kvtc_fp8_unpack(const void* in_dev, size_t in_bytes, int64_t n_tokens, int p,
                            void* x_out_dev, kvtc_dtype dtype, int64_t ld_x, kvtc_stream stream);

/*
 * ---- Features that are not contiguous in memory ------------------------------------------
 * A token's p features may come in blocks that lie apart: the heads of a cache kept as
 * [heads][tokens][d_head], or the per-layer tensors [layers][tokens][1024] whose concatenation a
 * cross-layer basis transforms (paper, Section "Feature decorrelation": keys or values of several
 * layers and heads are concatenated before the PCA).  Feature f of token t sits at
 *     x[t * token_stride + (f / block_features) * block_stride + f % block_features]     (elements).
 *   block_features   0: contiguous features (then this is the ld_x of the plain calls); else a power
 *                    of two >= 64 that divides p
 *   token_stride     >= block_features (>= p when contiguous), at most 2^21
 *   block_stride     >= block_features
 * Base and both strides 16-byte aligned.  Blocks must lie inside a token's row or tokens inside a
 * block's slab (anything else overlaps: KVTC_E_ARG; a batched call cannot see the token counts and
 * checks block_stride >= token_stride only).  The _blocked calls are the plain calls with a layout in
 * place of ld_x; everything else is as documented there.  In a batched call x_row0 counts tokens
 * (units of token_stride) from the base.
 */
typedef struct { int64_t token_stride; int32_t block_features; int32_t reserved; int64_t block_stride; } kvtc_layout;
kvtc_status kvtc_encode_blocked(const kvtc_plan* plan, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens,
                                const kvtc_layout* layout, void* out_dev, size_t out_cap, kvtc_stream stream);
kvtc_status kvtc_decode_blocked(const kvtc_plan* plan, const void* in_dev, size_t in_bytes, int64_t n_tokens,
                                void* x_out_dev, kvtc_dtype dtype, const kvtc_layout* layout, kvtc_stream stream);
kvtc_status kvtc_encode_batch_blocked(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                                      const void* x_base_dev, kvtc_dtype dtype, const kvtc_layout* layout,
                                      const uint64_t* offsets_dev, void* out_base_dev, size_t out_cap,
                                      uint32_t* status_dev, kvtc_stream stream);
kvtc_status kvtc_decode_batch_blocked(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                                      const void* in_base_dev, size_t in_bytes, const uint64_t* offsets_dev,
                                      void* x_out_base_dev, kvtc_dtype dtype, const kvtc_layout* layout,
                                      uint32_t* status_dev, kvtc_stream stream);

/*
 * ---- Plans over the concatenated features of several layers --------------------------------
 * (paper, Section "Feature decorrelation": the keys or values of l layers and h heads are concatenated
 * into p = l * h * d_head features under ONE basis; appendix "PCA matrix sizes": that basis is cut to its
 * first 8K or 10K components before the bit allocation removes more; appendix "PCA feature concat size
 * vs performance".)  Such a plan keeps thousands of coordinates, more than one record of the coder holds,
 * so its byte layout (on which the paper is silent) is cut into SECTIONS: consecutive kept groups are
 * gathered greedily into sections of at most 1024 coordinates and 64 groups; section c is coded exactly
 * as a plan made of its groups alone, and the stream of a tensor of T tokens is the T records of section
 * 0, then the T records of section 1, ..., each section starting on a 16-byte boundary of the stream.
 * The headers and codes are those of the unsectioned method (a group's quantisation never looks outside
 * the group); decoding sums the sections' products in fp32 and adds the mean once.
 *   kvtc_wide_create  arguments as kvtc_plan_create, with r and n_groups unbounded and every group of at
 *                     most 1024 coordinates (a multiple of 16).  Host arrays may be freed on return.
 *   kvtc_wide_encode  x_dev and layout as kvtc_encode_blocked (per-layer tensors [layers][tokens][1024]
 *                     are read in place: no concatenated copy); out_dev 16-byte aligned, out_cap >=
 *                     kvtc_wide_encoded_bytes(w, n_tokens) else KVTC_E_SMALL.  One launch per section.
 *   kvtc_wide_decode  x_out_dev and layout as kvtc_decode_blocked.  For bf16 output of a plan of several sections
 *                     the caller passes sum_dev, an fp32 workspace [n_tokens][p] (16-byte aligned): all sections
 *                     but the last are summed there, and the last section's launch reads that sum, adds its own
 *                     part and rounds to bf16 ONCE; for fp32 output the sections are summed in x_out_dev itself and
 *                     sum_dev is ignored (may be null; also for a plan of one section).  Sections between the first
 *                     and the last add with hardware float adds in memory; the launches are ordered on the stream,
 *                     so every element receives its terms in section order and results are reproducible.
 * Neither call allocates or synchronises.
 */
typedef struct kvtc_wide kvtc_wide;
kvtc_status kvtc_wide_create(kvtc_wide** out, int p, int r, const float* mu_host, const uint16_t* v_kept_bf16_host,
                             int n_groups, const kvtc_group* groups_host, kvtc_stream stream);
void kvtc_wide_destroy(kvtc_wide* w);
int kvtc_wide_sections(const kvtc_wide* w);
size_t kvtc_wide_section_record_bytes(const kvtc_wide* w, int section);      /* 0 outside 0..sections-1 */
size_t kvtc_wide_record_bytes(const kvtc_wide* w);                            /* bytes per token over all sections */
size_t kvtc_wide_encoded_bytes(const kvtc_wide* w, int64_t n_tokens);         /* stream length, alignment gaps included */
kvtc_status kvtc_wide_encode(const kvtc_wide* w, const void* x_dev, kvtc_dtype dtype, int64_t n_tokens,
                             const kvtc_layout* layout, void* out_dev, size_t out_cap, kvtc_stream stream);
kvtc_status kvtc_wide_decode(const kvtc_wide* w, const void* in_dev, size_t in_bytes, int64_t n_tokens, void* x_out_dev,
                             kvtc_dtype dtype, const kvtc_layout* layout, float* sum_dev, kvtc_stream stream);

/*
 * ---- Lossless stage over the packed records --------------------------------------------------
 * (paper, Section "Entropy coding": the quantiser's byte array is passed through a lossless coder on the
 * GPU -- a general-purpose DEFLATE in the paper's implementation; appendix "Ablations of lossless
 * compression".)  This library runs a byte-wise entropy coder matched to the records' fixed layout: a
 * static prefix code PER BYTE POSITION of the record (byte k of every record -- the high byte of a group's
 * shift, the third byte of the 4-bit codes -- has a distribution of its own).  The tables are data from
 * calibration: 256 code lengths (1..12, satisfying Kraft's inequality) per position; codes are canonical
 * (by length, then by symbol) and written most significant code bit first into a bit string that fills
 * bytes from their least significant bit.  Container of a tensor's n_tokens records, little-endian:
 *     uint32 chunk_off[n_chunks + 1]   byte offset of each 64-token chunk's bit string in the payload; last: payload length
 *     uint16 len_bits[64 * n_chunks]   bits of each token's code string (0 beyond the last token)
 *     payload                          the chunks' bit strings, each zero-padded to a multiple of 4 bytes; inside a
 *                                      chunk the tokens' strings follow each other bit by bit
 *   kvtc_entropy_create   n_tables table sets (one per tensor whose records share this size), code_len_host
 *                         [n_tables][record_bytes][256]; record_bytes a multiple of 4, at most 576
 *                         (KVTC_E_UNSUPPORTED beyond).  The array may be freed on return.
 *   kvtc_entropy_bound    bytes the container of n_tokens records can reach at most.
 *   kvtc_entropy_encode   records_dev: n_tokens records back to back (4-byte aligned), coded with table set `table`.
 *                         out_dev 4-byte aligned; out_cap must hold at least the directory (else KVTC_E_SMALL);
 *                         with out_cap >= kvtc_entropy_bound nothing can be cut short, otherwise chunks that would
 *                         end beyond out_cap are left unwritten.  *out_bytes_dev (device, 8-byte aligned) receives
 *                         the container's length -- compare it with out_cap after synchronising.  Three launches.
 *   kvtc_entropy_decode   in_dev/in_bytes: a container; records_out_dev: n_tokens * record_bytes bytes
 *                         (out_cap smaller: KVTC_E_SMALL).  Reads are clamped to in_bytes: a damaged container
 *                         gives wrong bytes, never a fault.
 *   the _batch calls      many tensors in the same launches (three for encode, one for decode).  jobs_dev is a
 *                         device array (8-byte aligned): table set, token count (at most max_tokens, the host's
 *                         bound for sizing the launch), the byte offset of the job's records from records_base_dev,
 *                         of its container from coded_base_dev, and coded_cap = the room for the container
 *                         (encode) or the container's length (decode); offsets 4-byte aligned.  The host cannot see
 *                         the table, so a job that is out of range in any way (table, token count, an extent beyond
 *                         records_bytes / coded_cap, no room for its directory) is left alone by every launch and,
 *                         in encode, gets coded_bytes_dev[job] = all ones; other jobs get their container's length.
 *                         At most 65535 jobs per call.
 * No call allocates or synchronises.
 */
typedef struct kvtc_entropy kvtc_entropy;
typedef struct { int32_t table; int32_t n_tokens; uint64_t records_off; uint64_t coded_off; uint64_t coded_cap; } kvtc_entropy_job;
kvtc_status kvtc_entropy_create(kvtc_entropy** out, int record_bytes, int n_tables, const uint8_t* code_len_host, kvtc_stream stream);
void kvtc_entropy_destroy(kvtc_entropy* e);
size_t kvtc_entropy_bound(const kvtc_entropy* e, int64_t n_tokens);
kvtc_status kvtc_entropy_encode(const kvtc_entropy* e, int table, const void* records_dev, int64_t n_tokens, void* out_dev,
                                size_t out_cap, uint64_t* out_bytes_dev, kvtc_stream stream);
kvtc_status kvtc_entropy_decode(const kvtc_entropy* e, int table, const void* in_dev, size_t in_bytes, int64_t n_tokens,
                                void* records_out_dev, size_t out_cap, kvtc_stream stream);
kvtc_status kvtc_entropy_encode_batch(const kvtc_entropy* e, const kvtc_entropy_job* jobs_dev, int n_jobs, int64_t max_tokens,
                                      const void* records_base_dev, size_t records_bytes, void* coded_base_dev, size_t coded_cap,
                                      uint64_t* coded_bytes_dev, kvtc_stream stream);
kvtc_status kvtc_entropy_decode_batch(const kvtc_entropy* e, const kvtc_entropy_job* jobs_dev, int n_jobs, int64_t max_tokens,
                                      const void* coded_base_dev, size_t coded_bytes, void* records_base_dev, size_t records_cap,
                                      kvtc_stream stream);

/*
 * ---- Calibration: the error table of the bit allocation ----------------------------------------
 * (paper, Section "Quantization" and appendix "Dynamic programming algorithm": the dynamic programme
 * chooses, per block of subsequent PCA coordinates, a quantiser type by the error it causes on the
 * calibration data.)  Computes, for every candidate block (start, n) and every width b = 1..max_bits, the
 * change of the squared error against dropping the block,
 *     change[block][b - 1] = sum over tokens t and coordinates j of the block of (d - d_hat)^2 - d^2,
 * where d_hat is d after the coder's own quantiser at width b (shared fp16 shift rounded down and scale
 * rounded up per token and block, code decided in fp32, exactly as kvtc_encode decides it).  The heavy
 * part of calibration after the PCA: every (block, width) pair is a pass over the calibration tokens.
 *   coef_dev    [n_tokens][ld] fp32: the calibration coefficients P = (C - mu) V (device, 4-byte aligned)
 *   blocks_dev  n_blocks x {start, n} (device): 1 <= n <= 1024, start + n <= ld; a block outside these
 *               limits gets NaN in its row of the result (the list is not visible to the host)
 *   change_dev  [n_blocks][max_bits] fp64 (device, 8-byte aligned); max_bits in 1..8
 * One workgroup per block with fixed summation order: results are reproducible.  No allocation, no
 * synchronisation.  The PCA itself (an eigen-decomposition of a p x p matrix) is not part of this library.
 */
typedef struct { int32_t start; int32_t n; } kvtc_calib_block;
kvtc_status kvtc_calib_block_errors(const float* coef_dev, int64_t n_tokens, int64_t ld, const kvtc_calib_block* blocks_dev,
                                    int n_blocks, int max_bits, double* change_dev, kvtc_stream stream);

/*
 * Calibration: the one pass over the calibration tokens that the PCA needs (paper, Section "Feature
 * decorrelation", eq. 2: the mean and the SVD of the centred calibration matrix C - mu; the right singular
 * vectors are the eigenvectors of the centred second-moment matrix).  Computes, in double precision and
 * with a fixed summation order (token by token),
 *     sum_dev[f]      = sum over tokens of x[t][f]
 *     gram_dev[f][g]  = sum over tokens of x[t][f] * x[t][g]          (all p x p entries)
 * from which the caller forms mu = sum / n and the covariance gram / n - mu mu^T and decomposes it on the
 * host (a p x p eigen-problem, not part of this library).
 *   x_dev, dtype, layout  the calibration tokens as kvtc_encode_blocked takes them (per-layer tensors or
 *                         heads-major caches in place); p a multiple of 64
 *   sum_dev [p], gram_dev [p][p]  device, 8-byte aligned
 * No allocation, no synchronisation.
 */
kvtc_status kvtc_calib_moments(const void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int p, const kvtc_layout* layout,
                               double* sum_dev, double* gram_dev, kvtc_stream stream);

/*
 * ---- Positional rotation of keys ----------------------------------------------------------
 * (paper, Section "Feature decorrelation": the rotary positional embedding is removed from keys
 * before they are transform-coded, because it hides their low-rank structure, and decoded keys are
 * rotated again.)  kvtc_rope rotates a key tensor in place: inside every head the features are
 * paired, and the pair (a, b) of the token at position m becomes
 *     a' = a cos(m theta_j) - b sin(m theta_j),  b' = a sin(m theta_j) + b cos(m theta_j),
 *     theta_j = base^(-2 j / d_head),  j = 0 .. d_head/2 - 1;
 * inverse = 1 turns by the opposite angle (undoes it).  A cache of rotated keys is coded as
 * kvtc_rope(inverse = 1) then kvtc_encode, and read back as kvtc_decode then kvtc_rope(inverse = 0).
 *   x_dev           element (token t, head h, feature f) at x_dev[t * token_stride + h * head_stride + f];
 *                   token-major tensors [T][H * d_head] have head_stride = d_head, head-major caches
 *                   [H][T][d_head] have token_stride = d_head and head_stride = T * d_head.  Overlapping
 *                   strides give KVTC_E_ARG.  d_head even, at most 256.
 *   positions_dev   NULL (token t sits at position0 + t) or a device array of n_tokens positions
 *   pairing         which features form pair j: a convention of the model's code, not of the method
 * Angles, sines, cosines and the rotation are computed in double precision and the result is rounded
 * once (nearest even) to dtype.  Ordered on `stream`, allocates nothing, does not synchronise;
 * n_tokens == 0 is a no-op.
 */
typedef enum { KVTC_ROPE_HALF = 0 /* (j, j + d_head/2) */, KVTC_ROPE_INTERLEAVED = 1 /* (2j, 2j + 1) */ } kvtc_rope_pairing;
kvtc_status kvtc_rope(void* x_dev, kvtc_dtype dtype, int64_t n_tokens, int n_heads, int d_head,
                      int64_t token_stride, int64_t head_stride, const int32_t* positions_dev,
                      int64_t position0, double base, kvtc_rope_pairing pairing, int inverse,
                      kvtc_stream stream);

/*
 * Stream offsets for appending to caches that each own a region of the stream buffer, computed on
 * the GPU:  offsets_dev[j] = region_dev[j] + n_coded_dev[j] * R(plan of job j),  j < n_jobs, and
 * offsets_dev[n_jobs] = region_dev[n_jobs].  region_dev has n_jobs + 1 ascending entries (byte
 * offsets of the regions and the end of the last one), n_coded_dev[j] is the number of records
 * region j already holds and jobs_dev[j].n_tokens the number about to be added.  A job whose region
 * has no room for them (or whose entry is invalid) gets the offset 2^64 - 1, which
 * kvtc_encode_batch reports through *status_dev like any job that does not fit.
 */
kvtc_status kvtc_offsets_append(const kvtc_batch* batch, const kvtc_job* jobs_dev, int n_jobs,
                                const uint64_t* region_dev, const int64_t* n_coded_dev,
                                uint64_t* offsets_dev, kvtc_stream stream);

/* Thread-local text for the last non-OK status returned on this thread (static storage). */
const char* kvtc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KVTC_H */
