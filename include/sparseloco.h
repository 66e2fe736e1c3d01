/*
 * sparseloco.h - C ABI of the MI355X (gfx950) SparseLoCo compress + aggregate library.
 *
 * The library implements, for a list of fp32 tensors that live in flat device
 * arenas, the two communication-side blocks of SparseLoCo's outer step
 * (arXiv 2508.15706, Algorithm 1 and Eq. (2)):
 *
 *   compress   (Algorithm 1, "Compression + Error Feedback"; Eq. (2) lines 1-2)
 *       a = beta * e + delta ;  payload = Q(Top-k(a)) ;  e = a - dequantised payload
 *   aggregate  (Algorithm 1, "Aggregate + Outer Update"; Eq. (2) lines 3-4)
 *       theta = theta - lr * (1/R) * sum_r dequantised payload_r
 *
 * Top-k is chunk-wise (Section 3.3, last paragraph): 64x64 blocks of a 2-D
 * tensor, runs of 4096 elements of a 1-D tensor, k largest |a| per chunk.  Q is
 * the 2-bit statistical quantizer of Section 4 (per tensor: centre by the mean,
 * four uniform bins over [-6 sigma, 6 sigma], per-bin centroid look-up table).
 * Indices travel as 12-bit fields, or Rice-coded (appendix "Compression of indices in
 * Top-k"): sl_compress_coded / sl_decompress_avg_apply_coded.
 *
 * Conventions for every function
 *   - returns SL_OK (0) or a negative sl_status; never throws, never aborts;
 *   - arguments are validated on the host before anything is enqueued; on an
 *     argument error nothing is launched and no buffer is touched;
 *   - "device" pointers are HIP device memory of the device that was current
 *     when the plan was created; "host" pointers are ordinary host memory;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream);
 *     kernels are enqueued on it and the call returns without synchronising;
 *   - the caller owns every buffer it passes; the library owns only sl_plan.
 *   - results are deterministic: the same inputs give the same bytes;
 *   - no environment variable is read; the one tuning knob is a field of the plan
 *     (sl_plan_set_codes_wave_below).
 */
#ifndef SPARSELOCO_H
#define SPARSELOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SL_OK = 0,
    SL_ERR_INVALID_ARG = -1, /* null / misaligned pointer, bad k, R or shape        */
    SL_ERR_BAD_PAYLOAD = -2, /* sl_payload_validate found a malformed record        */
    SL_ERR_HIP = -3,         /* a HIP runtime call failed; see sl_last_hip_error()  */
    SL_ERR_NOMEM = -4,       /* host or device allocation failed (plan creation)    */
    SL_ERR_DEVICE = -5,      /* current device differs from the plan's device       */
    SL_ERR_TOO_LARGE = -6    /* sl_compress_noalloc: the plan needs more scratch
                                than SL_NOALLOC_SCRATCH_BYTES                      */
} sl_status;

enum { SL_LAYOUT_FLAT = 0,    /* chunks are runs of 4096 consecutive elements      */
       SL_LAYOUT_TILE64 = 1 };/* chunks are 64x64 blocks of the row-major matrix   */

/* flags of sl_compress */
enum { SL_COMPRESS_DEFAULT = 0,
       SL_COMPRESS_EF_FROZEN = 1, /* appendix "Freezing Error Feedback": the buffer
                                     is neither used nor accumulated, i.e. a = delta
                                     and e is left untouched                       */
       SL_COMPRESS_DEFER_RESIDUAL = 2 /* leave e = a: the subtraction of the sent
                                     values (Eq. (2) line 2) stays pending and is
                                     folded into the next call, see sl_compress   */ };

enum { SL_CHUNK = 4096, SL_MAX_WORKERS = 64 };

/* One tensor of the list: row-major rows x cols fp32 at element `offset` of the
 * arenas (a 1-D tensor is rows = 1).  offset must be a multiple of 4 elements
 * (16 bytes).  Chunks are numbered tensor by tensor; inside a TILE64 tensor
 * row-major over the block grid with local index j = 64*row_in_block +
 * col_in_block; inside a FLAT tensor j is the position in the run.  Edge chunks
 * are partial: positions outside the tensor are never candidates; every chunk
 * must still hold at least k elements. */
typedef struct {
    int64_t rows, cols, offset;
    int32_t layout;
    int32_t reserved; /* must be 0 */
} sl_tensor;

typedef struct sl_plan sl_plan; /* opaque: chunk work list and per-tensor tables */

/* Builds the work list for a tensor list and a per-chunk k (Section 3.3:
 * chunk-wise Top-k with a fixed k per chunk, density k/4096).  `tensors` is a
 * host array, copied.  k must be a multiple of 4 with 4 <= k <= 4096.  Limits:
 * rows*cols <= 2^46 per tensor, cols <= 2^23 for a TILE64 tensor, at most 2^27
 * chunks in the whole list (more than 288 GB of HBM can hold).  Allocates
 * small device tables on the current device (freed by sl_plan_destroy).
 * Errors: INVALID_ARG (shape, alignment, overlap, a chunk with fewer than k
 * elements), NOMEM, HIP. */
int sl_plan_create(const sl_tensor *tensors, int n_tensors, int k, sl_plan **out);
int sl_plan_destroy(sl_plan *plan);
/* Tuning knob of the code kernel of sl_compress* (Section 4 set-up: the 2-bit codes): lists of
 * fewer than `n_chunks` chunks give a chunk to a wavefront instead of a lane at any k (a lane
 * per chunk leaves most of the chip idle on a short list).  Default 32768.  The bytes written are
 * the same either way; takes effect at the next call on the plan. */
int sl_plan_set_codes_wave_below(sl_plan *plan, int64_t n_chunks);

/* sl_plan_create for another value width (the ablation "Effect of quantization
 * on loss": 1-, 2-, 3- and 4-bit values and full precision).  value_bits is
 * 1, 2, 3 or 4 - the quantizer of Section 4 with 2^bits uniform bins over
 * [-6 sigma, 6 sigma]: bin q covers [c_q, c_(q+1)) sigma around the mean with
 * c_j = 12 j / 2^bits - 6, end bins open-ended, per-bin centroid table - or 32:
 * the selected fp32 values travel unquantized and the error update leaves an
 * exact zero at every sent position.  Every other call works on such a plan
 * with the sizes and formats that follow from its width.  Wire format: per
 * tensor a header of 2^bits floats padded with zeros to 16 bytes (no header at
 * 32), then per chunk the k 12-bit indices followed by the k codes as a
 * little-endian stream of bits-wide fields, or by the k fp32 values; a record
 * is 3k/2 + k*bits/8 bytes.  k must be a multiple of 8 unless value_bits is 2.
 * value_bits = 2 is sl_plan_create. */
int sl_plan_create_bits(const sl_tensor *tensors, int n_tensors, int k, int value_bits, sl_plan **out);
int sl_plan_value_bits(const sl_plan *plan);       /* 1, 2, 3, 4 or 32; -1 for NULL   */

int64_t sl_plan_num_chunks(const sl_plan *plan);   /* chunks in the whole list        */
int64_t sl_plan_num_elements(const sl_plan *plan); /* sum of rows*cols                */
/* Size of one worker's payload:  sum over tensors of align16(16 + chunks*7k/4).
 * Wire format: per tensor, at a 16-byte aligned offset, float LUT[4] (little
 * endian) and then one record per chunk: the k selected local indices in
 * ascending order as a little-endian stream of 12-bit fields, then the k 2-bit
 * codes, four per byte, entry m in bits 2*(m mod 4).  Padding bytes are zero. */
size_t sl_payload_bytes(const sl_plan *plan);
/* Byte offset of tensor `t`'s block inside a payload, or (size_t)-1. */
size_t sl_payload_tensor_offset(const sl_plan *plan, int t);
/* Size of the scratch buffer sl_compress needs (selected values and partial
 * sums of the quantizer statistics).  Contents are undefined between calls. */
size_t sl_workspace_bytes(const sl_plan *plan);

/* Compression + error feedback (Algorithm 1, compression block; Eq. (2)):
 *   a = fma(beta, e, delta) in fp32; per chunk the k largest |a| (ties: lowest
 *   local index); per tensor the 2-bit quantizer over its selected values
 *   (fp64 statistics, fixed summation tree); payload written in the wire
 *   format; e <- a - LUT[code] at the selected positions, e <- a elsewhere.
 * e        inout, device, fp32 arena, 16-byte aligned
 * delta    in,    device, fp32 arena, 16-byte aligned, must not alias e
 * flags    SL_COMPRESS_DEFAULT, SL_COMPRESS_EF_FROZEN or SL_COMPRESS_DEFER_RESIDUAL
 * pending  in, device, or NULL: the payload of the previous call on this e if
 *          that call was made with SL_COMPRESS_DEFER_RESIDUAL.  Its values are
 *          subtracted from e while e is read (e_true = e - LUT[code] at its
 *          positions), so the error update of the previous round costs no
 *          scattered pass over e.  Must not be `payload`; 16-byte aligned.
 * payload  out,   device, sl_payload_bytes() bytes, 16-byte aligned
 * workspace       device, sl_workspace_bytes() bytes, 256-byte aligned
 * With SL_COMPRESS_DEFER_RESIDUAL the call leaves e = a everywhere; the true
 * error buffer of Eq. (2) is then e minus the dequantised `payload`, which the
 * caller obtains by passing `payload` as `pending` to the next call or by
 * sl_residual_apply.  Results (payloads, and e once nothing is pending) are
 * bit-identical between the two modes.  EF_FROZEN excludes both `pending` and
 * DEFER_RESIDUAL.  Elements of the arenas that belong to no tensor are neither
 * read nor written. */
int sl_compress(sl_plan *plan, float *e, const float *delta, float beta, int flags,
                const void *pending, void *payload, void *workspace, void *stream);

/* sl_compress for callers that cannot allocate device memory or bring a
 * workspace of their own: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The scratch that sl_compress takes from its
 * `workspace` argument lives in a device array inside the library,
 * SL_NOALLOC_SCRATCH_BYTES per GPU, held from the moment the library is loaded
 * until the process ends.  The call itself allocates and frees nothing, on the
 * host or on the device, and launches the same kernels as sl_compress: payload
 * and e are bit-identical to sl_compress's.
 * Arguments and errors as sl_compress (no `workspace`), and in addition
 *   SL_ERR_TOO_LARGE  sl_workspace_bytes(plan) > SL_NOALLOC_SCRATCH_BYTES
 *                     (64 MiB: lists of up to about 200,000 chunks at k = 64);
 *                     nothing is launched.
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's
 * contents; nothing in it has to be cleared between calls (each section is
 * written before it is read).  Two calls whose kernels may overlap on one GPU -
 * two streams, two threads, two plans - race on it: keep such calls on one
 * stream, or give the others a workspace of their own through sl_compress. */
enum { SL_NOALLOC_SCRATCH_BYTES = 64 * 1024 * 1024 };
int sl_compress_noalloc(sl_plan *plan, float *e, const float *delta, float beta, int flags,
                        const void *pending, void *payload, void *stream);

/* sl_compress with the pseudo-gradient formed on the fly (Section 3.1 and
 * Algorithm 1, "Pseudo-gradient": delta = theta_outer - theta_local, the
 * parameters before and after the worker's H inner steps): one fp32 subtraction
 * per element inside the accumulate pass, so delta never exists in memory.
 * theta_outer, theta_local: in, device, fp32 arenas, 16-byte aligned, distinct
 * from each other and from e.  Everything else as sl_compress. */
int sl_compress_params(sl_plan *plan, float *e, const float *theta_outer, const float *theta_local,
                       float beta, int flags, const void *pending, void *payload, void *workspace,
                       void *stream);

/* sl_compress with Random-k in place of Top-k (the ablation "SparseLoCo with
 * Random-k vs. Top-k sparsification": k randomly chosen positions per chunk,
 * "for the same number of indices selected").  The k-subset of a chunk is a
 * function of (seed, index of the chunk in the list) alone - every position
 * gets the key fmix32(fmix32(fmix32(seed) ^ chunk) ^ j) >> 1 (fmix32 = the
 * 32-bit finalizer of MurmurHash3) and the k largest keys are taken, ties to
 * the lower index - so a caller draws a fresh seed per round and worker.
 * Everything else (flags, pending, quantizer, error update, payload) as
 * sl_compress. */
int sl_compress_random_k(sl_plan *plan, float *e, const float *delta, float beta, int flags,
                         const void *pending, void *payload, void *workspace, uint32_t seed, void *stream);

/* The error update on its own (Eq. (2) line 2, second half; Algorithm 1 error
 * update): e[i] <- e[i] - LUT[code] at the positions `payload` transmits.  Ends
 * a chain of SL_COMPRESS_DEFER_RESIDUAL calls (e.g. before a checkpoint).
 * e inout device arena; payload in device, a payload of this plan. */
int sl_residual_apply(sl_plan *plan, float *e, const void *payload, void *stream);

/* Aggregate + outer update (Algorithm 1, aggregation block; Eq. (2) lines 3-4):
 *   per chunk a zero fp32 accumulator, workers added in the order r = 0..R-1
 *   (acc[j] += LUT_r[code]), then theta = fma(-lr, acc * (1/R), theta) for every
 *   element of the chunk; a coordinate a worker did not send counts as zero.
 * theta    inout, device, fp32 arena, 16-byte aligned
 * payloads in, HOST array of R DEVICE pointers, each a payload of this plan,
 *          16-byte aligned; read only during the call's kernels
 * R        1..SL_MAX_WORKERS
 * Indices in a payload are trusted to be < 4096 (they are 12-bit by format) and
 * to lie inside the tensor; payloads produced by sl_compress always do. */
int sl_decompress_avg_apply(sl_plan *plan, float *theta, const void *const *payloads, int R,
                            float lr, void *stream);

/* ---- Outer steps of the DiLoCo family (Eq. (1); Section 3.2; appendix "Exact
 * algorithmic description of DiLoCo variants").  SparseLoCo is built up from
 * these and compared with them; they reuse the chunk-wise Top-k and the sparse
 * aggregate above - on a 32-bit plan, since these variants have no quantizer -
 * and add the dense steps below.  Every "c*y + z" is one fp32 fused
 * multiply-add; only elements that belong to a tensor of the plan are touched;
 * all buffers are device fp32 arenas, 16-byte aligned.
 *   DiLoCo (Eq. (1))        sl_dense_avg_apply(theta, momentum, {delta_r})
 *   DiLoCo-LOM              sl_lom_direction per worker, then
 *                           sl_dense_avg_apply(theta, NULL, {dir_r})
 *   DiLoCo-LOM-Sub-k        the same, then sl_sub_topk(m_r) per worker
 *   DiLoCo+Top-k[+EF]       sl_compress (EF: beta = the EF decay; no EF:
 *                           SL_COMPRESS_EF_FROZEN), then
 *                           sl_decompress_avg_apply_nesterov
 *   DiLoCo-LOM+Top-k[+EF]   sl_lom_direction, sl_compress of dir, then
 *                           sl_decompress_avg_apply                          */

/* Local outer momentum and local Nesterov direction of one worker (Section 3.2):
 *   m <- mu*m + delta ;  dir <- delta + mu*m.
 * m inout; delta in; dir out, may be the same buffer as delta; m must be
 * distinct from both. */
int sl_lom_direction(sl_plan *plan, float *m, const float *delta, float mu, float *dir, void *stream);

/* Dense aggregate and outer step: avg = (1/R) * sum_r dirs[r], an fp32
 * accumulator that starts at +0.0f and adds the buffers in the order r = 0..R-1,
 * times 1/R rounded once.
 *   momentum == NULL: theta <- theta - lr*avg (last lines of the LOM outer step;
 *                     with the raw pseudo-gradients: plain averaging)
 *   momentum != NULL: Eq. (1): m <- mu*m + avg ; d <- avg + mu*m ;
 *                     theta <- theta - lr*d.
 * dirs: HOST array of R DEVICE pointers (1 <= R <= SL_MAX_WORKERS), distinct
 * from theta and momentum. */
int sl_dense_avg_apply(sl_plan *plan, float *theta, float *momentum, const float *const *dirs, int R,
                       float lr, float mu, void *stream);

/* sl_decompress_avg_apply followed by DiLoCo's global Nesterov momentum
 * (appendix algorithm "Outer step for DiLoCo+Top-k[+EF]"), in the same pass:
 *   avg as in sl_decompress_avg_apply ; m <- mu*m + avg ; d <- avg + mu*m ;
 *   theta <- theta - lr*d at EVERY element (the momentum is dense).
 * momentum inout, distinct from theta. */
int sl_decompress_avg_apply_nesterov(sl_plan *plan, float *theta, float *momentum,
                                     const void *const *payloads, int R, float lr, float mu, void *stream);

/* DiLoCo-LOM-Sub-k (Section 3.2): m <- m - Top-k(m) with the plan's chunk-wise
 * Top-k (same magnitude order and tie rule as sl_compress): the k selected
 * entries of every chunk become +0.0f, nothing else is written. */
int sl_sub_topk(sl_plan *plan, float *m, void *stream);

/* Checks a received payload before it is trusted by sl_decompress_avg_apply:
 * in every record the k indices must be strictly ascending and must address
 * positions inside the chunk (edge chunks are partial).  This call WAITS for
 * the stream (it returns a verdict): SL_OK or SL_ERR_BAD_PAYLOAD.
 * workspace: device, >= 256 bytes, 256-byte aligned (its first word is used). */
int sl_payload_validate(sl_plan *plan, const void *payload, void *workspace, void *stream);

/* The record encoder of the wire format on its own (appendix "Compression of
 * indices in Top-k": 12-bit indices + 2-bit values): for each of n_chunks
 * chunks, k ascending indices (< 4096) and k codes (0..3) -> one 7k/4-byte
 * record; records are written back to back, without LUT headers.
 * idx    in, device, uint16[n_chunks*k]
 * codes  in, device, uint8[n_chunks*k]
 * out    out, device, n_chunks*7k/4 bytes
 * No alignment is required beyond that of the element types (4-byte aligned
 * `codes` and `out` take a faster route when k is a multiple of 16; the bytes
 * written are the same).  Only the low 12 bits of an index and the low bits of a
 * code are used. */
int sl_pack_indices(const uint16_t *idx, const uint8_t *codes, int64_t n_chunks, int k, void *out,
                    void *stream);
/* The same for the other value widths of sl_plan_create_bits: codes (values
 * below 2^value_bits) for value_bits 1..4, or `values` (device, float
 * [n_chunks*k]) for value_bits 32; the unused one may be NULL.  Records are
 * 3k/2 + k*value_bits/8 bytes, back to back. */
int sl_pack_indices_bits(const uint16_t *idx, const uint8_t *codes, const float *values,
                         int64_t n_chunks, int k, int value_bits, void *out, void *stream);

/* ---- The coded wire format (appendix "Compression of indices in Top-k": the indices of a
 * payload travel compressed - the paper names its coder, "sub-chunking and Rice coding", and
 * the rates it reaches, 8.9 / 6.6 / 5.6 bits per index at k = 32 / 128 / 256, but not the
 * algorithm, so the format is this library's own; it reaches 8.8 / 6.6 / 5.5).
 *
 * Format "SLRICE02".  A chunk's ascending indices are coded as gaps g_0 = idx_0,
 * g_i = idx_i - idx_(i-1) - 1, each a Rice code with parameter b = floor(log2(2839 / k))
 * (0 when 2839 / k < 1), whose two halves are stored apart: the remainders (b low bits of g_i)
 * as k fields at fixed places, the quotients g_i >> b in unary - q_i one-bits, a zero bit -
 * back to back as one bit vector of k + Q bits per chunk (Q = sum of the quotients).  Bits fill
 * bytes LSB first.  Buffer:
 *   "SLRICE02", uint64 total bytes (little endian);
 *   per tensor, at a 16-byte aligned offset that follows from the list alone:
 *     the table header of the plain format (sl_plan_create_bits);
 *     directory, one entry per 16 consecutive chunks: uint32 offset of the group's run of bit
 *       vectors in 4-byte words from the start of the quotient section, then the 16 chunks' Q,
 *       one byte each when (4096 - k) >> b < 256, else two (unused fields 0);
 *     fixed records, one per chunk: the k remainders padded to 4 bytes, the k value fields as
 *       they stand in the plain record, padded to 4 bytes;
 *     zero padding to 16 bytes;
 *   quotient section: per group one run - its chunks' bit vectors back to back, zero-padded to
 *     4 bytes - in list order; zero padding to 16 bytes.
 * Everything but the section lies at offsets that sl_coded_fixed_bytes() bounds; the total
 * size varies with the data, at most sl_rice_max_bytes(), which is 0 for a list so long that
 * run offsets could pass 2^32 words (every coded call then returns INVALID_ARG).
 *
 * sl_compress_coded: sl_compress that ALSO emits the payload in the coded format, in the same
 *   kernels - no pass reads the plain payload back.
 *   record    out, device, sl_payload_bytes(): the payload in the plain format.  It stays with
 *             the worker: it is what `pending` of the next call takes (deferred error update)
 *             and what sl_residual_apply takes; it need not travel.
 *   coded     out, device, 16-byte aligned, capacity >= sl_rice_max_bytes() (else INVALID_ARG).
 *             When the stream work has completed, bytes 8..15 hold the coded size as a little
 *             endian uint64; only that many bytes travel.
 *   e, delta, beta, flags, pending, workspace: as sl_compress.
 * sl_decompress_avg_apply_coded (and _nesterov_coded): the aggregate and outer step of
 *   sl_decompress_avg_apply (sl_decompress_avg_apply_nesterov) over R coded payloads, decoded
 *   inside the kernel: theta is bit-identical to the plain call on the decoded payloads.
 *   coded        HOST array of R DEVICE pointers, 16-byte aligned
 *   coded_bytes  HOST array of the R buffers' sizes (>= sl_coded_fixed_bytes(), else
 *                INVALID_ARG).  No read leaves [coded[r], coded[r] + coded_bytes[r]); a
 *                malformed payload gives indices clamped into the chunk, never a fault.
 *                Any bound from the coded size up to the buffer's capacity will do: a caller
 *                that cannot read the size word back (stream capture) passes the capacity.
 * sl_rice_encode: payload (plain format, device) -> coded buffer `out` (device, 16-byte
 *   aligned, capacity >= sl_rice_max_bytes(), else INVALID_ARG): the same bytes as
 *   sl_compress_coded writes.  Indices of a record that are not strictly ascending are coded as
 *   if each repeated or descending one followed its predecessor directly (gap 0); nothing is
 *   written outside `out`.  `workspace`: device, sl_workspace_bytes() bytes, 256-byte aligned.
 * sl_rice_decode: coded buffer `in` of `in_bytes` bytes (device, 16-byte aligned) -> payload in
 *   the plain format, every byte written; reads bounded as above.  Lossless both ways, at every
 *   value width of sl_plan_create_bits. */
size_t sl_rice_max_bytes(const sl_plan *plan);
size_t sl_coded_fixed_bytes(const sl_plan *plan);
int sl_compress_coded(sl_plan *plan, float *e, const float *delta, float beta, int flags,
                      const void *pending, void *record, void *coded, size_t coded_capacity,
                      void *workspace, void *stream);
int sl_decompress_avg_apply_coded(sl_plan *plan, float *theta, const void *const *coded,
                                  const size_t *coded_bytes, int R, float lr, void *stream);
int sl_decompress_avg_apply_nesterov_coded(sl_plan *plan, float *theta, float *momentum,
                                           const void *const *coded, const size_t *coded_bytes, int R,
                                           float lr, float mu, void *stream);
int sl_rice_encode(sl_plan *plan, const void *payload, void *out, size_t out_capacity,
                   void *workspace, void *stream);
int sl_rice_decode(sl_plan *plan, const void *in, size_t in_bytes, void *payload, void *stream);

/* Per-kernel timing for benchmarks.  Between sl_profile_begin and
 * sl_profile_end every sl_compress / sl_decompress_avg_apply call on the plan
 * records HIP events on its stream around each of its kernels (no
 * synchronisation; at most `max_calls` calls of each kind are recorded, later
 * ones run unrecorded).  sl_profile_end waits for the recorded events and
 * writes, per phase, the mean milliseconds per call into ms[SL_PROF_PHASES] and
 * the number of calls averaged into calls[SL_PROF_PHASES]; either may be NULL.
 * A phase's time runs from the end of the previous kernel on the stream to the
 * end of its own, so it includes the launch gap before it. */
enum { SL_PROF_SELECT = 0,  /* accumulate + chunk Top-k          (sl_compress)   */
       SL_PROF_STATS = 1,   /* per-tensor mean / variance                        */
       SL_PROF_CODES = 2,   /* 2-bit codes + record codes                        */
       SL_PROF_LUT = 3,     /* per-tensor centroids                              */
       SL_PROF_RESIDUAL = 4,/* e <- a - LUT[code] at the selected positions      */
       SL_PROF_APPLY = 5,   /* sl_decompress_avg_apply[_coded]                   */
       SL_PROF_INDEX = 6,   /* coded format: placement of the quotient bit vectors
                               (sl_compress_coded)                               */
       SL_PROF_PHASES = 7 };
int sl_profile_begin(sl_plan *plan, int max_calls);
int sl_profile_end(sl_plan *plan, double *ms, int *calls);

const char *sl_strerror(int status);   /* static string                            */
const char *sl_last_hip_error(void);   /* text of the last HIP failure, or ""      */

#ifdef __cplusplus
}
#endif
#endif /* SPARSELOCO_H */
