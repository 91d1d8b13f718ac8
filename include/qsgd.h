/*
 * libqsgd -- the data-parallel hot path of QSGD on one MI355X (gfx950).
 *
 * Alistarh, Grubic, Li, Tomioka, Vojnovic: "QSGD: Communication-Efficient SGD
 * via Gradient Quantization and Encoding".  The three entry points are the
 * boxed calls and the last line of Algorithm 1:
 *
 *   qsgd_encode             M <- Encode(g) = Code(Q_s(g))        (Alg. 1; Sec. 3.1)
 *   qsgd_decode_accumulate  acc <- acc + sum_l Decode(M_l)       (Alg. 1; Sec. 3.1)
 *   qsgd_sgd_step           x <- x - (eta/K) sum_l Decode(M_l)   (Alg. 1, last line)
 *
 * Plain C ABI: pointers and sizes only.  Every pointer named *_dev is device
 * memory owned by the caller; everything else is host memory.  The calls on
 * the hot path allocate no device memory: scratch comes in through
 * `workspace_dev` (the one exception is qsgd_layout_create, which uploads two
 * small tables once per layout, outside the path).  All work is queued on the HIP stream passed in (a hipStream_t cast to void*,
 * NULL = the default stream) and the calls return without waiting for it.
 *
 * Return value: 0, or a negative QSGD_ERR_* found on the host before anything
 * was queued.  Conditions only the GPU can see (message capacity exceeded, a
 * malformed message) are recorded in a status word and fetched with
 * qsgd_message_status / qsgd_workspace_status; kernels never read or write
 * outside the buffers described here, whatever the message bytes are.
 */
#ifndef QSGD_H
#define QSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Vector code (how the tuple (||v||, sigma, zeta) of Sec. 3.1 becomes bits). */
#define QSGD_CODE_SPARSE 0u /* Code_s : Elias(gap), sign, Elias(level) per nonzero (Sec. 3.1, App. A.2) */
#define QSGD_CODE_DENSE  1u /* Code'_s: sign, Elias(level+1) for every coordinate (App. A.3)            */
#define QSGD_CODE_FIXED  2u /* b-bit fields + sign bits, the "b-bit QSGD" of Sec. 5                     */

/* Scale of a bucket. */
#define QSGD_NORM_L2  0u    /* ||v||_2 (Eq. 2)                                    */
#define QSGD_NORM_MAX 1u    /* max_i |v_i| (Sec. 4, second variation)             */

#define QSGD_OK               0
#define QSGD_ERR_INVALID_ARG (-1) /* bad parameter, null pointer, misaligned buffer        */
#define QSGD_ERR_CAPACITY    (-2) /* message or workspace buffer too small                 */
#define QSGD_ERR_CORRUPT     (-3) /* message does not parse / header does not match params */
#define QSGD_ERR_HIP         (-4) /* a HIP runtime call failed                             */
#define QSGD_ERR_UNSUPPORTED (-5) /* valid request this build has no kernel for            */
#define QSGD_ERR_SCRATCH     (-6) /* request needs more than the built-in scratch holds    */

#define QSGD_MAX_PEERS 64u        /* largest K                                             */
#define QSGD_HEADER_BYTES 64u

/* Parameters of one Encode, and of the messages a Decode expects.
 *   n          length of the gradient vector (Sec. 2), 0 <= n < 2^32
 *   d          bucket size (Sec. 4): consecutive runs of d values are quantized
 *              independently, each with its own scale; d >= n means one bucket
 *   seed       key of the Philox-4x32-10 generator behind the rounding draws
 *   s          number of quantization levels (Sec. 3.1), 1 <= s <= 65535
 *   code, norm QSGD_CODE_*, QSGD_NORM_*
 *   stream_id  peer id and
 *   iteration  iteration number: counter words 2 and 3 of the generator, so that
 *              peers and iterations draw independently (element i uses word i%4 of
 *              the block with counter (i/4 low, i/4 high, stream_id, iteration))
 */
typedef struct qsgd_params {
  uint64_t n;
  uint64_t d;
  uint64_t seed;
  uint32_t s;
  uint32_t code;
  uint32_t norm;
  uint32_t stream_id;
  uint32_t iteration;
  uint32_t reserved; /* must be 0 */
} qsgd_params;

/* Library version (major*10000 + minor*100 + patch). Host only. */
int qsgd_version(void);

/* Text for a QSGD_ERR_* code. Host only; the string is static. */
const char *qsgd_strerror(int err);

/* Worst-case size in bytes of a message for these parameters (every coordinate
 * nonzero at the top level).  A smaller buffer may be passed to qsgd_encode when
 * the data are known to be sparse; running out is reported, never overrun.
 * Host only.  Returns 0 for invalid parameters. */
size_t qsgd_max_encoded_bytes(const qsgd_params *p);

/* Bytes of scratch the calls below need for these parameters and up to K
 * messages (K = 0 or 1 for encode-only use).  Host only; does not depend on the
 * device.  Returns 0 for invalid parameters. */
size_t qsgd_workspace_bytes(const qsgd_params *p, uint32_t K);

/* Bytes of scratch qsgd_encode needs when the message buffer has msg_capacity bytes (a
 * caller that knows its gradients to be sparse passes a buffer far below the worst case,
 * and the staging of the bucket strings can shrink with it): at most
 * qsgd_workspace_bytes(p, 1).  qsgd_encode accepts any workspace from this size up; with
 * less than the worst case, a part of the vector that codes much longer than its share of
 * msg_capacity ends the call like a message that does not fit (status QSGD_ERR_CAPACITY
 * in the header, size needed in its length field).  Host only. */
size_t qsgd_encode_workspace_bytes(const qsgd_params *p, size_t msg_capacity);

/* Encode (Alg. 1, "M^i <- Encode(g)"; Q_s: Sec. 3.1 Eq. 2 per bucket of Sec. 4;
 * Code_s / Code'_s: Sec. 3.1, App. A.2-A.3).
 *   g_dev          in : n floats, device, 16-byte aligned, finite values
 *   msg_dev        out: the message, device, 16-byte aligned, msg_capacity bytes.
 *                  Layout: 64-byte header | table of bucket word offsets
 *                  (Elias codes only) | bucket strings, each word aligned.
 *                  The used length is in the header (qsgd_message_info).
 *   workspace_dev  scratch, device, 16-byte aligned, >= qsgd_workspace_bytes(p, 1), or
 *                  >= qsgd_encode_workspace_bytes(p, msg_capacity) for sparse data;
 *                  contents on entry are ignored, calls sharing it must not overlap
 *   hip_stream     the stream the kernels are queued on
 * Errors: INVALID_ARG, CAPACITY (buffers smaller than the fixed parts), HIP,
 * UNSUPPORTED.  Payload overflow is found on the device: the header's status
 * becomes QSGD_ERR_CAPACITY and its length field says what was needed. */
int qsgd_encode(const qsgd_params *p, const float *g_dev, void *msg_dev,
                size_t msg_capacity, void *workspace_dev, size_t workspace_bytes,
                void *hip_stream);

/* qsgd_encode for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The scratch is a 64 MiB array inside the library image
 * (qsgd_static_scratch_bytes()); each GPU the library runs on holds its copy until the
 * process ends.  Arguments, message and error behaviour as qsgd_encode, minus the
 * workspace; additionally QSGD_ERR_SCRATCH when qsgd_workspace_bytes(p, 1) exceeds the
 * array (nothing is queued then).  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine; while qsgd_timing_enable is on, timing events are taken
 * from the pool made when it was switched on).  Every call on a GPU shares that GPU's array: calls that
 * overlap in time on one GPU (different streams, different threads) race, also with
 * each other's messages; calls on one stream, or ordered by events, are safe.  Nothing
 * in the array has to survive between calls and nothing has to be cleared. */
int qsgd_encode_static(const qsgd_params *p, const float *g_dev, void *msg_dev,
                       size_t msg_capacity, void *hip_stream);
size_t qsgd_static_scratch_bytes(void);

/* Decode K messages and add them up (Alg. 1, "g^l <- Decode(M^l)" and the sum of
 * its last line):  acc_i <- acc_i + (((0 + g^0_i) + g^1_i) + ... + g^{K-1}_i),
 * g^l_i = ||v||_bucket * sgn_i * level_i / s  (Eq. 2), all in fp32.
 *   msgs_dev       host array of K device pointers (16-byte aligned messages made
 *                  with the same n, d, s, code, norm as *p), 1 <= K <= QSGD_MAX_PEERS
 *   msg_bytes      host array of K sizes: readable bytes behind each pointer (the
 *                  kernels never read past them, whatever a header claims)
 *   acc_dev        in/out: n floats, device, 16-byte aligned
 *   workspace_dev  >= qsgd_workspace_bytes(p, K); word 0 receives the status
 * Errors: INVALID_ARG, CAPACITY, HIP, UNSUPPORTED on the host; a header that does
 * not match *p or a string that does not parse sets the workspace status to
 * QSGD_ERR_CORRUPT (values written for that bucket are then unspecified, nothing
 * outside acc_dev[0..n) is touched). */
int qsgd_decode_accumulate(const qsgd_params *p, const void *const *msgs_dev,
                           const size_t *msg_bytes, uint32_t K, float *acc_dev,
                           void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* The fused receive side of Alg. 1:  x_i <- fma(-(eta/K), sum_l g^l_i, x_i) with the
 * sum taken as in qsgd_decode_accumulate.  Arguments as there; x_dev in/out. */
int qsgd_sgd_step(const qsgd_params *p, const void *const *msgs_dev,
                  const size_t *msg_bytes, uint32_t K, float eta, float *x_dev,
                  void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* ---- Tensor-aware messages (Sec. 5, "Protocol": matrices with fewer than 10K
 * elements are sent unquantized, and quantization buckets are laid out per matrix).
 *
 * The gradient (and x) is an ARENA of p->n floats on the device in which tensor j
 * occupies [offsets[j], offsets[j] + sizes[j]); tensors ascend, do not overlap, and
 * start at multiples of 4 elements (16 bytes), as tensors packed with allocator
 * alignment do.  A tensor with sizes[j] < bypass_below travels as raw fp32 behind
 * the bucket strings; every other tensor is cut into buckets of d values that
 * restart at its first value (its last bucket is shorter), so no bucket mixes two
 * tensors' scales.  Draws are indexed by arena position.  Messages carry header
 * version 2; decoding needs the same layout.  d must be a multiple of 4, <= 8192.
 *
 * qsgd_layout_create builds the layout from HOST arrays and uploads two small tables
 * to the current device (it allocates device memory; the layout is immutable and may
 * be shared by any number of calls on that device); qsgd_layout_destroy frees it.
 * The other calls mirror their flat namesakes: same arguments plus the layout, same
 * ownership, same error behaviour; p->d must equal the layout's d and p->n must
 * cover its extent.  Positions of the arena outside every tensor are never read or
 * written.  Returns QSGD_ERR_UNSUPPORTED for bucket sizes the layout path does not
 * take. */
typedef struct qsgd_layout qsgd_layout;
int qsgd_layout_create(const uint64_t *offsets, const uint64_t *sizes, uint32_t T, uint64_t d,
                       uint64_t bypass_below, qsgd_layout **out);
void qsgd_layout_destroy(qsgd_layout *layout);
int qsgd_layout_info(const qsgd_layout *layout, uint64_t *buckets, uint64_t *raw_values,
                     uint64_t *extent);
size_t qsgd_layout_max_encoded_bytes(const qsgd_params *p, const qsgd_layout *layout);
size_t qsgd_layout_workspace_bytes(const qsgd_params *p, const qsgd_layout *layout, uint32_t K);
int qsgd_encode_layout(const qsgd_params *p, const qsgd_layout *layout, const float *g_dev,
                       void *msg_dev, size_t msg_capacity, void *workspace_dev,
                       size_t workspace_bytes, void *hip_stream);
int qsgd_decode_accumulate_layout(const qsgd_params *p, const qsgd_layout *layout,
                                  const void *const *msgs_dev, const size_t *msg_bytes,
                                  uint32_t K, float *acc_dev, void *workspace_dev,
                                  size_t workspace_bytes, void *hip_stream);
int qsgd_sgd_step_layout(const qsgd_params *p, const qsgd_layout *layout,
                         const void *const *msgs_dev, const size_t *msg_bytes, uint32_t K,
                         float eta, float *x_dev, void *workspace_dev, size_t workspace_bytes,
                         void *hip_stream);

/* Encode of a SLICE of a longer vector: as qsgd_encode on the p->n values at g_dev,
 * with the rounding draws of positions index_base .. index_base + p->n - 1 of the
 * whole vector (index_base a multiple of 4, else QSGD_ERR_INVALID_ARG; any code and any
 * bucket size qsgd_encode takes).  If index_base is a multiple of the bucket size, the
 * buckets and levels are exactly those the whole vector would get. */
int qsgd_encode_slice(const qsgd_params *p, uint64_t index_base, const float *g_dev,
                      void *msg_dev, size_t msg_capacity, void *workspace_dev,
                      size_t workspace_bytes, void *hip_stream);

/* ---- Double-buffered pass (Sec. 5, "Protocol": quantization and communication are
 * double buffered so that they overlap with computation).  The vector of p->n values is
 * cut into chunks of chunk_elems (a multiple of the bucket size and of 4; any code and
 * bucket size the flat calls take).  For every chunk the K
 * peers' slices g_dev[k] + offset are encoded (peer k with stream_id p->stream_id + k)
 * on one internal stream, then decoded, summed and applied to x_dev + offset on a second
 * one, while the next chunk is already being encoded; msg_dev holds 2*K device buffers
 * of msg_capacity bytes each (two sets used alternately; size them with
 * qsgd_max_encoded_bytes for n = chunk_elems), and the two workspaces (distinct, each
 * workspace_bytes >= qsgd_workspace_bytes for n = chunk_elems) serve the encode and the
 * decode side.  The work starts after what is queued on hip_stream at the time of the
 * call, and hip_stream continues after the last chunk.  x ends up exactly as after one
 * qsgd_sgd_step over the K whole-vector messages.  Errors as the calls it is made of:
 * sizes and parameters of every chunk are checked before anything is queued, so a
 * negative return leaves x untouched (only a failing HIP call can end the pass half way;
 * the internal streams may then still hold work: synchronise the device).
 * qsgd_pipeline_create makes the two streams (default priority) and five events on the
 * current device; calls on one pipeline object must not overlap. */
typedef struct qsgd_pipeline qsgd_pipeline;
int qsgd_pipeline_create(qsgd_pipeline **out);
void qsgd_pipeline_destroy(qsgd_pipeline *pl);
int qsgd_pipeline_step(qsgd_pipeline *pl, const qsgd_params *p, uint64_t chunk_elems,
                       const float *const *g_dev, uint32_t K, float eta, float *x_dev,
                       void *const *msg_dev, size_t msg_capacity, void *enc_workspace_dev,
                       void *dec_workspace_dev, size_t workspace_bytes, void *hip_stream);

/* Reads a message header from a HOST copy of (at least) its first 64 bytes.
 * Fills *out (seed is not stored: 0) and *total_bytes (either may be NULL).
 * Returns 0, QSGD_ERR_CORRUPT (not a header), or the status the encoder left
 * (QSGD_ERR_CAPACITY: *total_bytes is the size that would have been needed). */
int qsgd_message_info(const void *header_host, qsgd_params *out, uint64_t *total_bytes);

/* Convenience: waits for `hip_stream`, copies the header of msg_dev to the host
 * and returns what qsgd_message_info returns (or QSGD_ERR_HIP). */
int qsgd_message_status(const void *msg_dev, uint64_t *total_bytes, void *hip_stream);

/* Waits for `hip_stream` and returns the status word the last decode call left
 * in workspace_dev (0 or QSGD_ERR_CORRUPT), or QSGD_ERR_HIP. */
int qsgd_workspace_status(const void *workspace_dev, void *hip_stream);

/* Kernel timing for benchmarks: while enabled, every kernel launch of the
 * library is bracketed by HIP events on its own stream.  qsgd_timing_get waits
 * for the recorded events and reports, for kernels whose name starts with
 * `prefix`, the summed duration in milliseconds and the launch count since the
 * last reset.  Off by default; not for use inside stream capture. */
int qsgd_timing_enable(int on);
int qsgd_timing_reset(void);
int qsgd_timing_get(const char *prefix, double *total_ms, uint64_t *launches);

/* Measurement aid, not part of the method: a plain copy kernel (16-byte loads and
 * stores, grid-stride) of `bytes` bytes (a multiple of 16) from src_dev to dst_dev,
 * both device pointers aligned to 16 bytes, on `hip_stream` (streaming accesses, one
 * contiguous 16 KiB piece per workgroup).  It gives the copy ceiling of the machine the
 * codec is compared with, and a kernel of known HBM traffic that hardware counters can
 * be calibrated against.  Timed as "copy_probe".
 * Returns 0, QSGD_ERR_INVALID_ARG or QSGD_ERR_HIP. */
int qsgd_copy_probe(void *dst_dev, const void *src_dev, size_t bytes, void *hip_stream);

/* Measurement aid, not part of the method: the same copy with ONE 4-byte load and one
 * 4-byte store per lane (bytes a multiple of 4), the request size of the kernels that read
 * message strings word by word.  A second kernel of known traffic, so that the factors of
 * the hardware counters are known for both request sizes.  Timed as "copywords_probe". */
int qsgd_copy_probe_words(void *dst_dev, const void *src_dev, size_t bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* QSGD_H */
