/*
 * QSGD CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded C implementation of the QSGD hot path
 * (Alistarh et al., "QSGD: Communication-Efficient SGD via Gradient
 * Quantization and Encoding"): the stochastic quantizer Q_s (Sec. 3.1, Eq. 2),
 * bucketing (Sec. 4), the recursive Elias code (App. A.2, Definition), the
 * vector codes Code_s (Sec. 3.1 / App. A.2) and Code'_s (App. A.3), a
 * fixed-width packing for the "b-bit QSGD" of Sec. 5, Decode, and the
 * aggregate-and-step of Algorithm 1.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may use it.
 * It shares no code, header, table or constant generator with the GPU library.
 *
 * Parity status of each part (what it is pinned to, see tests/):
 *   Q_s           pinned: exact enumeration on n<=4, Lemma 3.1 (i)-(iii),
 *                 closed-form second moment (proof of Lemma 3.1), d=1 identity.
 *   Elias omega   pinned: textbook code words, round trip 1..2^20, prefix-free.
 *   Code_s/Code'_s pinned: round trip + closed-form lengths (App. A.2 / A.3).
 *   Philox-4x32-10 (the paper names no generator): pinned to the published
 *                 known-answer vectors and an independent big-integer version.
 *   Step          pinned: K=1 d=1 equals plain SGD; linearity vs accumulate; the
 *                 bucket-range form equals the whole step restricted to the range.
 *   Slices        pinned: buckets i..j of the whole message word for word; beyond
 *                 2^34 against draws recomputed with the big-integer generator.
 *   Memory safety: the whole file runs under -fsanitize=address,undefined
 *                 (sanitize_check.c).
 *   Container (header, offset table, word alignment, bit order) and the
 *   fixed-width field layout: builder-defined, PARITY UNPINNED by the paper
 *   (it gives bit widths only); covered by round trip and size formulas.
 */
#ifndef QSGD_ORACLE_H
#define QSGD_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { QO_CODE_SPARSE = 0, QO_CODE_DENSE = 1, QO_CODE_FIXED = 2 };
enum { QO_NORM_L2 = 0, QO_NORM_MAX = 1 };

enum {
  QO_OK = 0,
  QO_ERR_INVALID_ARG = -1,
  QO_ERR_CAPACITY = -2,
  QO_ERR_CORRUPT = -3
};

typedef struct {
  uint64_t n;         /* gradient length (Sec. 2)                                  */
  uint64_t d;         /* bucket size, d >= n means one bucket (Sec. 4)             */
  uint64_t seed;      /* Philox key                                                */
  uint32_t s;         /* number of quantization levels, 1..65535 (Sec. 3.1)        */
  uint32_t code;      /* QO_CODE_*                                                 */
  uint32_t norm;      /* QO_NORM_*  (L2: Eq. 2; MAX: Sec. 4, second variation)     */
  uint32_t stream_id; /* peer id        -> Philox counter word 2                   */
  uint32_t iteration; /* iteration t    -> Philox counter word 3                   */
  uint32_t reserved;
} qo_params;

/* Philox-4x32 with 10 rounds (Salmon et al., SC'11). */
void qo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The uniform draw in [0,1) used for element `index` (global index in the n-vector). */
float qo_draw(const qo_params *p, uint64_t index);

/* Recursive Elias (omega) code of k >= 1 (App. A.2, Definition). */
uint32_t qo_omega_len(uint64_t k);
/* Writes the code word as a string of '0'/'1' characters (NUL terminated); returns length. */
uint32_t qo_omega_string(uint64_t k, char *out, size_t out_cap);
/* Decodes one code word from a '0'/'1' string; returns the number of characters
 * consumed (0 on malformed/truncated input) and stores the integer in *k. */
uint32_t qo_omega_decode_string(const char *bits, size_t nbits, uint64_t *k);

/* Number of k in [lo, hi] whose code word does not decode back to k. */
uint64_t qo_omega_roundtrip_failures(uint64_t lo, uint64_t hi);

/* Geometry helpers. */
uint64_t qo_bucket_size(const qo_params *p);  /* effective d                      */
uint64_t qo_num_buckets(const qo_params *p);
uint32_t qo_fixed_field_bits(uint32_t s);     /* B in {2,4,8,16}                  */

/* Q_s per bucket (Eq. 2 applied to each bucket, Sec. 4).
 *   g        n floats
 *   u_in     NULL -> draws come from Philox; else n floats used as the draws
 *   levels   n x u32 : zeta_i = s * xi_i in 0..s
 *   neg      n x u8  : 1 iff v_i < 0
 *   norms    num_buckets floats: the scale of each bucket (fp32, as sent)
 *   u_out,p_out  optional (may be NULL): the draw and the round-up probability
 *                of each element (p = -1 where no draw decides, i.e. level == s
 *                by clamping or the bucket norm is 0)
 */
int qo_quantize(const qo_params *p, const float *g, const float *u_in,
                uint32_t *levels, uint8_t *neg, float *norms,
                float *u_out, float *p_out);

/* Q_s of a slice of a longer vector: element i takes the draw of global index
 * index_offset + i (as qo_encode_slice does); qo_quantize is the case index_offset = 0. */
int qo_quantize_slice(const qo_params *p, const float *g, uint64_t index_offset,
                      const float *u_in, uint32_t *levels, uint8_t *neg, float *norms,
                      float *u_out, float *p_out);

/* Worst-case message size in bytes for these parameters. */
size_t qo_max_encoded_bytes(const qo_params *p);

/* Encode = Code(Q_s(g)) into the message container. *bytes_out = used bytes. */
int qo_encode(const qo_params *p, const float *g, void *msg, size_t capacity,
              size_t *bytes_out);
/* Same, but with the draws supplied by the caller. */
int qo_encode_with_draws(const qo_params *p, const float *g, const float *u_in,
                         void *msg, size_t capacity, size_t *bytes_out);

/* Encode of a slice of a longer vector: g holds p->n elements that sit at global
 * indices [index_offset, index_offset + n) of it, so element i takes the draw of
 * global index index_offset + i (index_offset a multiple of the bucket size
 * reproduces the corresponding buckets of the long vector's message). */
int qo_encode_slice(const qo_params *p, const float *g, uint64_t index_offset,
                    void *msg, size_t capacity, size_t *bytes_out);

/* Encode ONE bucket: `v` holds its m elements, `first_index` is the global
 * index of v[0] (it selects the Philox draws), bucket geometry is not taken
 * from p->n/p->d.  Output: the bucket's string as 32-bit words.
 * Returns the number of words, or a negative error. */
int64_t qo_encode_bucket(const qo_params *p, const float *v, uint64_t m,
                         uint64_t first_index, uint32_t *words, size_t cap_words);

/* Reads a message header: fills *p (seed is not stored in a message: set to 0)
 * and *total_bytes. */
int qo_message_info(const void *msg, size_t avail_bytes, qo_params *p,
                    uint64_t *total_bytes);

/* Decode to the tuple (norms, neg, levels) -- any output may be NULL. */
int qo_decode_tuple(const void *msg, size_t bytes, uint32_t *levels, uint8_t *neg,
                    float *norms);
/* Decode to the dense vector g_hat (n floats):
 * g_hat_i = norm_b * sgn_i * zeta_i / s (Eq. 2). */
int qo_decode(const void *msg, size_t bytes, float *g_hat);

/* acc_i <- acc_i + sum_{k<K} Decode(M_k)_i   (sum taken in k order, fp32). */
int qo_decode_accumulate(const void *const *msgs, const size_t *bytes, uint32_t K,
                         float *acc);
/* x_i <- x_i - (eta/K) * sum_{k<K} Decode(M_k)_i   (Algorithm 1, last line). */
int qo_sgd_step(const void *const *msgs, const size_t *bytes, uint32_t K, float eta,
                float *x);

/* The step of Algorithm 1 on the coordinates of buckets [bucket_begin, bucket_begin +
 * bucket_count) only (buckets are independent, Sec. 4); x points at the first coordinate
 * of bucket `bucket_begin`. */
int qo_sgd_step_buckets(const void *const *msgs, const size_t *bytes, uint32_t K, float eta,
                        float *x, uint64_t bucket_begin, uint64_t bucket_count);

/* Word offset (from the payload start) and word count of bucket b's string. */
int qo_bucket_extent(const void *msg, size_t bytes, uint64_t b, uint64_t *word_off,
                     uint64_t *word_cnt);
/* Byte offset of the payload inside the message. */
int qo_payload_offset(const void *msg, size_t bytes, uint64_t *byte_off);

/* ---- tensor-aware messages (Sec. 5, "Protocol": small matrices are not
 * quantized, buckets are laid out per matrix).  The gradient is an arena of
 * p->n floats; tensor j occupies [offset, offset + size), tensors ascending and
 * disjoint.  Tensors with size < bypass_below travel as raw fp32; the others
 * are cut into buckets of p->d values that restart at the tensor's first value.
 * Draws are indexed by arena position.  CONTAINER LAYOUT: PARITY UNPINNED (the
 * paper fixes only the rule, not a format); the quantized values are pinned
 * through the flat functions they reuse. */
typedef struct { uint64_t offset, size; } qo_tensor;
int qo_layout_counts(const qo_params *p, const qo_tensor *t, uint32_t T,
                     uint64_t bypass_below, uint64_t *buckets, uint64_t *raw_elems);
size_t qo_layout_max_encoded_bytes(const qo_params *p, const qo_tensor *t, uint32_t T,
                                   uint64_t bypass_below);
int qo_encode_layout(const qo_params *p, const qo_tensor *t, uint32_t T,
                     uint64_t bypass_below, const float *arena, void *msg,
                     size_t capacity, size_t *bytes_out);
int qo_decode_layout(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                     const void *msg, size_t bytes, float *arena_out);
int qo_decode_accumulate_layout(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                                const void *const *msgs, const size_t *bytes, uint32_t K,
                                float *acc);
int qo_sgd_step_layout(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                       const void *const *msgs, const size_t *bytes, uint32_t K, float eta,
                       float *x);

#ifdef __cplusplus
}
#endif
#endif
