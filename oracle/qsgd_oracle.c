/*
 * QSGD CPU oracle -- TEST INFRASTRUCTURE ONLY (see qsgd_oracle.h).
 *
 * Everything here follows the paper's order of steps, one element and one bit
 * at a time.  No blocking, no fusion, no tables.  Compile with
 * -ffp-contract=off so that every fp32 operation below rounds once, as written.
 */
#include "qsgd_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11).  The paper leaves the source of randomness open. */
/* ------------------------------------------------------------------------- */

void qo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u; /* round multipliers      */
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u; /* key schedule (Weyl)    */
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    uint64_t prod0 = M0 * (uint64_t)c0;
    uint64_t prod1 = M1 * (uint64_t)c2;
    uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
    uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
    uint32_t n0 = hi1 ^ c1 ^ k0;
    uint32_t n1 = lo1;
    uint32_t n2 = hi0 ^ c3 ^ k1;
    uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0;
    k1 += W1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Draw for global element `index`: one Philox block serves four consecutive
 * elements; key = seed, counter = (index/4 lo, index/4 hi, stream, iteration);
 * the top 24 bits of the word give u = m * 2^-24 in [0,1). */
float qo_draw(const qo_params *p, uint64_t index) {
  uint64_t q = index >> 2;
  uint32_t ctr[4] = {(uint32_t)q, (uint32_t)(q >> 32), p->stream_id, p->iteration};
  uint32_t key[2] = {(uint32_t)p->seed, (uint32_t)(p->seed >> 32)};
  uint32_t out[4];
  qo_philox4x32_10(ctr, key, out);
  uint32_t w = out[index & 3];
  return (float)(w >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------------- */
/* Bit strings.  Stream bit j lives in 32-bit word j/32 at bit 31-(j%32).      */
/* ------------------------------------------------------------------------- */

typedef struct {
  uint32_t *w;    /* zero-initialised by the caller */
  uint64_t cap;   /* capacity in bits               */
  uint64_t pos;   /* next bit                       */
  int overflow;
} bitw;

static void put_bit(bitw *b, unsigned bit) {
  if (b->pos >= b->cap) { b->overflow = 1; b->pos++; return; }
  if (bit) b->w[b->pos >> 5] |= 1u << (31 - (b->pos & 31));
  b->pos++;
}

/* most significant bit first */
static void put_bits(bitw *b, uint64_t value, unsigned nbits) {
  for (unsigned i = nbits; i-- > 0;) put_bit(b, (unsigned)((value >> i) & 1u));
}

typedef struct {
  const uint32_t *w;
  uint64_t end;   /* one past the last readable bit */
  uint64_t pos;
  int overrun;
} bitr;

static unsigned get_bit(bitr *b) {
  if (b->pos >= b->end) { b->overrun = 1; b->pos++; return 0; }
  unsigned bit = (b->w[b->pos >> 5] >> (31 - (b->pos & 31))) & 1u;
  b->pos++;
  return bit;
}

/* ------------------------------------------------------------------------- */
/* Recursive Elias coding (App. A.2, Definition).  The definition's stopping   */
/* test is read as "k = 1" (the decoder rule, and |Elias(1)| = 1, fix this):   */
/* a '0' goes at the end; while k > 1 the binary form of k is put in front and */
/* k becomes (number of bits just written) - 1.                                */
/* ------------------------------------------------------------------------- */

static unsigned bit_length(uint64_t k) { /* floor(log2 k) + 1, k >= 1 */
  unsigned n = 0;
  while (k) { n++; k >>= 1; }
  return n;
}

uint32_t qo_omega_len(uint64_t k) {
  uint32_t len = 1; /* the final '0' */
  while (k > 1) {
    unsigned nb = bit_length(k);
    len += nb;
    k = nb - 1;
  }
  return len;
}

/* The groups are prepended, so the one written first on the wire is the one
 * produced last: recurse before emitting. */
static void omega_groups(bitw *b, uint64_t k) {
  if (k <= 1) return;
  unsigned nb = bit_length(k);
  omega_groups(b, nb - 1);
  put_bits(b, k, nb);
}

static void put_omega(bitw *b, uint64_t k) {
  omega_groups(b, k);
  put_bit(b, 0);
}

/* Decoder rule of the Definition: N = 1; a 0 bit ends and outputs N; a 1 bit is
 * the first of N+1 bits whose binary value becomes the new N. */
static uint64_t get_omega(bitr *b) {
  uint64_t N = 1;
  for (;;) {
    unsigned bit = get_bit(b);
    if (b->overrun) return 0;
    if (bit == 0) return N;
    if (N > 63) { b->overrun = 1; return 0; } /* would not fit 64 bits: malformed */
    uint64_t v = 1;
    for (uint64_t i = 0; i < N; ++i) v = (v << 1) | get_bit(b);
    if (b->overrun) return 0;
    N = v;
  }
}

uint32_t qo_omega_string(uint64_t k, char *out, size_t out_cap) {
  uint32_t words[8] = {0};
  bitw b = {words, 256, 0, 0};
  if (k < 1) { if (out_cap) out[0] = 0; return 0; }
  put_omega(&b, k);
  uint32_t len = (uint32_t)b.pos;
  if (out_cap < (size_t)len + 1) { if (out_cap) out[0] = 0; return 0; }
  for (uint32_t j = 0; j < len; ++j)
    out[j] = ((words[j >> 5] >> (31 - (j & 31))) & 1u) ? '1' : '0';
  out[len] = 0;
  return len;
}

uint32_t qo_omega_decode_string(const char *bits, size_t nbits, uint64_t *k) {
  if (nbits > 256) nbits = 256;
  uint32_t words[8] = {0};
  for (size_t j = 0; j < nbits; ++j)
    if (bits[j] == '1') words[j >> 5] |= 1u << (31 - (j & 31));
  bitr r = {words, nbits, 0, 0};
  uint64_t v = get_omega(&r);
  if (r.overrun) return 0;
  *k = v;
  return (uint32_t)r.pos;
}

/* Encodes every k in [lo, hi] into a bit string, decodes it again and counts
 * the k for which the value, or the number of bits consumed, does not come
 * back (0 = the code round-trips on the whole range). */
uint64_t qo_omega_roundtrip_failures(uint64_t lo, uint64_t hi) {
  uint64_t bad = 0;
  for (uint64_t k = lo; k >= 1 && k <= hi; ++k) {
    uint32_t words[8] = {0};
    bitw b = {words, 256, 0, 0};
    put_omega(&b, k);
    bitr r = {words, b.pos, 0, 0};
    uint64_t v = get_omega(&r);
    if (r.overrun || v != k || r.pos != b.pos || b.pos != qo_omega_len(k)) bad++;
  }
  return bad;
}

/* ------------------------------------------------------------------------- */
/* Geometry (Sec. 4: bucket i is the sub-vector v[(i-1)d+1 : i d]).            */
/* ------------------------------------------------------------------------- */

uint64_t qo_bucket_size(const qo_params *p) {
  if (p->n == 0) return p->d ? p->d : 1;
  return p->d >= p->n ? p->n : p->d;
}

uint64_t qo_num_buckets(const qo_params *p) {
  if (p->n == 0) return 0;
  uint64_t d = qo_bucket_size(p);
  return (p->n + d - 1) / d;
}

static uint64_t bucket_len(const qo_params *p, uint64_t b) {
  uint64_t d = qo_bucket_size(p);
  uint64_t start = b * d;
  return (p->n - start < d) ? p->n - start : d;
}

/* Fixed-width level field: the narrowest of 2/4/8/16 bits that holds 0..s-1
 * (L2 scaling: level s is carried by the bucket's escape word) or 0..s (max
 * scaling, where level s is the common case). */
static uint32_t fixed_bits(uint32_t s, uint32_t norm) {
  uint32_t need = (norm == QO_NORM_MAX) ? s + 1 : s; /* number of code points */
  uint32_t B = 2;
  while (B < 16 && (1u << B) < need) B *= 2;
  return B;
}
uint32_t qo_fixed_field_bits(uint32_t s) { return fixed_bits(s, QO_NORM_L2); }

static int check_params(const qo_params *p) {
  if (!p) return QO_ERR_INVALID_ARG;
  if (p->s < 1 || p->s > 65535) return QO_ERR_INVALID_ARG;
  if (p->d < 1) return QO_ERR_INVALID_ARG;
  if (p->n > 0xFFFFFFFFull) return QO_ERR_INVALID_ARG;
  if (p->code > QO_CODE_FIXED) return QO_ERR_INVALID_ARG;
  if (p->norm > QO_NORM_MAX) return QO_ERR_INVALID_ARG;
  return QO_OK;
}

/* ------------------------------------------------------------------------- */
/* Q_s on one bucket (Eq. 2; bucketing of Sec. 4).                             */
/* ------------------------------------------------------------------------- */

static float bucket_scale(const qo_params *p, const float *v, uint64_t m) {
  if (p->norm == QO_NORM_MAX) {
    float mx = 0.0f;
    for (uint64_t i = 0; i < m; ++i) {
      float a = fabsf(v[i]);
      if (a > mx) mx = a;
    }
    return mx;
  }
  /* ||v||_2: squares summed in double in index order, rounded once to fp32
   * (the scale travels as 32 bits, Sec. 3.1). */
  double S = 0.0;
  for (uint64_t i = 0; i < m; ++i) S += (double)v[i] * (double)v[i];
  return (float)sqrt(S);
}

static void quantize_bucket(const qo_params *p, const float *v, uint64_t m,
                            uint64_t first_index, const float *u_in,
                            uint32_t *levels, uint8_t *neg, float *norm_out,
                            float *u_out, float *p_out) {
  const uint32_t s = p->s;
  float norm = bucket_scale(p, v, m);
  /* |v_i| / ||v|| * s is evaluated as |v_i| * fl(s / ||v||). */
  float inv = (norm > 0.0f) ? (float)s / norm : 0.0f;
  *norm_out = norm;
  for (uint64_t i = 0; i < m; ++i) {
    float t = fabsf(v[i]) * inv;          /* = a * s, a = |v_i| / ||v||       */
    float fl = floorf(t);
    uint32_t zeta;
    float prob = -1.0f, u = 0.0f;
    if (!(norm > 0.0f)) {
      zeta = 0;                           /* Q_s(0) = 0                       */
    } else if (fl >= (float)s) {
      zeta = s;                           /* a = 1 (or an ulp above): top level */
    } else {
      uint32_t l = (uint32_t)fl;          /* a in [l/s, (l+1)/s]              */
      prob = t - fl;                      /* p(a, s) = a s - l  (exact)       */
      u = u_in ? u_in[i] : qo_draw(p, first_index + i);
      zeta = l + ((u < prob) ? 1u : 0u);  /* (l+1)/s with probability p       */
    }
    levels[i] = zeta;
    neg[i] = (v[i] < 0.0f) ? 1 : 0;       /* sgn(0) = +1                      */
    if (u_out) u_out[i] = u;
    if (p_out) p_out[i] = prob;
  }
}

int qo_quantize_slice(const qo_params *p, const float *g, uint64_t index_offset,
                      const float *u_in, uint32_t *levels, uint8_t *neg, float *norms,
                      float *u_out, float *p_out) {
  int rc = check_params(p);
  if (rc) return rc;
  uint64_t d = qo_bucket_size(p), nb = qo_num_buckets(p);
  for (uint64_t b = 0; b < nb; ++b) {
    uint64_t start = b * d, m = bucket_len(p, b);
    quantize_bucket(p, g + start, m, index_offset + start, u_in ? u_in + start : NULL,
                    levels + start, neg + start, &norms[b],
                    u_out ? u_out + start : NULL, p_out ? p_out + start : NULL);
  }
  return QO_OK;
}

int qo_quantize(const qo_params *p, const float *g, const float *u_in,
                uint32_t *levels, uint8_t *neg, float *norms,
                float *u_out, float *p_out) {
  return qo_quantize_slice(p, g, 0, u_in, levels, neg, norms, u_out, p_out);
}

/* ------------------------------------------------------------------------- */
/* Vector codes.                                                               */
/* ------------------------------------------------------------------------- */

static uint32_t float_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* Worst-case bits of one bucket string of m elements. */
static uint64_t bucket_max_bits(const qo_params *p, uint64_t m) {
  if (p->code == QO_CODE_SPARSE) /* every element nonzero, gap 1, largest level */
    return 32 + m * (uint64_t)(1 + 1 + qo_omega_len(p->s)) + 1;
  if (p->code == QO_CODE_DENSE)
    return 32 + m * (uint64_t)(1 + qo_omega_len((uint64_t)p->s + 1));
  uint32_t B = fixed_bits(p->s, p->norm);
  return 64 + 32 * ((m * B + 31) / 32) + 32 * ((m + 31) / 32);
}

/* Entry points of long strings.  A prefix code can only be read from its start, so
 * a bucket of millions of values (the sparse regime of Sec. 3.1 uses one bucket
 * of n) would have to be decoded by a single sequential reader.  When the
 * bucket size exceeds 8192, a string of an Elias code is therefore followed by
 * a list of places where a reader may start: positions are cut into segments
 * of 2048; for segment j >= 1, start_j is the bit offset (in the string, scale
 * included) of the first record that belongs to a segment >= j and prev_j the
 * position (1-based, 0 = none) of the last coded coordinate before segment j;
 * segment j is listed iff floor(start_j / 1024) > floor(start_(j-1) / 1024)
 * (start_0 = 32) and start_j < 2^32.  After the string's last word come the
 * listed (start_j, prev_j) pairs as 32-bit words in ascending j and one word
 * with their count.  This is container metadata of the builder (about 3% of
 * the string), not part of the paper's code: CONTAINER LAYOUT, PARITY UNPINNED. */
#define QO_ENTRY_MIN_D 8192u
#define QO_ENTRY_SEG 2048u
#define QO_ENTRY_BITS 1024u
static int has_entries(const qo_params *p) {
  return p->code != QO_CODE_FIXED && qo_bucket_size(p) > QO_ENTRY_MIN_D;
}

/* Worst-case words of one bucket string of m elements, entry list included. */
static uint64_t bucket_max_words(const qo_params *p, uint64_t m) {
  uint64_t bits = bucket_max_bits(p, m), words = (bits + 31) / 32;
  if (has_entries(p)) {
    uint64_t segs = (m + QO_ENTRY_SEG - 1) / QO_ENTRY_SEG;
    uint64_t e = segs ? segs - 1 : 0;
    if (bits / QO_ENTRY_BITS < e) e = bits / QO_ENTRY_BITS;
    words += 2 * e + 1;
  }
  return words;
}

/* Code_s (Sec. 3.1; App. A.2): 32 bits of scale, then for every nonzero level in
 * order: Elias(distance from the previous nonzero; the first distance is the
 * 1-based position), one sign bit (1 = negative), Elias(level).
 * Code'_s (App. A.3): 32 bits of scale, then for EVERY coordinate a sign bit and
 * Elias(level + 1).
 * Fixed: scale word, escape word, level fields, sign bits (the paper gives bit
 * widths only, Sec. 5; this layout is the builder's). */
static uint64_t code_bucket(const qo_params *p, uint64_t m, float norm,
                            const uint32_t *levels, const uint8_t *neg, bitw *b) {
  uint64_t start_bit = b->pos;
  put_bits(b, float_bits(norm), 32);
  const int entries = has_entries(p);
  uint32_t *elist = NULL; /* (start, prev) pairs of the listed segments */
  uint64_t ecount = 0, ecap = 0, start_before = 32;
  if (p->code == QO_CODE_SPARSE || p->code == QO_CODE_DENSE) {
    uint64_t prev = 0; /* 1-based position of the previous coded coordinate */
    for (uint64_t i = 1; i <= m; ++i) {
      if (entries && i > 1 && (i - 1) % QO_ENTRY_SEG == 0) { /* a segment starts at i */
        uint64_t start = b->pos - start_bit;
        if (start / QO_ENTRY_BITS > start_before / QO_ENTRY_BITS && start < (1ull << 32)) {
          if (ecount == ecap) {
            ecap = ecap ? 2 * ecap : 64;
            elist = (uint32_t *)realloc(elist, ecap * 2 * sizeof(uint32_t));
          }
          elist[2 * ecount] = (uint32_t)start;
          elist[2 * ecount + 1] = (uint32_t)prev;
          ++ecount;
        }
        start_before = start;
      }
      if (p->code == QO_CODE_SPARSE) {
        if (levels[i - 1] == 0) continue;
        put_omega(b, i - prev);
        put_bit(b, neg[i - 1]);
        put_omega(b, levels[i - 1]);
      } else {
        put_bit(b, neg[i - 1]);
        put_omega(b, (uint64_t)levels[i - 1] + 1);
      }
      prev = i;
    }
    if (p->code == QO_CODE_SPARSE)
      put_bit(b, 1); /* stop marker: records end here (zeros pad the word) */
    if (entries) { /* the list follows the string's last word */
      b->pos = (b->pos + 31) & ~(uint64_t)31;
      for (uint64_t e = 0; e < 2 * ecount; ++e) put_bits(b, elist[e], 32);
      put_bits(b, ecount, 32);
    }
    free(elist);
  } else {
    /* Fixed width.  Word 1 is the escape: index of the one element whose level
     * does not fit the field (it can only be level s), else all ones.  Then
     * the level plane (element i's field at bits [iB, iB+B) counted from the
     * least significant bit of consecutive words) and the sign plane (element
     * i at bit i%32 of word i/32). */
    uint32_t B = fixed_bits(p->s, p->norm);
    uint32_t fmax = (1u << B) - 1u;
    uint64_t lw = (m * B + 31) / 32, sw = (m + 31) / 32;
    if (b->pos + 32 * (1 + lw + sw) > b->cap) {
      b->overflow = 1;
      b->pos += 32 * (1 + lw + sw);
      return b->pos - start_bit;
    }
    uint32_t *esc_word = b->w + (b->pos >> 5); /* strings are word aligned */
    uint32_t *level_plane = esc_word + 1;
    uint32_t *sign_plane = level_plane + lw;
    *esc_word = 0xFFFFFFFFu;
    for (uint64_t i = 0; i < m; ++i) {
      uint32_t f = levels[i];
      if (f > fmax) {            /* only level s = 2^B can be too wide */
        if (*esc_word != 0xFFFFFFFFu) b->overflow = 1; /* not representable */
        *esc_word = (uint32_t)i;
        f = fmax;
      }
      uint64_t bitpos = i * B;   /* B divides 32: a field never straddles */
      level_plane[bitpos >> 5] |= f << (bitpos & 31);
      if (neg[i]) sign_plane[i >> 5] |= 1u << (i & 31);
    }
    b->pos += 32 * (1 + lw + sw);
  }
  return b->pos - start_bit;
}

/* Container ---------------------------------------------------------------- */
/* 16 header words, then (codes with data-dependent length only) a table of    */
/* num_buckets+1 word offsets padded to a multiple of 4 words, then the bucket  */
/* strings, each starting on a word boundary and zero padded.                   */

#define QO_MAGIC 0x44475351u /* 'QSGD' */
enum { H_MAGIC = 0, H_VERSION, H_CODE, H_NORM, H_S, H_STREAM, H_D_LO, H_D_HI,
       H_N_LO, H_N_HI, H_NB_LO, H_NB_HI, H_PW_LO, H_PW_HI, H_STATUS, H_ITER,
       H_WORDS };

static uint64_t table_words(const qo_params *p) {
  if (p->code == QO_CODE_FIXED) return 0;
  uint64_t t = qo_num_buckets(p) + 1;
  return (t + 3) & ~(uint64_t)3;
}

size_t qo_max_encoded_bytes(const qo_params *p) {
  if (check_params(p)) return 0;
  uint64_t nb = qo_num_buckets(p), words = 0;
  for (uint64_t b = 0; b < nb; ++b) {
    /* all buckets but the last have the same length: avoid a long loop */
    if (b + 1 < nb) {
      words += (nb - 1) * bucket_max_words(p, qo_bucket_size(p));
      b = nb - 2;
      continue;
    }
    words += bucket_max_words(p, bucket_len(p, b));
  }
  return (size_t)(4 * (H_WORDS + table_words(p) + words));
}

static int encode_impl(const qo_params *p, const float *g, const float *u_in,
                       uint64_t index_offset, void *msg, size_t capacity,
                       size_t *bytes_out) {
  int rc = check_params(p);
  if (rc) return rc;
  uint64_t d = qo_bucket_size(p), nb = qo_num_buckets(p), tw = table_words(p);
  if (capacity < 4 * (H_WORDS + tw)) return QO_ERR_CAPACITY;
  uint32_t *w = (uint32_t *)msg;
  memset(w, 0, capacity - capacity % 4);
  uint32_t *table = w + H_WORDS;
  uint32_t *payload = table + tw;
  uint64_t cap_words = capacity / 4 - H_WORDS - tw;

  uint32_t *levels = (uint32_t *)malloc((d ? d : 1) * sizeof(uint32_t));
  uint8_t *neg = (uint8_t *)malloc(d ? d : 1);
  if (!levels || !neg) { free(levels); free(neg); return QO_ERR_INVALID_ARG; }

  bitw bw = {payload, cap_words * 32, 0, 0};
  for (uint64_t b = 0; b < nb; ++b) {
    uint64_t start = b * d, m = bucket_len(p, b);
    float norm;
    quantize_bucket(p, g + start, m, index_offset + start, u_in ? u_in + start : NULL,
                    levels, neg, &norm, NULL, NULL);
    if (tw) table[b] = (uint32_t)(bw.pos / 32);
    code_bucket(p, m, norm, levels, neg, &bw);
    bw.pos = (bw.pos + 31) & ~(uint64_t)31; /* next string starts on a word */
    if (bw.overflow || bw.pos > bw.cap) { free(levels); free(neg); return QO_ERR_CAPACITY; }
  }
  uint64_t pw = bw.pos / 32;
  if (tw) table[nb] = (uint32_t)pw;
  free(levels);
  free(neg);

  w[H_MAGIC] = QO_MAGIC; w[H_VERSION] = 1; w[H_CODE] = p->code; w[H_NORM] = p->norm;
  w[H_S] = p->s; w[H_STREAM] = p->stream_id;
  w[H_D_LO] = (uint32_t)d; w[H_D_HI] = (uint32_t)(d >> 32);
  w[H_N_LO] = (uint32_t)p->n; w[H_N_HI] = (uint32_t)(p->n >> 32);
  w[H_NB_LO] = (uint32_t)nb; w[H_NB_HI] = (uint32_t)(nb >> 32);
  w[H_PW_LO] = (uint32_t)pw; w[H_PW_HI] = (uint32_t)(pw >> 32);
  w[H_STATUS] = 0; w[H_ITER] = p->iteration;
  if (bytes_out) *bytes_out = (size_t)(4 * (H_WORDS + tw + pw));
  return QO_OK;
}

int qo_encode_with_draws(const qo_params *p, const float *g, const float *u_in,
                         void *msg, size_t capacity, size_t *bytes_out) {
  return encode_impl(p, g, u_in, 0, msg, capacity, bytes_out);
}

int qo_encode(const qo_params *p, const float *g, void *msg, size_t capacity,
              size_t *bytes_out) {
  return encode_impl(p, g, NULL, 0, msg, capacity, bytes_out);
}

int qo_encode_slice(const qo_params *p, const float *g, uint64_t index_offset,
                    void *msg, size_t capacity, size_t *bytes_out) {
  return encode_impl(p, g, NULL, index_offset, msg, capacity, bytes_out);
}

int64_t qo_encode_bucket(const qo_params *p, const float *v, uint64_t m,
                         uint64_t first_index, uint32_t *words, size_t cap_words) {
  int rc = check_params(p);
  if (rc) return rc;
  uint32_t *levels = (uint32_t *)malloc((m ? m : 1) * sizeof(uint32_t));
  uint8_t *neg = (uint8_t *)malloc(m ? m : 1);
  if (!levels || !neg) { free(levels); free(neg); return QO_ERR_INVALID_ARG; }
  float norm;
  quantize_bucket(p, v, m, first_index, NULL, levels, neg, &norm, NULL, NULL);
  memset(words, 0, cap_words * 4);
  bitw bw = {words, (uint64_t)cap_words * 32, 0, 0};
  code_bucket(p, m, norm, levels, neg, &bw);
  free(levels);
  free(neg);
  if (bw.overflow || bw.pos > bw.cap) return QO_ERR_CAPACITY;
  return (int64_t)((bw.pos + 31) / 32);
}

/* ------------------------------------------------------------------------- */
/* Decode.                                                                     */
/* ------------------------------------------------------------------------- */

typedef struct {
  qo_params p;
  uint64_t d, nb, tw, pw;
  const uint32_t *table, *payload;
} view;

static int open_msg(const void *msg, size_t bytes, view *v) {
  if (!msg || bytes < 4 * H_WORDS) return QO_ERR_CORRUPT;
  const uint32_t *w = (const uint32_t *)msg;
  if (w[H_MAGIC] != QO_MAGIC || w[H_VERSION] != 1) return QO_ERR_CORRUPT;
  if (w[H_STATUS] != 0) return QO_ERR_CORRUPT;
  memset(v, 0, sizeof *v);
  v->p.code = w[H_CODE]; v->p.norm = w[H_NORM]; v->p.s = w[H_S];
  v->p.stream_id = w[H_STREAM]; v->p.iteration = w[H_ITER];
  v->p.d = w[H_D_LO] | ((uint64_t)w[H_D_HI] << 32);
  v->p.n = w[H_N_LO] | ((uint64_t)w[H_N_HI] << 32);
  if (check_params(&v->p)) return QO_ERR_CORRUPT;
  v->d = qo_bucket_size(&v->p);
  v->nb = qo_num_buckets(&v->p);
  if (v->d != v->p.d) return QO_ERR_CORRUPT;
  if ((w[H_NB_LO] | ((uint64_t)w[H_NB_HI] << 32)) != v->nb) return QO_ERR_CORRUPT;
  v->tw = table_words(&v->p);
  v->pw = w[H_PW_LO] | ((uint64_t)w[H_PW_HI] << 32);
  if ((uint64_t)bytes / 4 < H_WORDS + v->tw + v->pw) return QO_ERR_CORRUPT;
  v->table = w + H_WORDS;
  v->payload = v->table + v->tw;
  return QO_OK;
}

static int bucket_extent_m(const view *v, uint64_t b, uint64_t m, uint64_t *off,
                           uint64_t *cnt) {
  if (b >= v->nb) return QO_ERR_INVALID_ARG;
  if (v->p.code == QO_CODE_FIXED) {
    uint64_t full = (bucket_max_bits(&v->p, v->d) + 31) / 32;
    *off = b * full;
    *cnt = (bucket_max_bits(&v->p, m) + 31) / 32;
  } else {
    uint64_t o0 = v->table[b], o1 = v->table[b + 1];
    if (o1 < o0) return QO_ERR_CORRUPT;
    *off = o0;
    *cnt = o1 - o0;
  }
  if (*off + *cnt > v->pw) return QO_ERR_CORRUPT;
  return QO_OK;
}

static int bucket_extent(const view *v, uint64_t b, uint64_t *off, uint64_t *cnt) {
  if (b >= v->nb) return QO_ERR_INVALID_ARG;
  return bucket_extent_m(v, b, bucket_len(&v->p, b), off, cnt);
}

int qo_message_info(const void *msg, size_t avail_bytes, qo_params *p,
                    uint64_t *total_bytes) {
  if (!msg || avail_bytes < 4 * H_WORDS) return QO_ERR_CORRUPT;
  const uint32_t *w = (const uint32_t *)msg;
  if (w[H_MAGIC] != QO_MAGIC || w[H_VERSION] != 1) return QO_ERR_CORRUPT;
  qo_params q;
  memset(&q, 0, sizeof q);
  q.code = w[H_CODE]; q.norm = w[H_NORM]; q.s = w[H_S];
  q.stream_id = w[H_STREAM]; q.iteration = w[H_ITER];
  q.d = w[H_D_LO] | ((uint64_t)w[H_D_HI] << 32);
  q.n = w[H_N_LO] | ((uint64_t)w[H_N_HI] << 32);
  if (check_params(&q)) return QO_ERR_CORRUPT;
  uint64_t pw = w[H_PW_LO] | ((uint64_t)w[H_PW_HI] << 32);
  if (p) *p = q;
  if (total_bytes) *total_bytes = 4 * (H_WORDS + table_words(&q) + pw);
  return w[H_STATUS] == 0 ? QO_OK : QO_ERR_CORRUPT;
}

int qo_bucket_extent(const void *msg, size_t bytes, uint64_t b, uint64_t *word_off,
                     uint64_t *word_cnt) {
  view v;
  int rc = open_msg(msg, bytes, &v);
  if (rc) return rc;
  return bucket_extent(&v, b, word_off, word_cnt);
}

int qo_payload_offset(const void *msg, size_t bytes, uint64_t *byte_off) {
  view v;
  int rc = open_msg(msg, bytes, &v);
  if (rc) return rc;
  *byte_off = 4 * (H_WORDS + v.tw);
  return QO_OK;
}

/* Reads bucket b back into (norm, levels[m], neg[m]); neg is only meaningful
 * where a sign was sent (sparse code: nonzero levels). */
static int decode_bucket_m(const view *v, uint64_t b, uint64_t m, float *norm,
                           uint32_t *levels, uint8_t *neg) {
  uint64_t off, cnt;
  int rc = bucket_extent_m(v, b, m, &off, &cnt);
  if (rc) return rc;
  if (cnt < 1) return QO_ERR_CORRUPT;
  const uint32_t *w = v->payload + off;
  /* long buckets: the entry list sits behind the string (see has_entries) */
  const uint32_t *elist = NULL;
  uint64_t ecount = 0, enext = 0;
  if (has_entries(&v->p)) {
    ecount = w[cnt - 1];
    if (2 * ecount + 1 >= cnt) return QO_ERR_CORRUPT;
    cnt -= 2 * ecount + 1;
    elist = w + cnt;
  }
  bitr r = {w, cnt * 32, 0, 0};
  uint32_t nbits = 0;
  for (int i = 0; i < 32; ++i) nbits = (nbits << 1) | get_bit(&r); /* the scale */
  *norm = bits_float(nbits);
  for (uint64_t i = 0; i < m; ++i) { levels[i] = 0; neg[i] = 0; }
  const uint32_t s = v->p.s;
  if (v->p.code == QO_CODE_SPARSE) {
    /* The string ends with a stop marker: a single 1 bit after the last
     * record, then zeros up to the word boundary.  So the last word is never
     * zero and the records end just before its lowest set bit. */
    uint32_t last = w[cnt - 1];
    if (last == 0) return QO_ERR_CORRUPT;
    unsigned tz = 0;
    while (((last >> tz) & 1u) == 0) tz++;
    uint64_t end = cnt * 32 - 1 - tz;
    if (end < 32) return QO_ERR_CORRUPT;
    r.end = end;
    /* positions and values of the nonzeros, until the records are used up */
    uint64_t pos = 0;
    while (r.pos < r.end) {
      if (enext < ecount && r.pos == elist[2 * enext]) { /* a listed place: it must agree */
        if (pos != elist[2 * enext + 1]) return QO_ERR_CORRUPT;
        ++enext;
      }
      uint64_t gap = get_omega(&r);
      if (r.overrun || gap == 0) return QO_ERR_CORRUPT;
      unsigned sign = get_bit(&r);
      uint64_t lev = get_omega(&r);
      if (r.overrun) return QO_ERR_CORRUPT;
      pos += gap;
      if (pos > m || lev < 1 || lev > s) return QO_ERR_CORRUPT;
      levels[pos - 1] = (uint32_t)lev;
      neg[pos - 1] = (uint8_t)sign;
    }
    /* segments after the last record are listed at the end of the records */
    while (enext < ecount && elist[2 * enext] == r.pos && elist[2 * enext + 1] == pos) ++enext;
    if (enext != ecount) return QO_ERR_CORRUPT;
  } else if (v->p.code == QO_CODE_DENSE) {
    for (uint64_t i = 0; i < m; ++i) {
      if (enext < ecount && r.pos == elist[2 * enext]) {
        if (i != elist[2 * enext + 1]) return QO_ERR_CORRUPT;
        ++enext;
      }
      unsigned sign = get_bit(&r);
      uint64_t lev1 = get_omega(&r);
      if (r.overrun || lev1 < 1 || lev1 > (uint64_t)s + 1) return QO_ERR_CORRUPT;
      levels[i] = (uint32_t)(lev1 - 1);
      neg[i] = (uint8_t)sign;
    }
    if (enext != ecount) return QO_ERR_CORRUPT;
  } else {
    uint32_t B = fixed_bits(s, v->p.norm);
    uint64_t lw = (m * B + 31) / 32, sw = (m + 31) / 32;
    if (cnt != 2 + lw + sw) return QO_ERR_CORRUPT;
    uint32_t esc = w[1];
    const uint32_t *lp = w + 2, *sp = w + 2 + lw;
    for (uint64_t i = 0; i < m; ++i) {
      uint64_t bitpos = i * B;
      uint32_t f = (lp[bitpos >> 5] >> (bitpos & 31)) & ((1u << B) - 1u);
      if (f > s) return QO_ERR_CORRUPT;
      levels[i] = f;
      neg[i] = (uint8_t)((sp[i >> 5] >> (i & 31)) & 1u);
    }
    if (esc != 0xFFFFFFFFu) {
      if (esc >= m) return QO_ERR_CORRUPT;
      levels[esc] = s;
    }
  }
  return QO_OK;
}

static int decode_bucket(const view *v, uint64_t b, float *norm, uint32_t *levels,
                         uint8_t *neg) {
  if (b >= v->nb) return QO_ERR_INVALID_ARG;
  return decode_bucket_m(v, b, bucket_len(&v->p, b), norm, levels, neg);
}

int qo_decode_tuple(const void *msg, size_t bytes, uint32_t *levels, uint8_t *neg,
                    float *norms) {
  view v;
  int rc = open_msg(msg, bytes, &v);
  if (rc) return rc;
  uint64_t d = v.d ? v.d : 1;
  uint32_t *lv = (uint32_t *)malloc(d * sizeof(uint32_t));
  uint8_t *ng = (uint8_t *)malloc(d);
  if (!lv || !ng) { free(lv); free(ng); return QO_ERR_INVALID_ARG; }
  for (uint64_t b = 0; b < v.nb && rc == QO_OK; ++b) {
    float norm;
    uint64_t m = bucket_len(&v.p, b);
    rc = decode_bucket(&v, b, &norm, lv, ng);
    if (rc) break;
    if (norms) norms[b] = norm;
    if (levels) memcpy(levels + b * v.d, lv, m * sizeof(uint32_t));
    if (neg) memcpy(neg + b * v.d, ng, m);
  }
  free(lv);
  free(ng);
  return rc;
}

/* g_hat_i = ||v|| * sgn(v_i) * zeta_i / s (Eq. 2), evaluated as
 * sign * (fl(||v|| / s) * zeta_i). */
int qo_decode(const void *msg, size_t bytes, float *g_hat) {
  view v;
  int rc = open_msg(msg, bytes, &v);
  if (rc) return rc;
  uint64_t d = v.d ? v.d : 1;
  uint32_t *lv = (uint32_t *)malloc(d * sizeof(uint32_t));
  uint8_t *ng = (uint8_t *)malloc(d);
  if (!lv || !ng) { free(lv); free(ng); return QO_ERR_INVALID_ARG; }
  for (uint64_t b = 0; b < v.nb; ++b) {
    float norm;
    uint64_t m = bucket_len(&v.p, b);
    rc = decode_bucket(&v, b, &norm, lv, ng);
    if (rc) break;
    float scale = norm / (float)v.p.s;
    for (uint64_t i = 0; i < m; ++i) {
      float mag = scale * (float)lv[i];
      g_hat[b * v.d + i] = (lv[i] != 0 && ng[i]) ? -mag : mag;
    }
  }
  free(lv);
  free(ng);
  return rc;
}

static int decode_all(const void *const *msgs, const size_t *bytes, uint32_t K,
                      uint64_t *n_out, float ***out) {
  if (K < 1 || !msgs || !bytes) return QO_ERR_INVALID_ARG;
  view v0;
  int rc = open_msg(msgs[0], bytes[0], &v0);
  if (rc) return rc;
  float **dec = (float **)calloc(K, sizeof(float *));
  if (!dec) return QO_ERR_INVALID_ARG;
  for (uint32_t k = 0; k < K && rc == QO_OK; ++k) {
    view vk;
    rc = open_msg(msgs[k], bytes[k], &vk);
    if (rc) break;
    if (vk.p.n != v0.p.n) { rc = QO_ERR_INVALID_ARG; break; }
    dec[k] = (float *)malloc((vk.p.n ? vk.p.n : 1) * sizeof(float));
    if (!dec[k]) { rc = QO_ERR_INVALID_ARG; break; }
    rc = qo_decode(msgs[k], bytes[k], dec[k]);
  }
  if (rc) {
    for (uint32_t k = 0; k < K; ++k) free(dec[k]);
    free(dec);
    return rc;
  }
  *n_out = v0.p.n;
  *out = dec;
  return QO_OK;
}

int qo_decode_accumulate(const void *const *msgs, const size_t *bytes, uint32_t K,
                         float *acc) {
  uint64_t n;
  float **dec;
  int rc = decode_all(msgs, bytes, K, &n, &dec);
  if (rc) return rc;
  for (uint64_t i = 0; i < n; ++i) {
    float sum = 0.0f;
    for (uint32_t k = 0; k < K; ++k) sum += dec[k][i];
    acc[i] = acc[i] + sum;
  }
  for (uint32_t k = 0; k < K; ++k) free(dec[k]);
  free(dec);
  return QO_OK;
}

/* Algorithm 1, last line: x <- x - (eta/K) * sum_l g_hat^l. */
int qo_sgd_step(const void *const *msgs, const size_t *bytes, uint32_t K, float eta,
                float *x) {
  uint64_t n;
  float **dec;
  int rc = decode_all(msgs, bytes, K, &n, &dec);
  if (rc) return rc;
  float c = eta / (float)K;
  for (uint64_t i = 0; i < n; ++i) {
    float sum = 0.0f;
    for (uint32_t k = 0; k < K; ++k) sum += dec[k][i];
    x[i] = fmaf(-c, sum, x[i]);
  }
  for (uint32_t k = 0; k < K; ++k) free(dec[k]);
  free(dec);
  return QO_OK;
}

/* The same step restricted to the buckets [bucket_begin, bucket_begin + bucket_count):
 * buckets are quantized and coded independently (Sec. 4), so the update of the
 * coordinates of a run of buckets only needs those buckets' strings.  x points at the
 * first coordinate of bucket `bucket_begin`.  Same arithmetic as qo_sgd_step, one
 * bucket at a time. */
int qo_sgd_step_buckets(const void *const *msgs, const size_t *bytes, uint32_t K, float eta,
                        float *x, uint64_t bucket_begin, uint64_t bucket_count) {
  if (K < 1 || !msgs || !bytes || !x) return QO_ERR_INVALID_ARG;
  view *vs = (view *)calloc(K, sizeof(view));
  if (!vs) return QO_ERR_INVALID_ARG;
  int rc = QO_OK;
  for (uint32_t k = 0; k < K && rc == QO_OK; ++k) {
    rc = open_msg(msgs[k], bytes[k], &vs[k]);
    if (rc == QO_OK && (vs[k].p.n != vs[0].p.n || vs[k].d != vs[0].d)) rc = QO_ERR_INVALID_ARG;
  }
  if (rc == QO_OK && (bucket_begin > vs[0].nb || bucket_count > vs[0].nb - bucket_begin))
    rc = QO_ERR_INVALID_ARG;
  if (rc) { free(vs); return rc; }
  uint64_t d = vs[0].d ? vs[0].d : 1;
  uint32_t *lv = (uint32_t *)malloc(d * sizeof(uint32_t));
  uint8_t *ng = (uint8_t *)malloc(d);
  float *dec = (float *)malloc((size_t)K * d * sizeof(float));
  if (!lv || !ng || !dec) { free(lv); free(ng); free(dec); free(vs); return QO_ERR_INVALID_ARG; }
  float c = eta / (float)K;
  for (uint64_t b = bucket_begin; b < bucket_begin + bucket_count && rc == QO_OK; ++b) {
    uint64_t m = bucket_len(&vs[0].p, b);
    for (uint32_t k = 0; k < K && rc == QO_OK; ++k) {
      float norm;
      rc = decode_bucket(&vs[k], b, &norm, lv, ng);
      if (rc) break;
      float scale = norm / (float)vs[k].p.s;
      for (uint64_t i = 0; i < m; ++i) {
        float mag = scale * (float)lv[i];
        dec[(size_t)k * d + i] = (lv[i] != 0 && ng[i]) ? -mag : mag;
      }
    }
    if (rc) break;
    float *xb = x + (b - bucket_begin) * vs[0].d;
    for (uint64_t i = 0; i < m; ++i) {
      float sum = 0.0f;
      for (uint32_t k = 0; k < K; ++k) sum += dec[(size_t)k * d + i];
      xb[i] = fmaf(-c, sum, xb[i]);
    }
  }
  free(lv); free(ng); free(dec); free(vs);
  return rc;
}

/* ------------------------------------------------------------------------- */
/* Tensor-aware messages (Sec. 5, "Protocol": matrices with fewer than 10K      */
/* elements are not quantized; quantization buckets are laid out per matrix).  */
/*                                                                             */
/* The gradient is an arena of p->n floats in which tensor j occupies           */
/* [offset_j, offset_j + size_j).  A tensor with size < bypass_below goes into  */
/* the message as raw fp32; any other tensor is cut into buckets of d values    */
/* that restart at the tensor's first value (its last bucket is shorter), so    */
/* no bucket mixes two tensors' scales.  Draws are indexed by arena position.   */
/* Message (version 2): header as before with nb = number of such buckets and  */
/* payload words = strings + raw words; offset table (Elias codes); bucket      */
/* strings in tensor order; then the raw tensors in tensor order.               */
/* ------------------------------------------------------------------------- */

static int layout_check(const qo_params *p, const qo_tensor *t, uint32_t T) {
  int rc = check_params(p);
  if (rc) return rc;
  if (T && !t) return QO_ERR_INVALID_ARG;
  uint64_t prev_end = 0;
  for (uint32_t j = 0; j < T; ++j) { /* ascending, disjoint, inside the arena */
    if (t[j].offset < prev_end || t[j].size > p->n || t[j].offset > p->n - t[j].size)
      return QO_ERR_INVALID_ARG;
    prev_end = t[j].offset + t[j].size;
  }
  return QO_OK;
}

int qo_layout_counts(const qo_params *p, const qo_tensor *t, uint32_t T,
                     uint64_t bypass_below, uint64_t *buckets, uint64_t *raw_elems) {
  int rc = layout_check(p, t, T);
  if (rc) return rc;
  uint64_t nb = 0, raw = 0;
  for (uint32_t j = 0; j < T; ++j) {
    if (t[j].size < bypass_below) raw += t[j].size;
    else nb += (t[j].size + p->d - 1) / p->d;
  }
  if (buckets) *buckets = nb;
  if (raw_elems) *raw_elems = raw;
  return QO_OK;
}

static uint64_t layout_table_words(const qo_params *p, uint64_t nb) {
  if (p->code == QO_CODE_FIXED) return 0;
  return (nb + 1 + 3) & ~(uint64_t)3;
}

size_t qo_layout_max_encoded_bytes(const qo_params *p, const qo_tensor *t, uint32_t T,
                                   uint64_t bypass_below) {
  uint64_t nb, raw;
  if (qo_layout_counts(p, t, T, bypass_below, &nb, &raw)) return 0;
  uint64_t words = 0, full = bucket_max_words(p, p->d);
  for (uint32_t j = 0; j < T; ++j) {
    if (t[j].size < bypass_below) continue;
    uint64_t q = t[j].size / p->d, r = t[j].size % p->d;
    words += q * full;
    if (r) words += p->code == QO_CODE_FIXED ? full : bucket_max_words(p, r);
  }
  return (size_t)(4 * (H_WORDS + layout_table_words(p, nb) + words + raw));
}

int qo_encode_layout(const qo_params *p, const qo_tensor *t, uint32_t T,
                     uint64_t bypass_below, const float *arena, void *msg,
                     size_t capacity, size_t *bytes_out) {
  uint64_t nb, raw;
  int rc = qo_layout_counts(p, t, T, bypass_below, &nb, &raw);
  if (rc) return rc;
  uint64_t d = p->d, tw = layout_table_words(p, nb);
  if (capacity < 4 * (H_WORDS + tw)) return QO_ERR_CAPACITY;
  uint32_t *w = (uint32_t *)msg;
  memset(w, 0, capacity - capacity % 4);
  uint32_t *table = w + H_WORDS;
  uint32_t *payload = table + tw;
  uint64_t cap_words = capacity / 4 - H_WORDS - tw;
  uint64_t full = (bucket_max_bits(p, d) + 31) / 32;

  uint32_t *levels = (uint32_t *)malloc(d * sizeof(uint32_t));
  uint8_t *neg = (uint8_t *)malloc(d);
  if (!levels || !neg) { free(levels); free(neg); return QO_ERR_INVALID_ARG; }
  bitw bw = {payload, cap_words * 32, 0, 0};
  uint64_t b = 0;
  for (uint32_t j = 0; j < T && rc == QO_OK; ++j) {
    if (t[j].size < bypass_below) continue;
    for (uint64_t o = 0; o < t[j].size; o += d, ++b) {
      uint64_t m = t[j].size - o < d ? t[j].size - o : d;
      uint64_t start = t[j].offset + o;
      float norm;
      quantize_bucket(p, arena + start, m, start, NULL, levels, neg, &norm, NULL, NULL);
      if (tw) table[b] = (uint32_t)(bw.pos / 32);
      else bw.pos = b * full * 32; /* fixed width: bucket b sits at b * words(full bucket) */
      code_bucket(p, m, norm, levels, neg, &bw);
      bw.pos = (bw.pos + 31) & ~(uint64_t)31;
      if (bw.overflow || bw.pos > bw.cap) { rc = QO_ERR_CAPACITY; break; }
    }
  }
  free(levels);
  free(neg);
  if (rc) return rc;
  uint64_t strings = tw ? bw.pos / 32 : nb * full;
  if (tw) table[nb] = (uint32_t)strings;
  if (strings + raw > cap_words) return QO_ERR_CAPACITY;
  uint64_t r = 0;
  for (uint32_t j = 0; j < T; ++j) { /* the small tensors, as they are */
    if (t[j].size >= bypass_below) continue;
    memcpy(payload + strings + r, arena + t[j].offset, t[j].size * 4);
    r += t[j].size;
  }
  uint64_t pw = strings + raw;
  w[H_MAGIC] = QO_MAGIC; w[H_VERSION] = 2; w[H_CODE] = p->code; w[H_NORM] = p->norm;
  w[H_S] = p->s; w[H_STREAM] = p->stream_id;
  w[H_D_LO] = (uint32_t)d; w[H_D_HI] = (uint32_t)(d >> 32);
  w[H_N_LO] = (uint32_t)p->n; w[H_N_HI] = (uint32_t)(p->n >> 32);
  w[H_NB_LO] = (uint32_t)nb; w[H_NB_HI] = (uint32_t)(nb >> 32);
  w[H_PW_LO] = (uint32_t)pw; w[H_PW_HI] = (uint32_t)(pw >> 32);
  w[H_STATUS] = 0; w[H_ITER] = p->iteration;
  if (bytes_out) *bytes_out = (size_t)(4 * (H_WORDS + tw + pw));
  return QO_OK;
}

/* Values of one message at their arena positions; positions outside every
 * tensor are left as they are. */
int qo_decode_layout(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                     const void *msg, size_t bytes, float *arena_out) {
  if (!msg || bytes < 4 * H_WORDS) return QO_ERR_CORRUPT;
  const uint32_t *w = (const uint32_t *)msg;
  if (w[H_MAGIC] != QO_MAGIC || w[H_VERSION] != 2 || w[H_STATUS] != 0) return QO_ERR_CORRUPT;
  view v;
  memset(&v, 0, sizeof v);
  v.p.code = w[H_CODE]; v.p.norm = w[H_NORM]; v.p.s = w[H_S];
  v.p.stream_id = w[H_STREAM]; v.p.iteration = w[H_ITER];
  v.p.d = w[H_D_LO] | ((uint64_t)w[H_D_HI] << 32);
  v.p.n = w[H_N_LO] | ((uint64_t)w[H_N_HI] << 32);
  uint64_t nb, raw;
  if (qo_layout_counts(&v.p, t, T, bypass_below, &nb, &raw)) return QO_ERR_CORRUPT;
  if ((w[H_NB_LO] | ((uint64_t)w[H_NB_HI] << 32)) != nb) return QO_ERR_CORRUPT;
  v.d = v.p.d; v.nb = nb;
  v.tw = layout_table_words(&v.p, nb);
  v.pw = w[H_PW_LO] | ((uint64_t)w[H_PW_HI] << 32);
  if ((uint64_t)bytes / 4 < H_WORDS + v.tw + v.pw) return QO_ERR_CORRUPT;
  v.table = w + H_WORDS;
  v.payload = v.table + v.tw;
  uint64_t full = (bucket_max_bits(&v.p, v.d) + 31) / 32;
  uint64_t strings = v.tw ? v.table[nb] : nb * full;
  if (strings + raw != v.pw) return QO_ERR_CORRUPT;

  uint32_t *lv = (uint32_t *)malloc(v.d * sizeof(uint32_t));
  uint8_t *ng = (uint8_t *)malloc(v.d);
  if (!lv || !ng) { free(lv); free(ng); return QO_ERR_INVALID_ARG; }
  int rc = QO_OK;
  uint64_t b = 0, r = 0;
  for (uint32_t j = 0; j < T && rc == QO_OK; ++j) {
    if (t[j].size < bypass_below) {
      memcpy(arena_out + t[j].offset, v.payload + strings + r, t[j].size * 4);
      r += t[j].size;
      continue;
    }
    for (uint64_t o = 0; o < t[j].size && rc == QO_OK; o += v.d, ++b) {
      uint64_t m = t[j].size - o < v.d ? t[j].size - o : v.d;
      float norm;
      rc = decode_bucket_m(&v, b, m, &norm, lv, ng);
      if (rc) break;
      float scale = norm / (float)v.p.s;
      float *out = arena_out + t[j].offset + o;
      for (uint64_t i = 0; i < m; ++i) {
        float mag = scale * (float)lv[i];
        out[i] = (lv[i] != 0 && ng[i]) ? -mag : mag;
      }
    }
  }
  free(lv);
  free(ng);
  return rc;
}

/* acc_i <- acc_i + sum_l (message l at i)   (step == 0), or
 * x_i <- fma(-(eta/K), sum_l (message l at i), x_i)   (Algorithm 1, last line),
 * over the positions that belong to a tensor; the sum runs over l ascending. */
static int layout_reduce(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                         const void *const *msgs, const size_t *bytes, uint32_t K,
                         int step, float eta, float *x) {
  if (K < 1 || !msgs || !bytes || bytes[0] < 4 * H_WORDS) return QO_ERR_INVALID_ARG;
  const uint32_t *w0 = (const uint32_t *)msgs[0];
  uint64_t n = w0[H_N_LO] | ((uint64_t)w0[H_N_HI] << 32);
  float **dec = (float **)calloc(K, sizeof(float *));
  if (!dec) return QO_ERR_INVALID_ARG;
  int rc = QO_OK;
  for (uint32_t k = 0; k < K && rc == QO_OK; ++k) {
    const uint32_t *wk = (const uint32_t *)msgs[k];
    if (bytes[k] < 4 * H_WORDS || (wk[H_N_LO] | ((uint64_t)wk[H_N_HI] << 32)) != n) {
      rc = QO_ERR_INVALID_ARG;
      break;
    }
    dec[k] = (float *)calloc(n ? n : 1, sizeof(float));
    if (!dec[k]) { rc = QO_ERR_INVALID_ARG; break; }
    rc = qo_decode_layout(t, T, bypass_below, msgs[k], bytes[k], dec[k]);
  }
  if (rc == QO_OK) {
    float c = eta / (float)K;
    for (uint32_t j = 0; j < T; ++j) {
      for (uint64_t i = t[j].offset; i < t[j].offset + t[j].size; ++i) {
        float sum = 0.0f;
        for (uint32_t k = 0; k < K; ++k) sum += dec[k][i];
        x[i] = step ? fmaf(-c, sum, x[i]) : x[i] + sum;
      }
    }
  }
  for (uint32_t k = 0; k < K; ++k) free(dec[k]);
  free(dec);
  return rc;
}

int qo_decode_accumulate_layout(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                                const void *const *msgs, const size_t *bytes, uint32_t K,
                                float *acc) {
  return layout_reduce(t, T, bypass_below, msgs, bytes, K, 0, 0.0f, acc);
}

int qo_sgd_step_layout(const qo_tensor *t, uint32_t T, uint64_t bypass_below,
                       const void *const *msgs, const size_t *bytes, uint32_t K, float eta,
                       float *x) {
  return layout_reduce(t, T, bypass_below, msgs, bytes, K, 1, eta, x);
}
