/*
 * Driver for running the QSGD CPU oracle under -fsanitize=address,undefined
 * (TEST INFRASTRUCTURE ONLY, like the oracle itself).  It walks every code
 * (Code_s, Code'_s, fixed width), both scalings, short and ragged buckets, a
 * long single bucket with its entry list, the slice and bucket-range calls and
 * the tensor-aware container, and checks the round trip
 * Decode(Encode(v)) = Q_s(v) on the way, so that the pointer arithmetic into
 * the message (fixed-width planes, entry lists, tables) is exercised with
 * red zones around every buffer.  Exit status 0 = no finding and every check held.
 *
 *   gcc -g -O1 -std=c99 -fsanitize=address,undefined -fno-sanitize-recover=all \
 *       -static-libasan -ffp-contract=off sanitize_check.c qsgd_oracle.c -lm
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "qsgd_oracle.h"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double rnd(void) { /* xorshift64*, uniform in (0,1) */
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return ((rng_state * 0x2545F4914F6CDD1Dull) >> 11) * (1.0 / 9007199254740992.0) + 1e-17;
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(rnd())) * cos(6.283185307179586 * rnd())); }

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

static void one_case(uint64_t n, uint32_t s, uint64_t d, uint32_t code, uint32_t norm, double density) {
  qo_params p;
  memset(&p, 0, sizeof p);
  p.n = n; p.s = s; p.d = d; p.code = code; p.norm = norm; p.seed = 77; p.stream_id = 3; p.iteration = 5;
  float *g = (float *)malloc((n ? n : 1) * sizeof(float));
  for (uint64_t i = 0; i < n; ++i) g[i] = (rnd() < density ? 40.0f : 0.01f) * gauss();
  size_t cap = qo_max_encoded_bytes(&p), used = 0;
  /* exactly `cap` bytes: a write past the worst case lands in the red zone */
  void *msg = malloc(cap ? cap : 1);
  CHECK(qo_encode(&p, g, msg, cap, &used) == QO_OK);
  CHECK(used <= cap);
  /* the reader gets exactly the used bytes */
  void *tight = malloc(used ? used : 1);
  memcpy(tight, msg, used);
  uint64_t nb = qo_num_buckets(&p);
  uint32_t *lev = (uint32_t *)malloc((n ? n : 1) * 4), *lev2 = (uint32_t *)malloc((n ? n : 1) * 4);
  uint8_t *neg = (uint8_t *)malloc(n ? n : 1), *neg2 = (uint8_t *)malloc(n ? n : 1);
  float *norms = (float *)malloc((nb ? nb : 1) * 4), *norms2 = (float *)malloc((nb ? nb : 1) * 4);
  CHECK(qo_quantize(&p, g, NULL, lev, neg, norms, NULL, NULL) == QO_OK);
  CHECK(qo_decode_tuple(tight, used, lev2, neg2, norms2) == QO_OK);
  for (uint64_t i = 0; i < n; ++i) {
    CHECK(lev[i] == lev2[i]);
    if (code != QO_CODE_SPARSE || lev[i]) CHECK(neg[i] == neg2[i]);
  }
  for (uint64_t b = 0; b < nb; ++b) CHECK(memcmp(&norms[b], &norms2[b], 4) == 0);
  /* step over the whole vector and over bucket ranges */
  float *x = (float *)malloc((n ? n : 1) * 4), *y = (float *)malloc((n ? n : 1) * 4);
  for (uint64_t i = 0; i < n; ++i) x[i] = y[i] = gauss();
  const void *msgs[2] = {tight, tight};
  size_t sizes[2] = {used, used};
  CHECK(qo_sgd_step(msgs, sizes, 2, 0.1f, x) == QO_OK);
  uint64_t deff = qo_bucket_size(&p);
  for (uint64_t b0 = 0; b0 < nb; b0 += 3) {
    uint64_t cnt = nb - b0 < 3 ? nb - b0 : 3;
    CHECK(qo_sgd_step_buckets(msgs, sizes, 2, 0.1f, y + b0 * deff, b0, cnt) == QO_OK);
  }
  CHECK(memcmp(x, y, n * 4) == 0);
  /* a slice that starts on a bucket boundary */
  if (nb >= 3) {
    qo_params q = p;
    uint64_t b0 = nb / 2;
    q.n = n - b0 * deff;
    size_t cap2 = qo_max_encoded_bytes(&q), used2 = 0;
    void *m2 = malloc(cap2);
    CHECK(qo_encode_slice(&q, g + b0 * deff, b0 * deff, m2, cap2, &used2) == QO_OK);
    uint64_t off, cnt, off2, cnt2, pay, pay2;
    CHECK(qo_bucket_extent(tight, used, b0, &off, &cnt) == QO_OK);
    CHECK(qo_bucket_extent(m2, used2, 0, &off2, &cnt2) == QO_OK);
    CHECK(qo_payload_offset(tight, used, &pay) == QO_OK && qo_payload_offset(m2, used2, &pay2) == QO_OK);
    CHECK(cnt == cnt2);
    if (cnt == cnt2)
      CHECK(memcmp((const char *)tight + pay + 4 * off, (const char *)m2 + pay2 + 4 * off2, 4 * cnt) == 0);
    free(m2);
  }
  /* truncated and damaged messages must be refused, not read past */
  if (used > 64) {
    float *sink = (float *)malloc((n ? n : 1) * 4);
    void *cut = malloc(used - 4);
    memcpy(cut, msg, used - 4);
    CHECK(qo_decode(cut, used - 4, sink) != QO_OK);
    free(cut);
    free(sink);
  }
  free(g); free(msg); free(tight); free(lev); free(lev2); free(neg); free(neg2);
  free(norms); free(norms2); free(x); free(y);
}

static void layout_case(uint32_t code) {
  qo_tensor t[5] = {{0, 37}, {40, 5000}, {5040, 9}, {5052, 777}, {5832, 2049}};
  uint64_t n = 5832 + 2049;
  qo_params p;
  memset(&p, 0, sizeof p);
  p.n = n; p.s = code == QO_CODE_FIXED ? 16 : 5; p.d = 512; p.code = code; p.seed = 9;
  float *g = (float *)malloc(n * 4), *out = (float *)malloc(n * 4), *x = (float *)malloc(n * 4);
  for (uint64_t i = 0; i < n; ++i) { g[i] = 0.01f * gauss(); x[i] = gauss(); }
  size_t cap = qo_layout_max_encoded_bytes(&p, t, 5, 600), used = 0;
  void *msg = malloc(cap);
  CHECK(qo_encode_layout(&p, t, 5, 600, g, msg, cap, &used) == QO_OK);
  void *tight = malloc(used);
  memcpy(tight, msg, used);
  CHECK(qo_decode_layout(t, 5, 600, tight, used, out) == QO_OK);
  for (uint64_t i = 0; i < 37; ++i) CHECK(out[i] == g[i]);   /* a raw tensor comes back as it was */
  const void *msgs[1] = {tight};
  size_t sizes[1] = {used};
  CHECK(qo_sgd_step_layout(t, 5, 600, msgs, sizes, 1, 0.5f, x) == QO_OK);
  free(g); free(out); free(x); free(msg); free(tight);
}

int main(void) {
  for (uint32_t code = 0; code < 3; ++code)
    for (uint32_t norm = 0; norm < 2; ++norm) {
      one_case(0, 4, 512, code, norm, 0.0);
      one_case(1, 1, 1, code, norm, 0.0);
      one_case(700, 4, 512, code, norm, 0.01);
      one_case(3000, 16, 512, code, norm, 0.0);
      one_case(1500, 256, 512, code, norm, 0.0);
      one_case(777, 3, 100, code, norm, 0.2);
      one_case(9000, 4, 8192, code, norm, 0.01);
      one_case(2600, 65535, 64, code, norm, 0.0);
      if (code != QO_CODE_FIXED) {                 /* long buckets: entry lists */
        one_case(300000, 1, 300000, code, norm, 0.01);
        one_case(70001, 3, 30000, code, norm, 0.2);
      }
    }
  for (uint32_t code = 0; code < 3; ++code) layout_case(code);
  printf(failures ? "sanitize_check: %d checks failed\n" : "sanitize_check: ok\n", failures);
  return failures ? 1 : 0;
}
