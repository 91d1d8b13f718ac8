// C ABI of libqsgd (see include/qsgd.h): parameter checks, geometry, kernel
// launches.  Scratch is the caller's; the only device memory allocated here is the two
// small tables of a tensor layout (qsgd_layout_create).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "qsgd.h"
#include "qsgd_device.hpp"
#include "qsgd_encode_wave.hpp"
#include "qsgd_kernels.hpp"

// Tensor-aware messages: where the tensors sit in the arena, which of them are
// quantized (and the buckets they are cut into) and which travel raw.  The tables
// live on the device the layout was created on.
struct qsgd_layout {
  uint64_t d = 0, bypass = 0;
  uint64_t extent = 0;        // one past the last arena position a tensor uses
  uint64_t nb = 0;            // quantization buckets
  uint64_t short_buckets = 0; // buckets with fewer than d values ...
  uint64_t short_values = 0;  // ... and the values in them
  uint64_t raw = 0;           // raw fp32 values
  uint32_t R = 0;             // pieces of raw tensors
  int device = 0;
  uint2* btab = nullptr;      // per bucket: (start / 4, length)
  uint4* rtab = nullptr;      // per piece of a raw tensor: (start / 4, length, offset in the raw section, 0)
  std::vector<uint32_t> short_len;  // lengths of the short buckets (size accounting)
};

namespace {

using namespace qsgd;

// workspace: words appended by each team (u32) and their exclusive prefix sums (u64)
constexpr uint64_t kTotalsBytes = (uint64_t)kMaxTeams * 4 + (uint64_t)kMaxTeams * 8;
constexpr uint64_t kStatusBytes = 256;                      // workspace: decode status word

uint32_t omega_len_host(uint64_t k) {
  uint32_t len = 1;
  while (k > 1) {
    uint32_t nb = 0;
    for (uint64_t t = k; t; t >>= 1) ++nb;
    len += nb;
    k = nb - 1;
  }
  return len;
}

struct Geometry {
  uint64_t n, d;       // d: effective bucket size
  uint64_t nb;         // buckets
  uint32_t s, code, norm;
  uint32_t per_elem;   // worst-case bits per coordinate (Elias codes)
  uint32_t fixed_bits;
  uint64_t table_words;

  uint64_t bucket_len(uint64_t b) const { return std::min(d, n - b * d); }
  // Worst-case words of a bucket string of m elements.
  uint64_t max_words(uint64_t m) const {
    if (code == QSGD_CODE_FIXED) return 2 + (m * fixed_bits + 31) / 32 + (m + 31) / 32;
    const uint64_t bits = 32 + m * per_elem + (code == QSGD_CODE_SPARSE ? 1 : 0);
    uint64_t words = (bits + 31) / 32;
    if (d > kEntryMinD) {   // long buckets carry a list of entry points behind the string
      const uint64_t segs = (m + kSeg - 1) / kSeg;
      words += 2 * std::min<uint64_t>(segs ? segs - 1 : 0, bits / kEntryBits) + 1;
    }
    return words;
  }
  uint64_t max_payload_words() const {
    if (nb == 0) return 0;
    return (nb - 1) * max_words(d) + max_words(bucket_len(nb - 1));
  }
  bool bucket_path() const { return n > 0 && d % 4 == 0 && d <= kMaxBucketFast; }
};

// General path (any d): segments of kSeg values, workspace layout.
struct GenPlan {
  uint64_t spb, nseg;
  uint32_t sub_words;
  uint64_t off_partial, off_scale, off_seginfo, off_segstart, off_seggap, off_segrank,
      off_segprev, off_bents, off_slots;
  uint64_t enc_bytes;   // encode scratch (after the status block)
  uint64_t dec_bytes;   // decode scratch: dense accumulator
};

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

void plan_general(const Geometry& g, GenPlan& pl) {
  pl.spb = (g.d + kSeg - 1) / kSeg;
  pl.nseg = g.nb * pl.spb;
  const uint64_t sub_bits = (uint64_t)kSeg * g.per_elem;
  pl.sub_words = (uint32_t)(((sub_bits + 31) / 32 + 2 + 1) & ~(uint64_t)1);
  uint64_t o = 0;
  pl.off_partial = o; o = align_up(o + 8 * pl.nseg, 256);
  pl.off_scale = o; o = align_up(o + 4 * g.nb, 256);
  pl.off_seginfo = o; o = align_up(o + 12 * pl.nseg, 256);
  pl.off_segstart = o; o = align_up(o + 8 * pl.nseg, 256);
  pl.off_seggap = o; o = align_up(o + 4 * pl.nseg, 256);
  pl.off_segrank = o; o = align_up(o + 4 * pl.nseg, 256);
  pl.off_segprev = o; o = align_up(o + 4 * pl.nseg, 256);
  pl.off_bents = o; o = align_up(o + 4 * g.nb, 256);
  pl.off_slots = o;
  if (g.code != QSGD_CODE_FIXED) o = align_up(o + 4 * pl.nseg * pl.sub_words, 256);
  pl.enc_bytes = o;
  // decode: the dense accumulator, then a list per long bucket (see kCollide)
  pl.dec_bytes = g.code == QSGD_CODE_FIXED ? 0 : align_up(4 * g.n, 256);
  if (g.code == QSGD_CODE_SPARSE && g.d > kEntryMinD) pl.dec_bytes += g.nb * (uint64_t)kCollideBytes;
}

int make_geometry(const qsgd_params* p, Geometry& g) {
  if (!p) return QSGD_ERR_INVALID_ARG;
  if (p->s < 1 || p->s > 65535 || p->d < 1 || p->n > 0xFFFFFFFFull ||
      p->code > QSGD_CODE_FIXED || p->norm > QSGD_NORM_MAX || p->reserved != 0)
    return QSGD_ERR_INVALID_ARG;
  g.n = p->n;
  g.d = p->n == 0 ? p->d : std::min<uint64_t>(p->d, p->n);
  g.nb = p->n == 0 ? 0 : (p->n + g.d - 1) / g.d;
  g.s = p->s; g.code = p->code; g.norm = p->norm;
  g.fixed_bits = fixed_field_bits(p->s, p->norm);
  if (p->code == QSGD_CODE_SPARSE) g.per_elem = 2 + omega_len_host(p->s);
  else if (p->code == QSGD_CODE_DENSE) g.per_elem = 1 + omega_len_host((uint64_t)p->s + 1);
  else g.per_elem = 0;
  g.table_words = p->code == QSGD_CODE_FIXED ? 0 : ((g.nb + 1 + 3) & ~(uint64_t)3);
  return QSGD_OK;
}

// Team shape of the bucket path: TW wavefronts x CPW chunks of 256 cover d.
void team_shape(uint64_t d, int& tw, int& cpw) {
  const uint64_t chunks = (d + kChunk - 1) / kChunk;
  if (chunks <= 1) { tw = 1; cpw = 1; }
  else if (chunks <= 2) { tw = 1; cpw = 2; }
  else if (chunks <= 4) { tw = 1; cpw = 4; }
  else if (chunks <= 8) { tw = 1; cpw = 8; }
  else if (chunks <= 16) { tw = 2; cpw = 8; }
  else { tw = 4; cpw = 8; }
}

int device_cus() {
  static int cus[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cus[dev] == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      v = 256;
    cus[dev] = v;
  }
  return cus[dev];
}

struct EncodePlan {
  int tw, cpw;
  uint32_t teams, bper;
  uint64_t region_words;
  uint32_t dst_words, sub_words;
  uint32_t ring;   // records in a wavefront's survivor ring (Code_s)
  size_t lds;
  uint64_t ws_bytes;
};

// `teams_target` <= kMaxTeams.  `ws_avail`: bytes of workspace behind the status block; a
// workspace below the worst case gives every team an equal, smaller region.
void plan_encode(const Geometry& g, uint32_t teams_target, uint64_t ws_avail, EncodePlan& pl) {
  team_shape(g.d, pl.tw, pl.cpw);
  const uint32_t nb = (uint32_t)g.nb;
  const uint32_t t = std::max(1u, std::min(nb, teams_target));
  pl.bper = (nb + t - 1) / t;
  pl.teams = (nb + pl.bper - 1) / pl.bper;
  if (g.code == QSGD_CODE_FIXED) {
    pl.region_words = 0; pl.dst_words = 2; pl.sub_words = 2;
    pl.ws_bytes = kTotalsBytes;
  } else {
    pl.region_words = ((uint64_t)pl.bper * g.max_words(g.d) + 3) & ~(uint64_t)3;
    pl.dst_words = (uint32_t)((g.max_words(g.d) + 2 + 1) & ~(uint64_t)1);
    const uint64_t sub_bits = (uint64_t)pl.cpw * kChunk * g.per_elem;
    pl.sub_words = (uint32_t)(((sub_bits + 31) / 32 + 2 + 1) & ~(uint64_t)1);
    if (ws_avail >= kTotalsBytes) {
      const uint64_t share = ((ws_avail - kTotalsBytes) / 4 / pl.teams) & ~(uint64_t)3;
      pl.region_words = std::min(pl.region_words, share);
    }
    pl.ws_bytes = kTotalsBytes + (uint64_t)pl.teams * pl.region_words * 4;
  }
  // Code_s where several wavefronts share a bucket: the survivors of all of a wavefront's
  // chunks are listed before they are coded when the list is expected to be at most half
  // full, the share of nonzero levels being at most s (s + sqrt(d)) / d (Lemma 3.1 (iii));
  // a wavefront whose list overflows after all starts over with the direct coder.
  pl.ring = 0;
  const uint32_t list = qsgd::list_records(pl.cpw);
  if (g.code == QSGD_CODE_SPARSE && pl.tw >= 2 &&
      2.0 * g.s * (g.s + std::sqrt((double)g.d)) * (pl.cpw * kChunk) <= (double)g.d * list)
    pl.ring = list;
  const size_t ring_words =
      g.code == QSGD_CODE_SPARSE ? qsgd::ring_words(pl.ring ? pl.ring : qsgd::kRing) : 0;
  pl.lds = 4 * ((size_t)pl.dst_words + (size_t)pl.tw * (pl.sub_words + ring_words)) + 8 * pl.tw +
           16 * pl.tw + 16 + (g.code == QSGD_CODE_SPARSE ? 4 * qsgd::kOmegaTab : 0);
}

// ---- optional kernel timing -----------------------------------------------------
// Event pairs are made when timing is switched on (and kept for reuse), so that a timed
// loop creates none.
struct TimedLaunch { std::string name; hipEvent_t start, stop; };
struct EventPair { hipEvent_t start, stop; };
std::mutex g_timing_mu;
bool g_timing_on = false;
std::vector<TimedLaunch> g_launches;
std::vector<EventPair> g_spare;
constexpr size_t kSpareEvents = 1024;

struct ScopedTiming {
  hipStream_t st; bool on; TimedLaunch t;
  ScopedTiming(const char* name, hipStream_t s) : st(s), on(false) {
    std::lock_guard<std::mutex> lk(g_timing_mu);
    if (!g_timing_on) return;
    if (!g_spare.empty()) {
      t.start = g_spare.back().start; t.stop = g_spare.back().stop;
      g_spare.pop_back();
    } else {
      if (hipEventCreate(&t.start) != hipSuccess) return;
      if (hipEventCreate(&t.stop) != hipSuccess) { (void)hipEventDestroy(t.start); return; }
    }
    t.name = name;
    on = hipEventRecord(t.start, st) == hipSuccess;
    if (!on) g_spare.push_back({t.start, t.stop});
  }
  ~ScopedTiming() {
    if (!on) return;
    (void)hipEventRecord(t.stop, st);
    std::lock_guard<std::mutex> lk(g_timing_mu);
    g_launches.push_back(t);
  }
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Geometry of a tensor-aware message: the layout says how many buckets there are.
int layout_geometry(const qsgd_params* p, const qsgd_layout* L, Geometry& g) {
  int rc = make_geometry(p, g);
  if (rc) return rc;
  if (!L) return QSGD_OK;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return QSGD_ERR_HIP;
  if (dev != L->device || p->d != L->d || p->n < L->extent) return QSGD_ERR_INVALID_ARG;
  g.d = L->d;
  g.nb = L->nb;
  g.table_words = p->code == QSGD_CODE_FIXED ? 0 : ((g.nb + 1 + 3) & ~(uint64_t)3);
  return QSGD_OK;
}

// Worst-case words of all bucket strings of a tensor-aware message.
uint64_t layout_string_words(const Geometry& g, const qsgd_layout* L) {
  if (g.code == QSGD_CODE_FIXED) return g.nb * g.max_words(g.d);   // one full slot per bucket
  uint64_t w = (g.nb - L->short_buckets) * g.max_words(g.d);
  for (uint32_t m : L->short_len) w += g.max_words(m);
  return w;
}

RawArgs raw_args(const Geometry& g, const qsgd_layout* L) {
  RawArgs r;
  std::memset(&r, 0, sizeof r);
  r.rtab = L->rtab; r.R = L->R; r.raw_words = L->raw;
  r.fixed_strings = g.code == QSGD_CODE_FIXED ? g.nb * g.max_words(g.d) : 0;
  r.nb = (uint32_t)g.nb;
  return r;
}

int run_decode(const qsgd_params* p, const qsgd_layout* L, const void* const* msgs_dev,
               const size_t* msg_bytes, uint32_t K, float c, uint32_t step, float* x_dev,
               void* ws, size_t ws_bytes, void* hip_stream) {
  Geometry g;
  int rc = layout_geometry(p, L, g);
  if (rc) return rc;
  if (L && !g.bucket_path()) return QSGD_ERR_UNSUPPORTED;
  if (!msgs_dev || !msg_bytes || K < 1 || K > QSGD_MAX_PEERS || !ws || !aligned16(ws))
    return QSGD_ERR_INVALID_ARG;
  if (g.n > 0 && (!x_dev || !aligned16(x_dev))) return QSGD_ERR_INVALID_ARG;
  if (ws_bytes < (L ? qsgd_layout_workspace_bytes(p, L, K) : qsgd_workspace_bytes(p, K)))
    return QSGD_ERR_CAPACITY;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);

  DecodeArgs a;
  std::memset(&a, 0, sizeof a);
  for (uint32_t k = 0; k < K; ++k) {
    if (!msgs_dev[k] || !aligned16(msgs_dev[k])) return QSGD_ERR_INVALID_ARG;
    a.msgs[k] = static_cast<const uint32_t*>(msgs_dev[k]);
    a.msg_words[k] = msg_bytes[k] / 4;
  }
  a.K = K; a.n = g.n; a.d = (uint32_t)g.d; a.nb = (uint32_t)g.nb; a.s = g.s; a.code = g.code;
  a.norm_mode = g.norm; a.table_words = (uint32_t)g.table_words;
  a.btab = L ? L->btab : nullptr;
  a.version = L ? 2 : 1;
  a.raw_words = L ? L->raw : 0;
  a.x = x_dev; a.c = c; a.step = step;
  a.status = static_cast<uint32_t*>(ws);
  a.fixed_bits = g.fixed_bits;
  a.fixed_words_full = (uint32_t)g.max_words(g.d);
  // Which apply step the Elias decoder takes.  The share of nonzero levels of Q_s grows
  // like s / sqrt(d) (Lemma 3.1 (iii)); above 1/8 a string has more records per
  // 256-position window than the counting apply handles well, and Code'_s has a
  // record for every coordinate.  (The counting apply keeps a bit per message in a 32-bit
  // word: more than 32 messages go the other way whatever the data.)
  a.kloop = (g.code == QSGD_CODE_DENSE || 64ull * g.s * g.s > g.d || K > 32) ? 1u : 0u;

  {
    ScopedTiming tm("decode_check", st);
    if (launch_decode_check(a, st) != hipSuccess) return QSGD_ERR_HIP;
  }
  if (g.n == 0) return QSGD_OK;
  const uint32_t cus = (uint32_t)device_cus();
  if (L && L->R) {   // the small tensors: raw values behind the strings
    ScopedTiming tm("decode_raw", st);
    if (launch_raw_apply(a, raw_args(g, L), st) != hipSuccess) return QSGD_ERR_HIP;
  }
  if (g.nb == 0) return QSGD_OK;
  if (!g.bucket_path()) {
    const uint32_t blocks = (uint32_t)std::min<uint64_t>((g.n + 255) / 256, (uint64_t)cus * 32);
    ScopedTiming tm("decode_general", st);
    if (g.code == QSGD_CODE_FIXED) {
      if (launch_gen_decode_fixed(a, blocks, st) != hipSuccess) return QSGD_ERR_HIP;
      return QSGD_OK;
    }
    float* acc = reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + kStatusBytes + kTotalsBytes);
    // Long buckets of Code_s: a message has at most q = s (s + sqrt(d)) nonzero levels in
    // expectation (Lemma 3.1 (iii)), so about K^2 q^2 / (2 d) coordinates are hit by two
    // messages.  Where that is a few hundred at most, the K messages are read at once.
    {
      const double q = (double)g.s * ((double)g.s + std::sqrt((double)g.d));
      a.together = (g.code == QSGD_CODE_SPARSE && g.d > kEntryMinD &&
                    (double)K * K * q * q <= 512.0 * (double)g.d) ? 1u : 0u;
    }
    if (launch_gen_zero(acc, g.n, blocks, st) != hipSuccess) return QSGD_ERR_HIP;
    if (a.together) {
      uint8_t* lists = reinterpret_cast<uint8_t*>(acc) + align_up(4 * g.n, 256);
      if (launch_gen_parse_together(a, acc, lists, st) != hipSuccess) return QSGD_ERR_HIP;
    } else if (launch_gen_parse(a, acc, g.d > kEntryMinD, st) != hipSuccess) {
      return QSGD_ERR_HIP;
    }
    if (launch_gen_apply(a, acc, blocks, st) != hipSuccess) return QSGD_ERR_HIP;
    return QSGD_OK;
  }

  if (g.code == QSGD_CODE_FIXED) {
    const uint32_t blocks = (uint32_t)std::min<uint64_t>((g.nb + 3) / 4, (uint64_t)cus * QSGD_FIXED_BPC);
    ScopedTiming tm("decode_fixed", st);
    if (launch_decode_fixed(a, blocks, st) != hipSuccess) return QSGD_ERR_HIP;
    return QSGD_OK;
  }
  // Elias codes: one lane per string.
  if (a.kloop && g.s <= 127) {
    // dense strings whose levels fit a byte: the tile decoder
    const uint32_t W = QSGD_TILE_WIN;
    uint32_t gw = 1;  // buckets per wavefront: a power of two, gw * K lanes
    while (gw * 2 * K <= 64 && gw * 2 <= 16) gw *= 2;
    while (gw > 1 && (g.nb + gw - 1) / gw < (uint64_t)cus * 8) gw /= 2;
    a.tile_w = W; a.gw = gw;
    a.win = (uint32_t)std::min<uint64_t>((g.d + 3) & ~(uint64_t)3, W);
    a.winp = W;
    const size_t lds = 64 * (size_t)W + 4 * 64 * ((size_t)kStrWin + 1) + 128;   // tile, string rings, Elias table
    const uint32_t blocks = (uint32_t)((g.nb + gw - 1) / gw);
    ScopedTiming tm("decode_elias", st);
    if (launch_decode_tile(a, blocks, lds, st) != hipSuccess) return QSGD_ERR_HIP;
    return QSGD_OK;
  }
  const uint32_t win = (uint32_t)std::min<uint64_t>((g.d + 3) & ~(uint64_t)3, 256);
  const uint32_t winp = (win + kChunk - 1) / kChunk * kChunk;
  uint32_t gw = 1;  // buckets per wavefront: a power of two, gw * K lanes, gw * winp floats
  while (gw * 2 * K <= 64 && gw * 2 <= 16) gw *= 2;
  while (gw > 1 && (g.nb + gw - 1) / gw < (uint64_t)cus * 8) gw /= 2;
  a.win = win; a.winp = winp; a.gw = gw; a.rec = std::min(16u, 64u / gw);
  // LDS: accumulator, record rings, string word rings, Elias table, dump words; the message-by-message
  // apply also keeps 3 x 64 words of ring state (the counting apply does not pay for them)
  a.q16 = (g.code == QSGD_CODE_SPARSE && !a.kloop && g.s <= 4) ? 1u : 0u;
  const size_t lds = 4 * ((size_t)gw * winp + rec_words(a.q16 != 0) + 64 * (kStrWin + 1) + 32 + 64 +
                          (a.kloop ? 192 : 0));
  const uint32_t blocks = (uint32_t)((g.nb + gw - 1) / gw);
  ScopedTiming tm("decode_elias", st);
  if (launch_decode_elias(a, blocks, lds, st) != hipSuccess) return QSGD_ERR_HIP;
  return QSGD_OK;
}

}  // namespace

namespace qsgd {

int validate_encode(const qsgd_params* p, uint64_t index_base, size_t msg_capacity,
                    size_t workspace_bytes) {
  Geometry g;
  int rc = make_geometry(p, g);
  if (rc) return rc;
  if (index_base % 4) return QSGD_ERR_INVALID_ARG;
  const uint64_t fixed_part = 4 * (H_WORDS + g.table_words);
  if (msg_capacity < fixed_part) return QSGD_ERR_CAPACITY;
  const uint64_t cap_words = (msg_capacity - fixed_part) / 4;
  if (g.n == 0) return QSGD_OK;
  if (!g.bucket_path()) {
    GenPlan gp;
    plan_general(g, gp);
    if (gp.nseg > 0x7FFFFFFFull) return QSGD_ERR_UNSUPPORTED;
    if (workspace_bytes < kStatusBytes + kTotalsBytes + gp.enc_bytes) return QSGD_ERR_CAPACITY;
    if (g.code == QSGD_CODE_FIXED && cap_words < g.max_payload_words()) return QSGD_ERR_CAPACITY;
    return QSGD_OK;
  }
  if (workspace_bytes < kStatusBytes + kTotalsBytes) return QSGD_ERR_CAPACITY;
  EncodePlan pl;
  int tw, cpw;
  team_shape(g.d, tw, cpw);
  const uint32_t target = std::min<uint32_t>(kMaxTeams, (uint32_t)device_cus() * (QSGD_ENC_TEAMS / tw));
  plan_encode(g, target, workspace_bytes - kStatusBytes, pl);
  if (g.code != QSGD_CODE_FIXED && pl.region_words < std::min<uint64_t>(64, g.max_words(g.d)))
    return QSGD_ERR_CAPACITY;
  if (g.code == QSGD_CODE_FIXED && cap_words < g.max_payload_words()) return QSGD_ERR_CAPACITY;
  return QSGD_OK;
}

int validate_decode(const qsgd_params* p, uint32_t K, size_t workspace_bytes) {
  Geometry g;
  int rc = make_geometry(p, g);
  if (rc) return rc;
  if (K < 1 || K > QSGD_MAX_PEERS) return QSGD_ERR_INVALID_ARG;
  if (workspace_bytes < qsgd_workspace_bytes(p, K)) return QSGD_ERR_CAPACITY;
  return QSGD_OK;
}

}  // namespace qsgd

// Plain copy, for calibration and as the machine's copy ceiling.  Each workgroup copies
// one contiguous piece of kCopyPiece bytes, a thread has four 16-byte streaming loads in
// flight before its four stores (measured against grid-stride and cached variants on
// 8 GB: 5.6 TB/s read + write against 4.6 - 5.4).
constexpr uint64_t kCopyPiece = 16384;
__global__ __launch_bounds__(256) void k_copy_probe(float* __restrict__ dst,
                                                    const float* __restrict__ src,
                                                    uint64_t quads) {
  const uint64_t q0 = (uint64_t)blockIdx.x * (kCopyPiece / 16);
  const uint64_t q1 = min(q0 + kCopyPiece / 16, quads);
  float4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint64_t i = q0 + (uint64_t)u * 256 + threadIdx.x;
    if (i < q1) v[u] = qsgd::load_stream(src + 4 * i);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint64_t i = q0 + (uint64_t)u * 256 + threadIdx.x;
    if (i < q1) qsgd::store_stream(dst + 4 * i, v[u]);
  }
}

// The same data read with one 4-byte load per lane and written with one 4-byte store per
// lane: a second kernel of known traffic, so that the counters' factors are known for both
// request sizes the library's kernels use.
__global__ __launch_bounds__(256) void k_copy_probe_words(uint32_t* __restrict__ dst,
                                                          const uint32_t* __restrict__ src,
                                                          uint64_t words) {
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < words;
       i += (uint64_t)gridDim.x * 256)
    dst[i] = src[i];
}

extern "C" {

int qsgd_version(void) { return 100; }

const char* qsgd_strerror(int err) {
  switch (err) {
    case QSGD_OK: return "ok";
    case QSGD_ERR_INVALID_ARG: return "invalid argument";
    case QSGD_ERR_CAPACITY: return "buffer too small";
    case QSGD_ERR_CORRUPT: return "corrupt or mismatching message";
    case QSGD_ERR_HIP: return "HIP runtime error";
    case QSGD_ERR_UNSUPPORTED: return "unsupported configuration";
    case QSGD_ERR_SCRATCH: return "request exceeds the library's built-in scratch";
    default: return "unknown error";
  }
}

size_t qsgd_max_encoded_bytes(const qsgd_params* p) {
  Geometry g;
  if (make_geometry(p, g)) return 0;
  return (size_t)(4 * (H_WORDS + g.table_words + g.max_payload_words()));
}

size_t qsgd_workspace_bytes(const qsgd_params* p, uint32_t K) {
  Geometry g;
  if (make_geometry(p, g) || K > QSGD_MAX_PEERS) return 0;
  uint64_t bytes = kStatusBytes + kTotalsBytes;
  if (g.n > 0 && !g.bucket_path()) {
    GenPlan gp;
    plan_general(g, gp);
    bytes += std::max(gp.enc_bytes, gp.dec_bytes);
  } else if (g.bucket_path() && g.code != QSGD_CODE_FIXED) {
    // teams * bper < nb + teams, teams <= min(nb, kMaxTeams)
    const uint64_t slots = g.nb + std::min<uint64_t>(g.nb, kMaxTeams);
    bytes += slots * (g.max_words(g.d) + 4) * 4;
  }
  return (size_t)((bytes + 255) & ~(uint64_t)255);
}

size_t qsgd_encode_workspace_bytes(const qsgd_params* p, size_t msg_capacity) {
  Geometry g;
  if (make_geometry(p, g)) return 0;
  const size_t worst = qsgd_workspace_bytes(p, 1);
  if (!g.bucket_path() || g.code == QSGD_CODE_FIXED) return worst;
  // every team may fill four times its even share of the message, plus one worst-case string
  const uint64_t teams = std::min<uint64_t>(g.nb, kMaxTeams);
  const uint64_t share = (uint64_t)msg_capacity / 4 / teams * 4 + g.max_words(g.d) + 8;
  const uint64_t bytes = kStatusBytes + kTotalsBytes + teams * share * 4;
  return (size_t)std::min<uint64_t>(worst, (bytes + 255) & ~(uint64_t)255);
}

static int encode_impl(const qsgd_params* p, const qsgd_layout* L, uint64_t index_base,
                       const float* g_dev, void* msg_dev, size_t msg_capacity,
                       void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  Geometry g;
  int rc = layout_geometry(p, L, g);
  if (rc) return rc;
  if (L && !g.bucket_path()) return QSGD_ERR_UNSUPPORTED;
  if (index_base % 4) return QSGD_ERR_INVALID_ARG;
  const uint64_t raw_words = L ? L->raw : 0;
  if (!msg_dev || !aligned16(msg_dev) || !workspace_dev || !aligned16(workspace_dev))
    return QSGD_ERR_INVALID_ARG;
  if (g.n > 0 && (!g_dev || !aligned16(g_dev))) return QSGD_ERR_INVALID_ARG;
  const uint64_t fixed_part = 4 * (H_WORDS + g.table_words);
  if (msg_capacity < fixed_part) return QSGD_ERR_CAPACITY;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  uint32_t* header = static_cast<uint32_t*>(msg_dev);
  uint32_t* table = g.table_words ? header + H_WORDS : nullptr;
  uint32_t* payload = header + H_WORDS + g.table_words;
  const uint64_t cap_words = (msg_capacity - fixed_part) / 4;

  if (g.n == 0 && !L) {
    ScopedTiming tm("encode_empty", st);
    if (launch_write_empty(header, table, g.code, g.norm, g.s, g.d, p->stream_id, p->iteration,
                           st) != hipSuccess)
      return QSGD_ERR_HIP;
    return QSGD_OK;
  }
  if (!g.bucket_path()) {
    GenPlan gp;
    plan_general(g, gp);
    if (gp.nseg > 0x7FFFFFFFull) return QSGD_ERR_UNSUPPORTED;
    if (workspace_bytes < kStatusBytes + kTotalsBytes + gp.enc_bytes) return QSGD_ERR_CAPACITY;
    if (g.code == QSGD_CODE_FIXED && cap_words < g.max_payload_words()) return QSGD_ERR_CAPACITY;
    uint8_t* wsb = static_cast<uint8_t*>(workspace_dev) + kStatusBytes + kTotalsBytes;
    GenArgs a;
    std::memset(&a, 0, sizeof a);
    a.g = g_dev; a.index_base = index_base; a.n = g.n; a.d = g.d; a.nb = g.nb; a.spb = gp.spb;
    a.nseg = gp.nseg;
    a.s = g.s; a.code = g.code; a.norm_mode = g.norm;
    a.key0 = (uint32_t)p->seed; a.key1 = (uint32_t)(p->seed >> 32);
    a.stream_id = p->stream_id; a.iteration = p->iteration;
    a.sub_words = gp.sub_words;
    a.header = header; a.table = table; a.payload = payload;
    a.cap_words = cap_words; a.table_words = g.table_words;
    a.partial = reinterpret_cast<double*>(wsb + gp.off_partial);
    a.scale = reinterpret_cast<float*>(wsb + gp.off_scale);
    a.seginfo = reinterpret_cast<uint32_t*>(wsb + gp.off_seginfo);
    a.segstart = reinterpret_cast<uint64_t*>(wsb + gp.off_segstart);
    a.seggap = reinterpret_cast<uint32_t*>(wsb + gp.off_seggap);
    a.segrank = reinterpret_cast<uint32_t*>(wsb + gp.off_segrank);
    a.segprev = reinterpret_cast<uint32_t*>(wsb + gp.off_segprev);
    a.bents = reinterpret_cast<uint32_t*>(wsb + gp.off_bents);
    a.entries = (g.code != QSGD_CODE_FIXED && g.d > kEntryMinD) ? 1u : 0u;
    a.slots = reinterpret_cast<uint32_t*>(wsb + gp.off_slots);
    a.fixed_bits = g.fixed_bits;
    a.fixed_words_full = g.max_words(g.d);
    a.fixed_payload_words = g.code == QSGD_CODE_FIXED ? g.max_payload_words() : 0;
    const bool aligned = g.d % 4 == 0;
    ScopedTiming tm("encode_general", st);
    if (launch_gen_partial(a, st) != hipSuccess) return QSGD_ERR_HIP;
    if (launch_gen_scale(a, st) != hipSuccess) return QSGD_ERR_HIP;
    if (launch_gen_encode(a, aligned, st) != hipSuccess) return QSGD_ERR_HIP;
    if (g.code != QSGD_CODE_FIXED) {
      if (launch_gen_scan(a, st) != hipSuccess) return QSGD_ERR_HIP;
      const uint32_t fill_blocks =
          (uint32_t)std::min<uint64_t>(std::max<uint64_t>(1, (cap_words + 2047) / 2048), 4096);
      if (launch_gen_fill(a, fill_blocks, st) != hipSuccess) return QSGD_ERR_HIP;
      if (launch_gen_place(a, st) != hipSuccess) return QSGD_ERR_HIP;
    }
    return QSGD_OK;
  }

  if (L && g.nb == 0) {   // every tensor travels raw: header (and an empty table) only
    if (cap_words < raw_words) return QSGD_ERR_CAPACITY;
    RawArgs ra = raw_args(g, L);
    ra.g = g_dev; ra.header = header; ra.table = table; ra.payload = payload;
    ra.cap_words = cap_words;
    ScopedTiming tm("encode_raw", st);
    if (launch_write_layout_header(header, table, g.code, g.norm, g.s, g.d, g.n, raw_words,
                                   p->stream_id, p->iteration, st) != hipSuccess)
      return QSGD_ERR_HIP;
    if (launch_raw_pack(ra, st) != hipSuccess) return QSGD_ERR_HIP;
    return QSGD_OK;
  }

  EncodePlan pl;
  int tw, cpw;
  team_shape(g.d, tw, cpw);
  const uint32_t target = std::min<uint32_t>(kMaxTeams, (uint32_t)device_cus() * (QSGD_ENC_TEAMS / tw));
  if (workspace_bytes < kStatusBytes + kTotalsBytes) return QSGD_ERR_CAPACITY;
  plan_encode(g, target, workspace_bytes - kStatusBytes, pl);
  // Elias codes: a region must at least hold one string of typical size; below the
  // worst case the device reports a region that ran out like a message that did
  if (g.code != QSGD_CODE_FIXED && pl.region_words < std::min<uint64_t>(64, g.max_words(g.d)))
    return QSGD_ERR_CAPACITY;
  // fixed width: the size of the message does not depend on the data
  const uint64_t fixed_words =
      g.code != QSGD_CODE_FIXED ? 0
      : (L ? layout_string_words(g, L) : g.max_payload_words()) + raw_words;
  if (g.code == QSGD_CODE_FIXED && cap_words < fixed_words) return QSGD_ERR_CAPACITY;

  uint8_t* wsb = static_cast<uint8_t*>(workspace_dev) + kStatusBytes;
  EncodeArgs a;
  std::memset(&a, 0, sizeof a);
  a.g = g_dev; a.n = g.n; a.d = (uint32_t)g.d; a.nb = (uint32_t)g.nb; a.s = g.s;
  a.norm_mode = g.norm;
  a.btab = L ? L->btab : nullptr;
  a.version = L ? 2 : 1;
  a.index_base = index_base;
  a.key0 = (uint32_t)p->seed; a.key1 = (uint32_t)(p->seed >> 32);
  a.stream_id = p->stream_id; a.iteration = p->iteration;
  a.bper = pl.bper; a.dst_words = pl.dst_words; a.sub_words = pl.sub_words; a.ring = pl.ring;
  a.header = header; a.table = table;
  a.totals = reinterpret_cast<uint32_t*>(wsb);
  a.staging = reinterpret_cast<uint32_t*>(wsb + kTotalsBytes);
  a.region_words = pl.region_words;
  a.payload = payload;
  a.fixed_bits = g.fixed_bits;
  a.fixed_words_full = (uint32_t)g.max_words(g.d);
  a.fixed_payload_words = fixed_words;
  RawArgs ra;
  if (L) {
    ra = raw_args(g, L);
    ra.g = g_dev; ra.header = header; ra.table = table; ra.payload = payload;
    ra.cap_words = cap_words;
  }
  if (g.code == QSGD_CODE_FIXED && g.d <= 1024) {
    // small buckets: several ride in one wavefront
    const int lpb = g.d <= 256 ? 16 : g.d <= 512 ? 32 : 64;
    const int cp = (int)((g.d + lpb * 4 - 1) / (lpb * 4));
    const uint32_t per_pass = 64u / lpb;
    const uint32_t groups = (uint32_t)((g.nb + per_pass - 1) / per_pass);
    const uint32_t want = (uint32_t)device_cus() * QSGD_FS_TEAMS;   // (no per-team state: no cap)
    const uint32_t t = std::max(1u, std::min(groups, want));
    a.bper = (groups + t - 1) / t;
    const uint32_t teams = (groups + a.bper - 1) / a.bper;
    {
      ScopedTiming tm("encode_bucket", st);
      if (launch_encode_fixed_small(a, lpb, cp, teams, st) != hipSuccess) return QSGD_ERR_HIP;
    }
    if (L && L->R) {
      ScopedTiming tm("encode_raw", st);
      if (launch_raw_pack(ra, st) != hipSuccess) return QSGD_ERR_HIP;
    }
    return QSGD_OK;
  }
  {
    ScopedTiming tm("encode_bucket", st);
    if (launch_encode_bucket(a, g.code, pl.tw, pl.cpw, pl.teams, pl.lds, st) != hipSuccess)
      return QSGD_ERR_HIP;
  }
  if (g.code != QSGD_CODE_FIXED) {
    CompactArgs c;
    c.staging = a.staging; c.region_words = pl.region_words; c.totals = a.totals;
    c.prefix = reinterpret_cast<unsigned long long*>(wsb + (uint64_t)kMaxTeams * 4);
    c.table = table; c.payload = payload; c.header = header; c.cap_words = cap_words;
    c.bper = pl.bper; c.nb = (uint32_t)g.nb; c.table_words = (uint32_t)g.table_words;
    c.raw_words = raw_words;
    ScopedTiming tm("encode_compact", st);
    if (launch_encode_compact(c, pl.teams, st) != hipSuccess) return QSGD_ERR_HIP;
  }
  if (L && L->R) {
    ScopedTiming tm("encode_raw", st);
    if (launch_raw_pack(ra, st) != hipSuccess) return QSGD_ERR_HIP;
  }
  return QSGD_OK;
}

// ---- scratch that is part of the library image, for callers that cannot allocate --------
// One array per GPU the library runs on, held until the process ends.  Host code never
// uses the array's name as an address: the device address is looked up once per device
// (hipGetSymbolAddress, with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[64] = {nullptr};

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return QSGD_ERR_HIP;
  if (dev < 0 || dev >= 64) return QSGD_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return QSGD_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return QSGD_OK;
}

int qsgd_encode_static(const qsgd_params* p, const float* g_dev, void* msg_dev,
                       size_t msg_capacity, void* hip_stream) {
  const size_t need = qsgd_workspace_bytes(p, 1);
  if (need == 0) return QSGD_ERR_INVALID_ARG;
  if (need > kStaticScratchBytes) return QSGD_ERR_SCRATCH;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc) return rc;
  // (the encoder ignores what its workspace holds on entry: every word it reads it has
  // written in the same call, so the last call's contents need no clearing)
  return encode_impl(p, nullptr, 0, g_dev, msg_dev, msg_capacity, ws, need, hip_stream);
}

size_t qsgd_static_scratch_bytes(void) { return kStaticScratchBytes; }

int qsgd_encode(const qsgd_params* p, const float* g_dev, void* msg_dev, size_t msg_capacity,
                void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  return encode_impl(p, nullptr, 0, g_dev, msg_dev, msg_capacity, workspace_dev,
                     workspace_bytes, hip_stream);
}

int qsgd_encode_slice(const qsgd_params* p, uint64_t index_base, const float* g_dev,
                      void* msg_dev, size_t msg_capacity, void* workspace_dev,
                      size_t workspace_bytes, void* hip_stream) {
  return encode_impl(p, nullptr, index_base, g_dev, msg_dev, msg_capacity, workspace_dev,
                     workspace_bytes, hip_stream);
}

int qsgd_encode_layout(const qsgd_params* p, const qsgd_layout* layout, const float* g_dev,
                       void* msg_dev, size_t msg_capacity, void* workspace_dev,
                       size_t workspace_bytes, void* hip_stream) {
  if (!layout) return QSGD_ERR_INVALID_ARG;
  return encode_impl(p, layout, 0, g_dev, msg_dev, msg_capacity, workspace_dev,
                     workspace_bytes, hip_stream);
}



int qsgd_decode_accumulate(const qsgd_params* p, const void* const* msgs_dev,
                           const size_t* msg_bytes, uint32_t K, float* acc_dev,
                           void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  return run_decode(p, nullptr, msgs_dev, msg_bytes, K, 0.f, 0, acc_dev, workspace_dev,
                    workspace_bytes, hip_stream);
}

int qsgd_sgd_step(const qsgd_params* p, const void* const* msgs_dev, const size_t* msg_bytes,
                  uint32_t K, float eta, float* x_dev, void* workspace_dev,
                  size_t workspace_bytes, void* hip_stream) {
  if (K < 1) return QSGD_ERR_INVALID_ARG;
  const float c = eta / (float)K;
  return run_decode(p, nullptr, msgs_dev, msg_bytes, K, c, 1, x_dev, workspace_dev,
                    workspace_bytes, hip_stream);
}

int qsgd_decode_accumulate_layout(const qsgd_params* p, const qsgd_layout* layout,
                                  const void* const* msgs_dev, const size_t* msg_bytes,
                                  uint32_t K, float* acc_dev, void* workspace_dev,
                                  size_t workspace_bytes, void* hip_stream) {
  if (!layout) return QSGD_ERR_INVALID_ARG;
  return run_decode(p, layout, msgs_dev, msg_bytes, K, 0.f, 0, acc_dev, workspace_dev,
                    workspace_bytes, hip_stream);
}

int qsgd_sgd_step_layout(const qsgd_params* p, const qsgd_layout* layout,
                         const void* const* msgs_dev, const size_t* msg_bytes, uint32_t K,
                         float eta, float* x_dev, void* workspace_dev, size_t workspace_bytes,
                         void* hip_stream) {
  if (!layout || K < 1) return QSGD_ERR_INVALID_ARG;
  return run_decode(p, layout, msgs_dev, msg_bytes, K, eta / (float)K, 1, x_dev, workspace_dev,
                    workspace_bytes, hip_stream);
}

int qsgd_layout_create(const uint64_t* offsets, const uint64_t* sizes, uint32_t T, uint64_t d,
                       uint64_t bypass_below, qsgd_layout** out) {
  if (!out || (T && (!offsets || !sizes)) || d < 4 || d % 4 || d > kMaxBucketFast)
    return d > kMaxBucketFast || (d % 4) ? QSGD_ERR_UNSUPPORTED : QSGD_ERR_INVALID_ARG;
  std::vector<uint2> bt;
  std::vector<uint4> rt;
  qsgd_layout* L = new (std::nothrow) qsgd_layout;
  if (!L) return QSGD_ERR_INVALID_ARG;
  L->d = d; L->bypass = bypass_below;
  uint64_t prev_end = 0;
  for (uint32_t j = 0; j < T; ++j) {   // ascending, disjoint, 16-byte aligned starts
    const uint64_t off = offsets[j], sz = sizes[j];
    if (off < prev_end || (off % 4) || off + sz > 0xFFFFFFFFull) { delete L; return QSGD_ERR_INVALID_ARG; }
    prev_end = off + sz;
    if (sz < bypass_below) {
      // pieces of kRawPiece values, one workgroup each
      for (uint64_t o = 0; o < sz; o += kRawPiece)
        rt.push_back(make_uint4((uint32_t)((off + o) / 4),
                                (uint32_t)std::min<uint64_t>(kRawPiece, sz - o),
                                (uint32_t)(L->raw + o), 0));
      L->raw += sz;
      continue;
    }
    for (uint64_t o = 0; o < sz; o += d) {
      const uint32_t m = (uint32_t)std::min<uint64_t>(d, sz - o);
      bt.push_back(make_uint2((uint32_t)((off + o) / 4), m));
      if (m < d) { L->short_buckets++; L->short_values += m; L->short_len.push_back(m); }
    }
  }
  L->extent = prev_end;
  L->nb = bt.size();
  L->R = (uint32_t)rt.size();
  if (L->nb > 0x7FFFFFFFull || L->raw > 0xFFFFFFFFull) { delete L; return QSGD_ERR_UNSUPPORTED; }
  bool ok = hipGetDevice(&L->device) == hipSuccess;
  if (ok && !bt.empty()) {
    ok = hipMalloc(reinterpret_cast<void**>(&L->btab), bt.size() * sizeof(uint2)) == hipSuccess &&
         hipMemcpy(L->btab, bt.data(), bt.size() * sizeof(uint2), hipMemcpyHostToDevice) == hipSuccess;
  }
  if (ok && !rt.empty()) {
    ok = hipMalloc(reinterpret_cast<void**>(&L->rtab), rt.size() * sizeof(uint4)) == hipSuccess &&
         hipMemcpy(L->rtab, rt.data(), rt.size() * sizeof(uint4), hipMemcpyHostToDevice) == hipSuccess;
  }
  if (!ok) { qsgd_layout_destroy(L); return QSGD_ERR_HIP; }
  *out = L;
  return QSGD_OK;
}

void qsgd_layout_destroy(qsgd_layout* layout) {
  if (!layout) return;
  if (layout->btab) (void)hipFree(layout->btab);
  if (layout->rtab) (void)hipFree(layout->rtab);
  delete layout;
}

int qsgd_layout_info(const qsgd_layout* layout, uint64_t* buckets, uint64_t* raw_values,
                     uint64_t* extent) {
  if (!layout) return QSGD_ERR_INVALID_ARG;
  if (buckets) *buckets = layout->nb;
  if (raw_values) *raw_values = layout->raw;
  if (extent) *extent = layout->extent;
  return QSGD_OK;
}

size_t qsgd_layout_max_encoded_bytes(const qsgd_params* p, const qsgd_layout* layout) {
  Geometry g;
  if (!layout || make_geometry(p, g) || p->d != layout->d || p->n < layout->extent) return 0;
  g.d = layout->d; g.nb = layout->nb;
  g.table_words = p->code == QSGD_CODE_FIXED ? 0 : ((g.nb + 1 + 3) & ~(uint64_t)3);
  return (size_t)(4 * (H_WORDS + g.table_words + layout_string_words(g, layout) + layout->raw));
}

size_t qsgd_layout_workspace_bytes(const qsgd_params* p, const qsgd_layout* layout, uint32_t K) {
  Geometry g;
  if (!layout || make_geometry(p, g) || K > QSGD_MAX_PEERS || p->d != layout->d) return 0;
  g.d = layout->d; g.nb = layout->nb;
  uint64_t bytes = kStatusBytes + kTotalsBytes;
  if (g.code != QSGD_CODE_FIXED) {
    const uint64_t slots = g.nb + std::min<uint64_t>(g.nb, kMaxTeams);
    bytes += slots * (g.max_words(g.d) + 4) * 4;
  }
  return (size_t)((bytes + 255) & ~(uint64_t)255);
}

int qsgd_message_info(const void* header_host, qsgd_params* out, uint64_t* total_bytes) {
  if (!header_host) return QSGD_ERR_INVALID_ARG;
  uint32_t h[H_WORDS];
  std::memcpy(h, header_host, sizeof h);
  if (h[H_MAGIC] != kMagic || (h[H_VERSION] != 1 && h[H_VERSION] != 2)) return QSGD_ERR_CORRUPT;
  qsgd_params q;
  std::memset(&q, 0, sizeof q);
  q.code = h[H_CODE]; q.norm = h[H_NORM]; q.s = h[H_S];
  q.stream_id = h[H_STREAM]; q.iteration = h[H_ITER];
  q.d = h[H_D_LO] | ((uint64_t)h[H_D_HI] << 32);
  q.n = h[H_N_LO] | ((uint64_t)h[H_N_HI] << 32);
  Geometry g;
  if (make_geometry(&q, g)) return QSGD_ERR_CORRUPT;
  const uint64_t pw = h[H_PW_LO] | ((uint64_t)h[H_PW_HI] << 32);
  if (h[H_VERSION] == 2) {   // tensor-aware: the bucket count is the layout's, not ceil(n / d)
    const uint64_t nb = h[H_NB_LO] | ((uint64_t)h[H_NB_HI] << 32);
    g.table_words = q.code == QSGD_CODE_FIXED ? 0 : ((nb + 1 + 3) & ~(uint64_t)3);
  }
  if (out) *out = q;
  if (total_bytes) *total_bytes = 4 * (H_WORDS + g.table_words + pw);
  const int status = (int)h[H_STATUS];
  if (status == 0) return QSGD_OK;
  return status == QSGD_ERR_CAPACITY ? QSGD_ERR_CAPACITY : QSGD_ERR_CORRUPT;
}

int qsgd_message_status(const void* msg_dev, uint64_t* total_bytes, void* hip_stream) {
  if (!msg_dev) return QSGD_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  uint32_t h[H_WORDS];
  if (hipStreamSynchronize(st) != hipSuccess) return QSGD_ERR_HIP;
  if (hipMemcpy(h, msg_dev, sizeof h, hipMemcpyDeviceToHost) != hipSuccess) return QSGD_ERR_HIP;
  return qsgd_message_info(h, nullptr, total_bytes);
}

int qsgd_workspace_status(const void* workspace_dev, void* hip_stream) {
  if (!workspace_dev) return QSGD_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  uint32_t w = 0;
  if (hipStreamSynchronize(st) != hipSuccess) return QSGD_ERR_HIP;
  if (hipMemcpy(&w, workspace_dev, sizeof w, hipMemcpyDeviceToHost) != hipSuccess)
    return QSGD_ERR_HIP;
  return (int)w == 0 ? QSGD_OK : QSGD_ERR_CORRUPT;
}

int qsgd_timing_enable(int on) {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  g_timing_on = on != 0;
  while (g_timing_on && g_spare.size() < kSpareEvents) {
    EventPair e;
    if (hipEventCreate(&e.start) != hipSuccess) return QSGD_ERR_HIP;
    if (hipEventCreate(&e.stop) != hipSuccess) { (void)hipEventDestroy(e.start); return QSGD_ERR_HIP; }
    g_spare.push_back(e);
  }
  return QSGD_OK;
}

int qsgd_timing_reset(void) {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  for (auto& t : g_launches) {
    if (g_spare.size() < kSpareEvents) {
      g_spare.push_back({t.start, t.stop});
    } else {
      (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop);
    }
  }
  g_launches.clear();
  return QSGD_OK;
}

int qsgd_copy_probe(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream) {
  if (!dst_dev || !src_dev || (bytes & 15u) || !aligned16(dst_dev) || !aligned16(src_dev))
    return QSGD_ERR_INVALID_ARG;
  if (bytes == 0) return QSGD_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const uint64_t quads = bytes / 16;
  const uint64_t blocks = (bytes + kCopyPiece - 1) / kCopyPiece;
  if (blocks > 0x7FFFFFFFull) return QSGD_ERR_UNSUPPORTED;
  ScopedTiming tm("copy_probe", st);
  hipLaunchKernelGGL(k_copy_probe, dim3((uint32_t)blocks), dim3(256), 0, st,
                     reinterpret_cast<float*>(dst_dev), reinterpret_cast<const float*>(src_dev),
                     quads);
  return hipGetLastError() == hipSuccess ? QSGD_OK : QSGD_ERR_HIP;
}

int qsgd_copy_probe_words(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream) {
  if (!dst_dev || !src_dev || (bytes & 3u) || !aligned16(dst_dev) || !aligned16(src_dev))
    return QSGD_ERR_INVALID_ARG;
  if (bytes == 0) return QSGD_OK;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  const uint64_t words = bytes / 4;
  const uint32_t blocks =
      (uint32_t)std::min<uint64_t>((words + 255) / 256, (uint64_t)device_cus() * 64);
  ScopedTiming tm("copywords_probe", st);
  hipLaunchKernelGGL(k_copy_probe_words, dim3(blocks), dim3(256), 0, st,
                     reinterpret_cast<uint32_t*>(dst_dev),
                     reinterpret_cast<const uint32_t*>(src_dev), words);
  return hipGetLastError() == hipSuccess ? QSGD_OK : QSGD_ERR_HIP;
}

int qsgd_timing_get(const char* prefix, double* total_ms, uint64_t* launches) {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  const std::string pre = prefix ? prefix : "";
  double ms = 0.0;
  uint64_t cnt = 0;
  for (auto& t : g_launches) {
    if (t.name.compare(0, pre.size(), pre) != 0) continue;
    if (hipEventSynchronize(t.stop) != hipSuccess) return QSGD_ERR_HIP;
    float e = 0.f;
    if (hipEventElapsedTime(&e, t.start, t.stop) != hipSuccess) return QSGD_ERR_HIP;
    ms += e;
    ++cnt;
  }
  if (total_ms) *total_ms = ms;
  if (launches) *launches = cnt;
  return QSGD_OK;
}

}  // extern "C"
