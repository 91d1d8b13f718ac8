// Decode kernels, fused with the sum over the K peers and the update
//   x <- x - (eta/K) sum_l Decode(M_l)          (Alg. 1, last line)
// Decode of one bucket string (Sec. 3.1, last sentences on the coding scheme):
// read the 32-bit scale, then the records; Eq. (2) turns (scale, sign, level)
// into a value.
//
// Elias codes are prefix codes: one string can only be read front to back.  The
// parallelism is across strings: every lane of a wavefront reads its own string
// (bucket g of message k), the wavefront owns gw buckets of all K messages, and
// the per-bucket offset table says where each string starts.  Records go through
// small per-string queues in LDS and are applied to an LDS accumulator such that
// every element's fp32 sum is the one taken message by message (k ascending);
// then the accumulator is streamed against x with float4 accesses.
#include <type_traits>

#include "qsgd_device.hpp"
#include "qsgd_kernels.hpp"

namespace qsgd {

constexpr uint32_t kRingStride = kStrWin + 1;   // words of a lane's string ring: kStrWin and the mirror of slot 0

namespace {

// A piece of a string: words [idx, idx + kStrFetch), zeros at and past nwords; idx is a
// multiple of kStrFetch.  Strings are word-aligned, so a whole piece is one 16-byte load.
static_assert(kStrFetch == 4 && kStrWin % kStrFetch == 0, "pieces of four words");
struct __attribute__((packed, aligned(4))) StrPiece { uint32_t w[kStrFetch]; };
__device__ __forceinline__ void load_piece(const uint32_t* str, uint32_t idx, uint32_t nwords,
                                           uint32_t (&t)[kStrFetch]) {
  if (idx + kStrFetch <= nwords) {
    const StrPiece p = *reinterpret_cast<const StrPiece*>(str + idx);
#pragma unroll
    for (uint32_t j = 0; j < kStrFetch; ++j) t[j] = p.w[j];
  } else {
#pragma unroll
    for (uint32_t j = 0; j < kStrFetch; ++j) t[j] = idx + j < nwords ? str[idx + j] : 0u;
  }
}
// Stores the piece that starts at word `idx` of the string into a lane's ring (word j of the
// string in slot j % kStrWin; slot kStrWin mirrors slot 0).
__device__ __forceinline__ void ring_put_piece(uint32_t* ring, uint32_t idx,
                                               const uint32_t (&t)[kStrFetch]) {
  const uint32_t sl = idx & (kStrWin - 1u);
  uint32_t* const at = ring + sl;
#pragma unroll
  for (uint32_t j = 0; j < kStrFetch; ++j) at[j] = t[j];
  if (sl == 0) ring[kStrWin] = t[0];
}

// Recursive Elias code (App. A.2), decoder rule unrolled: N = 1; a 0 bit outputs N,
// a 1 bit opens an (N+1)-bit group whose value is the new N.  `w` holds the next
// 32 stream bits, first bit on top.  G = most groups accepted (G = 1: k <= 3,
// 2: k <= 15, 3: k < 2^16, 4: every code word of at most 32 bits, k < 2^20).
// Returns 0 (len 0) for anything longer or malformed.
template <int G>
__device__ __forceinline__ uint32_t omega_peek(uint32_t w, uint32_t& len) {
  const uint32_t t0 = w >> 31;
  const uint32_t g1 = w >> 30;            // first group, 2 bits: 2 or 3
  const uint32_t w1 = w << 2;
  const uint32_t t1 = w1 >> 31;
  uint32_t v = 0, l = 0;
  if constexpr (G >= 2) {
    const uint32_t n1 = g1 + 1u;            // 3 or 4
    const uint32_t g2 = w1 >> (32u - n1);   // 4..15
    const uint32_t w2 = w1 << n1;
    const uint32_t t2 = w2 >> 31;
    if constexpr (G >= 3) {
      const uint32_t n2 = g2 + 1u;            // 5..16
      const uint32_t g3 = w2 >> (32u - n2);   // 16..65535
      const uint32_t w3 = w2 << n2;
      const uint32_t t3 = w3 >> 31;
      const uint32_t l3 = 3u + n1 + n2;       // length when the third group is the value
      if constexpr (G >= 4) {
        const uint32_t n3 = min(g3 + 1u, 31u);  // only used when the whole word fits 32 bits
        const uint32_t g4 = w3 >> (32u - n3);
        // a fourth group only counts if it and its closing 0 lie inside the 32 bits
        const bool fits4 = l3 + g3 + 1u <= 32u && ((w3 << n3) >> 31) == 0u;
        if (t3 && fits4) { v = g4; l = l3 + n3; }
      }
      if (!t3) { v = g3; l = l3; }
    }
    if (!t2) { v = g2; l = 3u + n1; }
  }
  if (!t1) { v = g1; l = 3u; }
  if (!t0) { v = 1u; l = 1u; }
  len = l;
  return v;
}

// Entry of the Elias table for the 7-bit pattern b7 (first stream bit on top): (after, more)
// = where the bits of the LAST group after its leading 1 start, and how many they are.  The
// value of the code word is then 2^more + those bits and its length after + more + 1:
//   0......  the value 1                         (after 0, more 0)
//   1x0....  one group: 2 or 3                   (after 1, more 1)
//   1x1ab0.  two groups, the second of x+3 bits  (after 3, more x+2)
//   1x1ab1.  a third group of (second group)+1 bits follows: values 16 .. 2^16 - 1
__device__ __forceinline__ uint8_t omega_table_entry(uint32_t b7) {
  uint32_t after = 0, more = 0;
  if (b7 & 64u) {
    const uint32_t g1 = 2u | ((b7 >> 5) & 1u);
    after = 1; more = 1;
    if (b7 & 16u) {
      const uint32_t n1 = g1 + 1u;                                   // bits of the second group
      const uint32_t g2 = (b7 >> (5u - n1)) & ((1u << n1) - 1u);
      after = 3; more = n1 - 1u;
      if ((b7 >> (4u - n1)) & 1u) {                                   // the third group's leading 1
        after = 2u + n1 + 1u;
        more = g2;
      }
    }
  }
  return (uint8_t)(after | (more << 3));
}

}  // namespace

// One thread per message: the header must describe the same code as the call.
__global__ void k_decode_check(DecodeArgs a) {
  const uint32_t k = threadIdx.x;
  if (k == 0) *a.status = 0;
  __syncthreads();
  if (k >= a.K) return;
  bool ok = a.msg_words[k] >= (uint64_t)H_WORDS + a.table_words;
  if (ok) {
    const uint32_t* h = a.msgs[k];
    const uint64_t pw = h[H_PW_LO] | ((uint64_t)h[H_PW_HI] << 32);
    ok = h[H_MAGIC] == kMagic && h[H_VERSION] == a.version && h[H_CODE] == a.code &&
         h[H_NORM] == a.norm_mode && h[H_S] == a.s && h[H_D_LO] == a.d && h[H_D_HI] == 0 &&
         h[H_N_LO] == (uint32_t)a.n && h[H_N_HI] == (uint32_t)(a.n >> 32) &&
         h[H_NB_LO] == a.nb && h[H_NB_HI] == 0 && h[H_STATUS] == 0 &&
         (uint64_t)H_WORDS + a.table_words + pw <= a.msg_words[k];
    if (ok && a.version == 2) {   // tensor-aware: the strings and the raw values fill the payload
      const uint64_t strings = a.table_words ? (uint64_t)h[H_WORDS + a.nb]
                                             : (uint64_t)a.nb * a.fixed_words_full;
      ok = strings + a.raw_words == pw;
    }
  }
  if (!ok) flag_corrupt(a.status);
}

// ---- fixed width: one wavefront per bucket ----------------------------------------
// Lane k < K keeps message k's scale and escape index.  A wavefront takes CH chunks
// of 256 positions at a time; for those it requests the level and sign words of
// KG messages together, so that enough bytes are in flight per wavefront, and so
// that the 128-byte lines of a message that two chunks (or the header and the
// first chunk) share are touched at one time instead of once per chunk with 15
// other messages in between (measured: the second touch came from memory again).
// The sum over the messages runs in k order in registers.
// CHECK: a field can hold a level above s (s + 1 is not a power of two).
template <int B, int CH, bool CHECK>
__global__ __launch_bounds__(256) void k_decode_fixed(DecodeArgs a) {
  if (*a.status != 0) return;
  constexpr int KG = CH >= 4 ? QSGD_FIXED_KG / 2 : QSGD_FIXED_KG;  // messages whose words are requested together
  const int lane = threadIdx.x & 63;
  const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
  const uint32_t wave_count = gridDim.x * 4;
  const uint32_t s = a.s, K = a.K;
  const float s_f = (float)s;
  constexpr uint32_t fmask = (1u << B) - 1u;
  constexpr int LW = B == 16 ? 2 : 1;       // level words a lane reads per message and chunk
  const uint64_t all_ok = K >= 64 ? ~0ull : ((1ull << K) - 1ull);

  for (uint32_t b = wave_global; b < a.nb; b += wave_count) {
    uint64_t base;
    uint32_t m;
    bucket_extent(a, b, base, m);
    const uint32_t lw = (m * B + 31u) >> 5, sw = (m + 31u) >> 5;
    const uint64_t str_off = (uint64_t)H_WORDS + (uint64_t)b * a.fixed_words_full;
    float my_scale = 0.f;
    uint32_t my_esc = 0xFFFFFFFFu, my_ok = 0;
    if ((uint32_t)lane < K) {
      if (str_off + 2u + lw + sw <= a.msg_words[lane]) {
        const uint32_t* str = a.msgs[lane] + str_off;
        my_scale = __uint_as_float(str[0]) / s_f;
        my_esc = str[1];
        my_ok = (my_esc == 0xFFFFFFFFu || my_esc < m) ? 1u : 0u;
      }
      if (!my_ok) { flag_corrupt(a.status); my_scale = 0.f; my_esc = 0xFFFFFFFFu; }
    }
    const uint64_t okmask = __builtin_amdgcn_ballot_w64(my_ok != 0);
    // every message is intact and every chunk of the group is complete: no per-load tests
    const bool whole = okmask == all_ok && m % (CH * kChunk) == 0;
    for (uint32_t g0 = 0; g0 < m; g0 += CH * kChunk) {
      float4 xv[CH];
      float acc[CH][4];
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const uint32_t e0 = g0 + (uint32_t)c * kChunk + (uint32_t)lane * 4u;
        const float* xp = a.x + base + e0;
        xv[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        acc[c][0] = acc[c][1] = acc[c][2] = acc[c][3] = 0.f;
        if (e0 + 3 < m) {
          xv[c] = load_stream(xp);
        } else if (e0 < m) {
          xv[c].x = xp[0];
          if (e0 + 1 < m) xv[c].y = xp[1];
          if (e0 + 2 < m) xv[c].z = xp[2];
        }
      }
      for (uint32_t k0 = 0; k0 < K; k0 += KG) {
        uint32_t wl[KG][CH][LW], ws[KG][CH];
        if (whole) {
#pragma unroll
          for (int t = 0; t < KG; ++t) {
            const uint32_t* lplane = a.msgs[min(k0 + t, K - 1u)] + str_off + 2;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
              const uint32_t e0 = g0 + (uint32_t)c * kChunk + (uint32_t)lane * 4u;
              const uint32_t li = (e0 * B) >> 5;
              wl[t][c][0] = lplane[li];
              if (LW == 2) wl[t][c][LW - 1] = lplane[li + 1];
              ws[t][c] = lplane[lw + (e0 >> 5)];
            }
          }
        } else {
#pragma unroll
          for (int t = 0; t < KG; ++t) {
            const uint32_t k = k0 + t;
            const bool live = k < K && ((okmask >> k) & 1ull);
            const uint32_t* lplane = live ? a.msgs[k] + str_off + 2 : nullptr;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
              const uint32_t e0 = g0 + (uint32_t)c * kChunk + (uint32_t)lane * 4u;
              const uint32_t li = (e0 * B) >> 5;
              wl[t][c][0] = 0; ws[t][c] = 0;
              if (LW == 2) wl[t][c][LW - 1] = 0;
              if (live && e0 < m) {
                wl[t][c][0] = lplane[li];
                if (LW == 2 && li + 1 < lw) wl[t][c][LW - 1] = lplane[li + 1];
                ws[t][c] = lplane[lw + (e0 >> 5)];
              }
            }
          }
        }
#pragma unroll
        for (int t = 0; t < KG; ++t) {
          const uint32_t k = k0 + t;
          if (k >= K) break;
          const float sc = __uint_as_float(lane_bcast(__float_as_uint(my_scale), (int)k));
          const uint32_t esc = lane_bcast(my_esc, (int)k);
#pragma unroll
          for (int c = 0; c < CH; ++c) {
            const uint32_t c0 = g0 + (uint32_t)c * kChunk;       // uniform
            const uint32_t e0 = c0 + (uint32_t)lane * 4u;
            uint32_t z[4];
            if (B == 8) {
              z[0] = wl[t][c][0] & 0xFFu; z[1] = (wl[t][c][0] >> 8) & 0xFFu;
              z[2] = (wl[t][c][0] >> 16) & 0xFFu; z[3] = wl[t][c][0] >> 24;
            } else if (B == 16) {
              z[0] = wl[t][c][0] & 0xFFFFu; z[1] = wl[t][c][0] >> 16;
              z[2] = wl[t][c][LW - 1] & 0xFFFFu; z[3] = wl[t][c][LW - 1] >> 16;
            } else {
              const uint32_t w = wl[t][c][0] >> ((e0 * B) & 31u);
              z[0] = w & fmask; z[1] = (w >> B) & fmask; z[2] = (w >> (2 * B)) & fmask;
              z[3] = (w >> (3 * B)) & fmask;
            }
            float mag[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) mag[j] = sc * (float)z[j];
            // rare, wave-uniform: this message's top-level value lies in this chunk
            if (esc - c0 < kChunk) {
              const float top = sc * s_f;
#pragma unroll
              for (int j = 0; j < 4; ++j)
                if (esc == e0 + j) mag[j] = top;
            }
            if (CHECK) {
              if (max(max(z[0], z[1]), max(z[2], z[3])) > s) flag_corrupt(a.status);
            }
            const uint32_t sg = ws[t][c] >> (e0 & 31u);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              // the sign bit goes into the product (-0 for a zero level adds like +0)
              acc[c][j] += __uint_as_float(((sg << (31 - j)) & 0x80000000u) | __float_as_uint(mag[j]));
            }
          }
        }
      }
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const uint32_t e0 = g0 + (uint32_t)c * kChunk + (uint32_t)lane * 4u;
        float* xp = a.x + base + e0;
        float4 v = xv[c];
        if (a.step) {
          v.x = fmaf(-a.c, acc[c][0], v.x); v.y = fmaf(-a.c, acc[c][1], v.y);
          v.z = fmaf(-a.c, acc[c][2], v.z); v.w = fmaf(-a.c, acc[c][3], v.w);
        } else {
          v.x += acc[c][0]; v.y += acc[c][1]; v.z += acc[c][2]; v.w += acc[c][3];
        }
        if (e0 + 3 < m) {
          store_stream(xp, v);
        } else if (e0 < m) {
          xp[0] = v.x;
          if (e0 + 1 < m) xp[1] = v.y;
          if (e0 + 2 < m) xp[2] = v.z;
        }
      }
    }
  }
}

// ---- Elias codes: one lane per string, gw buckets x K messages per wavefront -------
// The bucket is walked in windows of `win` (<= 256) positions.  Per wavefront:
//  (1) x of a window is requested into registers well ahead of its use (at the
//      start of the window, or a whole window earlier: see kAhead);
//  (2) every lane parses ahead into its own ring of records.  Its string comes
//      through a small per-lane ring of words in LDS that is refilled in pieces
//      (a 128-byte line of a message is then fetched a few times, not once per
//      code word), and the parser itself works on a 64-bit register of unread bits;
//  (3) records are applied to an LDS accumulator, but only up to the position
//      every string has been parsed to, and such that every element's terms are
//      added in message order (see the apply step below);
//  (4) registers and accumulator are combined and stored.
// The kernel is bound by latency and instruction issue, not by bytes: small LDS
// per wavefront (short rings, 256-position windows) buys occupancy, which
// measured better than longer rings or windows.

// CODE: sparse or dense Elias code.  LG: groups a level's code word may have.
// KLOOP: apply the queued records message by message (dense messages) instead of
// counting the terms of every position first (sparse ones); see the apply step.
// Q16: queued records are 16 bits wide (s <= 4: the level, stored minus one, fits two
// bits beside 13 bits of position and the sign); the smaller rings let two more
// wavefronts live on a compute unit (c5: 2.77 -> 2.60 ms).
template <int CODE, int LG, int NQ, bool KLOOP, bool Q16>
__device__ __forceinline__ void decode_elias_body(const DecodeArgs& a, float* acc,
                                                  std::conditional_t<Q16, uint16_t, uint32_t>* queue,
                                                  uint32_t* swin, uint32_t b0, uint32_t gcount) {
  using qrec_t = std::conditional_t<Q16, uint16_t, uint32_t>;
  constexpr uint32_t kLevBias = Q16 ? 1u : 0u;
  constexpr uint32_t kRecWords = rec_words(Q16);
  constexpr bool kSparse = CODE == QSGD_CODE_SPARSE;
  // a whole record in one 32-bit peek: gap <= 21 bits, sign, level <= 7 bits
  constexpr bool kNarrow = !kSparse || LG <= 2;
  const uint32_t K = a.K, gw = a.gw, win = a.win, s = a.s;
  // ring depth: the message-by-message apply hands ring slot r of string (g, k) to lane
  // (g, r), so gw * depth <= 64 there
  constexpr bool kloop = KLOOP;
  const uint32_t rec = kloop ? a.rec : kRec;
  // ring slot idx of lane l: lane-major where other lanes read a string's slots side
  // by side (message loop), slot-major where a lane only reads its own ring
  auto qidx = [&](uint32_t l, uint32_t idx) -> uint32_t {
    return kloop ? l * rec + idx : idx * 64u + l;
  };
  constexpr uint32_t winp = kChunk;  // accumulator stride per bucket
  const int lane = threadIdx.x;
  const uint64_t pay = (uint64_t)H_WORDS + a.table_words;

  // ---- open this lane's string -----------------------------------------------------
  const uint32_t g = lane / K, k = lane - g * K;
  const uint32_t b = b0 + g;
  // The record a lane has decoded and not yet queued: (pend_pos, pend_lev, pend_neg), pend_pos
  // 1-based, kDone when there is none (the string has ended or is damaged).  One number says
  // both whether there is a record and where it falls, and the parse loop below has one
  // predicate per trip: every instruction of that loop, scalar ones included, is a step of
  // a chain that a lane's string forces to be serial.
  constexpr uint32_t kDone = 0xFFFFFFFFu;
  uint32_t m = 0;         // elements in this lane's bucket
  uint32_t endbit = 0;    // records end here
  uint32_t bitpos = 32;   // next unread bit (after the scale)
  uint32_t nwords = 0;
  uint32_t pend_pos = kDone, pend_lev = 0, pend_neg = 0;
  const uint32_t* str = nullptr;
  bool open = false;
  float my_scale = 0.f;
  if (g < gcount) {
    uint64_t base_unused;
    bucket_extent(a, b, base_unused, m);
    const uint32_t* msg = a.msgs[k];
    const uint32_t o0 = msg[H_WORDS + b], o1 = msg[H_WORDS + b + 1];
    if (o0 < o1 && pay + o1 <= a.msg_words[k]) {
      nwords = o1 - o0;
      str = msg + pay + o0;
      my_scale = __uint_as_float(str[0]) / (float)s;
      open = true;
      if (kSparse) {
        const uint32_t last = str[nwords - 1];
        endbit = nwords * 32u - 1u - (uint32_t)(__ffs((int)last) - 1);
        if (last == 0 || endbit < 32u) open = false;
      } else {
        endbit = nwords * 32u;
      }
    }
    if (!open) flag_corrupt(a.status);
  }
  if (!open) my_scale = 0.f;

  // The lane's view of its string: the last kStrWin words fetched, as a ring in LDS: word j
  // of the string in slot j % kStrWin of the lane's kStrWin + 1 slots; the last slot mirrors
  // slot 0, so that two consecutive words are always two consecutive slots (one LDS read
  // of a pair), and the odd stride keeps the lanes on distinct banks.  A string is touched
  // once per kStrFetch words instead of once per record, and the touches of one wavefront
  // happen together at the top of a round, so a 128-byte line of a message is pulled from
  // memory a few times rather than once per code word.
  uint32_t* const ring = swin + (uint32_t)lane * kRingStride;
  uint8_t* const otab = reinterpret_cast<uint8_t*>(swin + 64u * kRingStride);   // Elias table
  uint32_t sfill = 0;   // words [sfill - kStrWin, sfill) of the string are in the ring
  auto fetch = [&]() {
    uint32_t t[kStrFetch];
    load_piece(str, sfill, nwords, t);
    ring_put_piece(ring, sfill, t);
    sfill += kStrFetch;
  };
  // The 32 stream bits from bit `at` on, out of the ring (bit j of the stream is bit
  // 31 - j % 32 of word j / 32).  The parser keeps a bit position instead of a shift
  // register: the vector ALU bounds this kernel, and this way it only aligns two words.
  auto peek = [&](uint32_t at) -> uint32_t {
    const uint32_t off = at & 31u;
    const uint32_t* const pw = ring + ((at >> 5) & (kStrWin - 1u));
    const uint32_t wa = pw[0], wb = pw[1];
    const uint32_t sh = __builtin_amdgcn_alignbit(wa, wb, 32u - off);   // (off = 0 gives wb)
    return off ? sh : wa;
  };
  // Recursive Elias code (App. A.2) through a table: the entry (after, more) of the next 7
  // bits says where the last group's bits after its leading 1 start and how many they are;
  // the value is 2^more + those bits, the code word after + more + 1 bits (with its closing
  // 0, which `open_end` checks: its top bit is set if the word does not end there).
  // Values below 2^16 (three groups).
  auto omega_tab = [&](uint32_t w, uint32_t& len, uint32_t& open_end) -> uint32_t {
    const uint32_t e = otab[w >> 25];
    const uint32_t after = e & 7u, more = e >> 3;
    const uint32_t y = w << after;
    const uint32_t rest = __builtin_amdgcn_ubfe(y, 32u - more, more);   // (more = 0: 0)
    open_end = y << more;
    len = after + more + 1u;
    return (1u << more) | rest;
  };
  // The code words of 1 .. 4 ("0", "100", "110", "101000") from their first three bits, for
  // s <= 4: nibble b of the two constants is the value and the length for the top bits b
  // ("111" would be a value of 8 or more, and "101" has to go on with "000").  No table
  // look-up, that is one LDS round trip less in the chain from one record to the next.
  auto omega_small = [&](uint32_t w, uint32_t& len, uint32_t& open_end) -> uint32_t {
    const uint32_t six = w >> 26, b = six >> 3;
    len = (0x03631111u >> (4u * b)) & 0xFu;
    open_end = ((b == 7u) | ((b == 5u) & (six != 0x28u))) ? 0x80000000u : 0u;
    return (0x03421111u >> (4u * b)) & 0xFu;
  };
  // A record reads at most the two words at bitpos / 32 (kNarrow) or one more, so a lane may
  // parse while bitpos is below this limit (none once the whole string is in the ring: past
  // its end the ring may hold anything, those bits lie behind endbit).
  auto parse_limit = [&]() -> uint32_t {
    return sfill >= nwords ? 0xFFFFFFFFu : (sfill - (kNarrow ? 1u : 2u)) * 32u;
  };

  // Reads the next record into pend_*; `pos` is the position of the one before (0 at the
  // start of the string).  pend_pos = kDone at the end of the string.
  uint32_t bad = 0;   // a record that cannot be: remembered here, reported after the parse pass
  auto advance = [&](uint32_t pos) {
    uint32_t w = peek(bitpos);
    if (kSparse) {
      const bool more = bitpos < endbit;
      uint32_t gl, ll, e1, e2;
      const uint32_t gap = omega_tab(w, gl, e1);
      if (!kNarrow) w = peek(bitpos + gl); else w <<= gl;
      pend_neg = w >> 31;
      const uint32_t lev = Q16 ? omega_small(w << 1, ll, e2) : omega_tab(w << 1, ll, e2);
      bitpos += gl + 1u + ll;
      pos += gap;
      pend_lev = lev;
      // (no short cuts between the tests: as plain mask arithmetic they cost no branch)
      const bool bad_rec = ((int)(e1 | e2) < 0) | (lev > s) | (pos > m) | (bitpos > endbit);
      bad |= (more & bad_rec) ? 1u : 0u;
      pend_pos = (more & !bad_rec) ? pos : kDone;
    } else {
      const bool more = pos < m;
      uint32_t ll, e2;
      const uint32_t lev1 = omega_tab(w << 1, ll, e2);
      bitpos += 1u + ll;
      pend_neg = w >> 31;
      pend_lev = lev1 - 1u;
      const bool bad_rec = ((int)e2 < 0) | (lev1 > s + 1u) | (bitpos > endbit);
      bad |= (more & bad_rec) ? 1u : 0u;
      pend_pos = (more & !bad_rec) ? pos + 1u : kDone;
    }
  };
  // the table: entry of the 7-bit pattern b7 (first stream bit on top)
  for (uint32_t b7 = lane; b7 < 128u; b7 += 64) otab[b7] = omega_table_entry(b7);
  if (open) {
    fetch();
    fetch();
  }
  __syncthreads();
  if (open) advance(0u);
  if (bad) { flag_corrupt(a.status); bad = 0; }

  for (uint32_t j = lane; j < gw * winp; j += 64) acc[j] = 0.f;
  __syncthreads();

  // A window is at most 256 positions (winp = 256): quad q of the x registers is
  // bucket q of this wavefront, lane l holds positions 4l..4l+3 of the window.
  uint32_t qhead = 0, qcnt = 0;            // this lane's ring of queued records
  uint32_t* const accu = reinterpret_cast<uint32_t*>(acc);
  const uint32_t grow = (g < gw ? g : 0u) * winp;   // this lane's accumulator row
  const uint32_t dump = gw * winp + kRecWords + 64u * kRingStride + 32u + (uint32_t)lane;
  uint32_t* const counts = accu + gw * winp + kRecWords + 64u * kRingStride + 32u + 64u;
  uint32_t* const heads = counts + 64;
  float* const scales = reinterpret_cast<float*>(counts + 128);
  const uint32_t i = (uint32_t)lane * 4u;
  // x of one window into registers: quad qi is bucket qi of this wavefront.
  // The common case, decided per window on the scalar unit: the wavefront has all its NQ
  // buckets and the window lies inside every one of them.  Then loads and stores need no
  // per-lane bounds (the general code below costs about a hundred vector instructions per
  // window, and the vector ALU is what bounds this kernel).
  uint64_t xbase[NQ];
  uint32_t xlen_min = 0xFFFFFFFFu;
#pragma unroll
  for (int qi = 0; qi < NQ; ++qi) {
    xbase[qi] = 0;
    uint32_t mb = 0;
    if ((uint32_t)qi < gcount) bucket_extent(a, b0 + (uint32_t)qi, xbase[qi], mb);
    xlen_min = min(xlen_min, mb);
  }
  auto whole_window = [&](uint32_t ws) -> bool { return ws + win <= xlen_min && win == kChunk; };
  auto load_x = [&](float4 (&dst)[NQ], uint32_t ws) {
    if (whole_window(ws)) {
#pragma unroll
      for (int qi = 0; qi < NQ; ++qi) dst[qi] = load_stream(a.x + xbase[qi] + ws + i);
      return;
    }
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
      dst[qi] = make_float4(0.f, 0.f, 0.f, 0.f);
      if ((uint32_t)qi < gcount) {
        uint64_t base;
        uint32_t mb;
        bucket_extent(a, b0 + (uint32_t)qi, base, mb);
        const uint32_t cntw = ws < mb ? min(win, mb - ws) : 0u;
        const float* xp = a.x + base + ws + i;
        if (i + 3 < cntw) {
          dst[qi] = load_stream(xp);
        } else {
          if (i + 0 < cntw) dst[qi].x = xp[0];
          if (i + 1 < cntw) dst[qi].y = xp[1];
          if (i + 2 < cntw) dst[qi].z = xp[2];
        }
      }
    }
  };
  // Order of the memory operations (the wait counter retires them in order): the x
  // values are requested at the start of a window and used at its end; the next piece
  // of a string is requested into registers at the top of a parse round (counting apply)
  // and at the end of a window, BEFORE that window's stores, and moved into the ring at
  // the top of the following round, so that waiting for string words never waits for a
  // store, and a round's own work hides their latency and that of the x values.
  uint32_t tw[kStrFetch], tw_base = 0;   // string words on their way: [tw_base, tw_base + kStrFetch)
  bool tw_pending = false;
  auto commit_pending = [&]() {
    if (tw_pending && sfill == tw_base) {   // (a fetch on demand may have overtaken them)
      ring_put_piece(ring, sfill, tw);
      sfill += kStrFetch;
    }
    tw_pending = false;
  };
  // Requests the next piece of the string into registers; commit_pending() moves it
  // into the ring later, so the round in between hides the latency.
  auto request_next = [&]() {
    tw_pending = pend_pos != kDone && sfill < nwords && sfill - (bitpos >> 5) <= kStrWin - kStrFetch;
    tw_base = sfill;
    if (tw_pending) load_piece(str, sfill, nwords, tw);
  };
  // Message-by-message apply: x is requested a whole window ahead, because its rounds
  // wait for string words at once and would wait for x with them.  Counting apply: the
  // string words of a round arrive a round later, so x is requested at the start of its
  // own window and one register set is enough (one more wavefront per SIMD).
  constexpr bool kAhead = KLOOP;
  float4 xr[NQ], xn[NQ];
  if constexpr (kAhead) load_x(xr, 0);
  for (uint32_t ws = 0; ws < a.d; ws += win) {
    const uint32_t wend = ws + win;  // positions (1-based) up to wend fall in this window
    if constexpr (kAhead) {
      if (wend < a.d) load_x(xn, wend);
    } else {
      load_x(xr, ws);
    }
    // ---- rounds: parse ahead into the rings, apply what is due --------------------------
    // A position may only be applied once EVERY string has been parsed past it,
    // or an element could receive message 5's term before message 2's.  `limit`
    // is the smallest position still pending in any string, minus 1, capped at
    // the window end; queued records past it wait in the ring.  Parsing is lazy:
    // nobody parses while every string is already past the window end, and when
    // some string is not, all of them fill their rings (fewer, fuller passes of
    // the divergent parse loop).
    for (;;) {
      // A parse pass costs as many trips of the divergent loop as its busiest lane
      // takes, so passes are short and start when most lanes can use all the trips
      // (their rings have room), or when a lane is out of records for this window.
      const uint64_t needy = __builtin_amdgcn_ballot_w64(pend_pos <= wend);
      const uint32_t nroom = (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(pend_pos != kDone && qcnt + kRoom <= rec));
      if (needy != 0 || nroom >= kParseLanes) {
        // top up the string rings together, then parse
        commit_pending();
        if constexpr (KLOOP) {
          // dense strings use up a piece in a round or two: have it now
          if (pend_pos != kDone && sfill < nwords && sfill - (bitpos >> 5) <= kStrWin - kStrFetch) fetch();
        } else {
          request_next();   // arrives while this round parses and applies
        }
        const uint32_t trips = __popcll(needy) >= 32 ? rec : kParse;   // dense data: no imbalance
        const uint32_t plim = parse_limit();
        for (uint32_t np = 0; np < trips; ++np) {
          const bool c1 = pend_pos != kDone, c2 = qcnt < rec, c3 = bitpos < plim;
          const bool act = c1 & c2 & c3;
          // (the wavefront's vote from the three comparisons' own masks: a vote on their
          // conjunction first turns it into a register and compares again)
          if ((__builtin_amdgcn_ballot_w64(c1) & __builtin_amdgcn_ballot_w64(c2) &
               __builtin_amdgcn_ballot_w64(c3)) == 0)
            break;
          if (act) {
            if (kSparse || pend_lev) {   // (Code_s records always carry a level >= 1)
              queue[qidx((uint32_t)lane, (qhead + qcnt) & (rec - 1))] =
                  (qrec_t)((pend_pos - 1u) | (pend_neg << 13) | ((pend_lev - kLevBias) << 14));
              ++qcnt;
            }
            advance(pend_pos);
          }
        }
        if (bad) { flag_corrupt(a.status); bad = 0; }
      }
      if constexpr (KLOOP) {
        // Dense data: nearly every ring slot is due in every round, so the records are
        // applied message by message: in turn kk, lane (g2, r) takes slot r of string
        // (g2, kk), and all strings of one message run side by side.
        uint32_t limit = wave_min_u32(pend_pos - 1u);   // (kDone - 1: no limit from this lane)
        limit = min(limit, wend);   // 0-based positions below `limit` are due
        counts[lane] = qcnt;
        heads[lane] = qhead;
        scales[lane] = my_scale;
        __syncthreads();
        const uint32_t g2 = (uint32_t)lane / rec, r = (uint32_t)lane - g2 * rec;
        for (uint32_t kk = 0; kk < K; ++kk) {
          if (g2 < gw) {
            const uint32_t sl = g2 * K + kk;
            if (r < counts[sl]) {
              const uint32_t q = queue[qidx(sl, (heads[sl] + r) & (rec - 1))];
              const uint32_t p0 = q & 0x1FFFu;
              if (p0 < limit) {
                const float mag = scales[sl] * (float)((q >> 14) + kLevBias);
                acc[g2 * winp + ((p0 - ws) & (winp - 1u))] += ((q >> 13) & 1u) ? -mag : mag;
              }
            }
          }
          __syncthreads();
        }
        // drop what was applied from the front of the ring
        while (qcnt && (queue[qidx((uint32_t)lane, qhead)] & 0x1FFFu) < limit) {
          qhead = (qhead + 1u) & (rec - 1);
          --qcnt;
        }
        if (limit == wend) break;
        continue;
      }
      // At most kApply records per lane are applied in a round: a lane that holds
      // more caps the limit at its first record beyond them.
      uint32_t qv[kApply + 1], ad[kApply];
#pragma unroll
      for (uint32_t t = 0; t <= kApply; ++t)
        qv[t] = queue[((qhead + t) & (kRec - 1)) * 64u + lane];
      const uint32_t cap = qcnt > kApply ? (qv[kApply] & 0x1FFFu) : 0xFFFFFFFFu;
      uint32_t limit = wave_min_u32(min(pend_pos - 1u, cap));   // (kDone - 1: no limit)
      limit = min(limit, wend);   // 0-based positions below `limit` are due
      // ---- apply the due records of this lane's own ring ---------------------------------
      // All records of one position become due in the same round, and the position's word of
      // the accumulator is 0 until then.  That word first collects WHO has a term there, a bit
      // per message (K <= 32 on this path): a record's rank among the set bits below its own is
      // its turn in the sum that Alg. 1's last line takes message by message.  Then
      //   turn 0    stores its term (0 + t = t),
      //   turn r    adds its term to what turns 0 .. r-1 left, r = 1, 2, ... while any lane
      //             still has a record waiting: as many passes as the busiest position of
      //             the round has terms, not one per message.
      // Every pass handles the ring entries in groups of kGrp with straight-line code: entries
      // that do not take part read and write the lane's dump word instead of branching, so
      // that the LDS operations of a group are in flight together.
      constexpr uint32_t kGrp = 4;
      {
        // (positions ascend along a string, so the due entries are the first `ndue` of the ring)
        bool due[kApply];
        uint32_t ndue = 0;
#pragma unroll
        for (uint32_t t = 0; t < kApply; ++t) {
          const uint32_t p0 = qv[t] & 0x1FFFu;
          ad[t] = grow + ((p0 - ws) & (winp - 1u));
          due[t] = (t < qcnt) & (p0 < limit);
          ndue += due[t] ? 1u : 0u;
        }
        // uniform: does any lane apply an entry of the group that starts at t0?  (a vote per
        // group costs a comparison; the wavefront's maximum would cost a dozen shuffles)
        bool grp[kApply / kGrp];
#pragma unroll
        for (uint32_t t0 = 0; t0 < kApply; t0 += kGrp)
          grp[t0 / kGrp] = __builtin_amdgcn_ballot_w64(ndue > t0) != 0;
        const uint32_t kbit = 1u << k;
#pragma unroll
        for (uint32_t t0 = 0; t0 < kApply; t0 += kGrp) {
          if (!grp[t0 / kGrp]) break;
#pragma unroll
          for (uint32_t j = 0; j < kGrp; ++j) atomicOr(&accu[ad[t0 + j]], due[t0 + j] ? kbit : 0u);
        }
        __syncthreads();
        // a byte per ring entry: its turn, 0xFF for an entry that is not due
        uint32_t turn[kApply / 4];
        static_assert(kApply % 4 == 0, "turns are packed four to a word");
#pragma unroll
        for (uint32_t t = 0; t < kApply / 4; ++t) turn[t] = 0xFFFFFFFFu;
        uint32_t last = 0;   // the highest turn of this lane's entries
#pragma unroll
        for (uint32_t t0 = 0; t0 < kApply; t0 += kGrp) {
          if (!grp[t0 / kGrp]) break;
          uint32_t who[kGrp];
#pragma unroll
          for (uint32_t j = 0; j < kGrp; ++j) who[j] = accu[ad[t0 + j]];
#pragma unroll
          for (uint32_t j = 0; j < kGrp; ++j) {
            const uint32_t t = t0 + j;
            const uint32_t mine = (uint32_t)__popc(who[j] & (kbit - 1u));
            const uint32_t sh = 8u * (t & 3u);
            turn[t / 4] = due[t] ? (turn[t / 4] & ~(0xFFu << sh)) | (mine << sh) : turn[t / 4];
            last = due[t] ? max(last, mine) : last;
          }
        }
        __syncthreads();
        float term[kApply];
#pragma unroll
        for (uint32_t t = 0; t < kApply; ++t) {
          const float mag = my_scale * (float)((qv[t] >> 14) + kLevBias);
          term[t] = ((qv[t] >> 13) & 1u) ? -mag : mag;
        }
#pragma unroll
        for (uint32_t t0 = 0; t0 < kApply; t0 += kGrp) {
          if (!grp[t0 / kGrp]) break;
#pragma unroll
          for (uint32_t j = 0; j < kGrp; ++j) {
            const uint32_t t = t0 + j;
            const bool now = ((turn[t / 4] >> (8u * (t & 3u))) & 0xFFu) == 0u;
            acc[now ? ad[t] : dump] = term[t];
          }
        }
        __syncthreads();
        for (uint32_t r = 1; __builtin_amdgcn_ballot_w64(last >= r) != 0; ++r) {
#pragma unroll
          for (uint32_t t0 = 0; t0 < kApply; t0 += kGrp) {
            if (!grp[t0 / kGrp]) break;
            float old[kGrp];
            uint32_t at[kGrp];
#pragma unroll
            for (uint32_t j = 0; j < kGrp; ++j) {
              const uint32_t t = t0 + j;
              const bool now = ((turn[t / 4] >> (8u * (t & 3u))) & 0xFFu) == r;
              at[j] = now ? ad[t] : dump;
              old[j] = acc[at[j]];
            }
#pragma unroll
            for (uint32_t j = 0; j < kGrp; ++j) acc[at[j]] = old[j] + term[t0 + j];
          }
          __syncthreads();
        }
        qhead = (qhead + ndue) & (kRec - 1);
        qcnt -= ndue;
        if (limit == wend) break;   // uniform: every string is parsed past this window
      }
    }
    // ---- string words requested a window ago arrive; request the next ones ---------------
    commit_pending();
    request_next();
    // ---- combine the accumulator with x and store ------------------------------------
    if (whole_window(ws)) {
#pragma unroll
      for (int qi = 0; qi < NQ; ++qi) {
        float* ap = acc + qi * winp + i;
        const float4 av = *reinterpret_cast<float4*>(ap);
        *reinterpret_cast<float4*>(ap) = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 xv = xr[qi];
        if (a.step) {
          xv.x = fmaf(-a.c, av.x, xv.x); xv.y = fmaf(-a.c, av.y, xv.y);
          xv.z = fmaf(-a.c, av.z, xv.z); xv.w = fmaf(-a.c, av.w, xv.w);
        } else {
          xv.x += av.x; xv.y += av.y; xv.z += av.z; xv.w += av.w;
        }
        store_stream(a.x + xbase[qi] + ws + i, xv);
      }
    } else {
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
      if ((uint32_t)qi < gcount) {
        uint64_t base;
        uint32_t mb;
        bucket_extent(a, b0 + (uint32_t)qi, base, mb);
        const uint32_t cntw = ws < mb ? min(win, mb - ws) : 0u;
        float* xp = a.x + base + ws + i;
        float* ap = acc + qi * winp + i;
        if (i < cntw) {
          const float4 av = *reinterpret_cast<float4*>(ap);
          *reinterpret_cast<float4*>(ap) = make_float4(0.f, 0.f, 0.f, 0.f);
          float4 xv = xr[qi];
          if (a.step) {
            xv.x = fmaf(-a.c, av.x, xv.x); xv.y = fmaf(-a.c, av.y, xv.y);
            xv.z = fmaf(-a.c, av.z, xv.z); xv.w = fmaf(-a.c, av.w, xv.w);
          } else {
            xv.x += av.x; xv.y += av.y; xv.z += av.z; xv.w += av.w;
          }
          if (i + 3 < cntw) {
            store_stream(xp, xv);
          } else {
            xp[0] = xv.x;
            if (i + 1 < cntw) xp[1] = xv.y;
            if (i + 2 < cntw) xp[2] = xv.z;
          }
        }
      }
    }
    }
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi)
      if constexpr (kAhead) xr[qi] = xn[qi];
    __syncthreads();
  }
}

template <int CODE, int LG, int NQ, bool KLOOP, bool Q16>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(NQ == 4 && !KLOOP ? QSGD_DEC_WAVES : 1)))
void k_decode_elias(DecodeArgs a) {
  if (*a.status != 0) return;
  extern __shared__ uint32_t smem[];
  // LDS: [acc: gw*winp floats][record rings][string rings: 64*kRingStride][Elias table: 32][dump 64]
  //      [counts 64][heads 64][scales 64]
  using qrec_t = std::conditional_t<Q16, uint16_t, uint32_t>;
  const uint32_t gw = a.gw, winp = a.winp;
  float* const acc = reinterpret_cast<float*>(smem);
  qrec_t* const queue = reinterpret_cast<qrec_t*>(smem + gw * winp);
  uint32_t* const swin = smem + gw * winp + rec_words(Q16);
  const uint32_t b0 = blockIdx.x * gw;
  const uint32_t gcount = min(gw, a.nb - b0);  // buckets this wavefront really has
  decode_elias_body<CODE, LG, NQ, KLOOP, Q16>(a, acc, queue, swin, b0, gcount);
}

// ---- Elias codes, dense strings: a tile of signed levels, summed in registers -----------
// Where most coordinates carry a nonzero level (Code'_s, or Code_s with s^2 of the order of
// d: Lemma 3.1 (iii)), a window of W positions holds about as many records per string as
// positions, and every position receives up to K terms whose fp32 sum has to be taken in
// message order.  So the two halves of the work are separated by the data layout instead of
// by queues and turns:
//   phase 1  every lane parses its own string (bucket g of message k) up to the end of the
//            window and writes each record's signed level as ONE byte into its own row of a
//            tile in LDS (64 rows of W bytes, zero = no record): plain stores, no two lanes
//            share a byte, nothing to wait for.  String words come through a small per-lane
//            ring that all lanes top up together every kTileBatch records, a batch ahead.
//   phase 2  lane l owns positions W/64 * l .. of the window in every bucket: for bucket g it
//            reads its bytes of the rows (g, 0) .. (g, K-1) in message order, turns each
//            into scale_k * level (the scale comes from the lane that parsed the string) and
//            adds them up in registers: the sum ((0 + g^0) + g^1) + ... of Alg. 1's last
//            line by construction, then the update of x (read at the start of the window).
// Levels must fit a signed byte (s <= 127).
#ifndef QSGD_TILE_BATCH
#define QSGD_TILE_BATCH 8
#endif
constexpr uint32_t kTileBatch = QSGD_TILE_BATCH;   // records a lane parses between two top-ups of its ring

// NARROW: a whole record (gap, sign, level) fits the 32 bits of one peek.
template <int CODE, int LG, int NQ, int W, bool NARROW>
__global__ __launch_bounds__(64) void k_decode_tile(DecodeArgs a) {
  if (*a.status != 0) return;
  extern __shared__ uint32_t smem[];
  constexpr bool kSparse = CODE == QSGD_CODE_SPARSE;
  constexpr bool kNarrow = !kSparse || NARROW;
  constexpr uint32_t VPL = W / 64;          // positions of a window a lane owns (2 or 4)
  static_assert(VPL == 1 || VPL == 2 || VPL == 4, "window of 64, 128 or 256 positions");
  int8_t* const tile = reinterpret_cast<int8_t*>(smem);          // [64][W]
  uint32_t* const swin = smem + 64 * W / 4;                       // [64][kRingStride]
  uint8_t* const otab = reinterpret_cast<uint8_t*>(swin + 64 * kRingStride);   // [128]
  const uint32_t K = a.K, gw = a.gw, s = a.s, win = a.win;
  const int lane = threadIdx.x;
  const uint32_t b0 = blockIdx.x * gw;
  const uint32_t gcount = min(gw, a.nb - b0);
  const uint64_t pay = (uint64_t)H_WORDS + a.table_words;

  // ---- open this lane's string -----------------------------------------------------
  const uint32_t g = lane / K, k = lane - g * K;
  const uint32_t b = b0 + g;
  // The record a lane has read and not yet stored: 1-based position (kDone: none, the
  // string has ended or is damaged), level and sign.  One number answers both "is there a
  // record" and "does it fall in this window", which keeps the parse loop's bookkeeping
  // off the scalar unit: every instruction of that loop, scalar ones included, is a step
  // of a chain that one lane's string forces to be serial.
  constexpr uint32_t kDone = 0xFFFFFFFFu;
  uint32_t m = 0, endbit = 0, nwords = 0;
  uint32_t pend_pos = kDone, pend_lev = 0, pend_neg = 0;
  const uint32_t* str = nullptr;
  bool open = false;
  float my_scale = 0.f;
  if (g < gcount) {
    uint64_t base_unused;
    bucket_extent(a, b, base_unused, m);
    const uint32_t* msg = a.msgs[k];
    const uint32_t o0 = msg[H_WORDS + b], o1 = msg[H_WORDS + b + 1];
    if (o0 < o1 && pay + o1 <= a.msg_words[k]) {
      nwords = o1 - o0;
      str = msg + pay + o0;
      my_scale = __uint_as_float(str[0]) / (float)s;
      open = true;
      if (kSparse) {
        const uint32_t last = str[nwords - 1];
        endbit = nwords * 32u - 1u - (uint32_t)(__ffs((int)last) - 1);
        if (last == 0 || endbit < 32u) open = false;
      } else {
        endbit = nwords * 32u;
      }
    }
    if (!open) flag_corrupt(a.status);
  }
  if (!open) my_scale = 0.f;

  // The lane's view of its string: the last kStrWin words fetched, as a ring in LDS: word j
  // of the string in slot j % kStrWin of the lane's kStrWin + 1 slots; the last slot mirrors
  // slot 0, so that two consecutive words are always two consecutive slots (one LDS read
  // of a pair), and the odd stride keeps the lanes on distinct banks.
  uint32_t* const ring = swin + (uint32_t)lane * kRingStride;
  uint32_t sfill = 0;   // words [sfill - kStrWin, sfill) of the string are in the ring
  auto fetch = [&]() {
    uint32_t t[kStrFetch];
    load_piece(str, sfill, nwords, t);
    ring_put_piece(ring, sfill, t);
    sfill += kStrFetch;
  };
  // The 32 stream bits from bit `at` on, out of the ring (bit j of the stream is bit
  // 31 - j % 32 of word j / 32).  No shift register to maintain: the parser keeps a bit
  // position, and the vector ALU, which bounds this kernel, only aligns two words.
  auto peek = [&](uint32_t at) -> uint32_t {
    const uint32_t off = at & 31u;
    const uint32_t* const pw = ring + ((at >> 5) & (kStrWin - 1u));
    const uint32_t wa = pw[0], wb = pw[1];
    const uint32_t sh = __builtin_amdgcn_alignbit(wa, wb, 32u - off);   // (off = 0 gives wb)
    return off ? sh : wa;
  };
  // Recursive Elias code through the table: entry (after, more) of the next 7 bits says
  // where the last group's bits after its leading 1 start and how many they are; the value
  // is 2^more + those bits, the code word after + more + 1 bits (with its closing 0, which
  // `open_end` checks: its top bit is set if the word does not end there).
  auto omega_tab = [&](uint32_t w, uint32_t& len, uint32_t& open_end) -> uint32_t {
    const uint32_t e = otab[w >> 25];
    const uint32_t after = e & 7u, more = e >> 3;
    const uint32_t y = w << after;
    const uint32_t rest = __builtin_amdgcn_ubfe(y, 32u - more, more);   // (more = 0: 0)
    open_end = y << more;
    len = after + more + 1u;
    return (1u << more) | rest;
  };
  uint32_t bp = 32;   // next unread bit (after the scale)
  // A record reads at most the two words at bp / 32 (NARROW) or one more, so the lane may
  // parse while bp is below `plim` (no limit once the whole string is in the ring: past its
  // end the ring may hold anything, those bits lie behind endbit).
  auto parse_limit = [&]() -> uint32_t {
    return sfill >= nwords ? 0xFFFFFFFFu : (sfill - (kNarrow ? 1u : 2u)) * 32u;
  };
  uint32_t bad = 0;   // a record that cannot be: remembered here, reported after the batch
  // Reads the next record; `pos` is the position of the one before (0 at the start).
  auto advance = [&](uint32_t pos) {
    uint32_t w = peek(bp);
    if (kSparse) {
      const bool more = bp < endbit;
      uint32_t gl, ll, e1, e2;
      const uint32_t gap = omega_tab(w, gl, e1);
      if (!kNarrow) w = peek(bp + gl); else w <<= gl;
      pend_neg = w >> 31;
      const uint32_t lev = omega_tab(w << 1, ll, e2);
      bp += gl + 1u + ll;
      pos += gap;
      pend_lev = lev;
      // (no short cuts between the tests: as plain mask arithmetic they cost no branch)
      const bool bad_rec = ((int)(e1 | e2) < 0) | (lev > s) | (pos > m) | (bp > endbit);
      bad |= (more & bad_rec) ? 1u : 0u;
      pend_pos = (more & !bad_rec) ? pos : kDone;
    } else {
      const bool more = pos < m;
      uint32_t ll, e2;
      const uint32_t lev1 = omega_tab(w << 1, ll, e2);
      bp += 1u + ll;
      pend_neg = w >> 31;
      pend_lev = lev1 - 1u;
      const bool bad_rec = ((int)e2 < 0) | (lev1 > s + 1u) | (bp > endbit);
      bad |= (more & bad_rec) ? 1u : 0u;
      pend_pos = (more & !bad_rec) ? pos + 1u : kDone;
    }
  };
  for (uint32_t b7 = lane; b7 < 128u; b7 += 64) otab[b7] = omega_table_entry(b7);
  if (open) {
    fetch();
    fetch();
  }
  __syncthreads();
  if (open) advance(0u);
  if (bad) { flag_corrupt(a.status); bad = 0; }

  // The next kStrFetch words of the string are always on their way (in registers) while the
  // ring still holds unread ones: they are requested at a top-up and enter the ring at a
  // later one, once the lane has used up enough of the ring, a batch of parsing in between.
  uint32_t tw[kStrFetch];
  bool tw_pending = false;
#pragma unroll
  for (uint32_t j = 0; j < kStrFetch; ++j) tw[j] = 0u;
  auto commit_pending = [&]() {
    if (tw_pending && sfill - (bp >> 5) <= kStrWin - kStrFetch) {
      ring_put_piece(ring, sfill, tw);
      sfill += kStrFetch;
      tw_pending = false;
    }
  };
  auto request_next = [&]() {
    if (!tw_pending && pend_pos != kDone && sfill < nwords) {
      tw_pending = true;
      load_piece(str, sfill, nwords, tw);
    }
  };

  for (uint32_t j = lane; j < 64u * W / 4u; j += 64) smem[j] = 0u;
  __syncthreads();

  int8_t* const row = tile + (uint32_t)lane * W;
  const uint32_t i = (uint32_t)lane * VPL;   // first window position this lane owns
  float xr[NQ][VPL];
  for (uint32_t ws = 0; ws < a.d; ws += win) {
    const uint32_t wend = ws + win;  // positions (1-based) up to wend fall in this window
    // ---- string words for this window's first batch; x of this window ---------------------
    commit_pending();
    request_next();
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
#pragma unroll
      for (uint32_t j = 0; j < VPL; ++j) xr[qi][j] = 0.f;
      if ((uint32_t)qi < gcount) {
        uint64_t base;
        uint32_t mb;
        bucket_extent(a, b0 + (uint32_t)qi, base, mb);
        const uint32_t cntw = ws < mb ? min(win, mb - ws) : 0u;
        const float* xp = a.x + base + ws + i;
        if (i + VPL - 1 < cntw) {
          if constexpr (VPL == 4) {
            const float4 v = load_stream(xp);
            xr[qi][0] = v.x; xr[qi][1] = v.y; xr[qi][2] = v.z; xr[qi][3] = v.w;
          } else if constexpr (VPL == 2) {
            const float2 v = *reinterpret_cast<const float2*>(xp);
            xr[qi][0] = v.x; xr[qi][1] = v.y;
          } else {
            xr[qi][0] = xp[0];
          }
        } else {
#pragma unroll
          for (uint32_t j = 0; j < VPL; ++j)
            if (i + j < cntw) xr[qi][j] = xp[j];
        }
      }
    }
    // ---- phase 1: this lane's records of the window into its row of the tile ---------------
    for (;;) {
      const uint32_t plim = parse_limit();
      for (uint32_t t = 0; t < kTileBatch; ++t) {
        const bool c1 = pend_pos <= wend, c2 = bp < plim;
        const bool act = c1 & c2;
        // (the wavefront's vote from the two comparisons' own masks: a vote on their
        // conjunction first turns it into a register and compares again)
        if ((__builtin_amdgcn_ballot_w64(c1) & __builtin_amdgcn_ballot_w64(c2)) == 0) break;
        if (act) {
          if (kSparse || pend_lev)
            row[pend_pos - 1u - ws] = (int8_t)(pend_neg ? -(int)pend_lev : (int)pend_lev);
          advance(pend_pos);
        }
      }
      if (__builtin_amdgcn_ballot_w64(pend_pos <= wend) == 0) break;
      commit_pending();
      request_next();
    }
    if (bad) { flag_corrupt(a.status); bad = 0; }
    __syncthreads();
    // ---- phase 2: sum the K rows of every bucket in message order, update x ---------------
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
      if ((uint32_t)qi < gcount) {
        float sum[VPL];
#pragma unroll
        for (uint32_t j = 0; j < VPL; ++j) sum[j] = 0.f;
        for (uint32_t kk = 0; kk < K; ++kk) {
          const uint32_t r = (uint32_t)qi * K + kk;   // the lane that parsed string (qi, kk)
          const float sc = __uint_as_float(lane_bcast(__float_as_uint(my_scale), (int)r));
          uint32_t w;
          if constexpr (VPL == 4) {
            uint32_t* const p = reinterpret_cast<uint32_t*>(tile + r * W) + lane;
            w = *p;
            *p = 0u;
          } else if constexpr (VPL == 2) {
            uint16_t* const p = reinterpret_cast<uint16_t*>(tile + r * W) + lane;
            w = *p;
            *p = 0;
          } else {
            uint8_t* const p = reinterpret_cast<uint8_t*>(tile + r * W) + lane;
            w = *p;
            *p = 0;
          }
#pragma unroll
          for (uint32_t j = 0; j < VPL; ++j) {
            const int lev = (int)(int8_t)(w >> (8u * j));
            sum[j] += sc * (float)lev;     // sign * (scale * level), Eq. (2)
          }
        }
        uint64_t base;
        uint32_t mb;
        bucket_extent(a, b0 + (uint32_t)qi, base, mb);
        const uint32_t cntw = ws < mb ? min(win, mb - ws) : 0u;
        float* xp = a.x + base + ws + i;
        float out[VPL];
#pragma unroll
        for (uint32_t j = 0; j < VPL; ++j)
          out[j] = a.step ? fmaf(-a.c, sum[j], xr[qi][j]) : xr[qi][j] + sum[j];
        if (i + VPL - 1 < cntw) {
          if constexpr (VPL == 4) {
            store_stream(xp, make_float4(out[0], out[1], out[2], out[3]));
          } else if constexpr (VPL == 2) {
            *reinterpret_cast<float2*>(xp) = make_float2(out[0], out[1]);
          } else {
            xp[0] = out[0];
          }
        } else {
#pragma unroll
          for (uint32_t j = 0; j < VPL; ++j)
            if (i + j < cntw) xp[j] = out[j];
        }
      }
    }
    __syncthreads();
  }
}

hipError_t launch_decode_check(const DecodeArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(k_decode_check, dim3(1), dim3(64), 0, st, a);
  return hipGetLastError();
}

template <int CH, bool CHECK>
static void launch_fixed_ch(const DecodeArgs& a, dim3 grid, dim3 block, hipStream_t st) {
  switch (a.fixed_bits) {
    case 2: hipLaunchKernelGGL((k_decode_fixed<2, CH, CHECK>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((k_decode_fixed<4, CH, CHECK>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((k_decode_fixed<8, CH, CHECK>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((k_decode_fixed<16, CH, CHECK>), grid, block, 0, st, a); break;
  }
}

template <bool CHECK>
static void launch_fixed_check(const DecodeArgs& a, dim3 grid, dim3 block, hipStream_t st) {
  if (a.d <= kChunk) launch_fixed_ch<1, CHECK>(a, grid, block, st);
  else if (a.d <= 2 * kChunk) launch_fixed_ch<2, CHECK>(a, grid, block, st);
  else launch_fixed_ch<4, CHECK>(a, grid, block, st);
}

hipError_t launch_decode_fixed(const DecodeArgs& a, uint32_t blocks, hipStream_t st) {
  const dim3 grid(blocks), block(256);
  const bool check = ((1ull << a.fixed_bits) - 1ull) > a.s;
  if (check) launch_fixed_check<true>(a, grid, block, st);
  else launch_fixed_check<false>(a, grid, block, st);
  return hipGetLastError();
}

template <int CODE, int NQ, bool KLOOP>
static hipError_t launch_elias_kl(const DecodeArgs& a, int lg, uint32_t blocks, size_t lds,
                                  hipStream_t st) {
  const dim3 grid(blocks), block(64);
  if constexpr (CODE == QSGD_CODE_SPARSE && !KLOOP) {
    if (a.q16) {  // s <= 4: one or two groups
      if (lg == 1) hipLaunchKernelGGL((k_decode_elias<CODE, 1, NQ, false, true>), grid, block, lds, st, a);
      else hipLaunchKernelGGL((k_decode_elias<CODE, 2, NQ, false, true>), grid, block, lds, st, a);
      return hipGetLastError();
    }
  }
  switch (lg) {
    case 1: hipLaunchKernelGGL((k_decode_elias<CODE, 1, NQ, KLOOP, false>), grid, block, lds, st, a); break;
    case 2: hipLaunchKernelGGL((k_decode_elias<CODE, 2, NQ, KLOOP, false>), grid, block, lds, st, a); break;
    case 3: hipLaunchKernelGGL((k_decode_elias<CODE, 3, NQ, KLOOP, false>), grid, block, lds, st, a); break;
    default: hipLaunchKernelGGL((k_decode_elias<CODE, 4, NQ, KLOOP, false>), grid, block, lds, st, a); break;
  }
  return hipGetLastError();
}

template <int CODE, int NQ>
static hipError_t launch_elias_nq(const DecodeArgs& a, int lg, uint32_t blocks, size_t lds,
                                  hipStream_t st) {
  return a.kloop ? launch_elias_kl<CODE, NQ, true>(a, lg, blocks, lds, st)
                 : launch_elias_kl<CODE, NQ, false>(a, lg, blocks, lds, st);
}

template <int CODE>
static hipError_t launch_elias_code(const DecodeArgs& a, int lg, uint32_t blocks, size_t lds,
                                    hipStream_t st) {
  const uint32_t nq = a.gw;  // float4 of x per lane per window: one per bucket
  if (nq <= 4) return launch_elias_nq<CODE, 4>(a, lg, blocks, lds, st);
  if (nq <= 8) return launch_elias_nq<CODE, 8>(a, lg, blocks, lds, st);
  return launch_elias_nq<CODE, 16>(a, lg, blocks, lds, st);
}

template <int CODE, int NQ, int W>
static hipError_t launch_tile_lg(const DecodeArgs& a, int lg, uint32_t blocks, size_t lds,
                                 hipStream_t st) {
  const dim3 grid(blocks), block(64);
  // the longest record: Elias(d) for the gap, the sign, Elias(s) for the level
  auto bits_of = [](uint32_t k) {   // length of Elias(k)
    uint32_t len = 1;
    while (k > 1) {
      uint32_t nb = 0;
      for (uint32_t t = k; t; t >>= 1) ++nb;
      len += nb;
      k = nb - 1;
    }
    return len;
  };
  const bool narrow = a.code != QSGD_CODE_SPARSE || lg <= 2 ||
                      bits_of(a.d) + 1u + bits_of(a.s) <= 32u;
#define QSGD_TILE(LGV)                                                                          \
  if (narrow) hipLaunchKernelGGL((k_decode_tile<CODE, LGV, NQ, W, true>), grid, block, lds, st, a); \
  else hipLaunchKernelGGL((k_decode_tile<CODE, LGV, NQ, W, false>), grid, block, lds, st, a)
  switch (lg) {
    case 1: QSGD_TILE(1); break;
    case 2: QSGD_TILE(2); break;
    default: QSGD_TILE(3); break;
  }
#undef QSGD_TILE
  return hipGetLastError();
}

template <int CODE, int W>
static hipError_t launch_tile_nq(const DecodeArgs& a, int lg, uint32_t blocks, size_t lds,
                                 hipStream_t st) {
  if (a.gw <= 4) return launch_tile_lg<CODE, 4, W>(a, lg, blocks, lds, st);
  if (a.gw <= 8) return launch_tile_lg<CODE, 8, W>(a, lg, blocks, lds, st);
  return launch_tile_lg<CODE, 16, W>(a, lg, blocks, lds, st);
}

// Dense strings, s <= 127 (a level fits a signed byte): a.tile_w = 128 or 256.
hipError_t launch_decode_tile(const DecodeArgs& a, uint32_t blocks, size_t lds, hipStream_t st) {
  const uint32_t top = a.code == QSGD_CODE_SPARSE ? a.s : a.s + 1u;
  const int lg = top <= 3 ? 1 : top <= 15 ? 2 : 3;
#define QSGD_TILE_W(CODEV)                                                              \
  switch (a.tile_w) {                                                                    \
    case 64: return launch_tile_nq<CODEV, 64>(a, lg, blocks, lds, st);                   \
    case 128: return launch_tile_nq<CODEV, 128>(a, lg, blocks, lds, st);                 \
    default: return launch_tile_nq<CODEV, 256>(a, lg, blocks, lds, st);                  \
  }
  if (a.code == QSGD_CODE_SPARSE) { QSGD_TILE_W(QSGD_CODE_SPARSE) }
  QSGD_TILE_W(QSGD_CODE_DENSE)
#undef QSGD_TILE_W
}

// Groups in the longest level code word: Elias(s) (sparse) or Elias(s + 1) (dense).
hipError_t launch_decode_elias(const DecodeArgs& a, uint32_t blocks, size_t lds, hipStream_t st) {
  const uint32_t top = a.code == QSGD_CODE_SPARSE ? a.s : a.s + 1u;
  const int lg = top <= 3 ? 1 : top <= 15 ? 2 : top <= 65535 ? 3 : 4;
  if (a.code == QSGD_CODE_SPARSE) return launch_elias_code<QSGD_CODE_SPARSE>(a, lg, blocks, lds, st);
  return launch_elias_code<QSGD_CODE_DENSE>(a, lg, blocks, lds, st);
}

}  // namespace qsgd
