// Argument blocks and launchers of the HIP kernels (internal to libqsgd).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qsgd.h"

namespace qsgd {

constexpr uint32_t kMaxBucketFast = 8192;  // largest bucket the register path holds
constexpr uint32_t kMaxTeams = 8192;       // most teams (regions) one encode uses
// Team encoder of the Elias codes: waves per SIMD the compiler budgets registers for, and
// wavefronts of persistent teams per compute unit.  Measured on c5 with the survivor ring:
// 4 / 32 -> 0.63 ms per 5e8 values, 4 / 96 -> 0.61, 6 / 96 -> 0.54.  With the survivor
// list (sparse data, teams of four wavefronts) LDS lets a compute unit hold five teams, so
// its kernels are budgeted for five waves and keep every value in a register; per 1e9
// values: 4 waves 1.09 ms, 5 waves 1.00, 6 waves (registers spilled) 1.00.
#ifndef QSGD_ENC_WAVES
#define QSGD_ENC_WAVES 6
#endif
// Ring decoder of the Elias codes: waves per SIMD its registers are budgeted for (LDS lets a
// compute unit hold twenty of its one-wavefront workgroups on the workload it is tuned on).
#ifndef QSGD_DEC_WAVES
#define QSGD_DEC_WAVES 5
#endif
#ifndef QSGD_ENC_WAVES_LIST
#define QSGD_ENC_WAVES_LIST 5
#endif
#ifndef QSGD_ENC_TEAMS
#define QSGD_ENC_TEAMS 128u
#endif
// Small-bucket fixed-width encoder: wavefronts per compute unit the grid may have.  A
// persistent grid (32 per CU) measured 0.19 ms on c3, one pass per wavefront 0.15 ms.
#ifndef QSGD_FS_TEAMS
#define QSGD_FS_TEAMS 1024u
#endif
// ... and waves per SIMD its registers are budgeted for (c3, in the benchmark: 5 -> 0.168 ms, 6 -> 0.163, 7 -> 0.169 on one box).
#ifndef QSGD_FS_WAVES
#define QSGD_FS_WAVES 6
#endif
#ifndef QSGD_FIXED_BPC
#define QSGD_FIXED_BPC 512  // fixed-width decode: workgroups per compute unit
#endif
#ifndef QSGD_FIXED_KG
#define QSGD_FIXED_KG 8     // fixed-width decode: messages requested together
#endif
#ifndef QSGD_STR_WIN
#define QSGD_STR_WIN 8
#endif
constexpr uint32_t kStrWin = QSGD_STR_WIN;  // Elias decode: words of a string a lane keeps in LDS
#ifndef QSGD_REC
#define QSGD_REC 16
#endif
constexpr uint32_t kRec = QSGD_REC;               // Elias decode: records a lane queues ahead
// LDS words of a wavefront's record rings: a record is (position, sign, level); with
// s <= 4 it fits 16 bits (13 + 1 + 2, the level stored minus one), else it takes 32.
__host__ __device__ constexpr uint32_t rec_words(bool q16) { return q16 ? 32u * kRec : 64u * kRec; }
#ifndef QSGD_APPLY
#define QSGD_APPLY 8
#endif
constexpr uint32_t kApply = QSGD_APPLY;              // Elias decode: records a lane applies per round
#ifndef QSGD_PARSE
#define QSGD_PARSE 8
#endif
#ifndef QSGD_PARSE_LANES
#define QSGD_PARSE_LANES 32
#endif
#ifndef QSGD_ROOM
#define QSGD_ROOM QSGD_PARSE
#endif
constexpr uint32_t kRoom = QSGD_ROOM;        // ring slots a lane must have free to count as "has room"
constexpr uint32_t kParse = QSGD_PARSE;      // Elias decode: trips of a short parse pass
constexpr uint32_t kParseLanes = QSGD_PARSE_LANES;  // lanes with room that start a pass
constexpr uint32_t kStrFetch = kStrWin / 2; // words fetched at a time

// Tensor-aware messages: bucket b covers values [4 * btab[b].x, 4 * btab[b].x + btab[b].y)
// of the arena (a null table means bucket b = [b*d, min(n, (b+1)*d))).
template <class Args>
__device__ __forceinline__ void bucket_extent(const Args& a, uint32_t b, uint64_t& base,
                                              uint32_t& m) {
  if (a.btab) {
    const uint2 e = a.btab[b];
    base = (uint64_t)e.x * 4u;
    m = e.y;
  } else {
    base = (uint64_t)b * a.d;
    m = (uint32_t)min((uint64_t)a.d, a.n - base);
  }
}

struct EncodeArgs {
  const float* g;
  const uint2* btab;    // per-bucket (start / 4, length) or null
  uint32_t version;     // header version: 1 flat, 2 tensor-aware
  uint64_t index_base;  // draw index of g[0] (a slice of a longer vector), multiple of 4
  uint64_t n;
  uint32_t d;           // bucket size (<= kMaxBucketFast on this path)
  uint32_t nb;          // number of buckets
  uint32_t s;
  uint32_t norm_mode;
  uint32_t key0, key1;  // Philox key (seed low, high)
  uint32_t stream_id, iteration;
  uint32_t bper;        // buckets per team
  uint32_t dst_words;   // LDS words of the bucket-string image (even)
  uint32_t sub_words;   // LDS words of one wave's sub-stream (even)
  uint32_t ring;        // records in a wavefront's survivor ring (Code_s): 256 or 128
  uint32_t* header;     // message header (16 words)
  uint32_t* table;      // nb+1 word offsets (Elias codes)
  uint32_t* staging;    // workspace: one region per team
  uint64_t region_words;
  uint32_t* totals;     // workspace: words appended by each team
  // fixed width only
  uint32_t* payload;
  uint32_t fixed_bits;
  uint32_t fixed_words_full;  // words of a full bucket's string
  uint64_t fixed_payload_words;
};

struct CompactArgs {
  const uint32_t* staging;
  uint64_t region_words;
  const uint32_t* totals;
  unsigned long long* prefix;  // workspace: words appended by the teams before each team
  uint32_t* table;
  uint32_t* payload;
  uint32_t* header;
  uint64_t cap_words;  // payload words the message buffer can hold
  uint32_t bper;
  uint32_t nb;
  uint32_t table_words;  // padded table length
  uint64_t raw_words;    // raw fp32 words that follow the strings (tensor-aware messages)
};

struct DecodeArgs {
  const uint32_t* msgs[QSGD_MAX_PEERS];
  uint64_t msg_words[QSGD_MAX_PEERS];  // readable words behind each pointer
  uint32_t K;
  const uint2* btab;     // per-bucket (start / 4, length) or null
  uint32_t version;      // header version the messages must carry
  uint64_t raw_words;    // tensor-aware messages: raw values behind the strings
  uint64_t n;
  uint32_t d;
  uint32_t nb;
  uint32_t s;
  uint32_t code;
  uint32_t norm_mode;
  uint32_t table_words;  // padded table length in words (0 for fixed width)
  float* x;              // acc (accumulate) or x (step)
  float c;               // eta / K (step)
  uint32_t step;         // 1: x <- fma(-c, sum, x); 0: x <- x + sum
  uint32_t* status;      // workspace word 0
  // Elias path geometry
  uint32_t gw;           // buckets per wavefront
  uint32_t win;          // window (positions per bucket per pass), multiple of 4
  uint32_t winp;         // accumulator stride per bucket: win rounded up to 256
  uint32_t rec;          // record slots per string (message-by-message apply)
  uint32_t kloop;        // 1: records are applied message by message (dense messages)
  uint32_t q16;          // 1: 16-bit records (counting apply, s <= 4)
  uint32_t together;     // 1: long buckets, all messages read at once (few shared coordinates)
  uint32_t tile_w;       // dense strings with s <= 127: window of the tile decoder (128 or 256), else 0
  // fixed width
  uint32_t fixed_bits;
  uint32_t fixed_words_full;
};

// Raw section of tensor-aware messages: the small tensors in pieces of kRawPiece values.
constexpr uint32_t kRawPiece = 1024;
struct RawArgs {
  const uint4* rtab;         // per piece: (start / 4, length, offset in the raw section, 0)
  uint32_t R;
  uint64_t raw_words;        // all raw values of a message
  uint64_t fixed_strings;    // fixed width: words of all bucket strings; else 0 (read the table)
  // encode
  const float* g;
  uint32_t* header;
  const uint32_t* table;
  uint32_t* payload;
  uint64_t cap_words;
  uint32_t nb;
};

constexpr uint32_t kSeg = 2048;  // values per segment on the general path
// Elias-coded buckets above kEntryMinD values: the string is followed by a list of places
// where a reader may start (at most one per kEntryBits bits, on segment boundaries).
constexpr uint32_t kEntryMinD = 8192;
constexpr uint32_t kEntryBits = 1024;

struct GenArgs {
  const float* g;
  uint64_t index_base;  // draw index of g[0] (a slice of a longer vector), multiple of 4
  uint64_t n, d, nb;
  uint64_t spb;        // segments per bucket
  uint64_t nseg;       // nb * spb
  uint32_t s, code, norm_mode;
  uint32_t key0, key1, stream_id, iteration;
  uint32_t sub_words;  // words of one segment's sub-stream slot (even)
  uint32_t* header;
  uint32_t* table;
  uint32_t* payload;
  uint64_t cap_words;
  uint64_t table_words;
  // workspace
  double* partial;     // nseg: sum of squares (or max) of each segment
  float* scale;        // nb
  uint32_t* seginfo;   // 3 * nseg: first position, last position, bits
  uint64_t* segstart;  // nseg: bit offset of the segment's gap code in its bucket string
  uint32_t* seggap;    // nseg: gap in front of the segment's first record (0: none)
  uint32_t* segrank;   // nseg: index of the segment in its bucket's entry list, or ~0
  uint32_t* segprev;   // nseg: position of the last coded coordinate before the segment
  uint32_t* bents;     // nb: entries listed by the bucket
  uint32_t entries;    // 1: strings are followed by an entry list (d > kEntryMinD)
  uint32_t* slots;     // nseg * sub_words
  // fixed width
  uint32_t fixed_bits;
  uint64_t fixed_words_full;
  uint64_t fixed_payload_words;
};

// Host-side checks of an encode / a decode call that only depend on the parameters and the
// buffer sizes (what the entry points test before they queue anything): 0 or a QSGD_ERR_*.
int validate_encode(const qsgd_params* p, uint64_t index_base, size_t msg_capacity,
                    size_t workspace_bytes);
int validate_decode(const qsgd_params* p, uint32_t K, size_t workspace_bytes);

hipError_t launch_encode_bucket(const EncodeArgs& a, uint32_t code, int tw, int cpw,
                                uint32_t teams, size_t lds, hipStream_t st);
hipError_t launch_encode_compact(const CompactArgs& a, uint32_t teams, hipStream_t st);
hipError_t launch_encode_fixed_small(const EncodeArgs& a, int lpb, int cp, uint32_t teams,
                                     hipStream_t st);
hipError_t launch_write_empty(uint32_t* header, uint32_t* table, uint32_t code, uint32_t norm,
                              uint32_t s, uint64_t d, uint32_t stream_id, uint32_t iteration,
                              hipStream_t st);

hipError_t launch_decode_check(const DecodeArgs& a, hipStream_t st);
hipError_t launch_decode_fixed(const DecodeArgs& a, uint32_t blocks, hipStream_t st);
hipError_t launch_decode_elias(const DecodeArgs& a, uint32_t blocks, size_t lds, hipStream_t st);
hipError_t launch_decode_tile(const DecodeArgs& a, uint32_t blocks, size_t lds, hipStream_t st);
#ifndef QSGD_TILE_WIN
#define QSGD_TILE_WIN 128
#endif

hipError_t launch_write_layout_header(uint32_t* header, uint32_t* table, uint32_t code,
                                      uint32_t norm, uint32_t s, uint64_t d, uint64_t n,
                                      uint64_t raw_words, uint32_t stream_id, uint32_t iteration,
                                      hipStream_t st);
hipError_t launch_raw_pack(const RawArgs& a, hipStream_t st);
hipError_t launch_raw_apply(const DecodeArgs& a, const RawArgs& r, hipStream_t st);
hipError_t launch_gen_partial(const GenArgs& a, hipStream_t st);
hipError_t launch_gen_scale(const GenArgs& a, hipStream_t st);
hipError_t launch_gen_encode(const GenArgs& a, bool aligned, hipStream_t st);
hipError_t launch_gen_scan(const GenArgs& a, hipStream_t st);
hipError_t launch_gen_fill(const GenArgs& a, uint32_t blocks, hipStream_t st);
hipError_t launch_gen_place(const GenArgs& a, hipStream_t st);
hipError_t launch_gen_zero(float* p, uint64_t n, uint32_t blocks, hipStream_t st);
hipError_t launch_gen_parse(const DecodeArgs& a, float* acc, bool entries, hipStream_t st);
// Long buckets read with all messages at once: records at coordinates that several
// messages hit go to a list per bucket (a count, then kCollide x (position, value, message)).
constexpr uint32_t kCollide = 1024;
constexpr uint32_t kCollideBytes = 256 + 12 * kCollide;
hipError_t launch_gen_parse_together(const DecodeArgs& a, float* acc, uint8_t* lists,
                                     hipStream_t st);
hipError_t launch_gen_apply(const DecodeArgs& a, const float* acc, uint32_t blocks, hipStream_t st);
hipError_t launch_gen_decode_fixed(const DecodeArgs& a, uint32_t blocks, hipStream_t st);

}  // namespace qsgd
