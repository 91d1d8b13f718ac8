// Wavefront-level encoders: one wavefront turns up to CPW chunks of 256 values
// (held in registers, 4 per lane) into a bit "sub-stream" in LDS.
//
// Code_s (Sec. 3.1, App. A.2) only has records for nonzero levels, and in its
// intended regime almost every level is zero.  So the work is split in two:
//   stage 1, every element: one Philox block per float4, t = |v| * fl(s/scale),
//            and the test "level != 0", which is exactly u < t (for t >= 1 it
//            holds since u < 1; for t < 1 the round-up probability is t itself).
//            Survivors are compacted, in position order, into a small LDS ring.
//   stage 2, survivors only, one per lane: level from Eq. (2), Elias(gap), sign,
//            Elias(level), a wavefront prefix sum of the code lengths and the OR
//            of the code words into the sub-stream.
// The gap of a wavefront's first record depends on the wavefronts before it and
// is left out; whoever joins the sub-streams adds it.
#pragma once

#include "qsgd_device.hpp"

#ifndef QSGD_PHILOX_TOGETHER
#define QSGD_PHILOX_TOGETHER 8
#endif

namespace qsgd {

// Records in a wavefront's ring (a power of two): 256 holds the survivors of a whole chunk
// whatever the data.  On sparse data (see encode_sparse_list) the same words are a plain
// list of list_records(CPW) records that takes the survivors of all of a wavefront's chunks.
constexpr uint32_t kRing = 256;
__host__ __device__ constexpr uint32_t list_records(int cpw) { return cpw >= 8 ? 256u : 128u; }
// Elias code words of 1 .. kOmegaTab - 1 as (code << 8) | length, entry 0 = 0 (at most 14 bits).
constexpr uint32_t kOmegaTab = 256;
__host__ __device__ constexpr uint32_t ring_words(uint32_t ring) { return 3u * ring; }
constexpr uint32_t kRingWords = ring_words(kRing);

struct QuantCtx {
  float inv;   // fl(s / scale), 0 for an all-zero bucket
  float s_f;
  uint32_t s;
  uint32_t key0, key1, stream_id, iteration;
};

struct WaveOut {
  uint32_t first_pos;  // 1-based bucket position of the first record (0: none)
  uint32_t last_pos;   // 1-based bucket position of the last record
  uint32_t bits;       // bits in the sub-stream
};

// Number of set bits of `mask` below this lane.
__device__ __forceinline__ uint32_t bits_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The four draw words of the elements gidx .. gidx+3.  ALIGNED: gidx is a multiple
// of 4 and they are one Philox block; otherwise they straddle two blocks.
template <bool ALIGNED>
__device__ __forceinline__ void draw4(uint64_t gidx, const QuantCtx& q, uint32_t r[4]) {
  const uint64_t quad = gidx >> 2;
  philox4x32_10((uint32_t)quad, (uint32_t)(quad >> 32), q.stream_id, q.iteration, q.key0, q.key1,
                r);
  if constexpr (!ALIGNED) {
    const uint32_t sh = (uint32_t)(gidx & 3u);
    if (sh) {
      uint32_t r2[4];
      const uint64_t q2 = quad + 1;
      philox4x32_10((uint32_t)q2, (uint32_t)(q2 >> 32), q.stream_id, q.iteration, q.key0,
                    q.key1, r2);
      const uint32_t all[8] = {r[0], r[1], r[2], r[3], r2[0], r2[1], r2[2], r2[3]};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t v = all[j + 1];
        if (sh == 2) v = all[j + 2];
        if (sh == 3) v = all[j + 3];
        r[j] = v;
      }
    }
  }
}

// True when every Philox block of the elements gidx_first .. gidx_last (each lane passes
// its own lowest and highest index) has the same high counter word in all lanes: always,
// unless the wavefront straddles a multiple of 2^34 elements.  `hi` receives that word.
__device__ __forceinline__ bool uniform_counter_hi(uint64_t gidx_first, uint64_t gidx_last,
                                                   uint32_t& hi) {
  hi = __builtin_amdgcn_readfirstlane((uint32_t)(gidx_first >> 34));
  return __builtin_amdgcn_ballot_w64((uint32_t)(gidx_first >> 34) != hi ||
                                     (uint32_t)(gidx_last >> 34) != hi) == 0;
}

// draw4 of an aligned block whose high counter word `hi` is the same in every lane.
__device__ __forceinline__ void draw4_uniform_hi(uint64_t gidx, uint32_t hi, const QuantCtx& q,
                                                 uint32_t r[4]) {
  philox4x32_10_uniform((uint32_t)(gidx >> 2), hi, q.stream_id, q.iteration, q.key0, q.key1, r);
}

// Draw words of every chunk a wavefront holds.  They do not depend on the data, so
// callers compute them while the loads of the values are still in flight.
template <int CPW, bool ALIGNED>
__device__ __forceinline__ void draw_all(uint64_t gidx0, int lane, const QuantCtx& q,
                                         uint32_t (&r)[CPW][4]) {
  // blocks drawn side by side, the largest of 8, 4, 2 that divides CPW: the round keys are
  // stepped once for all of them (the compiler still sinks each block's rounds into the
  // chunk that uses it; pinning them together, for more independent multiplies in flight,
  // measured 2% slower: the vector unit, not the chain, is what the draws wait for)
  constexpr int kWish = QSGD_PHILOX_TOGETHER;
  constexpr int kTogether = CPW % kWish == 0 ? kWish : (CPW % 4 == 0 && kWish > 4 ? 4 : (CPW % 2 == 0 && kWish > 1 ? 2 : 1));
  if constexpr (ALIGNED && kTogether > 1) {
#pragma unroll
    for (int c = 0; c < CPW; c += kTogether) {
      uint32_t lo[kTogether], hi[kTogether];
#pragma unroll
      for (int i = 0; i < kTogether; ++i) {
        const uint64_t quad = (gidx0 + (uint64_t)(c + i) * kChunk + (uint64_t)lane * 4u) >> 2;
        lo[i] = (uint32_t)quad; hi[i] = (uint32_t)(quad >> 32);
      }
      philox4x32_10_xn<kTogether>(lo, hi, q.stream_id, q.iteration, q.key0, q.key1, &r[c]);
    }
  } else {
#pragma unroll
    for (int c = 0; c < CPW; ++c)
      draw4<ALIGNED>(gidx0 + (uint64_t)c * kChunk + (uint64_t)lane * 4u, q, r[c]);
  }
}

// Codes up to 64 records, one per lane (`live`: this lane has one), and appends them to the
// sub-stream at bit `bits`; returns the bits after them.
//   gap   position minus the position of the record before (0: the sub-stream's first record,
//         whose gap whoever joins the sub-streams adds)
//   tsb   bits of t with the sign of the value,  word  the draw word
//   otab  Elias code words of 1 .. kOmegaTab - 1 as (code << 8) | length in LDS, or null
// When every gap and level of the batch is in the table a record's whole code fits 32 bits
// (at most 14 + 1 + 14); otherwise the code words are computed (64-bit arithmetic).
// WIDE: gaps may need more than 21 bits, emit gap and (sign, level) separately.
template <bool WIDE>
__device__ __forceinline__ uint32_t code_batch(bool live, uint32_t gap, uint32_t tsb,
                                               uint32_t word, int lane, const QuantCtx& q,
                                               const uint32_t* otab, uint32_t* sub,
                                               uint32_t bits) {
  const uint32_t z = live ? min(quantize_scaled(__uint_as_float(tsb), word), q.s) : 0u;
  gap = live ? gap : 0u;
  if (!WIDE && otab != nullptr && __ballot(max(z, gap) >= kOmegaTab) == 0) {
    const uint32_t ez = otab[z], eg = otab[gap];
    const uint32_t ll = ez & 0xFFu, gl = eg & 0xFFu;
    const uint32_t cl = live ? ll + 1u : 0u;
    const uint32_t cw = ((tsb >> 31) << ll) | (ez >> 8);
    const uint32_t code = ((eg >> 8) << cl) | cw;
    const uint32_t len = gl + cl;
    const uint32_t incl = wave_incl_scan_u32(len, lane);
    const uint32_t off = bits + incl - len;
    if (live) {
      const uint32_t top = code << (32u - len);
      const uint32_t w = off >> 5, sh = off & 31u;
      atomicOr(&sub[w], top >> sh);
      if (sh + len > 32u) atomicOr(&sub[w + 1], top << (32u - sh));
    }
    return bits + lane_bcast(incl, 63);
  }
  uint64_t gc = 0, cw = 0;
  uint32_t gl = 0, cl = 0;
  if (live) {
    uint64_t lc; uint32_t ll;
    omega_encode(z, lc, ll);
    cw = ((uint64_t)(tsb >> 31) << ll) | lc;
    cl = ll + 1u;
    if (gap) omega_encode(gap, gc, gl);
  }
  const uint32_t len = gl + cl;
  const uint32_t incl = wave_incl_scan_u32(len, lane);
  const uint32_t off = bits + incl - len;
  if (live) {
    if (WIDE) {
      if (gl) lds_emit(sub, off, gc, gl);
      lds_emit(sub, off + gl, cw, cl);
    } else {
      lds_emit(sub, off, (gc << cl) | cw, len);
    }
  }
  return bits + lane_bcast(incl, 63);
}

// Stage 2 on `take` (1..64) records starting at ring slot `head`.
template <bool WIDE, uint32_t RING = kRing>
__device__ __forceinline__ void sparse_flush(const uint32_t* ring, uint32_t head, uint32_t take,
                                             int lane, const QuantCtx& q, const uint32_t* otab,
                                             uint32_t* sub, WaveOut& out) {
  const uint32_t idx = (head + (uint32_t)lane) & (RING - 1);
  const bool live = (uint32_t)lane < take;
  uint32_t pos = 0, gap = 0, tsb = 0, word = 0;
  if (live) {
    pos = ring[idx];
    tsb = ring[RING + idx];
    word = ring[2 * RING + idx];
    const uint32_t prev = lane == 0 ? out.last_pos : ring[(idx - 1u) & (RING - 1)];
    gap = prev ? pos - prev : 0u;
  }
  out.bits = code_batch<WIDE>(live, gap, tsb, word, lane, q, otab, sub, out.bits);
  if (out.first_pos == 0) out.first_pos = lane_bcast(pos, 0);
  out.last_pos = lane_bcast(pos, (int)take - 1);
}

// Code_s sub-stream of the wavefront's values.
//   v[c]      lane's float4 of chunk c (zeros past the end of the data)
//   nchunks   chunks that hold data (<= CPW)
//   pos0      bucket position (0-based) of the wavefront's first value
//   rall      draw words of every chunk (draw_all)
//   ring      kRingWords words of LDS private to this wavefront
//   otab      table of Elias code words in LDS (code_batch), or null
//   sub       zero-initialised LDS words private to this wavefront
// Returns true when it gave up (RING < 256 only): the sub-stream and `out` then hold
// leftovers and the caller starts over with encode_sparse_direct.
template <int CPW, bool WIDE, uint32_t RING = kRing>
__device__ __forceinline__ bool encode_sparse_wave(const float4 (&v)[CPW],
                                                   const uint32_t (&rall)[CPW][4], int nchunks,
                                                   uint32_t pos0, int lane,
                                                   const QuantCtx& q, uint32_t* ring,
                                                   const uint32_t* otab, uint32_t* sub,
                                                   WaveOut& out) {
  uint32_t head = 0, count = 0;
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    if (c >= nchunks) break;
    const uint32_t (&r)[4] = rall[c];
    const float ts[4] = {v[c].x * q.inv, v[c].y * q.inv, v[c].z * q.inv, v[c].w * q.inv};
    bool nz[4];
    uint64_t mk[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float u = (float)(r[j] >> 8) * (1.0f / 16777216.0f);
      nz[j] = u < fabsf(ts[j]);
      mk[j] = __ballot(nz[j]);
    }
    const uint32_t cnt = (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) +
                                    __popcll(mk[3]));
    if (cnt == 0) continue;
    if constexpr (RING >= 256) {
      while (count + cnt > RING) {  // make room (only in very dense data)
        const uint32_t take = min(64u, count);
        sparse_flush<WIDE, RING>(ring, head, take, lane, q, otab, sub, out);
        head += take;
        count -= take;
      }
    } else {
      // the ring holds at most 63 records here
      if (cnt > RING - 63u) return true;
    }
    uint32_t slot = head + count + bits_below(mk[0]) + bits_below(mk[1]) + bits_below(mk[2]) +
                    bits_below(mk[3]);
    const uint32_t p1 = pos0 + (uint32_t)c * kChunk + (uint32_t)lane * 4u + 1u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (nz[j]) {
        const uint32_t i = slot & (RING - 1);
        ring[i] = p1 + j;
        ring[RING + i] = __float_as_uint(ts[j]);
        ring[2 * RING + i] = r[j];
        ++slot;
      }
    }
    count += cnt;
    __builtin_amdgcn_wave_barrier();
    while (count >= 64u) {
      sparse_flush<WIDE, RING>(ring, head, 64u, lane, q, otab, sub, out);
      head += 64u;
      count -= 64u;
    }
  }
  __builtin_amdgcn_wave_barrier();
  while (count > 0) {
    const uint32_t take = min(64u, count);
    sparse_flush<WIDE, RING>(ring, head, take, lane, q, otab, sub, out);
    head += take;
    count -= take;
  }
  return false;
}

// Code_s sub-stream of the wavefront's values on sparse data: stage 1 runs over all
// chunks first and lists the survivors (position, t with its sign, draw word) in LDS, then
// one loop codes the list 64 records at a time.  Compared with encode_sparse_wave there is
// one copy of stage 2 in the kernel instead of one per chunk, no wrap-around in the
// indices, and the Elias code words of gaps and levels below kOmegaTab come from a table
// in LDS (`otab`), which keeps a record's whole code inside 32 bits.
//   list   3 * LIST words of LDS private to this wavefront
// Returns true when the list would overflow: nothing has been written to `sub` or `out`
// then, and the caller starts over with encode_sparse_direct.
template <int CPW, uint32_t LIST>
__device__ __forceinline__ bool encode_sparse_list(const float4 (&v)[CPW],
                                                   const uint32_t (&rall)[CPW][4], int nchunks,
                                                   uint32_t pos0, int lane, const QuantCtx& q,
                                                   uint32_t* list, const uint32_t* otab,
                                                   uint32_t* sub, WaveOut& out) {
  // (chunks past the end of the data hold zeros, which never survive: no test of nchunks;
  // and a list that would overflow is not written to any more while the count goes on, so
  // that the loop has one way out)
  uint32_t count = 0;
  const uint32_t p1 = pos0 + (uint32_t)lane * 4u + 1u;
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    const uint32_t (&r)[4] = rall[c];
    const float ts[4] = {v[c].x * q.inv, v[c].y * q.inv, v[c].z * q.inv, v[c].w * q.inv};
    bool nz[4];
    uint64_t mk[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float u = (float)(r[j] >> 8) * (1.0f / 16777216.0f);
      nz[j] = u < fabsf(ts[j]);
      mk[j] = __ballot(nz[j]);
    }
    const uint64_t m01 = mk[0] | mk[1], m23 = mk[2] | mk[3], any = m01 | m23;
    if (((mk[0] & mk[1]) | (mk[2] & mk[3]) | (m01 & m23)) == 0) {
      // the usual case on sparse data, no lane with two survivors: the survivors are the
      // lanes of `any`, the lanes below count once each, and one slot serves whichever of
      // the lane's values survived
      const uint32_t cnt = (uint32_t)__popcll(any);
      if (cnt != 0 && count + cnt <= LIST) {   // (else nothing to list, or no room)
        uint32_t* const at = list + count + bits_below(any);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (nz[j]) {
            at[0] = p1 + (uint32_t)(c * kChunk + j);
            at[LIST] = __float_as_uint(ts[j]);
            at[2 * LIST] = r[j];
          }
        }
      }
      count += cnt;
    } else {
      const uint32_t cnt = (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) +
                                      __popcll(mk[3]));
      if (count + cnt <= LIST) {
        uint32_t* at = list + count + bits_below(mk[0]) + bits_below(mk[1]) +
                       bits_below(mk[2]) + bits_below(mk[3]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (nz[j]) {
            at[0] = p1 + (uint32_t)(c * kChunk + j);
            at[LIST] = __float_as_uint(ts[j]);
            at[2 * LIST] = r[j];
            ++at;
          }
        }
      }
      count += cnt;
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (count == 0) return false;
  if (count > LIST) return true;
  uint32_t bits = 0;
  for (uint32_t head = 0; head < count; head += kWave) {
    const uint32_t i = head + (uint32_t)lane;
    const bool live = i < count;
    uint32_t gap = 0, tsb = 0, word = 0;
    if (live) {
      const uint32_t pos = list[i];
      tsb = list[LIST + i];
      word = list[2 * LIST + i];
      gap = i ? pos - list[i - 1u] : 0u;
    }
    bits = code_batch<false>(live, gap, tsb, word, lane, q, otab, sub, bits);
  }
  out.bits = bits;
  out.first_pos = __builtin_amdgcn_readfirstlane(list[0]);
  out.last_pos = __builtin_amdgcn_readfirstlane(list[count - 1u]);
  return false;
}

// Inclusive prefix maximum over the 64 lanes.
__device__ __forceinline__ uint32_t wave_incl_max_u32(uint32_t v) {
  v = max(v, dpp_fetch<kDppShr1, 0xf>(v));
  v = max(v, dpp_fetch<kDppShr2, 0xf>(v));
  v = max(v, dpp_fetch<kDppShr4, 0xf>(v));
  v = max(v, dpp_fetch<kDppShr8, 0xf>(v));
  v = max(v, dpp_fetch<kDppBcast15, 0xa>(v));
  v = max(v, dpp_fetch<kDppBcast31, 0xc>(v));
  return v;
}

// Code_s of one chunk without the ring, for dense data: every lane codes its own four
// values (Eq. 2, then gap, sign, level); the position of the nonzero level before a lane's
// first one comes from a prefix maximum over the lanes.  Appends to `sub` and `out` like
// encode_sparse_wave.  p1: 1-based bucket position of the lane's first value.
template <bool WIDE>
__device__ __forceinline__ void encode_sparse_direct(const float4& v, const uint32_t (&r)[4],
                                                     uint32_t p1, int lane, const QuantCtx& q,
                                                     uint32_t* sub, WaveOut& out) {
  const float vv[4] = {v.x, v.y, v.z, v.w};
  uint32_t z[4], lastnz = 0, firstnz = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    z[j] = quantize_one(vv[j], q.inv, q.s_f, q.s, r[j]);
    if (z[j]) {
      lastnz = p1 + j;
      if (!firstnz) firstnz = p1 + j;
    }
  }
  const uint32_t incl_max = wave_incl_max_u32(lastnz);
  uint32_t prev = (uint32_t)__shfl_up((int)incl_max, 1);
  if (lane == 0) prev = 0;
  prev = max(prev, out.last_pos);   // 0: no record in this sub-stream yet
  uint64_t gc[4], cw[4];
  uint32_t gl[4], cl[4], tot = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    gc[j] = 0; cw[j] = 0; gl[j] = 0; cl[j] = 0;
    if (z[j]) {
      const uint32_t pos = p1 + j;
      if (prev != 0) omega_encode(pos - prev, gc[j], gl[j]);
      uint64_t lc; uint32_t ll;
      omega_encode(z[j], lc, ll);
      cw[j] = ((uint64_t)(vv[j] < 0.f ? 1u : 0u) << ll) | lc;
      cl[j] = ll + 1u;
      prev = pos;
      tot += gl[j] + cl[j];
    }
  }
  const uint32_t incl = wave_incl_scan_u32(tot, lane);
  uint32_t off = out.bits + incl - tot;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (cl[j]) {
      if (WIDE) {
        if (gl[j]) lds_emit(sub, off, gc[j], gl[j]);
        lds_emit(sub, off + gl[j], cw[j], cl[j]);
      } else {
        lds_emit(sub, off, (gc[j] << cl[j]) | cw[j], gl[j] + cl[j]);
      }
      off += gl[j] + cl[j];
    }
  }
  out.bits += lane_bcast(incl, 63);
  const uint64_t any = __ballot(firstnz != 0);
  if (any) {
    if (out.first_pos == 0) out.first_pos = lane_bcast(firstnz, __ffsll((unsigned long long)any) - 1);
    out.last_pos = lane_bcast(incl_max, 63);
  }
}

// Code'_s sub-stream (App. A.3): every coordinate sends its sign and Elias(level+1).
//   len_valid  values that exist in the wavefront's range (the rest is padding)
template <int CPW>
__device__ __forceinline__ void encode_dense_wave(const float4 (&v)[CPW],
                                                  const uint32_t (&rall)[CPW][4], int nchunks,
                                                  uint32_t len_valid, int lane,
                                                  const QuantCtx& q, uint32_t* sub,
                                                  WaveOut& out) {
#pragma unroll
  for (int c = 0; c < CPW; ++c) {
    if (c >= nchunks) break;
    const uint32_t (&r)[4] = rall[c];
    const float vv[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
    const uint32_t e0 = (uint32_t)c * kChunk + (uint32_t)lane * 4u;
    uint64_t code[4];
    uint32_t len[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (e0 + j < len_valid) {
        const uint32_t z = quantize_one(vv[j], q.inv, q.s_f, q.s, r[j]);
        uint64_t lc; uint32_t ll;
        omega_encode(z + 1u, lc, ll);
        code[j] = ((uint64_t)(vv[j] < 0.f ? 1u : 0u) << ll) | lc;
        len[j] = ll + 1u;
      }
    }
    const uint32_t tot = len[0] + len[1] + len[2] + len[3];
    const uint32_t incl = wave_incl_scan_u32(tot, lane);
    uint32_t off = out.bits + incl - tot;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (len[j]) {
        lds_emit(sub, off, code[j], len[j]);
        off += len[j];
      }
    }
    out.bits += lane_bcast(incl, 63);
  }
}

}  // namespace qsgd
