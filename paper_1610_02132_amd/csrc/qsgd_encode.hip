// Encode kernels: M <- Code(Q_s(g))  (Alg. 1; Q_s: Sec. 3.1 Eq. 2 per bucket of
// Sec. 4; Code_s / Code'_s: Sec. 3.1 and App. A.2-A.3; fixed-width: Sec. 5).
//
// Bucket path (d <= 8192, d % 4 == 0).  A team of TW wavefronts (= one
// workgroup) owns a contiguous run of buckets.  Per bucket: one coalesced
// float4 read of the data into registers, the scale by a wavefront shuffle
// reduction (fp64 accumulation), one Philox block per float4, stochastic
// rounding, code lengths, a wavefront prefix sum for bit offsets, and the code
// words OR-ed into an LDS image of the bucket's string.  Strings have
// data-dependent lengths, so a team appends them to its own region of the
// workspace and a second, small kernel moves the regions to their final place
// (exclusive sum over at most a few thousand team totals): no team ever waits
// for another one.  Fixed-width strings have closed-form offsets and go straight
// to the message.
#include "qsgd_device.hpp"
#include "qsgd_encode_wave.hpp"
#include "qsgd_kernels.hpp"

#ifndef QSGD_UHI
#define QSGD_UHI 1
#endif
namespace qsgd {

namespace {

// Loads the float4 of this lane for the chunk starting `eoff` elements into the
// bucket; elements at or past m read as 0.
__device__ __forceinline__ float4 load_quad(const float* __restrict__ gb, uint32_t eoff,
                                            uint32_t m) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (eoff + 3 < m) {
    v = load_stream(gb + eoff);  // read once: the team's staged strings stay cached
  } else {
    if (eoff + 0 < m) v.x = gb[eoff + 0];
    if (eoff + 1 < m) v.y = gb[eoff + 1];
    if (eoff + 2 < m) v.z = gb[eoff + 2];
  }
  return v;
}

}  // namespace

// TW wavefronts per bucket, each holding up to CPW chunks of 256 elements.
// LIST (Code_s only): 0 = survivors go through a ring that is coded as it fills
// (encode_sparse_wave); list_records(CPW) = sparse data, survivors of all chunks are listed first
// (encode_sparse_list).
template <int TW, int CPW, int CODE, uint32_t LIST = 0>
__global__ __launch_bounds__(64 * TW)
    __attribute__((amdgpu_waves_per_eu(CODE == 2 ? 1 : (LIST ? QSGD_ENC_WAVES_LIST : QSGD_ENC_WAVES))))
    void k_encode_bucket(EncodeArgs a) {
  extern __shared__ uint32_t smem[];
  // LDS: [dst image of the bucket string][TW sub-streams][TW record rings][scratch]
  constexpr uint32_t kRingW = (CODE == QSGD_CODE_SPARSE) ? ring_words(LIST ? LIST : kRing) : 0u;
  uint32_t* const dst = smem;
  uint32_t* const sub_all = smem + a.dst_words;
  uint32_t* const ring_all = sub_all + TW * a.sub_words;
  double* const red = reinterpret_cast<double*>(ring_all + TW * kRingW);
  WaveOut* const winfo = reinterpret_cast<WaveOut*>(red + TW);
  uint32_t* const otab = reinterpret_cast<uint32_t*>(winfo + TW);  // kOmegaTab words (Code_s)

  const int tid = threadIdx.x;
  // (the wavefront's number is the same in all its lanes: as a scalar, what depends on it --
  // chunk bounds, LDS bases, the loop over chunks -- stays off the vector unit)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  uint32_t* const sub = sub_all + wave * a.sub_words;
  uint32_t* const ring = ring_all + wave * kRingW;

  for (uint32_t j = tid; j < a.dst_words + TW * a.sub_words; j += 64 * TW) smem[j] = 0;
  if (CODE == QSGD_CODE_SPARSE) {
    for (uint32_t k = tid; k < kOmegaTab; k += 64 * TW) {
      uint64_t code = 0; uint32_t len = 0;
      if (k) omega_encode(k, code, len);
      otab[k] = ((uint32_t)code << 8) | len;
    }
  }

  if (blockIdx.x == 0 && tid == 0) {  // header; length and status are completed later
    uint32_t* h = a.header;
    h[H_MAGIC] = kMagic; h[H_VERSION] = a.version; h[H_CODE] = CODE; h[H_NORM] = a.norm_mode;
    h[H_S] = a.s; h[H_STREAM] = a.stream_id;
    h[H_D_LO] = (uint32_t)a.d; h[H_D_HI] = 0;
    h[H_N_LO] = (uint32_t)a.n; h[H_N_HI] = (uint32_t)(a.n >> 32);
    h[H_NB_LO] = a.nb; h[H_NB_HI] = 0;
    h[H_PW_LO] = (uint32_t)a.fixed_payload_words;
    h[H_PW_HI] = (uint32_t)(a.fixed_payload_words >> 32);
    h[H_STATUS] = 0; h[H_ITER] = a.iteration;
  }
  __syncthreads();

  const uint32_t b_begin = blockIdx.x * a.bper;
  const uint32_t b_end = min(b_begin + a.bper, a.nb);
  uint32_t* const region = a.staging + (uint64_t)blockIdx.x * a.region_words;
  uint32_t run = 0;  // words this team has appended to its region

  const uint32_t s = a.s;
  const float s_f = (float)s;

  // Extent of bucket b, as scalars: the same in every lane, and saying so keeps the bounds
  // and the addresses on the scalar unit.
  auto extent = [&](uint32_t b, uint64_t& base, uint32_t& m) {
    bucket_extent(a, b, base, m);
    base = ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(base >> 32)) << 32) |
           __builtin_amdgcn_readfirstlane((uint32_t)base);
    m = __builtin_amdgcn_readfirstlane(m);
  };
  constexpr uint32_t kFull = (uint32_t)(TW * CPW) * kChunk;

  for (uint32_t b = b_begin; b < b_end; ++b) {
    uint64_t base;
    uint32_t m;
    extent(b, base, m);
    const float* __restrict__ gb = a.g + base;

    // ---- read the bucket once, accumulate the scale --------------------------
    float4 v[CPW];
    float mx = 0.f;
    if (m == kFull) {  // a full bucket: no bounds to check
#pragma unroll
      for (int c = 0; c < CPW; ++c)
        v[c] = load_stream(gb + (uint32_t)(wave * CPW + c) * kChunk + lane * 4);
    } else {
#pragma unroll
      for (int c = 0; c < CPW; ++c) {
        const uint32_t cstart = (uint32_t)(wave * CPW + c) * kChunk;
        v[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (cstart < m) v[c] = load_quad(gb, cstart + lane * 4, m);
      }
    }
    // the draws need no data: they are computed while the loads are in flight
    const uint32_t wstart = (uint32_t)wave * CPW * kChunk;  // bucket position of this wave
    QuantCtx qc;
    qc.inv = 0.f; qc.s_f = s_f; qc.s = s; qc.key0 = a.key0; qc.key1 = a.key1;
    qc.stream_id = a.stream_id; qc.iteration = a.iteration;
    uint32_t rall[CPW][4];
    draw_all<CPW, true>(a.index_base + base + wstart, lane, qc, rall);
    // squares are exact in fp64, so the fused multiply-add rounds like multiply, add
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
      if (a.norm_mode == 0) {
        s0 = fma((double)v[c].x, (double)v[c].x, s0);
        s1 = fma((double)v[c].y, (double)v[c].y, s1);
        s2 = fma((double)v[c].z, (double)v[c].z, s2);
        s3 = fma((double)v[c].w, (double)v[c].w, s3);
      } else {
        mx = fmaxf(fmaxf(mx, fmaxf(fabsf(v[c].x), fabsf(v[c].y))),
                   fmaxf(fabsf(v[c].z), fabsf(v[c].w)));
      }
    }
    double ss = (s0 + s1) + (s2 + s3);
    float scale;
    if (a.norm_mode == 0) {
      ss = wave_sum_f64(ss);
      if (TW > 1) {
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        ss = 0.0;
#pragma unroll
        for (int w = 0; w < TW; ++w) ss += red[w];
      }
      scale = (float)sqrt(ss);
    } else {
      mx = wave_max_f32(mx);
      if (TW > 1) {
        if (lane == 0) red[wave] = (double)mx;
        __syncthreads();
        mx = 0.f;
#pragma unroll
        for (int w = 0; w < TW; ++w) mx = fmaxf(mx, (float)red[w]);
      }
      scale = mx;
    }
    const float inv = (scale > 0.f) ? s_f / scale : 0.f;

    // ---- fixed width: closed-form placement, straight to the message ---------
    if (CODE == QSGD_CODE_FIXED) {
      const uint32_t B = a.fixed_bits;
      const uint32_t fmax = (1u << B) - 1u;
      uint32_t* const str = a.payload + (uint64_t)b * a.fixed_words_full;
      const uint32_t lw = (m * B + 31u) >> 5, sw = (m + 31u) >> 5;
      uint32_t* const lplane = str + 2;
      uint32_t* const splane = lplane + lw;
      uint32_t esc = 0xFFFFFFFFu;
#pragma unroll
      for (int c = 0; c < CPW; ++c) {
        const uint32_t cstart = (uint32_t)(wave * CPW + c) * kChunk;
        if (cstart >= m) continue;
        const uint32_t e0 = cstart + lane * 4;
        const uint32_t (&r)[4] = rall[c];
        uint32_t z[4];
        z[0] = quantize_one(v[c].x, inv, s_f, s, r[0]);
        z[1] = quantize_one(v[c].y, inv, s_f, s, r[1]);
        z[2] = quantize_one(v[c].z, inv, s_f, s, r[2]);
        z[3] = quantize_one(v[c].w, inv, s_f, s, r[3]);
        const uint32_t nib = (v[c].x < 0.f ? 1u : 0u) | (v[c].y < 0.f ? 2u : 0u) |
                             (v[c].z < 0.f ? 4u : 0u) | (v[c].w < 0.f ? 8u : 0u);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (z[j] > fmax) { esc = e0 + j; z[j] = fmax; }
        // level plane: element i's field at bit i*B (LSB first)
        if (B == 8) {
          const uint32_t w = z[0] | (z[1] << 8) | (z[2] << 16) | (z[3] << 24);
          const uint32_t wi = e0 >> 2;
          if (wi < lw) lplane[wi] = w;
        } else if (B == 16) {
          const uint32_t wi = e0 >> 1;
          if (wi < lw) lplane[wi] = z[0] | (z[1] << 16);
          if (wi + 1 < lw) lplane[wi + 1] = z[2] | (z[3] << 16);
        } else if (B == 4) {
          uint32_t h = z[0] | (z[1] << 4) | (z[2] << 8) | (z[3] << 12);
          h |= dpp_fetch<kDppShl1, 0xf>(h) << 16;
          const uint32_t wi = e0 >> 3;
          if ((lane & 1) == 0 && wi < lw) lplane[wi] = h;
        } else {  // B == 2
          uint32_t h = z[0] | (z[1] << 2) | (z[2] << 4) | (z[3] << 6);
          h |= dpp_fetch<kDppShl1, 0xf>(h) << 8;
          h |= dpp_fetch<kDppShl2, 0xf>(h) << 16;
          const uint32_t wi = e0 >> 4;
          if ((lane & 3) == 0 && wi < lw) lplane[wi] = h;
        }
        // sign plane: element i at bit i%32 of word i/32
        uint32_t sg = nib;
        sg |= dpp_fetch<kDppShl1, 0xf>(sg) << 4;
        sg |= dpp_fetch<kDppShl2, 0xf>(sg) << 8;
        sg |= dpp_fetch<kDppShl4, 0xf>(sg) << 16;
        const uint32_t si = e0 >> 5;
        if ((lane & 7) == 0 && si < sw) splane[si] = sg;
      }
      // a short bucket inside a tensor-aware message keeps a full-size slot: zero its tail
      if (a.btab && m < a.d) {
        for (uint32_t w = 2u + lw + sw + (uint32_t)tid; w < a.fixed_words_full; w += 64 * TW)
          str[w] = 0;
      }
      // escape word: at most one lane of the team holds an index
      const uint64_t eb = __ballot(esc != 0xFFFFFFFFu);
      if (TW == 1) {
        if (eb) esc = lane_bcast(esc, __ffsll((unsigned long long)eb) - 1);
        if (lane == 0) { str[0] = __float_as_uint(scale); str[1] = esc; }
      } else {
        if (tid == 0) winfo[0].first_pos = 0xFFFFFFFFu;
        __syncthreads();
        if (esc != 0xFFFFFFFFu) winfo[0].first_pos = esc;
        __syncthreads();
        if (tid == 0) { str[0] = __float_as_uint(scale); str[1] = winfo[0].first_pos; }
        __syncthreads();
      }
      continue;
    }

    // ---- Elias codes: each wave builds its sub-stream in LDS -----------------
    qc.inv = inv;
    WaveOut wo;
    wo.first_pos = 0; wo.last_pos = 0; wo.bits = 0;
    {
      const uint32_t wlen = wstart < m ? min((uint32_t)CPW * kChunk, m - wstart) : 0u;
      const int nchunks = (int)((wlen + kChunk - 1) / kChunk);
      if (CODE == QSGD_CODE_SPARSE) {
        bool gave_up = false;
        if constexpr (LIST != 0) {
          gave_up = encode_sparse_list<CPW, LIST>(v, rall, nchunks, wstart, lane, qc, ring, otab,
                                                  sub, wo);
        } else {
          (void)encode_sparse_wave<CPW, false>(v, rall, nchunks, wstart, lane, qc, ring, otab, sub,
                                               wo);
        }
        if (LIST && gave_up) {
          // dense data after all: clear what the sub-stream holds and code the wavefront's
          // values chunk by chunk straight from memory
          const uint32_t dirty = min(a.sub_words, ((wo.bits + 31u) >> 5) + 2u);
          for (uint32_t j = lane; j < dirty; j += kWave) sub[j] = 0;
          wo.first_pos = 0; wo.last_pos = 0; wo.bits = 0;
          __builtin_amdgcn_wave_barrier();
#pragma unroll 1
          for (int c = 0; c < nchunks; ++c) {
            const uint32_t e0 = wstart + (uint32_t)c * kChunk + (uint32_t)lane * 4u;
            const float4 vc = load_quad(gb, e0, m);
            uint32_t rc[4];
            draw4<true>(a.index_base + base + e0, qc, rc);
            encode_sparse_direct<false>(vc, rc, e0 + 1u, lane, qc, sub, wo);
          }
        }
      } else {
        encode_dense_wave<CPW>(v, rall, nchunks, wlen, lane, qc, sub, wo);
      }
    }
    const uint32_t wbits = wo.bits;

    // ---- join the sub-streams into the bucket string --------------------------
    if (lane == 0) winfo[wave] = wo;
    __syncthreads();
    uint32_t cursor = 32;  // after the scale
    uint32_t my_start = 0, my_glen = 0, my_gap = 0;
    {
      uint32_t prev_last = 0;
#pragma unroll
      for (int w = 0; w < TW; ++w) {
        WaveOut wi;
        wi.first_pos = __builtin_amdgcn_readfirstlane(winfo[w].first_pos);
        wi.last_pos = __builtin_amdgcn_readfirstlane(winfo[w].last_pos);
        wi.bits = __builtin_amdgcn_readfirstlane(winfo[w].bits);
        uint32_t glen = 0, gap = 0;
        if (CODE == QSGD_CODE_SPARSE && wi.first_pos) {
          gap = wi.first_pos - prev_last;
          glen = omega_length(gap);
          prev_last = wi.last_pos;
        }
        if (w == wave) { my_start = cursor; my_glen = glen; my_gap = gap; }
        cursor += glen + wi.bits;
      }
    }
    const uint32_t stop = (CODE == QSGD_CODE_SPARSE) ? 1u : 0u;
    const uint32_t words = (cursor + stop + 31u) >> 5;
    if (tid == 0) {
      dst[0] = __float_as_uint(scale);
      if (stop) lds_emit(dst, cursor, 1ull, 1u);
    }
    if (lane == 0 && my_glen) {
      uint64_t gc; uint32_t gl;
      omega_encode(my_gap, gc, gl);
      lds_emit(dst, my_start, gc, gl);
    }
    {
      const uint32_t o = my_start + my_glen;
      const uint32_t w0 = o >> 5, sh = o & 31u;
      const uint32_t nsub = (wbits + 31u) >> 5;
      for (uint32_t j = lane; j < nsub; j += kWave) {
        const uint32_t x = sub[j];
        sub[j] = 0;
        if (x) {
          atomicOr(&dst[w0 + j], x >> sh);
          if (sh) atomicOr(&dst[w0 + j + 1], x << (32u - sh));
        }
      }
    }
    __syncthreads();

    // ---- append the string to the team's region --------------------------------
    // (a region smaller than the worst case may run out: the string is then dropped, the
    // count goes on, and the message ends up with the capacity status and the size needed)
    if (tid == 0) a.table[b] = run;  // relative to the region; rebased later
    const bool room = (uint64_t)run + words <= a.region_words;
    for (uint32_t j = tid; j < words; j += 64 * TW) {
      if (room) region[run + j] = dst[j];
      dst[j] = 0;
    }
    run += words;
    // no barrier here: the image is next written after two barriers of the next bucket
    // (scale exchange, sub-stream summaries), which every thread reaches after its zeroing
  }
  if (CODE != QSGD_CODE_FIXED && tid == 0) a.totals[blockIdx.x] = run;
}

// Fixed width, buckets of at most 1024 values: LPB lanes per bucket (64 / LPB buckets
// per wavefront at once), CP float4 per lane, B-bit fields.  Offsets are closed
// form, so the wavefront reads its buckets once and writes their strings in place;
// the per-bucket work (scale reduction, square root, divide) is shared by the
// buckets that ride in one wavefront.
template <int LPB, int CP, int B>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(QSGD_FS_WAVES)))
void k_encode_fixed_small(EncodeArgs a) {
  constexpr int NB = 64 / LPB;             // buckets per wavefront pass
  constexpr uint32_t kStep = LPB * 4;      // values one pass of the bucket's lanes covers
  constexpr uint32_t fmax = (1u << B) - 1u;
  const int lane = threadIdx.x;
  const uint32_t sb = lane / LPB, l = lane % LPB;
  const int last_lane = (int)(sb * LPB + LPB - 1);

  if (blockIdx.x == 0 && lane == 0) {
    uint32_t* h = a.header;
    h[H_MAGIC] = kMagic; h[H_VERSION] = a.version; h[H_CODE] = QSGD_CODE_FIXED; h[H_NORM] = a.norm_mode;
    h[H_S] = a.s; h[H_STREAM] = a.stream_id;
    h[H_D_LO] = (uint32_t)a.d; h[H_D_HI] = 0;
    h[H_N_LO] = (uint32_t)a.n; h[H_N_HI] = (uint32_t)(a.n >> 32);
    h[H_NB_LO] = a.nb; h[H_NB_HI] = 0;
    h[H_PW_LO] = (uint32_t)a.fixed_payload_words;
    h[H_PW_HI] = (uint32_t)(a.fixed_payload_words >> 32);
    h[H_STATUS] = 0; h[H_ITER] = a.iteration;
  }
  const uint32_t s = a.s;
  const float s_f = (float)s;
  QuantCtx qc;
  qc.inv = 0.f; qc.s_f = s_f; qc.s = s; qc.key0 = a.key0; qc.key1 = a.key1;
  qc.stream_id = a.stream_id; qc.iteration = a.iteration;

  const uint32_t g_begin = blockIdx.x * a.bper;               // bucket groups of this team
  const uint32_t g_end = min(g_begin + a.bper, (a.nb + NB - 1) / NB);
  for (uint32_t grp = g_begin; grp < g_end; ++grp) {
    const uint32_t b = grp * NB + sb;
    const bool live = b < a.nb;
    uint64_t base = 0;
    uint32_t m = 0;
    if (live) bucket_extent(a, b, base, m);
    const float* __restrict__ gb = a.g + base;
    // every lane's CP quads lie inside its bucket: no per-element bounds needed
    const bool all_full = __ballot(m == (uint32_t)CP * kStep) == ~0ull;

    float4 v[CP];
    uint32_t r[CP][4];
#pragma unroll
    for (int c = 0; c < CP; ++c) {
      const uint32_t e0 = (uint32_t)c * kStep + l * 4;
      if (all_full) {
        v[c] = *reinterpret_cast<const float4*>(gb + e0);
      } else {
        v[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (e0 + 3 < m) {
          v[c] = *reinterpret_cast<const float4*>(gb + e0);
        } else {
          if (e0 + 0 < m) v[c].x = gb[e0 + 0];
          if (e0 + 1 < m) v[c].y = gb[e0 + 1];
          if (e0 + 2 < m) v[c].z = gb[e0 + 2];
        }
      }
    }
    {
      const uint64_t g0 = a.index_base + base + l * 4;
      uint32_t hi;
      if (QSGD_UHI && uniform_counter_hi(g0, g0 + (uint64_t)(CP - 1) * kStep, hi)) {
#pragma unroll
        for (int c = 0; c < CP; ++c) draw4_uniform_hi(g0 + (uint64_t)c * kStep, hi, qc, r[c]);
      } else {
#pragma unroll
        for (int c = 0; c < CP; ++c) draw4<true>(g0 + (uint64_t)c * kStep, qc, r[c]);
      }
    }

    // ---- scale of each bucket: reduction over its LPB lanes -------------------------
    float scale;
    if (a.norm_mode == 0) {
      double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
      for (int c = 0; c < CP; ++c) {
        s0 = fma((double)v[c].x, (double)v[c].x, s0);
        s1 = fma((double)v[c].y, (double)v[c].y, s1);
        s2 = fma((double)v[c].z, (double)v[c].z, s2);
        s3 = fma((double)v[c].w, (double)v[c].w, s3);
      }
      double ss = (s0 + s1) + (s2 + s3);
      ss += dpp_fetch_f64<kDppShr1, 0xf>(ss);
      ss += dpp_fetch_f64<kDppShr2, 0xf>(ss);
      ss += dpp_fetch_f64<kDppShr4, 0xf>(ss);
      ss += dpp_fetch_f64<kDppShr8, 0xf>(ss);
      if (LPB >= 32) ss += dpp_fetch_f64<kDppBcast15, 0xa>(ss);
      if (LPB >= 64) ss += dpp_fetch_f64<kDppBcast31, 0xc>(ss);
      scale = (float)sqrt(ss);  // right in the last lane of each bucket
    } else {
      float mx = 0.f;
#pragma unroll
      for (int c = 0; c < CP; ++c)
        mx = fmaxf(fmaxf(mx, fmaxf(fabsf(v[c].x), fabsf(v[c].y))),
                   fmaxf(fabsf(v[c].z), fabsf(v[c].w)));
      mx = fmaxf(mx, __uint_as_float(dpp_fetch<kDppShr1, 0xf>(__float_as_uint(mx))));
      mx = fmaxf(mx, __uint_as_float(dpp_fetch<kDppShr2, 0xf>(__float_as_uint(mx))));
      mx = fmaxf(mx, __uint_as_float(dpp_fetch<kDppShr4, 0xf>(__float_as_uint(mx))));
      mx = fmaxf(mx, __uint_as_float(dpp_fetch<kDppShr8, 0xf>(__float_as_uint(mx))));
      if (LPB >= 32) mx = fmaxf(mx, __uint_as_float(dpp_fetch<kDppBcast15, 0xa>(__float_as_uint(mx))));
      if (LPB >= 64) mx = fmaxf(mx, __uint_as_float(dpp_fetch<kDppBcast31, 0xc>(__float_as_uint(mx))));
      scale = mx;
    }
    scale = __shfl(scale, last_lane, kWave);
    const float inv = (scale > 0.f) ? s_f / scale : 0.f;

    // ---- quantize, pack, store ------------------------------------------------------------
    uint32_t* const str = a.payload + (uint64_t)b * a.fixed_words_full;
    const uint32_t lw = (m * B + 31u) >> 5, sw = (m + 31u) >> 5;
    uint32_t* const lplane = str + 2;
    uint32_t* const splane = lplane + lw;
    uint32_t esc = 0xFFFFFFFFu;
    const uint32_t zlim = min(fmax, s);
#pragma unroll
    for (int c = 0; c < CP; ++c) {
      const uint32_t e0 = (uint32_t)c * kStep + l * 4;
      uint32_t z[4];
      z[0] = quantize_unclamped(v[c].x, inv, r[c][0]);
      z[1] = quantize_unclamped(v[c].y, inv, r[c][1]);
      z[2] = quantize_unclamped(v[c].z, inv, r[c][2]);
      z[3] = quantize_unclamped(v[c].w, inv, r[c][3]);
      const uint32_t nib = (v[c].x < 0.f ? 1u : 0u) | (v[c].y < 0.f ? 2u : 0u) |
                           (v[c].z < 0.f ? 4u : 0u) | (v[c].w < 0.f ? 8u : 0u);
      // rare: a level above s (clamped to s here) or one the field cannot hold (level s
      // with s = 2^B, which goes to the escape word)
      if (max(max(z[0], z[1]), max(z[2], z[3])) > zlim) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          z[j] = min(z[j], s);
          if (z[j] > fmax) { esc = e0 + j; z[j] = fmax; }
        }
      }
      if (B == 8) {
        const uint32_t wi = e0 >> 2;
        if (all_full || wi < lw) lplane[wi] = z[0] | (z[1] << 8) | (z[2] << 16) | (z[3] << 24);
      } else if (B == 16) {
        const uint32_t wi = e0 >> 1;
        if (all_full || wi < lw) lplane[wi] = z[0] | (z[1] << 16);
        if (all_full || wi + 1 < lw) lplane[wi + 1] = z[2] | (z[3] << 16);
      } else if (B == 4) {
        uint32_t h = z[0] | (z[1] << 4) | (z[2] << 8) | (z[3] << 12);
        h |= dpp_fetch<kDppShl1, 0xf>(h) << 16;
        const uint32_t wi = e0 >> 3;
        if ((l & 1) == 0 && (all_full || wi < lw)) lplane[wi] = h;
      } else {
        uint32_t h = z[0] | (z[1] << 2) | (z[2] << 4) | (z[3] << 6);
        h |= dpp_fetch<kDppShl1, 0xf>(h) << 8;
        h |= dpp_fetch<kDppShl2, 0xf>(h) << 16;
        const uint32_t wi = e0 >> 4;
        if ((l & 3) == 0 && (all_full || wi < lw)) lplane[wi] = h;
      }
      uint32_t sg = nib;
      sg |= dpp_fetch<kDppShl1, 0xf>(sg) << 4;
      sg |= dpp_fetch<kDppShl2, 0xf>(sg) << 8;
      sg |= dpp_fetch<kDppShl4, 0xf>(sg) << 16;
      const uint32_t si = e0 >> 5;
      if ((l & 7) == 0 && (all_full || si < sw)) splane[si] = sg;
    }
    // a short bucket inside a tensor-aware message keeps a full-size slot: zero its tail
    if (a.btab && live && m < a.d) {
      for (uint32_t w = 2u + lw + sw + l; w < a.fixed_words_full; w += LPB) str[w] = 0;
    }
    // escape word of each bucket: at most one of its lanes holds an index
    const uint64_t eb = __ballot(esc != 0xFFFFFFFFu);
    if (eb) {
      uint64_t mine = eb;
      if constexpr (LPB < 64) mine = (eb >> (sb * LPB)) & ((1ull << LPB) - 1ull);
      const int src = mine ? (int)(sb * LPB) + __ffsll((unsigned long long)mine) - 1 : lane;
      const uint32_t got = (uint32_t)__shfl((int)esc, src, kWave);
      esc = mine ? got : 0xFFFFFFFFu;
    }
    if (l == 0 && live) {
      str[0] = __float_as_uint(scale);
      str[1] = esc;
    }
  }
}

// Exclusive prefix sums of the teams' totals: one workgroup, up to kMaxTeams values.
__global__ __launch_bounds__(1024) void k_encode_prefix(CompactArgs a, uint32_t teams) {
  __shared__ unsigned long long wave_tot[16];
  __shared__ unsigned long long carry;
  constexpr uint32_t kPer = 8;   // totals per thread: kMaxTeams in one trip
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (uint32_t c0 = 0; c0 < teams; c0 += 1024 * kPer) {
    const uint32_t i0 = c0 + (uint32_t)tid * kPer;
    uint32_t v[kPer];
    unsigned long long sum = 0;
#pragma unroll
    for (uint32_t t = 0; t < kPer; ++t) {
      v[t] = i0 + t < teams ? a.totals[i0 + t] : 0u;
      sum += v[t];
    }
    unsigned long long incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const unsigned long long up = __shfl_up(incl, o, kWave);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    unsigned long long before = carry;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    unsigned long long run = before + incl - sum;
#pragma unroll
    for (uint32_t t = 0; t < kPer; ++t) {
      if (i0 + t < teams) a.prefix[i0 + t] = run;
      run += v[t];
    }
    __syncthreads();
    if (tid == 1023) carry = before + incl;
    __syncthreads();
  }
}

// Moves each team's region to its place in the message: base_j = words of the teams
// before j (k_encode_prefix).  One workgroup per team.
__global__ __launch_bounds__(256) void k_encode_compact(CompactArgs a) {
  const int tid = threadIdx.x;
  const uint32_t j = blockIdx.x;
  const uint64_t base = a.prefix[j];
  const uint32_t mine = a.totals[j];
  const uint32_t b_begin = j * a.bper;
  const uint32_t b_end = min(b_begin + a.bper, a.nb);
  // (a team whose region ran out has counted on without storing: nothing to copy)
  const bool fits = base + mine <= a.cap_words && base + mine <= 0xFFFFFFFFull &&
                    mine <= a.region_words;
  if (fits) {
    const uint32_t* __restrict__ src = a.staging + (uint64_t)j * a.region_words;
    uint32_t* __restrict__ dstp = a.payload + base;
    for (uint32_t i = tid; i < mine; i += 256) dstp[i] = src[i];
  }
  for (uint32_t b = b_begin + tid; b < b_end; b += 256)
    a.table[b] = (uint32_t)min(base + a.table[b], (uint64_t)0xFFFFFFFFull);
  if (tid == 0) {
    if (!fits) atomicExch(&a.header[H_STATUS], (uint32_t)QSGD_ERR_CAPACITY);
    if (j == gridDim.x - 1) {
      const uint64_t total = base + mine;
      a.table[a.nb] = (uint32_t)min(total, (uint64_t)0xFFFFFFFFull);
      for (uint32_t i = a.nb + 1; i < a.table_words; ++i) a.table[i] = 0;  // padding
      const uint64_t all = total + a.raw_words;   // the raw values follow the strings
      if (all > a.cap_words) atomicExch(&a.header[H_STATUS], (uint32_t)QSGD_ERR_CAPACITY);
      a.header[H_PW_LO] = (uint32_t)all;
      a.header[H_PW_HI] = (uint32_t)(all >> 32);
    }
  }
}

// Header of an empty message (n = 0).
__global__ void k_write_empty(uint32_t* header, uint32_t* table, uint32_t code, uint32_t norm,
                              uint32_t s, uint64_t d, uint32_t stream_id, uint32_t iteration) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    header[H_MAGIC] = kMagic; header[H_VERSION] = 1; header[H_CODE] = code;
    header[H_NORM] = norm; header[H_S] = s; header[H_STREAM] = stream_id;
    header[H_D_LO] = (uint32_t)d; header[H_D_HI] = (uint32_t)(d >> 32);
    header[H_N_LO] = 0; header[H_N_HI] = 0; header[H_NB_LO] = 0; header[H_NB_HI] = 0;
    header[H_PW_LO] = 0; header[H_PW_HI] = 0; header[H_STATUS] = 0;
    header[H_ITER] = iteration;
    if (table) { table[0] = 0; table[1] = 0; table[2] = 0; table[3] = 0; }
  }
}

// ---- launch table -------------------------------------------------------------
template <int TW, int CPW>
static hipError_t launch_tw_cpw(const EncodeArgs& a, uint32_t code, dim3 grid, size_t lds,
                                hipStream_t st) {
  switch (code) {
    case QSGD_CODE_SPARSE:
      if (TW >= 2 && a.ring == list_records(CPW))
        hipLaunchKernelGGL((k_encode_bucket<TW, CPW, QSGD_CODE_SPARSE, TW >= 2 ? list_records(CPW) : 0u>),
                           grid, dim3(64 * TW), lds, st, a);
      else
        hipLaunchKernelGGL((k_encode_bucket<TW, CPW, QSGD_CODE_SPARSE>), grid, dim3(64 * TW), lds,
                           st, a);
      break;
    case QSGD_CODE_DENSE:
      hipLaunchKernelGGL((k_encode_bucket<TW, CPW, QSGD_CODE_DENSE>), grid, dim3(64 * TW), lds,
                         st, a);
      break;
    default:
      hipLaunchKernelGGL((k_encode_bucket<TW, CPW, QSGD_CODE_FIXED>), grid, dim3(64 * TW), lds,
                         st, a);
      break;
  }
  return hipGetLastError();
}

hipError_t launch_encode_bucket(const EncodeArgs& a, uint32_t code, int tw, int cpw,
                                uint32_t teams, size_t lds, hipStream_t st) {
  const dim3 grid(teams);
  if (tw == 1 && cpw == 1) return launch_tw_cpw<1, 1>(a, code, grid, lds, st);
  if (tw == 1 && cpw == 2) return launch_tw_cpw<1, 2>(a, code, grid, lds, st);
  if (tw == 1 && cpw == 4) return launch_tw_cpw<1, 4>(a, code, grid, lds, st);
  if (tw == 1 && cpw == 8) return launch_tw_cpw<1, 8>(a, code, grid, lds, st);
  if (tw == 2 && cpw == 8) return launch_tw_cpw<2, 8>(a, code, grid, lds, st);
  if (tw == 4 && cpw == 8) return launch_tw_cpw<4, 8>(a, code, grid, lds, st);
  return hipErrorInvalidValue;
}

template <int LPB, int CP>
static hipError_t launch_fixed_small_b(const EncodeArgs& a, uint32_t teams, hipStream_t st) {
  const dim3 grid(teams), block(64);
  switch (a.fixed_bits) {
    case 2: hipLaunchKernelGGL((k_encode_fixed_small<LPB, CP, 2>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((k_encode_fixed_small<LPB, CP, 4>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((k_encode_fixed_small<LPB, CP, 8>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((k_encode_fixed_small<LPB, CP, 16>), grid, block, 0, st, a); break;
  }
  return hipGetLastError();
}

// d <= 1024, d % 4 == 0; a.bper counts groups of 64/lpb buckets per team.
hipError_t launch_encode_fixed_small(const EncodeArgs& a, int lpb, int cp, uint32_t teams,
                                     hipStream_t st) {
  if (lpb == 16 && cp <= 1) return launch_fixed_small_b<16, 1>(a, teams, st);
  if (lpb == 16 && cp <= 2) return launch_fixed_small_b<16, 2>(a, teams, st);
  if (lpb == 16) return launch_fixed_small_b<16, 4>(a, teams, st);
  if (lpb == 32) return launch_fixed_small_b<32, 4>(a, teams, st);
  return launch_fixed_small_b<64, 4>(a, teams, st);
}

hipError_t launch_encode_compact(const CompactArgs& a, uint32_t teams, hipStream_t st) {
  hipLaunchKernelGGL(k_encode_prefix, dim3(1), dim3(1024), 0, st, a, teams);
  hipLaunchKernelGGL(k_encode_compact, dim3(teams), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_write_empty(uint32_t* header, uint32_t* table, uint32_t code, uint32_t norm,
                              uint32_t s, uint64_t d, uint32_t stream_id, uint32_t iteration,
                              hipStream_t st) {
  hipLaunchKernelGGL(k_write_empty, dim3(1), dim3(64), 0, st, header, table, code, norm, s, d,
                     stream_id, iteration);
  return hipGetLastError();
}

}  // namespace qsgd
