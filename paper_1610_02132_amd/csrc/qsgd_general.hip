// General path: any bucket size d (d > 8192, d not a multiple of 4, d = n).
//
// Encode.  A bucket no longer fits one workgroup's registers, so it is cut into
// segments of 2048 values, one wavefront each, and the steps that the bucket path
// does inside a workgroup become kernels:
//   partial  per-segment sum of squares (fp64) or max            -> workspace
//   scale    per-bucket reduction of the partials, s/scale
//   encode   per-segment sub-stream (same wavefront code as the bucket path, with
//            code words wide enough for 32-bit gaps)              -> workspace slot
//   scan     one workgroup walks the segments in order: which nonzero precedes a
//            segment's first one (max-scan), the bit offset of every segment in
//            its bucket string (sum-scan), the word offset of every bucket
//   fill     zeroes the payload
//   place    per segment: ORs gap code, sub-stream and stop bit into the payload
// Decode.  Records are added to a dense fp32 accumulator in the workspace, bucket by
// bucket and inside a bucket message after message (so every coordinate's sum has
// the order k = 0, 1, ...); a last kernel applies the accumulator to x.  Buckets
// above 8192 values carry a list of entry points behind their string and are read
// by a workgroup, a thread per stretch; shorter ones by a thread per bucket.
#include "qsgd_device.hpp"
#include "qsgd_encode_wave.hpp"
#include "qsgd_kernels.hpp"

namespace qsgd {

namespace {

constexpr int kSegChunks = 8;  // kSeg / kChunk

struct SegRef {
  uint64_t b;        // bucket
  uint32_t j;        // segment within the bucket
  uint64_t m;        // elements in the bucket
  uint32_t pos0;     // bucket position of the segment's first element
  uint32_t len;      // elements in the segment (0: past the end of a short bucket)
  uint64_t gidx0;    // global index of its first element
};

__device__ __forceinline__ SegRef seg_ref(const GenArgs& a, uint64_t seg) {
  SegRef r;
  r.b = seg / a.spb;
  r.j = (uint32_t)(seg - r.b * a.spb);
  const uint64_t base = r.b * a.d;
  r.m = min(a.d, a.n - base);
  const uint64_t p0 = (uint64_t)r.j * kSeg;
  r.pos0 = (uint32_t)p0;
  r.len = p0 < r.m ? (uint32_t)min((uint64_t)kSeg, r.m - p0) : 0u;
  r.gidx0 = base + p0;
  return r;
}

// Lane's four values of chunk c of a segment; any alignment, zeros past the end.
__device__ __forceinline__ float4 load_quad_any(const float* __restrict__ g, uint64_t gidx,
                                                uint32_t e, uint32_t len) {
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  const float* p = g + gidx + e;
  if (e + 3 < len && (((gidx + e) & 3u) == 0)) {
    v = *reinterpret_cast<const float4*>(p);
  } else {
    if (e + 0 < len) v.x = p[0];
    if (e + 1 < len) v.y = p[1];
    if (e + 2 < len) v.z = p[2];
    if (e + 3 < len) v.w = p[3];
  }
  return v;
}

// Inclusive scans over a 1024-thread workgroup (16 wavefronts).
// 64-bit value of the lane a DPP control names (0 where there is none).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned long long dpp_fetch_u64(unsigned long long v) {
  const uint32_t lo = dpp_fetch<CTRL, ROW_MASK>((uint32_t)v);
  const uint32_t hi = dpp_fetch<CTRL, ROW_MASK>((uint32_t)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

// (the operations used here have 0 as their identity: sums and maxima of unsigned values)
template <typename T, typename Op>
__device__ __forceinline__ T block_incl_scan(T v, T identity, T* wave_tot, Op op) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = op(v, dpp_fetch_u64<kDppShr1, 0xf>(v));
  v = op(v, dpp_fetch_u64<kDppShr2, 0xf>(v));
  v = op(v, dpp_fetch_u64<kDppShr4, 0xf>(v));
  v = op(v, dpp_fetch_u64<kDppShr8, 0xf>(v));
  v = op(v, dpp_fetch_u64<kDppBcast15, 0xa>(v));
  v = op(v, dpp_fetch_u64<kDppBcast31, 0xc>(v));
  // (wave_tot is free here: every call ends with a barrier after its reads)
  if (lane == 63) wave_tot[wave] = v;
  __syncthreads();
  T pre = identity;
  for (int w = 0; w < wave; ++w) pre = op(pre, wave_tot[w]);
  __syncthreads();
  return op(pre, v);
}

struct OpSum { __device__ unsigned long long operator()(unsigned long long a, unsigned long long b) const { return a + b; } };
struct OpMax { __device__ unsigned long long operator()(unsigned long long a, unsigned long long b) const { return a > b ? a : b; } };

}  // namespace

// ---- encode --------------------------------------------------------------------------

__global__ __launch_bounds__(256) void k_gen_partial(GenArgs a) {
  const int lane = threadIdx.x & 63;
  const uint64_t seg = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (seg >= a.nseg) return;
  const SegRef r = seg_ref(a, seg);
  double ss = 0.0;
  float mx = 0.f;
  for (int c = 0; c < kSegChunks; ++c) {
    const uint32_t e = (uint32_t)c * kChunk + lane * 4;
    if ((uint32_t)c * kChunk >= r.len) break;
    const float4 v = load_quad_any(a.g, r.gidx0, e, r.len);
    if (a.norm_mode == 0) {
      ss = fma((double)v.x, (double)v.x, ss);
      ss = fma((double)v.y, (double)v.y, ss);
      ss = fma((double)v.z, (double)v.z, ss);
      ss = fma((double)v.w, (double)v.w, ss);
    } else {
      mx = fmaxf(fmaxf(mx, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
  }
  if (a.norm_mode == 0) ss = wave_sum_f64(ss);
  else ss = (double)wave_max_f32(mx);
  if (lane == 0) a.partial[seg] = ss;
}

__global__ __launch_bounds__(256) void k_gen_scale(GenArgs a) {
  const int lane = threadIdx.x & 63;
  const uint64_t b = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t* h = a.header;
    h[H_MAGIC] = kMagic; h[H_VERSION] = 1; h[H_CODE] = a.code; h[H_NORM] = a.norm_mode;
    h[H_S] = a.s; h[H_STREAM] = a.stream_id;
    h[H_D_LO] = (uint32_t)a.d; h[H_D_HI] = (uint32_t)(a.d >> 32);
    h[H_N_LO] = (uint32_t)a.n; h[H_N_HI] = (uint32_t)(a.n >> 32);
    h[H_NB_LO] = (uint32_t)a.nb; h[H_NB_HI] = (uint32_t)(a.nb >> 32);
    h[H_PW_LO] = (uint32_t)a.fixed_payload_words;
    h[H_PW_HI] = (uint32_t)(a.fixed_payload_words >> 32);
    h[H_STATUS] = 0; h[H_ITER] = a.iteration;
  }
  if (b >= a.nb) return;
  // sixteen independent chains per lane, their loads in flight together: with thousands of
  // segments in one bucket the memory latency of each trip sets the pace
  constexpr int kChains = 16;
  double accs[kChains];
#pragma unroll
  for (int t = 0; t < kChains; ++t) accs[t] = 0.0;
  uint64_t j = lane;
  for (; j + (kChains - 1) * kWave < a.spb; j += kChains * kWave) {
    double p[kChains];
#pragma unroll
    for (int t = 0; t < kChains; ++t) p[t] = a.partial[b * a.spb + j + (uint64_t)t * kWave];
#pragma unroll
    for (int t = 0; t < kChains; ++t)
      accs[t] = a.norm_mode == 0 ? accs[t] + p[t] : fmax(accs[t], p[t]);
  }
  for (; j < a.spb; j += kWave) {
    const double p = a.partial[b * a.spb + j];
    accs[0] = a.norm_mode == 0 ? accs[0] + p : fmax(accs[0], p);
  }
#pragma unroll
  for (int w = kChains / 2; w >= 1; w /= 2) {
#pragma unroll
    for (int t = 0; t < w; ++t)
      accs[t] = a.norm_mode == 0 ? accs[t] + accs[t + w] : fmax(accs[t], accs[t + w]);
  }
  const double acc = accs[0];
  float scale;
  if (a.norm_mode == 0) scale = (float)sqrt(wave_sum_f64(acc));
  else scale = wave_max_f32((float)acc);
  if (lane == 0) {
    a.scale[b] = scale;
    if (a.code == QSGD_CODE_FIXED) {
      uint32_t* str = a.payload + b * a.fixed_words_full;
      str[0] = __float_as_uint(scale);
      str[1] = 0xFFFFFFFFu;
    }
  }
}

template <int CODE, bool ALIGNED>
__global__ __launch_bounds__(64) void k_gen_encode(GenArgs a) {
  extern __shared__ uint32_t smem[];
  uint32_t* const sub = smem;
  uint32_t* const ring = smem + a.sub_words;
  const int lane = threadIdx.x;
  const uint64_t seg = blockIdx.x;
  const SegRef r = seg_ref(a, seg);
  if (CODE != QSGD_CODE_FIXED) {
    for (uint32_t j = lane; j < a.sub_words; j += kWave) sub[j] = 0;
    __syncthreads();
  }
  WaveOut wo;
  wo.first_pos = 0; wo.last_pos = 0; wo.bits = 0;
  if (r.len) {
    float4 v[kSegChunks];
#pragma unroll
    for (int c = 0; c < kSegChunks; ++c) {
      v[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if ((uint32_t)c * kChunk < r.len)
        v[c] = load_quad_any(a.g, r.gidx0, (uint32_t)c * kChunk + lane * 4, r.len);
    }
    const float scale = a.scale[r.b];
    QuantCtx qc;
    qc.s_f = (float)a.s;
    qc.inv = (scale > 0.f) ? qc.s_f / scale : 0.f;
    qc.s = a.s; qc.key0 = a.key0; qc.key1 = a.key1;
    qc.stream_id = a.stream_id; qc.iteration = a.iteration;
    const int nchunks = (int)((r.len + kChunk - 1) / kChunk);
    uint32_t rall[kSegChunks][4];
    draw_all<kSegChunks, ALIGNED>(a.index_base + r.gidx0, lane, qc, rall);
    if (CODE == QSGD_CODE_SPARSE) {
      encode_sparse_wave<kSegChunks, true>(v, rall, nchunks, r.pos0, lane, qc, ring, nullptr, sub, wo);
    } else if (CODE == QSGD_CODE_DENSE) {
      encode_dense_wave<kSegChunks>(v, rall, nchunks, r.len, lane, qc, sub, wo);
    } else {
      // fixed width: fields of 2048 values start on word boundaries in both planes
      const uint32_t B = a.fixed_bits, fmax = (1u << B) - 1u;
      uint32_t* const str = a.payload + r.b * a.fixed_words_full;
      const uint64_t lw = (r.m * B + 31) >> 5;
      uint32_t* const lplane = str + 2 + (((uint64_t)r.pos0 * B) >> 5);
      uint32_t* const splane = str + 2 + lw + (r.pos0 >> 5);
      const uint32_t lwn = (uint32_t)((r.len * B + 31u) >> 5), swn = (r.len + 31u) >> 5;
#pragma unroll
      for (int c = 0; c < kSegChunks; ++c) {
        if (c >= nchunks) break;
        const uint32_t e0 = (uint32_t)c * kChunk + lane * 4;
        const uint32_t (&rr)[4] = rall[c];
        const float vv[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
        uint32_t z[4], nib = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          z[j] = (e0 + j < r.len) ? quantize_one(vv[j], qc.inv, qc.s_f, qc.s, rr[j]) : 0u;
          if (z[j] > fmax) { str[1] = r.pos0 + e0 + j; z[j] = fmax; }
          nib |= (vv[j] < 0.f ? 1u : 0u) << j;
        }
        if (B == 8) {
          if ((e0 >> 2) < lwn) lplane[e0 >> 2] = z[0] | (z[1] << 8) | (z[2] << 16) | (z[3] << 24);
        } else if (B == 16) {
          if ((e0 >> 1) < lwn) lplane[e0 >> 1] = z[0] | (z[1] << 16);
          if ((e0 >> 1) + 1 < lwn) lplane[(e0 >> 1) + 1] = z[2] | (z[3] << 16);
        } else if (B == 4) {
          uint32_t h = z[0] | (z[1] << 4) | (z[2] << 8) | (z[3] << 12);
          h |= dpp_fetch<kDppShl1, 0xf>(h) << 16;
          if ((lane & 1) == 0 && (e0 >> 3) < lwn) lplane[e0 >> 3] = h;
        } else {
          uint32_t h = z[0] | (z[1] << 2) | (z[2] << 4) | (z[3] << 6);
          h |= dpp_fetch<kDppShl1, 0xf>(h) << 8;
          h |= dpp_fetch<kDppShl2, 0xf>(h) << 16;
          if ((lane & 3) == 0 && (e0 >> 4) < lwn) lplane[e0 >> 4] = h;
        }
        uint32_t sg = nib;
        sg |= dpp_fetch<kDppShl1, 0xf>(sg) << 4;
        sg |= dpp_fetch<kDppShl2, 0xf>(sg) << 8;
        sg |= dpp_fetch<kDppShl4, 0xf>(sg) << 16;
        if ((lane & 7) == 0 && (e0 >> 5) < swn) splane[e0 >> 5] = sg;
      }
    }
  }
  if (CODE == QSGD_CODE_FIXED) return;
  __syncthreads();
  if (lane == 0) {
    a.seginfo[3 * seg + 0] = wo.first_pos;
    a.seginfo[3 * seg + 1] = wo.last_pos;
    a.seginfo[3 * seg + 2] = wo.bits;
  }
  uint32_t* slot = a.slots + seg * a.sub_words;
  const uint32_t nw = (wo.bits + 31u) >> 5;
  for (uint32_t j = lane; j < nw; j += kWave) slot[j] = sub[j];
}

// One workgroup of 1024 threads walks all segments in order, kScanPer consecutive segments
// per thread and trip: a thread scans its own segments one after the other and the
// workgroup scans the threads' totals.
constexpr int kScanPer = 4;
constexpr uint32_t kScanTrip = 1024 * kScanPer;
__global__ __launch_bounds__(1024) void k_gen_scan(GenArgs a) {
  __shared__ unsigned long long wave_tot[16];
  __shared__ unsigned long long tmp[kScanTrip];   // one value per segment of the trip
  __shared__ unsigned long long tot[1024];        // one value per thread
  __shared__ unsigned long long carry[5];  // max global position, bits in open bucket, words,
                                           // bits of the last segment, entries in open bucket
  const int i = threadIdx.x;
  if (i == 0) {
    carry[0] = 0; carry[1] = 0; carry[2] = 0; carry[3] = 0; carry[4] = 0;
    a.table[0] = 0;
  }
  __syncthreads();
  const bool sparse = a.code == QSGD_CODE_SPARSE;
  for (uint64_t c0 = 0; c0 < a.nseg; c0 += kScanTrip) {
    uint64_t seg[kScanPer], b[kScanPer];
    uint32_t idx[kScanPer], j[kScanPer], first[kScanPer], last[kScanPer], bits[kScanPer];
    bool live[kScanPer];
    unsigned long long base[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      idx[t] = (uint32_t)i * kScanPer + t;
      seg[t] = c0 + idx[t];
      live[t] = seg[t] < a.nseg;
      b[t] = 0; j[t] = 0; first[t] = 0; last[t] = 0; bits[t] = 0;
      if (live[t]) {
        b[t] = seg[t] / a.spb; j[t] = (uint32_t)(seg[t] - b[t] * a.spb);
        first[t] = a.seginfo[3 * seg[t]]; last[t] = a.seginfo[3 * seg[t] + 1];
        bits[t] = a.seginfo[3 * seg[t] + 2];
      }
      base[t] = b[t] * a.d;
    }
    const unsigned long long c_max = carry[0], c_bits = carry[1], c_words = carry[2];
    const unsigned long long c_tb = carry[3], c_ents = carry[4];
    // which nonzero precedes each segment's first one: prefix maximum of the last positions
    unsigned long long m_loc[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      const unsigned long long lastg = (live[t] && first[t]) ? base[t] + last[t] : 0ull;
      m_loc[t] = t ? (m_loc[t - 1] > lastg ? m_loc[t - 1] : lastg) : lastg;
    }
    tot[i] = block_incl_scan<unsigned long long>(m_loc[kScanPer - 1], 0ull, wave_tot, OpMax());
    __syncthreads();
    const unsigned long long m_before = i ? tot[i - 1] : 0ull;   // threads before this one
    const unsigned long long chunk_max = tot[1023];
    uint32_t prev_in_bucket[kScanPer], gap[kScanPer];
    unsigned long long tb[kScanPer], s_loc[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      unsigned long long prevg = t ? (m_before > m_loc[t - 1] ? m_before : m_loc[t - 1]) : m_before;
      prevg = prevg > c_max ? prevg : c_max;
      prev_in_bucket[t] = prevg > base[t] ? (uint32_t)(prevg - base[t]) : 0u;
      gap[t] = (live[t] && first[t] && sparse) ? first[t] - prev_in_bucket[t] : 0u;
      const uint32_t glen = gap[t] ? omega_length(gap[t]) : 0u;
      tb[t] = (unsigned long long)glen + bits[t];
      s_loc[t] = (t ? s_loc[t - 1] : 0ull) + tb[t];
    }
    // bit offset of each segment inside its bucket string
    const unsigned long long s_tot =
        block_incl_scan<unsigned long long>(s_loc[kScanPer - 1], 0ull, wave_tot, OpSum());
    unsigned long long s_excl[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      s_excl[t] = s_tot - s_loc[kScanPer - 1] + s_loc[t] - tb[t];
      tmp[idx[t]] = s_excl[t];
    }
    tot[i] = tb[kScanPer - 1];   // (tot was last read before the scan's barriers)
    __syncthreads();
    unsigned long long before[kScanPer], tb_prev[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      // bits of this bucket's records before this segment
      if (j[t] <= idx[t]) before[t] = s_excl[t] - tmp[idx[t] - j[t]];
      else before[t] = c_bits + s_excl[t];
      tb_prev[t] = t ? tb[t - 1] : (i ? tot[i - 1] : c_tb);
    }
    __syncthreads();
    // entry list of long buckets: segment j >= 1 is listed iff its bit offset lies in a
    // later block of kEntryBits bits than the offset of segment j - 1
    bool listed[kScanPer];
    unsigned long long e_loc[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      const unsigned long long start = 32ull + before[t];
      const unsigned long long m_b = live[t] ? min((unsigned long long)a.d, a.n - base[t]) : 0ull;
      listed[t] = a.entries && live[t] && j[t] >= 1 && (unsigned long long)j[t] * kSeg < m_b &&
                  (start / kEntryBits) > ((start - tb_prev[t]) / kEntryBits) &&
                  start < (1ull << 32);
      e_loc[t] = (t ? e_loc[t - 1] : 0ull) + (listed[t] ? 1ull : 0ull);
    }
    const unsigned long long e_tot =
        block_incl_scan<unsigned long long>(e_loc[kScanPer - 1], 0ull, wave_tot, OpSum());
    unsigned long long e_excl[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      e_excl[t] = e_tot - e_loc[kScanPer - 1] + e_loc[t] - (listed[t] ? 1ull : 0ull);
      tmp[idx[t]] = e_excl[t];
    }
    __syncthreads();
    unsigned long long rank[kScanPer], ents[kScanPer], w_loc[kScanPer];
    bool is_end[kScanPer];
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      // listed segments of this bucket before this one
      if (j[t] <= idx[t]) rank[t] = e_excl[t] - tmp[idx[t] - j[t]];
      else rank[t] = c_ents + e_excl[t];
      is_end[t] = live[t] && j[t] == a.spb - 1;
      ents[t] = rank[t] + (listed[t] ? 1ull : 0ull);  // at the end: of the bucket
      unsigned long long words = 0;
      if (is_end[t]) {
        words = (32ull + before[t] + tb[t] + (sparse ? 1ull : 0ull) + 31ull) >> 5;
        if (a.entries) words += 2ull * ents[t] + 1ull;
      }
      w_loc[t] = (t ? w_loc[t - 1] : 0ull) + words;
    }
    const unsigned long long w_tot =
        block_incl_scan<unsigned long long>(w_loc[kScanPer - 1], 0ull, wave_tot, OpSum());
#pragma unroll
    for (int t = 0; t < kScanPer; ++t) {
      if (!live[t]) continue;
      const unsigned long long w_incl = w_tot - w_loc[kScanPer - 1] + w_loc[t];
      a.segstart[seg[t]] = 32ull + before[t];
      a.seggap[seg[t]] = gap[t];
      if (a.entries) {
        a.segrank[seg[t]] = listed[t] ? (uint32_t)rank[t] : 0xFFFFFFFFu;
        a.segprev[seg[t]] = sparse ? prev_in_bucket[t] : j[t] * kSeg;
        if (is_end[t]) a.bents[b[t]] = (uint32_t)ents[t];
      }
      if (is_end[t]) {
        const unsigned long long off = c_words + w_incl;
        a.table[b[t] + 1] = off > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)off;
      }
      // (the carries were read at the top of this trip, several barriers ago)
      if (idx[t] == kScanTrip - 1 || seg[t] == a.nseg - 1) {
        carry[0] = chunk_max > c_max ? chunk_max : c_max;
        carry[1] = is_end[t] ? 0ull : before[t] + tb[t];
        carry[2] = c_words + w_incl;
        carry[3] = tb[t];
        carry[4] = is_end[t] ? 0ull : ents[t];
      }
    }
    __syncthreads();
  }
  if (i == 0) {
    const unsigned long long total = carry[2];
    a.header[H_PW_LO] = (uint32_t)total;
    a.header[H_PW_HI] = (uint32_t)(total >> 32);
    for (uint64_t t = a.nb + 1; t < a.table_words; ++t) a.table[t] = 0;
    if (total > a.cap_words || total > 0xFFFFFFFFull)
      a.header[H_STATUS] = (uint32_t)QSGD_ERR_CAPACITY;
  }
}

__global__ __launch_bounds__(256) void k_gen_fill(GenArgs a) {
  const uint64_t total = a.header[H_PW_LO] | ((uint64_t)a.header[H_PW_HI] << 32);
  const uint64_t lim = min(total, a.cap_words);
  for (uint64_t w = (uint64_t)blockIdx.x * 256 + threadIdx.x; w < lim; w += (uint64_t)gridDim.x * 256)
    a.payload[w] = 0;
}

__global__ __launch_bounds__(64) void k_gen_place(GenArgs a) {
  if (a.header[H_STATUS] != 0) return;  // does not fit: nothing is written
  const int lane = threadIdx.x;
  const uint64_t seg = blockIdx.x;
  const uint64_t b = seg / a.spb;
  const uint32_t j = (uint32_t)(seg - b * a.spb);
  uint32_t* const str = a.payload + a.table[b];
  const uint32_t bits = a.seginfo[3 * seg + 2];
  const uint32_t gap = a.seggap[seg];
  const uint64_t start = a.segstart[seg];
  uint32_t glen = 0;
  if (lane == 0) {
    if (j == 0) str[0] = __float_as_uint(a.scale[b]);
    if (gap) {
      uint64_t gc;
      omega_encode(gap, gc, glen);
      global_emit(str, start, gc, glen);
    }
    if (j == a.spb - 1 && a.code == QSGD_CODE_SPARSE) global_emit(str, start + glen + bits, 1ull, 1u);
  }
  if (a.entries && lane == 0) {
    // the entry list sits behind the string's last word: pairs, then their count
    const uint32_t ents = a.bents[b];
    uint32_t* const list = a.payload + a.table[b + 1] - (2u * ents + 1u);
    const uint32_t r = a.segrank[seg];
    if (r != 0xFFFFFFFFu) {
      list[2u * r] = (uint32_t)start;
      list[2u * r + 1u] = a.segprev[seg];
    }
    if (j == a.spb - 1) list[2u * ents] = ents;
  }
  glen = lane_bcast(glen, 0);
  const uint64_t o = start + glen;
  const uint64_t w0 = o >> 5;
  const uint32_t sh = (uint32_t)(o & 31u);
  const uint32_t* slot = a.slots + seg * a.sub_words;
  const uint32_t nw = (bits + 31u) >> 5;
  for (uint32_t t = lane; t < nw; t += kWave) {
    const uint32_t x = slot[t];
    if (x) {
      atomicOr(&str[w0 + t], x >> sh);
      if (sh && (x << (32u - sh))) atomicOr(&str[w0 + t + 1], x << (32u - sh));
    }
  }
}

// ---- decode --------------------------------------------------------------------------

namespace {

// 64 stream bits starting at bit `bitpos` of a string of nwords words (zeros past the end).
__device__ __forceinline__ uint64_t peek64(const uint32_t* w, uint64_t nwords, uint64_t bitpos) {
  const uint64_t wi = bitpos >> 5;
  const uint32_t off = (uint32_t)(bitpos & 31u);
  const uint64_t a0 = wi < nwords ? w[wi] : 0u;
  const uint64_t a1 = wi + 1 < nwords ? w[wi + 1] : 0u;
  const uint64_t a2 = wi + 2 < nwords ? w[wi + 2] : 0u;
  const uint64_t hi = (a0 << 32) | a1;
  return off ? (hi << off) | (a2 >> (32u - off)) : hi;
}

// Decoder rule of the recursive Elias code (App. A.2) on a 64-bit window; values
// below 2^32.  Returns 0 for malformed input; `len` = bits used.
__device__ __forceinline__ uint32_t omega_loop(uint64_t w, uint32_t& len) {
  uint32_t N = 1, used = 0;
  for (;;) {
    if ((w >> 63) == 0) { len = used + 1; return N; }
    if (N > 31u || used + N + 2u > 64u) { len = 0; return 0; }
    const uint32_t v = (uint32_t)(w >> (63u - N));
    w <<= (N + 1u);
    used += N + 1u;
    N = v;
  }
}

}  // namespace

__global__ __launch_bounds__(256) void k_gen_zero(float* p, uint64_t n) {
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256)
    p[i] = 0.f;
}

// Four consecutive words of a string in registers (zeros past its end): three serve a
// 64-bit peek at any bit offset of the first one, the fourth is requested one word
// ahead of its use so that a reader does not wait for memory at every record.
struct WordWindow {
  const uint32_t* str;
  uint64_t nwords, wi;   // w0..w3 = words wi..wi+3
  uint32_t w0, w1, w2, w3;
  __device__ __forceinline__ uint32_t word(uint64_t i) const { return i < nwords ? str[i] : 0u; }
  __device__ __forceinline__ void open(const uint32_t* s, uint64_t n, uint64_t bitpos) {
    str = s; nwords = n; wi = bitpos >> 5;
    w0 = word(wi); w1 = word(wi + 1); w2 = word(wi + 2); w3 = word(wi + 3);
  }
  // The 64 stream bits from `bitpos` on; bitpos never moves backwards.
  __device__ __forceinline__ uint64_t peek(uint64_t bitpos) {
    while (wi < (bitpos >> 5)) {
      w0 = w1; w1 = w2; w2 = w3;
      w3 = word(wi + 4);
      ++wi;
    }
    const uint32_t off = (uint32_t)(bitpos & 31u);
    const uint64_t hi = ((uint64_t)w0 << 32) | w1;
    return off ? (hi << off) | (w2 >> (32u - off)) : hi;
  }
};

// One string, read front to back from (bitpos, pos) until `stop` (or, for the last
// stretch of a Code'_s string, until position m); values are ADDED to out[] with plain
// read-modify-writes: the caller guarantees that nobody else touches this bucket's
// part of out[] at the same time.  Returns false on malformed input.
__device__ __forceinline__ bool parse_stretch(const uint32_t* str, uint64_t nwords, bool sparse,
                                              bool to_end_of_bucket, uint64_t stop, uint64_t m,
                                              uint32_t s, float scale, uint64_t& bitpos,
                                              uint64_t& pos, float* out) {
  WordWindow win;
  win.open(str, nwords, bitpos);
  // Records are read kBatch at a time and then added together: the additions of one
  // message hit distinct coordinates, so their loads can all be in flight at once
  // instead of one memory round trip per record.
  constexpr int kBatch = 8;
  for (;;) {
    float* where[kBatch];
    float what[kBatch];
    bool done = false;
#pragma unroll
    for (int t = 0; t < kBatch; ++t) {
      where[t] = nullptr;
      what[t] = 0.f;
      if (done) continue;
      if (to_end_of_bucket ? pos >= m : bitpos >= stop) { done = true; continue; }
      uint32_t gl = 0, gap = 1;
      if (sparse) {
        gap = omega_loop(win.peek(bitpos), gl);
        if (gap == 0) return false;
      }
      const uint64_t w = win.peek(bitpos + gl);
      uint32_t ll;
      uint32_t lev = omega_loop(w << 1, ll);
      bitpos += gl + 1u + ll;
      pos += gap;
      if (lev == 0 || pos > m || bitpos > stop) return false;
      if (!sparse) lev -= 1u;
      if (lev > s) return false;
      if (lev) {
        const float mag = scale * (float)lev;
        where[t] = out + (pos - 1);
        what[t] = (w >> 63) ? -mag : mag;
      }
    }
    float old[kBatch];
#pragma unroll
    for (int t = 0; t < kBatch; ++t) old[t] = where[t] ? *where[t] : 0.f;
#pragma unroll
    for (int t = 0; t < kBatch; ++t)
      if (where[t]) *where[t] = old[t] + what[t];
    if (done) return true;
  }
}

// Where a bucket string of message k lies and where its records end.
struct StringRef {
  const uint32_t* str;
  uint64_t nwords;   // words of the string proper
  uint64_t endbit;   // records end here
  const uint32_t* list;
  uint64_t ents;     // entry points behind the string
  float scale;
};

__device__ __forceinline__ bool open_string(const DecodeArgs& a, uint32_t k, uint64_t b,
                                            bool entries, StringRef& r) {
  const uint32_t* msg = a.msgs[k];
  const uint64_t pay = (uint64_t)H_WORDS + a.table_words;
  const uint32_t o0 = msg[H_WORDS + b], o1 = msg[H_WORDS + b + 1];
  if (!(o0 < o1 && pay + o1 <= a.msg_words[k])) return false;
  r.str = msg + pay + o0;
  uint64_t words = o1 - o0;
  r.ents = 0;
  r.list = nullptr;
  if (entries) {
    r.ents = r.str[words - 1];
    if (2 * r.ents + 1 >= words) return false;
    words -= 2 * r.ents + 1;
    r.list = r.str + words;
  }
  r.nwords = words;
  r.scale = __uint_as_float(r.str[0]) / (float)a.s;
  r.endbit = words * 32;
  if (a.code == QSGD_CODE_SPARSE) {
    const uint32_t last = r.str[words - 1];
    if (last == 0) return false;
    r.endbit = words * 32 - 1 - (uint32_t)(__ffs((int)last) - 1);
    if (r.endbit < 32) return false;
  }
  return true;
}

// Short buckets of the general path (d <= kEntryMinD, d not a multiple of 4): one thread
// per bucket reads the K strings one after the other, so every coordinate receives its
// terms in message order.
__global__ __launch_bounds__(256) void k_gen_parse(DecodeArgs a, float* acc) {
  if (*a.status != 0) return;
  const uint64_t b = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (b >= a.nb) return;
  const uint64_t base = b * (uint64_t)a.d;
  const uint64_t m = min((uint64_t)a.d, a.n - base);
  const bool sparse = a.code == QSGD_CODE_SPARSE;
  for (uint32_t k = 0; k < a.K; ++k) {
    StringRef r;
    if (!open_string(a, k, b, false, r)) { flag_corrupt(a.status); return; }
    uint64_t bitpos = 32, pos = 0;
    if (!parse_stretch(r.str, r.nwords, sparse, !sparse, r.endbit, m, a.s, r.scale, bitpos, pos,
                       acc + base) ||
        (!sparse && bitpos > r.endbit)) {
      flag_corrupt(a.status);
      return;
    }
  }
}

// Opens the K strings of bucket b side by side (a chain of dependent reads each).
// Returns false (every thread) if one of them is malformed.  Ends with a barrier.
__device__ __forceinline__ bool open_strings(const DecodeArgs& a, uint64_t b, StringRef* refs,
                                             uint32_t* bad) {
  if (threadIdx.x < a.K) {
    StringRef mine;
    if (open_string(a, threadIdx.x, b, true, mine)) refs[threadIdx.x] = mine;
    else *bad = 1;
  }
  __syncthreads();
  return *bad == 0;
}

// The messages take their turns (a barrier in between), a thread per stretch between two
// entry points: every coordinate receives its terms in message order.  Every stretch must
// end exactly where the next one starts, at the position the list names.
__device__ __forceinline__ bool parse_in_turns(const DecodeArgs& a, const StringRef* refs,
                                               uint64_t m, float* out, uint32_t* bad) {
  const bool sparse = a.code == QSGD_CODE_SPARSE;
  for (uint32_t k = 0; k < a.K; ++k) {
    const StringRef sr = refs[k];
    int my_bad = 0;
    for (uint64_t r = threadIdx.x; r <= sr.ents; r += blockDim.x) {
      uint64_t bitpos = r ? sr.list[2 * (r - 1)] : 32;
      uint64_t pos = r ? sr.list[2 * (r - 1) + 1] : 0;
      const bool last_stretch = r == sr.ents;
      const uint64_t stop = last_stretch ? sr.endbit : sr.list[2 * r];
      bool ok = bitpos >= 32 && bitpos <= stop && stop <= sr.endbit && pos <= m;
      ok = ok && parse_stretch(sr.str, sr.nwords, sparse, last_stretch && !sparse, stop, m, a.s,
                               sr.scale, bitpos, pos, out);
      // the stretch ends where the next one starts, at the position the list names
      if (ok && !last_stretch) ok = bitpos == stop && pos == sr.list[2 * r + 1];
      if (ok && last_stretch && !sparse) ok = pos == m && bitpos <= sr.endbit;
      if (!ok) my_bad = 1;
    }
    // message k is in before message k + 1 adds to the same coordinates; the barrier also
    // carries the verdict, so that every thread leaves (or stays) together
    if (__syncthreads_or(my_bad)) {
      if (threadIdx.x == 0) *bad = 1;
      return false;
    }
  }
  return true;
}

// Long buckets (d > kEntryMinD): the string is followed by a list of entry points, so a
// workgroup reads one bucket with a thread per stretch, message after message.
__global__ __launch_bounds__(256) void k_gen_parse_entries(DecodeArgs a, float* acc) {
  if (*a.status != 0) return;
  __shared__ uint32_t bad;
  __shared__ StringRef refs[QSGD_MAX_PEERS];
  if (threadIdx.x == 0) bad = 0;
  const uint64_t b = blockIdx.x;
  const uint64_t base = b * (uint64_t)a.d;
  const uint64_t m = min((uint64_t)a.d, a.n - base);
  __syncthreads();
  if (!open_strings(a, b, refs, &bad) || !parse_in_turns(a, refs, m, acc + base, &bad)) {
    if (threadIdx.x == 0) flag_corrupt(a.status);
  }
}

// Code_s records of one stretch, handed to f eight at a time: f(positions (0-based; ~0 for
// an unused slot), values), so that f can have its memory accesses in flight together.
constexpr int kWalkBatch = 8;
template <class F>
__device__ __forceinline__ bool walk_stretch(const StringRef& sr, uint64_t stop, uint64_t m,
                                             uint32_t s, uint64_t& bitpos, uint64_t& pos, F&& f) {
  WordWindow win;
  win.open(sr.str, sr.nwords, bitpos);
  for (;;) {
    uint64_t where[kWalkBatch];
    float what[kWalkBatch];
    bool done = false;
#pragma unroll
    for (int t = 0; t < kWalkBatch; ++t) {
      where[t] = ~0ull;
      what[t] = 0.f;
      if (done) continue;
      if (bitpos >= stop) { done = true; continue; }
      uint32_t gl, ll;
      const uint32_t gap = omega_loop(win.peek(bitpos), gl);
      if (gap == 0) return false;
      const uint64_t w = win.peek(bitpos + gl);
      const uint32_t lev = omega_loop(w << 1, ll);
      bitpos += gl + 1u + ll;
      pos += gap;
      if (lev == 0 || lev > s || pos > m || bitpos > stop) return false;
      const float mag = sr.scale * (float)lev;
      where[t] = pos - 1;
      what[t] = (w >> 63) ? -mag : mag;
    }
    f(where, what);
    if (done) return true;
  }
}

// Long buckets of sparse Code_s messages (the host expects few coordinates that several
// messages hit): all K messages are read at the same time, a workgroup per (bucket,
// message) and a thread per stretch, in three kernels:
//   count    every record adds 1 to its coordinate's word of the accumulator (an integer);
//   store    the strings are read again: a record whose coordinate counts 1 stores its
//            value (0 + v = v, the sum in message order); the others go to the bucket's
//            list in the workspace;
//   resolve  a coordinate on the list is summed from 0 in message order by the thread that
//            holds its record of the lowest message.  A list that overflowed (the messages
//            collide after all) makes the bucket's workgroup clear the bucket and read the
//            messages in turns.
struct CollideList {
  uint32_t* count;
  uint32_t* pos;
  float* val;
  uint32_t* msg;
};
__device__ __forceinline__ CollideList collide_list(uint8_t* lists, uint64_t b) {
  uint8_t* const base = lists + b * (uint64_t)kCollideBytes;
  CollideList l;
  l.count = reinterpret_cast<uint32_t*>(base);
  l.pos = reinterpret_cast<uint32_t*>(base + 256);
  l.val = reinterpret_cast<float*>(base + 256 + 4 * kCollide);
  l.msg = reinterpret_cast<uint32_t*>(base + 256 + 8 * kCollide);
  return l;
}

__global__ __launch_bounds__(256) void k_gen_zero_lists(uint8_t* lists, uint64_t nb) {
  const uint64_t b = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (b < nb) *collide_list(lists, b).count = 0;
}

// STORE false: the counting pass; true: the storing pass.
template <bool STORE>
__global__ __launch_bounds__(256) void k_gen_walk(DecodeArgs a, float* acc, uint8_t* lists) {
  if (*a.status != 0) return;
  __shared__ StringRef ref;
  __shared__ uint32_t bad;
  const uint64_t b = blockIdx.x;
  const uint32_t k = blockIdx.y;
  if (threadIdx.x == 0) {
    StringRef mine;
    bad = open_string(a, k, b, true, mine) ? 0u : 1u;
    if (!bad) ref = mine;
  }
  __syncthreads();
  if (bad) {
    if (threadIdx.x == 0) flag_corrupt(a.status);
    return;
  }
  const StringRef sr = ref;
  const uint64_t base = b * (uint64_t)a.d;
  const uint64_t m = min((uint64_t)a.d, a.n - base);
  float* const out = acc + base;
  uint32_t* const outu = reinterpret_cast<uint32_t*>(out);
  const CollideList cl = collide_list(lists, b);
  for (uint64_t r = threadIdx.x; r <= sr.ents; r += blockDim.x) {
    uint64_t bitpos = r ? sr.list[2 * (r - 1)] : 32;
    uint64_t pos = r ? sr.list[2 * (r - 1) + 1] : 0;
    const bool last_stretch = r == sr.ents;
    const uint64_t stop = last_stretch ? sr.endbit : sr.list[2 * r];
    bool ok = bitpos >= 32 && bitpos <= stop && stop <= sr.endbit && pos <= m;
    ok = ok && walk_stretch(sr, stop, m, a.s, bitpos, pos,
                            [&](const uint64_t (&p)[kWalkBatch], const float (&v)[kWalkBatch]) {
      if (!STORE) {
#pragma unroll
        for (int t = 0; t < kWalkBatch; ++t)
          if (p[t] != ~0ull) atomicAdd(&outu[p[t]], 1u);
      } else {
        uint32_t c[kWalkBatch];
#pragma unroll
        for (int t = 0; t < kWalkBatch; ++t) c[t] = p[t] != ~0ull ? outu[p[t]] : 0u;
#pragma unroll
        for (int t = 0; t < kWalkBatch; ++t) {
          if (p[t] == ~0ull) continue;
          if (c[t] == 1u) {   // (only this record names the coordinate: nobody else touches it)
            out[p[t]] = v[t];
          } else {
            const uint32_t idx = atomicAdd(cl.count, 1u);
            if (idx < kCollide) {
              cl.pos[idx] = (uint32_t)p[t]; cl.val[idx] = v[t]; cl.msg[idx] = k;
            }
          }
        }
      }
    });
    // the stretch ends where the next one starts, at the position the list names
    if (ok && !last_stretch) ok = bitpos == stop && pos == sr.list[2 * r + 1];
    if (!ok) flag_corrupt(a.status);
  }
}

__global__ __launch_bounds__(1024) void k_gen_resolve(DecodeArgs a, float* acc, uint8_t* lists) {
  if (*a.status != 0) return;
  __shared__ uint32_t bad;
  __shared__ StringRef refs[QSGD_MAX_PEERS];
  __shared__ uint32_t lpos[kCollide];
  __shared__ float lval[kCollide];
  __shared__ uint8_t lk[kCollide];
  const uint64_t b = blockIdx.x;
  const uint64_t base = b * (uint64_t)a.d;
  const uint64_t m = min((uint64_t)a.d, a.n - base);
  float* const out = acc + base;
  const CollideList cl = collide_list(lists, b);
  const uint32_t L = *cl.count;
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  if (L > kCollide) {
    for (uint64_t p = threadIdx.x; p < m; p += blockDim.x) out[p] = 0.f;
    __syncthreads();
    if (!open_strings(a, b, refs, &bad) || !parse_in_turns(a, refs, m, out, &bad)) {
      if (threadIdx.x == 0) flag_corrupt(a.status);
    }
    return;
  }
  for (uint32_t e = threadIdx.x; e < L; e += blockDim.x) {
    lpos[e] = cl.pos[e]; lval[e] = cl.val[e]; lk[e] = (uint8_t)cl.msg[e];
  }
  __syncthreads();
  // (a message names a coordinate at most once: the terms of p are found in message order
  // by looking for the lowest message above the last one, terms + 1 scans of the list)
  for (uint32_t e = threadIdx.x; e < L; e += blockDim.x) {
    const uint32_t p = lpos[e];
    float sum = 0.f;
    int last = -1;
    for (;;) {
      uint32_t best = 0xFFFFFFFFu;
      float bestv = 0.f;
#pragma unroll 4
      for (uint32_t j = 0; j < L; ++j) {
        const uint32_t kj = lk[j];
        if (lpos[j] == p && (int)kj > last && kj < best) { best = kj; bestv = lval[j]; }
      }
      if (best == 0xFFFFFFFFu) break;
      if (last < 0 && best != lk[e]) break;   // another thread holds the lowest message: its job
      sum += bestv;
      last = (int)best;
    }
    if (last >= 0) out[p] = sum;
  }
}

__global__ __launch_bounds__(256) void k_gen_apply(DecodeArgs a, const float* acc) {
  if (*a.status != 0) return;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * 256)
    a.x[i] = a.step ? fmaf(-a.c, acc[i], a.x[i]) : a.x[i] + acc[i];
}

// Fixed width, any bucket size: one thread per coordinate, peers summed in order.
__global__ __launch_bounds__(256) void k_gen_decode_fixed(DecodeArgs a) {
  if (*a.status != 0) return;
  const uint32_t B = a.fixed_bits, fmask = (1u << B) - 1u;
  const float s_f = (float)a.s;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < a.n; i += (uint64_t)gridDim.x * 256) {
    const uint64_t b = i / (uint64_t)a.d;
    const uint64_t e = i - b * (uint64_t)a.d;
    const uint64_t m = min((uint64_t)a.d, a.n - b * (uint64_t)a.d);
    const uint64_t lw = (m * B + 31) >> 5, sw = (m + 31) >> 5;
    const uint64_t off = (uint64_t)H_WORDS + b * (uint64_t)a.fixed_words_full;
    float sum = 0.f;
    for (uint32_t k = 0; k < a.K; ++k) {
      if (off + 2 + lw + sw > a.msg_words[k]) { flag_corrupt(a.status); continue; }
      const uint32_t* str = a.msgs[k] + off;
      uint32_t z = (str[2 + ((e * B) >> 5)] >> ((e * B) & 31u)) & fmask;
      if (str[1] == (uint32_t)e) z = a.s;
      if (z > a.s) { flag_corrupt(a.status); z = 0; }
      const uint32_t neg = (str[2 + lw + (e >> 5)] >> (e & 31u)) & 1u;
      const float mag = (__uint_as_float(str[0]) / s_f) * (float)z;
      sum += (z && neg) ? -mag : mag;
    }
    a.x[i] = a.step ? fmaf(-a.c, sum, a.x[i]) : a.x[i] + sum;
  }
}

// ---- launchers -------------------------------------------------------------------------

hipError_t launch_gen_partial(const GenArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_partial, dim3((uint32_t)((a.nseg + 3) / 4)), dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_gen_scale(const GenArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_scale, dim3((uint32_t)((a.nb + 3) / 4)), dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_gen_encode(const GenArgs& a, bool aligned, hipStream_t st) {
  const dim3 grid((uint32_t)a.nseg), block(64);
  const size_t lds = 4 * ((size_t)a.sub_words + kRingWords);
#define QSGD_GEN(CODE)                                                                       \
  if (aligned) hipLaunchKernelGGL((k_gen_encode<CODE, true>), grid, block, lds, st, a);      \
  else hipLaunchKernelGGL((k_gen_encode<CODE, false>), grid, block, lds, st, a)
  if (a.code == QSGD_CODE_SPARSE) { QSGD_GEN(QSGD_CODE_SPARSE); }
  else if (a.code == QSGD_CODE_DENSE) { QSGD_GEN(QSGD_CODE_DENSE); }
  else { QSGD_GEN(QSGD_CODE_FIXED); }
#undef QSGD_GEN
  return hipGetLastError();
}
hipError_t launch_gen_scan(const GenArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_scan, dim3(1), dim3(1024), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_gen_fill(const GenArgs& a, uint32_t blocks, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_fill, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_gen_place(const GenArgs& a, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_place, dim3((uint32_t)a.nseg), dim3(64), 0, st, a);
  return hipGetLastError();
}
hipError_t launch_gen_zero(float* p, uint64_t n, uint32_t blocks, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_zero, dim3(blocks), dim3(256), 0, st, p, n);
  return hipGetLastError();
}
hipError_t launch_gen_parse(const DecodeArgs& a, float* acc, bool entries, hipStream_t st) {
  if (entries) {
    hipLaunchKernelGGL(k_gen_parse_entries, dim3(a.nb), dim3(256), 0, st, a, acc);
  } else {
    hipLaunchKernelGGL(k_gen_parse, dim3((a.nb + 255) / 256), dim3(256), 0, st, a, acc);
  }
  return hipGetLastError();
}
// lists: a.nb x kCollideBytes of workspace behind the accumulator.
hipError_t launch_gen_parse_together(const DecodeArgs& a, float* acc, uint8_t* lists,
                                     hipStream_t st) {
  hipLaunchKernelGGL(k_gen_zero_lists, dim3((a.nb + 255) / 256), dim3(256), 0, st, lists,
                     (uint64_t)a.nb);
  const dim3 grid(a.nb, a.K);
  hipLaunchKernelGGL((k_gen_walk<false>), grid, dim3(256), 0, st, a, acc, lists);
  hipLaunchKernelGGL((k_gen_walk<true>), grid, dim3(256), 0, st, a, acc, lists);
  hipLaunchKernelGGL(k_gen_resolve, dim3(a.nb), dim3(1024), 0, st, a, acc, lists);
  return hipGetLastError();
}
hipError_t launch_gen_apply(const DecodeArgs& a, const float* acc, uint32_t blocks, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_apply, dim3(blocks), dim3(256), 0, st, a, acc);
  return hipGetLastError();
}
hipError_t launch_gen_decode_fixed(const DecodeArgs& a, uint32_t blocks, hipStream_t st) {
  hipLaunchKernelGGL(k_gen_decode_fixed, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace qsgd
