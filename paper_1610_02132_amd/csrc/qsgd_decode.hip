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
// small per-string queues in LDS and are applied to an LDS accumulator message
// by message (k ascending), so the fp32 sum has one fixed order; then the
// accumulator is streamed against x with float4 accesses.
#include "qsgd_device.hpp"
#include "qsgd_kernels.hpp"

namespace qsgd {

namespace {

__device__ __forceinline__ void flag_corrupt(uint32_t* status) {
  atomicExch(status, (uint32_t)QSGD_ERR_CORRUPT);
}

// MSB-first bit reader over words [0, nwords) of one string; past the end it
// supplies zeros and never touches memory.
struct BitReader {
  const uint32_t* w;
  uint32_t nwords, widx;
  uint64_t buf;       // next bits, most significant first
  uint32_t avail;     // valid bits in buf (kept above 32)
  uint32_t consumed;  // stream position of the next bit

  __device__ __forceinline__ void refill() {
    while (avail <= 32u) {
      const uint32_t nw = (widx < nwords) ? w[widx] : 0u;
      ++widx;
      buf |= (uint64_t)nw << (32u - avail);
      avail += 32u;
    }
  }
  __device__ __forceinline__ void init(const uint32_t* words, uint32_t n, uint32_t first_word) {
    w = words; nwords = n; widx = first_word; buf = 0; avail = 0;
    consumed = first_word * 32u;
    refill();
  }
  __device__ __forceinline__ uint32_t take(uint32_t nbits) {  // 1..32
    const uint32_t v = (uint32_t)(buf >> (64u - nbits));
    buf <<= nbits;
    avail -= nbits;
    consumed += nbits;
    refill();
    return v;
  }
  // Decoder rule of the recursive Elias code (App. A.2): N = 1; a 0 bit outputs N;
  // a 1 bit opens an (N+1)-bit group whose value is the new N.  0 = malformed.
  __device__ __forceinline__ uint32_t omega() {
    uint32_t N = 1;
    for (;;) {
      if ((buf >> 63) == 0) { take(1); return N; }
      if (N > 31u) return 0;
      N = take(N + 1u);
    }
  }
};

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
    ok = h[H_MAGIC] == kMagic && h[H_VERSION] == 1 && h[H_CODE] == a.code &&
         h[H_NORM] == a.norm_mode && h[H_S] == a.s && h[H_D_LO] == a.d && h[H_D_HI] == 0 &&
         h[H_N_LO] == (uint32_t)a.n && h[H_N_HI] == (uint32_t)(a.n >> 32) &&
         h[H_NB_LO] == a.nb && h[H_NB_HI] == 0 && h[H_STATUS] == 0 &&
         (uint64_t)H_WORDS + a.table_words + pw <= a.msg_words[k];
  }
  if (!ok) flag_corrupt(a.status);
}

// ---- fixed width: one wavefront per bucket ----------------------------------------
__global__ __launch_bounds__(256) void k_decode_fixed(DecodeArgs a) {
  if (*a.status != 0) return;
  const int lane = threadIdx.x & 63;
  const uint32_t wave_global = blockIdx.x * 4 + (threadIdx.x >> 6);
  const uint32_t wave_count = gridDim.x * 4;
  const uint32_t B = a.fixed_bits, s = a.s;
  const float s_f = (float)s;
  const uint32_t fmask = (1u << B) - 1u;

  for (uint32_t b = wave_global; b < a.nb; b += wave_count) {
    const uint64_t base = (uint64_t)b * a.d;
    const uint32_t m = (uint32_t)min((uint64_t)a.d, a.n - base);
    const uint32_t lw = (m * B + 31u) >> 5, sw = (m + 31u) >> 5;
    const uint64_t str_off = (uint64_t)H_WORDS + (uint64_t)b * a.fixed_words_full;
    // lane k < K holds the scale and the escape index of message k's string
    float my_scale = 0.f;
    uint32_t my_esc = 0xFFFFFFFFu, my_ok = 0;
    if ((uint32_t)lane < a.K) {
      if (str_off + 2u + lw + sw <= a.msg_words[lane]) {
        const uint32_t* str = a.msgs[lane] + str_off;
        my_scale = __uint_as_float(str[0]) / s_f;
        my_esc = str[1];
        my_ok = 1;
        if (my_esc != 0xFFFFFFFFu && my_esc >= m) { my_ok = 0; }
      }
      if (!my_ok) flag_corrupt(a.status);
    }
    for (uint32_t e0 = lane * 4; e0 < m; e0 += kChunk) {
      float acc[4] = {0.f, 0.f, 0.f, 0.f};
      for (uint32_t k = 0; k < a.K; ++k) {
        if (!lane_bcast(my_ok, k)) continue;
        const float sc = __uint_as_float(lane_bcast(__float_as_uint(my_scale), k));
        const uint32_t esc = lane_bcast(my_esc, k);
        const uint32_t* lplane = a.msgs[k] + str_off + 2;
        const uint32_t* splane = lplane + lw;
        uint32_t z[4];
        if (B == 8) {
          const uint32_t w = lplane[e0 >> 2];
          z[0] = w & 0xFFu; z[1] = (w >> 8) & 0xFFu; z[2] = (w >> 16) & 0xFFu; z[3] = w >> 24;
        } else if (B == 16) {
          const uint32_t w0 = lplane[e0 >> 1];
          const uint32_t w1 = ((e0 >> 1) + 1 < lw) ? lplane[(e0 >> 1) + 1] : 0u;
          z[0] = w0 & 0xFFFFu; z[1] = w0 >> 16; z[2] = w1 & 0xFFFFu; z[3] = w1 >> 16;
        } else {
          const uint32_t w = lplane[(e0 * B) >> 5] >> ((e0 * B) & 31u);
          z[0] = w & fmask; z[1] = (w >> B) & fmask; z[2] = (w >> (2 * B)) & fmask;
          z[3] = (w >> (3 * B)) & fmask;
        }
        const uint32_t sg = splane[e0 >> 5] >> (e0 & 31u);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (esc == e0 + j) z[j] = s;
        bool bad = false;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (e0 + j < m) {
            bad |= z[j] > s;
            const float mag = sc * (float)z[j];
            acc[j] += (z[j] != 0 && ((sg >> j) & 1u)) ? -mag : mag;
          }
        }
        if (bad) flag_corrupt(a.status);
      }
      float* xp = a.x + base + e0;
      if (e0 + 3 < m) {
        float4 xv = *reinterpret_cast<float4*>(xp);
        if (a.step) {
          xv.x = fmaf(-a.c, acc[0], xv.x); xv.y = fmaf(-a.c, acc[1], xv.y);
          xv.z = fmaf(-a.c, acc[2], xv.z); xv.w = fmaf(-a.c, acc[3], xv.w);
        } else {
          xv.x += acc[0]; xv.y += acc[1]; xv.z += acc[2]; xv.w += acc[3];
        }
        *reinterpret_cast<float4*>(xp) = xv;
      } else {
        for (int j = 0; j < 4; ++j)
          if (e0 + j < m) xp[j] = a.step ? fmaf(-a.c, acc[j], xp[j]) : xp[j] + acc[j];
      }
    }
  }
}

// ---- Elias codes: one lane per string, gw buckets x K messages per wavefront -------
__global__ __launch_bounds__(64) void k_decode_elias(DecodeArgs a) {
  if (*a.status != 0) return;
  extern __shared__ uint32_t smem[];
  // LDS: [acc: gw*win floats][queues: 64*rec words][counts: 64][scales: 64]
  float* const acc = reinterpret_cast<float*>(smem);
  uint32_t* const queue = smem + a.gw * a.win;
  uint32_t* const counts = queue + 64u * a.rec;
  float* const scales = reinterpret_cast<float*>(counts + 64);

  const int lane = threadIdx.x;
  const uint32_t K = a.K, gw = a.gw, win = a.win, rec = a.rec, s = a.s;
  const bool sparse = a.code == QSGD_CODE_SPARSE;
  const uint32_t b0 = blockIdx.x * gw;

  // ---- open this lane's string -----------------------------------------------------
  const uint32_t g = lane / K, k = lane - g * K;
  const uint32_t b = b0 + g;
  bool have = false;      // a decoded record is waiting in (pend_pos, pend_lev, pend_neg)
  uint32_t m = 0;         // elements in this lane's bucket
  uint32_t endbit = 0;    // sparse: records end here
  uint32_t pend_pos = 0, pend_lev = 0, pend_neg = 0;  // pend_pos is 1-based
  BitReader rd;
  rd.init(nullptr, 0, 0);
  bool open = false;
  if (g < gw && b < a.nb) {
    m = (uint32_t)min((uint64_t)a.d, a.n - (uint64_t)b * a.d);
    const uint32_t* msg = a.msgs[k];
    const uint32_t o0 = msg[H_WORDS + b], o1 = msg[H_WORDS + b + 1];
    const uint64_t pay = (uint64_t)H_WORDS + a.table_words;
    if (o0 < o1 && pay + o1 <= a.msg_words[k]) {
      const uint32_t* str = msg + pay + o0;
      const uint32_t nwords = o1 - o0;
      scales[lane] = __uint_as_float(str[0]) / (float)s;
      open = true;
      if (sparse) {
        const uint32_t last = str[nwords - 1];
        endbit = nwords * 32u - 1u - (uint32_t)(__ffs((int)last) - 1);
        if (last == 0 || endbit < 32u) open = false;
      } else {
        endbit = nwords * 32u;
      }
      if (open) rd.init(str, nwords, 1);
    }
    if (!open) flag_corrupt(a.status);
  }
  if (!open) scales[lane] = 0.f;

  // Reads the next record into pend_*; clears `have` at the end of the string.
  auto advance = [&]() {
    if (sparse) {
      if (rd.consumed >= endbit) { have = false; return; }
      const uint32_t gap = rd.omega();
      pend_neg = rd.take(1);
      const uint32_t lev = rd.omega();
      pend_pos += gap;
      pend_lev = lev;
      if (gap == 0 || lev == 0 || lev > s || pend_pos > m || rd.consumed > endbit) {
        flag_corrupt(a.status);
        have = false;
      }
    } else {
      if (pend_pos >= m) { have = false; return; }
      pend_neg = rd.take(1);
      const uint32_t lev1 = rd.omega();
      pend_pos += 1;
      pend_lev = lev1 - 1u;
      if (lev1 == 0 || lev1 > s + 1u || rd.consumed > endbit) {
        flag_corrupt(a.status);
        have = false;
      }
    }
  };
  if (open) { have = true; advance(); }

  for (uint32_t j = lane; j < gw * win; j += 64) acc[j] = 0.f;
  __syncthreads();

  for (uint32_t ws = 0; ws < a.d; ws += win) {
    const uint32_t wend = ws + win;  // records with pend_pos <= wend fall in this window
    // ---- rounds: fill the queues, then apply them message by message --------------
    // A round may only apply positions that EVERY string has already queued up
    // to, or an element could receive message 5's term before message 2's.  The
    // limit is the smallest position some full queue still has pending, minus 1;
    // queued records past it stay in the queue for the next round.
    uint32_t cnt = 0;
    for (;;) {
      while (have && pend_pos <= wend && cnt < rec) {
        if (pend_lev)
          queue[lane * rec + cnt++] = (pend_pos - 1u - ws) | (pend_neg << 12) | (pend_lev << 13);
        advance();
      }
      const bool more = have && pend_pos <= wend;  // stopped on a full queue
      uint32_t limit = more ? pend_pos - 1u : wend;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) limit = min(limit, (uint32_t)__shfl_xor((int)limit, o, kWave));
      const uint32_t rel_limit = limit - ws;  // window-relative positions below this are due
      counts[lane] = cnt;
      __syncthreads();
      const uint32_t g2 = lane / rec, r = lane - g2 * rec;
      for (uint32_t kk = 0; kk < K; ++kk) {
        if (g2 < gw) {
          const uint32_t sl = g2 * K + kk;
          if (r < counts[sl]) {
            const uint32_t q = queue[sl * rec + r];
            if ((q & 0xFFFu) < rel_limit) {
              const float mag = scales[sl] * (float)(q >> 13);
              acc[g2 * win + (q & 0xFFFu)] += ((q >> 12) & 1u) ? -mag : mag;
            }
          }
        }
        __syncthreads();
      }
      // keep what was not due yet at the front of the queue
      if (limit == wend) {
        cnt = 0;
      } else {
        uint32_t done = 0;
        while (done < cnt && (queue[lane * rec + done] & 0xFFFu) < rel_limit) ++done;
        for (uint32_t i = done; i < cnt; ++i) queue[lane * rec + i - done] = queue[lane * rec + i];
        cnt -= done;
      }
      if (__ballot(more || cnt != 0) == 0) break;
    }
    // ---- stream the window against x -------------------------------------------------
    for (uint32_t gg = 0; gg < gw; ++gg) {
      const uint32_t bb = b0 + gg;
      if (bb >= a.nb) break;
      const uint64_t base = (uint64_t)bb * a.d;
      const uint32_t mb = (uint32_t)min((uint64_t)a.d, a.n - base);
      if (ws >= mb) continue;
      const uint32_t cntw = min(win, mb - ws);
      float* xw = a.x + base + ws;
      float* aw = acc + gg * win;
      for (uint32_t i = lane * 4; i < cntw; i += kChunk) {
        if (i + 3 < cntw) {
          const float4 av = *reinterpret_cast<float4*>(aw + i);
          *reinterpret_cast<float4*>(aw + i) = make_float4(0.f, 0.f, 0.f, 0.f);
          float4 xv = *reinterpret_cast<float4*>(xw + i);
          if (a.step) {
            xv.x = fmaf(-a.c, av.x, xv.x); xv.y = fmaf(-a.c, av.y, xv.y);
            xv.z = fmaf(-a.c, av.z, xv.z); xv.w = fmaf(-a.c, av.w, xv.w);
          } else {
            xv.x += av.x; xv.y += av.y; xv.z += av.z; xv.w += av.w;
          }
          *reinterpret_cast<float4*>(xw + i) = xv;
        } else {
          for (uint32_t j = i; j < cntw; ++j) {
            const float av = aw[j];
            aw[j] = 0.f;
            xw[j] = a.step ? fmaf(-a.c, av, xw[j]) : xw[j] + av;
          }
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

hipError_t launch_decode_fixed(const DecodeArgs& a, uint32_t blocks, hipStream_t st) {
  hipLaunchKernelGGL(k_decode_fixed, dim3(blocks), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_decode_elias(const DecodeArgs& a, uint32_t blocks, size_t lds, hipStream_t st) {
  hipLaunchKernelGGL(k_decode_elias, dim3(blocks), dim3(64), lds, st, a);
  return hipGetLastError();
}

}  // namespace qsgd
