// Raw section of tensor-aware messages (Sec. 5, "Protocol": matrices with fewer
// than 10K elements are not quantized).  The small tensors of the arena travel as
// fp32 words after the bucket strings, in tensor order.  One workgroup per piece of
// kRawPiece values, four values per thread.
#include "qsgd_device.hpp"
#include "qsgd_kernels.hpp"

namespace qsgd {

// Encode side: copies the small tensors behind the strings.  Runs after the
// kernels that fix the length of the strings (the table's last entry).
__global__ __launch_bounds__(256) void k_raw_pack(RawArgs a) {
  if (a.header[H_STATUS] != 0) return;   // the strings did not fit: nothing more to write
  const uint64_t strings = a.table ? (uint64_t)a.table[a.nb] : a.fixed_strings;
  if (strings + a.raw_words > a.cap_words) return;
  const uint4 e = a.rtab[blockIdx.x];
  const float* __restrict__ src = a.g + (uint64_t)e.x * 4u;
  uint32_t* __restrict__ dst = a.payload + strings + e.z;
  const uint32_t i = threadIdx.x * 4u;
  if (i + 3 < e.y) {
    const float4 v = *reinterpret_cast<const float4*>(src + i);   // tensors start at 16-byte multiples
    dst[i] = __float_as_uint(v.x); dst[i + 1] = __float_as_uint(v.y);
    dst[i + 2] = __float_as_uint(v.z); dst[i + 3] = __float_as_uint(v.w);
  } else {
    for (uint32_t j = i; j < e.y; ++j) dst[j] = __float_as_uint(src[j]);
  }
}

// Decode side: x_i <- x_i + sum_l raw_l[i]  or  x_i <- fma(-c, sum_l raw_l[i], x_i),
// the sum over the messages in ascending order.
__global__ __launch_bounds__(256) void k_raw_apply(DecodeArgs a, RawArgs r) {
  if (*a.status != 0) return;
  __shared__ uint64_t base[QSGD_MAX_PEERS];   // word index of the raw section in message k
  __shared__ uint32_t bad;
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  if (threadIdx.x < a.K) {
    const uint32_t k = threadIdx.x;
    const uint32_t* h = a.msgs[k];
    const uint64_t pay = (uint64_t)H_WORDS + a.table_words;
    const uint64_t strings = a.table_words ? (uint64_t)h[H_WORDS + a.nb] : r.fixed_strings;
    const uint64_t pw = h[H_PW_LO] | ((uint64_t)h[H_PW_HI] << 32);
    if (strings + r.raw_words != pw || pay + pw > a.msg_words[k]) bad = 1;
    base[k] = pay + strings;
  }
  __syncthreads();
  if (bad) {
    if (threadIdx.x == 0) flag_corrupt(a.status);
    return;
  }
  const uint4 e = r.rtab[blockIdx.x];
  float* __restrict__ x = a.x + (uint64_t)e.x * 4u;
  const uint32_t i0 = threadIdx.x * 4u;
  if (i0 >= e.y) return;
  const uint32_t cnt = min(4u, e.y - i0);
  float sum[4] = {0.f, 0.f, 0.f, 0.f};
  for (uint32_t k0 = 0; k0 < a.K; k0 += 4) {   // four messages' words in flight, summed in order
    float w[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t k = min(k0 + (uint32_t)t, a.K - 1u);
      const uint32_t* __restrict__ src = a.msgs[k] + base[k] + e.z + i0;
#pragma unroll
      for (int j = 0; j < 4; ++j) w[t][j] = (uint32_t)j < cnt ? __uint_as_float(src[j]) : 0.f;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (k0 + (uint32_t)t < a.K) {
#pragma unroll
        for (int j = 0; j < 4; ++j) sum[j] += w[t][j];
      }
    }
  }
  for (uint32_t j = 0; j < cnt; ++j)
    x[i0 + j] = a.step ? fmaf(-a.c, sum[j], x[i0 + j]) : x[i0 + j] + sum[j];
}

// Header (and empty offset table) of a message whose tensors all travel raw.
__global__ void k_write_layout_header(uint32_t* header, uint32_t* table, uint32_t code,
                                      uint32_t norm, uint32_t s, uint64_t d, uint64_t n,
                                      uint64_t raw_words, uint32_t stream_id,
                                      uint32_t iteration) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    header[H_MAGIC] = kMagic; header[H_VERSION] = 2; header[H_CODE] = code;
    header[H_NORM] = norm; header[H_S] = s; header[H_STREAM] = stream_id;
    header[H_D_LO] = (uint32_t)d; header[H_D_HI] = (uint32_t)(d >> 32);
    header[H_N_LO] = (uint32_t)n; header[H_N_HI] = (uint32_t)(n >> 32);
    header[H_NB_LO] = 0; header[H_NB_HI] = 0;
    header[H_PW_LO] = (uint32_t)raw_words; header[H_PW_HI] = (uint32_t)(raw_words >> 32);
    header[H_STATUS] = 0; header[H_ITER] = iteration;
    if (table) { table[0] = 0; table[1] = 0; table[2] = 0; table[3] = 0; }
  }
}

hipError_t launch_write_layout_header(uint32_t* header, uint32_t* table, uint32_t code,
                                      uint32_t norm, uint32_t s, uint64_t d, uint64_t n,
                                      uint64_t raw_words, uint32_t stream_id, uint32_t iteration,
                                      hipStream_t st) {
  hipLaunchKernelGGL(k_write_layout_header, dim3(1), dim3(64), 0, st, header, table, code, norm,
                     s, d, n, raw_words, stream_id, iteration);
  return hipGetLastError();
}

hipError_t launch_raw_pack(const RawArgs& a, hipStream_t st) {
  if (a.R == 0) return hipSuccess;
  hipLaunchKernelGGL(k_raw_pack, dim3(a.R), dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_raw_apply(const DecodeArgs& a, const RawArgs& r, hipStream_t st) {
  if (r.R == 0) return hipSuccess;
  hipLaunchKernelGGL(k_raw_apply, dim3(r.R), dim3(256), 0, st, a, r);
  return hipGetLastError();
}

}  // namespace qsgd
