// Device-side building blocks shared by the encode and decode kernels (gfx950,
// wave64).  Everything follows the definitions of the QSGD paper: the quantizer
// Q_s (Sec. 3.1, Eq. 2), the recursive Elias code (App. A.2, Definition) and the
// message layout documented in include/qsgd.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qsgd {

constexpr int kWave = 64;
constexpr int kChunk = 256;  // elements one wave covers per step: 64 lanes x float4

// ---- message header (16 words) ---------------------------------------------
constexpr uint32_t kMagic = 0x44475351u;  // 'QSGD'
enum HeaderWord : int {
  H_MAGIC = 0, H_VERSION, H_CODE, H_NORM, H_S, H_STREAM, H_D_LO, H_D_HI,
  H_N_LO, H_N_HI, H_NB_LO, H_NB_HI, H_PW_LO, H_PW_HI, H_STATUS, H_ITER, H_WORDS
};

// ---- Philox-4x32-10 (Salmon et al., SC'11): the rounding draws ----------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2,
                                              uint32_t c3, uint32_t k0, uint32_t k1,
                                              uint32_t out[4]) {
  // Keep the key schedule in two scalar registers per call (scalar adds per round)
  // instead of letting twenty precomputed round keys occupy scalar registers.
  asm volatile("" : "+s"(k0), "+s"(k1));
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    // three-input xor in one instruction (v_bitop3_b32, truth table 0x96)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// N blocks at once (counter words 0 and 1 per block, words 2 and 3 and the key shared): each
// round's key is stepped once for all of them.
template <int N>
__device__ __forceinline__ void philox4x32_10_xn(const uint32_t (&c0)[N], const uint32_t (&c1)[N],
                                                 uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1, uint32_t (*out)[4]) {
  asm volatile("" : "+s"(k0), "+s"(k1));
  uint32_t x0[N], x1[N], x2[N], x3[N];
#pragma unroll
  for (int i = 0; i < N; ++i) { x0[i] = c0[i]; x1[i] = c1[i]; x2[i] = c2; x3[i] = c3; }
#pragma unroll
  for (int r = 0; r < 10; ++r) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint64_t p0 = (uint64_t)0xD2511F53u * x0[i];
      const uint64_t p1 = (uint64_t)0xCD9E8D57u * x2[i];
      const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), x1[i], k0, 0x96);
      const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), x3[i], k1, 0x96);
      x1[i] = (uint32_t)p1; x3[i] = (uint32_t)p0; x0[i] = n0; x2[i] = n2;
    }
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
#pragma unroll
  for (int i = 0; i < N; ++i) { out[i][0] = x0[i]; out[i][1] = x1[i]; out[i][2] = x2[i]; out[i][3] = x3[i]; }
}

// The same block when c1, c2 and c3 are equal in all lanes (c0 is not).  Then the second
// product of round one and the first product of round two depend on wave-uniform values
// alone; stating that (readfirstlane) moves them to the scalar unit, two of the twenty
// 32 x 32 -> 64 bit multiplies, which are the expensive instructions here.
__device__ __forceinline__ void philox4x32_10_uniform(uint32_t c0, uint32_t c1, uint32_t c2,
                                                      uint32_t c3, uint32_t k0, uint32_t k1,
                                                      uint32_t out[4]) {
  asm volatile("" : "+s"(k0), "+s"(k1));
  c1 = __builtin_amdgcn_readfirstlane(c1);
  c2 = __builtin_amdgcn_readfirstlane(c2);
  c3 = __builtin_amdgcn_readfirstlane(c3);
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
    if (r == 0) n0 = __builtin_amdgcn_readfirstlane((uint32_t)(p1 >> 32) ^ c1 ^ k0);
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ---- Q_s on one coordinate (Eq. 2) ---------------------------------------------
// t = |v| * fl(s/scale) = a*s;  l = floor(t);  p = t - l;  level = l + [u < p],
// u = (word >> 8) * 2^-24;  t >= s (a = 1 up to rounding) gives the top level.
// quantize_unclamped leaves out the clamp: its result exceeds s (by one) only for t >= s.
// ts: t with the sign of the value (|v| * inv = |v * inv|, inv >= 0); the absolute value
// rides on the operands of the two instructions that read t instead of costing one of its own.
__device__ __forceinline__ uint32_t quantize_scaled(float ts, uint32_t word) {
  // t >= 0: the conversion truncates, which is floor(t) (saturating for huge or infinite
  // t), and the fraction instruction returns t - floor(t), exact and below 1
  const uint32_t l = (uint32_t)fabsf(ts);
  const float p = __builtin_amdgcn_fractf(fabsf(ts));
  const float u = (float)(word >> 8) * (1.0f / 16777216.0f);
  return l + ((u < p) ? 1u : 0u);
}

__device__ __forceinline__ uint32_t quantize_unclamped(float v, float inv, uint32_t word) {
  return quantize_scaled(v * inv, word);
}

__device__ __forceinline__ uint32_t quantize_one(float v, float inv, float s_f, uint32_t s,
                                                 uint32_t word) {
  // t >= s (a = 1 up to rounding) must give the top level: l + [u < p] >= s then
  return min(quantize_unclamped(v, inv, word), s);
}

// ---- recursive Elias code (App. A.2): a '0' at the end, binary groups in front ---
// Returns the code word right-aligned in `code` (first bit = most significant of
// the `len` low bits).  k >= 1, k < 2^32: len <= 43.
__device__ __forceinline__ void omega_encode(uint32_t k, uint64_t& code, uint32_t& len) {
  code = 0;
  len = 1;
  while (k > 1) {
    const uint32_t nb = 32u - (uint32_t)__clz(k);
    code |= (uint64_t)k << len;
    len += nb;
    k = nb - 1;
  }
}

__device__ __forceinline__ uint32_t omega_length(uint32_t k) {
  uint32_t len = 1;
  while (k > 1) {
    const uint32_t nb = 32u - (uint32_t)__clz(k);
    len += nb;
    k = nb - 1;
  }
  return len;
}

// ---- bit strings: stream bit j is bit 31-(j%32) of word j/32 --------------------
// ORs the `len` (1..64) low bits of `code` into zero-initialised LDS words so that
// the code's first bit lands on stream bit `bitoff`.
__device__ __forceinline__ void lds_emit(uint32_t* words, uint32_t bitoff, uint64_t code,
                                         uint32_t len) {
  const uint64_t top = code << (64u - len);
  const uint32_t w = bitoff >> 5, sh = bitoff & 31u;
  const uint64_t a = top >> sh;
  atomicOr(&words[w], (uint32_t)(a >> 32));
  if (sh + len > 32u) atomicOr(&words[w + 1], (uint32_t)a);
  if (sh + len > 64u) atomicOr(&words[w + 2], (uint32_t)top << (32u - sh));
}

// Same on global memory (words zero-initialised, shared by several writers).
__device__ __forceinline__ void global_emit(uint32_t* words, uint64_t bitoff, uint64_t code,
                                            uint32_t len) {
  const uint64_t top = code << (64u - len);
  const uint64_t w = bitoff >> 5;
  const uint32_t sh = (uint32_t)(bitoff & 31u);
  const uint64_t a = top >> sh;
  atomicOr(&words[w], (uint32_t)(a >> 32));
  if (sh + len > 32u) atomicOr(&words[w + 1], (uint32_t)a);
  if (sh + len > 64u) atomicOr(&words[w + 2], (uint32_t)top << (32u - sh));
}

// ---- streaming accesses ----------------------------------------------------------
// For data that is touched once (the gradient, x): the caches then keep what is
// touched again, such as message strings read piece by piece.
typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float* p) {
  const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float* p, const float4& x) {
  v4f v; v.x = x.x; v.y = x.y; v.z = x.z; v.w = x.w;
  __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
}

// ---- wavefront helpers ----------------------------------------------------------
// Cross-lane data movement uses DPP modifiers (row shifts inside rows of 16 lanes,
// then broadcasts of lane 15 / lane 31 into the following rows): one VALU
// instruction per step and no LDS traffic.  Lanes without a source read 0, which
// is the identity of every combination used here (sums, max of magnitudes).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_fetch(uint32_t v) {
  // all rows written: lanes without a source read 0 by themselves (bound_ctrl), so no
  // register has to be cleared for them first
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, ROW_MASK == 0xf);
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_fetch_or(uint32_t other, uint32_t v) {  // `other` where no source
  return (uint32_t)__builtin_amdgcn_update_dpp((int)other, (int)v, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppShl1 = 0x101, kDppShl2 = 0x102, kDppShl4 = 0x104;  // lane l reads lane l+k of its row
constexpr int kDppShr1 = 0x111, kDppShr2 = 0x112, kDppShr4 = 0x114, kDppShr8 = 0x118;
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_fetch_f64(double v) {
  const uint32_t lo = dpp_fetch<CTRL, ROW_MASK>((uint32_t)__double2loint(v));
  const uint32_t hi = dpp_fetch<CTRL, ROW_MASK>((uint32_t)__double2hiint(v));
  return __hiloint2double((int)hi, (int)lo);
}

// Sum over the 64 lanes, the same value returned to every lane.
__device__ __forceinline__ double wave_sum_f64(double v) {
  v += dpp_fetch_f64<kDppShr1, 0xf>(v);
  v += dpp_fetch_f64<kDppShr2, 0xf>(v);
  v += dpp_fetch_f64<kDppShr4, 0xf>(v);
  v += dpp_fetch_f64<kDppShr8, 0xf>(v);
  v += dpp_fetch_f64<kDppBcast15, 0xa>(v);
  v += dpp_fetch_f64<kDppBcast31, 0xc>(v);
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
  return __hiloint2double(hi, lo);
}

// Max over the 64 lanes of non-negative values.
__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, __uint_as_float(dpp_fetch<kDppShr1, 0xf>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_fetch<kDppShr2, 0xf>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_fetch<kDppShr4, 0xf>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_fetch<kDppShr8, 0xf>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_fetch<kDppBcast15, 0xa>(__float_as_uint(v))));
  v = fmaxf(v, __uint_as_float(dpp_fetch<kDppBcast31, 0xc>(__float_as_uint(v))));
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), 63));
}

// Min over the 64 lanes, returned to every lane.
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
  v = min(v, dpp_fetch_or<kDppShr1, 0xf>(0xFFFFFFFFu, v));
  v = min(v, dpp_fetch_or<kDppShr2, 0xf>(0xFFFFFFFFu, v));
  v = min(v, dpp_fetch_or<kDppShr4, 0xf>(0xFFFFFFFFu, v));
  v = min(v, dpp_fetch_or<kDppShr8, 0xf>(0xFFFFFFFFu, v));
  v = min(v, dpp_fetch_or<kDppBcast15, 0xa>(0xFFFFFFFFu, v));
  v = min(v, dpp_fetch_or<kDppBcast31, 0xc>(0xFFFFFFFFu, v));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Max over the 64 lanes, returned to every lane.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = max(v, dpp_fetch<kDppShr1, 0xf>(v));
  v = max(v, dpp_fetch<kDppShr2, 0xf>(v));
  v = max(v, dpp_fetch<kDppShr4, 0xf>(v));
  v = max(v, dpp_fetch<kDppShr8, 0xf>(v));
  v = max(v, dpp_fetch<kDppBcast15, 0xa>(v));
  v = max(v, dpp_fetch<kDppBcast31, 0xc>(v));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, int /*lane*/) {
  v += dpp_fetch<kDppShr1, 0xf>(v);
  v += dpp_fetch<kDppShr2, 0xf>(v);
  v += dpp_fetch<kDppShr4, 0xf>(v);
  v += dpp_fetch<kDppShr8, 0xf>(v);
  v += dpp_fetch<kDppBcast15, 0xa>(v);
  v += dpp_fetch<kDppBcast31, 0xc>(v);
  return v;
}

__device__ __forceinline__ uint32_t lane_bcast(uint32_t v, int src) {
  return (uint32_t)__builtin_amdgcn_readlane((int)v, src);
}

// Records "a message did not parse / did not match" in a status word.
__device__ __forceinline__ void flag_corrupt(uint32_t* status) {
  atomicExch(status, 0xFFFFFFFDu);  // QSGD_ERR_CORRUPT (-3)
}

// Width of the fixed-width level field: narrowest of 2/4/8/16 bits holding
// 0..s-1 (L2 scale: level s goes to the bucket's escape word) or 0..s (max scale).
__host__ __device__ inline uint32_t fixed_field_bits(uint32_t s, uint32_t norm_mode) {
  const uint32_t need = norm_mode ? s + 1u : s;
  uint32_t B = 2;
  while (B < 16 && (1u << B) < need) B *= 2;
  return B;
}

}  // namespace qsgd
