// Device-side helpers shared by the gfx950 kernels: vector types, streaming loads and stores,
// wavefront reductions, the counter-based Gaussian generator and the one rounding order of the
// CECA combine.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ceca {

typedef float vf4 __attribute__((ext_vector_type(4)));

template <int VEC> struct VecOf;
template <> struct VecOf<4> { using T = vf4; };
template <> struct VecOf<1> { using T = float; };

// State rows are touched once per round: stream them past the caches (nontemporal loads and stores).
template <typename V> __device__ __forceinline__ V ld_stream(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
}
template <typename V> __device__ __forceinline__ void st_stream(float* p, V v) {
  __builtin_nontemporal_store(v, reinterpret_cast<V*>(p));
}
template <typename V> __device__ __forceinline__ V ld_plain(const float* p) {
  return *reinterpret_cast<const V*>(p);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over the 64 lanes of a wavefront with data-parallel-primitive adds (no LDS traffic): pairs and
// quads by quad permutes, rows of 16 by the two row mirrors, then the last lane of row 0 into row 1
// and of row 2 into row 3, then lane 31 into rows 2 and 3.  Lane 63 ends up with the complete sum.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, false);
  return v + __builtin_bit_cast(float, moved);     // rows outside ROW_MASK receive +0
}
__device__ __forceinline__ float wave_sum_to_lane63(float v) {
  v = dpp_add<0xB1, 0xf>(v);    // quad_perm [1, 0, 3, 2]
  v = dpp_add<0x4E, 0xf>(v);    // quad_perm [2, 3, 0, 1]
  v = dpp_add<0x141, 0xf>(v);   // row_half_mirror
  v = dpp_add<0x140, 0xf>(v);   // row_mirror
  v = dpp_add<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v = dpp_add<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}
// Sums N per-lane values across the wavefront.  On return lane l < N holds the complete sum of value
// number `which` = l.  Every index is a compile-time constant, so the values stay in registers.
template <int N>
__device__ __forceinline__ float wave_sum_many(const float (&m)[N], int lane, int& which) {
  static_assert(N >= 1 && N <= 64, "one lane per value");
  float mine = 0.0f;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const float total = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wave_sum_to_lane63(m[k])), 63));
    mine = (lane == k) ? total : mine;
  }
  which = lane;
  return mine;
}

__device__ __forceinline__ float dot_v(vf4 a, vf4 b) { return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w; }
__device__ __forceinline__ float dot_v(float a, float b) { return a * b; }

// ---------------------------------------------------------------------------------------------
// Counter-based Gaussian noise (definition in ceca.h): one 32-bit word per uniform, Box-Muller
// on column pairs.  Transcendentals use the hardware's log2 / sin / cos (arguments in turns).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t mix32(uint32_t h) {
  h ^= h >> 16; h *= 0x7feb352du;
  h ^= h >> 15; h *= 0x846ca68bu;
  h ^= h >> 16;
  return h;
}
__device__ __forceinline__ uint32_t noise_word(uint32_t c, uint32_t k0, uint32_t k1) {
  uint32_t h = c ^ k0;
  h ^= h >> 16; h *= 0x7feb352du;
  h ^= h >> 15; h += k1; h *= 0x846ca68bu;
  h ^= h >> 16;
  return h;
}
struct NoiseKeys { uint32_t k0, k1; };
__device__ __forceinline__ NoiseKeys noise_keys(uint32_t seed, uint32_t k, uint32_t agent) {
  NoiseKeys nk;
  nk.k0 = mix32(mix32(seed + 0x9e3779b9u * k) ^ agent);
  nk.k1 = mix32(nk.k0 + 0x85ebca6bu);
  return nk;
}
__device__ __forceinline__ void normal_pair(uint32_t q, NoiseKeys nk, float& e0, float& e1) {
  const uint32_t w1 = noise_word(2u * q, nk.k0, nk.k1);
  const uint32_t w2 = noise_word(2u * q + 1u, nk.k0, nk.k1);
  const float u1 = (float)((w1 >> 8) + 1u) * 0x1p-24f;   // (0, 1], exact in fp32
  const float u2 = (float)(w2 >> 8) * 0x1p-24f;          // [0, 1), exact in fp32
  // -2 ln u1 = (-2 ln 2) log2 u1
  const float rad = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u1));
  e0 = rad * __builtin_amdgcn_cosf(u2);
  e1 = rad * __builtin_amdgcn_sinf(u2);
}
template <typename V> __device__ __forceinline__ V noise_group(int64_t col, NoiseKeys nk);
template <> __device__ __forceinline__ vf4 noise_group<vf4>(int64_t col, NoiseKeys nk) {
  vf4 e;
  float a, b;
  const uint32_t q = (uint32_t)(col >> 1);     // col is a multiple of 4 on this path
  normal_pair(q, nk, a, b);
  e.x = a; e.y = b;
  normal_pair(q + 1u, nk, a, b);
  e.z = a; e.w = b;
  return e;
}
template <> __device__ __forceinline__ float noise_group<float>(int64_t col, NoiseKeys nk) {
  float a, b;
  normal_pair((uint32_t)(col >> 1), nk, a, b);
  return (col & 1) ? b : a;
}

// w * self + wp * msg, with one fixed rounding order wherever it is evaluated.
__device__ __forceinline__ float combine(float w, float self, float wp, float msg) {
#pragma clang fp contract(off)
  const float t = wp * msg;
  return __builtin_fmaf(w, self, t);
}
__device__ __forceinline__ vf4 combine(float w, vf4 self, float wp, vf4 msg) {
  vf4 o;
  o.x = combine(w, self.x, wp, msg.x); o.y = combine(w, self.y, wp, msg.y);
  o.z = combine(w, self.z, wp, msg.z); o.w = combine(w, self.w, wp, msg.w);
  return o;
}

}  // namespace ceca
