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
// v + (v of lane ^ XOR).  Distances 1 and 2 are quad permutes on the data-parallel-primitive path (no
// LDS traffic); 4, 8 and 16 are swizzles inside each half of the wavefront; 32 is a lane exchange.
template <int XOR>
__device__ __forceinline__ float xor_add(float v) {
  const int bits = __builtin_bit_cast(int, v);
  int moved;
  if constexpr (XOR == 1) moved = __builtin_amdgcn_update_dpp(0, bits, 0xB1, 0xf, 0xf, false);        // quad_perm [1, 0, 3, 2]
  else if constexpr (XOR == 2) moved = __builtin_amdgcn_update_dpp(0, bits, 0x4E, 0xf, 0xf, false);   // quad_perm [2, 3, 0, 1]
  else if constexpr (XOR == 32) moved = __shfl_xor(bits, 32, 64);
  else moved = __builtin_amdgcn_ds_swizzle(bits, (XOR << 10) | 0x1f);                                  // xor mask, all lanes kept
  return v + __builtin_bit_cast(float, moved);
}
// One level of the halving butterfly below: every lane adds its partner's copy of each of the 2H values
// it still carries, then keeps the H values that belong to its side (`up`); with one value left (H = 0)
// both partners keep the pair sum.
template <int XOR, int H>
__device__ __forceinline__ void halve(float (&m)[16], bool up) {
  if constexpr (H >= 1) {
    float s[2 * H];
#pragma unroll
    for (int k = 0; k < 2 * H; ++k) s[k] = xor_add<XOR>(m[k]);
#pragma unroll
    for (int k = 0; k < H; ++k) m[k] = up ? s[k + H] : s[k];
  } else {
    m[0] = xor_add<XOR>(m[0]);
  }
}
// Sums N <= 16 per-lane values (N a power of two) across the 64 lanes of a wavefront.  The level with
// partner distance 2^t halves the number of values a lane carries while there is more than one (the
// partner sits on the other side of lane bit t and carries the same values), so N values cost about
// 2N adds instead of 6N.  On return lane l < N holds the complete sum of value number `which`.
// All array indices are compile-time constants: the values stay in registers.
template <int N>
__device__ __forceinline__ float wave_sum_many(const float (&in)[N], int lane, int& which) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16, "N must be a power of two up to 16");
  float m[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) m[k] = in[k < N ? k : 0];
  const bool u0 = lane & 1, u1 = lane & 2, u2 = lane & 4, u3 = lane & 8;
  halve<1, N / 2>(m, u0);
  halve<2, N / 4>(m, u1);
  halve<4, N / 8>(m, u2);
  halve<8, N / 16>(m, u3);
  which = (N >= 2 && u0 ? N / 2 : 0) + (N >= 4 && u1 ? N / 4 : 0) + (N >= 8 && u2 ? N / 8 : 0) + (N >= 16 && u3 ? 1 : 0);
  return xor_add<32>(xor_add<16>(m[0]));
}

// The 32-bit word of lane ^ XOR (XOR a power of two below 64): quad permutes for 1 and 2, swizzles inside
// each half of the wavefront for 4, 8 and 16, a lane exchange for 32.
template <int XOR>
__device__ __forceinline__ int xor_lane(int bits) {
  if constexpr (XOR == 1) return __builtin_amdgcn_update_dpp(0, bits, 0xB1, 0xf, 0xf, false);        // quad_perm [1, 0, 3, 2]
  else if constexpr (XOR == 2) return __builtin_amdgcn_update_dpp(0, bits, 0x4E, 0xf, 0xf, false);   // quad_perm [2, 3, 0, 1]
  else if constexpr (XOR == 32) return __shfl_xor(bits, 32, 64);
  else return __builtin_amdgcn_ds_swizzle(bits, (XOR << 10) | 0x1f);                                  // xor mask, all lanes kept
}
// The double that lane ^ XOR holds.
template <int XOR>
__device__ __forceinline__ double xor_lane(double v) {
  const int lo = xor_lane<XOR>(__double2loint(v));
  const int hi = xor_lane<XOR>(__double2hiint(v));
  return __hiloint2double(hi, lo);
}
// One level of a halving butterfly over doubles: a lane and its partner (lane ^ XOR) both carry 2H
// values; the lane keeps H of them (the upper half if `up`, which is the lane's own XOR bit) and adds the
// partner's copies of those.  With one value left (H = 0) both partners keep the pair sum.  The sum a
// lane forms is its own value plus the partner's, and the partner adds the same two numbers, so partners
// agree bit for bit.
template <int XOR, int H, int N>
__device__ __forceinline__ void halve_d(double (&v)[N], bool up) {
  if constexpr (H >= 1) {
    static_assert(2 * H <= N, "halving more values than the lane carries");
#pragma unroll
    for (int k = 0; k < H; ++k) {
      const double give = up ? v[k] : v[k + H];         // the half this lane drops is the half its partner keeps
      const double keep = up ? v[k + H] : v[k];
      v[k] = keep + xor_lane<XOR>(give);
    }
  } else {
    v[0] = v[0] + xor_lane<XOR>(v[0]);
  }
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

// w * self + wp * msg, with one fixed rounding order wherever it is evaluated: the product with self is
// rounded, then the peer's term is added by a fused multiply-add.  In this order the result can replace
// self in its own register (multiply in place, accumulate in place): kernels that carry self across a loop
// need no copy per element and round.
__device__ __forceinline__ float combine(float w, float self, float wp, float msg) {
#pragma clang fp contract(off)
  const float t = w * self;
  return __builtin_fmaf(wp, msg, t);
}
__device__ __forceinline__ vf4 combine(float w, vf4 self, float wp, vf4 msg) {
  vf4 o;
  o.x = combine(w, self.x, wp, msg.x); o.y = combine(w, self.y, wp, msg.y);
  o.z = combine(w, self.z, wp, msg.z); o.w = combine(w, self.w, wp, msg.w);
  return o;
}

}  // namespace ceca
