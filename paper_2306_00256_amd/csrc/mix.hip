// Shift-invariant gossip rounds for gfx950 (see ceca_mix_rounds in ceca.h): the comparison
// topologies of Table 1 -- ring, static exponential, one-peer exponential -- as circulant mixing of x.
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

__device__ __forceinline__ float fma_each(float w, float z, float t) { return __builtin_fmaf(w, z, t); }
__device__ __forceinline__ vf4 fma_each(float w, vf4 z, vf4 t) {
  vf4 o;
  o.x = __builtin_fmaf(w, z.x, t.x); o.y = __builtin_fmaf(w, z.y, t.y);
  o.z = __builtin_fmaf(w, z.z, t.z); o.w = __builtin_fmaf(w, z.w, t.w);
  return o;
}

// Wavefronts per SIMD the kernel is compiled for: workgroups wider than 256 threads must fit 128
// registers per thread (one 1024-thread workgroup or two 512-thread ones per compute unit).
template <int THREADS>
constexpr int mix_waves() { return THREADS > 256 ? 4 : 1; }

// Same tiling as the fused CECA rounds: a workgroup keeps a column tile of every agent's x in
// registers (RT rows per thread) and publishes it in LDS once per round, where each row picks up its
// peers.  One read and one write of x for any number of rounds.
template <int VEC, int RT, int THREADS>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(mix_waves<THREADS>())))
void mix_rounds_kernel(const MixArgs M) {
#pragma clang fp contract(off)
  using V = typename VecOf<VEC>::T;
  extern __shared__ float lds_x[];                 // [n][lanes] groups of VEC floats
  const int lanes = THREADS / M.row_lanes;
  const int tid = threadIdx.x;
  const int cg = tid % lanes;
  const int rg = tid / lanes;
  // workgroups go round-robin over the 8 XCDs, each with its own L2: when a row of the tile is
  // narrower than a 128-byte line, neighbouring tiles should meet in one L2, so every XCD takes a
  // contiguous run of tiles (xcd_tiles = tiles per XCD, 0 = plain order)
  int64_t tile = blockIdx.x;
  if (M.xcd_tiles > 0) tile = (int64_t)(blockIdx.x & 7) * M.xcd_tiles + (blockIdx.x >> 3);
  const int64_t g = tile * lanes + cg;
  const bool on = g < M.ngroups;
  const int64_t col = M.col0 + (on ? g : 0) * VEC; // lanes past the last column shadow column group 0

  V x[RT];
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = min(rg + k * M.row_lanes, M.n - 1);   // rows past the last agent shadow it
    x[k] = ld_stream<V>(M.xin + (int64_t)i * M.ld + col);
  }
  V* xs = reinterpret_cast<V*>(lds_x);
  // Row i, column group c sits in LDS slot i * lanes + c, so my row k is slot tid + k * THREADS
  // (row_lanes * lanes = THREADS).  rows_per_thread is the least that covers n, so only my last row can
  // lie past the last agent: it then shadows agent n - 1 and is never published.
  constexpr int L = RT - 1;
  const bool last_mine = rg + L * M.row_lanes < M.n;
  const int slot_last = last_mine ? tid + L * THREADS : (M.n - 1) * lanes + cg;
  const int wrap = M.n * lanes;
  int spec = M.k0 % M.period;
  for (int t = 0; t < M.rounds; ++t) {
    const int j0 = M.start[spec], j1 = M.start[spec + 1];
    const float ws = M.w_self[spec];
    if (j1 > j0) {                                  // a round without peers is the identity
#pragma unroll
      for (int k = 0; k < L; ++k) xs[tid + k * THREADS] = x[k];
      if (last_mine) xs[slot_last] = x[L];
      __syncthreads();
      // peer by peer, all of the thread's rows at once: the RT LDS reads of a peer are independent and
      // issue back to back (row by row they would each wait for the one before).  Per row the order of
      // operations is t = w_self x, then t = fma(w_j, z_j, t) peer after peer -- with one peer that of the
      // CECA combine -- so the new x grows in the registers of the old one.
#pragma unroll
      for (int k = 0; k < RT; ++k) x[k] = ws * x[k];
      for (int j = j0; j < j1; ++j) {
        const int back = M.shift[j] * lanes;
        const float w = M.w[j];
#pragma unroll
        for (int k = 0; k < RT; ++k) {
          int q = ((k == L) ? slot_last : tid + k * THREADS) - back;
          if (q < 0) q += wrap;
          x[k] = fma_each(w, xs[q], x[k]);
        }
      }
      __syncthreads();
    }
    if (++spec == M.period) spec = 0;
  }
  if (!on) return;
  // the row addresses are worked out here, after the rounds: nothing of them occupies registers meanwhile
  int rg_out = rg;
  asm volatile("" : "+v"(rg_out));
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg_out + k * M.row_lanes;
    if (i < M.n) st_stream<V>(M.xout + (int64_t)i * M.ld + col, x[k]);
  }
}


template <int VEC, int RT, int THREADS>
static hipError_t launch_mix(const MixArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  if (lds > 64 * 1024) {
    // more than 64 KB of LDS per workgroup has to be asked for
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mix_rounds_kernel<VEC, RT, THREADS>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  mix_rounds_kernel<VEC, RT, THREADS><<<dim3(blocks), dim3(THREADS), lds, st>>>(mm);
  return hipGetLastError();
}

// 256-thread workgroups: up to 32 rows per thread
template <int VEC>
static hipError_t launch_mix_256(const MixArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  switch (mm.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_mix<VEC, RT, 256>(mm, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
    CECA_RT(9); CECA_RT(10); CECA_RT(11); CECA_RT(12); CECA_RT(13); CECA_RT(14); CECA_RT(15); CECA_RT(16);
    CECA_RT(17); CECA_RT(18); CECA_RT(19); CECA_RT(20); CECA_RT(21); CECA_RT(22); CECA_RT(23); CECA_RT(24);
    CECA_RT(25); CECA_RT(26); CECA_RT(27); CECA_RT(28); CECA_RT(29); CECA_RT(30); CECA_RT(31); CECA_RT(32);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

// wider workgroups (16-byte groups only): up to kMixWideRows rows per thread fit their 128 registers
template <int THREADS>
static hipError_t launch_mix_wide(const MixArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  switch (mm.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_mix<4, RT, THREADS>(mm, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
    CECA_RT(9); CECA_RT(10); CECA_RT(11); CECA_RT(12); CECA_RT(13); CECA_RT(14); CECA_RT(15); CECA_RT(16);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

hipError_t launch_mix_rounds(const MixArgs& m, bool vec4, hipStream_t st) {
  if (m.ngroups <= 0) return hipSuccess;
  const int threads = m.threads > 0 ? m.threads : kBlock;
  if (threads != 256 && threads != 512 && threads != 1024) return hipErrorInvalidValue;
  if (!vec4 && threads != 256) return hipErrorInvalidValue;          // scalar columns: 256-thread tiles only
  if (m.row_lanes < 1 || m.row_lanes > threads || (m.row_lanes & (m.row_lanes - 1)) != 0) return hipErrorInvalidValue;
  // the kernel relies on rows_per_thread being the least that covers n (only a thread's last row can
  // lie past the last agent)
  if (m.rows_per_thread < 1 || m.rows_per_thread > 32 ||
      (int64_t)m.rows_per_thread * m.row_lanes < m.n || (int64_t)(m.rows_per_thread - 1) * m.row_lanes >= m.n)
    return hipErrorInvalidValue;
  const int lanes = threads / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  MixArgs mm = m;
  mm.xcd_tiles = 0;
  if (lanes * (vec4 ? 16 : 4) < 128 && blocks >= 1024 && !g_tuning.plain_tile_order) {
    mm.xcd_tiles = (int32_t)((blocks + 7) / 8);
    blocks = (int64_t)mm.xcd_tiles * 8;            // tiles past the last one find no columns and leave
  }
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  if (lds > kMultiMaxLds) return hipErrorInvalidValue;
  if (!vec4) return launch_mix_256<1>(mm, (unsigned)blocks, lds, st);
  if (threads == 256) return launch_mix_256<4>(mm, (unsigned)blocks, lds, st);
  if (threads == 512) return launch_mix_wide<512>(mm, (unsigned)blocks, lds, st);
  return launch_mix_wide<1024>(mm, (unsigned)blocks, lds, st);
}

}  // namespace ceca
