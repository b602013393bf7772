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

// Same tiling as the fused CECA rounds: a workgroup keeps a column tile of every agent's x in
// registers (RT rows per thread) and publishes it in LDS once per round, where each row picks up its
// peers.  One read and one write of x for any number of rounds.
template <int VEC, int RT>
__global__ __launch_bounds__(kBlock) void mix_rounds_kernel(const MixArgs M) {
#pragma clang fp contract(off)
  using V = typename VecOf<VEC>::T;
  extern __shared__ float lds_x[];                 // [n][lanes] groups of VEC floats
  const int lanes = kBlock / M.row_lanes;
  const int cg = threadIdx.x % lanes;
  const int rg = threadIdx.x / lanes;
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
  int spec = M.k0 % M.period;
  for (int t = 0; t < M.rounds; ++t) {
    const int j0 = M.start[spec], j1 = M.start[spec + 1];
    const float ws = M.w_self[spec];
    if (j1 > j0) {                                  // a round without peers is the identity
#pragma unroll
      for (int k = 0; k < RT; ++k) {
        const int i = rg + k * M.row_lanes;
        if (i < M.n) xs[i * lanes + cg] = x[k];
      }
      __syncthreads();
      // peer by peer, all of the thread's rows at once: the RT LDS reads of a peer are independent and
      // issue back to back (row by row they would each wait for the one before).  In the last, partly
      // filled group of rows the threads past the last agent shadow it.  The order of operations per row is still t = w_0 z_0, t = fma(w_j, z_j, t),
      // x+ = fma(w_self, x, t).
      V acc[RT];
      {
        const int sh = M.shift[j0];
        const float w = M.w[j0];
#pragma unroll
        for (int k = 0; k < RT; ++k) {
          int p = min(rg + k * M.row_lanes, M.n - 1) - sh;
          if (p < 0) p += M.n;
          acc[k] = w * xs[p * lanes + cg];
        }
      }
      for (int j = j0 + 1; j < j1; ++j) {
        const int sh = M.shift[j];
        const float w = M.w[j];
#pragma unroll
        for (int k = 0; k < RT; ++k) {
          int p = min(rg + k * M.row_lanes, M.n - 1) - sh;
          if (p < 0) p += M.n;
          acc[k] = fma_each(w, xs[p * lanes + cg], acc[k]);
        }
      }
#pragma unroll
      for (int k = 0; k < RT; ++k) x[k] = fma_each(ws, x[k], acc[k]);
      __syncthreads();
    }
    if (++spec == M.period) spec = 0;
  }
  if (!on) return;
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg + k * M.row_lanes;
    if (i < M.n) st_stream<V>(M.xout + (int64_t)i * M.ld + col, x[k]);
  }
}

std::atomic<int> g_mix_xcd{1};

hipError_t launch_mix_rounds(const MixArgs& m, bool vec4, hipStream_t st) {
  if (m.ngroups <= 0) return hipSuccess;
  const int lanes = kBlock / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  MixArgs mm = m;
  mm.xcd_tiles = 0;
  if (lanes * (vec4 ? 16 : 4) < 128 && blocks >= 1024 && g_mix_xcd) {
    mm.xcd_tiles = (int32_t)((blocks + 7) / 8);
    blocks = (int64_t)mm.xcd_tiles * 8;            // tiles past the last one find no columns and leave
  }
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  dim3 grid((unsigned)blocks), block(kBlock);
  // 16-byte groups: exactly the rows n needs (1..32 per thread); the few scalar tail columns round up
#define CECA_MIX4(RT) case RT: mix_rounds_kernel<4, RT><<<grid, block, lds, st>>>(mm); break
#define CECA_MIX1(RT) mix_rounds_kernel<1, RT><<<grid, block, lds, st>>>(mm)
  if (m.rows_per_thread < 1 || m.rows_per_thread > 32) return hipErrorInvalidValue;
  if (vec4) {
    switch (m.rows_per_thread) {
      CECA_MIX4(1); CECA_MIX4(2); CECA_MIX4(3); CECA_MIX4(4); CECA_MIX4(5); CECA_MIX4(6); CECA_MIX4(7); CECA_MIX4(8);
      CECA_MIX4(9); CECA_MIX4(10); CECA_MIX4(11); CECA_MIX4(12); CECA_MIX4(13); CECA_MIX4(14); CECA_MIX4(15); CECA_MIX4(16);
      CECA_MIX4(17); CECA_MIX4(18); CECA_MIX4(19); CECA_MIX4(20); CECA_MIX4(21); CECA_MIX4(22); CECA_MIX4(23); CECA_MIX4(24);
      CECA_MIX4(25); CECA_MIX4(26); CECA_MIX4(27); CECA_MIX4(28); CECA_MIX4(29); CECA_MIX4(30); CECA_MIX4(31); CECA_MIX4(32);
    }
  } else if (m.rows_per_thread <= 4) CECA_MIX1(4);
  else if (m.rows_per_thread <= 8) CECA_MIX1(8);
  else if (m.rows_per_thread <= 16) CECA_MIX1(16);
  else CECA_MIX1(32);
#undef CECA_MIX4
#undef CECA_MIX1
  return hipGetLastError();
}

}  // namespace ceca
