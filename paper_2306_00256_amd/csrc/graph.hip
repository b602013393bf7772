// Gossip rounds over an arbitrary graph for gfx950 (see ceca_graph_rounds in ceca.h): the mixing step
// x_i+ = w_self[i] x_i + sum_j w[i][j] x_{nbr[i][j]} of Table 1's non-circulant topologies (grid, torus,
// hypercube, ...) and of any graph the caller brings, any number of rounds in one pass over x.
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

__device__ __forceinline__ float fma_rows(float w, float z, float t) { return __builtin_fmaf(w, z, t); }
__device__ __forceinline__ vf4 fma_rows(float w, vf4 z, vf4 t) {
  vf4 o;
  o.x = __builtin_fmaf(w, z.x, t.x); o.y = __builtin_fmaf(w, z.y, t.y);
  o.z = __builtin_fmaf(w, z.z, t.z); o.w = __builtin_fmaf(w, z.w, t.w);
  return o;
}

template <int THREADS>
constexpr int graph_waves() { return THREADS > 256 ? 4 : 1; }

// Same tiling as the shift-invariant mixing kernel: a workgroup keeps a column tile of every agent's x in
// registers (RT rows per thread), publishes it in LDS once per round, and every row picks up its
// neighbours there; the neighbour table of the round comes from memory (a few KB, cached), neighbour by
// neighbour for all of a thread's rows at once.  Per row the order of operations is t = w_self x, then
// t = fma(w_j, z_j, t) neighbour after neighbour -- that of the shift-invariant kernel, so a circulant
// graph gives the same bits there and here.
// STAGE: the round's table (n * m entries of index and weight) is copied into LDS behind the tile --
// once for a static graph, every round for a time-varying one (each thread requests its share of the
// next round's entries right after the barrier) -- and the look-ups read it there instead of from
// memory.  Used when the table is small (kGraphStageEntries entries per thread at most).
template <int VEC, int RT, int THREADS, bool STAGE>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(graph_waves<THREADS>())))
void graph_rounds_kernel(const GraphArgs M) {
#pragma clang fp contract(off)
  using V = typename VecOf<VEC>::T;
  extern __shared__ float lds_x[];                 // [n][lanes] groups of VEC floats, then (STAGE) [n * m] entries
  const int lanes = THREADS / M.row_lanes;
  const int tid = threadIdx.x;
  const int cg = tid % lanes;
  const int rg = tid / lanes;
  int64_t tile = blockIdx.x;
  if (M.xcd_tiles > 0) tile = (int64_t)(blockIdx.x & 7) * M.xcd_tiles + (blockIdx.x >> 3);   // see mix_rounds_kernel
  const int64_t g = tile * lanes + cg;
  const bool on = g < M.ngroups;
  const int64_t col = M.col0 + (on ? g : 0) * VEC; // lanes past the last column shadow column group 0

  V x[RT];
  int row[RT];                                     // my rows; one past the last agent shadows it (never published or stored)
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    row[k] = min(rg + k * M.row_lanes, M.n - 1);
    x[k] = ld_stream<V>(M.xin + (int64_t)row[k] * M.ld + col);
  }
  V* xs = reinterpret_cast<V*>(lds_x);
  // (clamped index, weight bits) of entry i * m + j, on the next 8-byte boundary behind the tile
  int2* tab = reinterpret_cast<int2*>(reinterpret_cast<char*>(lds_x) + (((size_t)M.n * lanes * sizeof(V) + 7) & ~(size_t)7));
  const int entries = M.n * M.m;
  constexpr int L = RT - 1;                        // rows_per_thread is the least that covers n: only row L can be a shadow
  const bool last_mine = rg + L * M.row_lanes < M.n;
  int spec = M.k0 % M.period;
  // my share of a round's table: entries tid, tid + THREADS, ...
  int2 share[STAGE ? kGraphStageEntries : 1];
  auto request_share = [&](int sp) {
    const int64_t base = (int64_t)sp * entries;
#pragma unroll
    for (int e = 0; e < kGraphStageEntries; ++e) {
      const int q = tid + e * THREADS;
      if (q < entries) {
        share[STAGE ? e : 0].x = min(max(M.nbr[base + q], 0), M.n - 1);     // indices outside [0, n) are clamped, not followed
        share[STAGE ? e : 0].y = __float_as_int(M.w[base + q]);
      }
    }
  };
  if (STAGE) request_share(spec);
  for (int t = 0; t < M.rounds; ++t) {
    const int64_t base = (int64_t)spec * M.n;
    const int32_t* nbr = M.nbr + base * M.m;
    const float* w = M.w + base * M.m;
    const int next_spec = (spec + 1 == M.period) ? 0 : spec + 1;
    float ws[RT];                                  // requested before the barrier, used after it
#pragma unroll
    for (int k = 0; k < RT; ++k) ws[k] = M.w_self[base + row[k]];
#pragma unroll
    for (int k = 0; k < L; ++k) xs[tid + k * THREADS] = x[k];      // row i, group c sits in slot i * lanes + c = tid + k * THREADS
    if (last_mine) xs[tid + L * THREADS] = x[L];
    const bool restage = STAGE && (t == 0 || M.period > 1);        // the same for every thread
    if (restage) {
#pragma unroll
      for (int e = 0; e < kGraphStageEntries; ++e) {
        const int q = tid + e * THREADS;
        if (q < entries) tab[q] = share[STAGE ? e : 0];
      }
    }
    __syncthreads();
    if (STAGE && M.period > 1 && t + 1 < M.rounds) request_share(next_spec);
#pragma unroll
    for (int k = 0; k < RT; ++k) x[k] = ws[k] * x[k];             // the new x grows in the registers of the old one
    for (int j = 0; j < M.m; ++j) {
      int idx[RT];
      float wt[RT];
#pragma unroll
      for (int k = 0; k < RT; ++k) {
        if (STAGE) {
          const int2 en = tab[row[k] * M.m + j];
          idx[k] = en.x;
          wt[k] = __int_as_float(en.y);
        } else {
          idx[k] = min(max(nbr[(int64_t)row[k] * M.m + j], 0), M.n - 1);   // indices outside [0, n) are clamped, not followed
          wt[k] = w[(int64_t)row[k] * M.m + j];
        }
      }
#pragma unroll
      for (int k = 0; k < RT; ++k) x[k] = fma_rows(wt[k], xs[idx[k] * lanes + cg], x[k]);
    }
    __syncthreads();
    spec = next_spec;
  }
  if (!on) return;
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg + k * M.row_lanes;
    if (i < M.n) st_stream<V>(M.xout + (int64_t)i * M.ld + col, x[k]);
  }
}

template <int VEC, int RT, int THREADS>
static hipError_t launch_graph(const GraphArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  // small tables are staged in LDS behind the tile
  const int64_t entries = (int64_t)mm.n * mm.m;
  const size_t staged = ((lds + 7) & ~(size_t)7) + (size_t)entries * sizeof(int2);
  const bool stage = mm.stage && entries <= (int64_t)kGraphStageEntries * THREADS && staged <= kMultiMaxLds &&
                     (staged <= 64 * 1024 || lds > 32 * 1024);     // do not halve the resident workgroups of a small tile
  if (stage) lds = staged;
  const void* fn = stage ? reinterpret_cast<const void*>(&graph_rounds_kernel<VEC, RT, THREADS, true>)
                         : reinterpret_cast<const void*>(&graph_rounds_kernel<VEC, RT, THREADS, false>);
  if (lds > 64 * 1024) {
    // more than 64 KB of LDS per workgroup has to be asked for
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (stage) graph_rounds_kernel<VEC, RT, THREADS, true><<<dim3(blocks), dim3(THREADS), lds, st>>>(mm);
  else graph_rounds_kernel<VEC, RT, THREADS, false><<<dim3(blocks), dim3(THREADS), lds, st>>>(mm);
  return hipGetLastError();
}

// 256-thread workgroups: up to kGraphRows rows per thread
template <int VEC>
static hipError_t launch_graph_256(const GraphArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  switch (mm.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_graph<VEC, RT, 256>(mm, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
    CECA_RT(9); CECA_RT(10); CECA_RT(11); CECA_RT(12); CECA_RT(13); CECA_RT(14); CECA_RT(15); CECA_RT(16);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

// wider workgroups (16-byte groups only): 6 rows per thread fit their 128 registers, 8 spill a little
template <int THREADS>
static hipError_t launch_graph_wide(const GraphArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  switch (mm.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_graph<4, RT, THREADS>(mm, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

hipError_t launch_graph_rounds(const GraphArgs& m, bool vec4, hipStream_t st) {
  if (m.ngroups <= 0) return hipSuccess;
  const int threads = m.threads > 0 ? m.threads : kBlock;
  if (threads != 256 && threads != 512 && threads != 1024) return hipErrorInvalidValue;
  if (!vec4 && threads != 256) return hipErrorInvalidValue;          // scalar columns: 256-thread tiles only
  if (m.row_lanes < 1 || m.row_lanes > threads || (m.row_lanes & (m.row_lanes - 1)) != 0) return hipErrorInvalidValue;
  // the kernel relies on rows_per_thread being the least that covers n
  if (m.rows_per_thread < 1 || m.rows_per_thread > kGraphRows ||
      (int64_t)m.rows_per_thread * m.row_lanes < m.n || (int64_t)(m.rows_per_thread - 1) * m.row_lanes >= m.n)
    return hipErrorInvalidValue;
  const int lanes = threads / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  GraphArgs mm = m;
  mm.xcd_tiles = 0;
  if (lanes * (vec4 ? 16 : 4) < 128 && blocks >= 1024 && !g_tuning.plain_tile_order) {
    mm.xcd_tiles = (int32_t)((blocks + 7) / 8);
    blocks = (int64_t)mm.xcd_tiles * 8;            // tiles past the last one find no columns and leave
  }
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  if (lds > kMultiMaxLds) return hipErrorInvalidValue;
  if (!vec4) return launch_graph_256<1>(mm, (unsigned)blocks, lds, st);
  if (threads == 256) return launch_graph_256<4>(mm, (unsigned)blocks, lds, st);
  if (threads == 512) return launch_graph_wide<512>(mm, (unsigned)blocks, lds, st);
  return launch_graph_wide<1024>(mm, (unsigned)blocks, lds, st);
}

}  // namespace ceca
