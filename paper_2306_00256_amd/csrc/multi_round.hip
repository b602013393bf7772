// Fused gossip rounds for gfx950 (see ceca_gossip_rounds in ceca.h).
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

// ---------------------------------------------------------------------------------------------
// Several gossip rounds in one pass: a workgroup keeps a column tile of every agent's (x, y) in
// registers and passes the travelling variable through LDS, so `rounds` rounds cost one read of x
// and one write of x and y (12 bytes per agent-parameter) instead of `rounds` x 16.  Columns are
// independent instances of the recursion (Sec. 3.1), and every round uses the same combine() as the
// single-round kernel, so the result has the same bits as `rounds` separate calls.
// ---------------------------------------------------------------------------------------------
// Tiles per XCD for the XCD-contiguous workgroup order (rows of the tile narrower than a 128-byte line
// and enough tiles to matter), 0 for the plain order; rounds *blocks up to 8 runs of that many tiles
// (workgroups past the last tile find no columns and leave).
static int32_t xcd_run(int row_bytes, int64_t* blocks) {
  if (row_bytes >= 128 || *blocks < 1024 || !g_mix_xcd) return 0;   // small launches measured better in plain order
  const int64_t per = (*blocks + 7) / 8;
  *blocks = per * 8;
  return (int32_t)per;
}

template <int VEC, int RT>
__global__ __launch_bounds__(kBlock) void multi_round_kernel(const MultiArgs M) {
  using V = typename VecOf<VEC>::T;
  extern __shared__ float lds_z[];                 // [n][lanes] groups of VEC floats
  const int lanes = kBlock / M.row_lanes;          // column groups per row handled by this workgroup
  const int cg = threadIdx.x % lanes;              // my column group inside the tile
  const int rg = threadIdx.x / lanes;              // my first row; I own rows rg, rg + row_lanes, ...
  // narrow tiles: every XCD (workgroups go round-robin over 8 of them, each with its own L2) takes a
  // contiguous run of tiles, so that the two halves of a 128-byte line meet in one L2
  int64_t tile = blockIdx.x;
  if (M.xcd_tiles > 0) tile = (int64_t)(blockIdx.x & 7) * M.xcd_tiles + (blockIdx.x >> 3);
  const int64_t g = tile * lanes + cg;
  const bool on = g < M.ngroups;
  const int64_t col = M.col0 + (on ? g : 0) * VEC; // lanes past the last column shadow column group 0

  V x[RT], y[RT];
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    // rows past the last agent shadow the last one (their values are never stored): no branch
    // surrounds a load, so all of a thread's rows are in flight together
    const int i = min(rg + k * M.row_lanes, M.n - 1);
    x[k] = ld_stream<V>(M.xin + (int64_t)i * M.ld + col);
    y[k] = V(0.0f);                                // round 0 has b = 0: y(0) is never used
  }
  V* zs = reinterpret_cast<V*>(lds_z);
  // LDS slot of each of my rows (rows past the last agent shadow it and are never published)
  int slot[RT];
  bool mine[RT];
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg + k * M.row_lanes;
    mine[k] = i < M.n;
    slot[k] = min(i, M.n - 1) * lanes + cg;
  }
  const int wrap = M.n * lanes;
  for (int t = 0; t < M.rounds; ++t) {
    const MultiRound R = M.round[t];
    // the round's flags are the same for every thread: branches, not per-element selects
    if (R.exch_y) {
#pragma unroll
      for (int k = 0; k < RT; ++k) if (mine[k]) zs[slot[k]] = y[k];
    } else {
#pragma unroll
      for (int k = 0; k < RT; ++k) if (mine[k]) zs[slot[k]] = x[k];
    }
    __syncthreads();
    // no branch around the LDS reads, so a thread's RT reads issue back to back
    V zp[RT];
    const int back = R.shift * lanes;
    if (M.port == 2) {
#pragma unroll
      for (int k = 0; k < RT; ++k) {
        int q = slot[k] - back;
        if (q < 0) q += wrap;
        zp[k] = zs[q];
      }
    } else {
#pragma unroll
      for (int k = 0; k < RT; ++k) {
        const int i = min(rg + k * M.row_lanes, M.n - 1);
        int q = (i & 1) ? slot[k] - back : slot[k] + back;     // even rows look ahead, odd rows back (Eq. (7))
        if (q < 0) q += wrap;
        if (q >= wrap) q -= wrap;
        zp[k] = zs[q];
      }
    }
#pragma unroll
    for (int k = 0; k < RT; ++k) x[k] = combine(R.a, x[k], R.ap, zp[k]);
    if (R.read_y) {
#pragma unroll
      for (int k = 0; k < RT; ++k) y[k] = combine(R.b, y[k], R.bp, zp[k]);
    } else {
#pragma unroll
      for (int k = 0; k < RT; ++k) y[k] = R.bp * zp[k];
    }
    __syncthreads();
  }
  if (!on) return;
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg + k * M.row_lanes;
    if (i < M.n) {
      st_stream<V>(M.xout + (int64_t)i * M.ld + col, x[k]);
      if (M.yout) st_stream<V>(M.yout + (int64_t)i * M.ld + col, y[k]);   // same for every thread
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Several DSGD-CECA iterations with the quadratic-centre loss in one pass.  That loss is elementwise
// (e_i = z_i - c_i + noise), so columns stay independent through whole iterations, not just through
// the communication round: the workgroup keeps a column tile of every agent's x, y and c in registers,
// takes the local step in place, exchanges the messages through LDS and combines (Algorithm 1,
// Eqs. (8), (9)), `rounds` times.  20 bytes per agent-parameter for any number of iterations.  The
// arithmetic per iteration is that of the single-step kernel, operation for operation.
// ---------------------------------------------------------------------------------------------
template <int VEC, int RT>
__global__ __launch_bounds__(kBlock) void multi_step_kernel(const StepsArgs S) {
#pragma clang fp contract(off)
  using V = typename VecOf<VEC>::T;
  const MultiArgs& M = S.m;
  extern __shared__ float lds_z[];                 // [n][lanes] groups of VEC floats
  const int lanes = kBlock / M.row_lanes;
  const int cg = threadIdx.x % lanes;
  const int rg = threadIdx.x / lanes;
  // narrow tiles: every XCD (workgroups go round-robin over 8 of them, each with its own L2) takes a
  // contiguous run of tiles, so that the two halves of a 128-byte line meet in one L2
  int64_t tile = blockIdx.x;
  if (M.xcd_tiles > 0) tile = (int64_t)(blockIdx.x & 7) * M.xcd_tiles + (blockIdx.x >> 3);
  const int64_t g = tile * lanes + cg;
  const bool on = g < M.ngroups;
  const int64_t col = M.col0 + (on ? g : 0) * VEC; // lanes past the last column shadow column group 0

  V x[RT], y[RT], c[RT];
  const bool first_reads_y = M.round[0].read_y != 0;
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = min(rg + k * M.row_lanes, M.n - 1);   // rows past the last agent shadow it
    x[k] = ld_stream<V>(M.xin + (int64_t)i * M.ld + col);
    c[k] = ld_stream<V>(S.c + (int64_t)i * S.ldc + col);
  }
  if (first_reads_y) {                             // a first round with b = 0 never uses y(0)
#pragma unroll
    for (int k = 0; k < RT; ++k) {
      const int i = min(rg + k * M.row_lanes, M.n - 1);
      y[k] = ld_stream<V>(S.yin + (int64_t)i * M.ld + col);
    }
  } else {
#pragma unroll
    for (int k = 0; k < RT; ++k) y[k] = V(0.0f);
  }
  V* zs = reinterpret_cast<V*>(lds_z);
  for (int t = 0; t < M.rounds; ++t) {
    const MultiRound R = M.round[t];
    V ge[RT];
    // local step of row k at z (its x or y): lr * e stays in registers, the message v_i goes to LDS
    auto half_step = [&](int k, const V& z) {
      const int i = min(rg + k * M.row_lanes, M.n - 1);
      V e = z - c[k];
      if (S.noise_std != 0.0f) e += S.noise_std * noise_group<V>(col, noise_keys(S.seed, S.k0 + (uint32_t)t, (uint32_t)i));
      ge[k] = S.lr * e;
      if (rg + k * M.row_lanes < M.n) zs[i * lanes + cg] = z - ge[k];
    };
    // the round's flags are the same for every thread: branches, not per-element selects
    if (R.exch_y) {
#pragma unroll
      for (int k = 0; k < RT; ++k) half_step(k, y[k]);
    } else {
#pragma unroll
      for (int k = 0; k < RT; ++k) half_step(k, x[k]);
    }
    __syncthreads();
    V zp[RT];
#pragma unroll
    for (int k = 0; k < RT; ++k) {
      const int i = min(rg + k * M.row_lanes, M.n - 1);
      int p;
      if (M.port == 2) {
        p = i - R.shift; if (p < 0) p += M.n;
      } else {
        p = (i & 1) ? i - R.shift : i + R.shift;
        if (p < 0) p += M.n;
        if (p >= M.n) p -= M.n;
      }
      zp[k] = zs[p * lanes + cg];
    }
#pragma unroll
    for (int k = 0; k < RT; ++k) x[k] = combine(R.a, x[k] - ge[k], R.ap, zp[k]);
    if (R.read_y) {
#pragma unroll
      for (int k = 0; k < RT; ++k) y[k] = combine(R.b, y[k] - ge[k], R.bp, zp[k]);
    } else {
#pragma unroll
      for (int k = 0; k < RT; ++k) y[k] = R.bp * zp[k];
    }
    __syncthreads();
  }
  if (!on) return;
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg + k * M.row_lanes;
    if (i < M.n) {
      st_stream<V>(M.xout + (int64_t)i * M.ld + col, x[k]);
      st_stream<V>(M.yout + (int64_t)i * M.ld + col, y[k]);
    }
  }
}

hipError_t launch_multi_step(const StepsArgs& s, bool vec4, hipStream_t st) {
  const MultiArgs& m = s.m;
  if (m.ngroups <= 0) return hipSuccess;
  const int lanes = kBlock / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  StepsArgs ss = s;
  ss.m.xcd_tiles = xcd_run(lanes * (vec4 ? 16 : 4), &blocks);
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  dim3 grid((unsigned)blocks), block(kBlock);
#define CECA_STEPS4(RT) case RT: multi_step_kernel<4, RT><<<grid, block, lds, st>>>(ss); break
#define CECA_STEPS1(RT) multi_step_kernel<1, RT><<<grid, block, lds, st>>>(ss)
  if (m.rows_per_thread < 1 || m.rows_per_thread > kMultiRows) return hipErrorInvalidValue;
  if (vec4) {
    switch (m.rows_per_thread) {
      CECA_STEPS4(1); CECA_STEPS4(2); CECA_STEPS4(3); CECA_STEPS4(4); CECA_STEPS4(5); CECA_STEPS4(6);
      CECA_STEPS4(7); CECA_STEPS4(8); CECA_STEPS4(9); CECA_STEPS4(10); CECA_STEPS4(11); CECA_STEPS4(12);
      CECA_STEPS4(13); CECA_STEPS4(14); CECA_STEPS4(15); CECA_STEPS4(16);
    }
  } else if (m.rows_per_thread <= 4) CECA_STEPS1(4);
  else if (m.rows_per_thread <= 8) CECA_STEPS1(8);
  else CECA_STEPS1(16);
#undef CECA_STEPS4
#undef CECA_STEPS1
  return hipGetLastError();
}

hipError_t launch_multi_round(const MultiArgs& m, bool vec4, hipStream_t st) {
  if (m.ngroups <= 0) return hipSuccess;
  const int lanes = kBlock / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  MultiArgs mm = m;
  mm.xcd_tiles = xcd_run(lanes * (vec4 ? 16 : 4), &blocks);
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  dim3 grid((unsigned)blocks), block(kBlock);
  // 16-byte groups: exactly the rows n needs (1..16 per thread); the few scalar tail columns round up
#define CECA_MULTI4(RT) case RT: multi_round_kernel<4, RT><<<grid, block, lds, st>>>(mm); break
#define CECA_MULTI1(RT) multi_round_kernel<1, RT><<<grid, block, lds, st>>>(mm)
  if (m.rows_per_thread < 1 || m.rows_per_thread > kMultiRows) return hipErrorInvalidValue;
  if (vec4) {
    switch (m.rows_per_thread) {
      CECA_MULTI4(1); CECA_MULTI4(2); CECA_MULTI4(3); CECA_MULTI4(4); CECA_MULTI4(5); CECA_MULTI4(6);
      CECA_MULTI4(7); CECA_MULTI4(8); CECA_MULTI4(9); CECA_MULTI4(10); CECA_MULTI4(11); CECA_MULTI4(12);
      CECA_MULTI4(13); CECA_MULTI4(14); CECA_MULTI4(15); CECA_MULTI4(16);
    }
  } else if (m.rows_per_thread <= 4) CECA_MULTI1(4);
  else if (m.rows_per_thread <= 8) CECA_MULTI1(8);
  else CECA_MULTI1(16);
#undef CECA_MULTI4
#undef CECA_MULTI1
  return hipGetLastError();
}

}  // namespace ceca
