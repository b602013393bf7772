// Consensus observables for gfx950 (see consensus_error in ceca.h).
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

// ---------------------------------------------------------------------------------------------
// Consensus observables: fp64 column mean, then per-agent squared distance to it.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void acc4(double (&s)[4], vf4 v) { s[0] += v.x; s[1] += v.y; s[2] += v.z; s[3] += v.w; }
__device__ __forceinline__ void acc4(double (&s)[4], float v) { s[0] += v; }

template <int VEC>
__global__ __launch_bounds__(kBlock) void colsum_kernel(const ConsensusArgs C) {
  using V = typename VecOf<VEC>::T;
  const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
  if (col + VEC > C.d) return;
  const int grp = blockIdx.y;
  const int i_lo = grp * C.agents_per_group;
  const int i_hi = min(C.n, i_lo + C.agents_per_group);
  double s[4] = {0.0, 0.0, 0.0, 0.0};
  int i = i_lo;
  for (; i + 4 <= i_hi; i += 4) {
    V r[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) r[q] = ld_plain<V>(C.X + (int64_t)(i + q) * C.ld + col);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc4(s, r[q]);
  }
  for (; i < i_hi; ++i) acc4(s, ld_plain<V>(C.X + (int64_t)i * C.ld + col));
  double* dst = C.colsum + (int64_t)grp * C.d + col;
#pragma unroll
  for (int q = 0; q < VEC; ++q) dst[q] = s[q];
}

// slice 0 of colsum <- mean; optional fp32 copy; per-workgroup partial of ||xbar||^2
__global__ __launch_bounds__(kBlock) void mean_kernel(const ConsensusArgs C) {
  __shared__ double red[kBlock / 64];
  double sq = 0.0;
  const int64_t base = (int64_t)blockIdx.x * kConsTile;
  for (int q = 0; q < (int)(kConsTile / kBlock); ++q) {
    const int64_t col = base + q * kBlock + threadIdx.x;
    if (col < C.d) {
      double s = 0.0;
      for (int g = 0; g < C.agent_groups; ++g) s += C.colsum[(int64_t)g * C.d + col];
      const double m = s / (double)C.n;
      C.colsum[col] = m;
      if (C.xbar) C.xbar[col] = (float)m;
      sq += m * m;
    }
  }
  sq = wave_sum(sq);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sq;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < kBlock / 64; ++w) t += red[w];
    C.normpart[blockIdx.x] = t;
  }
}

__device__ __forceinline__ double sqdev(vf4 v, const double (&m)[4]) {
  const double a = (double)v.x - m[0], b = (double)v.y - m[1], c = (double)v.z - m[2], d = (double)v.w - m[3];
  return a * a + b * b + c * c + d * d;
}
__device__ __forceinline__ double sqdev(float v, const double (&m)[4]) {
  const double a = (double)v - m[0];
  return a * a;
}

// devpart[agent][tile] = sum over the tile's columns of (x[agent][col] - mean[col])^2
template <int VEC>
__global__ __launch_bounds__(kBlock) void dev_kernel(const ConsensusArgs C) {
  using V = typename VecOf<VEC>::T;
  __shared__ double red[kBlock / 64];
  const int64_t tile = blockIdx.x;
  constexpr int PER = (int)(kConsTile / kBlock) / VEC;   // column groups per thread
  double m[PER][4];
  int64_t col[PER];
  bool on[PER];
#pragma unroll
  for (int p = 0; p < PER; ++p) {
    col[p] = tile * kConsTile + ((int64_t)p * kBlock + threadIdx.x) * VEC;
    on[p] = col[p] + VEC <= C.d;
#pragma unroll
    for (int q = 0; q < 4; ++q) m[p][q] = (on[p] && q < VEC) ? C.colsum[col[p] + q] : 0.0;
  }
  const int i_lo = blockIdx.y * C.dev_agents;
  const int i_hi = min(C.n, i_lo + C.dev_agents);
  for (int i = i_lo; i < i_hi; ++i) {
    double s = 0.0;
#pragma unroll
    for (int p = 0; p < PER; ++p)
      if (on[p]) s += sqdev(ld_plain<V>(C.X + (int64_t)i * C.ld + col[p]), m[p]);
    s = wave_sum(s);
    __syncthreads();   // red[] of the previous agent has been consumed
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int w = 0; w < kBlock / 64; ++w) t += red[w];
      C.devpart[(int64_t)i * C.ntiles + tile] = t;
    }
  }
}

// Single pass: a workgroup holds a column tile of every agent (RT rows per thread, the tiling of the
// fused-round kernels), so x is read once: column sums across the workgroup through LDS (fp64, fixed
// order), the mean in registers, then every row's squared distance to it and the tile's share of
// ||xbar||^2.  Writes devpart[agent][tile], normpart[tile] and, if asked, xbar.
template <int VEC, int RT>
__global__ __launch_bounds__(kBlock) void cons_tile_kernel(const ConsensusArgs C) {
  using V = typename VecOf<VEC>::T;
  extern __shared__ double lds_d[];                // phase 1: [row_lanes][lanes * VEC]; phase 2: [n + 1][lanes]
  const int lanes = kBlock / C.row_lanes;
  const int cg = threadIdx.x % lanes;
  const int rg = threadIdx.x / lanes;
  const int64_t tile = blockIdx.x;
  const int64_t g = tile * lanes + cg;
  const int64_t ngroups = (C.d + VEC - 1) / VEC;   // d is a multiple of VEC on the vector path
  const bool on = g < ngroups;
  const int64_t col = (on ? g : 0) * VEC;          // lanes past the last column shadow column group 0
  V x[RT];
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = min(rg + k * C.row_lanes, C.n - 1);    // rows past the last agent shadow it (weight 0 below)
    x[k] = ld_stream<V>(C.X + (int64_t)i * C.ld + col);
  }
  double s[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int k = 0; k < RT; ++k)
    if (rg + k * C.row_lanes < C.n) acc4(s, x[k]);
#pragma unroll
  for (int q = 0; q < VEC; ++q) lds_d[(rg * lanes + cg) * VEC + q] = s[q];
  __syncthreads();
  double m[4] = {0.0, 0.0, 0.0, 0.0};
  for (int r = 0; r < C.row_lanes; ++r) {
#pragma unroll
    for (int q = 0; q < VEC; ++q) m[q] += lds_d[(r * lanes + cg) * VEC + q];
  }
#pragma unroll
  for (int q = 0; q < VEC; ++q) m[q] /= (double)C.n;
  __syncthreads();                                  // phase 1 values are consumed: the buffer changes shape
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg + k * C.row_lanes;
    if (i < C.n) lds_d[i * lanes + cg] = on ? sqdev(x[k], m) : 0.0;
  }
  if (rg == 0) {
    double sq = 0.0;
#pragma unroll
    for (int q = 0; q < VEC; ++q) sq += m[q] * m[q];
    lds_d[C.n * lanes + cg] = on ? sq : 0.0;
    if (on && C.xbar) {
#pragma unroll
      for (int q = 0; q < VEC; ++q) C.xbar[col + q] = (float)m[q];
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i <= C.n; i += kBlock) {
    double t = 0.0;
    for (int c = 0; c < lanes; ++c) t += lds_d[i * lanes + c];
    if (i < C.n) C.devpart[(int64_t)i * C.ntiles + tile] = t;
    else C.normpart[tile] = t;
  }
}

// Single pass, one wavefront per column strip: the 64 lanes of a wavefront hold a strip of every agent
// (lane = row lane * cgs + column group: cgs adjacent 16-byte groups of RT rows each, rows
// rg, rg + row_lanes, ...), so x is read once and nothing is shared between wavefronts: no LDS, no barrier.
// Column sums cross the row lanes and squared deviations cross the column groups through lane exchanges
// (fp64, fixed order).  A wavefront takes strips w, w + nwaves, ... and adds up every row's squared
// distance to the column means over all of them before it reduces across lanes once.
// Writes devpart[agent][wave] (row n: the wavefront's share of ||xbar||^2) and, if asked, xbar.
template <int VEC, int RT>
__global__ __launch_bounds__(kBlock) void cons_wave_kernel(const ConsensusArgs C) {
  using V = typename VecOf<VEC>::T;
  constexpr int RTP = RT <= 1 ? 1 : RT <= 2 ? 2 : RT <= 4 ? 4 : RT <= 8 ? 8 : RT <= 16 ? 16 : 32;
  constexpr int LOG_RTP = RTP == 1 ? 0 : RTP == 2 ? 1 : RTP == 4 ? 2 : RTP == 8 ? 3 : RTP == 16 ? 4 : 5;
  const int lane = threadIdx.x & 63;
  const int64_t w = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (w >= C.nwaves) return;                        // the whole wavefront leaves
  const int cgs = C.wave_cgs;                       // column groups per strip: a power of two, 1..64
  const int cg = lane & (cgs - 1);
  const int rg = lane >> C.cg_shift;
  const int row_lanes = 64 >> C.cg_shift;
  const int64_t ngroups = (C.d + VEC - 1) / VEC;    // d is a multiple of VEC on the vector path
  double acc[RTP];
#pragma unroll
  for (int k = 0; k < RTP; ++k) acc[k] = 0.0;
  double nrm = 0.0;
  // the loads of one strip: lanes past the last column shadow column group 0, rows past the last agent
  // shadow it (neither is ever counted), so no branch surrounds a load
  auto request = [&](int64_t strip, V (&x)[RT], bool& on, int64_t& col) {
    const int64_t g = strip * cgs + cg;
    on = g < ngroups;
    col = (on ? g : 0) * VEC;
    // my rows lie row_lanes rows apart: one address, stepped (only the last row may need the clamp)
    const float* p = C.X + (int64_t)rg * C.ld + col;
    const int64_t step = (int64_t)row_lanes * C.ld;
#pragma unroll
    for (int k = 0; k < RT - 1; ++k) {
      x[k] = ld_stream<V>(p);
      p += step;
    }
    const int i = min(rg + (RT - 1) * row_lanes, C.n - 1);
    x[RT - 1] = ld_stream<V>(C.X + (int64_t)i * C.ld + col);
  };
  V x[RT];
  bool on;
  int64_t col;
  int64_t strip = w;
  request(strip, x, on, col);
  while (true) {
    const int64_t next = strip + C.nwaves;
    const bool more = next < C.strips;              // the same for the whole wavefront
    // rows per lane is the least that covers n, so only a lane's last row can lie past the last agent: the
    // others need no test
    const bool last_mine = rg + (RT - 1) * row_lanes < C.n;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int k = 0; k < RT - 1; ++k) acc4(s, x[k]);
    if (last_mine) acc4(s, x[RT - 1]);
    // the row lanes of a column group sit cgs lanes apart: sum across them (every lane ends with the total)
#define CECA_ROWSUM(O)                                                \
    if (cgs <= O) {                                                   \
      _Pragma("unroll") for (int q = 0; q < VEC; ++q) s[q] += xor_lane<O>(s[q]); \
    }
    CECA_ROWSUM(1) CECA_ROWSUM(2) CECA_ROWSUM(4) CECA_ROWSUM(8) CECA_ROWSUM(16) CECA_ROWSUM(32)
#undef CECA_ROWSUM
    double m[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int q = 0; q < VEC; ++q) m[q] = s[q] / (double)C.n;
    if (on) {
#pragma unroll
      for (int k = 0; k < RT - 1; ++k) acc[k] += sqdev(x[k], m);
      if (last_mine) acc[RT - 1] += sqdev(x[RT - 1], m);
    }
    if (rg == 0 && on) {
#pragma unroll
      for (int q = 0; q < VEC; ++q) nrm += m[q] * m[q];
      if (C.xbar) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) C.xbar[col + q] = (float)m[q];
      }
    }
    if (!more) break;
    request(next, x, on, col);
    strip = next;
  }
  // Sum over the column groups (lane bits below cg_shift).  Level t halves the rows a lane still carries
  // while there is more than one: afterwards the lane holds complete sums of rows off, off + 1, ...
  if (cgs > 1) { halve_d<1, RTP / 2>(acc, (lane & 1) != 0); nrm += xor_lane<1>(nrm); }
  if (cgs > 2) { halve_d<2, RTP / 4>(acc, (lane & 2) != 0); nrm += xor_lane<2>(nrm); }
  if (cgs > 4) { halve_d<4, RTP / 8>(acc, (lane & 4) != 0); nrm += xor_lane<4>(nrm); }
  if (cgs > 8) { halve_d<8, RTP / 16>(acc, (lane & 8) != 0); nrm += xor_lane<8>(nrm); }
  if (cgs > 16) { halve_d<16, RTP / 32>(acc, (lane & 16) != 0); nrm += xor_lane<16>(nrm); }
  if (cgs > 32) { halve_d<32, RTP / 64>(acc, (lane & 32) != 0); nrm += xor_lane<32>(nrm); }
  const int halvings = C.cg_shift < LOG_RTP ? C.cg_shift : LOG_RTP;     // levels that dropped half of the rows
  int off = 0;
#pragma unroll
  for (int t = 0; t < LOG_RTP; ++t)
    if (t < halvings) off += ((lane >> t) & 1) * (RTP >> (t + 1));
  const int live = RTP >> halvings;
  // with more column groups than rows the later levels leave copies: the lane whose remaining bits are 0 writes
  const bool writer = (cg >> halvings) == 0;
#pragma unroll
  for (int j = 0; j < RTP; ++j) {
    const int k = j + off;
    const int i = rg + k * row_lanes;
    if (writer && j < live && k < RT && i < C.n) C.devpart[(int64_t)i * C.nwaves + w] = acc[j];
  }
  if (lane == 0) C.devpart[(int64_t)C.n * C.nwaves + w] = nrm;
}

// The five results from the per-agent squared deviations dev2[0..n) and the partials of ||xbar||^2 (every
// sum in a fixed order).  One workgroup.
__device__ __forceinline__ void finish_results(const ConsensusArgs& C, const double* dev2) {
  __shared__ double r0[kBlock / 64], r1[kBlock / 64], r2[kBlock / 64], r3[kBlock / 64];
  double frob = 0.0, resid = 0.0, mx = 0.0, nrm = 0.0;
  for (int a = threadIdx.x; a < C.n; a += kBlock) {
    const double d2 = dev2[a];
    const double dv = sqrt(d2);
    frob += d2; resid += dv; mx = fmax(mx, dv);
  }
  for (int64_t t = threadIdx.x; t < C.norm_count; t += kBlock) nrm += C.normpart[t];
  frob = wave_sum(frob); resid = wave_sum(resid); mx = wave_max(mx); nrm = wave_sum(nrm);
  if ((threadIdx.x & 63) == 0) {
    const int w = threadIdx.x >> 6;
    r0[w] = frob; r1[w] = resid; r2[w] = mx; r3[w] = nrm;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double a = 0.0, b = 0.0, c = 0.0, d = 0.0;
    for (int w = 0; w < kBlock / 64; ++w) { a += r0[w]; b += r1[w]; c = fmax(c, r2[w]); d += r3[w]; }
    C.out[0] = a; C.out[1] = b; C.out[2] = c; C.out[3] = sqrt(d); C.out[4] = (double)C.n;
  }
}

// dev2[row] = sum over tiles (or wavefronts) of devpart[row][.]; one workgroup per row
__global__ __launch_bounds__(kBlock) void devsum_kernel(const ConsensusArgs C) {
  __shared__ double red[kBlock / 64];
  const int i = blockIdx.x;
  double s = 0.0;
  for (int64_t t = threadIdx.x; t < C.ntiles; t += kBlock) s += C.devpart[(int64_t)i * C.ntiles + t];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < kBlock / 64; ++w) t += red[w];
    C.dev2[i] = t;
  }
}

__global__ __launch_bounds__(kBlock) void finish_kernel(const ConsensusArgs C) { finish_results(C, C.dev2); }

// Few partials in all (small problems, where every launch counts): one workgroup sums the rows of devpart in
// turn (same order of additions as devsum_kernel) and finishes, in one launch.
__global__ __launch_bounds__(kBlock) void close_small_kernel(const ConsensusArgs C) {
  __shared__ double red[kBlock / 64];
  for (int i = 0; i < C.close_rows; ++i) {
    double s = 0.0;
    for (int64_t t = threadIdx.x; t < C.ntiles; t += kBlock) s += C.devpart[(int64_t)i * C.ntiles + t];
    s = wave_sum(s);
    __syncthreads();                                 // red[] of the row before has been consumed
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
      double t = 0.0;
      for (int w = 0; w < kBlock / 64; ++w) t += red[w];
      C.dev2[i] = t;
    }
  }
  __threadfence_block();
  __syncthreads();                                   // this workgroup wrote dev2 itself: visible to all its threads
  finish_results(C, C.dev2);
}

// Closes a consensus call: dev2 from the partials of `rows` rows (n, or n + 1 with ||xbar||^2 as the last), then
// the results.
static void launch_close(ConsensusArgs& c, int rows, hipStream_t st) {
  c.close_rows = rows;
  if ((int64_t)rows * c.ntiles <= 16384) {
    close_small_kernel<<<dim3(1), dim3(kBlock), 0, st>>>(c);
  } else {
    devsum_kernel<<<dim3((unsigned)rows), dim3(kBlock), 0, st>>>(c);
    finish_kernel<<<dim3(1), dim3(kBlock), 0, st>>>(c);
  }
}

// out[10] = out[0] + out[5]: the two halves' Frobenius terms of ||phi||_F^2
__global__ void phi_kernel(double* out) {
  if (threadIdx.x == 0) out[10] = out[0] + out[5];
}

hipError_t launch_phi(double* out, hipStream_t st) {
  phi_kernel<<<dim3(1), dim3(64), 0, st>>>(out);
  return hipGetLastError();
}

static hipError_t launch_cons_tile(ConsensusArgs c, bool vec4, hipStream_t st) {
  const int lanes = kBlock / c.row_lanes;
  const size_t lds = sizeof(double) * (size_t)((c.n + 1) * lanes > kBlock * (vec4 ? 4 : 1) ? (c.n + 1) * lanes : kBlock * (vec4 ? 4 : 1));
  if (c.ntiles < 1 || c.ntiles >= (1LL << 24) || lds > 65536 || c.rows_per_thread < 1 || c.rows_per_thread > 32)
    return hipErrorInvalidConfiguration;
  dim3 grid((unsigned)c.ntiles), block(kBlock);
#define CECA_CONS4(RT) case RT: cons_tile_kernel<4, RT><<<grid, block, lds, st>>>(c); break
#define CECA_CONS1(RT) cons_tile_kernel<1, RT><<<grid, block, lds, st>>>(c)
  if (vec4) {
    switch (c.rows_per_thread) {
      CECA_CONS4(1); CECA_CONS4(2); CECA_CONS4(3); CECA_CONS4(4); CECA_CONS4(5); CECA_CONS4(6); CECA_CONS4(7); CECA_CONS4(8);
      CECA_CONS4(9); CECA_CONS4(10); CECA_CONS4(11); CECA_CONS4(12); CECA_CONS4(13); CECA_CONS4(14); CECA_CONS4(15); CECA_CONS4(16);
      CECA_CONS4(17); CECA_CONS4(18); CECA_CONS4(19); CECA_CONS4(20); CECA_CONS4(21); CECA_CONS4(22); CECA_CONS4(23); CECA_CONS4(24);
      CECA_CONS4(25); CECA_CONS4(26); CECA_CONS4(27); CECA_CONS4(28); CECA_CONS4(29); CECA_CONS4(30); CECA_CONS4(31); CECA_CONS4(32);
    }
  } else if (c.rows_per_thread <= 4) CECA_CONS1(4);
  else if (c.rows_per_thread <= 8) CECA_CONS1(8);
  else if (c.rows_per_thread <= 16) CECA_CONS1(16);
  else CECA_CONS1(32);
#undef CECA_CONS4
#undef CECA_CONS1
  launch_close(c, c.n, st);
  return hipGetLastError();
}

static hipError_t launch_cons_wave(const ConsensusArgs& c0, bool vec4, hipStream_t st) {
  ConsensusArgs c = c0;
  const int cgs = c.wave_cgs;
  if (cgs < 1 || cgs > 64 || (cgs & (cgs - 1)) != 0 || (1 << c.cg_shift) != cgs) return hipErrorInvalidValue;
  const int row_lanes = 64 / cgs;
  // the kernel relies on rows_per_thread being the least that covers n
  if (c.rows_per_thread < 1 || c.rows_per_thread > 32 || (int64_t)c.rows_per_thread * row_lanes < c.n ||
      (int64_t)(c.rows_per_thread - 1) * row_lanes >= c.n)
    return hipErrorInvalidValue;
  if (c.nwaves < 1 || c.nwaves > c.strips || c.nwaves >= (1LL << 30)) return hipErrorInvalidConfiguration;
  // few wavefronts: one per workgroup, so that they spread over the compute units
  const int block = c.nwaves <= 2048 ? 64 : kBlock;
  const int64_t per = block / 64;
  dim3 grid((unsigned)((c.nwaves + per - 1) / per));
  c.ntiles = c.nwaves;            // row length of devpart for the reduction kernels
  c.normpart = c.dev2 + c.n;      // devsum's row n is ||xbar||^2
  c.norm_count = 1;
#define CECA_CW4(RT) case RT: cons_wave_kernel<4, RT><<<grid, dim3(block), 0, st>>>(c); break
#define CECA_CW1(RT) case RT: cons_wave_kernel<1, RT><<<grid, dim3(block), 0, st>>>(c); break
  if (vec4) {
    switch (c.rows_per_thread) {
      CECA_CW4(1); CECA_CW4(2); CECA_CW4(3); CECA_CW4(4); CECA_CW4(5); CECA_CW4(6); CECA_CW4(7); CECA_CW4(8);
      CECA_CW4(9); CECA_CW4(10); CECA_CW4(11); CECA_CW4(12); CECA_CW4(13); CECA_CW4(14); CECA_CW4(15); CECA_CW4(16);
      CECA_CW4(17); CECA_CW4(18); CECA_CW4(19); CECA_CW4(20); CECA_CW4(21); CECA_CW4(22); CECA_CW4(23); CECA_CW4(24);
      CECA_CW4(25); CECA_CW4(26); CECA_CW4(27); CECA_CW4(28); CECA_CW4(29); CECA_CW4(30); CECA_CW4(31); CECA_CW4(32);
    }
  } else {
    switch (c.rows_per_thread) {
      CECA_CW1(1); CECA_CW1(2); CECA_CW1(3); CECA_CW1(4); CECA_CW1(5); CECA_CW1(6); CECA_CW1(7); CECA_CW1(8);
      CECA_CW1(9); CECA_CW1(10); CECA_CW1(11); CECA_CW1(12); CECA_CW1(13); CECA_CW1(14); CECA_CW1(15); CECA_CW1(16);
      CECA_CW1(17); CECA_CW1(18); CECA_CW1(19); CECA_CW1(20); CECA_CW1(21); CECA_CW1(22); CECA_CW1(23); CECA_CW1(24);
      CECA_CW1(25); CECA_CW1(26); CECA_CW1(27); CECA_CW1(28); CECA_CW1(29); CECA_CW1(30); CECA_CW1(31); CECA_CW1(32);
    }
  }
#undef CECA_CW4
#undef CECA_CW1
  launch_close(c, c.n + 1, st);
  return hipGetLastError();
}

hipError_t launch_consensus(const ConsensusArgs& c0, bool vec4, hipStream_t st) {
  if (c0.wave_cgs > 0) return launch_cons_wave(c0, vec4, st);
  ConsensusArgs c = c0;
  c.norm_count = c.ntiles;        // one partial of ||xbar||^2 per column tile
  if (c.rows_per_thread > 0) return launch_cons_tile(c, vec4, st);
  const int vec = vec4 ? 4 : 1;
  const int64_t groups = (c.d + vec - 1) / vec;
  const int64_t gx = (groups + kBlock - 1) / kBlock;
  const int64_t dev_gy = ((int64_t)c.n + c.dev_agents - 1) / c.dev_agents;
  if (gx > 0x7fffffffLL || c.ntiles > 0x7fffffffLL || c.agent_groups > 65535 || dev_gy > 65535 || c.n > 0x7fffffff)
    return hipErrorInvalidConfiguration;
  dim3 block(kBlock);
  {
    dim3 grid((unsigned)gx, (unsigned)c.agent_groups);
    if (vec4) colsum_kernel<4><<<grid, block, 0, st>>>(c);
    else colsum_kernel<1><<<grid, block, 0, st>>>(c);
  }
  mean_kernel<<<dim3((unsigned)c.ntiles), block, 0, st>>>(c);
  {
    dim3 grid((unsigned)c.ntiles, (unsigned)dev_gy);
    if (vec4) dev_kernel<4><<<grid, block, 0, st>>>(c);
    else dev_kernel<1><<<grid, block, 0, st>>>(c);
  }
  launch_close(c, c.n, st);
  return hipGetLastError();
}

}  // namespace ceca
