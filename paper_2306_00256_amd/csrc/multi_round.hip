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
  if (row_bytes >= 128 || *blocks < 1024 || g_tuning.plain_tile_order) return 0;   // small launches measured better in plain order
  const int64_t per = (*blocks + 7) / 8;
  *blocks = per * 8;
  return (int32_t)per;
}

// Wavefronts per SIMD the kernel is compiled for: workgroups wider than 256 threads hold many agents'
// rows and must fit 128 registers per thread (four wavefronts per SIMD: one 1024-thread workgroup or two
// 512-thread ones per compute unit); 256-thread workgroups take what their rows need.
template <int THREADS>
constexpr int multi_round_waves() { return THREADS > 256 ? 4 : 1; }
// The gossip-rounds kernel with 256 threads also comes in a register-lean form (LEAN > 0: that many
// wavefronts per SIMD, peers read from LDS two rows at a time): more workgroups are resident, so that some
// load or store while others exchange.
template <int THREADS, int LEAN>
constexpr int rounds_waves() { return LEAN > 0 ? LEAN : multi_round_waves<THREADS>(); }

// Peer slots of a round, per thread: my row k < RT - 1 sits in slot tid + k * THREADS and reads the slot
// `shift` rows before it (two ports), or `shift` rows ahead (even rows) / back (odd rows) with one port
// (Eq. (7)), modulo the tile.  base[p] is that slot for k = 0 with p the parity of k (my rows share one
// parity unless I hold consecutive rows); row k adds k * THREADS, which can pass the end of the tile once.
struct PeerSlots {
  int base[2];
  int last;     // peer slot of my last row (which may shadow agent n - 1)
};
template <int THREADS>
__device__ __forceinline__ int peer_slot(const PeerSlots& P, int k, int wrap) {
  const int t = P.base[k & 1] + k * THREADS;               // in [0, 2 * wrap)
  return (int)min((unsigned)t, (unsigned)(t - wrap));      // t - wrap when that is not negative
}
__device__ __forceinline__ int wrap_slot(int s, int wrap) {   // s in (-wrap, 2 * wrap)
  if (s < 0) s += wrap;
  return (int)min((unsigned)s, (unsigned)(s - wrap));
}

template <int VEC, int RT, int THREADS, int LEAN>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(rounds_waves<THREADS, LEAN>())))
void multi_round_kernel(const MultiArgs M) {
  using V = typename VecOf<VEC>::T;
  extern __shared__ float lds_z[];                 // [n][lanes] groups of VEC floats
  const int lanes = THREADS / M.row_lanes;         // column groups per row handled by this workgroup
  const int tid = threadIdx.x;
  const int cg = tid % lanes;                      // my column group inside the tile
  const int rg = tid / lanes;                      // my first row; I own rows rg, rg + row_lanes, ...
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
    y[k] = V(-0.0f);                               // y(0) is never read: the first round has b = 0
  }
  V* zs = reinterpret_cast<V*>(lds_z);
  // Row i, column group c sits in LDS slot i * lanes + c, so my row k is slot tid + k * THREADS
  // (row_lanes * lanes = THREADS).  rows_per_thread is the least that covers n, so only my last row can
  // lie past the last agent: it then shadows agent n - 1 and is never published.
  constexpr int L = RT - 1;
  const bool last_mine = rg + L * M.row_lanes < M.n;
  const int slot_last = last_mine ? tid + L * THREADS : (M.n - 1) * lanes + cg;
  const int wrap = M.n * lanes;
  // one port: even rows look ahead, odd rows back (Eq. (7)); my rows rg + k * row_lanes share rg's parity
  // unless I hold consecutive rows (row_lanes = 1, then rg = 0 and row k has the parity of k)
  const bool odd0 = (rg & 1) != 0;
  const bool odd1 = M.row_lanes == 1 ? !odd0 : odd0;
  const bool odd_last = ((min(rg + L * M.row_lanes, M.n - 1)) & 1) != 0;
  // a thread with no row below its last one (RT = 1 past the last agent) keeps tid inside the tile
  const int slot0 = min(tid, wrap - 1);
  // rows whose messages are read from LDS together: all of them, or a few at a time where registers are short
  constexpr int KB = ((THREADS > 256 || LEAN > 0) && RT > 4) ? (RT > 7 || LEAN > 0 ? 2 : 4) : RT;
  // The loop body below is one straight line that replaces x and y where they are: the round's flags only
  // steer which variable is published and whether y restarts, never two versions of the arithmetic (with
  // several bodies to choose from, the compiler keeps a second copy of the tile and moves it back every round).
  for (int t = 0; t < M.rounds; ++t) {
    const MultiRound R = M.round[t];
    if (R.exch_y) {
#pragma unroll
      for (int k = 0; k < L; ++k) zs[tid + k * THREADS] = y[k];
      if (last_mine) zs[slot_last] = y[L];
    } else {
#pragma unroll
      for (int k = 0; k < L; ++k) zs[tid + k * THREADS] = x[k];
      if (last_mine) zs[slot_last] = x[L];
    }
    // b = 0 (round 0 of a cycle): y is not used.  From y = -0 the combine below gives b_peer * z to the
    // bit (0 * -0 = -0, and adding -0 changes nothing, not even the sign of a zero).
    if (!R.read_y) {
#pragma unroll
      for (int k = 0; k < RT; ++k) y[k] = V(-0.0f);
    }
    const int back = R.shift * lanes;
    const int fwd = M.port == 2 ? -back : back;    // two ports: every row reads `shift` rows back
    PeerSlots P;
    P.base[0] = wrap_slot(slot0 + (odd0 ? -back : fwd), wrap);
    P.base[1] = wrap_slot(slot0 + (odd1 ? -back : fwd), wrap);
    P.last = wrap_slot(slot_last + (odd_last ? -back : fwd), wrap);
    __syncthreads();
#pragma unroll
    for (int k0 = 0; k0 < RT; k0 += KB) {
      // no branch around the LDS reads, so the reads of a batch issue back to back
      V zp[KB];
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        const int k = k0 + j;
        if (k < RT) zp[j] = zs[k == L ? P.last : peer_slot<THREADS>(P, k, wrap)];
      }
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        const int k = k0 + j;
        if (k < RT) {
          x[k] = combine(R.a, x[k], R.ap, zp[j]);
          y[k] = combine(R.b, y[k], R.bp, zp[j]);
        }
      }
      if (KB < RT) __builtin_amdgcn_sched_barrier(0);    // keep the batches apart
    }
    __syncthreads();
  }
  if (!on) return;
  // the row addresses are worked out here, after the rounds: nothing of them occupies registers meanwhile
  int rg_out = rg;
  asm volatile("" : "+v"(rg_out));
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg_out + k * M.row_lanes;
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
template <int VEC, int RT, int THREADS>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(multi_round_waves<THREADS>())))
void multi_step_kernel(const StepsArgs S) {
#pragma clang fp contract(off)
  using V = typename VecOf<VEC>::T;
  const MultiArgs& M = S.m;
  extern __shared__ float lds_z[];                 // [n][lanes] groups of VEC floats
  const int lanes = THREADS / M.row_lanes;
  const int tid = threadIdx.x;
  const int cg = tid % lanes;
  const int rg = tid / lanes;
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
  // Row i, column group c sits in LDS slot i * lanes + c, so my row k is slot tid + k * THREADS
  // (row_lanes * lanes = THREADS).  rows_per_thread is the least that covers n, so only my last row can
  // lie past the last agent: it then shadows agent n - 1 and is never published.
  constexpr int L = RT - 1;
  const bool last_mine = rg + L * M.row_lanes < M.n;
  const int slot_last = last_mine ? tid + L * THREADS : (M.n - 1) * lanes + cg;
  const int wrap = M.n * lanes;
  const bool alternate = M.row_lanes == 1;         // one port: my rows share rg's parity unless consecutive
  const bool rg_odd = (rg & 1) != 0;
  for (int t = 0; t < M.rounds; ++t) {
    const MultiRound R = M.round[t];
    // Local step of row k at z (its x or y): both x and y move by lr * e (Algorithm 1; x - lr e and
    // y - lr e are what Eqs. (8), (9) combine), and the moved z is the message v.
    auto local_step = [&](int k, const V& z) {
      const int i = min(rg + k * M.row_lanes, M.n - 1);
      V e = z - c[k];
      if (S.noise_std != 0.0f) e += S.noise_std * noise_group<V>(col, noise_keys(S.seed, S.k0 + (uint32_t)t, (uint32_t)i));
      const V ge = S.lr * e;
      x[k] = x[k] - ge;
      y[k] = y[k] - ge;
    };
    // the round's flags are the same for every thread: branches, not per-element selects
    if (R.exch_y) {
#pragma unroll
      for (int k = 0; k < RT; ++k) {
        local_step(k, y[k]);
        if (k < L) zs[tid + k * THREADS] = y[k];
        else if (last_mine) zs[slot_last] = y[k];
        if (THREADS > 256) __builtin_amdgcn_sched_barrier(0);     // row by row where registers are short
      }
    } else {
#pragma unroll
      for (int k = 0; k < RT; ++k) {
        local_step(k, x[k]);
        if (k < L) zs[tid + k * THREADS] = x[k];
        else if (last_mine) zs[slot_last] = x[k];
        if (THREADS > 256) __builtin_amdgcn_sched_barrier(0);     // row by row where registers are short
      }
    }
    __syncthreads();
    const int back = R.shift * lanes;
    // rows whose messages are read from LDS together: all of them, or two at a time where registers are short
    constexpr int KB = (THREADS > 256 && RT > 2) ? 2 : RT;
#pragma unroll
    for (int k0 = 0; k0 < RT; k0 += KB) {
      V zp[KB];
#pragma unroll
      for (int j = 0; j < KB; ++j) {
        const int k = k0 + j;
        if (k < RT) {
          const int s = (k == L) ? slot_last : tid + k * THREADS;
          int q;
          if (M.port == 2) {
            q = s - back;
            if (q < 0) q += wrap;
          } else {
            const bool odd = alternate ? ((k & 1) != 0) : rg_odd;   // even rows look ahead, odd rows back (Eq. (7))
            q = odd ? s - back : s + back;
            if (q < 0) q += wrap;
            if (q >= wrap) q -= wrap;
          }
          zp[j] = zs[q];
        }
      }
#pragma unroll
      for (int j = 0; j < KB; ++j)
        if (k0 + j < RT) x[k0 + j] = combine(R.a, x[k0 + j], R.ap, zp[j]);
      if (R.read_y) {
#pragma unroll
        for (int j = 0; j < KB; ++j)
          if (k0 + j < RT) y[k0 + j] = combine(R.b, y[k0 + j], R.bp, zp[j]);
      } else {
#pragma unroll
        for (int j = 0; j < KB; ++j)
          if (k0 + j < RT) y[k0 + j] = R.bp * zp[j];
      }
      if (KB < RT) __builtin_amdgcn_sched_barrier(0);    // keep the batches apart
    }
    __syncthreads();
  }
  if (!on) return;
  // the row addresses are worked out here, after the iterations: nothing of them occupies registers meanwhile
  int rg_out = rg;
  asm volatile("" : "+v"(rg_out));
#pragma unroll
  for (int k = 0; k < RT; ++k) {
    const int i = rg_out + k * M.row_lanes;
    if (i < M.n) {
      st_stream<V>(M.xout + (int64_t)i * M.ld + col, x[k]);
      st_stream<V>(M.yout + (int64_t)i * M.ld + col, y[k]);
    }
  }
}

template <int VEC, int RT, int THREADS>
static hipError_t launch_steps(const StepsArgs& ss, unsigned blocks, size_t lds, hipStream_t st) {
  if (lds > 64 * 1024) {
    // more than 64 KB of LDS per workgroup has to be asked for
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&multi_step_kernel<VEC, RT, THREADS>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  multi_step_kernel<VEC, RT, THREADS><<<dim3(blocks), dim3(THREADS), lds, st>>>(ss);
  return hipGetLastError();
}

// 256-thread workgroups: up to 16 rows per thread
template <int VEC>
static hipError_t launch_steps_256(const StepsArgs& ss, unsigned blocks, size_t lds, hipStream_t st) {
  switch (ss.m.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_steps<VEC, RT, 256>(ss, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
    CECA_RT(9); CECA_RT(10); CECA_RT(11); CECA_RT(12); CECA_RT(13); CECA_RT(14); CECA_RT(15); CECA_RT(16);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

// wider workgroups (16-byte groups only): x, y and c of up to kStepsWideRows rows fit their 128 registers
template <int THREADS>
static hipError_t launch_steps_wide(const StepsArgs& ss, unsigned blocks, size_t lds, hipStream_t st) {
  switch (ss.m.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_steps<4, RT, THREADS>(ss, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

hipError_t launch_multi_step(const StepsArgs& s, bool vec4, hipStream_t st) {
  const MultiArgs& m = s.m;
  if (m.ngroups <= 0) return hipSuccess;
  const int threads = m.threads > 0 ? m.threads : kBlock;
  if (threads != 256 && threads != 512 && threads != 1024) return hipErrorInvalidValue;
  if (!vec4 && threads != 256) return hipErrorInvalidValue;          // scalar columns: 256-thread tiles only
  if (m.row_lanes < 1 || m.row_lanes > threads || (m.row_lanes & (m.row_lanes - 1)) != 0) return hipErrorInvalidValue;
  // the kernel relies on rows_per_thread being the least that covers n (only a thread's last row can
  // lie past the last agent)
  if (m.rows_per_thread < 1 || m.rows_per_thread > kMultiRows ||
      (int64_t)m.rows_per_thread * m.row_lanes < m.n || (int64_t)(m.rows_per_thread - 1) * m.row_lanes >= m.n)
    return hipErrorInvalidValue;
  const int lanes = threads / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  StepsArgs ss = s;
  ss.m.xcd_tiles = xcd_run(lanes * (vec4 ? 16 : 4), &blocks);
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  if (lds > kMultiMaxLds) return hipErrorInvalidValue;
  if (!vec4) return launch_steps_256<1>(ss, (unsigned)blocks, lds, st);
  if (threads == 256) return launch_steps_256<4>(ss, (unsigned)blocks, lds, st);
  if (threads == 512) return launch_steps_wide<512>(ss, (unsigned)blocks, lds, st);
  return launch_steps_wide<1024>(ss, (unsigned)blocks, lds, st);
}

template <int VEC, int RT, int THREADS, int LEAN>
static hipError_t launch_rounds(const MultiArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  if (lds > 64 * 1024) {
    // more than 64 KB of LDS per workgroup has to be asked for
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&multi_round_kernel<VEC, RT, THREADS, LEAN>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  multi_round_kernel<VEC, RT, THREADS, LEAN><<<dim3(blocks), dim3(THREADS), lds, st>>>(mm);
  return hipGetLastError();
}

template <int VEC, int THREADS, int LEAN = 0>
static hipError_t launch_rounds_rt(const MultiArgs& mm, unsigned blocks, size_t lds, hipStream_t st) {
  switch (mm.rows_per_thread) {
#define CECA_RT(RT) case RT: return launch_rounds<VEC, RT, THREADS, LEAN>(mm, blocks, lds, st)
    CECA_RT(1); CECA_RT(2); CECA_RT(3); CECA_RT(4); CECA_RT(5); CECA_RT(6); CECA_RT(7); CECA_RT(8);
    CECA_RT(9); CECA_RT(10); CECA_RT(11); CECA_RT(12); CECA_RT(13); CECA_RT(14); CECA_RT(15); CECA_RT(16);
#undef CECA_RT
  }
  return hipErrorInvalidValue;
}

hipError_t launch_multi_round(const MultiArgs& m, bool vec4, hipStream_t st) {
  if (m.ngroups <= 0) return hipSuccess;
  const int threads = m.threads > 0 ? m.threads : kBlock;
  if (threads != 256 && threads != 512 && threads != 1024) return hipErrorInvalidValue;
  if (!vec4 && threads != 256) return hipErrorInvalidValue;          // scalar columns: 256-thread tiles only
  if (m.row_lanes < 1 || m.row_lanes > threads || (m.row_lanes & (m.row_lanes - 1)) != 0) return hipErrorInvalidValue;
  // the kernel relies on rows_per_thread being the least that covers n (only a thread's last row can
  // lie past the last agent)
  if (m.rows_per_thread < 1 || m.rows_per_thread > kMultiRows ||
      (int64_t)m.rows_per_thread * m.row_lanes < m.n || (int64_t)(m.rows_per_thread - 1) * m.row_lanes >= m.n)
    return hipErrorInvalidValue;
  const int lanes = threads / m.row_lanes;
  int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  MultiArgs mm = m;
  mm.xcd_tiles = xcd_run(lanes * (vec4 ? 16 : 4), &blocks);
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  if (lds > kMultiMaxLds) return hipErrorInvalidValue;
  if (!vec4) return launch_rounds_rt<1, 256>(mm, (unsigned)blocks, lds, st);
  if (threads == 256 && m.lean == 4) return launch_rounds_rt<4, 256, 4>(mm, (unsigned)blocks, lds, st);
  if (threads == 256 && m.lean == 5) return launch_rounds_rt<4, 256, 5>(mm, (unsigned)blocks, lds, st);
  if (threads == 256 && m.lean == 6) return launch_rounds_rt<4, 256, 6>(mm, (unsigned)blocks, lds, st);
  if (threads == 256) return launch_rounds_rt<4, 256>(mm, (unsigned)blocks, lds, st);
  if (threads == 512) return launch_rounds_rt<4, 512>(mm, (unsigned)blocks, lds, st);
  return launch_rounds_rt<4, 1024>(mm, (unsigned)blocks, lds, st);
}

}  // namespace ceca
