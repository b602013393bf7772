// gfx950 kernels of the DSGD-CECA hot path.
//
// Layout: the state is 2n rows of ld floats (x rows then y rows); a workgroup is 256 threads
// (4 wavefronts of 64) and every thread owns 16-byte column groups, so each row access of a
// workgroup is one contiguous 4 KiB run.
//
// Chain walk.  In a round every row i needs the message of exactly one other row, peer(i), and
// peer is a permutation (Eqs. (5)-(7)): following i -> (i + stride) mod n visits rows in the
// order in which each one's message is needed by the next.  A thread therefore walks a stretch of
// such a cycle for its columns, keeping the message of the row it just finished in registers for
// the row it visits next, and every row is read from memory once per round instead of twice.
// A stretch that covers a whole cycle ("closed") holds its first row's terms until the walk comes
// back round; an open stretch fetches only the message of the row before its first one.
// One-port rounds are the closed two-row case of the same walk.
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

// ---------------------------------------------------------------------------------------------
// Chain-walk kernel: gossip round, fused quadratic-centre step, and combine-from-messages.
// ---------------------------------------------------------------------------------------------
template <typename V, int MODE, bool READ_Y> struct Raw { V x, y, aux; };

template <typename V, int MODE, bool READ_Y>
__device__ __forceinline__ Raw<V, MODE, READ_Y> load_raw(const ChainArgs& A, int agent, int64_t col) {
  Raw<V, MODE, READ_Y> r;
  const int64_t off = (int64_t)agent * A.ld + col;
  r.x = ld_stream<V>(A.xin + off);
  if (READ_Y) r.y = ld_stream<V>(A.yin + off); else r.y = V(0.0f);
  if (MODE != MODE_GOSSIP) r.aux = ld_stream<V>(A.aux + (int64_t)agent * A.ldaux + col); else r.aux = V(0.0f);
  return r;
}

// Self terms xs = x - lr e, ys = y - lr e and message v = z - lr e of one agent (Eqs. (8), (9)).
template <typename V, int MODE, bool EXCH_Y, bool READ_Y>
__device__ __forceinline__ void agent_terms(const ChainArgs& A, const Raw<V, MODE, READ_Y>& r, int agent,
                                            int64_t col, V& xs, V& ys, V& v) {
  // no fused multiply-add here or in message_only: a message must have the same bits whether its
  // own stretch or a neighbouring one computes it, so results do not depend on the launch shape
#pragma clang fp contract(off)
  const V z = EXCH_Y ? r.y : r.x;
  if (MODE == MODE_GOSSIP) {
    xs = r.x; ys = r.y; v = z;
  } else if (MODE == MODE_QUAD) {
    V e = z - r.aux;
    if (A.noise_std != 0.0f) e += A.noise_std * noise_group<V>(col, noise_keys(A.seed, A.k, (uint32_t)agent));
    const V ge = A.lr * e;
    xs = r.x - ge; ys = r.y - ge; v = z - ge;
  } else if (MODE == MODE_GRAD) {
    const V ge = A.lr * r.aux;
    xs = r.x - ge; ys = r.y - ge; v = z - ge;
  } else {  // MODE_FROMV: aux = v, so -lr e = v - z
    v = r.aux;
    const V dz = v - z;
    xs = EXCH_Y ? r.x + dz : v;
    ys = EXCH_Y ? v : r.y + dz;
  }
}

// Message of an agent whose own update belongs to another chain stretch.
template <typename V, int MODE, bool EXCH_Y>
__device__ __forceinline__ V message_only(const ChainArgs& A, int agent, int64_t col) {
#pragma clang fp contract(off)
  const int64_t off = (int64_t)agent * A.ld + col;
  if (MODE == MODE_FROMV) return ld_plain<V>(A.aux + (int64_t)agent * A.ldaux + col);
  const V z = ld_plain<V>((EXCH_Y ? A.yin : A.xin) + off);
  if (MODE == MODE_GOSSIP) return z;
  if (MODE == MODE_GRAD) return z - A.lr * ld_plain<V>(A.aux + (int64_t)agent * A.ldaux + col);
  V e = z - ld_plain<V>(A.aux + (int64_t)agent * A.ldaux + col);
  if (A.noise_std != 0.0f) e += A.noise_std * noise_group<V>(col, noise_keys(A.seed, A.k, (uint32_t)agent));
  const V ge = A.lr * e;
  return z - ge;
}

// Per-thread walk state: where the thread is on its cycle and the message of the row before.
template <typename V> struct Walk {
  int c;        // next row to visit
  V vprev;      // message of the row visited last
  V xs0, ys0;   // self terms of a closed stretch's first row, combined when the walk returns to it
};

template <typename V>
__device__ __forceinline__ void put_row(const ChainArgs& A, int row, int64_t col, V xs, V ys, V msg, bool read_y) {
  const int64_t off = (int64_t)row * A.ld + col;
  st_stream<V>(A.xout + off, combine(A.a, xs, A.ap, msg));
  st_stream<V>(A.yout + off, read_y ? combine(A.b, ys, A.bp, msg) : A.bp * msg);
}

// Q consecutive rows of the walk: all their loads are issued first, then the rows are finished in
// order (only the message passes from one to the next).  FIRST marks the opening block of a closed
// stretch, whose first row is held back instead of stored.
template <typename V, int MODE, bool EXCH_Y, bool READ_Y, int Q, bool FIRST>
__device__ __forceinline__ void walk_block(const ChainArgs& A, int64_t col, Walk<V>& w) {
  Raw<V, MODE, READ_Y> raw[Q];
  int row[Q];
#pragma unroll
  for (int j = 0; j < Q; ++j) {
    row[j] = w.c;
    w.c += A.stride;
    if (w.c >= A.n) w.c -= A.n;
  }
#pragma unroll
  for (int j = 0; j < Q; ++j) raw[j] = load_raw<V, MODE, READ_Y>(A, row[j], col);
#pragma unroll
  for (int j = 0; j < Q; ++j) {
    V xs, ys, v;
    agent_terms<V, MODE, EXCH_Y, READ_Y>(A, raw[j], row[j], col, xs, ys, v);
    if (FIRST && j == 0) {
      w.xs0 = xs; w.ys0 = ys;
    } else {
      put_row<V>(A, row[j], col, xs, ys, w.vprev, READ_Y);
    }
    w.vprev = v;
  }
}

template <typename V, int MODE, bool EXCH_Y, bool READ_Y, int R, bool FIRST>
__device__ __forceinline__ int walk_upto(const ChainArgs& A, int64_t col, Walk<V>& w, int remaining) {
  // one block of min(R, remaining) rows; returns how many rows it took
  if (remaining >= R) { walk_block<V, MODE, EXCH_Y, READ_Y, R, FIRST>(A, col, w); return R; }
  if (R > 4 && remaining >= 4) { walk_block<V, MODE, EXCH_Y, READ_Y, 4, FIRST>(A, col, w); return 4; }
  if (R > 2 && remaining >= 2) { walk_block<V, MODE, EXCH_Y, READ_Y, 2, FIRST>(A, col, w); return 2; }
  walk_block<V, MODE, EXCH_Y, READ_Y, 1, FIRST>(A, col, w);
  return 1;
}

template <int VEC, int MODE, bool EXCH_Y, bool READ_Y, int R>
__global__ __launch_bounds__(kBlock) void chain_kernel(const ChainArgs A) {
  using V = typename VecOf<VEC>::T;

  // Which stretch of which cycle this workgroup walks.  Workgroups are numbered band by band: a band
  // is `band` adjacent column tiles, and inside a band all tiles of one stretch come before the
  // next stretch along the cycle.  The device then sweeps a few rows of one band at a time, and the
  // message an open stretch re-reads was fetched by the stretch before it only moments earlier.
  const uint32_t per_band = A.band * A.nsegs;
  const uint32_t bnd = blockIdx.x / per_band;
  const uint32_t rem = blockIdx.x - bnd * per_band;
  const uint32_t width = min(A.band, A.tiles - bnd * A.band);     // the last band may be narrower
  const uint32_t seg = rem / width;
  const uint32_t tile = bnd * A.band + (rem - seg * width);
  const int64_t g = (int64_t)tile * kBlock + threadIdx.x;
  if (g >= A.ngroups) return;          // no barriers below: lanes past the last column just leave
  const int64_t col = A.col0 + g * VEC;

  const int cyc = (int)(seg / (uint32_t)A.segs_per_cycle);
  const int q = (int)seg - cyc * A.segs_per_cycle;
  const int t0 = q * A.seg_len;
  int remaining = min(A.seg_len, A.cyc_len - t0);
  const bool closed = (A.segs_per_cycle == 1);

  Walk<V> w;
  w.c = (int)(((int64_t)cyc * A.c0_mul + (int64_t)t0 * A.stride) % A.n);
  const int c_first = w.c;
  if (closed) {
    remaining -= walk_upto<V, MODE, EXCH_Y, READ_Y, R, true>(A, col, w, remaining);
  } else {
    int pred = w.c - A.stride;
    if (pred < 0) pred += A.n;
    w.vprev = message_only<V, MODE, EXCH_Y>(A, pred, col);
  }
  while (remaining >= R) {
    walk_block<V, MODE, EXCH_Y, READ_Y, R, false>(A, col, w);
    remaining -= R;
  }
  while (remaining > 0) remaining -= walk_upto<V, MODE, EXCH_Y, READ_Y, R, false>(A, col, w, remaining);
  if (closed) put_row<V>(A, c_first, col, w.xs0, w.ys0, w.vprev, READ_Y);
}

template <int VEC, int MODE, int R>
static hipError_t launch_chain_t(ChainArgs a, hipStream_t st) {
  const int64_t tiles = (a.ngroups + kBlock - 1) / kBlock;
  const int64_t ncyc = (int64_t)a.n / a.cyc_len;   // cycles are equal-length and cover all agents
  const int64_t blocks = tiles * ncyc * a.segs_per_cycle;
  // the runtime addresses at most 2^32 threads per launch
  if (tiles < 1 || blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  a.tiles = (uint32_t)tiles;
  a.nsegs = (uint32_t)(ncyc * a.segs_per_cycle);
  if (a.band == 0 || a.band > a.tiles) a.band = a.tiles;
  dim3 grid((unsigned)blocks), block(kBlock);
  // Unused dynamic LDS caps the workgroups resident on a CU (160 KiB of LDS each): fewer, fatter
  // workgroups keep the rows the device touches at any moment few, which the memory system rewards.
  size_t lds = 0;
  if (a.wg_per_cu > 0) {
    lds = (size_t)(160 * 1024 / a.wg_per_cu) & ~(size_t)1023;
    if (lds > 64 * 1024) lds = 64 * 1024;
  }
  if (a.exch_y) {
    // y travels only when delta_r = 0, and then b = 1/2: y is always read
    chain_kernel<VEC, MODE, true, true, R><<<grid, block, lds, st>>>(a);
  } else if (a.read_y) {
    chain_kernel<VEC, MODE, false, true, R><<<grid, block, lds, st>>>(a);
  } else {
    chain_kernel<VEC, MODE, false, false, R><<<grid, block, lds, st>>>(a);
  }
  return hipGetLastError();
}

hipError_t launch_chain(const ChainArgs& a, int mode, bool vec4, int rows, hipStream_t st) {
  if (a.ngroups <= 0) return hipSuccess;
#define CECA_CHAIN(M)                                                   \
  do {                                                                  \
    if (!vec4) return launch_chain_t<1, M, 2>(a, st);                   \
    switch (rows) {                                                     \
      case 1: return launch_chain_t<4, M, 1>(a, st);                    \
      case 2: return launch_chain_t<4, M, 2>(a, st);                    \
      case 8: return launch_chain_t<4, M, 8>(a, st);                    \
      default: return launch_chain_t<4, M, 4>(a, st);                   \
    }                                                                   \
  } while (0)
  switch (mode) {
    case MODE_GOSSIP: CECA_CHAIN(MODE_GOSSIP);
    case MODE_QUAD: CECA_CHAIN(MODE_QUAD);
    case MODE_FROMV: CECA_CHAIN(MODE_FROMV);
    case MODE_GRAD: CECA_CHAIN(MODE_GRAD);
  }
#undef CECA_CHAIN
  return hipErrorInvalidValue;
}

}  // namespace ceca
