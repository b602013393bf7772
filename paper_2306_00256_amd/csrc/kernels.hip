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
#include "launch.h"

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
  } else {  // MODE_FROMV: aux = v, so -lr e = v - z
    v = r.aux;
    const V dz = v - z;
    xs = EXCH_Y ? r.x + dz : v;
    ys = EXCH_Y ? v : r.y + dz;
  }
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

// Message of an agent whose own update belongs to another chain stretch.
template <typename V, int MODE, bool EXCH_Y>
__device__ __forceinline__ V message_only(const ChainArgs& A, int agent, int64_t col) {
#pragma clang fp contract(off)
  const int64_t off = (int64_t)agent * A.ld + col;
  if (MODE == MODE_FROMV) return ld_plain<V>(A.aux + (int64_t)agent * A.ldaux + col);
  const V z = ld_plain<V>((EXCH_Y ? A.yin : A.xin) + off);
  if (MODE == MODE_GOSSIP) return z;
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
  }
#undef CECA_CHAIN
  return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// Several gossip rounds in one pass: a workgroup keeps a column tile of every agent's (x, y) in
// registers and passes the travelling variable through LDS, so `rounds` rounds cost one read of x
// and one write of x and y (12 bytes per agent-parameter) instead of `rounds` x 16.  Columns are
// independent instances of the recursion (Sec. 3.1), and every round uses the same combine() as the
// single-round kernel, so the result has the same bits as `rounds` separate calls.
// ---------------------------------------------------------------------------------------------
template <int VEC, int RT>
__global__ __launch_bounds__(kBlock) void multi_round_kernel(const MultiArgs M) {
  using V = typename VecOf<VEC>::T;
  extern __shared__ float lds_z[];                 // [n][lanes] groups of VEC floats
  const int lanes = kBlock / M.row_lanes;          // column groups per row handled by this workgroup
  const int cg = threadIdx.x % lanes;              // my column group inside the tile
  const int rg = threadIdx.x / lanes;              // my first row; I own rows rg, rg + row_lanes, ...
  const int64_t g = (int64_t)blockIdx.x * lanes + cg;
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
  for (int t = 0; t < M.rounds; ++t) {
    const MultiRound R = M.round[t];
#pragma unroll
    for (int k = 0; k < RT; ++k) {
      const int i = rg + k * M.row_lanes;
      if (i < M.n) zs[i * lanes + cg] = R.exch_y ? y[k] : x[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < RT; ++k) {
      const int i = rg + k * M.row_lanes;
      if (i < M.n) {
        int p;
        if (M.port == 2) {
          p = i - R.shift; if (p < 0) p += M.n;
        } else {
          p = (i & 1) ? i - R.shift : i + R.shift;
          if (p < 0) p += M.n;
          if (p >= M.n) p -= M.n;
        }
        const V zp = zs[p * lanes + cg];
        x[k] = combine(R.a, x[k], R.ap, zp);
        y[k] = R.read_y ? combine(R.b, y[k], R.bp, zp) : R.bp * zp;
      }
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

hipError_t launch_multi_round(const MultiArgs& m, bool vec4, hipStream_t st) {
  if (m.ngroups <= 0) return hipSuccess;
  const int lanes = kBlock / m.row_lanes;
  const int64_t blocks = (m.ngroups + lanes - 1) / lanes;
  if (blocks < 1 || blocks >= (1LL << 24)) return hipErrorInvalidConfiguration;
  const size_t lds = (size_t)m.n * lanes * (vec4 ? 16 : 4);
  dim3 grid((unsigned)blocks), block(kBlock);
  if (vec4) multi_round_kernel<4, kMultiRows><<<grid, block, lds, st>>>(m);
  else multi_round_kernel<1, kMultiRows><<<grid, block, lds, st>>>(m);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Minibatch gradients of the GEMV-shaped losses: margins a_ij . z_i, then e_i and the message.
// ---------------------------------------------------------------------------------------------
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
// Sums N per-lane values across the 64 lanes of a wavefront at once.  Each butterfly step halves the
// number of values a lane carries (partners swap the halves they do not keep), so N values cost
// N - 1 + (6 - log2 N) lane exchanges instead of 6 N.  On return lane l < N holds the complete sum
// of value number `which`.
template <int N>
__device__ __forceinline__ float wave_sum_many(float (&m)[N], int lane, int& which) {
  static_assert(N >= 1 && N <= 64 && (N & (N - 1)) == 0, "N must be a power of two");
  which = 0;
  int bit = 0;
#pragma unroll
  for (int len = N; len > 1; len >>= 1, ++bit) {
    const bool up = (lane >> bit) & 1;
    const int half = len / 2;
#pragma unroll
    for (int k = 0; k < half; ++k) {
      const float send = up ? m[k] : m[k + half];
      const float keep = up ? m[k + half] : m[k];
      m[k] = keep + __shfl_xor(send, 1 << bit, 64);
    }
    which += up ? half : 0;
  }
  float v = m[0];
#pragma unroll
  for (int b = bit; b < 6; ++b) v += __shfl_xor(v, 1 << b, 64);
  return v;
}

__device__ __forceinline__ float dot_v(vf4 a, vf4 b) { return a.x * b.x + a.y * b.y + a.z * b.z + a.w * b.w; }
__device__ __forceinline__ float dot_v(float a, float b) { return a * b; }

// Minibatch row numbers are the same for every lane: keep them in scalar registers so that row
// addresses are scalar and all row loads can be issued back to back.
__device__ __forceinline__ int32_t uniform_i32(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
// A sampled row number, forced into [0, N): a bad index must not become a wild read.
__device__ __forceinline__ int32_t sample_row(int32_t v, int32_t N) { return min(max(uniform_i32(v), 0), N - 1); }

// partial[(agent * nchunks + chunk) * B + j] = sum over the chunk's columns of A[row_j][col] * z[agent][col].
// A workgroup takes one column chunk of kRowGroup sampled rows of one agent (grid: chunks x agents x row groups),
// so few agents still spread over many workgroups.
template <int VEC>
__global__ __launch_bounds__(kBlock) void margins_kernel(const GemvArgs G) {
  using V = typename VecOf<VEC>::T;
  __shared__ float red[kBlock / 64][kRowGroup];
  const int agent = blockIdx.y;
  const int chunk = blockIdx.x;
  const int j0 = blockIdx.z * kRowGroup;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // lanes past the last column read column 0 instead and carry z = 0: no branch surrounds a load
  const int64_t c = (int64_t)chunk * G.chunk_cols + (int64_t)threadIdx.x * VEC;
  const bool on = c + VEC <= G.d;
  const int64_t col = on ? c : 0;
  const V zv = ld_plain<V>(G.zin + (int64_t)agent * G.ld + col);
  const V z = on ? zv : V(0.0f);
  const int32_t* idx = G.batch_idx + (int64_t)agent * G.B;
  const float* Abase = G.A + (int64_t)agent * G.N * G.lda + col;
  V a[kRowGroup];
#pragma unroll
  for (int jj = 0; jj < kRowGroup; ++jj) {
    const int32_t rj = sample_row(idx[min(j0 + jj, G.B - 1)], G.N);   // rows past B repeat the last one
    a[jj] = ld_stream<V>(Abase + (int64_t)rj * G.lda);
  }
  float acc[kRowGroup];
#pragma unroll
  for (int jj = 0; jj < kRowGroup; ++jj) acc[jj] = dot_v(a[jj], z);
  int jj;
  const float s = wave_sum_many<kRowGroup>(acc, lane, jj);
  if (lane < kRowGroup) red[wave][jj] = s;
  __syncthreads();
  if ((int)threadIdx.x < kRowGroup && j0 + (int)threadIdx.x < G.B) {
    float t = 0.0f;
#pragma unroll
    for (int w = 0; w < kBlock / 64; ++w) t += red[w][threadIdx.x];
    G.partial[((int64_t)agent * G.nchunks + chunk) * G.B + j0 + threadIdx.x] = t;
  }
}

// Loss derivative at margin m with target / label t, already divided by the batch size.
__device__ __forceinline__ float loss_coef(int kind, float m, float t, float scale) {
  // LOGISTIC: -t * sigma(-t m) with sigma(-u) = 1 / (1 + e^u); e^u = inf gives 0, e^u = 0 gives 1
  const float cf = (kind == CECA_LOSS_LSQ) ? (m - t) : (-t / (1.0f + expf(t * m)));
  return cf * scale;
}

// v_i = z_i - lr * e_i with e_i = sum_j coef_j a_ij; coef_j folds the loss derivative and the 1/B.
template <int VEC>
__global__ __launch_bounds__(kBlock) void halfstep_kernel(const GemvArgs G) {
  using V = typename VecOf<VEC>::T;
  __shared__ float coef[64 + kRowGroup];
  __shared__ int32_t rowid[64 + kRowGroup];
  const int agent = blockIdx.y;
  if ((int)threadIdx.x < 64 + kRowGroup) {
    const int j = min((int)threadIdx.x, G.B - 1);
    float m = 0.0f;
    for (int ch = 0; ch < G.nchunks; ++ch) m += G.partial[((int64_t)agent * G.nchunks + ch) * G.B + j];
    const int32_t row = min(max(G.batch_idx[(int64_t)agent * G.B + j], 0), G.N - 1);
    const float t = G.t[(int64_t)agent * G.N + row];
    // entries past B repeat the last row with coefficient 0, so the row loop needs no bounds test
    coef[threadIdx.x] = ((int)threadIdx.x < G.B) ? loss_coef(G.kind, m, t, G.scale) : 0.0f;
    rowid[threadIdx.x] = row;
  }
  __syncthreads();
  const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
  if (col + VEC > G.d) return;
  V e = V(0.0f);
  const float* base = G.A + (int64_t)agent * G.N * G.lda + col;
  for (int j0 = 0; j0 < G.B; j0 += kRowGroup) {
    V r[kRowGroup];
#pragma unroll
    for (int jj = 0; jj < kRowGroup; ++jj) r[jj] = ld_stream<V>(base + (int64_t)uniform_i32(rowid[j0 + jj]) * G.lda);
#pragma unroll
    for (int jj = 0; jj < kRowGroup; ++jj) e += coef[j0 + jj] * r[jj];
  }
  if (G.noise_std != 0.0f) e += G.noise_std * noise_group<V>(col, noise_keys(G.seed, G.k, (uint32_t)agent));
  const V z = ld_plain<V>(G.zin + (int64_t)agent * G.ld + col);
  *reinterpret_cast<V*>(G.v + (int64_t)agent * G.ldv + col) = z - G.lr * e;
}

// One pass over the minibatch rows: a workgroup owns an agent, keeps its B sampled rows of A in
// registers (B x G 16-byte groups per thread), reduces the B margins across the workgroup, and forms
// v = z - lr * e from the same registers, so A is read from memory once per iteration.
template <int THREADS, int BMAX, int G>
__global__ __launch_bounds__(THREADS) void grad_onepass_kernel(const GemvArgs P) {
  constexpr int WAVES = THREADS / 64;
  __shared__ float red[WAVES][BMAX];
  __shared__ float coef[BMAX];
  const int agent = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // lanes past the last column read column 0 instead and carry z = 0: no branch surrounds a load
  int64_t col[G];
  bool on[G];
  vf4 z[G];
#pragma unroll
  for (int u = 0; u < G; ++u) {
    const int64_t c = ((int64_t)u * THREADS + threadIdx.x) * 4;
    on[u] = c < P.d;                       // d is a multiple of 4 on this path
    col[u] = on[u] ? c : 0;
    const vf4 zv = ld_plain<vf4>(P.zin + (int64_t)agent * P.ld + col[u]);
    z[u] = on[u] ? zv : vf4(0.0f);
  }
  const int32_t* idx = P.batch_idx + (int64_t)agent * P.B;
  const float* Abase = P.A + (int64_t)agent * P.N * P.lda;
  int32_t rowid[BMAX];
#pragma unroll
  for (int j = 0; j < BMAX; ++j) rowid[j] = sample_row(idx[min(j, P.B - 1)], P.N);   // rows past B repeat the last
  vf4 a[BMAX][G];
#pragma unroll
  for (int j = 0; j < BMAX; ++j) {
    const float* row = Abase + (int64_t)rowid[j] * P.lda;
#pragma unroll
    for (int u = 0; u < G; ++u) a[j][u] = ld_stream<vf4>(row + col[u]);
  }
  float m[BMAX];
#pragma unroll
  for (int j = 0; j < BMAX; ++j) {
    m[j] = 0.0f;
#pragma unroll
    for (int u = 0; u < G; ++u) m[j] += dot_v(a[j][u], z[u]);
  }
  int jrow;
  const float msum = wave_sum_many<BMAX>(m, lane, jrow);
  if (lane < BMAX) red[wave][jrow] = msum;
  __syncthreads();
  if ((int)threadIdx.x < BMAX) {
    const int j = threadIdx.x;
    float m = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) m += red[w][j];
    const float t = P.t[(int64_t)agent * P.N + min(max(idx[min(j, P.B - 1)], 0), P.N - 1)];
    coef[j] = (j < P.B) ? loss_coef(P.kind, m, t, P.scale) : 0.0f;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < G; ++u) {
    vf4 e = vf4(0.0f);
#pragma unroll
    for (int j = 0; j < BMAX; ++j) e += coef[j] * a[j][u];
    if (P.noise_std != 0.0f) e += P.noise_std * noise_group<vf4>(col[u], noise_keys(P.seed, P.k, (uint32_t)agent));
    if (on[u]) *reinterpret_cast<vf4*>(P.v + (int64_t)agent * P.ldv + col[u]) = z[u] - P.lr * e;
  }
}

// Picks the one-pass variant whose register tile covers (B, d); false if none does.
bool launch_grad_onepass(const GemvArgs& g, hipStream_t st, hipError_t* err) {
  const int64_t d4 = g.d / 4;
  dim3 grid((unsigned)g.n);
#define CECA_ONEPASS(T, BM, GG)                                          \
  if (g.B <= BM && d4 <= (int64_t)T * GG) {                              \
    grad_onepass_kernel<T, BM, GG><<<grid, dim3(T), 0, st>>>(g);         \
    *err = hipGetLastError();                                            \
    return true;                                                         \
  }
  CECA_ONEPASS(256, 16, 1)
  CECA_ONEPASS(256, 32, 1)
  CECA_ONEPASS(1024, 8, 1)
  CECA_ONEPASS(1024, 16, 1)
  CECA_ONEPASS(1024, 8, 2)
  CECA_ONEPASS(1024, 4, 4)
#undef CECA_ONEPASS
  return false;
}

hipError_t launch_margins(const GemvArgs& g, bool vec4, hipStream_t st) {
  if (g.nchunks < 1 || g.n > 65535) return hipErrorInvalidConfiguration;
  dim3 grid((unsigned)g.nchunks, (unsigned)g.n, (unsigned)((g.B + kRowGroup - 1) / kRowGroup)), block(kBlock);
  if (vec4) margins_kernel<4><<<grid, block, 0, st>>>(g);
  else margins_kernel<1><<<grid, block, 0, st>>>(g);
  return hipGetLastError();
}

hipError_t launch_halfstep(const GemvArgs& g, bool vec4, hipStream_t st) {
  const int vec = vec4 ? 4 : 1;
  const int64_t groups = (g.d + vec - 1) / vec;
  const int64_t gx = (groups + kBlock - 1) / kBlock;
  if (gx < 1 || gx > 0x7fffffffLL || g.n > 65535) return hipErrorInvalidConfiguration;
  dim3 grid((unsigned)gx, (unsigned)g.n), block(kBlock);
  if (vec4) halfstep_kernel<4><<<grid, block, 0, st>>>(g);
  else halfstep_kernel<1><<<grid, block, 0, st>>>(g);
  return hipGetLastError();
}

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

// dev2[agent] = sum over tiles of devpart[agent][tile]
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

__global__ __launch_bounds__(kBlock) void finish_kernel(const ConsensusArgs C) {
  __shared__ double r0[kBlock / 64], r1[kBlock / 64], r2[kBlock / 64], r3[kBlock / 64];
  double frob = 0.0, resid = 0.0, mx = 0.0, nrm = 0.0;
  for (int i = threadIdx.x; i < C.n; i += kBlock) {
    const double d2 = C.dev2[i];
    const double dv = sqrt(d2);
    frob += d2; resid += dv; mx = fmax(mx, dv);
  }
  for (int64_t t = threadIdx.x; t < C.ntiles; t += kBlock) nrm += C.normpart[t];
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

hipError_t launch_consensus(const ConsensusArgs& c, bool vec4, hipStream_t st) {
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
  devsum_kernel<<<dim3((unsigned)c.n), block, 0, st>>>(c);
  finish_kernel<<<dim3(1), block, 0, st>>>(c);
  return hipGetLastError();
}

}  // namespace ceca
