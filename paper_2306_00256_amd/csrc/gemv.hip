// Minibatch gradients of the GEMV-shaped losses for gfx950: margins a_ij . z_i, then e_i and the message.
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

// Minibatch row numbers are the same for every lane: keep them in scalar registers so that row
// addresses are scalar and all row loads can be issued back to back.
__device__ __forceinline__ int32_t uniform_i32(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }
// Sampled row numbers are forced into [0, N) wherever they are used: a bad index must not become a
// wild read.

// partial[(agent * nchunks + chunk) * B + j] = sum over the chunk's columns of A[row_j][col] * z[agent][col].
// A workgroup takes one column chunk of kRowGroup sampled rows of one agent (grid: chunks x agents x row groups),
// so few agents still spread over many workgroups.
// FUSE: the workgroup first finishes the iteration before for its agent and columns -- x+, y+ from x, y,
// its own message and its peer's (Eqs. (8), (9), with the arithmetic of the combine kernel, operation
// for operation) -- and takes the margins at the new z.  Every row group of an (agent, chunk) pair
// computes the same x+, y+; the first one stores them, into a buffer other than the one they are read
// from (the row groups run at the same time).
template <int VEC, bool FUSE>
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
  V zv;
  if (FUSE) {
#pragma clang fp contract(off)
    int p;
    if (G.p_port == 2) {
      p = agent - G.p_shift; if (p < 0) p += G.n;
    } else {
      p = (agent & 1) ? agent - G.p_shift : agent + G.p_shift;
      if (p < 0) p += G.n;
      if (p >= G.n) p -= G.n;
    }
    const int64_t off = (int64_t)agent * G.ld + col;
    const V x = ld_plain<V>(G.px + off);
    const V y = G.p_read_y || G.p_exch_y ? ld_plain<V>(G.py + off) : V(0.0f);
    const V v = ld_plain<V>(G.pv + (int64_t)agent * G.ldv + col);
    const V msg = ld_plain<V>(G.pv + (int64_t)p * G.ldv + col);
    const V dz = v - (G.p_exch_y ? y : x);          // -lr e of the iteration before
    const V xs = G.p_exch_y ? x + dz : v;
    const V ys = G.p_exch_y ? v : y + dz;
    const V xn = combine(G.pa, xs, G.pap, msg);
    const V yn = G.p_read_y ? combine(G.pb, ys, G.pbp, msg) : G.pbp * msg;
    if (on && blockIdx.z == 0) {
      const int64_t oo = (int64_t)agent * G.ldo + col;
      *reinterpret_cast<V*>(G.ox + oo) = xn;
      *reinterpret_cast<V*>(G.oy + oo) = yn;
    }
    zv = G.new_exch_y ? yn : xn;
  } else {
    zv = ld_plain<V>(G.zin + (int64_t)agent * G.ld + col);
  }
  const V z = on ? zv : V(0.0f);
  const int32_t* idx = G.batch_idx + (int64_t)agent * G.B;
  const float* Abase = G.A + (int64_t)agent * G.N * G.lda + col;
  // one vector load for the group's sample numbers (lane jj holds sample j0 + jj; samples past B repeat
  // the last), made scalar lane by lane: scalar loads would each wait for the one before
  const int32_t myidx = idx[min(j0 + min(lane, kRowGroup - 1), G.B - 1)];
  V a[kRowGroup];
#pragma unroll
  for (int jj = 0; jj < kRowGroup; ++jj) {
    const int32_t rj = min(max(__builtin_amdgcn_readlane(myidx, jj), 0), G.N - 1);
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
  __shared__ float red[2][WAVES][BMAX];   // alternating between a workgroup's agents: one barrier per agent
  static_assert(BMAX <= 64, "one lane per sampled row");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // lanes past the last column read column 0 instead and carry z = 0: no branch surrounds a load
  int64_t col[G];
  bool on[G];
#pragma unroll
  for (int u = 0; u < G; ++u) {
    const int64_t c = ((int64_t)u * THREADS + threadIdx.x) * 4;
    on[u] = c < P.d;                       // d is a multiple of 4 on this path
    col[u] = on[u] ? c : 0;
  }
  // A workgroup takes agents blockIdx.x, blockIdx.x + gridDim.x, ...  The next agent's batch numbers
  // and z are requested while the current agent is being worked on, so only the first agent of a
  // workgroup waits for them before its rows can be requested.
  // One vector load brings a whole batch into a wavefront (lane j holds sample j; samples past B repeat
  // the last); the row numbers then become scalars lane by lane: B scalar loads would each wait for
  // the one before, because scalar loads return out of order.
  int agent = blockIdx.x;
  int32_t idx_next = P.batch_idx[(int64_t)agent * P.B + min(lane, P.B - 1)];
  vf4 z_next[G];
#pragma unroll
  for (int u = 0; u < G; ++u) z_next[u] = ld_plain<vf4>(P.zin + (int64_t)agent * P.ld + col[u]);
  for (int turn = 0; agent < P.n; agent += gridDim.x, turn ^= 1) {
    const int32_t myidx = idx_next;
    vf4 z[G];
#pragma unroll
    for (int u = 0; u < G; ++u) z[u] = on[u] ? z_next[u] : vf4(0.0f);
    const float* Abase = P.A + (int64_t)agent * P.N * P.lda;
    int32_t rowid[BMAX];
#pragma unroll
    for (int j = 0; j < BMAX; ++j) rowid[j] = min(max(__builtin_amdgcn_readlane(myidx, j), 0), P.N - 1);
    vf4 a[BMAX][G];
#pragma unroll
    for (int j = 0; j < BMAX; ++j) {
      const float* row = Abase + (int64_t)rowid[j] * P.lda;
#pragma unroll
      for (int u = 0; u < G; ++u) a[j][u] = ld_stream<vf4>(row + col[u]);
    }
    // the target of "my" sampled row (lanes 0 .. BMAX-1 of every wavefront turn margins into
    // coefficients later) is requested here, behind the rows, so that nothing waits for it after the
    // barrier; the row number comes from the scalar row ids, so nothing has to arrive first
    int32_t rmine = rowid[0];
#pragma unroll
    for (int j = 1; j < BMAX; ++j) rmine = (lane == j) ? rowid[j] : rmine;
    const float tmine = P.t[(int64_t)agent * P.N + rmine];
    // what the next agent of this workgroup needs first (the last one re-reads its own: no branch)
    const int nxt = agent + (int)gridDim.x < P.n ? agent + (int)gridDim.x : agent;
    idx_next = P.batch_idx[(int64_t)nxt * P.B + min(lane, P.B - 1)];
#pragma unroll
    for (int u = 0; u < G; ++u) z_next[u] = ld_plain<vf4>(P.zin + (int64_t)nxt * P.ld + col[u]);
    // every load above is issued before any arithmetic below: the scheduler must not trade loads in
    // flight for registers here (it split the rows into two dependent batches when left alone)
    __builtin_amdgcn_sched_barrier(0);
    float m[BMAX];
#pragma unroll
    for (int j = 0; j < BMAX; ++j) {
      m[j] = 0.0f;
#pragma unroll
      for (int u = 0; u < G; ++u) m[j] += dot_v(a[j][u], z[u]);
    }
    constexpr int CH = BMAX < 16 ? BMAX : 16;        // margins are summed across the wavefront 16 at a time
#pragma unroll
    for (int c0 = 0; c0 < BMAX; c0 += CH) {
      float part[CH];
#pragma unroll
      for (int k = 0; k < CH; ++k) part[k] = m[c0 + k];
      int jrow;
      const float msum = wave_sum_many<CH>(part, lane, jrow);
      if (lane < CH) red[turn][wave][c0 + jrow] = msum;
    }
    __syncthreads();
    // every wavefront turns the margins into coefficients for itself (lane j: sample j, same summation
    // order everywhere), so no second barrier and no LDS round trip for the coefficients
    float cmine = 0.0f;
    {
      const int j = min(lane, BMAX - 1);
      float mj = 0.0f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) mj += red[turn][w][j];
      cmine = (lane < P.B) ? loss_coef(P.kind, mj, tmine, P.scale) : 0.0f;
    }
    float coef[BMAX];                                 // wavefront-uniform: scalar registers
#pragma unroll
    for (int j = 0; j < BMAX; ++j) coef[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cmine), j));
#pragma unroll
    for (int u = 0; u < G; ++u) {
      vf4 e = vf4(0.0f);
#pragma unroll
      for (int j = 0; j < BMAX; ++j) e += coef[j] * a[j][u];
      if (P.noise_std != 0.0f) e += P.noise_std * noise_group<vf4>(col[u], noise_keys(P.seed, P.k, (uint32_t)agent));
      if (on[u]) *reinterpret_cast<vf4*>(P.v + (int64_t)agent * P.ldv + col[u]) = z[u] - P.lr * e;
    }
  }
}

// The same computation with the batch taken CH rows at a time: only CH rows of A are in registers at
// once, so two 1024-thread workgroups fit a compute unit and one computes while the other waits for
// its rows.  e accumulates over the samples in the same order as in the kernel above.
// (One column group per thread fits 64 registers, i.e. two 1024-thread workgroups per unit; wider rows
// take up to 128 registers and one such workgroup per unit, but still any batch size.)
// FUSE: the workgroup first finishes the iteration before for its agent -- x+, y+ from x, y, its own
// message and its peer's (Eqs. (8), (9), with the arithmetic of the combine kernel, operation for
// operation) -- stores them, and takes the gradient at the new z.  One launch per iteration instead
// of two, and the state rows (cache resident at these sizes) are touched once.
// FUSE = 2: the state between iterations is kept in half-step form -- rows xs = x - lr e, ys = y - lr e of
// the iteration before (the travelling one of the two IS that iteration's message, bit for bit) -- so the
// prologue reads its own two rows and one row of its peer, combines in registers without storing x+, y+,
// and the epilogue writes the new half-step rows to the other buffer: 20 bytes of state traffic per
// agent-parameter and iteration instead of 28, with the arithmetic of FUSE = 1 operation for operation.
// VEC = 1 is the same kernel on single columns, for layouts that are not 16-byte aligned.
template <int VEC, int THREADS, int CH, int G, int FUSE>
__global__ __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(G == 1 ? 8 : 4, 8)))
void grad_chunked_kernel(const GemvArgs P) {
  using V = typename VecOf<VEC>::T;
  constexpr int WAVES = THREADS / 64;
  __shared__ float red[2][WAVES][CH];     // alternating between chunks: one barrier per chunk
  static_assert(CH <= 16, "one wavefront sum per chunk");
  const int agent = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t col[G];
  bool on[G];
  V z[G], e[G];
  // FUSE = 2: the variable that does not travel this iteration, after the combine.  It is needed again only in
  // the epilogue and waits in LDS meanwhile (in registers it pushed three others out to scratch memory,
  // 8 MB of extra writes per iteration at n = 1023, d = 4096); a thread reads back what it wrote itself.
  __shared__ V other_s[FUSE == 2 ? THREADS * G : 1];
#pragma unroll
  for (int u = 0; u < G; ++u) {
    const int64_t c = ((int64_t)u * THREADS + threadIdx.x) * VEC;
    on[u] = c < P.d;                       // d is a multiple of VEC
    col[u] = on[u] ? c : 0;
  }
  const float* Abase = P.A + (int64_t)agent * P.N * P.lda;
  // lane j holds sample j of the whole batch (B <= 64; samples past B repeat the last)
  const int32_t myidx = min(max(P.batch_idx[(int64_t)agent * P.B + min(lane, P.B - 1)], 0), P.N - 1);
  const float tmine = P.t[(int64_t)agent * P.N + myidx];
  V a[CH][G];
  // rows c0 .. c0 + CH - 1 of the batch into the register tile
  auto request_rows = [&](int c0) {
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const int32_t rj = __builtin_amdgcn_readlane(myidx, min(c0 + j, 63));
      const float* row = Abase + (int64_t)rj * P.lda;
#pragma unroll
      for (int u = 0; u < G; ++u) a[j][u] = ld_stream<V>(row + col[u]);
    }
  };
  // without the prologue the first rows are requested before z; with it they follow it: the prologue
  // needs 24 registers of its own, and loads return in order anyway
  if (FUSE == 0) request_rows(0);
#pragma unroll
  for (int u = 0; u < G; ++u) {
    V zv;
    if (FUSE == 2) {
#pragma clang fp contract(off)
      const int64_t off = (int64_t)agent * P.ld + col[u];
      const V hx = ld_plain<V>(P.px + off);
      const V hy = ld_plain<V>(P.py + off);
      V xn = hx, yn = hy;                  // the call's first iteration starts from x, y themselves
      if (!P.p_first) {
        int p;
        if (P.p_port == 2) {
          p = agent - P.p_shift; if (p < 0) p += P.n;
        } else {
          p = (agent & 1) ? agent - P.p_shift : agent + P.p_shift;
          if (p < 0) p += P.n;
          if (p >= P.n) p -= P.n;
        }
        // the peer's message is the travelling row of its half-step state
        const V msg = ld_plain<V>((P.p_exch_y ? P.py : P.px) + (int64_t)p * P.ld + col[u]);
        xn = combine(P.pa, hx, P.pap, msg);
        yn = P.p_read_y ? combine(P.pb, hy, P.pbp, msg) : P.pbp * msg;
      }
      zv = P.new_exch_y ? yn : xn;
      other_s[u * THREADS + threadIdx.x] = P.new_exch_y ? xn : yn;
    } else if (FUSE == 1) {
#pragma clang fp contract(off)
      int p;
      if (P.p_port == 2) {
        p = agent - P.p_shift; if (p < 0) p += P.n;
      } else {
        p = (agent & 1) ? agent - P.p_shift : agent + P.p_shift;
        if (p < 0) p += P.n;
        if (p >= P.n) p -= P.n;
      }
      const int64_t off = (int64_t)agent * P.ld + col[u];
      const V x = ld_plain<V>(P.px + off);
      const V y = P.p_read_y || P.p_exch_y ? ld_plain<V>(P.py + off) : V(0.0f);
      const V v = ld_plain<V>(P.pv + (int64_t)agent * P.ldv + col[u]);
      const V msg = ld_plain<V>(P.pv + (int64_t)p * P.ldv + col[u]);
      const V dz = v - (P.p_exch_y ? y : x);        // -lr e of the iteration before
      const V xs = P.p_exch_y ? x + dz : v;
      const V ys = P.p_exch_y ? v : y + dz;
      const V xn = combine(P.pa, xs, P.pap, msg);
      const V yn = P.p_read_y ? combine(P.pb, ys, P.pbp, msg) : P.pbp * msg;
      if (on[u]) {
        *reinterpret_cast<V*>(P.ox + off) = xn;
        *reinterpret_cast<V*>(P.oy + off) = yn;
      }
      zv = P.new_exch_y ? yn : xn;
    } else {
      zv = ld_plain<V>(P.zin + (int64_t)agent * P.ld + col[u]);
    }
    z[u] = on[u] ? zv : V(0.0f);
    e[u] = V(0.0f);
  }
  if (FUSE != 0) request_rows(0);
  int turn = 0;
  for (int c0 = 0; c0 < P.B; c0 += CH, turn ^= 1) {
    float m[CH];
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      m[j] = 0.0f;
#pragma unroll
      for (int u = 0; u < G; ++u) m[j] += dot_v(a[j][u], z[u]);
    }
    int jrow;
    const float msum = wave_sum_many<CH>(m, lane, jrow);
    if (lane < CH) red[turn][wave][jrow] = msum;
    __syncthreads();
    // lane c0 + j of every wavefront turns margin j of this chunk into its coefficient
    const int jm = min(max(lane - c0, 0), CH - 1);
    float mj = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) mj += red[turn][w][jm];
    const float cmine = (lane >= c0 && lane < P.B) ? loss_coef(P.kind, mj, tmine, P.scale) : 0.0f;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
      const float cj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cmine), min(c0 + j, 63)));
#pragma unroll
      for (int u = 0; u < G; ++u) e[u] += cj * a[j][u];
    }
    if (c0 + CH < P.B) request_rows(c0 + CH);       // same for every thread
  }
#pragma unroll
  for (int u = 0; u < G; ++u) {
    V ee = e[u];
    if (P.noise_std != 0.0f) ee += P.noise_std * noise_group<V>(col[u], noise_keys(P.seed, P.k, (uint32_t)agent));
    const V v = z[u] - P.lr * ee;
    if (FUSE == 2) {
      // half-step rows for the next iteration's combine: the travelling variable becomes the message itself,
      // the other moves by the same -lr e = v - z (the arithmetic of the combine kernel on stored messages)
      const V dz = v - z[u];
      const V moved = other_s[u * THREADS + threadIdx.x] + dz;
      if (on[u]) {
        const int64_t off = (int64_t)agent * P.ldo + col[u];
        *reinterpret_cast<V*>(P.ox + off) = P.new_exch_y ? moved : v;
        *reinterpret_cast<V*>(P.oy + off) = P.new_exch_y ? v : moved;
      }
    } else {
      if (on[u]) *reinterpret_cast<V*>(P.v + (int64_t)agent * P.ldv + col[u]) = v;
    }
  }
}

// The chunked kernel for rows of d4 16-byte groups.  Workgroup size and column groups per thread are a
// function of d4 alone and equal those of the one-pass variant for the same d4, so either kernel (and
// the fused form) produces the same bits.
template <int FUSE>
static hipError_t launch_chunked(const GemvArgs& g, hipStream_t st) {
  const int64_t d4 = g.d / 4;
  dim3 grid((unsigned)g.n);
  if (d4 <= 256) grad_chunked_kernel<4, 256, 8, 1, FUSE><<<grid, dim3(256), 0, st>>>(g);
  else if (d4 <= 1024) grad_chunked_kernel<4, 1024, 8, 1, FUSE><<<grid, dim3(1024), 0, st>>>(g);
  else if (d4 <= 2048) grad_chunked_kernel<4, 1024, 4, 2, FUSE><<<grid, dim3(1024), 0, st>>>(g);
  else grad_chunked_kernel<4, 1024, 2, 4, FUSE><<<grid, dim3(1024), 0, st>>>(g);
  return hipGetLastError();
}

// Layouts that are not 16-byte aligned: one column per thread, rows of at most 1024 columns, any batch.
template <int FUSE>
static hipError_t launch_chunked_scalar(const GemvArgs& g, hipStream_t st) {
  dim3 grid((unsigned)g.n);
  if (g.d <= 64) grad_chunked_kernel<1, 64, 8, 1, FUSE><<<grid, dim3(64), 0, st>>>(g);
  else if (g.d <= 256) grad_chunked_kernel<1, 256, 8, 1, FUSE><<<grid, dim3(256), 0, st>>>(g);
  else grad_chunked_kernel<1, 1024, 8, 1, FUSE><<<grid, dim3(1024), 0, st>>>(g);
  return hipGetLastError();
}

// A one-pass variant with the whole batch in registers exists for (B, d4).
static bool onepass_tile_exists(int32_t B, int64_t d4) {
  return (B <= 32 && d4 <= 256) || (B <= 16 && d4 <= 1024) || (B <= 8 && d4 <= 2048) || (B <= 4 && d4 <= 4096);
}

// With many agents and long rows the chunked kernel is the default for a single step.
static bool chunked_by_default(int32_t n, int64_t d4) { return n >= 128 && d4 > 256 && d4 <= 4096; }

// Shapes whose iterations can run as one fused kernel each with the bits of single steps: those where a
// single step already uses the chunked kernel, and those where it uses a one-pass variant (same bits).
// Few agents with a batch too large for a register tile stay with the two-pass kernels: a handful of
// workgroups walking megabytes of rows would be slower than three launches.
// (d a multiple of 4, vector layouts: checked by the caller.)
bool grad_fused_covers(int32_t n, int64_t d, int32_t B, bool vec4) {
  if (!vec4) return n >= 2 && d <= 1024;          // the scalar chunked kernel is what a single step uses there
  const int64_t d4 = d / 4;
  return n >= 2 && d4 <= 4096 && (chunked_by_default(n, d4) || onepass_tile_exists(B, d4));
}

bool launch_grad_fused(const GemvArgs& g, bool vec4, hipStream_t st, hipError_t* err) {
  if (!grad_fused_covers(g.n, g.d, g.B, vec4)) return false;
  *err = vec4 ? launch_chunked<1>(g, st) : launch_chunked_scalar<1>(g, st);
  return true;
}

// The same with the state kept in half-step form between iterations (px, py -> ox, oy: two different buffers).
bool launch_grad_half(const GemvArgs& g, bool vec4, hipStream_t st, hipError_t* err) {
  if (!grad_fused_covers(g.n, g.d, g.B, vec4)) return false;
  if (g.px == g.ox && !g.p_first) { *err = hipErrorInvalidValue; return true; }     // peers' rows are read while rows are written
  *err = vec4 ? launch_chunked<2>(g, st) : launch_chunked_scalar<2>(g, st);
  return true;
}

// The gradient of a single step on a layout that is not 16-byte aligned; false when the rows are too long
// for one workgroup (then the two-pass kernels run).
bool launch_grad_scalar(const GemvArgs& g, hipStream_t st, hipError_t* err) {
  if (g.d > 1024) return false;
  *err = launch_chunked_scalar<0>(g, st);
  return true;
}

// Picks the one-pass variant whose register tile covers (B, d); false if none does.
bool launch_grad_onepass(const GemvArgs& g, hipStream_t st, hipError_t* err) {
  const int64_t d4 = g.d / 4;
  const int apw = g_tuning.agents_per_wg;
  // many agents, long rows: the chunked kernel (any B up to 64, d up to 16384), two workgroups per
  // compute unit; a handful of agents cannot fill the device that way and stays with the kernels below
  if (chunked_by_default(g.n, d4) && !g_tuning.never_chunked) {
    *err = launch_chunked<0>(g, st);
    return true;
  }
  // 1024-thread workgroups fill a compute unit alone: one per unit, each looping over its agents;
  // 256-thread workgroups leave room for several per unit
#define CECA_ONEPASS(T, BM, GG)                                          \
  if (g.B <= BM && d4 <= (int64_t)T * GG) {                              \
    const int per_wg = apw > 0 ? apw : (T == 1024 ? (g.n + 255) / 256 : 1); \
    dim3 grid((unsigned)((g.n + per_wg - 1) / per_wg));                  \
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
  if (vec4) margins_kernel<4, false><<<grid, block, 0, st>>>(g);
  else margins_kernel<1, false><<<grid, block, 0, st>>>(g);
  return hipGetLastError();
}

hipError_t launch_margins_fused(const GemvArgs& g, bool vec4, hipStream_t st) {
  if (g.nchunks < 1 || g.n > 65535) return hipErrorInvalidConfiguration;
  // the row groups of an (agent, chunk) pair all read the old rows while the first one stores the new ones
  if (g.px == g.ox || g.py == g.oy) return hipErrorInvalidValue;
  dim3 grid((unsigned)g.nchunks, (unsigned)g.n, (unsigned)((g.B + kRowGroup - 1) / kRowGroup)), block(kBlock);
  if (vec4) margins_kernel<4, true><<<grid, block, 0, st>>>(g);
  else margins_kernel<1, true><<<grid, block, 0, st>>>(g);
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

}  // namespace ceca
