// C ABI of the DSGD-CECA hot path: argument checking, round schedule, launch shapes.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <numeric>

#include "ceca.h"
#include "ceca_test.h"
#include "launch.h"
#include "schedule.h"

namespace ceca {
thread_local Tuning g_tuning{};     // all zero: the library's own launch shapes
}

namespace {

using ceca::g_tuning;

thread_local char g_msg[256] = "";
thread_local int32_t g_hip = 0;

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_msg, sizeof g_msg, fmt, ap);
  va_end(ap);
  return code;
}

int32_t hip_fail(hipError_t e, const char* what) {
  g_hip = (int32_t)e;
  (void)hipGetLastError();   // clear the sticky launch error so later calls start clean
  return fail(CECA_EHIP, "%s: %s", what, hipGetErrorString(e));
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

inline bool overlaps(const void* a, int64_t na, const void* b, int64_t nb) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

// Shared checks of the two state-updating calls.  On success fills `rd` (left zeroed with n = 1).
int32_t check_state_call(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld, int32_t r,
                         int32_t port, ceca_round_t* rd) {
  if (!S_in || !S_out) return fail(CECA_EINVAL, "null state pointer");
  if (n < 1) return fail(CECA_EINVAL, "n = %d: need at least one agent", n);
  if (d < 1 || ld < d) return fail(CECA_EINVAL, "need 1 <= d <= ld (d = %lld, ld = %lld)", (long long)d, (long long)ld);
  if (port != 1 && port != 2) return fail(CECA_EINVAL, "port = %d: must be 1 or 2", port);
  const int32_t tau = ceca::tau_of(n);
  if (n == 1 ? r != 0 : (r < 0 || r >= tau)) return fail(CECA_EINVAL, "round r = %d outside [0, tau = %d)", r, tau);
  if (port == 1 && n > 1 && (n & 1)) return fail(CECA_EODD1P, "one-port CECA needs an even number of agents (n = %d)", n);
  const int64_t bytes = 2 * (int64_t)n * ld * (int64_t)sizeof(float);
  const bool same = (const void*)S_in == (const void*)S_out;
  if (overlaps(S_in, bytes, S_out, bytes) && !same)
    return fail(CECA_EINVAL, "S_out partially overlaps S_in");
  *rd = ceca_round_t{};
  rd->n = n;
  if (n > 1) ceca::fill_round(n, r, port, rd);
  return CECA_OK;
}

// Chain shape for the round: which cycles the walk has and how they are cut into stretches.
void shape_chain(const ceca_round_t& rd, int32_t n, int32_t port, bool in_place, int32_t default_seg, int64_t groups,
                 ceca::ChainArgs* a) {
  a->n = n;
  if (n == 1) {
    // a lone agent: one closed stretch of one row; weights make x+ = x - lr e, and y+ follows the call
    a->stride = 0; a->cyc_len = 1; a->segs_per_cycle = 1; a->seg_len = 1; a->c0_mul = 1;
    return;
  }
  a->stride = rd.shift;
  if (port == 1) {
    // pairs (2j, 2j + shift): closed two-row cycles starting at the even rows (Eq. (7))
    a->cyc_len = 2; a->segs_per_cycle = 1; a->seg_len = 2; a->c0_mul = 2;
    return;
  }
  const int32_t g = std::gcd(n, rd.shift);   // a shift by s splits the ring into gcd(n, s) cycles
  const int32_t len = n / g;
  a->cyc_len = len;
  a->c0_mul = 1;
  // In place only whole cycles are safe.  Out of place, measurements on MI355X favour one-row
  // stretches: the device then sweeps the rows of a column band one at a time (few concurrent DRAM
  // streams), and the message a stretch re-reads is still in L2 from the stretch before it.
  int32_t seg_len = in_place ? len : g_tuning.segment;
  if (seg_len <= 0) seg_len = default_seg;
  if (seg_len > len) seg_len = len;
  // a launch addresses fewer than 2^24 workgroups: huge problems walk longer stretches
  const int64_t tiles = (groups + ceca::kBlock - 1) / ceca::kBlock;
  while (seg_len < len && tiles * g * ((len + seg_len - 1) / seg_len) >= (1LL << 24)) seg_len *= 2;
  if (seg_len > len) seg_len = len;
  a->seg_len = seg_len;
  a->segs_per_cycle = (len + seg_len - 1) / seg_len;
}

// Launch shape of a chain kernel for this call: rows in flight, band, workgroups per compute unit (written
// into `a`) and the default stretch length.
struct ChainPlan { int rows; int32_t default_seg; bool in_place; };

ChainPlan plan_chain(ceca::ChainArgs* a, int mode, int64_t d, int32_t port) {
  ChainPlan p;
  int rows = g_tuning.rows;
  a->band = (uint32_t)g_tuning.band;
  a->wg_per_cu = g_tuning.wg_per_cu;
  // combining from stored messages reads no other agent's state rows, so it can overwrite the state
  // row by row with any stretch length; the other modes may only run whole cycles in place
  const bool in_place = a->xin == a->xout && mode != ceca::MODE_FROMV;
  const bool pairs = port == 1 || a->n == 1;
  // rows in flight per thread: closed pairs and in-place cycles of the fused step like the fattest
  // variant (it also runs fewer workgroups per CU); one-row stretches want more, lighter workgroups
  // round 0 of the fused step (y not read: half the traffic is writes) measured best with the lightest
  // variant, two-row stretches, wider bands and at most 4 workgroups per CU
  const bool fused_step = mode == ceca::MODE_QUAD || mode == ceca::MODE_GRAD;     // x, y and one more array stream in
  const bool quad_round0 = fused_step && !a->read_y && !(pairs || in_place);
  // a state that stays in the last-level cache (minibatch losses on many small agents) is not a
  // streaming problem: measured on MI355X at n = 1023, d = 4096, 16-row stretches with two rows in
  // flight beat one-row stretches (fewer, longer workgroups; 18.5 -> 14 us for the combine)
  // (only when one-row stretches would make thousands of workgroups: a handful of agents or columns
  // needs every workgroup it can get)
  const bool cached = mode == ceca::MODE_FROMV && !(pairs || in_place) &&
                      2 * (int64_t)a->n * a->ld * (int64_t)sizeof(float) <= (64LL << 20) &&
                      (int64_t)a->n * ((d + 4 * ceca::kBlock - 1) / (4 * ceca::kBlock)) >= 2048;
  p.default_seg = quad_round0 ? 2 : (cached ? 16 : 1);
  if (rows == 0) rows = quad_round0 ? 1 : cached ? 2 : (fused_step && (pairs || in_place)) ? 8 : 4;
  if (cached && a->band == 0) a->band = 2;
  if (quad_round0) {
    if (a->band == 0) a->band = 512;
    if (a->wg_per_cu == 0) a->wg_per_cu = 4;
  }
  // band: about 7-10 MB of traffic between a row's own read and its re-read as a message, so that the
  // re-read hits L2 (32 MB over 8 XCDs; a tile and its successor land on the same XCD when the band
  // is a multiple of 8)
  // closed stretches re-read nothing: they sweep whole rows, one pair or cycle after the other
  if (a->band == 0 && !(pairs || in_place)) a->band = fused_step ? 256 : 512;
  p.rows = rows;
  p.in_place = in_place;
  return p;
}

int32_t run_chain(ceca::ChainArgs a, int mode, int64_t d, bool can_vec, const ceca_round_t& rd, int32_t port,
                  hipStream_t st) {
  const ChainPlan pl = plan_chain(&a, mode, d, port);
  const int rows = pl.rows;
  const bool in_place = pl.in_place;
  const int32_t default_seg = pl.default_seg;
  const int64_t d4 = can_vec ? d / 4 : 0;
  if (d4 > 0) {
    a.col0 = 0;
    a.ngroups = d4;
    shape_chain(rd, a.n, port, in_place, default_seg, d4, &a);
    const hipError_t e = ceca::launch_chain(a, mode, true, rows, st);
    if (e != hipSuccess) return hip_fail(e, "chain kernel launch");
  }
  const int64_t rest = d - 4 * d4;
  if (rest > 0) {
    a.col0 = 4 * d4;
    a.ngroups = rest;
    shape_chain(rd, a.n, port, in_place, default_seg, rest, &a);
    const hipError_t e = ceca::launch_chain(a, mode, false, rows, st);
    if (e != hipSuccess) return hip_fail(e, "chain kernel launch (scalar columns)");
  }
  return CECA_OK;
}

void set_weights(const ceca_round_t& rd, int32_t n, bool gossip_only, ceca::ChainArgs* a) {
  if (n == 1) {
    // x+ = x - lr e;  y+ = y for a gossip "round" of one agent, y+ = x+ for a training step
    a->a = 1.0f; a->ap = 0.0f;
    a->b = gossip_only ? 1.0f : 0.0f; a->bp = gossip_only ? 0.0f : 1.0f;
    a->exch_y = 0; a->read_y = gossip_only ? 1 : 0;
    return;
  }
  a->a = rd.a; a->ap = rd.a_peer; a->b = rd.b; a->bp = rd.b_peer;
  a->exch_y = rd.exchange_y;
  a->read_y = (rd.b_num != 0) ? 1 : 0;
}

// dsgd_ceca_run's copy of the state: 2n rows at the caller's pitch, for pitches up to round_up(d, 64)
int64_t run_state_bytes(int32_t n, int64_t d) { return round_up(2 * (int64_t)n * round_up(d, 64) * (int64_t)sizeof(float), 256); }

struct GemvPlan {
  int64_t ldv, v_bytes, partial_bytes;
  int32_t nchunks_max;
};

GemvPlan gemv_plan(int32_t n, int64_t d, int32_t B) {
  GemvPlan p;
  p.ldv = round_up(d, 4);
  p.v_bytes = round_up((int64_t)n * p.ldv * (int64_t)sizeof(float), 256);
  const int64_t scalar_chunk = (int64_t)ceca::kBlock * ceca::kChunkGroups;     // the narrowest chunk in use
  p.nchunks_max = (int32_t)((d + scalar_chunk - 1) / scalar_chunk);
  p.partial_bytes = round_up((int64_t)n * p.nchunks_max * B * (int64_t)sizeof(float), 256);
  return p;
}

int32_t check_loss(const ceca_loss_t* loss, int64_t d, bool need_batch, const int32_t* batch_idx) {
  if (!loss) return fail(CECA_EINVAL, "null loss");
  switch (loss->kind) {
    case CECA_LOSS_LSQ:
    case CECA_LOSS_LOGISTIC:
      if (loss->N < 1 || loss->B < 1 || loss->B > 64)
        return fail(CECA_EINVAL, "need N >= 1 and 1 <= B <= 64 (N = %d, B = %d)", loss->N, loss->B);
      if (!loss->A || !loss->t || loss->lda < d) return fail(CECA_EINVAL, "minibatch loss needs A, t and lda >= d");
      if (need_batch && !batch_idx) return fail(CECA_EINVAL, "minibatch loss needs batch_idx");
      if (!(loss->noise_std >= 0.0f) || !(loss->grad_scale >= 0.0f))
        return fail(CECA_EINVAL, "noise_std and grad_scale must be >= 0");
      return CECA_OK;
    case CECA_LOSS_QUAD_CENTER:
      if (!loss->c || loss->ldc < d) return fail(CECA_EINVAL, "quadratic-centre loss needs c and ldc >= d");
      if (!(loss->noise_std >= 0.0f)) return fail(CECA_EINVAL, "noise_std must be >= 0");
      return CECA_OK;
    case CECA_LOSS_GRADIENT:
      if (!loss->c || loss->ldc < d) return fail(CECA_EINVAL, "caller-supplied gradients need c and ldc >= d");
      return CECA_OK;
    default:
      return fail(CECA_EINVAL, "unknown loss kind %d", loss->kind);
  }
}

// Consensus observables come in three forms (all deterministic, fp64 accumulation):
//   WAVE      one pass, a wavefront holds a column strip of every agent (no LDS): up to 64 x 32 agents
//   TILE      one pass, a workgroup holds a column tile of every agent and reduces through LDS
//   TWO_PASS  column sums, mean, then per-agent squared deviations (x read twice)
enum ConsForm { CONS_TWO_PASS = 1, CONS_TILE = 2, CONS_WAVE = 3 };

// Partial sums of the WAVE form are capped at this many bytes whatever the launch shape, so that the
// workspace bound does not depend on the calling thread's tuning.
constexpr int64_t kConsWavePartialBytes = 12LL << 20;
constexpr int64_t kConsWaves = 1024;     // wavefronts of the WAVE form: one per SIMD of an MI355X

struct ConsPlan {
  // two-pass form
  int64_t ntiles;
  int32_t agent_groups, agents_per_group, dev_agents;
  int64_t off_norm, off_devpart, off_dev2, two_pass_total;
  // TILE form: rows per thread (0 = not available for this n), row lanes, tiles for 16-byte / scalar groups
  int32_t rows_per_thread, row_lanes;
  int64_t tile_ntiles_vec, tile_ntiles_scalar;
  int64_t tile_total;          // workspace of the TILE form on a layout without 16-byte alignment (the larger one)
  // WAVE form: column groups per strip (0 = not available), rows per lane, most wavefronts
  int32_t wave_cgs, wave_shift, wave_rows;
  int64_t wave_cap;            // most wavefronts (bounds the partial sums)
  bool wave_default;           // the library's own choice for this n
  int64_t bound;               // workspace that covers every form and launch shape
};

struct ConsWave { int64_t strips, nwaves, off_dev2, total; };

// The WAVE form's launch for this layout: strips of wave_cgs column groups, strips per wavefront.
ConsWave cons_wave(const ConsPlan& p, int32_t n, int64_t d, bool vec4) {
  ConsWave w;
  const int64_t ngroups = vec4 ? (d + 3) / 4 : d;
  w.strips = (ngroups + p.wave_cgs - 1) / p.wave_cgs;
  // Measured on MI355X (n = 16 ... 130, 0.3 to 3 GB): the pass is fastest with exactly one wavefront per SIMD
  // (256 compute units x 4), each holding many rows in flight and walking its share of the strips; at
  // n = 31, d = 25.6 M that streams 7.0 TB/s, what a plain read-only kernel reaches, against 5.4 TB/s with
  // 50,000 short-lived wavefronts.  More wavefronts only add row streams that compete for DRAM pages.
  int64_t per = g_tuning.cons_strips;
  if (per <= 0) per = std::max<int64_t>((w.strips + kConsWaves - 1) / kConsWaves, 1);
  per = std::max(per, (w.strips + p.wave_cap - 1) / p.wave_cap);
  w.nwaves = (w.strips + per - 1) / per;
  w.off_dev2 = round_up(((int64_t)n + 1) * w.nwaves * 8, 256);
  w.total = w.off_dev2 + round_up(((int64_t)n + 1) * 8, 256);
  return w;
}

ConsPlan cons_plan(int32_t n, int64_t d) {
  ConsPlan p;
  p.ntiles = (d + ceca::kConsTile - 1) / ceca::kConsTile;
  // column sums: slice the agents when there are too few column tiles to fill the device
  // (at most 32 slices: the mean kernel adds them up serially per column)
  int64_t want = (1024 + p.ntiles - 1) / p.ntiles;
  if (want > 32) want = 32;
  if (want > (n + 3) / 4) want = (n + 3) / 4;
  if (want < 1) want = 1;
  p.agents_per_group = (int32_t)((n + want - 1) / want);
  p.agent_groups = (n + p.agents_per_group - 1) / p.agents_per_group;
  // deviations: one workgroup walks dev_agents rows of its column tile with the mean in registers
  int64_t rows = (4096 + p.ntiles - 1) / p.ntiles;      // wanted workgroups along the agents
  int64_t per = (n + rows - 1) / rows;
  if (per < 1) per = 1;
  while ((n + per - 1) / per > 65535) ++per;
  p.dev_agents = (int32_t)per;
  int64_t off = round_up((int64_t)p.agent_groups * d * 8, 256);
  p.off_norm = off;     off += round_up(p.ntiles * 8, 256);
  p.off_devpart = off;  off += round_up((int64_t)n * p.ntiles * 8, 256);
  p.off_dev2 = off;     off += round_up((int64_t)n * 8, 256);
  p.two_pass_total = off;
  p.bound = off;
  // TILE form: every agent's column tile in one workgroup (x-only tiling of the fused-round kernels)
  p.rows_per_thread = 0;
  p.row_lanes = 0;
  p.tile_total = 0;
  {
    // the widest tile (32 rows per thread) bounds the workspace of every tuned shape: fewer rows per thread
    // mean more row lanes, narrower tiles and more of them
    int32_t cap = g_tuning.rows;
    if (cap < 4 || cap > 32) cap = n <= 32 ? 16 : 32;     // wide tiles measured best on MI355X (n = 31, 100, 1023)
    int32_t row_lanes = 1;
    while (row_lanes * cap < n) row_lanes *= 2;
    while (row_lanes <= ceca::kBlock && ((int64_t)n + 1) * (ceca::kBlock / row_lanes) * 8 > 65536) row_lanes *= 2;
    // rows of the tile narrower than 128 bytes read poorly: with that many agents the single pass is kept
    // only for small problems, where the two-pass form is bound by its five launches
    const bool wide_enough = ceca::kBlock / (row_lanes < ceca::kBlock ? row_lanes : ceca::kBlock) >= 8 ||
                             (int64_t)n * d * 4 <= (64LL << 20);
    if (row_lanes <= ceca::kBlock && (n + row_lanes - 1) / row_lanes <= 32 && wide_enough) {
      p.row_lanes = row_lanes;
      p.rows_per_thread = (n + row_lanes - 1) / row_lanes;
      const int64_t lanes = ceca::kBlock / row_lanes;
      p.tile_ntiles_vec = ((d + 3) / 4 + lanes - 1) / lanes;
      p.tile_ntiles_scalar = (d + lanes - 1) / lanes;
    }
    if (p.rows_per_thread > 0) {
      p.tile_total = round_up(p.tile_ntiles_scalar * 8, 256) + round_up((int64_t)n * p.tile_ntiles_scalar * 8, 256) +
                     round_up((int64_t)n * 8, 256);
    }
  }
  // WAVE form
  p.wave_cgs = 0;
  p.wave_default = false;
  {
    // Rows per lane, measured on MI355X with one wavefront per SIMD: 16 up to 64 agents (n = 31: two row lanes
    // beat one lane with 31 rows, n = 64: four beat two), 32 beyond (n = 100, 128: four row lanes with 25 / 32
    // rows beat eight with 13 / 16: a strip is 256 bytes per agent instead of 128)
    int32_t cap = g_tuning.rows;
    if (cap < 1 || cap > 32) cap = n <= 64 ? 16 : 32;
    int32_t row_lanes = 1;
    while (row_lanes * cap < n) row_lanes *= 2;
    if (row_lanes <= 64) {
      p.wave_cgs = 64 / row_lanes;
      p.wave_shift = 0;
      while ((1 << p.wave_shift) < p.wave_cgs) ++p.wave_shift;
      p.wave_rows = (n + row_lanes - 1) / row_lanes;
      p.wave_cap = std::max<int64_t>(kConsWavePartialBytes / (((int64_t)n + 1) * 8), 64);
      // strips of 128 bytes per agent still win (n = 130: 0.072 against 0.077 ms for the workgroup tiles on
      // 273 MB); at 64 bytes (n = 258) the tiles do
      p.wave_default = p.wave_cgs >= 8;
    }
  }
  // the WAVE form never exceeds its cap whatever its launch shape; the TILE form's share follows the
  // calling thread's tuning (ask for the size after setting the options)
  const int64_t wave_bound = round_up(((int64_t)n + 1) * std::max<int64_t>(kConsWavePartialBytes / (((int64_t)n + 1) * 8), 64) * 8, 256) +
                             round_up(((int64_t)n + 1) * 8, 256);
  p.bound = std::max(p.bound, wave_bound);
  p.bound = std::max(p.bound, p.tile_total);
  return p;
}


// Tile of the register-tile kernels (fused rounds, fused iterations, mixing): threads per workgroup,
// threads that share a column group (a power of two) and rows per thread (the least that covers n);
// ok = false when no such tile holds n agents.
struct TileShape {
  int32_t threads, row_lanes, rows_per_thread;
  bool ok;
  // bytes of one agent's row inside the tile
  int32_t row_bytes(bool vec4) const { return (threads / std::max(row_lanes, 1)) * (vec4 ? 16 : 4); }
};

// The tile with at most `cap` rows per thread: the fewest row lanes that cover n give the widest rows.
TileShape shape_tile(int32_t n, bool vec4, int32_t threads, int32_t cap) {
  TileShape t{};
  t.threads = threads;
  t.row_lanes = 1;
  while ((int64_t)t.row_lanes * cap < n) t.row_lanes *= 2;
  t.rows_per_thread = (n + t.row_lanes - 1) / t.row_lanes;
  const int64_t lds = t.row_lanes <= t.threads ? (int64_t)n * (t.threads / t.row_lanes) * (vec4 ? 16 : 4) : 0;
  t.ok = t.row_lanes <= t.threads && lds <= (int64_t)ceca::kMultiMaxLds;
  return t;
}

// A kernel's tile policy: threads per workgroup for n agents, and the most rows per thread for that
// width.  The option knobs override it when the tile they ask for holds n agents (scalar columns always
// run 256-thread workgroups).
template <typename Threads, typename Cap>
TileShape pick_tile(int32_t n, bool vec4, int32_t cap_lo, int32_t cap_hi_256, int32_t cap_hi_wide, Threads threads_for, Cap cap_for) {
  const int32_t dflt_threads = vec4 ? threads_for(n) : ceca::kBlock;
  const TileShape dflt = shape_tile(n, vec4, dflt_threads, cap_for(dflt_threads));
  int32_t threads = vec4 ? g_tuning.tile_threads : ceca::kBlock;
  if (threads == 0) threads = dflt_threads;
  int32_t cap = g_tuning.rows;
  if (cap < cap_lo || cap > (threads == ceca::kBlock ? cap_hi_256 : cap_hi_wide)) cap = cap_for(threads);
  const TileShape t = shape_tile(n, vec4, threads, cap);
  return t.ok ? t : dflt;
}

// Fused gossip rounds (x and y of every row in registers); with_y = false: exact averaging, which
// stores no y.
TileShape rounds_tile(int32_t n, bool vec4, bool with_y = true) {
  // Measured on MI355X (n = 8 ... 4096) with the straight-line round body.  Up to 256 agents: 256-thread
  // workgroups.  The fused rounds, two thirds of whose traffic is writes, do best with many small
  // workgroups while the rows of the tile stay wide: up to 80 agents 5 rows per thread (n = 8: 0.30 against
  // 0.36 ms, n = 31: 0.29 against 0.31, n = 72: 0.29 against 0.32 for 9 rows), beyond that up to 9.  Exact
  // averaging, lighter on memory, prefers fewer row lanes and up to 12 rows per thread between 33 and 192
  // agents (n = 56: 0.19 against 0.225 ms, n = 72: 0.20 against 0.24, n = 176: 0.23 against 0.26) and 5 rows
  // below that (n = 8: 0.18 against 0.21).
  // More agents: 512-thread workgroups with up to 10 rows per thread (the tile then takes at most half of
  // a compute unit's LDS: two workgroups per compute unit) make the rows of the tile two to four times wider
  // than 256-thread ones; 12 rows per thread carry them to 12 x 128 agents (n = 1500: 0.75 ms against 0.79
  // with 1024 threads), beyond that only a 1024-thread workgroup keeps the rows at 64 bytes.  Exact averaging
  // does better with 256-thread workgroups holding up to 16 rows per thread where the rows stay 128 bytes
  // wide (up to 512 agents; n = 400: 0.26 ms against 0.34) or a thread gets at least 12 rows (705 to 1024
  // agents; n = 800: 0.31 ms against 0.40).
  if (n <= 256) {
    const int32_t cap = with_y ? (n <= 80 ? 5 : 9) : (n <= 32 ? 5 : (n <= 192 ? 12 : 9));
    return pick_tile(n, vec4, 4, ceca::kMultiRows, ceca::kMultiRows, [](int32_t) { return ceca::kBlock; },
                     [cap](int32_t threads) { return threads == ceca::kBlock ? cap : 9; });
  }
  const bool narrow_group = !with_y && (n <= 512 || (n > 704 && n <= 1024));
  return pick_tile(n, vec4, 4, ceca::kMultiRows, ceca::kMultiRows,
                   [narrow_group](int32_t m) { return narrow_group ? ceca::kBlock : (m > 12 * 128 ? 1024 : 512); },
                   [n](int32_t threads) { return threads == ceca::kBlock ? ceca::kMultiRows : (threads == 512 ? (n > 10 * 128 ? 12 : 10) : 9); });
}

// Register-lean form of the fused-rounds kernel for a 256-thread tile with this many rows per thread (the
// wavefronts per SIMD it is compiled for, peers read from LDS two rows at a time; 0 = the plain form, all of
// a thread's peers read at once).  Measured on MI355X: with 5 to 8 rows five wavefronts per SIMD (n = 128,
// 8 rows: exact averaging 0.235 -> 0.21 ms), with 9 rows four; from 10 rows on the lean forms spill and the
// plain form is the one to use.
int32_t rounds_lean(const TileShape& t, bool vec4) {
  const int32_t forced = g_tuning.lean_tiles;
  if (!vec4 || t.threads != ceca::kBlock || forced == 1) return 0;
  if (forced >= 4) return forced;
  if (t.rows_per_thread >= 5 && t.rows_per_thread <= 8) return 5;
  if (t.rows_per_thread == 9) return 4;
  return 0;
}

// Fused iterations (x, y and c of every row in registers).
TileShape steps_tile(int32_t n, bool vec4, int32_t steps) {
  // With noise the kernel is bound by the generator's arithmetic: few rows per thread (small register
  // footprint, many resident wavefronts) measured best on MI355X.  More agents need wider workgroups
  // to keep a row of the tile 64 bytes wide: x, y and c of 5 rows fit the 128 registers of a 512-thread
  // (two per compute unit) or 1024-thread workgroup.  Measured against 256-thread tiles, 4 iterations,
  // 2^26 elements: n = 258 0.19 -> 0.13 ms, n = 640 0.27 -> 0.23, n = 1026 0.72 -> 0.26, n = 2050
  // 1.39 -> 0.62.
  return pick_tile(n, vec4, 1, ceca::kMultiRows, 8,
                   [](int32_t m) { return m <= 128 ? ceca::kBlock : (m <= 5 * 128 ? 512 : 1024); },
                   [n, steps](int32_t threads) {
                     if (threads != ceca::kBlock) return 5;
                     if (n <= 128) return 4;
                     if (n <= 512) return 8;
                     return (steps <= 16 || n > 8 * ceca::kBlock) ? 16 : 8;     // 8 rows x 256 row lanes hold 2048 agents
                   });
}

// Mixing rounds of the comparison topologies (x of every row in registers); heavy = four or more
// peers in some round.
TileShape mix_tile(int32_t n, bool vec4, bool heavy) {
  // Measured on MI355X (n = 31 ... 4096, all three topologies; x alone in registers, 67 registers at 9 rows
  // per thread).  What counts is how many workgroups a compute unit holds: the LDS tile is n x tile row.
  // Up to 256 agents: 256 threads, up to 12 rows per thread (n = 64 ring: 0.20 against 0.25 ms with 16,
  // n = 100: 0.215 against 0.24).  257 to 512 agents: one or two peers per round run 512-thread workgroups
  // with up to 9 rows (n = 258 ring: 0.33 against 0.40 ms), many peers per round (LDS-read bound) 256 threads
  // with up to 16.  Up to 9 x 128 agents: 512 threads x at most 9 rows, i.e. 64-byte tile rows and three
  // workgroups per compute unit rather than 128-byte rows and one (n = 800: ring 0.31 against 0.50 ms, static
  // exponential 0.81 against 1.20).  Beyond: 512 threads x 13 rows up to 13 x 128 agents and 1024 threads
  // after that for few peers; many peers keep 512 threads x 9 rows up to 2304 agents (n = 1500: 0.98 against
  // 1.51 ms, n = 2050: 1.34 against 1.59).
  return pick_tile(n, vec4, 4, 32, 16,
                   [heavy](int32_t m) {
                     if (m <= 256) return ceca::kBlock;
                     if (m <= 512) return heavy ? ceca::kBlock : 512;
                     if (m <= 9 * 128) return 512;
                     if (heavy) return m <= 9 * 256 ? 512 : 1024;
                     return m <= 13 * 128 ? 512 : 1024;
                   },
                   [n, heavy](int32_t threads) {
                     if (threads == ceca::kBlock) return n <= 256 ? 12 : (n <= 512 ? 16 : (heavy ? 16 : 24));
                     if (threads == 512) return (heavy || n <= 9 * 128) ? 9 : 13;
                     return 13;
                   });
}

// Gossip over an arbitrary graph (x of every row in registers, plus a neighbour index and weight per row
// in flight).  Measured on MI355X (ring, torus; n = 130 ... 2048): 256-thread workgroups up to about 384
// agents, 512-thread ones up to 768 (n = 520: torus 0.81 -> 0.72 ms, ring 0.59 -> 0.53 against 1024 threads),
// 1024-thread ones beyond, with up to 8 rows per thread so that the rows of the tile stay 64 bytes wide up to
// 2048 agents (n = 2048 ring: 1.13 -> 0.70 ms against 6 rows and 32-byte rows).
TileShape graph_tile(int32_t n, bool vec4) {
  return pick_tile(n, vec4, 4, ceca::kGraphRows, 8,
                   [](int32_t m) { return m <= 384 ? ceca::kBlock : (m <= 768 ? 512 : 1024); },
                   [n](int32_t threads) {
                     if (threads == ceca::kBlock) return n <= 192 ? 8 : ceca::kGraphRows;
                     return 8;
                   });
}

// ---- scratch memory of the allocation-free entry point (consensus_error_noalloc) ----
// One array per GPU, held from the moment the library's code is loaded on that GPU until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address it yields
// (a different one on every GPU) is what kernels and copies are given.
constexpr int64_t kScratchBytes = 16LL << 20;
__device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of the scratch array (looked up once per device, with that device current).
int32_t scratch_of_current_device(char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(CECA_EINVAL, "device %d: the allocation-free entry point serves devices 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!p || (reinterpret_cast<uintptr_t>(p) & 255u) != 0) return fail(CECA_EHIP, "the scratch array has no 256-byte aligned device address");
    g_scratch_ptr[dev] = p;
  }
  *out = reinterpret_cast<char*>(g_scratch_ptr[dev]);
  return CECA_OK;
}

}  // namespace

extern "C" {

const char* ceca_last_error(void) { return g_msg; }
int32_t ceca_last_hip_error(void) { return g_hip; }

int32_t ceca_set_option(int32_t option, int32_t value) {
  ceca::Tuning& t = ceca::g_tuning;
  switch (option) {
    case CECA_OPT_SEGMENT:
      if (value < 0) return fail(CECA_EINVAL, "segment length must be >= 0");
      t.segment = value;
      return CECA_OK;
    case CECA_OPT_ROWS:
      if (value < 0 || value > 32) return fail(CECA_EINVAL, "rows must be 0..32");
      t.rows = value;
      return CECA_OK;
    case CECA_OPT_WG_PER_CU:
      if (value < 0 || value > 8) return fail(CECA_EINVAL, "workgroups per CU must be 0..8");
      t.wg_per_cu = value;
      return CECA_OK;
    case CECA_OPT_ONEPASS:
      t.two_pass_gradient = value == 0;
      return CECA_OK;
    case CECA_OPT_CONS_SINGLE_PASS:
      if (value < 0 || value > 3) return fail(CECA_EINVAL, "consensus form must be 0..3");
      t.cons_form = value == 1 ? 0 : (value == 0 ? 1 : value);
      return CECA_OK;
    case CECA_OPT_TILE_THREADS:
      if (value != 0 && value != 256 && value != 512 && value != 1024)
        return fail(CECA_EINVAL, "tile threads must be 0, 256, 512 or 1024");
      t.tile_threads = value;
      return CECA_OK;
    case CECA_OPT_XCD_TILE_ORDER:
      t.plain_tile_order = value == 0;
      return CECA_OK;
    case CECA_OPT_AGENTS_PER_WG:
      if (value < 0) return fail(CECA_EINVAL, "agents per workgroup must be >= 0");
      t.agents_per_wg = value;
      return CECA_OK;
    case CECA_OPT_BAND:
      if (value < 0) return fail(CECA_EINVAL, "band width must be >= 0");
      t.band = value;
      return CECA_OK;
    case CECA_OPT_GRAPH_STAGE:
      t.graph_tables_in_memory = value == 0;
      return CECA_OK;
    case CECA_OPT_CHUNKED_GRADIENT:
      t.never_chunked = value == 0;
      return CECA_OK;
    case CECA_OPT_HALF_STEP_RUN:
      t.no_half_step = value == 0;
      return CECA_OK;
    case CECA_OPT_LEAN_TILES:
      if (value != 0 && value != 1 && (value < 4 || value > 6)) return fail(CECA_EINVAL, "lean tiles must be 0, 1, 4, 5 or 6");
      t.lean_tiles = value;
      return CECA_OK;
    case CECA_OPT_PROBE_VARIANT:
      if (value < 0 || value > 399) return fail(CECA_EINVAL, "probe variant must be 0..399");
      t.probe_variant = value;
      return CECA_OK;
    case CECA_OPT_PROBE_WAVES:
      if (value < 0 || value > (1 << 20)) return fail(CECA_EINVAL, "probe wavefronts must be 0..2^20");
      t.probe_waves = value;
      return CECA_OK;
    case CECA_OPT_CONS_STRIPS:
      if (value < 0 || value > 4096) return fail(CECA_EINVAL, "strips per wavefront must be 0..4096");
      t.cons_strips = value;
      return CECA_OK;
    default:
      return fail(CECA_EINVAL, "unknown option %d", option);
  }
}

int32_t ceca_reset_options(void) {
  ceca::g_tuning = ceca::Tuning{};
  return CECA_OK;
}

int32_t ceca_tau(int32_t n) {
  if (n < 1) return fail(CECA_EINVAL, "n = %d: need at least one agent", n);
  return ceca::tau_of(n);
}

int32_t ceca_schedule(int32_t n, int32_t r, int32_t port, ceca_round_t* out, int32_t* peer) {
  if (n < 2) return fail(CECA_EINVAL, "n = %d: a schedule needs at least two agents", n);
  if (port != 1 && port != 2) return fail(CECA_EINVAL, "port = %d: must be 1 or 2", port);
  const int32_t tau = ceca::tau_of(n);
  if (r < 0 || r >= tau) return fail(CECA_EINVAL, "round r = %d outside [0, tau = %d)", r, tau);
  if (port == 1 && (n & 1)) return fail(CECA_EODD1P, "one-port CECA needs an even number of agents (n = %d)", n);
  ceca_round_t rd;
  ceca::fill_round(n, r, port, &rd);
  if (out) *out = rd;
  if (peer)
    for (int32_t i = 0; i < n; ++i) peer[i] = ceca::peer_of(rd, i);
  return CECA_OK;
}

int32_t ceca_gossip_round(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld, int32_t r,
                          int32_t port, void* hip_stream) {
  ceca_round_t rd;
  const int32_t rc = check_state_call(S_in, S_out, n, d, ld, r, port, &rd);
  if (rc != CECA_OK) return rc;
  ceca::ChainArgs a{};
  a.xin = S_in;  a.yin = S_in + (int64_t)n * ld;
  a.xout = S_out; a.yout = S_out + (int64_t)n * ld;
  a.ld = ld;
  a.n = n;
  set_weights(rd, n, /*gossip_only=*/true, &a);
  const bool can_vec = aligned16(S_in) && aligned16(S_out) && ld % 4 == 0;
  return run_chain(a, ceca::MODE_GOSSIP, d, can_vec, rd, port, (hipStream_t)hip_stream);
}

int32_t ceca_gossip_rounds(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld, int32_t rounds,
                           int32_t port, void* hip_stream) {
  ceca_round_t rd;
  const int32_t rc = check_state_call(S_in, S_out, n, d, ld, 0, port, &rd);
  if (rc != CECA_OK) return rc;
  if (rounds < 1) return fail(CECA_EINVAL, "rounds = %d: need at least one", rounds);
  hipStream_t st = (hipStream_t)hip_stream;
  const int32_t tau = ceca::tau_of(n);
  const TileShape tv = rounds_tile(n, true), ts = rounds_tile(n, false);
  const bool can_vec = aligned16(S_in) && aligned16(S_out) && ld % 4 == 0;
  // A single round is the streaming kernel's job, and tiles with rows narrower than a 128-byte line pay
  // off only over a few rounds (measured: the fused pass costs about 1.5, 2.5 and 4.7 single rounds at
  // n = 1026, 2050 and 4096).
  const int32_t row_bytes = can_vec ? tv.row_bytes(true) : ts.row_bytes(false);
  const int32_t worth = row_bytes >= 64 ? (tv.threads == 1024 && can_vec ? 3 : 2) : 5;
  const bool knobs = g_tuning.rows != 0 || g_tuning.tile_threads != 0;
  // (rounds after the first run in place on S_out: with two ports those walk whole cycles, which needs
  // many column tiles to fill the device)
  const bool rounds_fill = port == 1 || d >= 1024 * 1024 || rounds == 1;
  if (n == 1 || !tv.ok || !ts.ok || (rounds < worth && rounds_fill && !knobs)) {
    // too many agents for one workgroup's registers (or too little to fuse): one launch per round, the
    // first from S_in to S_out, the rest in place on S_out (whole cycles / pairs read before they write)
    for (int32_t t = 0; t < rounds; ++t) {
      const int32_t r1 = ceca_gossip_round(t == 0 ? S_in : S_out, S_out, n, d, ld, n == 1 ? 0 : t % tau, port, st);
      if (r1 != CECA_OK) return r1;
    }
    return CECA_OK;
  }
  const int64_t d4 = can_vec ? d / 4 : 0;
  // one kernel takes up to kMultiMaxRounds rounds; longer runs go in pieces of whole cycles (the
  // kernel starts at round 0, which reads no y), the first from S_in to S_out and the rest in place
  // on S_out (a workgroup holds its whole tile before it writes)
  const int32_t piece = ceca::kMultiMaxRounds / tau * tau;     // tau <= 12 for the agent counts that reach here
  for (int32_t t0 = 0; t0 < rounds; t0 += piece) {
    const int32_t cnt = std::min(rounds - t0, piece);
    ceca::MultiArgs m{};
    m.xin = t0 == 0 ? S_in : S_out;
    m.xout = S_out;  m.yout = S_out + (int64_t)n * ld;
    m.ld = ld;
    m.n = n;  m.port = port;  m.rounds = cnt;
    m.lean = rounds_lean(tv, true);
    for (int32_t t = 0; t < cnt; ++t) {
      ceca::fill_round(n, (t0 + t) % tau, port, &rd);
      ceca::MultiRound& R = m.round[t];
      R.shift = rd.shift;  R.exch_y = rd.exchange_y;  R.read_y = rd.b_num != 0;
      R.a = rd.a;  R.ap = rd.a_peer;  R.b = rd.b;  R.bp = rd.b_peer;
    }
    if (d4 > 0) {
      m.col0 = 0;  m.ngroups = d4;
      m.threads = tv.threads;  m.row_lanes = tv.row_lanes;  m.rows_per_thread = tv.rows_per_thread;
      const hipError_t e = ceca::launch_multi_round(m, true, st);
      if (e != hipSuccess) return hip_fail(e, "multi-round kernel launch");
    }
    if (d - 4 * d4 > 0) {
      m.col0 = 4 * d4;  m.ngroups = d - 4 * d4;
      m.threads = ts.threads;  m.row_lanes = ts.row_lanes;  m.rows_per_thread = ts.rows_per_thread;
      const hipError_t e = ceca::launch_multi_round(m, false, st);
      if (e != hipSuccess) return hip_fail(e, "multi-round kernel launch (scalar columns)");
    }
  }
  return CECA_OK;
}

int32_t ceca_average(const float* X_in, float* X_out, int32_t n, int64_t d, int64_t ld, int32_t port, void* hip_stream) {
  if (!X_in || !X_out) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || n > 4096) return fail(CECA_EINVAL, "n = %d: exact averaging in one pass takes 1 to 4096 agents", n);
  if (d < 1 || ld < d) return fail(CECA_EINVAL, "need 1 <= d <= ld (d = %lld, ld = %lld)", (long long)d, (long long)ld);
  if (port != 1 && port != 2) return fail(CECA_EINVAL, "port = %d: must be 1 or 2", port);
  if (port == 1 && n > 1 && (n & 1)) return fail(CECA_EODD1P, "one-port CECA needs an even number of agents (n = %d)", n);
  const int64_t bytes = (int64_t)n * ld * (int64_t)sizeof(float);
  if (overlaps(X_in, bytes, X_out, bytes) && (const void*)X_in != (const void*)X_out)
    return fail(CECA_EINVAL, "X_out partially overlaps X_in");
  hipStream_t st = (hipStream_t)hip_stream;
  const int32_t tau = ceca::tau_of(n);
  const TileShape tv = rounds_tile(n, true, false), ts = rounds_tile(n, false, false);
  if (!tv.ok || !ts.ok) return fail(CECA_EINVAL, "internal: no tile holds n = %d agents", n);
  ceca::MultiArgs m{};
  m.xin = X_in;
  m.xout = X_out;  m.yout = nullptr;
  m.ld = ld;
  m.n = n;  m.port = port;  m.rounds = tau;          // n = 1: no rounds, the kernel copies
  m.lean = rounds_lean(tv, true);
  ceca_round_t rd;
  for (int32_t t = 0; t < tau; ++t) {
    ceca::fill_round(n, t, port, &rd);
    ceca::MultiRound& R = m.round[t];
    R.shift = rd.shift;  R.exch_y = rd.exchange_y;  R.read_y = rd.b_num != 0;
    R.a = rd.a;  R.ap = rd.a_peer;  R.b = rd.b;  R.bp = rd.b_peer;
  }
  const bool can_vec = aligned16(X_in) && aligned16(X_out) && ld % 4 == 0;
  const int64_t d4 = can_vec ? d / 4 : 0;
  if (d4 > 0) {
    m.col0 = 0;  m.ngroups = d4;
    m.threads = tv.threads;  m.row_lanes = tv.row_lanes;  m.rows_per_thread = tv.rows_per_thread;
    const hipError_t e = ceca::launch_multi_round(m, true, st);
    if (e != hipSuccess) return hip_fail(e, "averaging kernel launch");
  }
  if (d - 4 * d4 > 0) {
    m.col0 = 4 * d4;  m.ngroups = d - 4 * d4;
    m.threads = ts.threads;  m.row_lanes = ts.row_lanes;  m.rows_per_thread = ts.rows_per_thread;
    const hipError_t e = ceca::launch_multi_round(m, false, st);
    if (e != hipSuccess) return hip_fail(e, "averaging kernel launch (scalar columns)");
  }
  return CECA_OK;
}

int64_t dsgd_ceca_workspace_bytes(int32_t n, int64_t d, const ceca_loss_t* loss) {
  if (n < 1 || d < 1) return fail(CECA_EINVAL, "need n >= 1 and d >= 1");
  const int32_t rc = check_loss(loss, d, false, nullptr);
  if (rc != CECA_OK) return rc;
  if (loss->kind == CECA_LOSS_QUAD_CENTER || loss->kind == CECA_LOSS_GRADIENT) return 0;
  const GemvPlan p = gemv_plan(n, d, loss->B);
  return p.v_bytes + p.partial_bytes;
}

int32_t dsgd_ceca_step(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld, const ceca_loss_t* loss,
                       const int32_t* batch_idx, float lr, int32_t r, int32_t port, void* workspace,
                       int64_t workspace_bytes, void* hip_stream) {
  ceca_round_t rd;
  int32_t rc = check_state_call(S_in, S_out, n, d, ld, r, port, &rd);
  if (rc != CECA_OK) return rc;
  rc = check_loss(loss, d, true, batch_idx);
  if (rc != CECA_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;

  ceca::ChainArgs a{};
  a.xin = S_in;  a.yin = S_in + (int64_t)n * ld;
  a.xout = S_out; a.yout = S_out + (int64_t)n * ld;
  a.ld = ld;
  a.n = n;
  a.lr = lr;
  set_weights(rd, n, /*gossip_only=*/false, &a);
  const bool state_vec = aligned16(S_in) && aligned16(S_out) && ld % 4 == 0;

  if (loss->kind == CECA_LOSS_QUAD_CENTER || loss->kind == CECA_LOSS_GRADIENT) {
    const int64_t sbytes = 2 * (int64_t)n * ld * 4, cbytes = (int64_t)n * loss->ldc * 4;
    if (overlaps(loss->c, cbytes, S_out, sbytes)) return fail(CECA_EINVAL, "centres or gradients overlap S_out");
    a.aux = loss->c;
    a.ldaux = loss->ldc;
    const bool can_vec = state_vec && aligned16(loss->c) && loss->ldc % 4 == 0;
    if (loss->kind == CECA_LOSS_GRADIENT) return run_chain(a, ceca::MODE_GRAD, d, can_vec, rd, port, st);
    a.noise_std = loss->noise_std;
    a.seed = loss->seed;
    a.k = loss->k;
    return run_chain(a, ceca::MODE_QUAD, d, can_vec, rd, port, st);
  }

  // GEMV-shaped losses: margins -> messages v (workspace) -> combine
  if (n > 65535) return fail(CECA_EINVAL, "minibatch losses support at most 65535 agents");
  const GemvPlan p = gemv_plan(n, d, loss->B);
  if (!workspace || workspace_bytes < p.v_bytes + p.partial_bytes)
    return fail(CECA_EWORKSPACE, "workspace of %lld bytes needed, %lld given", (long long)(p.v_bytes + p.partial_bytes),
                (long long)(workspace ? workspace_bytes : 0));
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return fail(CECA_EWORKSPACE, "workspace must be 256-byte aligned");
  if (overlaps(workspace, p.v_bytes + p.partial_bytes, S_out, 2 * (int64_t)n * ld * 4) ||
      overlaps(workspace, p.v_bytes + p.partial_bytes, S_in, 2 * (int64_t)n * ld * 4))
    return fail(CECA_EINVAL, "workspace overlaps the state");

  ceca::GemvArgs g{};
  g.zin = a.exch_y ? a.yin : a.xin;
  g.ld = ld;
  g.A = loss->A;  g.lda = loss->lda;  g.t = loss->t;
  g.batch_idx = batch_idx;
  g.v = reinterpret_cast<float*>(workspace);
  g.ldv = p.ldv;
  g.partial = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + p.v_bytes);
  g.d = d;
  g.n = n;  g.N = loss->N;  g.B = loss->B;  g.kind = loss->kind;
  g.lr = lr;
  g.scale = loss->grad_scale > 0.0f ? loss->grad_scale : 1.0f / (float)loss->B;
  g.noise_std = loss->noise_std;
  g.seed = loss->seed;
  g.k = loss->k;
  const bool gemv_vec = aligned16(S_in) && ld % 4 == 0 && aligned16(loss->A) && loss->lda % 4 == 0 && d % 4 == 0;
  g.chunk_cols = ceca::kBlock * ceca::kChunkGroups * (gemv_vec ? 4 : 1);
  g.nchunks = (int32_t)((d + g.chunk_cols - 1) / g.chunk_cols);
  hipError_t e = hipSuccess;
  const bool onepass = !g_tuning.two_pass_gradient &&
                       (gemv_vec ? ceca::launch_grad_onepass(g, st, &e) : ceca::launch_grad_scalar(g, st, &e));
  if (onepass) {
    if (e != hipSuccess) return hip_fail(e, "one-pass gradient kernel launch");
  } else {
    e = ceca::launch_margins(g, gemv_vec, st);
    if (e != hipSuccess) return hip_fail(e, "margins kernel launch");
    e = ceca::launch_halfstep(g, gemv_vec, st);
    if (e != hipSuccess) return hip_fail(e, "half-step kernel launch");
  }

  a.aux = g.v;
  a.ldaux = g.ldv;
  return run_chain(a, ceca::MODE_FROMV, d, state_vec, rd, port, st);
}

int64_t dsgd_ceca_run_workspace_bytes(int32_t n, int64_t d, const ceca_loss_t* loss) {
  if (n < 1 || d < 1) return fail(CECA_EINVAL, "need n >= 1 and d >= 1");
  const int32_t rc = check_loss(loss, d, false, nullptr);
  if (rc != CECA_OK) return rc;
  if (loss->kind != CECA_LOSS_LSQ && loss->kind != CECA_LOSS_LOGISTIC)
    return fail(CECA_EINVAL, "dsgd_ceca_run takes minibatch losses (LSQ, LOGISTIC)");
  const GemvPlan p = gemv_plan(n, d, loss->B);
  // two message buffers (iterations alternate) + partial margins + a copy of the state (iterations on the
  // two-pass gradient kernels alternate between it and S_out)
  return 2 * p.v_bytes + p.partial_bytes + run_state_bytes(n, d);
}

int32_t dsgd_ceca_run(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld, const ceca_loss_t* loss,
                      const int32_t* batch_idx, float lr, int32_t r0, int32_t iters, int32_t port, void* workspace,
                      int64_t workspace_bytes, void* hip_stream) {
  ceca_round_t rd;
  int32_t rc = check_state_call(S_in, S_out, n, d, ld, r0, port, &rd);
  if (rc != CECA_OK) return rc;
  rc = check_loss(loss, d, true, batch_idx);
  if (rc != CECA_OK) return rc;
  if (loss->kind != CECA_LOSS_LSQ && loss->kind != CECA_LOSS_LOGISTIC)
    return fail(CECA_EINVAL, "dsgd_ceca_run takes minibatch losses (LSQ, LOGISTIC)");
  if (iters < 1) return fail(CECA_EINVAL, "iters = %d: need at least one", iters);
  const GemvPlan p = gemv_plan(n, d, loss->B);
  const int64_t need = 2 * p.v_bytes + p.partial_bytes + run_state_bytes(n, d);
  if (!workspace || workspace_bytes < need)
    return fail(CECA_EWORKSPACE, "workspace of %lld bytes needed, %lld given", (long long)need,
                (long long)(workspace ? workspace_bytes : 0));
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return fail(CECA_EWORKSPACE, "workspace must be 256-byte aligned");
  const int64_t sbytes = 2 * (int64_t)n * ld * 4;
  if (overlaps(workspace, need, S_out, sbytes) || overlaps(workspace, need, S_in, sbytes))
    return fail(CECA_EINVAL, "workspace overlaps the state");
  hipStream_t st = (hipStream_t)hip_stream;
  const int32_t tau = ceca::tau_of(n);
  char* w = reinterpret_cast<char*>(workspace);
  const int64_t nb = (int64_t)n * loss->B;
  // the gradient kernel of an iteration is chosen by the layout of the state it reads (S_in first, then
  // S_out): the fused form needs the two to agree
  const bool lay = ld % 4 == 0 && aligned16(loss->A) && loss->lda % 4 == 0 && d % 4 == 0;
  const bool vec = lay && aligned16(S_in);
  const bool same_layout = vec == (lay && aligned16(S_out));
  const bool fused = same_layout && n > 1 && iters > 1 && !g_tuning.two_pass_gradient && !g_tuning.never_chunked &&
                     ceca::grad_fused_covers(n, d, loss->B, vec);
  // Shapes whose single step takes the two-pass gradient (margins, then half step): the combine of the
  // iteration before becomes the prologue of the margins kernel -- two launches per iteration instead of
  // three, same bits.  The row groups of that kernel all read the old rows while one of them stores the
  // new ones, so the state alternates between S_out and a copy in the workspace.
  const bool two_pass = g_tuning.two_pass_gradient || !(vec ? ceca::grad_fused_covers(n, d, loss->B, true) : d <= 1024);
  const bool copy_fits = 2 * (int64_t)n * ld * (int64_t)sizeof(float) <= run_state_bytes(n, d);     // the copy keeps the caller's pitch
  if (!fused && two_pass && same_layout && copy_fits && n > 1 && iters > 1 && n <= 65535) {
    float* V2[2] = {reinterpret_cast<float*>(w), reinterpret_cast<float*>(w + p.v_bytes)};
    float* W = reinterpret_cast<float*>(w + 2 * p.v_bytes + p.partial_bytes);
    ceca::GemvArgs g{};
    g.A = loss->A;  g.lda = loss->lda;  g.t = loss->t;
    g.ldv = p.ldv;
    g.partial = reinterpret_cast<float*>(w + 2 * p.v_bytes);
    g.d = d;
    g.n = n;  g.N = loss->N;  g.B = loss->B;  g.kind = loss->kind;
    g.lr = lr;
    g.scale = loss->grad_scale > 0.0f ? loss->grad_scale : 1.0f / (float)loss->B;
    g.noise_std = loss->noise_std;
    g.seed = loss->seed;
    g.chunk_cols = ceca::kBlock * ceca::kChunkGroups * (vec ? 4 : 1);
    g.nchunks = (int32_t)((d + g.chunk_cols - 1) / g.chunk_cols);
    // where the state lives before iteration t's prologue: S_in, then the copy and S_out in turn
    const float* cur = S_in;
    ceca_round_t prev{};
    g.ld = ld;  g.ldo = ld;
    for (int32_t t = 0; t < iters; ++t) {
      ceca::fill_round(n, (r0 + t) % tau, port, &rd);
      g.batch_idx = batch_idx + (int64_t)t * nb;
      g.k = loss->k + (uint32_t)t;
      g.v = V2[t & 1];
      hipError_t e;
      if (t == 0) {
        g.zin = rd.exchange_y ? S_in + (int64_t)n * ld : S_in;
        e = ceca::launch_margins(g, vec, st);
      } else {
        float* dst = (cur == W) ? S_out : W;
        g.px = cur;  g.py = cur + (int64_t)n * ld;
        g.ox = dst;  g.oy = dst + (int64_t)n * ld;
        g.pv = V2[(t - 1) & 1];
        g.p_shift = prev.shift;  g.p_port = port;
        g.p_exch_y = prev.exchange_y;  g.p_read_y = prev.b_num != 0;
        g.pa = prev.a;  g.pap = prev.a_peer;  g.pb = prev.b;  g.pbp = prev.b_peer;
        g.new_exch_y = rd.exchange_y;
        e = ceca::launch_margins_fused(g, vec, st);
        cur = dst;
        g.zin = rd.exchange_y ? cur + (int64_t)n * ld : cur;          // the half step reads z where the prologue put it
      }
      if (e != hipSuccess) return hip_fail(e, "margins kernel launch");
      e = ceca::launch_halfstep(g, vec, st);
      if (e != hipSuccess) return hip_fail(e, "half-step kernel launch");
      prev = rd;
    }
    // the last iteration's combine, from wherever the state lives into S_out
    ceca::ChainArgs a{};
    a.xin = cur;  a.yin = cur + (int64_t)n * ld;
    a.xout = S_out;  a.yout = S_out + (int64_t)n * ld;
    a.ld = ld;
    a.n = n;
    a.lr = lr;
    set_weights(prev, n, /*gossip_only=*/false, &a);
    a.aux = V2[(iters - 1) & 1];
    a.ldaux = p.ldv;
    return run_chain(a, ceca::MODE_FROMV, d, vec && aligned16(S_out) && ld % 4 == 0, prev, port, st);
  }
  ceca_loss_t one = *loss;
  if (!fused) {
    // one dsgd_ceca_step per iteration: the first from S_in to S_out, the rest in place on S_out
    for (int32_t t = 0; t < iters; ++t) {
      one.k = loss->k + (uint32_t)t;
      rc = dsgd_ceca_step(t == 0 ? S_in : S_out, S_out, n, d, ld, &one, batch_idx + (int64_t)t * nb, lr,
                          n == 1 ? 0 : (r0 + t) % tau, port, w + p.v_bytes, p.v_bytes + p.partial_bytes, st);
      if (rc != CECA_OK) return rc;
    }
    return CECA_OK;
  }
  if (copy_fits && !g_tuning.no_half_step) {
    // Between the iterations of this call the state lives in half-step form: rows xs = x - lr e, ys = y - lr e,
    // of which the travelling one is the iteration's message bit for bit (Eqs. (8), (9) combine exactly these).
    // Iteration t's kernel combines its agent's two rows with one row of its peer in registers, takes the
    // gradient at the new z and writes the next half-step rows to the other of two buffers (the copy in the
    // workspace and S_out): no message buffers, x+ and y+ never stored -- 20 bytes of state traffic per
    // agent-parameter and iteration instead of 28.  A closing combine (a gossip round's arithmetic on the
    // last half-step rows) writes x, y into S_out; the buffers alternate so that it reads the copy.
    float* W = reinterpret_cast<float*>(w + 2 * p.v_bytes + p.partial_bytes);
    auto H = [&](int32_t t) { return ((iters - 1 - t) & 1) == 0 ? W : S_out; };
    ceca::GemvArgs g{};
    g.ld = ld;  g.ldo = ld;
    g.A = loss->A;  g.lda = loss->lda;  g.t = loss->t;
    g.ldv = p.ldv;
    g.d = d;
    g.n = n;  g.N = loss->N;  g.B = loss->B;  g.kind = loss->kind;
    g.lr = lr;
    g.scale = loss->grad_scale > 0.0f ? loss->grad_scale : 1.0f / (float)loss->B;
    g.noise_std = loss->noise_std;
    g.seed = loss->seed;
    ceca_round_t prev{};
    for (int32_t t = 0; t < iters; ++t) {
      ceca::fill_round(n, (r0 + t) % tau, port, &rd);
      g.batch_idx = batch_idx + (int64_t)t * nb;
      g.k = loss->k + (uint32_t)t;
      const float* src = t == 0 ? S_in : H(t - 1);
      float* dst = H(t);
      g.px = src;  g.py = src + (int64_t)n * ld;
      g.ox = dst;  g.oy = dst + (int64_t)n * ld;
      g.p_first = t == 0;
      g.p_shift = prev.shift;  g.p_port = port;
      g.p_exch_y = prev.exchange_y;  g.p_read_y = prev.b_num != 0;
      g.pa = prev.a;  g.pap = prev.a_peer;  g.pb = prev.b;  g.pbp = prev.b_peer;
      g.new_exch_y = rd.exchange_y;
      hipError_t e = hipSuccess;
      if (!ceca::launch_grad_half(g, vec, st, &e)) return fail(CECA_EINVAL, "internal: fused gradient kernel does not cover this shape");
      if (e != hipSuccess) return hip_fail(e, "gradient kernel launch");
      prev = rd;
    }
    // x+ = a xs + (1 - a) v_peer, y+ = b ys + (1 - b) v_peer with v = the travelling half-step row: the
    // gradient-free round's kernel with the last iteration's weights, from the copy into S_out
    ceca::ChainArgs a{};
    a.xin = W;  a.yin = W + (int64_t)n * ld;
    a.xout = S_out;  a.yout = S_out + (int64_t)n * ld;
    a.ld = ld;
    a.n = n;
    set_weights(prev, n, /*gossip_only=*/true, &a);
    return run_chain(a, ceca::MODE_GOSSIP, d, vec && aligned16(S_out), prev, port, st);
  }
  float* V[2] = {reinterpret_cast<float*>(w), reinterpret_cast<float*>(w + p.v_bytes)};
  ceca::GemvArgs g{};
  g.ld = ld;
  g.A = loss->A;  g.lda = loss->lda;  g.t = loss->t;
  g.ldv = p.ldv;
  g.partial = reinterpret_cast<float*>(w + 2 * p.v_bytes);
  g.d = d;
  g.n = n;  g.N = loss->N;  g.B = loss->B;  g.kind = loss->kind;
  g.lr = lr;
  g.scale = loss->grad_scale > 0.0f ? loss->grad_scale : 1.0f / (float)loss->B;
  g.noise_std = loss->noise_std;
  g.seed = loss->seed;
  g.chunk_cols = ceca::kBlock * ceca::kChunkGroups * 4;
  g.nchunks = (int32_t)((d + g.chunk_cols - 1) / g.chunk_cols);
  const float* xin = S_in;
  const float* yin = S_in + (int64_t)n * ld;
  float* xout = S_out;
  float* yout = S_out + (int64_t)n * ld;
  hipError_t e = hipSuccess;
  ceca_round_t prev{};
  for (int32_t t = 0; t < iters; ++t) {
    ceca::fill_round(n, (r0 + t) % tau, port, &rd);
    g.batch_idx = batch_idx + (int64_t)t * nb;
    g.k = loss->k + (uint32_t)t;
    g.v = V[t & 1];
    if (t == 0) {
      g.zin = rd.exchange_y ? yin : xin;
      if (!(vec ? ceca::launch_grad_onepass(g, st, &e) : ceca::launch_grad_scalar(g, st, &e)))
        return fail(CECA_EINVAL, "internal: gradient kernel does not cover this shape");
    } else {
      // the state before iteration t-1's combine: S_in for t = 1, then S_out (updated row by row in place)
      g.px = (t == 1) ? xin : xout;
      g.py = (t == 1) ? yin : yout;
      g.ox = xout;  g.oy = yout;
      g.pv = V[(t - 1) & 1];
      g.p_shift = prev.shift;  g.p_port = port;
      g.p_exch_y = prev.exchange_y;  g.p_read_y = prev.b_num != 0;
      g.pa = prev.a;  g.pap = prev.a_peer;  g.pb = prev.b;  g.pbp = prev.b_peer;
      g.new_exch_y = rd.exchange_y;
      if (!ceca::launch_grad_fused(g, vec, st, &e)) return fail(CECA_EINVAL, "internal: fused gradient kernel does not cover this shape");
    }
    if (e != hipSuccess) return hip_fail(e, "gradient kernel launch");
    prev = rd;
  }
  // the last iteration's combine: from the state before it (S_out, or S_in when there was one iteration)
  ceca::ChainArgs a{};
  a.xin = xout;  a.yin = yout;
  a.xout = xout; a.yout = yout;
  a.ld = ld;
  a.n = n;
  a.lr = lr;
  set_weights(prev, n, /*gossip_only=*/false, &a);
  a.aux = V[(iters - 1) & 1];
  a.ldaux = p.ldv;
  return run_chain(a, ceca::MODE_FROMV, d, aligned16(S_out) && ld % 4 == 0, prev, port, st);
}

int32_t dsgd_ceca_steps(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld, const ceca_loss_t* loss,
                        float lr, int32_t r0, int32_t steps, int32_t port, void* hip_stream) {
  ceca_round_t rd;
  int32_t rc = check_state_call(S_in, S_out, n, d, ld, r0, port, &rd);
  if (rc != CECA_OK) return rc;
  rc = check_loss(loss, d, false, nullptr);
  if (rc != CECA_OK) return rc;
  if (loss->kind != CECA_LOSS_QUAD_CENTER)
    return fail(CECA_EINVAL, "fused iterations need an elementwise loss (CECA_LOSS_QUAD_CENTER)");
  if (steps < 1) return fail(CECA_EINVAL, "steps = %d: need at least one", steps);
  const int64_t sbytes = 2 * (int64_t)n * ld * 4, cbytes = (int64_t)n * loss->ldc * 4;
  if (overlaps(loss->c, cbytes, S_out, sbytes)) return fail(CECA_EINVAL, "centres overlap S_out");
  hipStream_t st = (hipStream_t)hip_stream;
  const int32_t tau = ceca::tau_of(n);
  const TileShape tv = steps_tile(n, true, steps), ts = steps_tile(n, false, steps);
  const bool can_vec = aligned16(S_in) && aligned16(S_out) && ld % 4 == 0 && aligned16(loss->c) && loss->ldc % 4 == 0;
  // A tile row narrower than a 128-byte line reads and writes HBM several times less efficiently than
  // the streaming single-step kernel, which only pays off over enough iterations (measured at n = 1026,
  // 2050, 4096: the fused pass costs about 2, 6 and 11 single steps at 64, 32 and 16 bytes).
  const int32_t row_bytes = can_vec ? tv.row_bytes(true) : ts.row_bytes(false);
  const int32_t worth = row_bytes >= 128 ? 1 : (row_bytes >= 64 ? 3 : (row_bytes >= 32 ? 8 : 14));
  // (the steps after the first run in place on S_out: with two ports those walk whole cycles, which
  // needs many column tiles to fill the device)
  const bool steps_fill = port == 1 || d >= 1024 * 1024;
  const bool knobs = g_tuning.rows != 0 || g_tuning.tile_threads != 0;
  if (n == 1 || !tv.ok || !ts.ok || (steps < worth && steps_fill && !knobs)) {
    ceca_loss_t one = *loss;
    for (int32_t t = 0; t < steps; ++t) {
      one.k = loss->k + (uint32_t)t;
      const int32_t r1 = dsgd_ceca_step(t == 0 ? S_in : S_out, S_out, n, d, ld, &one, nullptr, lr,
                                        n == 1 ? 0 : (r0 + t) % tau, port, nullptr, 0, st);
      if (r1 != CECA_OK) return r1;
    }
    return CECA_OK;
  }
  const int64_t d4 = can_vec ? d / 4 : 0;
  // one kernel takes up to kMultiMaxRounds iterations; longer runs go in pieces, the first from S_in
  // to S_out and the rest in place on S_out (a workgroup holds its whole tile before it writes)
  for (int32_t t0 = 0; t0 < steps; t0 += ceca::kMultiMaxRounds) {
    const int32_t cnt = std::min(steps - t0, ceca::kMultiMaxRounds);
    const float* src = t0 == 0 ? S_in : S_out;
    ceca::StepsArgs a{};
    ceca::MultiArgs& m = a.m;
    m.xin = src;
    m.xout = S_out;  m.yout = S_out + (int64_t)n * ld;
    m.ld = ld;
    m.n = n;  m.port = port;  m.rounds = cnt;
    for (int32_t t = 0; t < cnt; ++t) {
      ceca::fill_round(n, (r0 + t0 + t) % tau, port, &rd);
      ceca::MultiRound& R = m.round[t];
      R.shift = rd.shift;  R.exch_y = rd.exchange_y;  R.read_y = rd.b_num != 0;
      R.a = rd.a;  R.ap = rd.a_peer;  R.b = rd.b;  R.bp = rd.b_peer;
    }
    a.yin = src + (int64_t)n * ld;
    a.c = loss->c;  a.ldc = loss->ldc;
    a.lr = lr;  a.noise_std = loss->noise_std;  a.seed = loss->seed;  a.k0 = loss->k + (uint32_t)t0;
    if (d4 > 0) {
      m.col0 = 0;  m.ngroups = d4;
      m.threads = tv.threads;  m.row_lanes = tv.row_lanes;  m.rows_per_thread = tv.rows_per_thread;
      const hipError_t e = ceca::launch_multi_step(a, true, st);
      if (e != hipSuccess) return hip_fail(e, "multi-step kernel launch");
    }
    if (d - 4 * d4 > 0) {
      m.col0 = 4 * d4;  m.ngroups = d - 4 * d4;
      m.threads = ts.threads;  m.row_lanes = ts.row_lanes;  m.rows_per_thread = ts.rows_per_thread;
      const hipError_t e = ceca::launch_multi_step(a, false, st);
      if (e != hipSuccess) return hip_fail(e, "multi-step kernel launch (scalar columns)");
    }
  }
  return CECA_OK;
}

int32_t ceca_topology_round(int32_t kind, int32_t n, int32_t k, ceca_mix_t* out) {
  if (!out) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || k < 0) return fail(CECA_EINVAL, "need n >= 1 and k >= 0");
  if (!ceca::fill_topology(kind, n, k, out)) return fail(CECA_EINVAL, "topology kind %d with n = %d: unknown kind, or more than %d peers", kind, n, CECA_MIX_MAX);
  return CECA_OK;
}

int32_t ceca_mix_rounds(const float* X_in, float* X_out, int32_t n, int64_t d, int64_t ld, const ceca_mix_t* specs,
                        int32_t period, int32_t k0, int32_t rounds, void* hip_stream) {
  if (!X_in || !X_out || !specs) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || n > 4096) return fail(CECA_EINVAL, "n = %d: mixing rounds take 1 to 4096 agents", n);
  if (d < 1 || ld < d) return fail(CECA_EINVAL, "need 1 <= d <= ld (d = %lld, ld = %lld)", (long long)d, (long long)ld);
  if (period < 1 || period > ceca::kMixMaxPeriod) return fail(CECA_EINVAL, "period = %d outside [1, %d]", period, ceca::kMixMaxPeriod);
  if (k0 < 0 || rounds < 1) return fail(CECA_EINVAL, "need k0 >= 0 and rounds >= 1");
  const int64_t bytes = (int64_t)n * ld * (int64_t)sizeof(float);
  if (overlaps(X_in, bytes, X_out, bytes) && (const void*)X_in != (const void*)X_out)
    return fail(CECA_EINVAL, "X_out partially overlaps X_in");
  ceca::MixArgs m{};
  int32_t total = 0;
  for (int32_t q = 0; q < period; ++q) {
    const ceca_mix_t& sp = specs[q];
    if (sp.m < 0 || sp.m > CECA_MIX_MAX) return fail(CECA_EINVAL, "round %d: m = %d outside [0, %d]", q, sp.m, CECA_MIX_MAX);
    if (total + sp.m > ceca::kMixMaxPeers) return fail(CECA_EINVAL, "more than %d peers over the period", ceca::kMixMaxPeers);
    m.start[q] = total;
    m.w_self[q] = sp.w_self;
    for (int32_t j = 0; j < sp.m; ++j) {
      if (sp.shift[j] < 0 || sp.shift[j] >= n) return fail(CECA_EINVAL, "round %d: shift %d outside [0, n)", q, sp.shift[j]);
      m.shift[total] = sp.shift[j];
      m.w[total] = sp.w[j];
      ++total;
    }
  }
  m.start[period] = total;
  m.xin = X_in;  m.xout = X_out;  m.ld = ld;
  m.n = n;  m.rounds = rounds;  m.period = period;  m.k0 = k0 % period;
  int32_t most = 0;
  for (int32_t q = 0; q < period; ++q) most = std::max(most, specs[q].m);
  const TileShape tv = mix_tile(n, true, most >= 4), ts = mix_tile(n, false, most >= 4);
  if (!tv.ok || !ts.ok) return fail(CECA_EINVAL, "internal: no tile holds n = %d agents", n);
  hipStream_t st = (hipStream_t)hip_stream;
  const bool can_vec = aligned16(X_in) && aligned16(X_out) && ld % 4 == 0;
  const int64_t d4 = can_vec ? d / 4 : 0;
  if (d4 > 0) {
    m.col0 = 0;  m.ngroups = d4;
    m.threads = tv.threads;  m.row_lanes = tv.row_lanes;  m.rows_per_thread = tv.rows_per_thread;
    const hipError_t e = ceca::launch_mix_rounds(m, true, st);
    if (e != hipSuccess) return hip_fail(e, "mixing kernel launch");
  }
  if (d - 4 * d4 > 0) {
    m.col0 = 4 * d4;  m.ngroups = d - 4 * d4;
    m.threads = ts.threads;  m.row_lanes = ts.row_lanes;  m.rows_per_thread = ts.rows_per_thread;
    const hipError_t e = ceca::launch_mix_rounds(m, false, st);
    if (e != hipSuccess) return hip_fail(e, "mixing kernel launch (scalar columns)");
  }
  return CECA_OK;
}

int32_t ceca_graph_rounds(const float* X_in, float* X_out, int32_t n, int64_t d, int64_t ld, const int32_t* nbr,
                          const float* w, const float* w_self, int32_t m, int32_t period, int32_t k0, int32_t rounds,
                          void* hip_stream) {
  if (!X_in || !X_out || !nbr || !w || !w_self) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || n > 4096) return fail(CECA_EINVAL, "n = %d: graph gossip rounds take 1 to 4096 agents", n);
  if (d < 1 || ld < d) return fail(CECA_EINVAL, "need 1 <= d <= ld (d = %lld, ld = %lld)", (long long)d, (long long)ld);
  if (m < 1 || m > ceca::kGraphMaxDegree) return fail(CECA_EINVAL, "m = %d outside [1, %d]", m, ceca::kGraphMaxDegree);
  if (period < 1 || k0 < 0 || rounds < 1) return fail(CECA_EINVAL, "need period >= 1, k0 >= 0 and rounds >= 1");
  const int64_t bytes = (int64_t)n * ld * (int64_t)sizeof(float);
  if (overlaps(X_in, bytes, X_out, bytes) && (const void*)X_in != (const void*)X_out)
    return fail(CECA_EINVAL, "X_out partially overlaps X_in");
  const int64_t entries = (int64_t)period * n * m;
  if (overlaps(nbr, entries * 4, X_out, bytes) || overlaps(w, entries * 4, X_out, bytes) ||
      overlaps(w_self, (int64_t)period * n * 4, X_out, bytes))
    return fail(CECA_EINVAL, "the graph tables overlap X_out");
  const TileShape tv = graph_tile(n, true), ts = graph_tile(n, false);
  if (!tv.ok || !ts.ok) return fail(CECA_EINVAL, "internal: no tile holds n = %d agents", n);
  ceca::GraphArgs g{};
  g.xin = X_in;  g.xout = X_out;  g.ld = ld;
  g.nbr = nbr;  g.w = w;  g.w_self = w_self;
  g.n = n;  g.m = m;  g.rounds = rounds;  g.period = period;  g.k0 = k0 % period;
  g.stage = !g_tuning.graph_tables_in_memory;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool can_vec = aligned16(X_in) && aligned16(X_out) && ld % 4 == 0;
  const int64_t d4 = can_vec ? d / 4 : 0;
  if (d4 > 0) {
    g.col0 = 0;  g.ngroups = d4;
    g.threads = tv.threads;  g.row_lanes = tv.row_lanes;  g.rows_per_thread = tv.rows_per_thread;
    const hipError_t e = ceca::launch_graph_rounds(g, true, st);
    if (e != hipSuccess) return hip_fail(e, "graph gossip kernel launch");
  }
  if (d - 4 * d4 > 0) {
    g.col0 = 4 * d4;  g.ngroups = d - 4 * d4;
    g.threads = ts.threads;  g.row_lanes = ts.row_lanes;  g.rows_per_thread = ts.rows_per_thread;
    const hipError_t e = ceca::launch_graph_rounds(g, false, st);
    if (e != hipSuccess) return hip_fail(e, "graph gossip kernel launch (scalar columns)");
  }
  return CECA_OK;
}

int32_t ceca_describe_step_launch(int32_t n, int64_t d, int64_t ld, int32_t r, int32_t port, int32_t kind,
                                  int32_t in_place, int32_t* out) {
  if (!out) return fail(CECA_EINVAL, "null pointer");
  if (kind < 0 || kind > 2) return fail(CECA_EINVAL, "kind must be 0 (gossip round), 1 (fused quadratic-centre step) or 2 (combine of a minibatch step)");
  // stand-in addresses (never dereferenced): only their equality and alignment enter the launch shape
  const float* S_in = reinterpret_cast<const float*>(uintptr_t(1) << 20);
  float* S_out = in_place ? const_cast<float*>(S_in) : reinterpret_cast<float*>(uintptr_t(1) << 50);
  ceca_round_t rd;
  const int32_t rc = check_state_call(S_in, S_out, n, d, ld, r, port, &rd);
  if (rc != CECA_OK) return rc;
  ceca::ChainArgs a{};
  a.xin = S_in;  a.yin = S_in + (int64_t)n * ld;
  a.xout = S_out; a.yout = S_out + (int64_t)n * ld;
  a.ld = ld;
  a.n = n;
  set_weights(rd, n, /*gossip_only=*/kind == 0, &a);
  const int mode = kind == 1 ? ceca::MODE_QUAD : (kind == 2 ? ceca::MODE_FROMV : ceca::MODE_GOSSIP);
  const ChainPlan pl = plan_chain(&a, mode, d, port);
  const bool vec = ld % 4 == 0;
  const int64_t groups = vec ? d / 4 : d;
  shape_chain(rd, n, port, pl.in_place, pl.default_seg, std::max<int64_t>(groups, 1), &a);
  out[0] = pl.rows;
  out[1] = (int32_t)a.band;
  out[2] = a.wg_per_cu;
  out[3] = a.seg_len;
  out[4] = a.segs_per_cycle;
  out[5] = vec ? 4 : 1;
  return CECA_OK;
}

int32_t ceca_stream_probe(const float* a, const float* b, const float* c, float* o1, float* o2, int64_t count,
                          int32_t reads, int32_t writes, void* hip_stream) {
  if (reads < 1 || reads > 3 || writes < 0 || writes > 2) return fail(CECA_EINVAL, "the probe takes 1..3 reads and 0..2 writes");
  if (!a || (reads >= 2 && !b) || (reads >= 3 && !c) || !o1 || (writes >= 2 && !o2)) return fail(CECA_EINVAL, "null pointer");
  if (count < 4 || count % 4 != 0) return fail(CECA_EINVAL, "count must be a positive multiple of 4");
  if (!aligned16(a) || !aligned16(b) || !aligned16(c) || !aligned16(o1) || !aligned16(o2))
    return fail(CECA_EINVAL, "the probe takes 16-byte aligned arrays");
  const hipError_t e = ceca::launch_stream_probe(a, b, c, o1, o2, count / 4, reads, writes, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "probe kernel launch");
  return CECA_OK;
}

int64_t consensus_error_workspace_bytes(int32_t n, int64_t d) {
  if (n < 1 || d < 1) return fail(CECA_EINVAL, "need n >= 1 and d >= 1");
  return cons_plan(n, d).bound;
}

namespace {

// The consensus kernels on `workspace` (checked by the caller to be 256-byte aligned); *need receives the
// bytes this problem's form uses, and nothing is launched when `have` is smaller.
int32_t run_consensus(const float* X, int32_t n, int64_t d, int64_t ld, double* out, float* xbar_or_null,
                      char* w, int64_t have, int64_t* need, hipStream_t st) {
  const ConsPlan p = cons_plan(n, d);
  ceca::ConsensusArgs c{};
  c.X = X;  c.ld = ld;  c.d = d;  c.n = n;
  c.out = out;
  c.xbar = xbar_or_null;
  const bool vec = aligned16(X) && ld % 4 == 0 && d % 4 == 0;
  const int32_t forced = g_tuning.cons_form;
  int form = CONS_TWO_PASS;
  if (forced == CONS_WAVE ? p.wave_cgs > 0 : (forced == 0 && p.wave_cgs > 0 && p.wave_default)) form = CONS_WAVE;
  else if (forced != CONS_TWO_PASS && p.rows_per_thread > 0) form = CONS_TILE;
  if (form == CONS_WAVE) {
    const ConsWave cw = cons_wave(p, n, d, vec);
    *need = cw.total;
    if (have < cw.total) return CECA_EWORKSPACE;
    c.wave_cgs = p.wave_cgs;  c.cg_shift = p.wave_shift;  c.rows_per_thread = p.wave_rows;
    c.strips = cw.strips;  c.nwaves = cw.nwaves;
    c.devpart = reinterpret_cast<double*>(w);
    c.dev2 = reinterpret_cast<double*>(w + cw.off_dev2);
  } else if (form == CONS_TILE) {
    // single pass over x; the workspace then holds only the partials: normpart[ntiles], devpart[n][ntiles], dev2[n]
    c.ntiles = vec ? p.tile_ntiles_vec : p.tile_ntiles_scalar;
    const int64_t off_devpart = round_up(c.ntiles * 8, 256);
    const int64_t off_dev2 = off_devpart + round_up((int64_t)n * c.ntiles * 8, 256);
    *need = off_dev2 + round_up((int64_t)n * 8, 256);
    if (have < *need) return CECA_EWORKSPACE;
    c.rows_per_thread = p.rows_per_thread;
    c.row_lanes = p.row_lanes;
    c.normpart = reinterpret_cast<double*>(w);
    c.devpart = reinterpret_cast<double*>(w + off_devpart);
    c.dev2 = reinterpret_cast<double*>(w + off_dev2);
  } else {
    *need = p.two_pass_total;
    if (have < p.two_pass_total) return CECA_EWORKSPACE;
    c.agent_groups = p.agent_groups;
    c.agents_per_group = p.agents_per_group;
    c.dev_agents = p.dev_agents;
    c.ntiles = p.ntiles;
    c.colsum = reinterpret_cast<double*>(w);
    c.normpart = reinterpret_cast<double*>(w + p.off_norm);
    c.devpart = reinterpret_cast<double*>(w + p.off_devpart);
    c.dev2 = reinterpret_cast<double*>(w + p.off_dev2);
  }
  const hipError_t e = ceca::launch_consensus(c, vec, st);
  if (e != hipSuccess) return hip_fail(e, "consensus kernels launch");
  return CECA_OK;
}

}  // namespace

int32_t consensus_error(const float* X, int32_t n, int64_t d, int64_t ld, double* out, float* xbar_or_null,
                        void* workspace, int64_t workspace_bytes, void* hip_stream) {
  if (!X || !out) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || d < 1 || ld < d) return fail(CECA_EINVAL, "need n >= 1 and 1 <= d <= ld");
  const int64_t bound = cons_plan(n, d).bound;
  if (!workspace || workspace_bytes < bound)
    return fail(CECA_EWORKSPACE, "workspace of %lld bytes needed, %lld given", (long long)bound,
                (long long)(workspace ? workspace_bytes : 0));
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return fail(CECA_EWORKSPACE, "workspace must be 256-byte aligned");
  int64_t need = 0;
  const int32_t rc = run_consensus(X, n, d, ld, out, xbar_or_null, reinterpret_cast<char*>(workspace), workspace_bytes, &need,
                                   (hipStream_t)hip_stream);
  if (rc == CECA_EWORKSPACE)
    return fail(CECA_EWORKSPACE, "internal: this launch shape needs %lld bytes of workspace, the bound is %lld", (long long)need,
                (long long)bound);
  return rc;
}

int32_t consensus_error_noalloc(const float* X, int32_t n, int64_t d, int64_t ld, double* out, float* xbar_or_null,
                                void* hip_stream) {
  if (!X || !out) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || d < 1 || ld < d) return fail(CECA_EINVAL, "need n >= 1 and 1 <= d <= ld");
  char* w = nullptr;
  int32_t rc = scratch_of_current_device(&w);
  if (rc != CECA_OK) return rc;
  // every partial sum the kernels read was written by an earlier kernel of this same call, so the array
  // needs no clearing between calls
  int64_t need = 0;
  rc = run_consensus(X, n, d, ld, out, xbar_or_null, w, kScratchBytes, &need, (hipStream_t)hip_stream);
  if (rc == CECA_EWORKSPACE)
    return fail(CECA_EWORKSPACE, "n = %d, d = %lld needs %lld bytes of scratch memory, the allocation-free entry point holds %lld: "
                "use consensus_error with a workspace", n, (long long)d, (long long)need, (long long)kScratchBytes);
  return rc;
}

int32_t ceca_state_consensus(const float* S, int32_t n, int64_t d, int64_t ld, double* out, void* workspace,
                             int64_t workspace_bytes, void* hip_stream) {
  if (!S || !out) return fail(CECA_EINVAL, "null pointer");
  if (n < 1 || d < 1 || ld < d) return fail(CECA_EINVAL, "need n >= 1 and 1 <= d <= ld");
  int32_t rc = consensus_error(S, n, d, ld, out, nullptr, workspace, workspace_bytes, hip_stream);
  if (rc != CECA_OK) return rc;
  rc = consensus_error(S + (int64_t)n * ld, n, d, ld, out + 5, nullptr, workspace, workspace_bytes, hip_stream);
  if (rc != CECA_OK) return rc;
  const hipError_t e = ceca::launch_phi(out, (hipStream_t)hip_stream);
  if (e != hipSuccess) return hip_fail(e, "phi kernel launch");
  return CECA_OK;
}

}  // extern "C"
