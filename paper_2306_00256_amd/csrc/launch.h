// Internal interface between the C ABI (api.cpp) and the gfx950 kernels (chain.hip, multi_round.hip,
// gemv.hip, consensus.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ceca {

// What an agent contributes in one iteration (Algorithm 1): its "self" terms x_i - lr e_i and
// y_i - lr e_i, and the message v_i = z_i - lr e_i it sends.
enum ChainMode : int {
  MODE_GOSSIP = 0,  // e = 0: self terms are x, y and the message is z             (Sec. 3 recursions)
  MODE_QUAD = 1,    // e = z - c + noise, generated in the kernel                  (fused step)
  MODE_FROMV = 2,   // message v was written by the half-step kernel; x - lr e = x + (v - z)
  MODE_GRAD = 3     // e is read from memory (the caller's gradients)
};

struct ChainArgs {
  const float* xin;   // row 0 of x in S_in
  const float* yin;   // row 0 of y in S_in
  float* xout;
  float* yout;
  int64_t ld;
  const float* aux;   // MODE_QUAD: centres c;  MODE_FROMV: messages v;  MODE_GRAD: gradients e
  int64_t ldaux;
  int64_t col0;       // first column of this launch
  int64_t ngroups;    // VEC-wide column groups in this launch
  uint32_t tiles;     // workgroups per chain stretch (set by the launcher)
  uint32_t nsegs;     // stretches over all cycles (set by the launcher)
  uint32_t band;      // column tiles per band of the launch order (0 = all tiles in one band)
  int32_t wg_per_cu;  // cap on resident workgroups per CU (0 = whatever fits)
  int32_t n;
  int32_t stride;     // walk step: the agent after c is (c + stride) mod n, and it receives from c
  int32_t cyc_len;    // agents per cycle of the walk
  int32_t segs_per_cycle;
  int32_t seg_len;    // agents per chain segment (last segment of a cycle may be shorter)
  int32_t c0_mul;     // first agent of cycle j is j * c0_mul
  int32_t exch_y;     // 1: z = y
  int32_t read_y;     // 0: b == 0, y rows are not read
  float a, ap, b, bp;
  float lr, noise_std;
  uint32_t seed, k;
};

// One round of the multi-round kernel: weights and travelling variable (Algorithm 1's a, b, z).
struct MultiRound {
  int32_t shift, exch_y, read_y;
  float a, ap, b, bp;
};

constexpr int kMultiRows = 16;       // most rows of (x, y) a thread of the multi-round kernel keeps in registers
constexpr int kMultiMaxRounds = 64;
constexpr size_t kMultiMaxLds = 160 * 1024;   // LDS one workgroup can have on gfx950

struct MultiArgs {
  const float* xin;    // row 0 of x in S_in (y of S_in is not read: round 0 overwrites it)
  float* xout;
  float* yout;         // NULL: y is not stored (exact averaging only needs x)
  int64_t ld;
  int64_t col0;
  int64_t ngroups;
  int32_t n, port, rounds;
  int32_t xcd_tiles;        // > 0: workgroup b takes tile (b % 8) * xcd_tiles + b / 8 (set by the launcher)
  int32_t rows_per_thread;  // 1 to 16 rows of (x, y) in a thread's registers
  int32_t row_lanes;   // power of two, row_lanes * rows_per_thread >= n: threads of a workgroup that share a column group
  int32_t threads;     // threads per workgroup of the gossip-rounds kernel: 0 = 256, or 512 / 1024 (16-byte groups only);
                       // 512 / 1024 keep at most 9 rows per thread in registers without spilling
  int32_t lean;        // gossip-rounds kernel, 256 threads, 16-byte groups: 4, 5 or 6 = register-lean form compiled
                       // for that many wavefronts per SIMD (0 = the plain form)
  MultiRound round[kMultiMaxRounds];
};

struct GemvArgs {
  const float* zin;       // row 0 of the variable the gradient is taken at (x or y rows of S_in)
  int64_t ld;
  const float* A;
  int64_t lda;
  const float* t;
  const int32_t* batch_idx;
  float* partial;         // [n][nchunks][B] partial margins
  float* v;               // [n][ldv] messages
  int64_t ldv;
  int64_t d;
  int32_t n, N, B, kind;
  int32_t nchunks;
  int32_t chunk_cols;
  float lr;
  float scale;            // factor on sum_j coef_j a_ij: 1/B, or the caller's grad_scale
  float noise_std;        // additive Gaussian gradient noise (0 = none), keyed by (seed, k)
  uint32_t seed, k;
  // Fused form only (launch_grad_fused): the combine of the iteration before runs as a prologue.
  // z is then the x or y row (new_exch_y) of the state this prologue produces.
  const float* px;        // row 0 of x, y before that combine
  const float* py;
  float* ox;              // row 0 of x, y after it (launch_grad_fused: may be px, py, a workgroup touches only its
  float* oy;              // agent's rows, pitch ld; launch_margins_fused: another buffer, pitch ldo)
  int64_t ldo;
  const float* pv;        // messages of the iteration before, [n][ldv]
  int32_t p_shift, p_port, p_exch_y, p_read_y;
  float pa, pap, pb, pbp; // its weights
  int32_t new_exch_y;
  int32_t p_first;        // half-step form only: 1 = no iteration before (px, py are x, y themselves)
};

struct ConsensusArgs {
  const float* X;
  int64_t ld;
  int64_t d;
  int32_t n;
  int32_t agent_groups;    // partial column sums are taken over this many slices of the agents
  int32_t agents_per_group;
  int32_t dev_agents;      // agents one workgroup of the deviation kernel walks
  int64_t ntiles;          // column tiles of 1024
  double* colsum;          // [agent_groups][d]; slice 0 becomes the fp64 mean
  double* normpart;        // [ntiles] partial ||xbar||^2
  double* devpart;         // [n][ntiles] partial squared deviations
  double* dev2;            // [n]
  double* out;             // 5 results
  float* xbar;             // optional
  // single-pass form (every agent's column tile in one workgroup's registers); 0 rows = two-pass form
  int32_t rows_per_thread; // 1..32 rows of x per thread
  int32_t row_lanes;       // power of two, row_lanes * rows_per_thread >= n
  // wavefront-per-strip form of the single pass (wave_cgs > 0): devpart is [n + 1][nwaves], dev2 has n + 1 entries
  int32_t wave_cgs;        // column groups per strip: a power of two, 64 / wave_cgs row lanes share a group
  int32_t cg_shift;        // log2(wave_cgs)
  int64_t strips;          // column strips in all
  int64_t nwaves;          // wavefronts launched; wavefront w takes strips w, w + nwaves, ...
  int64_t norm_count;      // entries of normpart (set by the launcher)
  int32_t close_rows;      // rows of devpart the closing kernels reduce (set by the launcher)
};

// Fused iterations with the quadratic-centre loss: the rounds of MultiArgs plus what the gradient needs.
// Iteration t uses round m.round[t] and the noise counter k0 + t.
struct StepsArgs {
  MultiArgs m;
  const float* yin;     // row 0 of y in S_in
  const float* c;       // centres
  int64_t ldc;
  float lr, noise_std;
  uint32_t seed, k0;
};

constexpr int kMixMaxPeriod = 16;    // distinct rounds of a mixing sequence
constexpr int kMixMaxPeers = 64;     // peers summed over those rounds

// Shift-invariant mixing rounds on x alone: round t applies entries
// [start[(k0 + t) % period], start[(k0 + t) % period + 1]) of (shift, w) and w_self of that round.
struct MixArgs {
  const float* xin;
  float* xout;
  int64_t ld;
  int64_t col0;
  int64_t ngroups;
  int32_t n, rounds, period, k0;
  int32_t rows_per_thread;  // rows of x in a thread's registers: 1 to 32, the least that covers n
  int32_t row_lanes;        // power of two, row_lanes * rows_per_thread >= n
  int32_t threads;          // threads per workgroup: 0 = 256, or 512 / 1024 (16-byte groups only, at most 16 rows per thread)
  int32_t xcd_tiles;        // > 0: workgroup b takes tile (b % 8) * xcd_tiles + b / 8 (set by the launcher)
  int32_t start[kMixMaxPeriod + 1];
  float w_self[kMixMaxPeriod];
  int32_t shift[kMixMaxPeers];
  float w[kMixMaxPeers];
};

constexpr int kGraphRows = 16;      // most rows of x a thread of the graph-gossip kernel keeps in registers
constexpr int kGraphMaxDegree = 64; // most neighbours per vertex and round
constexpr int kGraphStageEntries = 12;   // a round's table is staged in LDS when each thread copies at most this many entries

struct GraphArgs {
  const float* xin;
  float* xout;
  int64_t ld;
  int64_t col0;
  int64_t ngroups;
  const int32_t* nbr;       // device, [period][n][m]: neighbour j of vertex i in the round's graph
  const float* w;           // device, [period][n][m]: its weight
  const float* w_self;      // device, [period][n]
  int32_t n, m, rounds, period, k0;
  int32_t rows_per_thread;  // 1 to kGraphRows, the least that covers n
  int32_t row_lanes;        // power of two, row_lanes * rows_per_thread >= n
  int32_t threads;          // threads per workgroup: 0 = 256, or 512 / 1024 (16-byte groups only)
  int32_t stage;            // 1: stage small tables in LDS (0: always read them from memory)
  int32_t xcd_tiles;        // set by the launcher
};

// Launch-shape overrides of the calling thread, set through the test and measurement interface
// (ceca_test.h).  Zero everywhere = the library's own choices, which is all the product ABI ever sees on a
// thread that never touched that interface.
struct Tuning {
  int32_t segment;              // agents a two-port chain walks before it starts a new one
  int32_t rows;                 // rows in flight (streaming kernels) / most rows per thread (register-tile kernels)
  int32_t band;                 // column tiles per band of the launch order
  int32_t wg_per_cu;            // cap on workgroups resident per compute unit
  int32_t tile_threads;         // threads per workgroup of the register-tile kernels: 256, 512, 1024
  int32_t agents_per_wg;        // agents one workgroup of the looping one-pass gradient kernel takes in turn
  int32_t two_pass_gradient;    // 1: minibatch gradients always take the margins / half-step kernels
  int32_t never_chunked;        // 1: single steps never take the chunked gradient kernel
  int32_t cons_form;            // consensus observables: 1 two-pass, 2 workgroup tiles, 3 wavefront strips
  int32_t cons_strips;          // strips one wavefront of the consensus kernel takes in turn
  int32_t plain_tile_order;     // 1: register-tile kernels never use the XCD-contiguous tile order
  int32_t graph_tables_in_memory;  // 1: graph gossip reads its tables from memory at every look-up
  int32_t no_half_step;         // 1: dsgd_ceca_run keeps full states and message buffers between fused iterations
  int32_t lean_tiles;           // gossip-rounds kernel with 256 threads: 4, 5, 6 = the register-lean form for that many wavefronts per SIMD
  int32_t probe_variant;        // 3-read / 2-write probe: policy * 100 + threads code * 10 + column groups per thread
  int32_t probe_waves;          // probe kernels: that many long-lived wavefronts instead of one thread per column group
};
extern thread_local Tuning g_tuning;

// rows: state rows whose loads a thread keeps in flight together (1, 2, 4 or 8)
hipError_t launch_chain(const ChainArgs& a, int mode, bool vec4, int rows, hipStream_t st);
// one-pass gradient (vector layouts only): returns false when no register tile covers (B, d)
bool launch_grad_onepass(const GemvArgs& g, hipStream_t st, hipError_t* err);
// gradient kernel with the previous iteration's combine as its prologue; false when the shape is not covered
bool launch_grad_fused(const GemvArgs& g, bool vec4, hipStream_t st, hipError_t* err);
bool grad_fused_covers(int32_t n, int64_t d, int32_t B, bool vec4);
// the fused form with the state in half-step rows between iterations: reads px, py (pitch ld), writes ox, oy
// (pitch ldo, another buffer unless p_first); false when the shape is not covered
bool launch_grad_half(const GemvArgs& g, bool vec4, hipStream_t st, hipError_t* err);
// single-step gradient for layouts that are not 16-byte aligned (rows up to 1024 columns); false otherwise
bool launch_grad_scalar(const GemvArgs& g, hipStream_t st, hipError_t* err);
hipError_t launch_multi_round(const MultiArgs& m, bool vec4, hipStream_t st);
hipError_t launch_mix_rounds(const MixArgs& m, bool vec4, hipStream_t st);
hipError_t launch_multi_step(const StepsArgs& s, bool vec4, hipStream_t st);
hipError_t launch_graph_rounds(const GraphArgs& m, bool vec4, hipStream_t st);
hipError_t launch_margins(const GemvArgs& g, bool vec4, hipStream_t st);
// margins with the previous iteration's combine as prologue: reads px, py (pitch ld), stores ox, oy (pitch ldo)
hipError_t launch_margins_fused(const GemvArgs& g, bool vec4, hipStream_t st);
hipError_t launch_halfstep(const GemvArgs& g, bool vec4, hipStream_t st);
hipError_t launch_consensus(const ConsensusArgs& c, bool vec4, hipStream_t st);
// measurement aid: o1, o2 <- elementwise functions of a, b, c (ngroups groups of 4 floats, 16-byte aligned);
// reads 1..3 of a, b, c and writes 0..2 of o1, o2 are touched
hipError_t launch_stream_probe(const float* a, const float* b, const float* c, float* o1, float* o2, int64_t ngroups,
                               int reads, int writes, hipStream_t st);
// out[10] = out[0] + out[5] (11 doubles on the device)
hipError_t launch_phi(double* out, hipStream_t st);

constexpr int kBlock = 256;          // threads per workgroup: 4 wavefronts of 64
constexpr int kChunkGroups = 1;      // column groups per thread in the margins kernel
constexpr int kRowGroup = 8;         // sampled rows whose loads the two-pass gradient kernels keep in flight
constexpr int64_t kConsTile = 1024;  // columns per workgroup in the consensus kernels

}  // namespace ceca
