/*
 * ceca.h -- C ABI of the DSGD-CECA hot path for one AMD MI355X (gfx950).
 *
 * All n agents of a decentralized run are simulated on one device as rows of a
 * stacked state S = [x; y]: 2n rows of `ld` floats, rows 0..n-1 hold the models
 * x_i, rows n..2n-1 the auxiliary models y_i (stacked notation of Sec. 4.1 and
 * App. A of the DSGD-CECA paper, arXiv 2306.00256).  One iteration = one local
 * stochastic-gradient step per agent plus one CECA communication round
 * (Algorithm 1); tau = ceil(log2 n) gradient-free rounds leave every x_i equal
 * to the global mean for any n (Sec. 3).
 *
 * Conventions
 *   - Every function returns an int32 status (0 = CECA_OK, negative = error) or a
 *     byte count; nothing aborts or throws.  ceca_last_error() gives a message for
 *     the calling thread's most recent failure.
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     never allocates, frees or retains them.  "host" pointers are ordinary memory.
 *   - Device calls are asynchronous on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream); the library never synchronizes.
 *   - Agents and rounds are 0-based: row i is the paper's agent i+1, r = k mod tau
 *     is the ordinary remainder in [0, tau) (Algorithm 1).
 *   - Any base pointer / leading dimension is accepted; 16-byte aligned bases with
 *     leading dimensions that are multiples of 4 take the vectorized kernels, other
 *     layouts silently take a scalar kernel with identical results.
 *   - The functions declared here keep no mutable state between calls beyond the calling
 *     thread's last error (ceca_last_error, ceca_last_hip_error) and may be called from
 *     several threads at once.  Launch shapes are the library's own; the per-thread
 *     overrides that tests and measurement sweeps use live in ceca_test.h, which is not
 *     part of this interface.
 */
#ifndef CECA_H
#define CECA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CECA_OK = 0,
  CECA_EINVAL = -1,     /* bad size, round, port, leading dimension, null pointer, or forbidden aliasing */
  CECA_EODD1P = -2,     /* port == 1 with odd n: CECA-1P exists for even n only (Table 1, Sec. 3.2) */
  CECA_EWORKSPACE = -3, /* workspace missing or smaller than the matching *_workspace_bytes() */
  CECA_EHIP = -4        /* a HIP runtime call failed; see ceca_last_hip_error() */
};

enum { CECA_LOSS_LSQ = 0, CECA_LOSS_LOGISTIC = 1, CECA_LOSS_QUAD_CENTER = 2, CECA_LOSS_GRADIENT = 3 };

/* One CECA round, as Algorithm 1 uses it (Sec. 3.1 Eqs. (2), (3); Sec. 4.1). */
typedef struct {
  int32_t n, tau, r, port;
  int32_t delta;        /* delta_r: bit tau-1-r of n-1 (Eq. (2), most significant first) */
  int32_t n_r;          /* window size before the round (Eq. (3)) */
  int32_t shift;        /* 2 ports: n_r + delta_r, row i receives from row i - shift (Eqs. (5), (6));
                           1 port: 2 n_r + 1, even rows pair with i + shift, odd rows with i - shift (Eq. (7)) */
  int32_t exchange_y;   /* 0: z = x travels (delta_r = 1);  1: z = y travels (delta_r = 0) */
  int32_t a_num, a_den; /* self-weight a of the x update: 1/2 or (n_r+1)/(2 n_r+1) */
  int32_t b_num, b_den; /* self-weight b of the y update: n_r/(2 n_r+1) or 1/2 */
  float a, a_peer;      /* (float)((double)a_num/a_den), (float)((double)(a_den-a_num)/a_den) */
  float b, b_peer;      /* same for b */
} ceca_round_t;

/* Per-agent stochastic gradient e_i = grad F(z_i; xi_i), evaluated once per agent per
 * iteration at z_i (Algorithm 1).  With s = grad_scale (0 selects the minibatch mean, s = 1/B):
 *   LSQ         e_i = s sum_j (a_ij . z_i - t_ij) a_ij + noise_std * eps_i
 *               (s = 1, B = N, batch_idx = 0..N-1 and noise_std = sigma_n give the least-squares
 *               experiment of Sec. 5: full gradient of 1/2 ||A_i x - b_i||^2 plus N(0, sigma_n^2 I))
 *   LOGISTIC    e_i = -s sum_j t_ij sigma(-t_ij a_ij . z_i) a_ij + noise_std * eps_i,  labels t_ij = +-1
 *   QUAD_CENTER e_i = z_i - c_i + noise_std * eps_i
 *   GRADIENT    e_i = row i of c: the caller evaluated the stochastic gradient of any loss at z_i (the x
 *               row when ceca_schedule's exchange_y is 0, the y row when it is 1) and passes it in;
 *               N, B, seed, k, noise_std, grad_scale, A, t are ignored
 * eps_i ~ N(0, I) comes from the counter-based generator below, keyed by (seed, k, agent, column).
 *
 * Noise generator (uint32 arithmetic, wrapping; agent and column 0-based):
 *   mix(h):   h ^= h >> 16; h *= 0x7feb352d; h ^= h >> 15; h *= 0x846ca68b; h ^= h >> 16
 *   keys:     k0 = mix(mix(seed + 0x9e3779b9 * k) ^ agent);  k1 = mix(k0 + 0x85ebca6b)
 *   word(c):  h = c ^ k0; h ^= h >> 16; h *= 0x7feb352d; h ^= h >> 15; h += k1; h *= 0x846ca68b; h ^= h >> 16
 *   pair q = column >> 1:  u1 = ((word(2q) >> 8) + 1) / 2^24 in (0, 1],  u2 = (word(2q+1) >> 8) / 2^24 in [0, 1)
 *   Box-Muller: rad = sqrt(-2 ln u1);  eps[2q] = rad cos(2 pi u2),  eps[2q+1] = rad sin(2 pi u2)
 * The integer part is exact; the device evaluates log / sqrt / sin / cos with its fp32 hardware units
 * (absolute error of eps below 2e-5). */
typedef struct {
  int32_t kind;         /* CECA_LOSS_* */
  int32_t N;            /* samples per agent (minibatch losses) */
  int32_t B;            /* minibatch rows per agent per iteration, 1..64 */
  uint32_t seed;        /* noise seed */
  uint32_t k;           /* iteration number fed to the noise counter */
  float noise_std;      /* scale of the additive Gaussian gradient noise, 0 = none */
  float grad_scale;     /* minibatch losses: factor s on the summed gradient; 0 = 1/B */
  const float* A;       /* device, n*N rows of lda floats: row i*N + j is sample j of agent i */
  int64_t lda;          /* >= d */
  const float* t;       /* device, n*N floats: targets (LSQ) or labels +-1 (LOGISTIC) */
  const float* c;       /* device, n rows of ldc floats: centres (QUAD_CENTER) or gradients (GRADIENT) */
  int64_t ldc;          /* >= d */
} ceca_loss_t;

/* tau = ceil(log2 n), computed as the bit length of n-1 (Sec. 3.1); n = 1 gives 0; n < 1 gives CECA_EINVAL. */
int32_t ceca_tau(int32_t n);

/* Schedule of round r (host only, integer exact).  `out` (host, may be NULL) receives the round;
 * `peer` (host, caller-owned, n entries, may be NULL) receives the 0-based receive-from map:
 * row i combines its own rows with the message of row peer[i] (Eqs. (5)-(7)).
 * Errors: CECA_EINVAL for n < 2, r outside [0, tau), port not 1 or 2; CECA_EODD1P. */
int32_t ceca_schedule(int32_t n, int32_t r, int32_t port, ceca_round_t* out, int32_t* peer);

/* One gradient-free CECA round (Sec. 3.1 / 3.2 "Main recursions" with I = x, J = y):
 *   x_i+ = a x_i + (1-a) z_peer(i),   y_i+ = b y_i + (1-b) z_peer(i),   z = x or y by delta_r.
 * Every kernel of the library evaluates such a combination as t = a x (rounded to fp32), then fma(a_peer, z, t)
 * with the float weights of ceca_round_t, so single rounds, fused rounds and fused steps agree bit for bit.
 * S_in, S_out: device, 2n rows of ld floats (d used); S_out is either disjoint from S_in or S_in
 * itself.  In place, a thread reads every row of a pair (port 1) or of a whole shift cycle (port 2)
 * before it writes it; out of place, two-port rounds are cut into one-row stretches that sweep the
 * state band by band, which is the faster form on MI355X.  Partial overlap is CECA_EINVAL.
 * In place with two ports, one workgroup per 1024 columns walks a whole cycle of up to n rows in turn:
 * fine with many columns (within 10-20 % of out of place from d = 2^17), but with few columns and many
 * agents it is latency-bound (n = 4097, d = 1024: 1 ms against 15 us) -- alternate two buffers there.
 * n = 1 copies (r must be 0).
 * In round 0 (b = 0) the y rows of S_in are not read. */
int32_t ceca_gossip_round(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld,
                          int32_t r, int32_t port, void* hip_stream);

/* `rounds` consecutive gradient-free CECA rounds r = 0, 1, ..., taken cyclically (round t uses
 * r = t mod tau), in one pass over the state: rounds = tau leaves every x_i at the global mean
 * (Sec. 3.1 problem statement; matrix-consensus lemma, first identity), rounds = tau + 1 also every
 * y_i (Lemma 4.2) -- the global averaging that Theorem 4.3 asks for before the first iteration.
 * The result has the same bits as `rounds` calls of ceca_gossip_round.  Because the sequence starts
 * at round 0, the y rows of S_in are never read.  S_out may be S_in or disjoint from it.
 * Up to 4096 agents run through kernels that move 12 bytes per agent-parameter for as many whole cycles
 * as fit in 64 rounds each (longer runs take several such kernels, in place on S_out after the first).
 * More agents, a single round, and -- with one port or at least 2^20 columns -- fewer than 3-5 rounds on
 * more than about 1150 agents (where the fused pass costs more than that many streaming rounds) take one
 * launch per round instead (in place on S_out after the first).  With more than about 100 agents a row of
 * a workgroup's tile is 64-256 bytes wide: an ld that is a multiple of 32 floats keeps those rows on
 * 128-byte lines (up to 1.7x faster than an odd ld at n = 130-400). */
int32_t ceca_gossip_rounds(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld,
                           int32_t rounds, int32_t port, void* hip_stream);

/* Exact averaging (the problem CECA solves, Sec. 3.1): X_out row i = (1/n) sum_j X_in row j for every i,
 * reached by tau = ceil(log2 n) CECA rounds carried through registers, with the arithmetic of
 * ceca_gossip_rounds(rounds = tau) -- the x rows have the same bits -- but the auxiliary y is neither
 * read nor written: 8 bytes per agent-parameter.  X_in, X_out: device, n rows of ld floats; X_out may be
 * X_in or disjoint from it.  port = 1 needs even n.  Limits: n <= 4096 (CECA_EINVAL beyond; use
 * ceca_gossip_rounds on a full state there). */
int32_t ceca_average(const float* X_in, float* X_out, int32_t n, int64_t d, int64_t ld, int32_t port,
                     void* hip_stream);

/* Bytes of device workspace dsgd_ceca_step needs for this problem (0 for QUAD_CENTER); < 0 on error. */
int64_t dsgd_ceca_workspace_bytes(int32_t n, int64_t d, const ceca_loss_t* loss);

/* One DSGD-CECA iteration (Algorithm 1, Eqs. (8), (9)) with the gradient fused in:
 *   e_i = grad at z_i,  v_i = z_i - lr e_i,
 *   x_i+ = a (x_i - lr e_i) + (1-a) v_peer(i),   y_i+ = b (y_i - lr e_i) + (1-b) v_peer(i).
 * batch_idx: device, n*B int32 in [0, N), row i = agent i's sampled rows (NULL for QUAD_CENTER);
 *   values outside [0, N) are clamped into it rather than followed.
 * workspace: device, 256-byte aligned, at least dsgd_ceca_workspace_bytes() (may be NULL when that is 0);
 * its contents are scratch.  Aliasing rules as ceca_gossip_round.  n = 1: plain SGD on x, y+ = x+. */
int32_t dsgd_ceca_step(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld,
                       const ceca_loss_t* loss, const int32_t* batch_idx, float lr,
                       int32_t r, int32_t port, void* workspace, int64_t workspace_bytes,
                       void* hip_stream);

/* `steps` consecutive DSGD-CECA iterations with the quadratic-centre loss in one pass over the state.
 * Iteration t (t = 0 .. steps-1) uses round (r0 + t) mod tau and the noise counter loss->k + t, at the
 * one step size lr; the result has the same bits as `steps` calls of dsgd_ceca_step.  Only
 * CECA_LOSS_QUAD_CENTER is taken (CECA_EINVAL otherwise): its gradient is elementwise, so columns stay
 * independent across whole iterations and a workgroup can carry a column tile of x, y and c through all
 * of them in registers -- 20 bytes per agent-parameter for the whole call instead of per iteration.
 * S_out may be S_in or disjoint from it.  Up to 4096 agents run as one kernel per 64 iterations (in place
 * on S_out after the first).  More agents, and -- with one port or at least 2^20 columns -- runs too short
 * to repay a narrow tile (fewer than 3, 8 or 14 iterations on more than 640, 1280 or 2560 agents), take one
 * dsgd_ceca_step per iteration (likewise). */
int32_t dsgd_ceca_steps(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld,
                        const ceca_loss_t* loss, float lr, int32_t r0, int32_t steps, int32_t port,
                        void* hip_stream);

/* Bytes of device workspace dsgd_ceca_run needs for this problem; < 0 on error. */
int64_t dsgd_ceca_run_workspace_bytes(int32_t n, int64_t d, const ceca_loss_t* loss);

/* `iters` consecutive DSGD-CECA iterations with a minibatch loss (LSQ or LOGISTIC) in one call.
 * Iteration t (t = 0 .. iters-1) uses round (r0 + t) mod tau, the noise counter loss->k + t, the batch
 * rows batch_idx + t * n * B (device, iters * n * B int32) and the one step size lr; the result has the
 * same bits as `iters` calls of dsgd_ceca_step.  Where a workgroup can take an agent's whole rows
 * (16-byte aligned layouts with d <= 16384 and either n >= 128 with d > 1024 or a batch that fits a
 * register tile: B <= 32 at d <= 1024, 16 at 4096, 8 at 8192, 4 at 16384; any other layout with
 * d <= 1024) each iteration after the first is ONE kernel: the workgroup that takes agent i's gradient
 * first finishes the iteration before for that agent (Eqs. (8), (9)) from its own and its peer's
 * message.  Other shapes take the gradient in two passes (margins, then half step); there the margins
 * kernel finishes the iteration before, TWO kernels per iteration instead of three, with the state
 * alternating between S_out and a copy in the workspace (used when ld <= d rounded up to a multiple of
 * 64; beyond that, and when S_in and S_out differ in 16-byte alignment, the call loops over
 * dsgd_ceca_step).
 * S_out may be S_in or disjoint from it; when disjoint, S_in is left unchanged.
 * workspace: device, 256-byte aligned, at least dsgd_ceca_run_workspace_bytes(); contents are scratch. */
int32_t dsgd_ceca_run(const float* S_in, float* S_out, int32_t n, int64_t d, int64_t ld,
                      const ceca_loss_t* loss, const int32_t* batch_idx, float lr, int32_t r0,
                      int32_t iters, int32_t port, void* workspace, int64_t workspace_bytes,
                      void* hip_stream);

/* Bytes of device workspace consensus_error needs; < 0 on error. */
int64_t consensus_error_workspace_bytes(int32_t n, int64_t d);

/* Consensus observables of X (device, n rows of ld floats), accumulated in fp64:
 *   out[0] = ||X - 1 xbar^T||_F^2      (consensus distance of the descent lemma, App. B.3)
 *   out[1] = sum_i ||x_i - xbar||      (the residue of Sec. 5 taken about the CURRENT row mean xbar; the paper's
 *                                       residue is about x* = the mean of the initial x_i(0).  The two agree
 *                                       whenever the rounds preserve the mean: gradient-free CECA from
 *                                       y(0) = x(0), and the doubly stochastic comparison topologies.  They
 *                                       differ along a DSGD trajectory, where xbar moves by -lr ebar per
 *                                       iteration, and for graph weights that do not preserve the mean: there
 *                                       out[1] / n is the mean distance to the averaged model, not to x*)
 *   out[2] = max_i ||x_i - xbar||
 *   out[3] = ||xbar||
 *   out[4] = n
 * out: device, 5 doubles.  xbar_or_null: device, d floats, receives the mean when not NULL. */
int32_t consensus_error(const float* X, int32_t n, int64_t d, int64_t ld, double* out,
                        float* xbar_or_null, void* workspace, int64_t workspace_bytes,
                        void* hip_stream);

/* consensus_error for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same kernels, same
 * results.  The partial sums live in a 16 MiB array in the library's own device image (one copy per GPU, held
 * until the process ends); the call allocates and frees nothing.  Problems whose partial sums need more than
 * 16 MiB return CECA_EWORKSPACE with the size in ceca_last_error() -- take consensus_error with a workspace
 * there.  Up to 512 agents every d fits (the single pass caps its partial sums at 12 MiB); with more agents
 * the partial sums grow with n * d (n = 1023 on a 16-byte aligned layout: d up to about 60,000), and where only the two-pass form applies
 * (more than 4095 agents) the fp64 column sums alone take 8 d bytes or more.  The array needs no clearing
 * (every partial a kernel reads was written earlier in the same call), but all calls on one GPU share it: two calls that
 * overlap in time on one GPU -- different streams or different threads -- race and give wrong results;
 * calls on one stream, or on streams the caller orders, are safe.  The device whose array is used is the
 * calling thread's current device, which must be the one X, out and the stream belong to. */
int32_t consensus_error_noalloc(const float* X, int32_t n, int64_t d, int64_t ld, double* out,
                                float* xbar_or_null, void* hip_stream);

/* Consensus observables of both halves of a state S = [x; y] (device, 2n rows of ld floats), each half
 * about its own mean, and the squared norm of the stacked deviation phi that the consensus lemma
 * bounds (App. B.3, definition of phi):
 *   out[0..4]  = the five values of consensus_error for the x rows,
 *   out[5..9]  = the same for the y rows,
 *   out[10]    = ||phi||_F^2 = out[0] + out[5].
 * out: device, 11 doubles.  workspace: as consensus_error (same size; the two halves use it in turn). */
int32_t ceca_state_consensus(const float* S, int32_t n, int64_t d, int64_t ld, double* out,
                             void* workspace, int64_t workspace_bytes, void* hip_stream);

/* ---- Shift-invariant gossip averaging (the comparison topologies of Table 1 and of the consensus
 * comparison in Sec. 5; their definitions are those of the works cited there) ----
 * One round:  x_i+ = w_self x_i + sum_{j < m} w[j] x_{(i - shift[j]) mod n}   on x alone (n rows).
 * Evaluated as t = w_self x (rounded), then t = fma(w[j], z_j, t) for j = 0, 1, .. in that order, x+ = t, so a
 * round with m = 1 has the bits of a CECA round with the same weights. */
#define CECA_MIX_MAX 16
typedef struct {
  int32_t m;                      /* 0 .. CECA_MIX_MAX peers */
  float   w_self;
  int32_t shift[CECA_MIX_MAX];    /* each in [0, n) */
  float   w[CECA_MIX_MAX];
} ceca_mix_t;

enum {
  CECA_TOPO_RING = 0,             /* shifts 1 and n-1, weights 1/3 (n = 2: 1/2, 1/2; n = 1: identity)       */
  CECA_TOPO_STATIC_EXP = 1,       /* shifts 2^0 .. 2^(tau-1), every weight 1/(tau+1)                        */
  CECA_TOPO_ONE_PEER_EXP = 2      /* round k: shift 2^(k mod tau), weights 1/2, 1/2 (CECA when n = 2^tau)   */
};

/* Host: round k of a topology.  w[j] = (float) of the exact weight, w_self = (float)(1 - sum_j w[j])
 * so that the rounded weights still sum to one.  Static topologies ignore k.  Returns CECA_EINVAL
 * for n < 1, k < 0 or an unknown kind. */
int32_t ceca_topology_round(int32_t kind, int32_t n, int32_t k, ceca_mix_t* out);

/* `rounds` mixing rounds in one pass over X (device, n rows of ld floats): round t applies
 * specs[(k0 + t) mod period] (specs: host, `period` entries, at most 64 peers over the period).
 * A workgroup keeps a column tile of every agent in registers and passes rows through LDS, so any number
 * of rounds moves 8 bytes per agent-parameter.  X_out may be X_in or disjoint from it.  Limits: n <= 4096.
 * Asynchronous on the stream; specs is read before the call returns. */
int32_t ceca_mix_rounds(const float* X_in, float* X_out, int32_t n, int64_t d, int64_t ld,
                        const ceca_mix_t* specs, int32_t period, int32_t k0, int32_t rounds,
                        void* hip_stream);

/* Gossip averaging over an arbitrary graph (the non-circulant topologies of Table 1 -- grid, torus,
 * hypercube -- and any graph or weight rule the caller brings; their definitions are not the paper's):
 *   x_i+ = w_self[i] x_i + sum_{j < m} w[i*m + j] x_{nbr[i*m + j]}
 * for `rounds` rounds in one pass over X (8 bytes per agent-parameter); round t uses the tables at index
 * (k0 + t) mod period.  nbr: device, period*n*m int32 (0-based vertices; rows with fewer than m neighbours
 * are padded with any valid vertex at weight 0; values outside [0, n) are clamped into it rather than
 * followed); w: device, period*n*m floats; w_self: device, period*n floats.  The tables must not overlap
 * X_out.  Evaluated as t = w_self x (rounded), then t = fma(w_j, z_j, t) in the order of the table: a circulant
 * graph gives the bits of ceca_mix_rounds.  X_out may be X_in or disjoint from it.  Limits: n <= 4096, 1 <= m <= 64. */
int32_t ceca_graph_rounds(const float* X_in, float* X_out, int32_t n, int64_t d, int64_t ld,
                          const int32_t* nbr, const float* w, const float* w_self, int32_t m,
                          int32_t period, int32_t k0, int32_t rounds, void* hip_stream);

/* Message for the calling thread's most recent error ("" if none); valid until its next failing call. */
const char* ceca_last_error(void);
/* hipError_t value behind the calling thread's most recent CECA_EHIP (0 if none). */
int32_t ceca_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CECA_H */
