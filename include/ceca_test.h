/*
 * ceca_test.h -- test and measurement interface of libceca.so.  NOT part of the product ABI (ceca.h does
 * not include it): launch-shape overrides that let tests reach every kernel variant and let sweeps time
 * them, and elementwise probe kernels that show what the device gives the simplest kernel with a given
 * mix of streaming reads and writes.
 *
 * The overrides belong to the calling thread (thread-local): a call on another thread, whatever its stream,
 * never sees them, and a thread that never calls ceca_set_option always gets the library's own shapes.
 * They change which kernel variant or launch shape runs, never what a call computes beyond the last bits
 * of the fp64 consensus sums (every state-updating kernel is bit-identical across shapes; tested).
 * Workspace sizes that depend on a tile shape (consensus_error_workspace_bytes) follow the overrides in
 * force when they are asked for: set the options first, then ask.
 */
#ifndef CECA_TEST_H
#define CECA_TEST_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Options (value 0 = library default unless stated otherwise):
 *   CECA_OPT_SEGMENT  agents a 2-port chain walks before it starts a new one
 *   CECA_OPT_ROWS     0..32.  Single rounds and steps: state rows whose loads one thread keeps in flight,
 *                     1, 2, 4 or 8 (other values: 4).  Register-tile kernels: most rows of the tile a thread
 *                     holds -- 4..16 for ceca_gossip_rounds / ceca_average, 1..16 for dsgd_ceca_steps, 4..32 for
 *                     ceca_mix_rounds and the workgroup-tile consensus kernel, 1..32 for the wavefront-strip
 *                     consensus kernel (values outside a kernel's range leave that kernel at its default)
 *   CECA_OPT_BAND     column tiles (of 1024 columns) per band of the launch order
 *   CECA_OPT_WG_PER_CU  cap on workgroups resident per compute unit, 2..8
 *   CECA_OPT_ONEPASS  1 (default): minibatch gradients keep the sampled rows in registers and read A once when
 *                     (B, d) fits; 0: always the two-pass margins / half-step kernels
 *   CECA_OPT_AGENTS_PER_WG  agents one workgroup of the looping one-pass gradient kernel takes in turn
 *   CECA_OPT_CONS_SINGLE_PASS  consensus observables: 1 (default) the library's choice; 0 always the two-pass
 *                     kernels; 2 the single pass with workgroup tiles (LDS) where a tile holds n agents;
 *                     3 the single pass with one wavefront per column strip (up to 64 x rows agents)
 *   CECA_OPT_XCD_TILE_ORDER  1 (default): register-tile kernels whose tile rows are narrower than 128 bytes give
 *                     each of the 8 XCDs a contiguous run of tiles; 0: plain order
 *   CECA_OPT_TILE_THREADS  threads per workgroup of the fused rounds, fused iterations and mixing kernels:
 *                     256, 512 or 1024; more threads make the rows of a tile wider.  A tile shape that cannot
 *                     hold n agents is replaced by the library's own
 *   CECA_OPT_GRAPH_STAGE  1 (default): ceca_graph_rounds stages small neighbour tables in LDS; 0: it reads them
 *                     from memory at every look-up
 *   CECA_OPT_CHUNKED_GRADIENT  1 (default): single steps with many agents and long rows take the chunked
 *                     gradient kernel; 0: never (the looping one-pass kernels run instead, and dsgd_ceca_run
 *                     does not fuse iterations)
 *   CECA_OPT_CONS_STRIPS  column strips one wavefront of the wavefront-strip consensus kernel takes in turn,
 *                     0..4096 (raised where the partial sums would outgrow their 12 MiB share of the workspace)
 *   CECA_OPT_LEAN_TILES  fused gossip rounds / exact averaging with 256-thread workgroups: 4, 5 or 6 = the
 *                     register-lean form compiled for that many wavefronts per SIMD, 1 = always the plain form
 *   CECA_OPT_HALF_STEP_RUN  1 (default): dsgd_ceca_run keeps the state in half-step form between fused iterations
 *                     (no message buffers); 0: it keeps full states and two message buffers
 *   CECA_OPT_PROBE_VARIANT  the 3-read / 2-write probe in another shape: 100 * policy (0 streaming loads and stores,
 *                     1 plain loads, 2 plain stores, 3 both plain) + 10 * threads code (1 = 256, 2 = 512,
 *                     4 = 1024 per workgroup) + column groups per thread (1, 2, 4, 8 with 256 threads)
 *   CECA_OPT_PROBE_WAVES  ceca_stream_probe: that many long-lived wavefronts walk the arrays (each thread keeps four
 *                     column groups of every array in flight) instead of one short-lived thread per column group
 * Returns CECA_EINVAL for an unknown option or value. */
enum { CECA_OPT_SEGMENT = 1, CECA_OPT_ROWS = 2, CECA_OPT_BAND = 3, CECA_OPT_WG_PER_CU = 4, CECA_OPT_ONEPASS = 5,
       CECA_OPT_AGENTS_PER_WG = 7, CECA_OPT_CONS_SINGLE_PASS = 8, CECA_OPT_XCD_TILE_ORDER = 9,
       CECA_OPT_TILE_THREADS = 10, CECA_OPT_GRAPH_STAGE = 11, CECA_OPT_CHUNKED_GRADIENT = 12,
       CECA_OPT_CONS_STRIPS = 13, CECA_OPT_PROBE_WAVES = 14, CECA_OPT_LEAN_TILES = 15, CECA_OPT_PROBE_VARIANT = 16, CECA_OPT_HALF_STEP_RUN = 17 };
int32_t ceca_set_option(int32_t option, int32_t value);

/* Every option of the calling thread back to the library default. */
int32_t ceca_reset_options(void);

/* Launch shape the library picks (under the calling thread's overrides) for the state-updating kernel of one
 * ceca_gossip_round (kind = 0), of one dsgd_ceca_step with the quadratic-centre loss (kind = 1) or of one
 * dsgd_ceca_step with a minibatch loss (kind = 2: the combine from stored messages) on a 16-byte aligned
 * state of 2n rows of ld floats, out of place (in_place = 0) or in place: out[0] = state rows a thread keeps
 * in flight, out[1] = column tiles per band of the launch order (0 = one band), out[2] = cap on workgroups
 * per compute unit (0 = none), out[3] = agents per chain stretch, out[4] = stretches per cycle, out[5] =
 * floats per column group (4 or 1).  Nothing is launched.  A benchmark uses it to tell whether a stored
 * hardware-counter profile still describes the kernels it is about to time.  out: host, 6 int32. */
int32_t ceca_describe_step_launch(int32_t n, int64_t d, int64_t ld, int32_t r, int32_t port, int32_t kind,
                                  int32_t in_place, int32_t* out);

/* An elementwise kernel with `reads` streaming reads (1..3: a, then b, then c) and `writes` streaming
 * writes (1..2: o1, then o2) per element, so that a benchmark can report, from the same run, the bandwidth
 * the device gives the simplest kernel with a step's traffic mix: 3 reads + 2 writes for a full round of
 * the fused quadratic-centre step, 2 + 2 for its round 0, 2 + 2 / 1 + 2 for gossip rounds, 1 + 0 is not
 * offered (use reads = 1, writes = 1).  o1, o2 may be a, b.  All pointers device, 16-byte aligned
 * (unused ones may be NULL), count floats (a multiple of 4). */
int32_t ceca_stream_probe(const float* a, const float* b, const float* c, float* o1, float* o2, int64_t count,
                          int32_t reads, int32_t writes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* CECA_TEST_H */
