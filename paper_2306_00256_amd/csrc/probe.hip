// Measurement aid (see ceca_stream_probe in ceca_test.h): the simplest elementwise kernel with a given
// number of streaming reads and streaming writes per element, so that a benchmark can put the bandwidth
// the real kernels reach next to what the device gives such a kernel in the same run.
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

template <int R, int W>
__global__ __launch_bounds__(kBlock) void stream_probe_kernel(const float* a, const float* b, const float* c,
                                                              float* o1, float* o2, int64_t ngroups) {
  const int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (g >= ngroups) return;
  const vf4 x = ld_stream<vf4>(a + 4 * g);
  vf4 y = x, z = x;
  if constexpr (R >= 2) y = ld_stream<vf4>(b + 4 * g);
  if constexpr (R >= 3) z = ld_stream<vf4>(c + 4 * g);
  const vf4 p = 0.5f * x + 0.5f * (y - 0.1f * (y - z));
  const vf4 q = 0.4f * y + 0.6f * (x - 0.1f * (x - z));
  if constexpr (W >= 1) st_stream<vf4>(o1 + 4 * g, p);
  if constexpr (W >= 2) st_stream<vf4>(o2 + 4 * g, q);
  if constexpr (W == 0) {
    // read-only: the loads must not be optimised away; no finite input produces this value
    if (p.x + q.y + p.z + q.w == __builtin_inff()) st_stream<vf4>(o1 + 4 * g, p);
  }
}

// The same elementwise work as a fixed number of long-lived wavefronts: every thread walks the arrays with
// a stride of the whole grid and keeps U column groups of every array in flight.
template <int R, int W, int U>
__global__ __launch_bounds__(kBlock) void stream_probe_loop_kernel(const float* a, const float* b, const float* c,
                                                                   float* o1, float* o2, int64_t ngroups) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t g0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g0 < ngroups; g0 += U * stride) {
    vf4 x[U], y[U], z[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t g = g0 + u * stride < ngroups ? g0 + u * stride : g0;      // past the end: shadow the first group
      x[u] = ld_stream<vf4>(a + 4 * g);
      y[u] = x[u];
      z[u] = x[u];
      if constexpr (R >= 2) y[u] = ld_stream<vf4>(b + 4 * g);
      if constexpr (R >= 3) z[u] = ld_stream<vf4>(c + 4 * g);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t g = g0 + u * stride;
      if (g >= ngroups) continue;
      const vf4 p = 0.5f * x[u] + 0.5f * (y[u] - 0.1f * (y[u] - z[u]));
      const vf4 q = 0.4f * y[u] + 0.6f * (x[u] - 0.1f * (x[u] - z[u]));
      if constexpr (W >= 1) st_stream<vf4>(o1 + 4 * g, p);
      if constexpr (W >= 2) st_stream<vf4>(o2 + 4 * g, q);
      if constexpr (W == 0) {
        if (p.x + q.y + p.z + q.w == __builtin_inff()) st_stream<vf4>(o1 + 4 * g, p);
      }
    }
  }
}

// Variants of the 3-read / 2-write probe for exploring what the memory system rewards: U consecutive
// column groups per thread (a workgroup then covers U * THREADS * 16 contiguous bytes of every array,
// thread t taking groups t, t + THREADS, ...), THREADS per workgroup, streaming (nontemporal) or plain
// loads and stores.
template <int U, int THREADS, bool NTL, bool NTS>
__global__ __launch_bounds__(THREADS) void stream_probe_variant_kernel(const float* a, const float* b, const float* c,
                                                                       float* o1, float* o2, int64_t ngroups) {
  const int64_t base = (int64_t)blockIdx.x * (U * THREADS) + threadIdx.x;
  vf4 x[U], y[U], z[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t g = base + u * THREADS < ngroups ? base + u * THREADS : 0;
    x[u] = NTL ? ld_stream<vf4>(a + 4 * g) : ld_plain<vf4>(a + 4 * g);
    y[u] = NTL ? ld_stream<vf4>(b + 4 * g) : ld_plain<vf4>(b + 4 * g);
    z[u] = NTL ? ld_stream<vf4>(c + 4 * g) : ld_plain<vf4>(c + 4 * g);
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t g = base + u * THREADS;
    if (g >= ngroups) continue;
    const vf4 p = 0.5f * x[u] + 0.5f * (y[u] - 0.1f * (y[u] - z[u]));
    const vf4 q = 0.4f * y[u] + 0.6f * (x[u] - 0.1f * (x[u] - z[u]));
    if (NTS) { st_stream<vf4>(o1 + 4 * g, p); st_stream<vf4>(o2 + 4 * g, q); }
    else { *reinterpret_cast<vf4*>(o1 + 4 * g) = p; *reinterpret_cast<vf4*>(o2 + 4 * g) = q; }
  }
}

template <int U, int THREADS>
static hipError_t launch_probe_variant(const float* a, const float* b, const float* c, float* o1, float* o2,
                                       int64_t ngroups, int policy, hipStream_t st) {
  const int64_t blocks = (ngroups + (int64_t)U * THREADS - 1) / ((int64_t)U * THREADS);
  if (blocks < 1 || blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  const dim3 grid((unsigned)blocks), block(THREADS);
  switch (policy) {
    case 0: stream_probe_variant_kernel<U, THREADS, true, true><<<grid, block, 0, st>>>(a, b, c, o1, o2, ngroups); break;
    case 1: stream_probe_variant_kernel<U, THREADS, false, true><<<grid, block, 0, st>>>(a, b, c, o1, o2, ngroups); break;
    case 2: stream_probe_variant_kernel<U, THREADS, true, false><<<grid, block, 0, st>>>(a, b, c, o1, o2, ngroups); break;
    default: stream_probe_variant_kernel<U, THREADS, false, false><<<grid, block, 0, st>>>(a, b, c, o1, o2, ngroups); break;
  }
  return hipGetLastError();
}

hipError_t launch_stream_probe(const float* a, const float* b, const float* c, float* o1, float* o2, int64_t ngroups,
                               int reads, int writes, hipStream_t st) {
  const int64_t blocks = (ngroups + kBlock - 1) / kBlock;
  if (blocks < 1 || blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  const dim3 grid((unsigned)blocks), block(kBlock);
  const int variant = g_tuning.probe_variant;       // decimal digits: policy (0..3), threads (1 = 256, 2 = 512, 4 = 1024), groups per thread
  if (variant > 0 && reads == 3 && writes == 2) {
    const int U = variant % 10, T = (variant / 10) % 10, pol = (variant / 100) % 10;
#define CECA_PV(UU, TT, THR) if (U == UU && T == TT) return launch_probe_variant<UU, THR>(a, b, c, o1, o2, ngroups, pol, st);
    CECA_PV(1, 1, 256) CECA_PV(2, 1, 256) CECA_PV(4, 1, 256) CECA_PV(8, 1, 256)
    CECA_PV(1, 2, 512) CECA_PV(2, 2, 512) CECA_PV(4, 2, 512)
    CECA_PV(1, 4, 1024) CECA_PV(2, 4, 1024) CECA_PV(4, 4, 1024)
#undef CECA_PV
    return hipErrorInvalidValue;
  }
  const int waves = g_tuning.probe_waves;
  if (waves > 0) {
    // long-lived wavefronts, in workgroups of one wavefront so that they spread over the SIMDs
    const dim3 lgrid((unsigned)waves), lblock(64);
#define CECA_PROBE_LOOP(R, W) if (reads == R && writes == W) { stream_probe_loop_kernel<R, W, 4><<<lgrid, lblock, 0, st>>>(a, b, c, o1, o2, ngroups); return hipGetLastError(); }
    CECA_PROBE_LOOP(1, 0) CECA_PROBE_LOOP(2, 0) CECA_PROBE_LOOP(3, 0)
    CECA_PROBE_LOOP(1, 1) CECA_PROBE_LOOP(2, 1) CECA_PROBE_LOOP(3, 1)
    CECA_PROBE_LOOP(1, 2) CECA_PROBE_LOOP(2, 2) CECA_PROBE_LOOP(3, 2)
#undef CECA_PROBE_LOOP
    return hipErrorInvalidValue;
  }
#define CECA_PROBE(R, W) if (reads == R && writes == W) { stream_probe_kernel<R, W><<<grid, block, 0, st>>>(a, b, c, o1, o2, ngroups); return hipGetLastError(); }
  CECA_PROBE(1, 0) CECA_PROBE(2, 0) CECA_PROBE(3, 0)
  CECA_PROBE(1, 1) CECA_PROBE(2, 1) CECA_PROBE(3, 1)
  CECA_PROBE(1, 2) CECA_PROBE(2, 2) CECA_PROBE(3, 2)
#undef CECA_PROBE
  return hipErrorInvalidValue;
}

}  // namespace ceca
