// Measurement aid (see ceca_stream_probe in ceca.h): the simplest kernel with the traffic mix of the
// fused quadratic-centre step -- three streaming reads and two streaming writes per element -- so that
// a benchmark can put the bandwidth the real kernels reach next to what the device gives such a kernel.
#include <hip/hip_runtime.h>

#include "ceca.h"
#include "device_util.h"
#include "launch.h"

namespace ceca {

__global__ __launch_bounds__(kBlock) void stream_probe_kernel(const float* a, const float* b, const float* c,
                                                              float* o1, float* o2, int64_t ngroups) {
  const int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (g >= ngroups) return;
  const vf4 x = ld_stream<vf4>(a + 4 * g), y = ld_stream<vf4>(b + 4 * g), z = ld_stream<vf4>(c + 4 * g);
  st_stream<vf4>(o1 + 4 * g, 0.5f * x + 0.5f * (y - 0.1f * (y - z)));
  st_stream<vf4>(o2 + 4 * g, 0.4f * y + 0.6f * (x - 0.1f * (x - z)));
}

hipError_t launch_stream_probe(const float* a, const float* b, const float* c, float* o1, float* o2, int64_t ngroups,
                               hipStream_t st) {
  const int64_t blocks = (ngroups + kBlock - 1) / kBlock;
  if (blocks < 1 || blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  stream_probe_kernel<<<dim3((unsigned)blocks), dim3(kBlock), 0, st>>>(a, b, c, o1, o2, ngroups);
  return hipGetLastError();
}

}  // namespace ceca
