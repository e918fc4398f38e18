// Measurement aid: the rate at which this GPU delivers B rows fetched the way the brick
// kernel fetches them -- rows picked at random from a buffer, each read as 16 lanes x 16
// contiguous bytes per half row, several loads in flight per wavefront.  With a buffer far
// larger than the caches this is the ceiling for inputs whose B rows cannot be reused
// (random brick positions); with a cache-sized buffer it is the ceiling of the L2 path.
#include "../../include/spmm.h"
#include "exec_common.h"

namespace spmm {
namespace {

__device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

constexpr int kInFlight = 8;   // load instructions in flight per wavefront

// every wavefront reads `loads` x 4 rows x 256 bytes; n_rows is a power of two, rows are 512 B
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_gather_rows(
    const char* __restrict__ buf, uint32_t row_mask, int loads, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const uint32_t wid = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < loads; it += kInFlight) {
    float4_t v[kInFlight];
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) {
      // load (it+u) covers half h of rows 4k .. 4k+3 of this wavefront's random sequence
      const uint32_t seq = (uint32_t)(it + u);
      const uint32_t r = mix32(wid * 0x9e3779b9u ^ ((seq >> 1) * 4u + (uint32_t)(lane >> 4))) & row_mask;
      v[u] = *reinterpret_cast<const float4_t*>(buf + (size_t)r * 512 + (seq & 1u) * 256 +
                                                (lane & 15) * 16);
    }
#pragma unroll
    for (int u = 0; u < kInFlight; ++u) acc += v[u];
  }
  // never true for the zero-filled or finite buffers callers pass; keeps the loads alive
  if (acc[0] + acc[1] + acc[2] + acc[3] == 12345.678f) sink[threadIdx.x] = acc[0];
}

}  // namespace
}  // namespace spmm

extern "C" int spmm_calibrate_gather(const float* buf, int64_t n_rows, int64_t loads_per_wave,
                                     int64_t n_waves, float* sink, void* stream) {
  using namespace spmm;
  if (!buf || !sink || n_rows < 1 || (n_rows & (n_rows - 1)) != 0 || n_rows > (int64_t(1) << 31) ||
      loads_per_wave < kInFlight || loads_per_wave % kInFlight != 0 ||
      loads_per_wave > (int64_t(1) << 24) || n_waves < kWavesPerBlock ||
      n_waves % kWavesPerBlock != 0 || n_waves > (int64_t(1) << 24))
    return SPMM_EINVAL;
  hipLaunchKernelGGL(k_gather_rows, dim3((unsigned)(n_waves / kWavesPerBlock)),
                     dim3(64 * kWavesPerBlock), 0, (hipStream_t)stream,
                     reinterpret_cast<const char*>(buf), (uint32_t)(n_rows - 1), (int)loads_per_wave,
                     sink);
  return hipGetLastError() == hipSuccess ? SPMM_OK : SPMM_EHIP;
}
