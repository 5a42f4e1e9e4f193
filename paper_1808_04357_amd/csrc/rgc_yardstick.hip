// rgc_yardstick.hip -- what the streaming pass's memory traffic costs by itself.
//
// The compression call's streaming pass (Algorithm 1's accumulate with the momentum correction of
// Section 2.5) reads G, V and u and writes V and u: 20 bytes per element, two fifths of them writes.
// The kernel below does exactly that and nothing else -- no keys, no lists, no histogram -- with the
// same decomposition (one wave per contiguous wave-chunk, 16 bytes per lane and access, consecutive
// calls walking the tensors in opposite directions).  Its time is the yardstick a benchmark holds the
// streaming pass against: the share of the HBM peak that this mix of reads and writes reaches on the
// device at all.  A diagnostic (rgc_diag.h); no product call uses it.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/rgc_diag.h"
#include "rgc_internal.h"

namespace rgc {
namespace {

typedef float yf4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kYardThreads = 256;      // four waves, as in the streaming pass
constexpr uint32_t kYardChunk = 8192;       // elements per wave
constexpr uint32_t kYardInFlight = 2;       // 16-byte accesses per lane and array in flight

__global__ void __launch_bounds__(kYardThreads) yardstick_kernel(const float* __restrict__ g, float* __restrict__ v,
                                                                 float* __restrict__ u, uint64_t n, float m,
                                                                 uint32_t reverse) {
  const uint32_t wg = reverse ? gridDim.x - 1u - blockIdx.x : blockIdx.x;
  const uint64_t wave = static_cast<uint64_t>(wg) * (kYardThreads / 64u) + (threadIdx.x >> 6);
  const uint32_t lane = threadIdx.x & 63u;
  const uint64_t n4 = n / 4u;                                  // whole 16-byte groups
  const uint64_t b = wave * (kYardChunk / 4u);
  uint64_t e = b + kYardChunk / 4u;
  if (e > n4) e = n4;
  const yf4* g4 = reinterpret_cast<const yf4*>(g);
  yf4* v4 = reinterpret_cast<yf4*>(v);
  yf4* u4 = reinterpret_cast<yf4*>(u);
  for (uint64_t i = b + lane; i < e; i += 64u * kYardInFlight) {
    yf4 gg[kYardInFlight], vv[kYardInFlight], uu[kYardInFlight];
#pragma unroll
    for (uint32_t j = 0; j < kYardInFlight; ++j) {
      const uint64_t p = i + 64u * j;
      if (p < e) { gg[j] = g4[p]; vv[j] = v4[p]; uu[j] = u4[p]; }
    }
#pragma unroll
    for (uint32_t j = 0; j < kYardInFlight; ++j) {
      const uint64_t p = i + 64u * j;
      if (p < e) {
        uu[j] = m * uu[j] + gg[j];      // (no contraction: the library is built without fma fusion)
        vv[j] = vv[j] + uu[j];
        u4[p] = uu[j];
        v4[p] = vv[j];
      }
    }
  }
  // the up to three elements behind the last whole group
  if (wg == 0u && threadIdx.x < (n & 3u)) {
    const uint64_t p = n4 * 4u + threadIdx.x;
    const float un = m * u[p] + g[p];
    u[p] = un;
    v[p] = v[p] + un;
  }
}

}  // namespace
}  // namespace rgc

extern "C" int rgc_stream_yardstick(const float* grad, float* residual, float* velocity, int64_t n, float momentum,
                                    int reverse, void* hip_stream) {
  if (!grad || !residual || !velocity || n < 1 || n >= (int64_t(1) << 40)) return RGC_EINVAL;
  if ((reinterpret_cast<uintptr_t>(grad) | reinterpret_cast<uintptr_t>(residual) | reinterpret_cast<uintptr_t>(velocity)) & 15u)
    return RGC_EINVAL;
  const uint64_t per_wg = static_cast<uint64_t>(rgc::kYardChunk) * (rgc::kYardThreads / 64u);
  const uint64_t wgs = (static_cast<uint64_t>(n) + per_wg - 1u) / per_wg;
  if (wgs > 0x7FFFFFFFull) return RGC_EINVAL;
  rgc::yardstick_kernel<<<dim3(static_cast<uint32_t>(wgs)), dim3(rgc::kYardThreads), 0, static_cast<hipStream_t>(hip_stream)>>>(
      grad, residual, velocity, static_cast<uint64_t>(n), momentum, reverse ? 1u : 0u);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return rgc::fail_hip(e, "rgc_stream_yardstick launch");
  return RGC_OK;
}
