// Measurement aid: a plain 128-bit streaming read of a device buffer.  It gives the
// HBM read rate this GPU reaches with nothing but loads, the practical ceiling the
// decode-attention rate is reported against next to the published peak.
#include <hip/hip_runtime.h>

#include "../../include/cocktail.h"
#include "common.h"

namespace cocktail {

constexpr int kProbeUnroll = 8;  // 16-byte loads in flight per lane

__global__ void __launch_bounds__(64) stream_read_kernel(const u32x4* __restrict__ in, size_t vec_per_wave,
                                                         uint32_t* __restrict__ sink) {
  const u32x4* p = in + (size_t)blockIdx.x * vec_per_wave + threadIdx.x;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = 0; i < vec_per_wave; i += 64 * kProbeUnroll) {
    u32x4 v[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) v[u] = __builtin_nontemporal_load(&p[i + u * 64]);   // read-once data
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc ^= v[u];
  }
  // keeps the loads alive; the store itself almost never happens
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;
}

}  // namespace cocktail

extern "C" int cocktail_stream_read_probe(const void* buf, size_t bytes, void* sink, size_t* bytes_read,
                                          void* stream) {
  using namespace cocktail;
  if (!buf || !sink || !bytes_read) return fail(COCKTAIL_EINVAL, "stream_read_probe: NULL argument");
  if (reinterpret_cast<uintptr_t>(buf) % 16 != 0 || reinterpret_cast<uintptr_t>(sink) % 4 != 0)
    return fail(COCKTAIL_EALIGN, "stream_read_probe: buf must be 16-byte aligned, sink 4-byte aligned");
  constexpr size_t kWaves = 2048;
  constexpr size_t kQuantum = 64 * kProbeUnroll * 16;  // bytes one wave reads per loop trip
  const size_t per_wave = bytes / kWaves / kQuantum * kQuantum;
  if (per_wave == 0) return fail(COCKTAIL_EINVAL, "stream_read_probe: buffer smaller than %zu bytes", kWaves * kQuantum);
  *bytes_read = per_wave * kWaves;
  hipLaunchKernelGGL(stream_read_kernel, dim3(kWaves), dim3(64), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(buf), per_wave / 16, static_cast<uint32_t*>(sink));
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(COCKTAIL_EHIP, "stream_read_probe: launch failed: %s", hipGetErrorString(e));
  return COCKTAIL_OK;
}
