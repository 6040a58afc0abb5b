// Measurement aid, not part of the method: a pure read stream shaped like the decode step's
// (one wave per contiguous region, 1 KiB per load instruction, non-temporal 16-byte loads, a few
// KiB in flight per wave), so that the benchmark can put the rate this chip sustains for such a
// stream beside the published peak.
#include "lessdec_wave.h"

namespace lessdec {

constexpr int kProbeDepth = 7;

__global__ __launch_bounds__(512) void probe_stream_kernel(const unsigned char *buf, size_t per_wave, unsigned *sink)
{
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  const unsigned char *p = buf + wave * per_wave;
  const int n = (int)(per_wave / 1024);                      // loads of this wave
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(p), 0, (int)per_wave, 0x00020000);
  u4v ring[kProbeDepth];
#pragma unroll
  for (int j = 0; j < kProbeDepth; ++j) ring[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, j * 1024, 2);
  unsigned acc = 0;
  for (int base = 0; base < n; base += kProbeDepth) {
#pragma unroll
    for (int j = 0; j < kProbeDepth; ++j) {
      acc ^= ring[j].x ^ ring[j].y ^ ring[j].z ^ ring[j].w;  // loads past the region read as zero
      ring[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, lane * 16, (base + j + kProbeDepth) * 1024, 2);
    }
  }
  if (acc == 0x9e3779b9u) sink[wave] = acc;                  // keeps the loads alive; practically never taken
}

}  // namespace lessdec

extern "C" int lessdec_probe_stream_read(const void *buf, size_t bytes, int32_t waves, uint32_t *sink, void *hip_stream)
{
  if (!buf || !sink || waves < 8 || waves % 8 || (reinterpret_cast<uintptr_t>(buf) & 15)) return LESSDEC_EINVAL;
  const size_t per_wave = bytes / (size_t)waves / 1024 * 1024;
  if (per_wave < 1024 || per_wave > (size_t)1 << 30) return LESSDEC_EINVAL;
  lessdec::probe_stream_kernel<<<(unsigned)(waves / 8), 512, 0, (hipStream_t)hip_stream>>>(
      static_cast<const unsigned char *>(buf), per_wave, sink);
  return hipGetLastError() == hipSuccess ? LESSDEC_OK : LESSDEC_EHIP;
}
