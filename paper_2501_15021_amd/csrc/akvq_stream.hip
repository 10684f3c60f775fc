// Measurement aid, not part of the method: a plain streaming read of a device buffer with 128-bit loads, the same
// access shape the cache kernels use (one 16-byte load per lane, fully coalesced, several loads in flight per lane)
// and no arithmetic beyond an exclusive-or.  Its rate is the practical ceiling to hold the cache kernels against,
// beside the published peak.
#include "akvq_device.h"
#include "akvq_kernels.h"

namespace akvq {

namespace {

constexpr int kStreamThreads = 256;
constexpr int kStreamUnroll = 8;                                         // 16-byte loads in flight per lane
constexpr size_t kStreamChunk = (size_t)kStreamThreads * 16 * kStreamUnroll;  // 32 KB per workgroup

// NT: loads carry the non-temporal hint (the form the decode kernels use for the cache stream)
template <bool NT>
__global__ __launch_bounds__(kStreamThreads) void stream_read_kernel(const u32x4 *src, size_t n_vec, uint32_t *sink) {
  const size_t base = (size_t)blockIdx.x * (kStreamThreads * kStreamUnroll) + threadIdx.x;
  u32x4 v[kStreamUnroll];
#pragma unroll
  for (int i = 0; i < kStreamUnroll; ++i) {
    const size_t idx = base + (size_t)i * kStreamThreads;
    const u32x4 *p = src + (idx < n_vec ? idx : n_vec - 1);  // unconditional loads, clamped address
    v[i] = NT ? stream_load(p) : *p;
  }
  u32x4 acc = v[0];
#pragma unroll
  for (int i = 1; i < kStreamUnroll; ++i) acc ^= v[i];
  const uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  // keeps the loads alive; never true for the benchmark's buffers (sink receives the value if it ever is)
  if (r == 0x9E3779B9u && (acc[0] & acc[1] & acc[2]) == 0xFFFFFFFFu) sink[0] = r;
}

}  // namespace

hipError_t launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int non_temporal, hipStream_t stream) {
  const size_t n_vec = bytes / 16;
  const size_t n_wg = (bytes + kStreamChunk - 1) / kStreamChunk;
  if (non_temporal)
    hipLaunchKernelGGL(stream_read_kernel<true>, dim3((unsigned)n_wg), dim3(kStreamThreads), 0, stream,
                       static_cast<const u32x4 *>(src), n_vec, sink);
  else
    hipLaunchKernelGGL(stream_read_kernel<false>, dim3((unsigned)n_wg), dim3(kStreamThreads), 0, stream,
                       static_cast<const u32x4 *>(src), n_vec, sink);
  return hipGetLastError();
}

}  // namespace akvq
