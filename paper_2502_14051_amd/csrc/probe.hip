// Measurement aid, not a step of the method: a plain streaming read of a device buffer, to put a
// measured HBM read ceiling beside the published 8 TB/s when the decode kernels are priced against
// the bandwidth roofline (the decode step of Algorithm 1 in arXiv 2502.14051 is bandwidth-bound by
// the paper's own accounting, Section 3.4).
#include "common.h"

namespace rkv {

constexpr int kProbeThreads = 256;
constexpr int kProbeInFlight = 8;  // 16-byte loads a thread keeps in flight

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Every workgroup owns one contiguous chunk and each load instruction of a wavefront covers 1 KiB of
// whole cache lines; the loads carry the streaming hint.  (Of the variants tried this one reads
// fastest: 7.0 TB/s, against 6.2 without the hint and 6.5 with the chunks interleaved.)
__global__ __launch_bounds__(kProbeThreads)
void stream_read_kernel(const u32x4* __restrict__ src, int64_t n16, uint32_t* __restrict__ sink) {
  const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const int64_t b0 = blockIdx.x * per;
  const int64_t b1 = b0 + per < n16 ? b0 + per : n16;
  int64_t i = b0 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + (kProbeInFlight - 1) * kProbeThreads < b1; i += kProbeInFlight * kProbeThreads) {
    u32x4 v[kProbeInFlight];
#pragma unroll
    for (int u = 0; u < kProbeInFlight; ++u) v[u] = __builtin_nontemporal_load(src + i + u * kProbeThreads);
#pragma unroll
    for (int u = 0; u < kProbeInFlight; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < b1; i += kProbeThreads) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  // one word per wavefront keeps the loads alive without adding measurable write traffic
  for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
  if ((threadIdx.x & (kWave - 1)) == 0)
    sink[blockIdx.x * (kProbeThreads / kWave) + threadIdx.x / kWave] = acc;
}

int probe_read_workgroups() { return 256 * 16; }

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(probe_read_workgroups()), dim3(kProbeThreads), 0, st,
                     static_cast<const u32x4*>(src), (int64_t)(bytes / sizeof(u32x4)), sink);
  return hipGetLastError();
}

}  // namespace rkv
