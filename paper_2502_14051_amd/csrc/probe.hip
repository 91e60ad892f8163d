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

// The K and V tiles of a page list, read with the attention kernels' own work split and load pattern
// (a wavefront takes page pairs of its share of the list; per page four 16-byte loads per lane for the
// K tile and eight 8-byte loads for the V tile, streaming hint) and nothing else: no logits, no
// softmax, no merge.  What a launch of this takes is the floor under Step 3 on this GPU for that list.
template <int WAVES>
__global__ __launch_bounds__(WAVES* kWave)
void gather_read_kernel(CacheView c, const int32_t* __restrict__ pages, int row_len, int chunk, int per_wave,
                        uint32_t* __restrict__ sink) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int unit = blockIdx.x, split = blockIdx.y;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int e_begin = split * chunk, e_end = min(e_begin + chunk, row_len);
  const int wb = e_begin + wave * per_wave, we = min(wb + per_wave, e_end);
  const bf16_t* k_lane = c.k_pool + (int64_t)g * c.stride_head + hn * kHeadDim + kg * 8;
  const bf16_t* v_lane = c.v_pool + (int64_t)g * c.stride_head + hn * kAttnPage + kg * 4;
  uint32_t acc = 0;
  for (int base = wb; base < we; base += kWave) {
    // the page ids of up to 64 entries with one load, as the attention kernels do; lane i holds entry base + i
    int my_id = -1;
    if (base + lane < we) my_id = pages[(int64_t)unit * row_len + base + lane];
    if (my_id >= c.pages_cap) my_id = -1;
    const int64_t my_pp = my_id >= 0 ? phys_page(c, b, my_id) : -1;
    const int64_t my_off = (my_pp >= 0 ? my_pp : 0) * c.stride_page;
    const int cnt = min(kWave, we - base);
    // pages a wavefront requests before it looks at any of them: a pair, as in the attention kernels.
    // (With four, i.e. with everything a wavefront owns at the benchmark shape in flight at once, the
    // launch takes the same time, 13.7 against 13.8 us: the gather is not short of requests in flight.)
    constexpr int kDepth = 2;
    for (int i = 0; i < cnt; i += kDepth) {
      u32x4 kf[kDepth][4];
      u32x2 vf[kDepth][8];
      bool present[kDepth];  // an absent entry reads page 0, as in the attention kernels, and is left out of the checksum
#pragma unroll
      for (int x = 0; x < kDepth; ++x) {
        const int e = (i + x) & (kWave - 1);
        present[x] = i + x < cnt && __builtin_amdgcn_readlane((int)(my_pp >> 32), e) >= 0;
        const int64_t off = ((int64_t)__builtin_amdgcn_readlane((int)(my_off >> 32), e) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)(my_off & 0xffffffff), e);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          kf[x][j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(k_lane + off + j * 32));
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
          vf[x][cb] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(v_lane + off + cb * 16 * kAttnPage));
      }
#pragma unroll
      for (int x = 0; x < kDepth; ++x) {
        uint32_t t = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) t ^= kf[x][j].x ^ kf[x][j].y ^ kf[x][j].z ^ kf[x][j].w;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) t ^= vf[x][cb].x ^ vf[x][cb].y;
        acc ^= present[x] ? t : 0u;
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
  if (lane == 0) sink[((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * WAVES + wave] = acc;
}

// geometry of the list split: that of the attention launch over the same list without the channel shares
static AttendPlan gather_plan(const CacheView& c, int row_len) {
  AttendPlan p = plan_attend(c, row_len, true);
  if (p.n_csplit > 1) {  // the probe reads whole tiles: fold the channel shares back into one workgroup per list share
    p.n_csplit = 1;
  }
  return p;
}

size_t probe_gather_sink_words(const CacheView& c, int row_len) {
  const AttendPlan p = gather_plan(c, row_len);
  return (size_t)c.batch * c.n_kv_heads * p.n_split * p.waves;
}

hipError_t launch_stream_gather(const CacheView& c, const int32_t* pages, int row_len, uint32_t* sink, hipStream_t st) {
  const AttendPlan p = gather_plan(c, row_len);
  const dim3 grid(c.batch * c.n_kv_heads, p.n_split);
  if (p.waves == 8)
    hipLaunchKernelGGL(gather_read_kernel<8>, grid, dim3(8 * kWave), 0, st, c, pages, row_len, p.chunk, p.per_wave, sink);
  else
    hipLaunchKernelGGL(gather_read_kernel<4>, grid, dim3(4 * kWave), 0, st, c, pages, row_len, p.chunk, p.per_wave, sink);
  return hipGetLastError();
}

int probe_read_workgroups() { return 256 * 16; }

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(probe_read_workgroups()), dim3(kProbeThreads), 0, st,
                     static_cast<const u32x4*>(src), (int64_t)(bytes / sizeof(u32x4)), sink);
  return hipGetLastError();
}

}  // namespace rkv
