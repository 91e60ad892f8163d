// Stand-alone HSA Step 2 kernel (Algorithm 1 of arXiv 2502.14051: i1, g, P, s1, i2): one 256-thread
// workgroup per (sequence, KV head) runs the workgroup-level selection routine and writes the page
// list to global memory.
#include "select_core.h"

namespace rkv {

constexpr int kSelThreads = 256;

__global__ __launch_bounds__(kSelThreads) void hsa_select_kernel(CacheView c, SelectArgs a) {
  extern __shared__ uint32_t keys[];  // [ceil8(pages_cap)] order keys of the page scores
  __shared__ SelectShared<kSelThreads> sh;
  const int unit = blockIdx.x;
  const int n = c.seq_lens[unit / c.n_kv_heads];
  const TailPatch none = {-1, 0, nullptr, nullptr};
  select_block<kSelThreads>(c, a, unit, n, sh, keys, nullptr, true, none);
}

hipError_t launch_hsa_select(const CacheView& c, const SelectArgs& a, hipStream_t st) {
  const size_t smem = (size_t)((c.pages_cap + 7) / 8 * 8) * sizeof(uint32_t);
  hipLaunchKernelGGL(hsa_select_kernel, dim3(c.batch * c.n_kv_heads), dim3(kSelThreads), smem, st,
                     c, a);
  return hipGetLastError();
}

}  // namespace rkv
