// Stand-alone HSA Step 2 kernels (Algorithm 1 of arXiv 2502.14051: i1, g, P, s1, i2).  Small
// summaries: one 256-thread workgroup per (sequence, KV head) runs the whole workgroup-level selection
// routine and writes the page list to global memory.  Large ones (small pages and many channels, the
// operating points Section 3.6 derives, where Step 2 moves as many bytes as Step 3): the page scores
// are formed by several workgroups per (sequence, KV head), each on a slice of the pages, and a
// second launch picks the top pages from the scores.
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

constexpr int kScoreRuns = 64;  // eight-page runs per workgroup of the split score launch

__global__ __launch_bounds__(kSelThreads) void hsa_score_kernel(CacheView c, SelectArgs a) {
  __shared__ SelectShared<kSelThreads> sh;
  const int unit = blockIdx.y;
  const int n = c.seq_lens[unit / c.n_kv_heads];  // not needed until the channels are picked
  select_channels<kSelThreads>(c, a, unit, sh, blockIdx.x == 0);
  int P = (n + c.page_size - 1) / c.page_size;
  if (P > c.pages_cap) P = c.pages_cap;
  const int o_begin = blockIdx.x * kScoreRuns;
  const int n_runs = min(kScoreRuns, (P + 7) / 8 - o_begin);
  if (n_runs > 0) score_chunk<kSelThreads>(c, a, unit, P, sh, o_begin, n_runs, a.out_scores + (int64_t)unit * c.pages_cap);
}

// one workgroup per (sequence, KV head) and a whole compute unit's worth of threads for it: the pick is
// short dependent phases of per-score work, so lanes are what shortens it
constexpr int kPickThreads = 1024;
__global__ __launch_bounds__(kPickThreads) void hsa_pick_kernel(CacheView c, SelectArgs a) {
  extern __shared__ uint32_t keys[];
  __shared__ PickShared<kPickThreads> sh;
  const int unit = blockIdx.x;
  const int n = c.seq_lens[unit / c.n_kv_heads];
  (&sh.hist[0][0])[threadIdx.x] = 0;
  __syncthreads();
  pick_from_scores<kPickThreads>(c, a, unit, n, sh, keys);
}

bool select_wants_split(const CacheView& c, int k1) {
  return (int64_t)k1 * c.pages_cap * (int64_t)sizeof(bf16_t) >= 128 * 1024;
}

hipError_t launch_hsa_select(const CacheView& c, const SelectArgs& a, hipStream_t st) {
  const size_t smem = (size_t)((c.pages_cap + 7) / 8 * 8) * sizeof(uint32_t);
  const int units = c.batch * c.n_kv_heads;
  if (a.out_scores && select_wants_split(c, a.k1)) {
    const int chunks = ((c.pages_cap + 7) / 8 + kScoreRuns - 1) / kScoreRuns;
    hipLaunchKernelGGL(hsa_score_kernel, dim3(chunks, units), dim3(kSelThreads), 0, st, c, a);
    SelectArgs b = a;
    b.in_scores = a.out_scores;
    b.out_channels = nullptr;  // written by the score launch
    b.zero_counters = nullptr;
    hipLaunchKernelGGL(hsa_pick_kernel, dim3(units), dim3(kPickThreads), smem, st, c, b);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(hsa_select_kernel, dim3(units), dim3(kSelThreads), smem, st, c, a);
  return hipGetLastError();
}

}  // namespace rkv
