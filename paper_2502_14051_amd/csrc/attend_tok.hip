// Stand-alone Step 3 kernel over token-major caches (see attend_tok_core.h): driven by a page list in
// global memory, or the identity list for the Full-KV baseline; optionally through the index of
// RocketKV-MT.
#include "attend_tok_core.h"

namespace rkv {

template <int WAVES, bool INDEXED>
__global__ __launch_bounds__(WAVES* kWave) __attribute__((amdgpu_waves_per_eu(2)))
void attend_tokens_kernel(CacheView c, AttendArgs a, TokenRun t) {
  extern __shared__ float smem[];  // sO[WAVES][G][128], sM[WAVES][G], sL[WAVES][G]
  __shared__ int s_last;
  const int unit = blockIdx.y, split = blockIdx.x;
  const int b = unit / c.n_kv_heads;
  const int n = INDEXED ? t.n_logical[b] : c.seq_lens[b];
  const int32_t* list = a.pages ? a.pages + (int64_t)unit * a.row_len : nullptr;
  const TokenPatch none = {-1, nullptr, nullptr};
  attend_tokens_block<WAVES, INDEXED>(c, a, t, unit, split, n, list, smem, &s_last, none);
}

hipError_t launch_attend_tokens(const CacheView& c, const bf16_t* q, const int32_t* pages, int row_len,
                                bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                                const LogicalView* lv, hipStream_t st) {
  const int units = c.batch * c.n_kv_heads;
  AttendArgs a;
  a.q = q;
  a.pages = pages;
  a.row_len = row_len;
  a.out = out;
  a.out_lse = out_lse;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + plan.partial_off);
  a.counters = attend_counters(ws, plan);
  a.n_split = plan.n_split;
  a.chunk = plan.chunk * kAttnPage;        // the plan counts 16-token entries
  a.per_wave = plan.per_wave * kAttnPage;  // even number of entries: a multiple of 32 slots
  a.n_csplit = 1;
  TokenRun t;
  t.ps = lv ? lv->page_size : c.page_size;
  t.tokens = row_len * t.ps;
  t.index = lv ? lv->token_index : nullptr;
  t.index_stride = lv ? lv->pages_cap * lv->page_size : 0;
  t.n_logical = lv ? lv->n_indexed : nullptr;
  t.logical_pages_cap = lv ? lv->pages_cap : 0;
  const size_t smem = (size_t)plan.waves * c.group * (kHeadDim + 2) * sizeof(float);
  const dim3 grid(plan.n_split, units);
  if (plan.waves == 8) {
    if (lv)
      hipLaunchKernelGGL((attend_tokens_kernel<8, true>), grid, dim3(8 * kWave), smem, st, c, a, t);
    else
      hipLaunchKernelGGL((attend_tokens_kernel<8, false>), grid, dim3(8 * kWave), smem, st, c, a, t);
  } else {
    if (lv)
      hipLaunchKernelGGL((attend_tokens_kernel<4, true>), grid, dim3(4 * kWave), smem, st, c, a, t);
    else
      hipLaunchKernelGGL((attend_tokens_kernel<4, false>), grid, dim3(4 * kWave), smem, st, c, a, t);
  }
  return hipGetLastError();
}

}  // namespace rkv
