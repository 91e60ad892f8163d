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

// ---- large summaries: scores by several workgroups per (sequence, KV head), then the top-k ---------
//
// NT threads score NT/4 eight-page runs.  Two shapes are launched:
//   <256, APPEND, false>  small workgroups for the score launch of rocketkv_hsa_select, which has no
//                         workspace for counters and leaves the top-k to hsa_pick_kernel;
//   <1024, APPEND, true>  the decode step: a (sequence, KV head) is covered by one to four workgroups of
//                         a compute unit's worth of threads; the scores go out with device-scope stores,
//                         each workgroup reports to the unit's counter, and the last one to report
//                         picks the top-k right there, a launch boundary and a round trip earlier.
//
// APPEND: the launch also takes in the token generated at this step (Section 3.4 Step 1, last
// sentence).  Every workgroup reads the old length at its start, scores with the new key folded into the tail
// page's bound from an LDS copy (so it does not matter whether the write-back has landed), and reports
// its read; workgroup 0 of each (sequence, KV head) writes the key row, the value row or column and
// the summary column.  Reports go to two levels of counters so that none sees more than a handful of
// arrivals: the workgroups of a (sequence, KV head) meet at its counter, the last of them goes on to
// the sequence's, and the last one there stores the new length: no reader of this launch sees it
// change.  unit_counters ([units]) and seq_counters ([batch]) are zero on entry and on exit.
constexpr int kPickThreads = 1024;

template <int NT, bool PICK>
struct ScoreLds {
  static constexpr size_t kPick = PICK ? sizeof(PickShared<NT>) : 0;
  static constexpr size_t kBytes = sizeof(SelectShared<NT>) > kPick ? sizeof(SelectShared<NT>) : kPick;
};

template <int NT, bool APPEND, bool PICK>
__global__ __launch_bounds__(NT) void hsa_score_kernel(CacheView c, SelectArgs a, AppendArgs ap,
                                                       uint32_t* unit_counters, uint32_t* seq_counters) {
  __shared__ __align__(16) unsigned char lds[ScoreLds<NT, PICK>::kBytes];  // selection state, then the pick's
  __shared__ int s_last;
  __shared__ bf16_t s_knew[kHeadDim];
  SelectShared<NT>& sh = *reinterpret_cast<SelectShared<NT>*>(lds);
  const int tid = threadIdx.x;
  const int unit = blockIdx.y;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  // q, the new key / value and the length: all requested before anything is used (one round trip)
  uint32_t qv[kMaxGroup];  // one bf16 each, kept in a register of its own (no packing, hence no early use)
  load_q_column(c, a, unit, qv);
  int n = 0;
  bf16_t kb = 0, vb = 0;
  n = c.seq_lens[b + opaque_zero()];  // a vector load beside the others; not needed until the channels are picked
  if (APPEND) {
    if (tid < kHeadDim) {
      kb = ap.k_new[(int64_t)unit * kHeadDim + tid];
      if (blockIdx.x == 0) vb = ap.v_new[(int64_t)unit * kHeadDim + tid];
      s_knew[tid] = kb;
    }
  }
  select_channels<NT>(c, a, unit, sh, blockIdx.x == 0, qv);  // its barriers publish s_knew
  n = __builtin_amdgcn_readfirstlane(n);  // the same in every lane: a scalar from here on
  TailPatch tp = {-1, 0, s_knew, nullptr};
  bool room = false;
  if (APPEND) {
    room = n < c.pages_cap * c.page_size;
    if (room) {
      tp.page = n / c.page_size;
      tp.slot = n % c.page_size;
      n += 1;
    }
  }
  // the summary column the new key goes into: fetched beside the row loads, stored at the end
  const bool writer = APPEND && room && blockIdx.x == 0 && tid < kHeadDim;
  const int64_t sum_off = ((int64_t)unit * kHeadDim + (tid & (kHeadDim - 1))) * c.pages_cap + (room ? tp.page : 0);
  bf16_t old_max = 0, old_min = 0;
  if (writer && tp.slot != 0) {
    old_max = ap.kmax[sum_off];
    old_min = ap.kmin[sum_off];
  }
  int P = (n + c.page_size - 1) / c.page_size;
  if (P > c.pages_cap) P = c.pages_cap;
  // the runs of the cache (not just of the sequence: the split must not depend on data) in equal shares
  const int share = ((c.pages_cap + 7) / 8 + gridDim.x - 1) / gridDim.x;  // <= NT / 4 by the launch's grid
  const int o_begin = blockIdx.x * share;
  const int n_runs = min(share, (P + 7) / 8 - o_begin);
  if (n_runs > 0)
    score_chunk<NT, PICK>(c, a, unit, P, sh, o_begin, n_runs, a.out_scores + (int64_t)unit * c.pages_cap, tp);
  if (writer) {
    const int64_t pp = phys_page(c, b, tp.page);
    if (pp >= 0) {
      const int64_t base = pp * c.stride_page + (int64_t)g * c.stride_head;
      c.k_pool[base + tp.slot * kHeadDim + tid] = kb;
      c.v_pool[base + (c.v_token_major ? tp.slot * kHeadDim + tid : tid * c.page_size + tp.slot)] = vb;
    }
    const float x = bf16_to_f32(kb);
    if (tp.slot == 0 || x > bf16_to_f32(old_max)) ap.kmax[sum_off] = kb;
    if (tp.slot == 0 || x < bf16_to_f32(old_min)) ap.kmin[sum_off] = kb;
  }
  if (!APPEND && !PICK) return;
  // (score_chunk ended with a wait for the stores' acknowledgement and a barrier: with PICK, this
  // workgroup's scores are visible device-wide before thread 0 reports)
  if (tid == 0) {
    const bool last = __hip_atomic_fetch_add(&unit_counters[unit], 1u, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT) == gridDim.x - 1u;
    if (last) {
      __hip_atomic_store(&unit_counters[unit], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (APPEND && __hip_atomic_fetch_add(&seq_counters[b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                        (uint32_t)c.n_kv_heads - 1u) {
        if (room) c.seq_lens[b] = n;
        __hip_atomic_store(&seq_counters[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    s_last = last;
  }
  if (!PICK) return;
  __syncthreads();  // also: every thread is done with the selection state in `lds`
  if (!s_last) return;
  PickShared<NT>& ph = *reinterpret_cast<PickShared<NT>*>(lds);
  for (int i = tid; i < 4 * 256; i += NT) (&ph.hist[0][0])[i] = 0;
  __syncthreads();
  SelectArgs pa = a;
  pa.in_scores = a.out_scores;
  pick_from_scores<NT, true>(c, pa, unit, n, ph);
}

// one workgroup per (sequence, KV head) and a whole compute unit's worth of threads for it: the pick is
// short dependent phases of per-score work, so lanes are what shortens it
__global__ __launch_bounds__(kPickThreads) void hsa_pick_kernel(CacheView c, SelectArgs a) {
  __shared__ PickShared<kPickThreads> sh;
  const int unit = blockIdx.x;
  const int n = c.seq_lens[unit / c.n_kv_heads];
  (&sh.hist[0][0])[threadIdx.x] = 0;
  __syncthreads();
  pick_from_scores<kPickThreads>(c, a, unit, n, sh);
}

// Picked summary rows of this size or more per (sequence, KV head) are streamed by several workgroups:
// one workgroup reads them at about 11 GB/s, i.e. 128 KiB already costs it some 12 us.
constexpr int64_t kSplitSummaryBytes = 128 * 1024;

bool select_wants_split(const CacheView& c, int k1) {
  return c.pages_cap > kSingleSelectPages ||
         (int64_t)k1 * c.pages_cap * (int64_t)sizeof(bf16_t) >= kSplitSummaryBytes;
}

hipError_t launch_hsa_select(const CacheView& c, const SelectArgs& a, hipStream_t st) {
  const size_t smem = (size_t)((c.pages_cap + 7) / 8 * 8) * sizeof(uint32_t);
  const int units = c.batch * c.n_kv_heads;
  if (a.out_scores && select_wants_split(c, a.k1)) {
    const AppendArgs none = {nullptr, nullptr, nullptr, nullptr};
    return launch_hsa_select_split(c, a, none, nullptr, nullptr, st);
  }
  hipLaunchKernelGGL(hsa_select_kernel, dim3(units), dim3(kSelThreads), smem, st, c, a);
  return hipGetLastError();
}

hipError_t launch_hsa_select_split(const CacheView& c, const SelectArgs& a, const AppendArgs& ap,
                                   uint32_t* unit_counters, uint32_t* seq_counters, hipStream_t st) {
  const int units = c.batch * c.n_kv_heads;
  const int runs = (c.pages_cap + 7) / 8;
  if (unit_counters) {
    // with counters to meet at: scores and top-k in one launch
    const dim3 grid((runs + kPickThreads / 4 - 1) / (kPickThreads / 4), units);
    if (ap.k_new)
      hipLaunchKernelGGL((hsa_score_kernel<kPickThreads, true, true>), grid, dim3(kPickThreads), 0, st, c, a, ap,
                         unit_counters, seq_counters);
    else
      hipLaunchKernelGGL((hsa_score_kernel<kPickThreads, false, true>), grid, dim3(kPickThreads), 0, st, c, a, ap,
                         unit_counters, seq_counters);
    return hipGetLastError();
  }
  const dim3 grid((runs + kSelThreads / 4 - 1) / (kSelThreads / 4), units);
  hipLaunchKernelGGL((hsa_score_kernel<kSelThreads, false, false>), grid, dim3(kSelThreads), 0, st, c, a, ap,
                     unit_counters, seq_counters);
  SelectArgs b = a;
  b.in_scores = a.out_scores;
  b.out_channels = nullptr;  // written by the score launch
  hipLaunchKernelGGL(hsa_pick_kernel, dim3(units), dim3(kPickThreads), 0, st, c, b);
  return hipGetLastError();
}

}  // namespace rkv
