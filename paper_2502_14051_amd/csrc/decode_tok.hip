// One HSA decode step in one launch for caches with token-major V, and for the logical sequences of
// RocketKV-MT (Algorithm 1 of arXiv 2502.14051 end to end; Section 3.5 for the indexed variant).
// Same structure as the channel-major fused kernel: every workgroup of a (sequence, KV head) unit runs
// Step 2 for itself, keeps the page list in LDS and goes on to Step 3 over its share of the token
// slots.  Used when the picked summary rows are small enough to be read twice per unit; larger ones
// (small pages, many channels) take the score / pick / attention launches.
//
// APPEND also takes in the token generated at this step (Section 3.4 Step 1, last sentence): every
// reader patches its key / value rows in from LDS copies; split 0 of the unit writes them to the cache,
// updates the tail page's summary column and, under an index, records the token's cache position as
// the next entry of the logical sequence.  The lengths (the cache's, and the logical one under an
// index) are bumped by whichever workgroup of the sequence is last to have read the old ones.
#include "attend_tok_core.h"
#include "select_core.h"

namespace rkv {

namespace {
__host__ __device__ constexpr size_t tok_round16(size_t x) { return (x + 15) / 16 * 16; }
constexpr size_t kTokStageBytes = 2 * kHeadDim * sizeof(bf16_t);  // staged new key and value
}  // namespace

// `c`: the cache (pools, its own paging, its lengths).  `lc`: what Step 2 works on, i.e. lengths, page
// size and page capacity of the logical sequence (equal to `c` without an index).
template <int WAVES, bool APPEND, bool INDEXED>
__global__ __launch_bounds__(WAVES* kWave) __attribute__((amdgpu_waves_per_eu(2)))
void hsa_decode_tok_kernel(CacheView c, CacheView lc, SelectArgs sa, AttendArgs aa, TokenRun t, AppendArgs ap,
                           uint32_t* seq_counters) {
  constexpr int NT = WAVES * kWave;
  extern __shared__ __align__(16) unsigned char dsm[];  // [staged k,v][list][selection scratch | merge buffer]
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int unit = blockIdx.x, split = blockIdx.y;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  // q, the new key / value and the lengths: all requested before anything else is done or used (one
  // round trip, through the first kernel arguments fetched; the set-up below runs while they travel)
  uint32_t qv[kMaxGroup];  // one bf16 each, kept in a register of its own (no packing, hence no early use)
  load_q_column(lc, sa, unit, qv);
  int n = lc.seq_lens[b + opaque_zero()];  // a vector load beside the others; not needed until the channels are picked
  int pos0 = 0;  // where the new token goes in the cache
  uint32_t arrivals = 0;
  bf16_t kb = 0, vb = 0;
  if (APPEND) {
    // every thread has read the old lengths (see the header comment for how the workgroup reports that)
    if (INDEXED) pos0 = c.seq_lens[b + opaque_zero()];
    if (tid < kHeadDim) {
      const int64_t src = (int64_t)unit * kHeadDim + tid;
      kb = ap.k_new[src];
      vb = ap.v_new[src];
    }
  }

  bf16_t* s_knew = reinterpret_cast<bf16_t*>(dsm);
  bf16_t* s_vnew = s_knew + kHeadDim;
  int32_t* list = reinterpret_cast<int32_t*>(dsm + kTokStageBytes);
  unsigned char* region = dsm + kTokStageBytes + tok_round16((size_t)sa.row_len * sizeof(int32_t));
  SelectShared<NT>& sh = *reinterpret_cast<SelectShared<NT>*>(region);
  uint32_t* keys = reinterpret_cast<uint32_t*>(region + tok_round16(sizeof(SelectShared<NT>)));
  const int ps = lc.page_size;
  TailPatch tp = {-1, 0, s_knew, s_vnew};
  TokenPatch tokp = {-1, s_knew, s_vnew};
  for (int i = tid; i < sa.row_len; i += NT) list[i] = -1;
  if (APPEND && tid < kHeadDim) {
    s_knew[tid] = kb;
    s_vnew[tid] = vb;
  }
  select_channels<NT>(lc, sa, unit, sh, split == 0, qv);  // ends with a barrier: the staging is visible
  n = __builtin_amdgcn_readfirstlane(n);  // the same in every lane: scalars from here on
  pos0 = __builtin_amdgcn_readfirstlane(pos0);
  bool room = false;
  if (APPEND) {
    const int n0 = n;
    if (!INDEXED) pos0 = n0;
    room = n0 < lc.pages_cap * ps && pos0 < c.pages_cap * c.page_size;
    if (room) {
      tp.page = n0 / ps;
      tp.slot = n0 % ps;
      tokp.j_new = n0;
      n = n0 + 1;
    }
  }
  // the summary column the new key goes into, fetched now (beside the row loads) and stored at the end
  uint32_t old_max = 0, old_min = 0;  // bf16 bits, not looked at before the write-back
  const int64_t sum_off = ((int64_t)unit * kHeadDim + (tid & (kHeadDim - 1))) * lc.pages_cap + (room ? tp.page : 0);
  if (APPEND && room && split == 0 && tid < kHeadDim && tp.slot != 0) {
    old_max = ap.kmax[sum_off];
    old_min = ap.kmin[sum_off];
  }
  select_pages<NT>(lc, sa, unit, n, sh, keys, list, split == 0, tp);
  __syncthreads();  // list complete; the selection scratch is dead and becomes the merge buffer
  auto write_back = [&]() {
    if (!APPEND) return;
    if (tid == 0)  // this workgroup's read of the old lengths, reported where the answer's latency hides under the merges
      arrivals = __hip_atomic_fetch_add(&seq_counters[b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (room && split == 0 && tid < kHeadDim) {
      const int sp = pos0 / c.page_size, ss = pos0 % c.page_size;
      const int64_t pp = phys_page(c, b, sp);
      if (pp >= 0) {
        const int64_t at = pp * c.stride_page + (int64_t)g * c.stride_head + ss * kHeadDim + tid;
        c.k_pool[at] = kb;
        c.v_pool[at] = vb;
      }
      if (INDEXED && tid == 0)
        const_cast<int32_t*>(t.index)[(int64_t)unit * t.index_stride + tokp.j_new] = pos0;
      const float x = bf16_to_f32(kb);
      if (tp.slot == 0 || x > bf16_to_f32((bf16_t)use_late(old_max))) ap.kmax[sum_off] = kb;
      if (tp.slot == 0 || x < bf16_to_f32((bf16_t)use_late(old_min))) ap.kmin[sum_off] = kb;
    }
  };
  attend_tokens_block<WAVES, INDEXED, APPEND>(c, aa, t, unit, split, n, list, reinterpret_cast<float*>(region),
                                             &s_last, tokp, write_back);
  if (APPEND) {
    // the last workgroup of the sequence to have read the old lengths stores the new ones
    if (tid == 0 && arrivals == (uint32_t)c.n_kv_heads * gridDim.y - 1u) {
      if (room) {
        lc.seq_lens[b] = n;
        if (INDEXED) c.seq_lens[b] = pos0 + 1;
      }
      __hip_atomic_store(&seq_counters[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

size_t fused_decode_tok_lds_bytes(const CacheView& lc, int row_len, const AttendPlan& plan) {
  const size_t sel = tok_round16(plan.waves == 8 ? sizeof(SelectShared<512>) : sizeof(SelectShared<256>)) +
                     (size_t)((lc.pages_cap + 7) / 8 * 8) * sizeof(uint32_t);
  const size_t mrg = (size_t)plan.waves * lc.group * (kHeadDim + 2) * sizeof(float);
  return kTokStageBytes + tok_round16((size_t)row_len * sizeof(int32_t)) + (sel > mrg ? sel : mrg);
}

hipError_t launch_hsa_decode_tok_fused(const CacheView& c, const LogicalView* lv, const SelectArgs& sa,
                                       const AppendArgs& ap, bf16_t* out, float* out_lse, void* ws,
                                       const AttendPlan& plan, hipStream_t st) {
  CacheView lc = c;
  if (lv) {
    lc.seq_lens = lv->n_indexed;
    lc.page_size = lv->page_size;
    lc.pages_cap = lv->pages_cap;
  }
  AttendArgs a;
  a.q = sa.q;
  a.pages = nullptr;
  a.row_len = sa.row_len;
  a.out = out;
  a.out_lse = out_lse;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + plan.partial_off);
  a.counters = attend_counters(ws, plan);
  a.n_split = plan.n_split;
  a.chunk = plan.chunk * kAttnPage;
  a.per_wave = plan.per_wave * kAttnPage;
  a.n_csplit = 1;
  TokenRun t;
  t.ps = lc.page_size;
  t.tokens = sa.row_len * t.ps;
  t.index = lv ? lv->token_index : nullptr;
  t.index_stride = lv ? lv->pages_cap * lv->page_size : 0;
  t.n_logical = lv ? lv->n_indexed : nullptr;
  t.logical_pages_cap = lv ? lv->pages_cap : 0;
  uint32_t* seq_counters = decode_seq_counters(ws, plan);
  const size_t smem = fused_decode_tok_lds_bytes(lc, sa.row_len, plan);
  const dim3 grid(c.batch * c.n_kv_heads, plan.n_split);
  const bool append = ap.k_new != nullptr;
#define RKV_LAUNCH_TOK(W, A, I)                                                                              \
  hipLaunchKernelGGL((hsa_decode_tok_kernel<W, A, I>), grid, dim3(W * kWave), smem, st, c, lc, sa, a, t, ap, \
                     seq_counters)
  if (plan.waves == 8) {
    if (append) { if (lv) RKV_LAUNCH_TOK(8, true, true); else RKV_LAUNCH_TOK(8, true, false); }
    else        { if (lv) RKV_LAUNCH_TOK(8, false, true); else RKV_LAUNCH_TOK(8, false, false); }
  } else {
    if (append) { if (lv) RKV_LAUNCH_TOK(4, true, true); else RKV_LAUNCH_TOK(4, true, false); }
    else        { if (lv) RKV_LAUNCH_TOK(4, false, true); else RKV_LAUNCH_TOK(4, false, false); }
  }
#undef RKV_LAUNCH_TOK
  return hipGetLastError();
}

}  // namespace rkv
