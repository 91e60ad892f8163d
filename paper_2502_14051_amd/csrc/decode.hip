// One HSA decode step in one launch (Algorithm 1 of arXiv 2502.14051 end to end): every workgroup
// of a (sequence, KV head) unit first runs Step 2 on its own (the selection is cheap and
// deterministic, so the splits of a unit arrive at the same page list without talking to each other),
// keeps the list in LDS, and goes straight on to Step 3 over its share of the list.  This removes a
// dependent launch (about 2.7 us on MI355X) and the round trip of the list through memory from a step
// whose whole budget is a few tens of microseconds.  The unit index is the fast grid dimension, so the
// splits of a unit land on the same XCD and the second reader of the summary rows hits in L2.
//
// The APPEND variant also takes in the token generated at this step (Section 3.4 Step 1: the
// summaries are updated each time a new key is generated): the first workgroup of each unit writes
// the key row, the value column and the updated summary column for later steps, while every
// workgroup patches the new key / value into what it reads from LDS copies, so nobody depends on
// those writes having landed.  The sequence length is bumped by whichever workgroup of the sequence
// is last to have read the old one (a per-sequence arrival counter in the workspace header).
#include "attend_core.h"
#include "select_core.h"

namespace rkv {

__host__ __device__ constexpr size_t round16(size_t x) { return (x + 15) / 16 * 16; }
constexpr size_t kStageBytes = 2 * kHeadDim * sizeof(bf16_t);  // staged new key and value
constexpr size_t kSeqCounterOff = ROCKETKV_WS_HEADER_BYTES / 2;  // per-sequence arrival counters

// CB: channel blocks of the output a workgroup computes (8: all; 4: the unit's channels are divided
// between two workgroups, see attend_block); blockIdx.y counts (list split, channel share) pairs.
template <int WAVES, bool APPEND, bool STREAM_K, int CB>
__global__ __launch_bounds__(WAVES* kWave) __attribute__((amdgpu_waves_per_eu(2)))
void hsa_decode_kernel(CacheView c, SelectArgs sa, AttendArgs aa, AppendArgs ap, uint32_t* seq_counters) {
  constexpr int NT = WAVES * kWave;
  extern __shared__ __align__(16) unsigned char dsm[];  // [staged k,v][list][selection scratch | merge buffer]
  __shared__ int s_last;
  const int tid = threadIdx.x;
  const int unit = blockIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  RKV_STAMP(0);
  // Everything the selection starts from is requested before anything else is done or used, so that q,
  // the new key / value and the length cost one memory round trip together, and so that the kernel
  // arguments they go through are the first ones fetched (the rest of the set-up below runs while
  // the loads travel).
  uint32_t qv[kMaxGroup];  // one bf16 each, kept in a register of its own (no packing, hence no early use)
  load_q_column(c, sa, unit, qv);
  int n = c.seq_lens[b + opaque_zero()];  // a vector load beside the others; not needed until the channels are picked
  uint32_t arrivals = 0;
  bf16_t kb = 0, vb = 0;
  if (APPEND && tid < kHeadDim) {
    const int64_t src = ((int64_t)b * c.n_kv_heads + g) * kHeadDim + tid;
    kb = ap.k_new[src];
    vb = ap.v_new[src];
  }

  const int split = blockIdx.y / aa.n_csplit, cs = blockIdx.y % aa.n_csplit;
  const bool first = blockIdx.y == 0;  // the workgroup of the unit that writes what is written once
  bf16_t* s_knew = reinterpret_cast<bf16_t*>(dsm);
  bf16_t* s_vnew = s_knew + kHeadDim;
  int32_t* list = reinterpret_cast<int32_t*>(dsm + kStageBytes);
  unsigned char* region = dsm + kStageBytes + round16((size_t)sa.row_len * sizeof(int32_t));
  SelectShared<NT>& sh = *reinterpret_cast<SelectShared<NT>*>(region);
  uint32_t* keys = reinterpret_cast<uint32_t*>(region + round16(sizeof(SelectShared<NT>)));
  TailPatch tp = {-1, 0, s_knew, s_vnew};
  for (int i = tid; i < sa.row_len; i += NT) list[i] = -1;
  if (APPEND && tid < kHeadDim) {
    // Every thread has read the old length.  Behind its K/V stream the workgroup reports that read to
    // the per-sequence counter, and the one that finds every other workgroup of the sequence has
    // reported stores the new length at its very end: no thread anywhere sees the length change
    // under it.
    s_knew[tid] = kb;
    s_vnew[tid] = vb;
  }
  select_channels<NT>(c, sa, unit, sh, first, qv);  // ends with a barrier: the staging is visible
  n = __builtin_amdgcn_readfirstlane(n);  // the same in every lane: a scalar from here on
  RKV_STAMP(1);
  bool room = false;
  if (APPEND) {
    const int n0 = n;
    room = n0 < c.pages_cap * kAttnPage;
    if (room) {
      tp.page = n0 / kAttnPage;
      tp.slot = n0 % kAttnPage;
      n = n0 + 1;
    }
  }
  // the summary column the new key goes into, and where the token's page lives: requested behind the
  // thread's last K/V tiles (see `report`), looked at in the write-back
  uint32_t old_max = 0, old_min = 0;  // bf16 bits
  const auto summary_slot = [&]() {
    return ((int64_t)unit * kHeadDim + (tid & (kHeadDim - 1))) * c.pages_cap + (room ? tp.page : 0);
  };
  int32_t pp_new = -1;
  // what the write-back needs from memory (the page's old bounds, its place in the pools)
  auto request = [&]() {
    if (APPEND && room && first && tid < kHeadDim) {
      pp_new = phys_page_request(c, b, tp.page);
      if (tp.slot != 0) {
        old_max = ap.kmax[summary_slot()];
        old_min = ap.kmin[summary_slot()];
      }
    }
  };
  // One workgroup per compute unit (eight wavefronts, all channels): the request goes out here, while
  // memory is idle, and its 256 scattered lines per unit are long back when the stream starts
  // (0.3 us off the step at the benchmark shape).  With two workgroups per compute unit the other
  // one is streaming at this point and the same move costs 0.5 us; there, and where the registers of
  // the selection are needed (a share of the channels), it goes out later (see below).
  constexpr bool kRequestEarly = CB == 8 && WAVES == 8;
  if (kRequestEarly) request();
  // Launches of more than 256 units (four wavefronts, two workgroups per compute unit) are bound by
  // bandwidth from start to end, and there the 256 lines per unit that hold the old bounds, two useful
  // bytes each, are worth avoiding.  The same bounds are the extremes of the rows the receiving page
  // already holds, at most 15 rows of 256 contiguous bytes: the thread of a channel reads its column
  // of them here, all loads in flight across the selection, and folds them when the selection is
  // done (1-2 us off the step at batch 64-128).  A page without storage keeps to the summary column.
  // (With one workgroup per compute unit the extra instructions in front of the stream cost more
  // than the lines: 26.6 against 26.0 us at the benchmark shape when it was tried.)
  constexpr bool kBoundsFromRows = APPEND && CB == 8 && WAVES == 4;
  constexpr int kOldRows = kAttnPage - 1;
  uint32_t old_row[kBoundsFromRows ? kOldRows : 1];
  bool from_rows = false;
  if (kBoundsFromRows && room && first && tid < kHeadDim) {
    pp_new = phys_page_request(c, b, tp.page);
    if (tp.slot != 0) {
      const int64_t pp = phys_page_resolve(c, pp_new);
      if (pp >= 0) {
        from_rows = true;
        const bf16_t* col = c.k_pool + pp * c.stride_page + (int64_t)g * c.stride_head + tid;
#pragma unroll
        for (int r = 0; r < kOldRows; ++r)  // rows beyond the last one held repeat it: harmless, and no branch
          old_row[r] = col[min(r, tp.slot - 1) * kHeadDim];
      } else {
        old_max = ap.kmax[summary_slot()];
        old_min = ap.kmin[summary_slot()];
      }
    }
  }
  select_pages<NT>(c, sa, unit, n, sh, keys, list, first, tp);
  if (kBoundsFromRows && from_rows) {
    float mx = -INFINITY, mn = INFINITY;
#pragma unroll
    for (int r = 0; r < kOldRows; ++r) {
      const float x = bf16_to_f32((bf16_t)use_late(old_row[r]));
      mx = fmaxf(mx, x);
      mn = fminf(mn, x);
    }
    old_max = __float_as_uint(mx) >> 16;
    old_min = __float_as_uint(mn) >> 16;
  }
  __syncthreads();  // list complete; the selection scratch is dead and becomes the merge buffer
  RKV_STAMP(5);
  // The token generated at this step goes to memory for later steps (the first workgroup of the unit
  // writes the key row, the value column and the updated summary column), and the workgroup reports
  // its read of the old length.  None of this is on the way of the result, so each piece sits where
  // its memory latency hides:
  //   request: the loads above;
  //   report:  the add to the sequence's counter, behind the loads of thread 0's last K/V tiles, so
  //            that its answer travels with them;
  //   store:   the write-back itself.
  // The stores follow the thread's last tile and drain under the merges.  Where the request has not
  // gone out yet, it goes out with the report if the workgroup's registers allow (a share of the
  // channels, CB < 8), otherwise in front of the stream, where its answers arrive with the first tiles.
  auto store = [&]() {
    if (APPEND && room && first && tid < kHeadDim) {
      const int64_t sum_off = summary_slot();
      const int64_t pp = phys_page_resolve(c, pp_new);
      if (pp >= 0) {
        const int64_t base = pp * c.stride_page + (int64_t)g * c.stride_head;
        c.k_pool[base + tp.slot * kHeadDim + tid] = kb;
        c.v_pool[base + tid * kAttnPage + tp.slot] = vb;
      }
      const float x = bf16_to_f32(kb);
      if (tp.slot == 0 || x > bf16_to_f32((bf16_t)use_late(old_max))) ap.kmax[sum_off] = kb;
      if (tp.slot == 0 || x < bf16_to_f32((bf16_t)use_late(old_min))) ap.kmin[sum_off] = kb;
    }
  };
  auto last_round = [&]() {
    if (!APPEND) return;
    if (tid == 0)
      arrivals = __hip_atomic_fetch_add(&seq_counters[b], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (CB < 8) request();
  };
  if (CB == 8 && !kRequestEarly && !kBoundsFromRows) request();
  attend_block<WAVES, 1, STREAM_K, CB>(c, aa, unit, split, cs, n, list, reinterpret_cast<float*>(region), &s_last, tp,
                                       store, last_round);

  RKV_STAMP(12);
  if (APPEND) {
    // the last workgroup of the sequence to have read the old length stores the new one
    if (tid == 0 && arrivals == (uint32_t)c.n_kv_heads * gridDim.y - 1u) {
      if (room) c.seq_lens[b] = n;
      __hip_atomic_store(&seq_counters[b], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

#ifdef RKV_STAMPS
extern "C" int rocketkv_debug_stamps(void* host, size_t bytes, int clear) {
  if (clear) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_stamps)) != hipSuccess) return -1;
    return hipMemset(p, 0, sizeof(unsigned long long) * kStampSlots * 2 * kStampWaves * kStampMarks) == hipSuccess ? 0 : -1;
  }
  return hipMemcpyFromSymbol(host, HIP_SYMBOL(g_stamps), bytes) == hipSuccess ? 0 : -1;
}
#endif

size_t fused_decode_lds_bytes(const CacheView& c, int row_len, const AttendPlan& plan) {
  const size_t sel = round16(plan.waves == 8 ? sizeof(SelectShared<512>) : sizeof(SelectShared<256>)) +
                     (size_t)((c.pages_cap + 7) / 8 * 8) * sizeof(uint32_t);
  const size_t mrg = (size_t)plan.waves * c.group * (kHeadDim / plan.n_csplit + 2) * sizeof(float);
  return kStageBytes + round16((size_t)row_len * sizeof(int32_t)) + (sel > mrg ? sel : mrg);
}

uint32_t* decode_seq_counters(void* ws, const AttendPlan& plan) {
  return reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + plan.counter_off + kSeqCounterOff);
}

hipError_t launch_hsa_decode_fused(const CacheView& c, const SelectArgs& sa, const AppendArgs& ap,
                                   bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                                   hipStream_t st) {
  AttendArgs a;
  a.q = sa.q;
  a.pages = nullptr;
  a.row_len = sa.row_len;
  a.out = out;
  a.out_lse = out_lse;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + plan.partial_off);
  a.counters = attend_counters(ws, plan);
  a.n_split = plan.n_split;
  a.chunk = plan.chunk;
  a.per_wave = plan.per_wave;
  a.n_csplit = plan.n_csplit;
  uint32_t* seq_counters = decode_seq_counters(ws, plan);
  const size_t smem = fused_decode_lds_bytes(c, sa.row_len, plan);
  const dim3 grid(c.batch * c.n_kv_heads, plan.n_split * plan.n_csplit);
  const bool append = ap.k_new != nullptr;
  const bool stream_k = wants_stream_k(c, sa.row_len);
#define RKV_LAUNCH_DECODE(W, A, S, CB) \
  hipLaunchKernelGGL((hsa_decode_kernel<W, A, S, CB>), grid, dim3(W * kWave), smem, st, c, sa, a, ap, seq_counters)
#define RKV_LAUNCH_DECODE_S(W, A) \
  do { if (stream_k) RKV_LAUNCH_DECODE(W, A, true, 8); else RKV_LAUNCH_DECODE(W, A, false, 8); } while (0)
  if (plan.n_csplit == 2) {
    // (eight wavefronts by the plan.  K tiles are read by both workgroups of a pair: plain loads, so that
    // the second reader finds them in L2; with the streaming hint it does not, measured 2.7 us slower.)
    if (append) RKV_LAUNCH_DECODE(8, true, false, 4); else RKV_LAUNCH_DECODE(8, false, false, 4);
  } else if (plan.waves == 8) {
    if (append) RKV_LAUNCH_DECODE_S(8, true); else RKV_LAUNCH_DECODE_S(8, false);
  } else {
    if (append) RKV_LAUNCH_DECODE_S(4, true); else RKV_LAUNCH_DECODE_S(4, false);
  }
#undef RKV_LAUNCH_DECODE_S
#undef RKV_LAUNCH_DECODE
  return hipGetLastError();
}

}  // namespace rkv
