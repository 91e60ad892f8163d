// Internal declarations shared by the gfx950 kernels and the C-ABI front end.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rocketkv.h"

namespace rkv {

constexpr int kHeadDim = 128;      // channels per head handled by every kernel
constexpr int kWave = 64;          // CDNA wavefront
constexpr int kMaxGroup = 16;      // query heads per KV head that fit one MFMA tile
constexpr int kAttnPage = 16;      // page size of the matrix-core attention path
constexpr int kSingleSelectPages = 8192;  // most pages a one-workgroup selection keeps in LDS

typedef uint16_t bf16_t;           // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// 16-byte load; STREAM marks data that is read once per launch (streaming hint: it does not displace
// what the caches hold for reuse, and large one-pass reads measure about a tenth faster with it)
typedef uint32_t raw_u32x4 __attribute__((ext_vector_type(4)));
template <bool STREAM>
__device__ __forceinline__ uint4 ld16(const void* p) {
  if (STREAM) {
    const raw_u32x4 v = __builtin_nontemporal_load(static_cast<const raw_u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
  }
  return *static_cast<const uint4*>(p);
}

__device__ __forceinline__ float bf16lo_to_f32(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs; NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// Hand-off of data between workgroups of one launch, as used by every last-arriver scheme here:
//   producer: device-scope (write-through) stores; drain_stores() in EVERY storing thread; a workgroup
//             barrier; one thread adds to a device-scope counter.
//   consumer: the workgroup whose add returns the last count reads the data with device-scope loads
//             (issued after a barrier that follows the add, hence after its answer).
// drain_stores() is what orders the stores before the counter: it holds the wavefront until the
// memory system has acknowledged every vector store (and load) it has issued, so once the barrier
// has let the adding thread through, all of the workgroup's data is visible device-wide.  A barrier
// alone does not wait for stores in flight.
__device__ __forceinline__ void drain_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Diagnostic build only (-DRKV_STAMPS, never the shipped library): lane 0 of every wavefront of a few
// workgroups of the fused decode kernel notes the 100 MHz clock at phase boundaries.
#ifdef RKV_STAMPS
constexpr int kStampSlots = 64, kStampWaves = 8, kStampMarks = 16;
static __device__ unsigned long long g_stamps[kStampSlots * 2 * kStampWaves * kStampMarks];
#define RKV_STAMP(k)                                                                                          \
  do {                                                                                                        \
    if (threadIdx.x % 64 == 0 && blockIdx.x % 16 == 3 && blockIdx.x / 16 < rkv::kStampSlots && blockIdx.y < 2) \
      rkv::g_stamps[(((blockIdx.x / 16) * 2 + blockIdx.y) * rkv::kStampWaves + threadIdx.x / 64) *            \
                        rkv::kStampMarks + (k)] = __builtin_amdgcn_s_memrealtime();                          \
  } while (0)
#define RKV_STAMP_VAL(k, v)                                                                                   \
  do {                                                                                                        \
    if (threadIdx.x % 64 == 0 && blockIdx.x % 16 == 3 && blockIdx.x / 16 < rkv::kStampSlots && blockIdx.y < 2) \
      rkv::g_stamps[(((blockIdx.x / 16) * 2 + blockIdx.y) * rkv::kStampWaves + threadIdx.x / 64) *            \
                        rkv::kStampMarks + (k)] = (unsigned long long)(v);                                    \
  } while (0)
#else
#define RKV_STAMP(k) do { } while (0)
#define RKV_STAMP_VAL(k, v) do { } while (0)
#endif

// A zero the compiler cannot see through.  Added to an index whose value is the same for the whole
// workgroup, it keeps the load a vector load issued where the source says, beside the other vector
// loads of a phase (as a scalar load it may be issued, and waited for, only after them).
__device__ __forceinline__ int opaque_zero() {
  int z;
  asm volatile("v_mov_b32 %0, 0" : "=v"(z));
  return z;
}

// A loaded value that is not needed until much later: calling this where the value is first used keeps
// the compiler from deriving anything from it (and hence from waiting for the load) any earlier, so the
// load's latency hides under whatever lies between.
__device__ __forceinline__ uint32_t use_late(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves (four
// shifts inside each row of 16 lanes, then two row broadcasts): six adds and no LDS round trips.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);  // row_shr:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);  // row_shr:2
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);  // row_shr:4
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);  // row_shr:8
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);  // row_bcast:15 -> rows 1,3
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);  // row_bcast:31 -> rows 2,3
  return x;
}

// Minimum / maximum over the 64 lanes of a wavefront with the same lane moves (a lane that has no
// source keeps its own value); every lane gets the result.
__device__ __forceinline__ float wave_min_f32(float x) {
#define RKV_DPP_MIN(ctrl, rows) \
  x = fminf(x, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), ctrl, rows, 0xf, false)))
  RKV_DPP_MIN(0x111, 0xf);
  RKV_DPP_MIN(0x112, 0xf);
  RKV_DPP_MIN(0x114, 0xf);
  RKV_DPP_MIN(0x118, 0xf);
  RKV_DPP_MIN(0x142, 0xa);
  RKV_DPP_MIN(0x143, 0xc);
#undef RKV_DPP_MIN
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), kWave - 1));
}
__device__ __forceinline__ float wave_max_f32(float x) {
#define RKV_DPP_MAX(ctrl, rows) \
  x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), ctrl, rows, 0xf, false)))
  RKV_DPP_MAX(0x111, 0xf);
  RKV_DPP_MAX(0x112, 0xf);
  RKV_DPP_MAX(0x114, 0xf);
  RKV_DPP_MAX(0x118, 0xf);
  RKV_DPP_MAX(0x142, 0xa);
  RKV_DPP_MAX(0x143, 0xc);
#undef RKV_DPP_MAX
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), kWave - 1));
}

// Device view of a cache (copied by value into kernel arguments).
struct CacheView {
  int32_t batch, n_q_heads, n_kv_heads, group;
  int32_t page_size, pages_cap;
  int64_t n_phys_pages, stride_page, stride_head;
  int32_t* seq_lens;
  const int32_t* block_table;
  bf16_t* k_pool;
  bf16_t* v_pool;
  int32_t v_token_major;  // V tile [page_size][128] instead of [128][page_size]
};

// physical page of logical page p of sequence b, or -1 when absent
__device__ __forceinline__ int64_t phys_page(const CacheView& c, int b, int p) {
  int64_t pp = c.block_table ? (int64_t)c.block_table[(int64_t)b * c.pages_cap + p]
                             : (int64_t)b * c.pages_cap + p;
  return (pp >= 0 && pp < c.n_phys_pages) ? pp : -1;
}

// The same lookup in two parts, for a caller that needs the answer much later: phys_page_request
// returns what the block table holds (or the identity mapping) without looking at it, so nothing waits
// for the load; phys_page_resolve turns it into the page or -1.
__device__ __forceinline__ int32_t phys_page_request(const CacheView& c, int b, int p) {
  return c.block_table ? c.block_table[(int64_t)b * c.pages_cap + p] : b * c.pages_cap + p;
}
__device__ __forceinline__ int64_t phys_page_resolve(const CacheView& c, int32_t raw) {
  const int64_t pp = (int32_t)use_late((uint32_t)raw);
  return (pp >= 0 && pp < c.n_phys_pages) ? pp : -1;
}

__host__ __device__ __forceinline__ int pages_to_pick(int n, int ps, int T) {
  int P = (n + ps - 1) / ps;
  if (P == 0) return 0;
  if (T >= n) return P;
  int kp = T / ps;
  if (kp < 1) kp = 1;
  return kp < P ? kp : P;
}

// A token that is being appended in the same launch that attends to it (Section 3.4 Step 1: the
// summaries follow every new key).  Its key / value are not read back from the pools: every consumer
// patches them in from these LDS copies, so it does not matter whether the workgroup that writes them
// to memory has got there yet.  page < 0: nothing is being appended.
struct TailPatch {
  int page;            // logical page that receives the token
  int slot;            // position inside that page
  const bf16_t* knew;  // LDS, [128]
  const bf16_t* vnew;  // LDS, [128]
};

// ---- launchers (defined next to their kernels); all return hipError_t ----
hipError_t launch_page_summaries(const CacheView& c, bf16_t* kmax, bf16_t* kmin, int first_page,
                                 int n_pages, hipStream_t st);

struct SelectArgs {
  const bf16_t* q;
  const bf16_t* kmax;
  const bf16_t* kmin;
  int k1, T, n_recent;
  int32_t* out_pages;     // [units][row_len], may be the workspace list
  int row_len;
  int32_t* out_pages2;    // optional second copy (caller's out_pages) with its own row length
  int row_len2;
  int32_t* out_channels;  // optional
  float* out_scores;      // optional
  const float* in_scores; // set by the launcher when the scores come from a separate launch
};
struct AppendArgs {      // all null: plain decode
  const bf16_t* k_new;   // [B][Hkv][128]
  const bf16_t* v_new;
  bf16_t* kmax;          // writable views of the summaries
  bf16_t* kmin;
};
// One launch when the picked summary rows are small enough for a workgroup per (sequence, KV head);
// otherwise, and only if a.out_scores gives it somewhere to put the scores, a score launch split over
// the pages followed by the top-k launch.
bool select_wants_split(const CacheView& c, int k1);
hipError_t launch_hsa_select(const CacheView& c, const SelectArgs& a, hipStream_t st);

struct AttendPlan {
  int waves;          // wavefronts per workgroup (4 or 8)
  int n_csplit;       // workgroups a unit's output channels are divided between (1 or 2)
  int n_split;        // workgroups a unit's page list is divided between (each of the n_csplit shares)
  int chunk;          // page-list entries per workgroup
  int per_wave;       // page-list entries per wavefront (even)
  size_t partial_off; // workspace offsets (bytes)
  size_t counter_off;
  size_t total_bytes;
};
AttendPlan plan_attend(const CacheView& c, int row_len, bool gather);
hipError_t launch_attend(const CacheView& c, const bf16_t* q, const int32_t* pages, int row_len,
                         bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                         hipStream_t st);
hipError_t launch_zero(void* p, size_t bytes, hipStream_t st);
// The logical sequence of RocketKV-MT (Section 3.5): token j of (sequence, KV head) u sits at
// position token_index[u * pages_cap * page_size + j] of the cache.
struct LogicalView {
  int32_t* token_index;
  int32_t* n_indexed;  // [batch]
  int32_t page_size, pages_cap;
};
// Step 3 over token-major caches of any page size; `row_len` counts list entries (pages), the plan
// comes from plan_attend on the 16-slot entries they add up to.  `lv` (optional): the list addresses
// pages of that logical sequence.
hipError_t launch_attend_tokens(const CacheView& c, const bf16_t* q, const int32_t* pages, int row_len,
                                bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                                const LogicalView* lv, hipStream_t st);
// Step 2 + Step 3 (+ the token append) in one launch for token-major caches; `lv` (optional): over the
// logical sequence of RocketKV-MT.  Usable when fused_decode_tok_lds_bytes() fits kMaxLdsBytes and the
// summaries are not large enough to want the split selection.
size_t fused_decode_tok_lds_bytes(const CacheView& lc, int row_len, const AttendPlan& plan);
hipError_t launch_hsa_decode_tok_fused(const CacheView& c, const LogicalView* lv, const SelectArgs& sa,
                                       const AppendArgs& ap, bf16_t* out, float* out_lse, void* ws,
                                       const AttendPlan& plan, hipStream_t st);
hipError_t launch_page_summaries_indexed(const CacheView& c, const LogicalView& lv, bf16_t* kmax,
                                         bf16_t* kmin, int first_page, int n_pages, hipStream_t st);
hipError_t launch_append_indexed(const CacheView& c, const LogicalView& lv, const bf16_t* k_new,
                                 const bf16_t* v_new, bf16_t* kmax, bf16_t* kmin, hipStream_t st);
// Step 2 + Step 3 in one launch; usable when fused_decode_lds_bytes() fits kMaxLdsBytes
constexpr size_t kMaxLdsBytes = 64 * 1024;
size_t fused_decode_lds_bytes(const CacheView& c, int row_len, const AttendPlan& plan);
// The large-summary path of Step 2 (a.out_scores must be set).  With `unit_counters` ([units]) and
// `seq_counters` ([batch]; both zero on entry and on exit) it is one launch and, given ap.k_new, also
// takes in the generated token; without counters (and without append) a score launch and a top-k
// launch.
hipError_t launch_hsa_select_split(const CacheView& c, const SelectArgs& a, const AppendArgs& ap,
                                   uint32_t* unit_counters, uint32_t* seq_counters, hipStream_t st);
uint32_t* decode_seq_counters(void* ws, const AttendPlan& plan);
hipError_t launch_hsa_decode_fused(const CacheView& c, const SelectArgs& sa, const AppendArgs& ap,
                                   bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                                   hipStream_t st);
uint32_t* attend_counters(void* ws, const AttendPlan& plan);
// measurement aid: one streaming read of a buffer; `sink` holds a word per wavefront launched
int probe_read_workgroups();
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);
// measurement aid: the K/V tiles of a page list read with the attention kernels' work split and load
// pattern, nothing computed; `sink` holds probe_gather_sink_words() words
size_t probe_gather_sink_words(const CacheView& c, int row_len);
hipError_t launch_stream_gather(const CacheView& c, const int32_t* pages, int row_len, uint32_t* sink, hipStream_t st);

hipError_t launch_append(const CacheView& c, const bf16_t* k_new, const bf16_t* v_new, bf16_t* kmax,
                         bf16_t* kmin, hipStream_t st);

struct SnapPlan {
  size_t stats_off, votes_off, pooled_off, kept_off, sel_off, total_bytes;
  int sel_split;  // workgroups per unit in the select of a long prompt (0: one, in a single launch)
  int n_chunks;  // key-axis chunks per (sequence, head group) in the two score passes
  int chunk_pages;
};
SnapPlan plan_snapkv(const CacheView& src, int window, int keep);
// dst == nullptr: filter only (indices to kept_idx, rows of kept_stride entries; counts to n_out)
hipError_t launch_snapkv(const bf16_t* q_obs, const CacheView& src, int window, int pool_kernel,
                         int keep, const CacheView* dst, int32_t* kept_idx, int kept_stride,
                         int32_t* n_out, void* ws, const SnapPlan& plan, hipStream_t st);

}  // namespace rkv
