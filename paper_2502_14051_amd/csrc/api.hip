// C-ABI front end: argument validation on the host, workspace carving, kernel launches.
// Every exported function validates before it enqueues anything and never synchronises.
#include <math.h>
#include <mutex>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include "common.h"

using namespace rkv;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(ROCKETKV_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
}

// Checks the host-visible part of a cache description.  `need_pools` is false for queries that only
// size a workspace.
int check_cache(const rocketkv_cache_t* c, bool need_pools, const char* who) {
  if (!c) return fail(ROCKETKV_INVALID_ARG, "%s: cache is NULL", who);
  if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1)
    return fail(ROCKETKV_INVALID_ARG, "%s: batch and head counts must be positive", who);
  if (c->n_q_heads % c->n_kv_heads != 0)
    return fail(ROCKETKV_INVALID_ARG, "%s: n_q_heads (%d) is not a multiple of n_kv_heads (%d)", who,
                c->n_q_heads, c->n_kv_heads);
  if (c->head_dim != kHeadDim)
    return fail(c->head_dim < 1 ? ROCKETKV_INVALID_ARG : ROCKETKV_UNSUPPORTED,
                "%s: head_dim %d (this build handles %d)", who, c->head_dim, kHeadDim);
  if (c->n_q_heads / c->n_kv_heads > kMaxGroup)
    return fail(ROCKETKV_UNSUPPORTED, "%s: group size %d exceeds %d", who,
                c->n_q_heads / c->n_kv_heads, kMaxGroup);
  if (c->v_layout != ROCKETKV_V_CHANNEL_MAJOR && c->v_layout != ROCKETKV_V_TOKEN_MAJOR)
    return fail(ROCKETKV_INVALID_ARG, "%s: unknown v_layout %d", who, c->v_layout);
  if (c->page_size < 1) return fail(ROCKETKV_INVALID_ARG, "%s: page_size must be >= 1", who);
  if (c->page_size > 64) return fail(ROCKETKV_UNSUPPORTED, "%s: page_size %d > 64", who, c->page_size);
  if (c->pages_cap < 1 || c->pages_cap % 8 != 0)
    return fail(ROCKETKV_INVALID_ARG, "%s: pages_cap (%d) must be a positive multiple of 8", who,
                c->pages_cap);
  if ((int64_t)c->batch * c->n_kv_heads * 4 > ROCKETKV_WS_HEADER_BYTES / 2)
    return fail(ROCKETKV_UNSUPPORTED, "%s: batch * n_kv_heads exceeds %d", who, ROCKETKV_WS_HEADER_BYTES / 8);
  if ((int64_t)c->pages_cap * c->page_size > (int64_t)1 << 30)
    return fail(ROCKETKV_INVALID_ARG, "%s: pages_cap * page_size overflows", who);
  if (need_pools) {
    if (!c->seq_lens || !c->k_pool || !c->v_pool)
      return fail(ROCKETKV_INVALID_ARG, "%s: seq_lens / k_pool / v_pool must not be NULL", who);
    const int64_t tile = (int64_t)c->page_size * kHeadDim;
    if (c->stride_head < tile || c->stride_page < (int64_t)c->n_kv_heads * tile || c->stride_head % 8 ||
        c->stride_page % 8)
      return fail(ROCKETKV_INVALID_ARG,
                  "%s: strides must be multiples of 8 elements with stride_head >= page_size*head_dim "
                  "and stride_page >= n_kv_heads*page_size*head_dim", who);
    if (c->n_phys_pages < 1) return fail(ROCKETKV_INVALID_ARG, "%s: n_phys_pages must be positive", who);
    if (c->n_phys_pages > 2147483647ll)
      return fail(ROCKETKV_UNSUPPORTED, "%s: n_phys_pages %lld exceeds 2^31 - 1", who, (long long)c->n_phys_pages);
    if (!c->block_table && c->n_phys_pages < (int64_t)c->batch * c->pages_cap)
      return fail(ROCKETKV_INVALID_ARG,
                  "%s: identity block table needs n_phys_pages >= batch * pages_cap", who);
    if (((uintptr_t)c->k_pool | (uintptr_t)c->v_pool) & 15)
      return fail(ROCKETKV_INVALID_ARG, "%s: pools must be 16-byte aligned", who);
  }
  return ROCKETKV_OK;
}

CacheView view_of(const rocketkv_cache_t* c) {
  CacheView v;
  v.batch = c->batch;
  v.n_q_heads = c->n_q_heads;
  v.n_kv_heads = c->n_kv_heads;
  v.group = c->n_q_heads / c->n_kv_heads;
  v.page_size = c->page_size;
  v.pages_cap = c->pages_cap;
  v.n_phys_pages = c->n_phys_pages;
  v.stride_page = c->stride_page;
  v.stride_head = c->stride_head;
  v.seq_lens = c->seq_lens;
  v.block_table = c->block_table;
  v.k_pool = static_cast<bf16_t*>(c->k_pool);
  v.v_pool = static_cast<bf16_t*>(c->v_pool);
  v.v_token_major = c->v_layout == ROCKETKV_V_TOKEN_MAJOR;
  return v;
}

int list_len_for_budget(const rocketkv_cache_t* c, int T) {
  int64_t need = ((int64_t)T + c->page_size - 1) / c->page_size;
  if (need < 1) need = 1;
  if (need > c->pages_cap) need = c->pages_cap;
  return (int)need;
}

int check_select_args(const rocketkv_cache_t* c, const void* q, const void* kmax, const void* kmin,
                      int k1, int T, int n_recent, const char* who) {
  if (!q || !kmax || !kmin) return fail(ROCKETKV_INVALID_ARG, "%s: q / kmax / kmin must not be NULL", who);
  if (k1 < 1 || k1 > c->head_dim)
    return fail(ROCKETKV_INVALID_ARG, "%s: channel_budget %d outside [1, %d]", who, k1, c->head_dim);
  if (T < 1) return fail(ROCKETKV_INVALID_ARG, "%s: token_budget must be >= 1", who);
  if (n_recent < 0) return fail(ROCKETKV_INVALID_ARG, "%s: n_recent_pages must be >= 0", who);
  if (c->pages_cap > ROCKETKV_MAX_PAGES)
    return fail(ROCKETKV_UNSUPPORTED, "%s: pages_cap %d exceeds %d", who, c->pages_cap, ROCKETKV_MAX_PAGES);
  if (((uintptr_t)q | (uintptr_t)kmax | (uintptr_t)kmin) & 15)
    return fail(ROCKETKV_INVALID_ARG, "%s: q / kmax / kmin must be 16-byte aligned", who);
  return ROCKETKV_OK;
}

int check_attend_shape(const rocketkv_cache_t* c, const char* who) {
  if (c->v_layout == ROCKETKV_V_CHANNEL_MAJOR && c->page_size != kAttnPage)
    return fail(ROCKETKV_UNSUPPORTED, "%s: attention over channel-major V needs page_size %d (got %d)", who,
                kAttnPage, c->page_size);
  return ROCKETKV_OK;
}

// Launch geometry of Step 3 over `row_len` list entries.  The plan counts 16-token entries; a
// token-major cache of another page size is planned on the token slots its entries add up to.
// `gather`: a page list drives the launch (false: the identity list of the Full-KV baseline).
AttendPlan attend_plan_for(const CacheView& v, int row_len, bool gather) {
  if (!v.v_token_major) return plan_attend(v, row_len, gather);
  // whole entries only: the kernel's last wavefront absorbs a remainder of fewer than 16 slots
  const int64_t slots = (int64_t)row_len * v.page_size;
  return plan_attend(v, slots >= kAttnPage ? (int)(slots / kAttnPage) : 1, gather);
}

hipError_t launch_attend_any(const CacheView& v, const bf16_t* q, const int32_t* pages, int row_len,
                             bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                             hipStream_t st) {
  return v.v_token_major ? launch_attend_tokens(v, q, pages, row_len, out, out_lse, ws, plan, nullptr, st)
                         : launch_attend(v, q, pages, row_len, out, out_lse, ws, plan, st);
}

// argument rules of Stage 1 that involve the source only
int check_snapkv_args(const void* q_obs, const rocketkv_cache_t* src, int32_t window, int32_t pool_kernel,
                      int32_t keep_budget, const char* who) {
  if (!q_obs) return fail(ROCKETKV_INVALID_ARG, "%s: q_obs must not be NULL", who);
  if (((uintptr_t)q_obs) & 15) return fail(ROCKETKV_INVALID_ARG, "%s: q_obs must be 16-byte aligned", who);
  if (src->page_size != kAttnPage)
    return fail(ROCKETKV_UNSUPPORTED, "%s: src needs page_size %d (got %d)", who, kAttnPage, src->page_size);
  if (window < 1 || window > 128 || window % 16 != 0)
    return fail(window < 1 ? ROCKETKV_INVALID_ARG : ROCKETKV_UNSUPPORTED,
                "%s: window %d must be a multiple of 16 in [16, 128]", who, window);
  if ((src->n_q_heads / src->n_kv_heads) * window > 256)
    return fail(ROCKETKV_UNSUPPORTED, "%s: group size x window (%d) exceeds 256", who,
                (src->n_q_heads / src->n_kv_heads) * window);
  if (pool_kernel < 1 || pool_kernel % 2 == 0)
    return fail(ROCKETKV_INVALID_ARG, "%s: pool_kernel %d must be odd and positive", who, pool_kernel);
  if (pool_kernel > 1023) return fail(ROCKETKV_UNSUPPORTED, "%s: pool_kernel %d > 1023", who, pool_kernel);
  if (keep_budget <= window)
    return fail(ROCKETKV_INVALID_ARG, "%s: keep_budget %d must exceed window %d", who, keep_budget, window);
  return ROCKETKV_OK;
}

struct DecodePlan {
  AttendPlan attend;
  int row_len;
  size_t list_off, scores_off, attend_off, total;
};

DecodePlan plan_decode(const rocketkv_cache_t* c, int T) {
  DecodePlan d;
  const CacheView v = view_of(c);
  d.row_len = list_len_for_budget(c, T);
  d.attend = attend_plan_for(v, d.row_len, true);
  size_t off = 0;
  d.attend_off = off;  // first, so that the counters sit in the header workspace_init clears
  off += d.attend.total_bytes;
  d.list_off = off;
  off += ((size_t)c->batch * c->n_kv_heads * d.row_len * sizeof(int32_t) + 255) / 256 * 256;
  d.scores_off = off;  // page scores, for selections that run as a score launch plus a top-k launch
  off += ((size_t)c->batch * c->n_kv_heads * c->pages_cap * sizeof(float) + 255) / 256 * 256;
  d.total = off;
  return d;
}

}  // namespace

extern "C" {

const char* rocketkv_last_error(void) { return g_err; }

int32_t rocketkv_version(void) { return 100; }

size_t rocketkv_workspace_bytes(int32_t op, const rocketkv_cache_t* cache, int32_t a, int32_t b) {
  g_err[0] = 0;
  if (check_cache(cache, false, "rocketkv_workspace_bytes")) return 0;
  const CacheView v = view_of(cache);
  switch (op) {
    case ROCKETKV_OP_HSA_DECODE:
      if (a < 1) { fail(ROCKETKV_INVALID_ARG, "rocketkv_workspace_bytes: token_budget must be >= 1"); return 0; }
      return plan_decode(cache, a).total;
    case ROCKETKV_OP_DENSE_DECODE:
      return attend_plan_for(v, cache->pages_cap, false).total_bytes;
    case ROCKETKV_OP_ATTEND:
      if (a < 0) { fail(ROCKETKV_INVALID_ARG, "rocketkv_workspace_bytes: pages_row_len must be >= 0"); return 0; }
      return attend_plan_for(v, a > 0 ? a : cache->pages_cap, a > 0).total_bytes;
    case ROCKETKV_OP_SNAPKV:
      if (a < 1 || b <= a) { fail(ROCKETKV_INVALID_ARG, "rocketkv_workspace_bytes: need 1 <= window < keep_budget"); return 0; }
      return plan_snapkv(v, a, b).total_bytes;
    default:
      fail(ROCKETKV_INVALID_ARG, "rocketkv_workspace_bytes: unknown op %d", op);
      return 0;
  }
}

int32_t rocketkv_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  if (!workspace) return fail(ROCKETKV_INVALID_ARG, "rocketkv_workspace_init: workspace is NULL");
  if ((uintptr_t)workspace & 255)
    return fail(ROCKETKV_INVALID_ARG, "rocketkv_workspace_init: workspace must be 256-byte aligned");
  const size_t n = workspace_bytes < ROCKETKV_WS_HEADER_BYTES ? workspace_bytes : (size_t)ROCKETKV_WS_HEADER_BYTES;
  const hipError_t e = launch_zero(workspace, n / 4 * 4, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, "rocketkv_workspace_init");
}

int32_t rocketkv_build_page_summaries(const rocketkv_cache_t* cache, void* kmax, void* kmin,
                                      int32_t first_page, int32_t n_pages, void* stream) {
  g_err[0] = 0;
  if (int r = check_cache(cache, true, "rocketkv_build_page_summaries")) return r;
  if (!kmax || !kmin) return fail(ROCKETKV_INVALID_ARG, "rocketkv_build_page_summaries: kmax / kmin must not be NULL");
  if (first_page < 0 || first_page > cache->pages_cap)
    return fail(ROCKETKV_INVALID_ARG, "rocketkv_build_page_summaries: first_page %d outside [0, %d]",
                first_page, cache->pages_cap);
  const hipError_t e = launch_page_summaries(view_of(cache), static_cast<bf16_t*>(kmax),
                                             static_cast<bf16_t*>(kmin), first_page, n_pages,
                                             static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, "rocketkv_build_page_summaries");
}

int32_t rocketkv_hsa_select(const rocketkv_cache_t* cache, const void* q, const void* kmax,
                            const void* kmin, int32_t channel_budget, int32_t token_budget,
                            int32_t n_recent_pages, int32_t* out_pages, int32_t pages_row_len,
                            int32_t* out_channels, float* out_scores, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_hsa_select";
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_select_args(cache, q, kmax, kmin, channel_budget, token_budget, n_recent_pages, who)) return r;
  if (!out_pages) return fail(ROCKETKV_INVALID_ARG, "%s: out_pages must not be NULL", who);
  if (cache->pages_cap > kSingleSelectPages && !out_scores)
    return fail(ROCKETKV_UNSUPPORTED, "%s: pages_cap %d > %d needs out_scores", who, cache->pages_cap,
                kSingleSelectPages);
  if (pages_row_len < list_len_for_budget(cache, token_budget))
    return fail(ROCKETKV_INVALID_ARG, "%s: pages_row_len %d < %d needed for this budget", who,
                pages_row_len, list_len_for_budget(cache, token_budget));
  SelectArgs a;
  a.q = static_cast<const bf16_t*>(q);
  a.kmax = static_cast<const bf16_t*>(kmax);
  a.kmin = static_cast<const bf16_t*>(kmin);
  a.k1 = channel_budget;
  a.T = token_budget;
  a.n_recent = n_recent_pages;
  a.out_pages = out_pages;
  a.row_len = pages_row_len;
  a.out_pages2 = nullptr;
  a.row_len2 = 0;
  a.out_channels = out_channels;
  a.out_scores = out_scores;
  a.in_scores = nullptr;
  const hipError_t e = launch_hsa_select(view_of(cache), a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

int32_t rocketkv_attend(const rocketkv_cache_t* cache, const void* q, const int32_t* pages,
                        int32_t pages_row_len, void* out, float* out_lse, void* workspace,
                        size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_attend";
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_attend_shape(cache, who)) return r;
  if (!q || !out) return fail(ROCKETKV_INVALID_ARG, "%s: q / out must not be NULL", who);
  if (((uintptr_t)q) & 15) return fail(ROCKETKV_INVALID_ARG, "%s: q must be 16-byte aligned", who);
  if (pages && pages_row_len < 1) return fail(ROCKETKV_INVALID_ARG, "%s: pages_row_len must be >= 1", who);
  const int row_len = pages ? pages_row_len : cache->pages_cap;
  const CacheView v = view_of(cache);
  const AttendPlan plan = attend_plan_for(v, row_len, pages != nullptr);
  if (plan.total_bytes && (!workspace || workspace_bytes < plan.total_bytes))
    return fail(ROCKETKV_WORKSPACE_TOO_SMALL, "%s: workspace %zu bytes < %zu needed", who,
                workspace ? workspace_bytes : (size_t)0, plan.total_bytes);
  if ((uintptr_t)workspace & 255) return fail(ROCKETKV_INVALID_ARG, "%s: workspace must be 256-byte aligned", who);
  const hipError_t e = launch_attend_any(v, static_cast<const bf16_t*>(q), pages, row_len,
                                         static_cast<bf16_t*>(out), out_lse, workspace, plan,
                                         static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

int32_t rocketkv_dense_decode(const rocketkv_cache_t* cache, const void* q, void* out,
                              float* out_lse, void* workspace, size_t workspace_bytes,
                              void* stream) {
  return rocketkv_attend(cache, q, nullptr, 0, out, out_lse, workspace, workspace_bytes, stream);
}

namespace {

// Shared body of rocketkv_hsa_decode and rocketkv_hsa_decode_append (k_new == NULL: no append).
int decode_impl(const char* who, const rocketkv_cache_t* cache, const void* q, const void* k_new,
                const void* v_new, void* kmax, void* kmin, int32_t channel_budget, int32_t token_budget,
                int32_t n_recent_pages, void* out, float* out_lse, int32_t* out_pages,
                int32_t* out_channels, void* workspace, size_t workspace_bytes, void* stream) {
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_attend_shape(cache, who)) return r;
  if (int r = check_select_args(cache, q, kmax, kmin, channel_budget, token_budget, n_recent_pages, who)) return r;
  if (!out) return fail(ROCKETKV_INVALID_ARG, "%s: out must not be NULL", who);
  const DecodePlan d = plan_decode(cache, token_budget);
  if (!workspace || workspace_bytes < d.total)
    return fail(ROCKETKV_WORKSPACE_TOO_SMALL, "%s: workspace %zu bytes < %zu needed", who,
                workspace ? workspace_bytes : (size_t)0, d.total);
  if ((uintptr_t)workspace & 255) return fail(ROCKETKV_INVALID_ARG, "%s: workspace must be 256-byte aligned", who);
  const CacheView v = view_of(cache);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  SelectArgs a;
  a.q = static_cast<const bf16_t*>(q);
  a.kmax = static_cast<const bf16_t*>(kmax);
  a.kmin = static_cast<const bf16_t*>(kmin);
  a.k1 = channel_budget;
  a.T = token_budget;
  a.n_recent = n_recent_pages;
  a.row_len = d.row_len;
  a.out_channels = out_channels;
  a.out_scores = nullptr;
  a.in_scores = nullptr;
  AppendArgs ap = {static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new),
                   static_cast<bf16_t*>(kmax), static_cast<bf16_t*>(kmin)};
  hipError_t e;
  if (!v.v_token_major && fused_decode_lds_bytes(v, d.row_len, d.attend) + 64 <= kMaxLdsBytes) {
    // one launch: every workgroup selects for itself and keeps the list in LDS
    a.out_pages = out_pages;
    a.out_pages2 = nullptr;
    a.row_len2 = 0;
    e = launch_hsa_decode_fused(v, a, ap, static_cast<bf16_t*>(out), out_lse, ws + d.attend_off, d.attend, st);
    return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
  }
  if (v.v_token_major && !select_wants_split(v, a.k1) &&
      fused_decode_tok_lds_bytes(v, d.row_len, d.attend) + 64 <= kMaxLdsBytes) {
    a.out_pages = out_pages;
    a.out_pages2 = nullptr;
    a.row_len2 = 0;
    e = launch_hsa_decode_tok_fused(v, nullptr, a, ap, static_cast<bf16_t*>(out), out_lse, ws + d.attend_off,
                                    d.attend, st);
    return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
  }
  a.out_pages = reinterpret_cast<int32_t*>(ws + d.list_off);
  a.out_pages2 = out_pages;
  a.row_len2 = d.row_len;
  if (select_wants_split(v, a.k1)) {
    // score launch (which also takes in the new token) + top-k launch
    a.out_scores = reinterpret_cast<float*>(ws + d.scores_off);
    e = launch_hsa_select_split(v, a, ap, attend_counters(ws + d.attend_off, d.attend),
                                decode_seq_counters(ws + d.attend_off, d.attend), st);
  } else {
    if (k_new) {
      e = launch_append(v, ap.k_new, ap.v_new, ap.kmax, ap.kmin, st);
      if (e != hipSuccess) return hip_fail(e, who);
    }
    e = launch_hsa_select(v, a, st);
  }
  if (e != hipSuccess) return hip_fail(e, who);
  e = launch_attend_any(v, a.q, a.out_pages, d.row_len, static_cast<bf16_t*>(out), out_lse,
                        ws + d.attend_off, d.attend, st);
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

}  // namespace

int32_t rocketkv_hsa_decode(const rocketkv_cache_t* cache, const void* q, const void* kmax,
                            const void* kmin, int32_t channel_budget, int32_t token_budget,
                            int32_t n_recent_pages, void* out, float* out_lse,
                            int32_t* out_pages, int32_t* out_channels, void* workspace,
                            size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  return decode_impl("rocketkv_hsa_decode", cache, q, nullptr, nullptr, const_cast<void*>(kmax),
                     const_cast<void*>(kmin), channel_budget, token_budget, n_recent_pages, out, out_lse,
                     out_pages, out_channels, workspace, workspace_bytes, stream);
}

// ---- rocketkv_hsa_decode with the library's own scratch memory ------------------------------------
// One array per GPU, owned by the library's code object on that GPU until the process ends.  In host
// code the array's name is only a handle for the runtime: the device address comes from
// hipGetSymbolAddress, once per device, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[ROCKETKV_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, null until first use there

// The address of `scratch` on the current device (looked up on the first call there), or null with
// the reason in g_err.
void* scratch_on_current_device(const char* who) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { hip_fail(e, who); return nullptr; }
  if (dev < 0 || dev >= kMaxDevices) {
    fail(ROCKETKV_UNSUPPORTED, "%s: device ordinal %d outside [0, %d)", who, dev, kMaxDevices);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { hip_fail(e, who); return nullptr; }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}
}  // namespace

int32_t rocketkv_hsa_decode_noalloc(const rocketkv_cache_t* cache, const void* q, const void* kmax,
                                    const void* kmin, int32_t channel_budget, int32_t token_budget,
                                    int32_t n_recent_pages, void* out, float* out_lse,
                                    int32_t* out_pages, int32_t* out_channels, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_hsa_decode_noalloc";
  if (int r = check_cache(cache, true, who)) return r;
  if (token_budget < 1) return fail(ROCKETKV_INVALID_ARG, "%s: token_budget must be >= 1", who);
  const size_t need = plan_decode(cache, token_budget).total;
  if (need > (size_t)ROCKETKV_NOALLOC_SCRATCH_BYTES)
    return fail(ROCKETKV_UNSUPPORTED,
                "%s: this shape needs %zu bytes of scratch, the built-in buffer holds %zu; use "
                "rocketkv_hsa_decode with a workspace of the caller's", who, need,
                (size_t)ROCKETKV_NOALLOC_SCRATCH_BYTES);
  void* ws = scratch_on_current_device(who);
  if (!ws) return g_err[0] ? ROCKETKV_HIP_ERROR : ROCKETKV_HIP_ERROR;
  // The buffer keeps whatever the last call on this GPU left in it.  What a call expects to find at
  // zero, the arrival counters in the leading header, is cleared here by a fill kernel (a launch, not a
  // memset node, so the call can be captured into a graph); everything else is written before it is read.
  const hipError_t e = launch_zero(ws, ROCKETKV_WS_HEADER_BYTES, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, who);
  return decode_impl(who, cache, q, nullptr, nullptr, const_cast<void*>(kmax), const_cast<void*>(kmin),
                     channel_budget, token_budget, n_recent_pages, out, out_lse, out_pages, out_channels, ws,
                     (size_t)ROCKETKV_NOALLOC_SCRATCH_BYTES, stream);
}

int32_t rocketkv_hsa_decode_append(const rocketkv_cache_t* cache, const void* q, const void* k_new,
                                   const void* v_new, void* kmax, void* kmin, int32_t channel_budget,
                                   int32_t token_budget, int32_t n_recent_pages, void* out,
                                   float* out_lse, int32_t* out_pages, int32_t* out_channels,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_hsa_decode_append";
  if (!k_new || !v_new) return fail(ROCKETKV_INVALID_ARG, "%s: k_new / v_new must not be NULL", who);
  return decode_impl(who, cache, q, k_new, v_new, kmax, kmin, channel_budget, token_budget,
                     n_recent_pages, out, out_lse, out_pages, out_channels, workspace, workspace_bytes,
                     stream);
}

int32_t rocketkv_append_kv(const rocketkv_cache_t* cache, const void* k_new, const void* v_new,
                           void* kmax, void* kmin, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_append_kv";
  if (int r = check_cache(cache, true, who)) return r;
  if (!k_new || !v_new || !kmax || !kmin)
    return fail(ROCKETKV_INVALID_ARG, "%s: k_new / v_new / kmax / kmin must not be NULL", who);
  const hipError_t e = launch_append(view_of(cache), static_cast<const bf16_t*>(k_new),
                                     static_cast<const bf16_t*>(v_new), static_cast<bf16_t*>(kmax),
                                     static_cast<bf16_t*>(kmin), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

size_t rocketkv_stream_read_sink_bytes(void) { return (size_t)probe_read_workgroups() * 4 * sizeof(uint32_t); }

int32_t rocketkv_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_stream_read";
  if (!src || !sink) return fail(ROCKETKV_INVALID_ARG, "%s: src / sink must not be NULL", who);
  if ((bytes & 15) || ((uintptr_t)src & 15))
    return fail(ROCKETKV_INVALID_ARG, "%s: src and bytes must be multiples of 16", who);
  if (bytes == 0) return ROCKETKV_OK;
  const hipError_t e = launch_stream_read(src, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

size_t rocketkv_stream_gather_sink_bytes(const rocketkv_cache_t* cache, int32_t pages_row_len) {
  g_err[0] = 0;
  if (check_cache(cache, false, "rocketkv_stream_gather_sink_bytes")) return 0;
  if (pages_row_len < 1) { fail(ROCKETKV_INVALID_ARG, "rocketkv_stream_gather_sink_bytes: pages_row_len must be >= 1"); return 0; }
  return probe_gather_sink_words(view_of(cache), pages_row_len) * sizeof(uint32_t);
}

int32_t rocketkv_stream_gather(const rocketkv_cache_t* cache, const int32_t* pages, int32_t pages_row_len,
                               void* sink, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_stream_gather";
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_attend_shape(cache, who)) return r;
  if (cache->v_layout != ROCKETKV_V_CHANNEL_MAJOR)
    return fail(ROCKETKV_UNSUPPORTED, "%s: the probe reads channel-major V tiles of 16-token pages", who);
  if (!pages || !sink) return fail(ROCKETKV_INVALID_ARG, "%s: pages / sink must not be NULL", who);
  if (pages_row_len < 1) return fail(ROCKETKV_INVALID_ARG, "%s: pages_row_len must be >= 1", who);
  const hipError_t e = launch_stream_gather(view_of(cache), pages, pages_row_len, static_cast<uint32_t*>(sink),
                                            static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

int32_t rocketkv_snapkv_compress(const void* q_obs, const rocketkv_cache_t* src, int32_t window,
                                 int32_t pool_kernel, int32_t keep_budget,
                                 const rocketkv_cache_t* dst, int32_t* kept_idx, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_snapkv_compress";
  if (int r = check_cache(src, true, who)) return r;
  if (int r = check_cache(dst, true, who)) return r;
  if (int r = check_snapkv_args(q_obs, src, window, pool_kernel, keep_budget, who)) return r;
  if (src->batch != dst->batch || src->n_q_heads != dst->n_q_heads || src->n_kv_heads != dst->n_kv_heads)
    return fail(ROCKETKV_INVALID_ARG, "%s: src and dst must agree on batch and head counts", who);
  if (dst->v_layout == ROCKETKV_V_CHANNEL_MAJOR && dst->page_size != kAttnPage)
    return fail(ROCKETKV_UNSUPPORTED, "%s: a dst with channel-major V needs page_size %d (got %d)", who,
                kAttnPage, dst->page_size);
  if ((int64_t)dst->pages_cap * dst->page_size < keep_budget)
    return fail(ROCKETKV_INVALID_ARG, "%s: dst holds %lld tokens per sequence < keep_budget %d", who,
                (long long)dst->pages_cap * dst->page_size, keep_budget);
  if (src->k_pool == dst->k_pool || src->v_pool == dst->v_pool)
    return fail(ROCKETKV_INVALID_ARG, "%s: src and dst pools must be distinct", who);
  const CacheView sv = view_of(src), dv = view_of(dst);
  const SnapPlan plan = plan_snapkv(sv, window, keep_budget);
  if (!workspace || workspace_bytes < plan.total_bytes)
    return fail(ROCKETKV_WORKSPACE_TOO_SMALL, "%s: workspace %zu bytes < %zu needed", who,
                workspace ? workspace_bytes : (size_t)0, plan.total_bytes);
  if ((uintptr_t)workspace & 255) return fail(ROCKETKV_INVALID_ARG, "%s: workspace must be 256-byte aligned", who);
  const hipError_t e = launch_snapkv(static_cast<const bf16_t*>(q_obs), sv, window, pool_kernel,
                                     keep_budget, &dv, kept_idx, keep_budget, dv.seq_lens, workspace, plan,
                                     static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

int32_t rocketkv_decompose(int64_t seq_len, int32_t token_budget, int32_t head_dim,
                           rocketkv_split_t* out) {
  g_err[0] = 0;
  const char* who = "rocketkv_decompose";
  if (!out) return fail(ROCKETKV_INVALID_ARG, "%s: out is NULL", who);
  if (seq_len < 1 || token_budget < 1 || head_dim < 1)
    return fail(ROCKETKV_INVALID_ARG, "%s: seq_len, token_budget and head_dim must be positive", who);
  if (seq_len > ((int64_t)1 << 40)) return fail(ROCKETKV_INVALID_ARG, "%s: seq_len too large", who);
  rocketkv_split_t s;
  s.c = fmax(1.0, (double)seq_len / (double)token_budget);
  s.r = fmin(0.2 + 0.06 * log2(s.c), 0.8);
  s.stage1 = pow(s.c, s.r);
  s.stage2 = pow(s.c, 1.0 - s.r);
  const double seq_ratio = ceil(pow(s.c, 0.5 * (1.0 - s.r)));  // sequence-dimension share, a whole page size
  s.head_ratio = s.stage2 / seq_ratio;
  s.page_size = (int32_t)seq_ratio;
  const double keep = floor((double)seq_len / s.stage1 + 0.5);
  s.keep_budget = (int32_t)fmin(fmax(keep, 1.0), fmin((double)seq_len, 2147483647.0));
  const double ch = floor((double)head_dim / s.head_ratio + 0.5);
  s.channel_budget = (int32_t)fmin(fmax(ch, 1.0), (double)head_dim);
  s.attend_tokens = token_budget / 2 > 1 ? token_budget / 2 : 1;
  const double aux = 2.0 / pow(s.c, 0.5 * (1.0 + s.r));  // K_max and K_min, Table 1's accounting
  s.storage = 1.0 / s.stage1 + aux;
  s.storage_mt = 1.0 + aux;
  s.traffic = 1.0 / s.c;
  *out = s;
  return ROCKETKV_OK;
}

}  // extern "C"

namespace {

int check_index(const rocketkv_cache_t* c, const rocketkv_index_t* ix, const char* who) {
  if (!ix) return fail(ROCKETKV_INVALID_ARG, "%s: index is NULL", who);
  if (!ix->token_index || !ix->n_indexed)
    return fail(ROCKETKV_INVALID_ARG, "%s: index->token_index / n_indexed must not be NULL", who);
  if (ix->page_size < 1) return fail(ROCKETKV_INVALID_ARG, "%s: index->page_size must be >= 1", who);
  if (ix->page_size > 64) return fail(ROCKETKV_UNSUPPORTED, "%s: index->page_size %d > 64", who, ix->page_size);
  if (ix->pages_cap < 1 || ix->pages_cap % 8 != 0)
    return fail(ROCKETKV_INVALID_ARG, "%s: index->pages_cap (%d) must be a positive multiple of 8", who,
                ix->pages_cap);
  if ((int64_t)ix->pages_cap * ix->page_size > (int64_t)1 << 30)
    return fail(ROCKETKV_INVALID_ARG, "%s: index->pages_cap * page_size overflows", who);
  if (c->v_layout != ROCKETKV_V_TOKEN_MAJOR)
    return fail(ROCKETKV_UNSUPPORTED, "%s: the cache behind an index needs token-major V", who);
  return ROCKETKV_OK;
}

LogicalView logical_of(const rocketkv_index_t* ix) {
  LogicalView lv;
  lv.token_index = ix->token_index;
  lv.n_indexed = ix->n_indexed;
  lv.page_size = ix->page_size;
  lv.pages_cap = ix->pages_cap;
  return lv;
}

// The cache as Step 2 sees it under an index: lengths, page size and page capacity of the logical
// sequence (the selection never touches the pools).
rocketkv_cache_t logical_cache(const rocketkv_cache_t* c, const rocketkv_index_t* ix) {
  rocketkv_cache_t lc = *c;
  lc.seq_lens = ix->n_indexed;
  lc.page_size = ix->page_size;
  lc.pages_cap = ix->pages_cap;
  return lc;
}

int mt_decode_impl(const char* who, const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                   const void* q, const void* k_new, const void* v_new, void* kmax, void* kmin,
                   int32_t channel_budget, int32_t token_budget, int32_t n_recent_pages, void* out,
                   float* out_lse, int32_t* out_pages, int32_t* out_channels, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_index(cache, index, who)) return r;
  const rocketkv_cache_t lc = logical_cache(cache, index);
  if (int r = check_select_args(&lc, q, kmax, kmin, channel_budget, token_budget, n_recent_pages, who)) return r;
  if (!out) return fail(ROCKETKV_INVALID_ARG, "%s: out must not be NULL", who);
  const DecodePlan d = plan_decode(&lc, token_budget);
  if (!workspace || workspace_bytes < d.total)
    return fail(ROCKETKV_WORKSPACE_TOO_SMALL, "%s: workspace %zu bytes < %zu needed", who,
                workspace ? workspace_bytes : (size_t)0, d.total);
  if ((uintptr_t)workspace & 255) return fail(ROCKETKV_INVALID_ARG, "%s: workspace must be 256-byte aligned", who);
  const CacheView v = view_of(cache), lcv = view_of(&lc);
  const LogicalView lv = logical_of(index);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  hipError_t e;
  SelectArgs a;
  a.q = static_cast<const bf16_t*>(q);
  a.kmax = static_cast<const bf16_t*>(kmax);
  a.kmin = static_cast<const bf16_t*>(kmin);
  a.k1 = channel_budget;
  a.T = token_budget;
  a.n_recent = n_recent_pages;
  a.row_len = d.row_len;
  a.out_channels = out_channels;
  if (!select_wants_split(lcv, a.k1) && fused_decode_tok_lds_bytes(lcv, d.row_len, d.attend) + 64 <= kMaxLdsBytes) {
    // one launch: selection on the logical sequence, attention through the index, append folded in
    const AppendArgs ap = {static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new),
                           static_cast<bf16_t*>(kmax), static_cast<bf16_t*>(kmin)};
    a.out_pages = out_pages;
    a.out_pages2 = nullptr;
    a.row_len2 = 0;
    a.out_scores = nullptr;
    a.in_scores = nullptr;
    e = launch_hsa_decode_tok_fused(v, &lv, a, ap, static_cast<bf16_t*>(out), out_lse, ws + d.attend_off,
                                    d.attend, st);
    return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
  }
  if (k_new) {
    e = launch_append_indexed(v, lv, static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new),
                              static_cast<bf16_t*>(kmax), static_cast<bf16_t*>(kmin), st);
    if (e != hipSuccess) return hip_fail(e, who);
  }
  a.out_pages = reinterpret_cast<int32_t*>(ws + d.list_off);
  a.out_pages2 = out_pages;
  a.row_len2 = d.row_len;
  a.out_scores = select_wants_split(lcv, a.k1) ? reinterpret_cast<float*>(ws + d.scores_off) : nullptr;
  a.in_scores = nullptr;
  e = launch_hsa_select(lcv, a, st);
  if (e != hipSuccess) return hip_fail(e, who);
  e = launch_attend_tokens(v, a.q, a.out_pages, d.row_len, static_cast<bf16_t*>(out), out_lse,
                           ws + d.attend_off, d.attend, &lv, st);
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

}  // namespace

extern "C" {

int32_t rocketkv_snapkv_filter(const void* q_obs, const rocketkv_cache_t* src, int32_t window,
                               int32_t pool_kernel, int32_t keep_budget, const rocketkv_index_t* index,
                               void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_snapkv_filter";
  if (int r = check_cache(src, true, who)) return r;
  if (int r = check_snapkv_args(q_obs, src, window, pool_kernel, keep_budget, who)) return r;
  if (!index || !index->token_index || !index->n_indexed)
    return fail(ROCKETKV_INVALID_ARG, "%s: index and its arrays must not be NULL", who);
  if (index->page_size < 1 || index->pages_cap < 1 ||
      (int64_t)index->pages_cap * index->page_size < keep_budget)
    return fail(ROCKETKV_INVALID_ARG, "%s: index rows hold %lld entries < keep_budget %d", who,
                (long long)index->pages_cap * index->page_size, keep_budget);
  const CacheView sv = view_of(src);
  const SnapPlan plan = plan_snapkv(sv, window, keep_budget);
  if (!workspace || workspace_bytes < plan.total_bytes)
    return fail(ROCKETKV_WORKSPACE_TOO_SMALL, "%s: workspace %zu bytes < %zu needed", who,
                workspace ? workspace_bytes : (size_t)0, plan.total_bytes);
  if ((uintptr_t)workspace & 255) return fail(ROCKETKV_INVALID_ARG, "%s: workspace must be 256-byte aligned", who);
  const hipError_t e = launch_snapkv(static_cast<const bf16_t*>(q_obs), sv, window, pool_kernel, keep_budget,
                                     nullptr, index->token_index, index->pages_cap * index->page_size,
                                     index->n_indexed, workspace, plan, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

int32_t rocketkv_mt_build_page_summaries(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                                         void* kmax, void* kmin, int32_t first_page, int32_t n_pages,
                                         void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_mt_build_page_summaries";
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_index(cache, index, who)) return r;
  if (!kmax || !kmin) return fail(ROCKETKV_INVALID_ARG, "%s: kmax / kmin must not be NULL", who);
  if (first_page < 0 || first_page > index->pages_cap)
    return fail(ROCKETKV_INVALID_ARG, "%s: first_page %d outside [0, %d]", who, first_page, index->pages_cap);
  const hipError_t e = launch_page_summaries_indexed(view_of(cache), logical_of(index),
                                                     static_cast<bf16_t*>(kmax), static_cast<bf16_t*>(kmin),
                                                     first_page, n_pages, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

size_t rocketkv_mt_workspace_bytes(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                                   int32_t token_budget) {
  g_err[0] = 0;
  const char* who = "rocketkv_mt_workspace_bytes";
  if (check_cache(cache, false, who)) return 0;
  if (!index || index->page_size < 1 || index->page_size > 64 || index->pages_cap < 1 || index->pages_cap % 8) {
    fail(ROCKETKV_INVALID_ARG, "%s: index needs page_size in [1, 64] and pages_cap a positive multiple of 8", who);
    return 0;
  }
  if (token_budget < 1) { fail(ROCKETKV_INVALID_ARG, "%s: token_budget must be >= 1", who); return 0; }
  rocketkv_cache_t lc = *cache;
  lc.page_size = index->page_size;
  lc.pages_cap = index->pages_cap;
  lc.v_layout = ROCKETKV_V_TOKEN_MAJOR;
  return plan_decode(&lc, token_budget).total;
}

int32_t rocketkv_mt_hsa_decode(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                               const void* q, const void* kmax, const void* kmin,
                               int32_t channel_budget, int32_t token_budget, int32_t n_recent_pages,
                               void* out, float* out_lse, int32_t* out_pages, int32_t* out_channels,
                               void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  return mt_decode_impl("rocketkv_mt_hsa_decode", cache, index, q, nullptr, nullptr, const_cast<void*>(kmax),
                        const_cast<void*>(kmin), channel_budget, token_budget, n_recent_pages, out, out_lse,
                        out_pages, out_channels, workspace, workspace_bytes, stream);
}

int32_t rocketkv_mt_append_kv(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                              const void* k_new, const void* v_new, void* kmax, void* kmin,
                              void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_mt_append_kv";
  if (int r = check_cache(cache, true, who)) return r;
  if (int r = check_index(cache, index, who)) return r;
  if (!k_new || !v_new || !kmax || !kmin)
    return fail(ROCKETKV_INVALID_ARG, "%s: k_new / v_new / kmax / kmin must not be NULL", who);
  const hipError_t e = launch_append_indexed(view_of(cache), logical_of(index),
                                             static_cast<const bf16_t*>(k_new), static_cast<const bf16_t*>(v_new),
                                             static_cast<bf16_t*>(kmax), static_cast<bf16_t*>(kmin),
                                             static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ROCKETKV_OK : hip_fail(e, who);
}

int32_t rocketkv_mt_hsa_decode_append(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                                      const void* q, const void* k_new, const void* v_new, void* kmax,
                                      void* kmin, int32_t channel_budget, int32_t token_budget,
                                      int32_t n_recent_pages, void* out, float* out_lse,
                                      int32_t* out_pages, int32_t* out_channels, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  const char* who = "rocketkv_mt_hsa_decode_append";
  if (!k_new || !v_new) return fail(ROCKETKV_INVALID_ARG, "%s: k_new / v_new must not be NULL", who);
  return mt_decode_impl(who, cache, index, q, k_new, v_new, kmax, kmin, channel_budget, token_budget,
                        n_recent_pages, out, out_lse, out_pages, out_channels, workspace, workspace_bytes,
                        stream);
}

}  // extern "C"
