// HSA Step 1 (Section 3.4 of arXiv 2502.14051): per-page element-wise max / min of the keys,
// stored channel-major with the page index contiguous, plus the per-token append that keeps the
// tail page's summary current.
//
// Bandwidth-bound: one pass over K.  Sixteen lanes x 16 B cover one 256 B token row; each group of 16
// lanes reduces whole pages of its own, four rows in flight, so a wavefront has four pages under way at
// any page size and nothing crosses lanes; the workgroup transposes its 64 pages through LDS so that
// every summary row is written as one 128 B run.
#include "common.h"

namespace rkv {

constexpr int kSumPages = 64;   // pages per workgroup
constexpr int kSumPad = 66;     // LDS row pitch in bf16 (33 dwords: conflict-free column writes)

__global__ __launch_bounds__(256) void page_summaries_kernel(CacheView c, bf16_t* __restrict__ kmax,
                                                             bf16_t* __restrict__ kmin,
                                                             int first_page, int last_page) {
  __shared__ bf16_t tmax[kHeadDim * kSumPad];
  __shared__ bf16_t tmin[kHeadDim * kSumPad];
  const int unit = blockIdx.y;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int n = c.seq_lens[b];
  const int ps = c.page_size;
  int P = (n + ps - 1) / ps;
  if (P > c.pages_cap) P = c.pages_cap;
  const int p0 = first_page + blockIdx.x * kSumPages;
  const int pend = min(min(p0 + kSumPages, last_page), P);
  if (p0 >= pend) return;
  const int npg = pend - p0;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int tg = lane / 16, cl = lane % 16;

  // every 16-lane group takes whole pages of its own (no cross-lane step), four rows in flight
  for (int pl = wave * 4 + tg; pl < npg; pl += 16) {
    const int p = p0 + pl;
    const int64_t pp = phys_page(c, b, p);
    const int ntok = min(ps, n - p * ps);
    float mx[8], mn[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { mx[i] = -INFINITY; mn[i] = INFINITY; }
    if (pp >= 0) {
      const bf16_t* tile = c.k_pool + pp * c.stride_page + (int64_t)g * c.stride_head + cl * 8;
      for (int t0 = 0; t0 < ntok; t0 += 4) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          v[u] = ld16<true>(tile + min(t0 + u, ntok - 1) * kHeadDim);  // read once: streamed; a repeat is harmless
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float lo = bf16lo_to_f32(w[i]), hi = bf16hi_to_f32(w[i]);
            mx[2 * i] = fmaxf(mx[2 * i], lo); mn[2 * i] = fminf(mn[2 * i], lo);
            mx[2 * i + 1] = fmaxf(mx[2 * i + 1], hi); mn[2 * i + 1] = fminf(mn[2 * i + 1], hi);
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      // an absent page contributes neutral zeros
      const float a = pp >= 0 ? mx[i] : 0.f, z = pp >= 0 ? mn[i] : 0.f;
      tmax[(cl * 8 + i) * kSumPad + pl] = (bf16_t)(__float_as_uint(a) >> 16);
      tmin[(cl * 8 + i) * kSumPad + pl] = (bf16_t)(__float_as_uint(z) >> 16);
    }
  }
  __syncthreads();
  const int64_t row0 = (int64_t)unit * kHeadDim;
  for (int idx = threadIdx.x; idx < kHeadDim * kSumPages; idx += 256) {
    const int ch = idx / kSumPages, pl = idx % kSumPages;
    if (pl < npg) {
      const int64_t o = (row0 + ch) * c.pages_cap + p0 + pl;
      kmax[o] = tmax[ch * kSumPad + pl];
      kmin[o] = tmin[ch * kSumPad + pl];
    }
  }
}

hipError_t launch_page_summaries(const CacheView& c, bf16_t* kmax, bf16_t* kmin, int first_page,
                                 int n_pages, hipStream_t st) {
  int last = (n_pages < 0) ? c.pages_cap : first_page + n_pages;
  if (last > c.pages_cap) last = c.pages_cap;
  if (first_page >= last) return hipSuccess;
  dim3 grid((last - first_page + kSumPages - 1) / kSumPages, c.batch * c.n_kv_heads);
  hipLaunchKernelGGL(page_summaries_kernel, grid, dim3(256), 0, st, c, kmax, kmin, first_page, last);
  return hipGetLastError();
}

// One generated token per sequence: write its key row and value column into the tail page, fold the
// key into that page's summary, then bump the length.  One workgroup per sequence, one thread per
// (KV head, channel) where that fits, so that every load of the step is in flight at once; every
// thread reads the old length before the barrier that precedes the increment.
constexpr int kAppendThreads = 1024;
__global__ __launch_bounds__(kAppendThreads) void append_kv_kernel(CacheView c, const bf16_t* __restrict__ k_new,
                                                                   const bf16_t* __restrict__ v_new,
                                                                   bf16_t* __restrict__ kmax,
                                                                   bf16_t* __restrict__ kmin) {
  const int b = blockIdx.x;
  const int n = c.seq_lens[b];
  const int ps = c.page_size;
  const bool room = n < c.pages_cap * ps;
  if (room) {
    const int p = n / ps, slot = n % ps;
    const int64_t pp = phys_page(c, b, p);
    for (int idx = threadIdx.x; idx < c.n_kv_heads * kHeadDim; idx += blockDim.x) {
      const int g = idx / kHeadDim, ch = idx % kHeadDim;
      const int64_t src = ((int64_t)b * c.n_kv_heads + g) * kHeadDim + ch;
      const int64_t o = (((int64_t)b * c.n_kv_heads + g) * kHeadDim + ch) * c.pages_cap + p;
      const bf16_t kb = k_new[src], vb = v_new[src];
      const bf16_t old_max = kmax[o], old_min = kmin[o];
      if (pp >= 0) {
        const int64_t base = pp * c.stride_page + (int64_t)g * c.stride_head;
        c.k_pool[base + slot * kHeadDim + ch] = kb;
        c.v_pool[base + (c.v_token_major ? slot * kHeadDim + ch : ch * ps + slot)] = vb;
      }
      const float x = bf16_to_f32(kb);
      if (slot == 0 || x > bf16_to_f32(old_max)) kmax[o] = kb;
      if (slot == 0 || x < bf16_to_f32(old_min)) kmin[o] = kb;
    }
  }
  __syncthreads();
  if (room && threadIdx.x == 0) c.seq_lens[b] = n + 1;
}

hipError_t launch_append(const CacheView& c, const bf16_t* k_new, const bf16_t* v_new, bf16_t* kmax,
                         bf16_t* kmin, hipStream_t st) {
  int threads = c.n_kv_heads * kHeadDim;
  if (threads > kAppendThreads) threads = kAppendThreads;
  hipLaunchKernelGGL(append_kv_kernel, dim3(c.batch), dim3(threads), 0, st, c, k_new, v_new, kmax, kmin);
  return hipGetLastError();
}

// ---- RocketKV-MT (Section 3.5): the same two steps over a logical sequence ---------------------------
// Page p of the logical order holds logical tokens p*ps .. p*ps+ps-1, each at its own position of the
// cache, so a page is a gather of rows rather than a tile.  Same workgroup shape and LDS transpose as
// above; four row groups of 16 lanes take the page's tokens in turn.
__global__ __launch_bounds__(256) void page_summaries_indexed_kernel(CacheView c, LogicalView lv,
                                                                     bf16_t* __restrict__ kmax,
                                                                     bf16_t* __restrict__ kmin,
                                                                     int first_page, int last_page) {
  __shared__ bf16_t tmax[kHeadDim * kSumPad];
  __shared__ bf16_t tmin[kHeadDim * kSumPad];
  const int unit = blockIdx.y;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int ps = lv.page_size;
  int n = lv.n_indexed[b];
  if (n > lv.pages_cap * ps) n = lv.pages_cap * ps;
  const int P = (n + ps - 1) / ps;
  const int p0 = first_page + blockIdx.x * kSumPages;
  const int pend = min(min(p0 + kSumPages, last_page), P);
  if (p0 >= pend) return;
  const int npg = pend - p0;
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  const int tg = lane / 16, cl = lane % 16;
  const int32_t* idx = lv.token_index + (int64_t)unit * lv.pages_cap * ps;

  for (int pl = wave; pl < npg; pl += 4) {
    const int p = p0 + pl;
    const int ntok = min(ps, n - p * ps);
    float mx[8], mn[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { mx[i] = -INFINITY; mn[i] = INFINITY; }
    bool any = false;
    for (int t = tg; t < ntok; t += 4) {
      const int pos = idx[p * ps + t];
      const int sp = pos / c.page_size, ss = pos - sp * c.page_size;
      const int64_t pp = (pos >= 0 && sp < c.pages_cap) ? phys_page(c, b, sp) : -1;
      if (pp < 0) continue;  // a token whose cache page is absent contributes nothing
      any = true;
      const uint4 v = ld16<true>(c.k_pool + pp * c.stride_page + (int64_t)g * c.stride_head + ss * kHeadDim + cl * 8);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float lo = bf16lo_to_f32(w[i]), hi = bf16hi_to_f32(w[i]);
        mx[2 * i] = fmaxf(mx[2 * i], lo); mn[2 * i] = fminf(mn[2 * i], lo);
        mx[2 * i + 1] = fmaxf(mx[2 * i + 1], hi); mn[2 * i + 1] = fminf(mn[2 * i + 1], hi);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 16)); mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 32));
      mn[i] = fminf(mn[i], __shfl_xor(mn[i], 16)); mn[i] = fminf(mn[i], __shfl_xor(mn[i], 32));
    }
    any = __any(any);
    if (tg == 0) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float a = any ? mx[i] : 0.f, z = any ? mn[i] : 0.f;
        tmax[(cl * 8 + i) * kSumPad + pl] = (bf16_t)(__float_as_uint(a) >> 16);
        tmin[(cl * 8 + i) * kSumPad + pl] = (bf16_t)(__float_as_uint(z) >> 16);
      }
    }
  }
  __syncthreads();
  const int64_t row0 = (int64_t)unit * kHeadDim;
  for (int i = threadIdx.x; i < kHeadDim * kSumPages; i += 256) {
    const int ch = i / kSumPages, pl = i % kSumPages;
    if (pl < npg) {
      const int64_t o = (row0 + ch) * lv.pages_cap + p0 + pl;
      kmax[o] = tmax[ch * kSumPad + pl];
      kmin[o] = tmin[ch * kSumPad + pl];
    }
  }
}

hipError_t launch_page_summaries_indexed(const CacheView& c, const LogicalView& lv, bf16_t* kmax,
                                         bf16_t* kmin, int first_page, int n_pages, hipStream_t st) {
  int last = (n_pages < 0) ? lv.pages_cap : first_page + n_pages;
  if (last > lv.pages_cap) last = lv.pages_cap;
  if (first_page >= last) return hipSuccess;
  dim3 grid((last - first_page + kSumPages - 1) / kSumPages, c.batch * c.n_kv_heads);
  hipLaunchKernelGGL(page_summaries_indexed_kernel, grid, dim3(256), 0, st, c, lv, kmax, kmin, first_page,
                     last);
  return hipGetLastError();
}

// One generated token per sequence into the cache (position seq_lens[b]) and into the logical
// sequence (entry n_indexed[b] of every KV head's index row, logical tail page's summary).  One
// workgroup per sequence; both lengths are read by every thread before the barrier in front of
// their increment.
__global__ __launch_bounds__(kAppendThreads) void append_indexed_kernel(CacheView c, LogicalView lv,
                                                                       const bf16_t* __restrict__ k_new,
                                                                       const bf16_t* __restrict__ v_new,
                                                                       bf16_t* __restrict__ kmax,
                                                                       bf16_t* __restrict__ kmin) {
  const int b = blockIdx.x;
  const int pos = c.seq_lens[b];   // where the token goes in the cache
  const int j = lv.n_indexed[b];   // its place in the logical order
  const int ps = lv.page_size;
  const bool room = pos < c.pages_cap * c.page_size && j < lv.pages_cap * ps;
  if (room) {
    const int sp = pos / c.page_size, ss = pos % c.page_size;
    const int p = j / ps, slot = j % ps;
    const int64_t pp = phys_page(c, b, sp);
    for (int i = threadIdx.x; i < c.n_kv_heads * kHeadDim; i += blockDim.x) {
      const int g = i / kHeadDim, ch = i % kHeadDim;
      const int64_t unit = (int64_t)b * c.n_kv_heads + g;
      const int64_t src = unit * kHeadDim + ch;
      const int64_t o = (unit * kHeadDim + ch) * lv.pages_cap + p;
      const bf16_t kb = k_new[src], vb = v_new[src];
      const bf16_t old_max = kmax[o], old_min = kmin[o];
      if (pp >= 0) {
        const int64_t base = pp * c.stride_page + (int64_t)g * c.stride_head + ss * kHeadDim + ch;
        c.k_pool[base] = kb;
        c.v_pool[base] = vb;  // token-major V (checked on the host)
      }
      if (ch == 0) lv.token_index[unit * lv.pages_cap * ps + j] = pos;
      const float x = bf16_to_f32(kb);
      if (slot == 0 || x > bf16_to_f32(old_max)) kmax[o] = kb;
      if (slot == 0 || x < bf16_to_f32(old_min)) kmin[o] = kb;
    }
  }
  __syncthreads();
  if (room && threadIdx.x == 0) {
    c.seq_lens[b] = pos + 1;
    lv.n_indexed[b] = j + 1;
  }
}

hipError_t launch_append_indexed(const CacheView& c, const LogicalView& lv, const bf16_t* k_new,
                                 const bf16_t* v_new, bf16_t* kmax, bf16_t* kmin, hipStream_t st) {
  int threads = c.n_kv_heads * kHeadDim;
  if (threads > kAppendThreads) threads = kAppendThreads;
  hipLaunchKernelGGL(append_indexed_kernel, dim3(c.batch), dim3(threads), 0, st, c, lv, k_new, v_new, kmax,
                     kmin);
  return hipGetLastError();
}

}  // namespace rkv
