// HSA Step 2 (Algorithm 1 of arXiv 2502.14051, assignments i1, g, P, s1, i2): one workgroup per
// (sequence, KV head) picks the top-k1 channels of the group-summed |q|, streams only those rows of
// the channel-major page summaries (K_max where the group-summed q is >= 0, K_min otherwise),
// forms one fp32 score per page in LDS and keeps the top-kp pages with an exact 4-pass radix
// select.  Ties go to the lower index in both picks; the page list comes out ascending.
//
// Traffic: k1 rows of P bf16 values per unit, read as 16-byte runs of eight pages; everything else
// lives in LDS.  Summation order is fixed, so results are bit-reproducible run to run.
#include "common.h"

namespace rkv {

constexpr int kSelThreads = 256;

__device__ __forceinline__ uint32_t f32_order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger float <=> larger unsigned key
}

// exclusive prefix sum of one uint32 per thread over the 256-thread workgroup
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wsum /*[4]*/) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint32_t inc = wave_incl_scan(v);
  if (lane == kWave - 1) wsum[wave] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += wsum[w];
  __syncthreads();
  return base + inc - v;
}

__global__ __launch_bounds__(kSelThreads) void hsa_select_kernel(CacheView c, SelectArgs a) {
  extern __shared__ uint32_t keys[];  // [ceil8(P)] order keys of the page scores
  __shared__ __align__(16) float s_abs[kHeadDim];
  __shared__ float s_sum[kHeadDim];
  __shared__ int s_chan[kHeadDim];
  __shared__ float s_wgt[kHeadDim];
  __shared__ float partial[kSelThreads * 8];
  __shared__ __align__(16) uint32_t hist[4][256];  // one histogram per radix pass
  __shared__ int s_rank[kSelThreads];
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t sh_cnt0;

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int unit = blockIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int G = c.group, ps = c.page_size;
  const int n = c.seq_lens[b];
  int P = (n + ps - 1) / ps;
  if (P > c.pages_cap) P = c.pages_cap;
  int kp = pages_to_pick(n, ps, a.T);
  if (kp > P) kp = P;
  if (kp > a.row_len) kp = a.row_len;

  if (a.zero_counters && tid == 0) a.zero_counters[unit] = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) hist[i][tid] = 0;

  // -1 padding of the list rows beyond kp
  for (int i = kp + tid; i < a.row_len; i += kSelThreads) a.out_pages[(int64_t)unit * a.row_len + i] = -1;
  if (a.out_pages2)
    for (int i = kp + tid; i < a.row_len2; i += kSelThreads) a.out_pages2[(int64_t)unit * a.row_len2 + i] = -1;

  // ---- a[c] = sum_h |q|, s[c] = sum_h q (fp32, head order) -----------------------------------
  if (tid < kHeadDim) {
    float sa = 0.f, ss = 0.f;
    const bf16_t* qp = a.q + ((int64_t)b * c.n_q_heads + (int64_t)g * G) * kHeadDim + tid;
    bf16_t qv[kMaxGroup];
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) qv[h] = h < G ? qp[h * kHeadDim] : (bf16_t)0;
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) {
      if (h < G) {
        const float x = bf16_to_f32(qv[h]);
        sa += fabsf(x);
        ss += x;
      }
    }
    s_abs[tid] = sa;
    s_sum[tid] = ss;
  }
  __syncthreads();
  // ---- i1: rank by counting, compact ascending --------------------------------------------------
  // every thread ranks channel (tid mod 128) against one half of the channels, 4 at a time
  {
    const int ch = tid & (kHeadDim - 1), half = tid >> 7;
    const float mine = s_abs[ch];
    const float4* v4 = reinterpret_cast<const float4*>(s_abs + half * 64);
    int rank = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float4 v = v4[i];
      const int o = half * 64 + 4 * i;
      rank += (v.x > mine) || (v.x == mine && o + 0 < ch);
      rank += (v.y > mine) || (v.y == mine && o + 1 < ch);
      rank += (v.z > mine) || (v.z == mine && o + 2 < ch);
      rank += (v.w > mine) || (v.w == mine && o + 3 < ch);
    }
    s_rank[tid] = rank;
  }
  __syncthreads();
  bool sel = false;
  if (tid < kHeadDim) sel = s_rank[tid] + s_rank[tid + kHeadDim] < a.k1;
  const unsigned long long bal = __ballot(sel);
  if (tid == 0) sh_cnt0 = (uint32_t)__popcll(bal);
  __syncthreads();
  if (sel) {
    const int pos = __popcll(bal & ((1ull << lane) - 1ull)) + (wave == 1 ? (int)sh_cnt0 : 0);
    s_chan[pos] = tid;
    s_wgt[pos] = s_sum[tid];
    if (a.out_channels) a.out_channels[(int64_t)unit * a.k1 + pos] = tid;
  }
  __syncthreads();
  if (P == 0) return;

  // ---- s1: page scores ---------------------------------------------------------------------------
  const int n_oct = (P + 7) / 8;
  const int64_t rows = (int64_t)unit * kHeadDim;
  if (n_oct < kSelThreads) {
    int npow = 1;
    while (npow < n_oct) npow <<= 1;
    const int R = kSelThreads / npow;  // row groups summed separately, then in order
    const int r = tid / npow, o = tid % npow;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    if (o < n_oct) {
      // eight rows per batch: all loads of a batch are in flight before the first is used
      for (int j0 = r; j0 < a.k1; j0 += 8 * R) {
        uint4 v[8];
        float w[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int j = j0 + t * R;
          w[t] = 0.f;
          v[t] = make_uint4(0, 0, 0, 0);
          if (j < a.k1) {
            w[t] = s_wgt[j];
            const bf16_t* row = (w[t] >= 0.f ? a.kmax : a.kmin) + (rows + s_chan[j]) * c.pages_cap + o * 8;
            v[t] = *reinterpret_cast<const uint4*>(row);
          }
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const uint32_t x[4] = {v[t].x, v[t].y, v[t].z, v[t].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[2 * i] = fmaf(w[t], bf16lo_to_f32(x[i]), acc[2 * i]);
            acc[2 * i + 1] = fmaf(w[t], bf16hi_to_f32(x[i]), acc[2 * i + 1]);
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) partial[(r * npow + o) * 8 + i] = acc[i];
    __syncthreads();
    for (int p = tid; p < npow * 8; p += kSelThreads) {
      float s = 0.f;
      for (int rr = 0; rr < R; ++rr) s += partial[rr * npow * 8 + p];
      if (p < n_oct * 8) {
        if (p < P && a.out_scores) a.out_scores[(int64_t)unit * c.pages_cap + p] = s;
        if (p >= P) s = -INFINITY;
        else if (p >= P - a.n_recent) s = INFINITY;
        keys[p] = f32_order_key(s);
      }
    }
  } else {
    for (int o = tid; o < n_oct; o += kSelThreads) {
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
      for (int j0 = 0; j0 < a.k1; j0 += 8) {
        uint4 v[8];
        float w[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int j = j0 + t;
          w[t] = 0.f;
          v[t] = make_uint4(0, 0, 0, 0);
          if (j < a.k1) {
            w[t] = s_wgt[j];
            const bf16_t* row = (w[t] >= 0.f ? a.kmax : a.kmin) + (rows + s_chan[j]) * c.pages_cap + o * 8;
            v[t] = *reinterpret_cast<const uint4*>(row);
          }
        }
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const uint32_t x[4] = {v[t].x, v[t].y, v[t].z, v[t].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[2 * i] = fmaf(w[t], bf16lo_to_f32(x[i]), acc[2 * i]);
            acc[2 * i + 1] = fmaf(w[t], bf16hi_to_f32(x[i]), acc[2 * i + 1]);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int p = o * 8 + i;
        float s = acc[i];
        if (p < P && a.out_scores) a.out_scores[(int64_t)unit * c.pages_cap + p] = s;
        if (p >= P) s = -INFINITY;
        else if (p >= P - a.n_recent) s = INFINITY;
        keys[p] = f32_order_key(s);
      }
    }
  }
  __syncthreads();

  // ---- i2: exact kp-th largest key by 4 x 8-bit radix passes -------------------------------------
  uint32_t tau = 0, need_eq = (uint32_t)P;  // defaults select everything (kp == P)
  if (kp < P) {
    uint32_t prefix = 0, mask = 0, k = (uint32_t)kp;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      for (int p = tid; p < P; p += kSelThreads) {
        const uint32_t key = keys[p];
        if ((key & mask) == prefix) atomicAdd(&hist[pass][(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      // every wavefront finds the bucket holding the k-th largest on its own (no broadcast needed):
      // lane L owns bins 4(63-L)..4(63-L)+3, so a prefix sum over lanes counts the keys in higher bins
      const int b0 = 4 * (kWave - 1 - lane);
      const uint4 h = *reinterpret_cast<const uint4*>(&hist[pass][b0]);
      const uint32_t s3 = h.w, s2 = h.z + s3, s1 = h.y + s2, s0 = h.x + s1;  // suffix sums inside the lane
      const uint32_t above = wave_incl_scan(s0) - s0;                          // keys in bins of lower lanes
      const uint32_t in[4] = {above + s0, above + s1, above + s2, above + s3};
      const uint32_t hc[4] = {h.x, h.y, h.z, h.w};
      int found = -1;
      uint32_t newk = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t exc = in[j] - hc[j];
        if (exc < k && k <= in[j]) {
          found = b0 + j;
          newk = k - exc;
        }
      }
      const unsigned long long who = __ballot(found >= 0);
      const int src = __ffsll((long long)who) - 1;
      const uint32_t bucket = (uint32_t)__builtin_amdgcn_readlane(found, src);
      k = (uint32_t)__builtin_amdgcn_readlane((int)newk, src);
      prefix |= bucket << shift;
      mask |= 0xffu << shift;
    }
    tau = prefix;
    need_eq = k;
  }

  // ---- emit ascending: every key > tau, plus the first need_eq keys == tau -----------------------
  const int ipt = (P + kSelThreads - 1) / kSelThreads;
  const int lo = min(P, tid * ipt), hi = min(P, lo + ipt);
  uint32_t cnt = 0;  // low 16 bits: keys > tau, high 16 bits: keys == tau
  for (int p = lo; p < hi; ++p) {
    const uint32_t key = keys[p];
    cnt += (key > tau) ? 1u : 0u;
    cnt += (key == tau) ? 0x10000u : 0u;
  }
  const uint32_t before = block_excl_scan(cnt, wsum);
  uint32_t gt = before & 0xffffu, eq = before >> 16;
  for (int p = lo; p < hi; ++p) {
    const uint32_t key = keys[p];
    bool take = key > tau;
    if (key == tau) {
      take = eq < need_eq;
      ++eq;
    }
    if (take) {
      const uint32_t eq_taken = (key == tau) ? eq - 1 : min(eq, need_eq);
      const uint32_t pos = gt + eq_taken;
      if ((int)pos < kp) {
        a.out_pages[(int64_t)unit * a.row_len + pos] = p;
        if (a.out_pages2 && (int)pos < a.row_len2) a.out_pages2[(int64_t)unit * a.row_len2 + pos] = p;
      }
    }
    if (key > tau) ++gt;
  }
}

hipError_t launch_hsa_select(const CacheView& c, const SelectArgs& a, hipStream_t st) {
  const size_t smem = (size_t)((c.pages_cap + 7) / 8 * 8) * sizeof(uint32_t);
  hipLaunchKernelGGL(hsa_select_kernel, dim3(c.batch * c.n_kv_heads), dim3(kSelThreads), smem, st,
                     c, a);
  return hipGetLastError();
}

}  // namespace rkv
