// HSA Step 3 (Algorithm 1 of arXiv 2502.14051, y = attn(q, K[i2], V[i2])) and the Full-KV baseline of
// Table 1: exact GQA decode attention over a list of 16-token pages, split over workgroups along the
// list, with online softmax and a last-arriver merge of the split partials.
//
// The work is a stream of 4 KiB K tiles and 4 KiB V tiles per page and is HBM-bound; the arithmetic
// (G flop per byte plus the softmax) would not fit the vector ALUs beside the stream, so both
// contractions run on the matrix cores with the query heads of the group padded to one 16-wide tile:
//
//   S[token][head]   = K[token][:] . Q[head][:]       A = K tile (rows: 16 tokens), B = Q^T
//   O^T[chan][head] += V^T[chan][token] . P[token][head]   A = V tile (rows: 16 channels), B = P
//
// Both products have the head index as the MFMA column, so a lane owns one head throughout: its
// S values, running max / sum and O accumulators never need to move between lanes.  The V pool is
// channel-major inside a page precisely so that the contraction index (tokens) is contiguous per lane.
// A 16x16x32 MFMA contracts 32 tokens: two pages per step, lane group kg contributing tokens
// 4kg..4kg+3 of each, which is exactly how the S tiles come out of the first product.
#include "common.h"

namespace rkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kPartialStride = kHeadDim + 2;  // O[128], running max (log2 domain), running sum
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;

union Frag {
  uint4 u;
  bf16x8 v;
};

struct AttendArgs {
  const bf16_t* q;
  const int32_t* pages;  // NULL = identity list
  int row_len;           // entries per unit in `pages` (or pages_cap for identity)
  bf16_t* out;
  float* out_lse;
  float* partial;        // [units][n_split][G][kPartialStride]
  uint32_t* counters;    // [units]
  int n_split, chunk;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

__global__ __launch_bounds__(kAttnThreads) void attend_mfma_kernel(CacheView c, AttendArgs a) {
  __shared__ float sO[kAttnWaves][kMaxGroup][kHeadDim];
  __shared__ float sM[kAttnWaves][kMaxGroup];
  __shared__ float sL[kAttnWaves][kMaxGroup];
  __shared__ int s_last;

  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int unit = blockIdx.y, split = blockIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int G = c.group;
  const int n = c.seq_lens[b];
  int P = (n + kAttnPage - 1) / kAttnPage;
  if (P > c.pages_cap) P = c.pages_cap;

  // Q as the B operand of the first product: lane (head hn, group kg) holds channels j*32+kg*8..+7
  Frag qf[4];
  if (hn < G) {
    const bf16_t* qp = a.q + ((int64_t)b * c.n_q_heads + (int64_t)g * G + hn) * kHeadDim + kg * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) qf[j].u = *reinterpret_cast<const uint4*>(qp + j * 32);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j) qf[j].u = make_uint4(0, 0, 0, 0);
  }

  f32x4 O[8];
#pragma unroll
  for (int cb = 0; cb < 8; ++cb) O[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = kNegBig, l = 0.f;
  const float sc = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)

  const int e_begin = split * a.chunk;
  const int e_end = min(e_begin + a.chunk, a.row_len);
  const int32_t* list = a.pages ? a.pages + (int64_t)unit * a.row_len : nullptr;
  const int64_t head_off = (int64_t)g * c.stride_head;

  for (int e = e_begin + 2 * wave; e < e_end; e += 2 * kAttnWaves) {
    int id[2];
    int64_t pp[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      int v = -1;
      if (e + x < e_end) v = list ? list[e + x] : e + x;
      if (v < 0 || v >= P) v = -1;
      v = __builtin_amdgcn_readfirstlane(v);
      id[x] = v;
      pp[x] = v >= 0 ? phys_page(c, b, v) : -1;
      if (pp[x] < 0) id[x] = -1;
    }
    if (id[0] < 0 && id[1] < 0) continue;

    Frag kf[2][4];
    uint2 vf[2][8];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      if (id[x] >= 0) {
        const bf16_t* kt = c.k_pool + pp[x] * c.stride_page + head_off + hn * kHeadDim + kg * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) kf[x][j].u = *reinterpret_cast<const uint4*>(kt + j * 32);
        const bf16_t* vt = c.v_pool + pp[x] * c.stride_page + head_off + hn * kAttnPage + kg * 4;
#pragma unroll
        for (int cb = 0; cb < 8; ++cb)
          vf[x][cb] = *reinterpret_cast<const uint2*>(vt + cb * 16 * kAttnPage);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) kf[x][j].u = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) vf[x][cb] = make_uint2(0, 0);
      }
    }

    // S tiles: s[x][r] = logit of token id[x]*16 + 4kg + r for head hn
    float s[2][4];
    float mx = kNegBig;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[x][j].v, qf[j].v, acc, 0, 0, 0);
      const int tok0 = id[x] * kAttnPage + kg * 4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool ok = id[x] >= 0 && tok0 + r < n;
        s[x][r] = ok ? acc[r] * sc : -INFINITY;
        mx = fmaxf(mx, s[x][r]);
      }
      // a partial tail page may hold anything beyond the sequence end: keep it out of P.V
      if (id[x] >= 0 && id[x] * kAttnPage + kAttnPage > n) {
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
          uint32_t w0 = vf[x][cb].x, w1 = vf[x][cb].y;
          if (tok0 + 0 >= n) w0 &= 0xffff0000u;
          if (tok0 + 1 >= n) w0 &= 0x0000ffffu;
          if (tok0 + 2 >= n) w1 &= 0xffff0000u;
          if (tok0 + 3 >= n) w1 &= 0x0000ffffu;
          vf[x][cb] = make_uint2(w0, w1);
        }
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    float p[2][4], psum = 0.f;
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[x][r] = fast_exp2(s[x][r] - m_new);
        psum += p[x][r];
      }
    l = l * alpha + psum;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) O[cb] *= alpha;
    Frag pf;
    pf.u = make_uint4(pack_bf16x2(p[0][0], p[0][1]), pack_bf16x2(p[0][2], p[0][3]),
                      pack_bf16x2(p[1][0], p[1][1]), pack_bf16x2(p[1][2], p[1][3]));
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      Frag vv;
      vv.u = make_uint4(vf[0][cb].x, vf[0][cb].y, vf[1][cb].x, vf[1][cb].y);
      O[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vv.v, pf.v, O[cb], 0, 0, 0);
    }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);

  // ---- merge the four waves through LDS --------------------------------------------------------
  if (hn < G) {
#pragma unroll
    for (int cb = 0; cb < 8; ++cb)
      *reinterpret_cast<float4*>(&sO[wave][hn][cb * 16 + kg * 4]) =
          make_float4(O[cb][0], O[cb][1], O[cb][2], O[cb][3]);
    if (kg == 0) {
      sM[wave][hn] = m;
      sL[wave][hn] = l;
    }
  }
  __syncthreads();
  const int ch = tid % kHeadDim;
  const int64_t out_base = ((int64_t)b * c.n_q_heads + (int64_t)g * G) * kHeadDim;
  for (int h = tid / kHeadDim; h < G; h += kAttnThreads / kHeadDim) {
    float M = sM[0][h];
#pragma unroll
    for (int w = 1; w < kAttnWaves; ++w) M = fmaxf(M, sM[w][h]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      const float f = fast_exp2(sM[w][h] - M);
      num += f * sO[w][h][ch];
      den += f * sL[w][h];
    }
    if (a.n_split == 1) {
      a.out[out_base + h * kHeadDim + ch] = f32_to_bf16(den > 0.f ? num / den : 0.f);
      if (ch == 0 && a.out_lse)
        a.out_lse[(int64_t)b * c.n_q_heads + g * G + h] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
    } else {
      float* pr = a.partial + (((int64_t)unit * a.n_split + split) * G + h) * kPartialStride;
      pr[ch] = num;
      if (ch == 0) {
        pr[kHeadDim] = M;
        pr[kHeadDim + 1] = den;
      }
    }
  }
  if (a.n_split == 1) return;

  // ---- last workgroup of the unit merges the split partials --------------------------------------
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const uint32_t old = atomicAdd(&a.counters[unit], 1u);
    s_last = (old == (uint32_t)a.n_split - 1u);
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  for (int h = tid / kHeadDim; h < G; h += kAttnThreads / kHeadDim) {
    const float* pr = a.partial + ((int64_t)unit * a.n_split * G + h) * kPartialStride;
    const int64_t sstride = (int64_t)G * kPartialStride;
    float M = kNegBig;
    for (int s2 = 0; s2 < a.n_split; ++s2)
      M = fmaxf(M, __hip_atomic_load(pr + s2 * sstride + kHeadDim, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    float num = 0.f, den = 0.f;
    for (int s2 = 0; s2 < a.n_split; ++s2) {
      const float ms = __hip_atomic_load(pr + s2 * sstride + kHeadDim, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const float ls = __hip_atomic_load(pr + s2 * sstride + kHeadDim + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const float os = __hip_atomic_load(pr + s2 * sstride + ch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const float f = fast_exp2(ms - M);
      num += f * os;
      den += f * ls;
    }
    a.out[out_base + h * kHeadDim + ch] = f32_to_bf16(den > 0.f ? num / den : 0.f);
    if (ch == 0 && a.out_lse)
      a.out_lse[(int64_t)b * c.n_q_heads + g * G + h] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
  }
  if (tid == 0) a.counters[unit] = 0;  // leave the counter ready for the next call
}

__global__ void zero_u32_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

static int g_target_wgs = 512;    // workgroups aimed for along (units x splits)
static int g_min_chunk = 8;       // page-list entries per workgroup, multiple of 8

void tune_attend(int target_wgs, int min_chunk) {
  if (target_wgs > 0) g_target_wgs = target_wgs;
  if (min_chunk > 0) g_min_chunk = (min_chunk + 7) / 8 * 8;
}

AttendPlan plan_attend(const CacheView& c, int row_len) {
  AttendPlan p;
  const int units = c.batch * c.n_kv_heads;
  int want = (g_target_wgs + units - 1) / units;
  const int max_split = (row_len + g_min_chunk - 1) / g_min_chunk;
  if (want > max_split) want = max_split;
  if (want < 1) want = 1;
  int chunk = (row_len + want - 1) / want;
  chunk = (chunk + 7) / 8 * 8;
  if (chunk < g_min_chunk) chunk = g_min_chunk;
  p.chunk = chunk;
  p.n_split = (row_len + chunk - 1) / chunk;
  if (p.n_split < 1) p.n_split = 1;
  size_t off = 0;
  p.counter_off = off;
  off += ((size_t)units * sizeof(uint32_t) + 255) / 256 * 256;
  p.partial_off = off;
  off += ((size_t)units * p.n_split * c.group * kPartialStride * sizeof(float) + 255) / 256 * 256;
  p.total_bytes = off;
  return p;
}

hipError_t launch_attend(const CacheView& c, const bf16_t* q, const int32_t* pages, int row_len,
                         bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                         hipStream_t st) {
  const int units = c.batch * c.n_kv_heads;
  AttendArgs a;
  a.q = q;
  a.pages = pages;
  a.row_len = row_len;
  a.out = out;
  a.out_lse = out_lse;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + plan.partial_off);
  a.counters = reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + plan.counter_off);
  a.n_split = plan.n_split;
  a.chunk = plan.chunk;
  if (plan.n_split > 1) {
    hipLaunchKernelGGL(zero_u32_kernel, dim3((units + 255) / 256), dim3(256), 0, st, a.counters, units);
  }
  hipLaunchKernelGGL(attend_mfma_kernel, dim3(plan.n_split, units), dim3(kAttnThreads), 0, st, c, a);
  return hipGetLastError();
}

}  // namespace rkv
