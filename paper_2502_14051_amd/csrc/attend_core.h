// HSA Step 3 (Algorithm 1 of arXiv 2502.14051, y = attn(q, K[i2], V[i2])) and the Full-KV baseline of
// Table 1: exact GQA decode attention over a list of 16-token pages, split over workgroups along the
// list, with online softmax and a last-arriver merge of the split partials.
//
// The work is a stream of 4 KiB K tiles and 4 KiB V tiles per page and is HBM-bound; the arithmetic
// (G flop per byte plus the softmax) would not fit the vector ALUs beside the stream, so both
// contractions run on the matrix cores with the query heads of the group padded to one 16-wide tile:
//
//   S[token][head]   = K[token][:] . Q[head][:]            A = K tile (rows: 16 tokens), B = Q^T
//   O^T[chan][head] += V^T[chan][token] . P[token][head]   A = V tile (rows: 16 channels), B = P
//
// Both products have the head index as the MFMA column, so a lane owns one head throughout: its
// S values, running max / sum and O accumulators never move between lanes.  The V pool is
// channel-major inside a page precisely so that the contraction index (tokens) is contiguous per lane.
// A 16x16x32 MFMA contracts 32 tokens: two pages per step, lane group kg contributing tokens
// 4kg..4kg+3 of each, which is exactly how the S tiles come out of the first product.
//
// Latency matters as much as bandwidth here (a layer moves only tens of MB): a wavefront reads the
// page ids of its whole share with one load and requests a page pair's 16 KiB in one go (one pair in
// flight per wavefront, the other wavefronts of the SIMD cover its softmax step), and the split
// partials are handed over with write-through stores, an explicit wait for their acknowledgement and
// a relaxed device-scope counter instead of cache-flushing fences.
#pragma once

#include "common.h"

namespace rkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kPartialStride = kHeadDim + 2;  // O[128], running max (log2 domain), running sum
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// K and V tiles are read once per launch.  Loading them with the streaming hint keeps them out of
// the way in the caches and measures 10-13 % faster on a plain read of a large buffer (7.0 against
// 6.2 TB/s on MI355X).  V tiles always take it (every load instruction of a wavefront covers whole
// cache lines of a V tile).  A K load instruction covers half of each line it touches, the next one
// the other half; with the hint that measured slower for dense reads, for token-major caches and for
// small launches, and faster only for large gathers of 16-token pages, so the host picks the kernel
// variant with it (STREAM_K) there.
template <class T>
__device__ __forceinline__ T ld_stream(const bf16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
}
template <class T>
__device__ __forceinline__ T ld_plain(const bf16_t* p) {
  return *reinterpret_cast<const T*>(p);
}
// gathers of at least this many bytes of keys per launch use the streaming hint for K
constexpr int64_t kStreamKBytes = 24ll << 20;
inline bool wants_stream_k(const CacheView& c, int row_len) {
  return (int64_t)c.batch * c.n_kv_heads * row_len * kAttnPage * kHeadDim * (int64_t)sizeof(bf16_t) >= kStreamKBytes;
}

// Fragments are plain ext-vector values (no unions or structs of arrays): anything the compiler
// cannot split into scalars ends up in scratch memory, which costs far more than the arithmetic.
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

struct AttendArgs {
  const bf16_t* q;
  const int32_t* pages;  // NULL = identity list
  int row_len;           // entries per unit in `pages` (or pages_cap for identity)
  bf16_t* out;
  float* out_lse;
  float* partial;        // [units][n_csplit][n_split][G][kPartialStride]
  uint32_t* counters;    // [units][n_csplit]
  int n_split, chunk, per_wave;
  int n_csplit;          // workgroups a unit's output channels are divided between (1 or 2)
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two fp32 -> packed bf16, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  const bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<const uint32_t*>(&r);
}

__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Online-softmax update and second product for the NP page pairs of one round: `acc` holds the raw
// logits S[token][head] (masked entries -inf), `vf` the V operand (lane: channel cb*16+hn, tokens
// 4kg..4kg+3 of each page).  One max / rescale per round, the logit scale folded into the exponent's
// FMA, hardware bf16 packing.
template <int NP, int CB>
__device__ __forceinline__ void softmax_pv(f32x4 (&acc)[NP][2], u32x2 (&vf)[NP][2][CB],
                                           f32x4 (&O)[CB], float& m, float& l, bool have_acc, float sc) {
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < NP; ++u)
#pragma unroll
    for (int x = 0; x < 2; ++x)
      mx = fmaxf(fmaxf(mx, fmaxf(acc[u][x][0], acc[u][x][1])), fmaxf(acc[u][x][2], acc[u][x][3]));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx * sc);  // running max in the scaled log2 domain
  if (have_acc) {
    const float alpha = fast_exp2(m - m_new);
    l *= alpha;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) O[cb] *= alpha;
    }
  }
  m = m_new;
  float psum = 0.f;
  u32x4 pf[NP];
#pragma unroll
  for (int u = 0; u < NP; ++u) {
    float p[2][4];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[x][r] = fast_exp2(fmaf(acc[u][x][r], sc, -m_new));
        psum += p[x][r];
      }
    pf[u] = (u32x4){pack_bf16x2(p[0][0], p[0][1]), pack_bf16x2(p[0][2], p[0][3]),
                    pack_bf16x2(p[1][0], p[1][1]), pack_bf16x2(p[1][2], p[1][3])};
  }
  l += psum;
#pragma unroll
  for (int u = 0; u < NP; ++u)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const u32x4 vv = {vf[u][0][cb].x, vf[u][0][cb].y, vf[u][1][cb].x, vf[u][1][cb].y};
      O[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), as_bf16x8(pf[u]), O[cb], 0, 0, 0);
    }
}

// Online-softmax step over the NP page pairs of one round.  The vector ALUs issue one wave64
// instruction per four cycles and share the SIMD with the next wave, so instruction count is what
// this step is built around: one max / rescale per round instead of per page, the logit scale folded
// into the exponent's FMA, hardware bf16 packing, and the per-token masks compiled only into the
// MASK variant, which a round takes when it holds an absent page or the sequence's partial tail page.
// `cs`: which share of the output channels this workgroup computes (channel blocks cs*CB .. cs*CB+CB-1).
template <int NP, bool MASK, int CB>
__device__ __forceinline__ void softmax_round(u32x4 (&kf)[NP][2][4], u32x2 (&vf)[NP][2][CB],
                                              const int (&ids)[NP][2], const u32x4 (&qf)[4],
                                              f32x4 (&O)[CB], float& m, float& l, bool have_acc, int n,
                                              int hn, int kg, float sc, const TailPatch& tp, int cs) {
  if (MASK && tp.page >= 0) {
    // the page receiving a token in this launch: take that token's key row and value column from the
    // staged copies rather than from memory
#pragma unroll
    for (int u = 0; u < NP; ++u)
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        if (ids[u][x] == tp.page) {
          if (hn == tp.slot) {
#pragma unroll
            for (int j = 0; j < 4; ++j) kf[u][x][j] = *reinterpret_cast<const u32x4*>(tp.knew + j * 32 + kg * 8);
          }
          if (kg == (tp.slot >> 2)) {
            const int e = tp.slot & 3;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
              const uint32_t val = tp.vnew[(cs * CB + cb) * 16 + hn];
              uint32_t w0 = vf[u][x][cb].x, w1 = vf[u][x][cb].y;
              if (e == 0) w0 = (w0 & 0xffff0000u) | val;
              if (e == 1) w0 = (w0 & 0x0000ffffu) | (val << 16);
              if (e == 2) w1 = (w1 & 0xffff0000u) | val;
              if (e == 3) w1 = (w1 & 0x0000ffffu) | (val << 16);
              vf[u][x][cb] = (u32x2){w0, w1};
            }
          }
        }
      }
  }
  f32x4 acc[NP][2];
#pragma unroll
  for (int u = 0; u < NP; ++u)
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      acc[u][x] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[u][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[u][x][j]), as_bf16x8(qf[j]),
                                                            acc[u][x], 0, 0, 0);
    }
  if (MASK) {
#pragma unroll
    for (int u = 0; u < NP; ++u)
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const int tok0 = ids[u][x] * kAttnPage + kg * 4;
        const bool gone = ids[u][x] < 0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (gone || tok0 + r >= n) acc[u][x][r] = -INFINITY;
        // what lies in an absent page, or beyond the sequence end in the tail page, may be anything:
        // its probability is zero, but 0 x NaN is not, so it is cleared out of the V operand too
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          uint32_t w0 = vf[u][x][cb].x, w1 = vf[u][x][cb].y;
          if (gone || tok0 + 0 >= n) w0 &= 0xffff0000u;
          if (gone || tok0 + 1 >= n) w0 &= 0x0000ffffu;
          if (gone || tok0 + 2 >= n) w1 &= 0xffff0000u;
          if (gone || tok0 + 3 >= n) w1 &= 0x0000ffffu;
          vf[u][x][cb] = (u32x2){w0, w1};
        }
      }
  }
  softmax_pv<NP, CB>(acc, vf, O, m, l, have_acc, sc);
}

// Merges of one workgroup's result: the wavefronts' (O, max, sum) through LDS, then, when the unit's
// list is split over several workgroups, the hand-over of the partial and the last arriver's merge of
// all of them.  `O`, `m`, `l` are the lane's online-softmax state with `l` already summed over the four
// token groups; `smem` holds WAVES*G*(CB*16+2) floats, `s_last` one int.  The workgroup owns output
// channels cs*CB*16 .. +CB*16-1 of the unit; workgroups with different `cs` never meet.
template <int WAVES, int CB = 8>
__device__ __forceinline__ void attend_merge(const CacheView& c, const AttendArgs& a, int unit, int split, int cs,
                                             const f32x4 (&O)[CB], float m, float l, float* smem,
                                             int* s_last, int b, int g) {
  constexpr int kThreads = WAVES * kWave;
  constexpr int CW = CB * 16;  // output channels of this workgroup
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int G = c.group;
  float* sO = smem;
  float* sM = smem + WAVES * G * CW;
  float* sL = sM + WAVES * G;

  // ---- merge the waves through LDS ---------------------------------------------------------------
  if (hn < G) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
      *reinterpret_cast<float4*>(&sO[(wave * G + hn) * CW + cb * 16 + kg * 4]) =
          make_float4(O[cb][0], O[cb][1], O[cb][2], O[cb][3]);
    if (kg == 0) {
      sM[wave * G + hn] = m;
      sL[wave * G + hn] = l;
    }
  }
  __syncthreads();
  RKV_STAMP(8);
  const int64_t out_base = ((int64_t)b * c.n_q_heads + (int64_t)g * G) * kHeadDim + cs * CW;
  const int64_t group = (int64_t)unit * a.n_csplit + cs;  // the workgroups that merge with each other
  for (int idx = tid; idx < G * CW; idx += kThreads) {
    const int h = idx / CW, ch = idx % CW;
    float M = sM[h];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) M = fmaxf(M, sM[w * G + h]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float f = fast_exp2(sM[w * G + h] - M);
      num += f * sO[(w * G + h) * CW + ch];
      den += f * sL[w * G + h];
    }
    if (a.n_split == 1) {
      a.out[out_base + h * kHeadDim + ch] = f32_to_bf16(den > 0.f ? num / den : 0.f);
      if (ch == 0 && cs == 0 && a.out_lse)
        a.out_lse[(int64_t)b * c.n_q_heads + g * G + h] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
    } else {
      // write-through stores: visible device-wide once acknowledged, no cache flush needed
      float* pr = a.partial + ((group * a.n_split + split) * G + h) * kPartialStride;
      st_agent(pr + ch, num);
      if (ch == 0) {
        st_agent(pr + kHeadDim, M);
        st_agent(pr + kHeadDim + 1, den);
      }
    }
  }
  if (a.n_split == 1) return;

  // ---- last workgroup of the group merges the split partials -------------------------------------
  RKV_STAMP(9);
  drain_stores();   // this thread's partials (and whatever else it stored) have been acknowledged ...
  __syncthreads();  // ... and so have every other thread's, before thread 0 reports
  if (tid == 0) {
    const uint32_t old = __hip_atomic_fetch_add(&a.counters[group], 1u, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
    *s_last = (old == (uint32_t)a.n_split - 1u);
  }
  __syncthreads();
  RKV_STAMP(10);
  if (!*s_last) return;
  for (int idx = tid; idx < G * CW; idx += kThreads) {
    const int h = idx / CW, ch = idx % CW;
    const float* pr = a.partial + (group * a.n_split * G + h) * kPartialStride;
    const int64_t sstride = (int64_t)G * kPartialStride;
    float M = kNegBig, num = 0.f, den = 0.f;
    // eight splits per batch, every load of a batch in flight before the first use
    for (int s0 = 0; s0 < a.n_split; s0 += 8) {
      float ms[8], ls[8], os[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const bool ok = s0 + t < a.n_split;
        const float* ps = pr + (ok ? s0 + t : s0) * sstride;
        ms[t] = ld_agent(ps + kHeadDim);
        ls[t] = ld_agent(ps + kHeadDim + 1);
        os[t] = ld_agent(ps + ch);
        if (!ok) { ms[t] = kNegBig; ls[t] = 0.f; os[t] = 0.f; }
      }
      float Mb = M;
#pragma unroll
      for (int t = 0; t < 8; ++t) Mb = fmaxf(Mb, ms[t]);
      const float fo = fast_exp2(M - Mb);
      num *= fo;
      den *= fo;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float f = fast_exp2(ms[t] - Mb);
        num += f * os[t];
        den += f * ls[t];
      }
      M = Mb;
    }
    a.out[out_base + h * kHeadDim + ch] = f32_to_bf16(den > 0.f ? num / den : 0.f);
    if (ch == 0 && cs == 0 && a.out_lse)
      a.out_lse[(int64_t)b * c.n_q_heads + g * G + h] = den > 0.f ? (M + log2f(den)) * kLn2 : -INFINITY;
  }
  if (tid == 0) __hip_atomic_store(&a.counters[group], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  RKV_STAMP(11);
}

// The attention of one workgroup: its share (`split`) of the page list of `unit`, then the merges.
// `list` points at the unit's page ids (global memory or LDS; null = identity), `smem` at
// WAVES*G*130 floats of LDS for the wave merge, `s_last` at one LDS int.
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};

// `after_stream` runs once per thread after the last K/V tile has been consumed and before the
// merges: a place for stores whose latency should hide under the merge.
//
// CB < 8: the unit's output channels are divided between 8 / CB workgroups (`cs` says which share is
// this one's) instead of, or on top of, its page list.  Each of them reads every K tile of its pages
// (the second reader of a tile finds it in the L2 of the XCD the unit's workgroups share, which is why
// those loads are plain ones), forms the same logits and softmax weights, and takes only its own
// channel blocks of the V tiles: the same HBM bytes, but workgroups that never have to meet, so a
// unit split two ways needs no hand-over of partials through memory at all.
//
// `last_round` runs once per thread right after the loads of its last round have been requested (or
// before `after_stream` if it has no round at all): a place for a memory operation whose answer
// should travel with those loads instead of being waited for on its own.
template <int WAVES, int NP, bool STREAM_K, int CB = 8, typename Hook = NoHook, typename Hook2 = NoHook>
__device__ __forceinline__ void attend_block(const CacheView& c, const AttendArgs& a, int unit, int split, int cs,
                                             int n, const int32_t* list, float* smem, int* s_last,
                                             const TailPatch& tp, const Hook& after_stream = Hook(),
                                             const Hook2& last_round = Hook2()) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int G = c.group;
  int P = (n + kAttnPage - 1) / kAttnPage;
  if (P > c.pages_cap) P = c.pages_cap;

  // this wave's share of the list
  const int e_begin = split * a.chunk;
  const int e_end = min(e_begin + a.chunk, a.row_len);
  const int wb = e_begin + wave * a.per_wave;
  const int we = min(wb + a.per_wave, e_end);

  // first batch of page ids: issued before anything else
  int my_id = -1;
  if (wb + lane < we) my_id = list ? list[wb + lane] : wb + lane;

  // Q as the B operand of the first product: lane (head hn, group kg) holds channels j*32+kg*8..+7
  u32x4 qf[4];
  {
    const bf16_t* qp = a.q + ((int64_t)b * c.n_q_heads + (int64_t)g * G + (hn < G ? hn : 0)) * kHeadDim + kg * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      qf[j] = *reinterpret_cast<const u32x4*>(qp + j * 32);
      if (hn >= G) qf[j] = (u32x4){0u, 0u, 0u, 0u};
    }
  }

  f32x4 O[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) O[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = kNegBig, l = 0.f;
  bool have_acc = false;
  const float sc = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)
  // lane-dependent part of every tile address
  const bf16_t* k_lane = c.k_pool + (int64_t)g * c.stride_head + hn * kHeadDim + kg * 8;
  const bf16_t* v_lane = c.v_pool + (int64_t)g * c.stride_head + (cs * CB * 16 + hn) * kAttnPage + kg * 4;

  for (int base = wb; base < we; base += kWave) {
    if (base != wb) {
      my_id = -1;
      if (base + lane < we) my_id = list ? list[base + lane] : base + lane;
    }
    if (my_id >= P) my_id = -1;
    int64_t my_pp = my_id >= 0 ? phys_page(c, b, my_id) : -1;
    if (my_pp < 0) my_id = -1;
    // element offset of this lane's page (an absent page reads page 0 and is masked out)
    const int64_t my_off = (my_id >= 0 ? my_pp : 0) * c.stride_page;
    const unsigned long long special =
        __ballot(my_id < 0 || my_id * kAttnPage + kAttnPage > n || my_id == tp.page);
    const int cnt = min(kWave, we - base);
    const int npairs = (cnt + 1) / 2;

    // NP pairs per round: all their loads go out back to back (K tiles first, the first product
    // needs them first), then one softmax step consumes them.  Nothing is carried between rounds in
    // registers; the other wavefronts of the SIMD cover the gap.
    for (int i = 0; i < npairs; i += NP) {
      u32x4 kf[NP][2][4];
      u32x2 vf[NP][2][CB];
      int ids[NP][2];
      const bf16_t* vt[NP][2];
      const int e0 = __builtin_amdgcn_readfirstlane(2 * i);
#pragma unroll
      for (int u = 0; u < NP; ++u)
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          const int e = (e0 + 2 * u + x) & (kWave - 1);
          ids[u][x] = 2 * (i + u) + x < kWave ? __builtin_amdgcn_readlane(my_id, e) : -1;
          const int64_t off = ((int64_t)__builtin_amdgcn_readlane((int)(my_off >> 32), e) << 32) |
                              (uint32_t)__builtin_amdgcn_readlane((int)(my_off & 0xffffffff), e);
          const bf16_t* kt = k_lane + off;
          vt[u][x] = v_lane + off;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            kf[u][x][j] = STREAM_K ? ld_stream<u32x4>(kt + j * 32) : ld_plain<u32x4>(kt + j * 32);
        }
#pragma unroll
      for (int u = 0; u < NP; ++u)
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
          for (int cb = 0; cb < CB; ++cb)
            vf[u][x][cb] = ld_stream<u32x2>(vt[u][x] + cb * 16 * kAttnPage);
      if (base + kWave >= we && i + NP >= npairs) last_round();
      const bool masked = ((special >> e0) & ((1ull << (2 * NP)) - 1ull)) != 0ull || e0 + 2 * NP > kWave;
      if (!masked)
        softmax_round<NP, false, CB>(kf, vf, ids, qf, O, m, l, have_acc, n, hn, kg, sc, tp, cs);
      else
        softmax_round<NP, true, CB>(kf, vf, ids, qf, O, m, l, have_acc, n, hn, kg, sc, tp, cs);
      if (!have_acc) RKV_STAMP(6);
      have_acc = true;
    }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  RKV_STAMP(7);
  if (wb >= we) last_round();
  after_stream();
  attend_merge<WAVES, CB>(c, a, unit, split, cs, O, m, l, smem, s_last, b, g);
}

}  // namespace rkv
