// Stage 1 of RocketKV (Section 3.3 of arXiv 2502.14051; window / kernel sizes from Appendix A.3):
// GQA-aware SnapKV.  Per (sequence, KV head):
//   pass 1  row statistics (max, sum-exp) of the causal softmax of every (head, window row) over the
//           whole prompt, split along the key axis, then merged;
//   pass 2  probabilities recomputed from the statistics and summed over heads and window rows into
//           one vote per prefix token;
//   pool    stride-1 max-pool of the votes (odd kernel, clipped at the ends);
//   select  exact top-(N-W) of the pooled votes by radix select, ties to the lower position, emitted
//           ascending, followed by the W window positions;
//   gather  K rows and V columns of the kept tokens copied into the destination cache.
// The two score passes are the one dense contraction of the method (G*W query rows against every
// key): they run on the matrix cores with the (head, window-row) index as the MFMA column, so a lane
// owns a fixed set of softmax rows and their statistics stay in registers.
#include <type_traits>

#include "common.h"

namespace rkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kSnapColBlocks = 8;    // 16-column blocks per wavefront (128 softmax rows)
constexpr float kLog2eS = 1.4426950408889634f;
constexpr float kNegBigS = -1.0e30f;

union FragS {
  uint4 u;
  bf16x8 v;
};

struct SnapArgs {
  const bf16_t* qobs;
  int W, NC, CG, n_chunks, chunk_pages, keep, s_cap, pool_r;
  float* stats_part;  // [units][n_chunks][NC][2]
  float* stats;       // [units][NC][2]   (max in log2 domain, 1/sum)
  float* votes;       // [units][s_cap]
  float* pooled;      // [units][s_cap]
  int32_t* kept;      // [units][keep]
  int32_t* kept_user; // optional copy for the caller, rows of kept_stride entries
  int kept_stride;
  int32_t* n_out;     // [batch]: number of tokens kept per sequence
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

template <bool PASS2>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void snap_score_kernel(CacheView c, SnapArgs a) {
  __shared__ float sM[4][kSnapColBlocks * 16], sZ[4][kSnapColBlocks * 16];
  __shared__ float sV[4][16];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int unit = blockIdx.y, chunk = blockIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int L = S - a.W;
  const int cgi = wave % a.CG, pw = wave / a.CG, npw = 4 / a.CG;
  // 16-column blocks this wavefront owns that hold real softmax rows (same for all its lanes)
  const int n_cb = __builtin_amdgcn_readfirstlane(min(kSnapColBlocks, (a.NC + 15) / 16 - cgi * kSnapColBlocks));
  const int p_begin = chunk * a.chunk_pages;
  const int p_limit = PASS2 ? (L + kAttnPage - 1) / kAttnPage : (S + kAttnPage - 1) / kAttnPage;
  const int p_end = min(p_begin + a.chunk_pages, p_limit);

  FragS qf[kSnapColBlocks][4];
  int limit[kSnapColBlocks];
  float M2[kSnapColBlocks], invZ[kSnapColBlocks];
#pragma unroll
  for (int cb = 0; cb < kSnapColBlocks; ++cb) {
    const int col = (cgi * kSnapColBlocks + cb) * 16 + hn;
    if (col < a.NC) {
      const int h = col / a.W, w = col % a.W;
      const bf16_t* qp =
          a.qobs + (((int64_t)b * c.n_q_heads + (int64_t)g * c.group + h) * a.W + w) * kHeadDim + kg * 8;
#pragma unroll
      for (int j = 0; j < 4; ++j) qf[cb][j].u = *reinterpret_cast<const uint4*>(qp + j * 32);
      limit[cb] = L + w;
      if (PASS2) {
        M2[cb] = a.stats[((int64_t)unit * a.NC + col) * 2];
        invZ[cb] = a.stats[((int64_t)unit * a.NC + col) * 2 + 1];
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) qf[cb][j].u = make_uint4(0, 0, 0, 0);
      limit[cb] = -1;
      M2[cb] = 0.f;
      invZ[cb] = 0.f;
    }
  }
  float m[kSnapColBlocks], z[kSnapColBlocks];
#pragma unroll
  for (int cb = 0; cb < kSnapColBlocks; ++cb) { m[cb] = kNegBigS; z[cb] = 0.f; }
  const float sc = kLog2eS * 0.08838834764831845f;
  const int64_t head_off = (int64_t)g * c.stride_head;

  // Key tiles are requested two pages ahead of the one being scored (two register buffers used in
  // rotation), so the memory latency is hidden behind the matrix and exponent work of the pages
  // in between.  An absent or out-of-range page reads tile 0 of the pool and is masked below: the
  // loads stay unconditional and the loop body straight-line.
  const int64_t lane_off = head_off + hn * kHeadDim + kg * 8;
  const auto fetch = [&](int p, uint4* kf) -> bool {
    const int64_t pp = p < p_end ? phys_page(c, b, p) : -1;
    const bf16_t* kt = c.k_pool + (pp >= 0 ? pp : 0) * c.stride_page + lane_off;
#pragma unroll
    for (int j = 0; j < 4; ++j) kf[j] = ld16<false>(kt + j * 32);
    return pp >= 0;
  };
  const int n_it = p_end > p_begin ? (p_end - p_begin + npw - 1) / npw : 0;
  // one page: consume buffer kn (its tile arrived by now), refill it with the page two steps on
  const auto step = [&](int it, uint4* kn, bool& present_buf) {
    const int p = p_begin + it * npw + pw;
    const bool live = p < p_end;
    const bool present = present_buf;
    bf16x8 kf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kf[j] = __builtin_bit_cast(bf16x8, kn[j]);
    present_buf = fetch(p + 2 * npw, kn);
    const int tok0 = p * kAttnPage + kg * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    // A page that lies wholly inside the prefix is visible to every window row: no causal mask.
    // Column blocks go four at a time: four independent accumulator chains keep the matrix pipe
    // busy, and the softmax update is branch-free so the whole group schedules as one block.
    const auto score_page = [&](auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
      for (int qd = 0; qd < kSnapColBlocks / 4; ++qd) {
        if (qd * 4 >= n_cb) break;  // wave-uniform: the rest of this wavefront's blocks are unused
        f32x4 acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j], qf[qd * 4 + i][j].v, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int cb = qd * 4 + i;
          float s[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            s[r] = acc[i][r] * sc;
            if (MASKED) s[r] = (present && tok0 + r <= limit[cb]) ? s[r] : -INFINITY;
          }
          if (!PASS2) {
            const float mn = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), m[cb]);
            z[cb] = z[cb] * exp2_fast(m[cb] - mn) + exp2_fast(s[0] - mn) + exp2_fast(s[1] - mn) +
                    exp2_fast(s[2] - mn) + exp2_fast(s[3] - mn);
            m[cb] = mn;
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] += exp2_fast(s[r] - M2[cb]) * invZ[cb];
          }
        }
      }
    };
    if (present && p * kAttnPage + kAttnPage - 1 <= L)
      score_page(std::false_type{});
    else
      score_page(std::true_type{});
    if (PASS2) {
      // sum the 16 columns held by the lanes of one token group, then the column groups
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        v[r] += __shfl_xor(v[r], 1);
        v[r] += __shfl_xor(v[r], 2);
        v[r] += __shfl_xor(v[r], 4);
        v[r] += __shfl_xor(v[r], 8);
      }
      if (a.CG == 2) {
        if (cgi == 1 && hn == 0) {
#pragma unroll
          for (int r = 0; r < 4; ++r) sV[pw][kg * 4 + r] = v[r];
        }
        __syncthreads();
        if (cgi == 0) {
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] += sV[pw][kg * 4 + r];
        }
        __syncthreads();
      }
      if (live && cgi == 0 && hn == 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (tok0 + r < L) a.votes[(int64_t)unit * a.s_cap + tok0 + r] = v[r];
      }
    }
  };
  uint4 k0[4], k1[4];
  bool pr0 = false, pr1 = false;
  if (n_it > 0) {
    pr0 = fetch(p_begin + pw, k0);
    pr1 = fetch(p_begin + npw + pw, k1);
  }
  for (int it = 0; it < n_it; it += 2) {  // n_it is the same for every wavefront of the workgroup
    step(it, k0, pr0);
    if (it + 1 < n_it) step(it + 1, k1, pr1);
  }
  if (PASS2) return;

  // ---- pass 1: merge statistics over token groups, waves, and hand the chunk's partial out -------
#pragma unroll
  for (int cb = 0; cb < kSnapColBlocks; ++cb) {
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
      const float mo = __shfl_xor(m[cb], off), zo = __shfl_xor(z[cb], off);
      const float mn = fmaxf(m[cb], mo);
      z[cb] = z[cb] * exp2_fast(m[cb] - mn) + zo * exp2_fast(mo - mn);
      m[cb] = mn;
    }
    if (kg == 0) {
      sM[wave][cb * 16 + hn] = m[cb];
      sZ[wave][cb * 16 + hn] = z[cb];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < a.CG * kSnapColBlocks * 16; idx += 256) {
    const int cg2 = idx / (kSnapColBlocks * 16), lc = idx % (kSnapColBlocks * 16);
    const int col = cg2 * kSnapColBlocks * 16 + lc;
    if (col >= a.NC) continue;
    float mm = kNegBigS, zz = 0.f;
    for (int w2 = cg2; w2 < 4; w2 += a.CG) {
      const float mo = sM[w2][lc], zo = sZ[w2][lc];
      const float mn = fmaxf(mm, mo);
      zz = zz * exp2_fast(mm - mn) + zo * exp2_fast(mo - mn);
      mm = mn;
    }
    float* o = a.stats_part + (((int64_t)unit * a.n_chunks + chunk) * a.NC + col) * 2;
    o[0] = mm;
    o[1] = zz;
  }
}

// merge the per-chunk statistics of one unit: one thread per softmax row
__global__ __launch_bounds__(256) void snap_stats_kernel(CacheView c, SnapArgs a) {
  const int unit = blockIdx.x;
  const int b = unit / c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int chunks = ((S + kAttnPage - 1) / kAttnPage + a.chunk_pages - 1) / a.chunk_pages;
  for (int col = threadIdx.x; col < a.NC; col += 256) {
    float mm = kNegBigS, zz = 0.f;
    for (int ch = 0; ch < chunks; ++ch) {
      const float* o = a.stats_part + (((int64_t)unit * a.n_chunks + ch) * a.NC + col) * 2;
      const float mo = o[0], zo = o[1];
      const float mn = fmaxf(mm, mo);
      zz = zz * exp2_fast(mm - mn) + zo * exp2_fast(mo - mn);
      mm = mn;
    }
    a.stats[((int64_t)unit * a.NC + col) * 2] = mm;
    a.stats[((int64_t)unit * a.NC + col) * 2 + 1] = zz > 0.f ? 1.f / zz : 0.f;
  }
}

// stride-1 max-pool over the prefix votes, window [j-r, j+r] clipped to [0, L)
constexpr int kPoolTile = 1024;
__global__ __launch_bounds__(256) void snap_pool_kernel(CacheView c, SnapArgs a) {
  extern __shared__ float tile[];  // kPoolTile + 2r
  const int unit = blockIdx.y;
  const int b = unit / c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int L = S - a.W, r = a.pool_r;
  const int j0 = blockIdx.x * kPoolTile;
  if (j0 >= L) return;
  const float* v = a.votes + (int64_t)unit * a.s_cap;
  for (int i = threadIdx.x; i < kPoolTile + 2 * r; i += 256) {
    const int j = j0 - r + i;
    tile[i] = (j >= 0 && j < L) ? v[j] : -INFINITY;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kPoolTile; i += 256) {
    const int j = j0 + i;
    if (j >= L) break;
    float mx = tile[i];
    for (int d = 1; d <= 2 * r; ++d) mx = fmaxf(mx, tile[i + d]);
    a.pooled[(int64_t)unit * a.s_cap + j] = mx;
  }
}

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exact top-(keep-W) of pooled[0, L) + the window, ascending; one 1024-thread workgroup per unit
constexpr int kSelT = 1024;
__global__ __launch_bounds__(kSelT) void snap_select_kernel(CacheView c, SnapArgs a) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t wsum[kSelT / kWave];
  __shared__ uint32_t sh_bucket, sh_k;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int unit = blockIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int S = c.seq_lens[b];
  int32_t* kept = a.kept + (int64_t)unit * a.keep;
  int32_t* kept2 = a.kept_user ? a.kept_user + (int64_t)unit * a.kept_stride : nullptr;
  const bool small = S <= a.keep;
  const bool bad = S > c.pages_cap * kAttnPage;
  if (small || bad) {
    const int cnt = bad ? 0 : S;
    for (int i = tid; i < a.keep; i += kSelT) {
      const int v = i < cnt ? i : -1;
      kept[i] = v;
      if (kept2) kept2[i] = v;
    }
    if (g == 0 && tid == 0) a.n_out[b] = cnt;
    return;
  }
  const int L = S - a.W;
  const int k_pref = a.keep - a.W;
  const float* pv = a.pooled + (int64_t)unit * a.s_cap;

  uint32_t prefix = 0, mask = 0, k = (uint32_t)k_pref;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < L; j += kSelT) {
      const uint32_t key = order_key(pv[j]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    uint32_t v = 0, inc = 0;
    if (tid < 256) {  // bins are owned by the first four wavefronts
      v = hist[tid];
      inc = v;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t y = __shfl_down(inc, off);
        if (lane + off < kWave) inc += y;
      }
      if (lane == 0) wsum[wave] = inc;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = wave + 1; w < 4; ++w) inc += wsum[w];
      const uint32_t exc = inc - v;
      if (exc < k && k <= inc) {
        sh_bucket = (uint32_t)tid;
        sh_k = k - exc;
      }
    }
    __syncthreads();
    prefix |= sh_bucket << shift;
    mask |= 0xffu << shift;
    k = sh_k;
    __syncthreads();
  }
  const uint32_t tau = prefix, need_eq = k;

  // ordered emission: thread t owns a contiguous range of positions
  const int ipt = (L + kSelT - 1) / kSelT;
  const int lo = min(L, tid * ipt), hi = min(L, lo + ipt);
  uint32_t cgt = 0, ceq = 0;
  for (int j = lo; j < hi; ++j) {
    const uint32_t key = order_key(pv[j]);
    cgt += key > tau;
    ceq += key == tau;
  }
  // two block scans (counts can exceed 16 bits here)
  uint32_t before_gt, before_eq;
  {
    uint32_t inc = cgt;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint32_t y = __shfl_up(inc, off);
      if (lane >= off) inc += y;
    }
    if (lane == kWave - 1) wsum[wave] = inc;
    __syncthreads();
    uint32_t base = 0;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    before_gt = base + inc - cgt;
    __syncthreads();
    inc = ceq;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const uint32_t y = __shfl_up(inc, off);
      if (lane >= off) inc += y;
    }
    if (lane == kWave - 1) wsum[wave] = inc;
    __syncthreads();
    base = 0;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    before_eq = base + inc - ceq;
  }
  uint32_t gt = before_gt, eq = before_eq;
  for (int j = lo; j < hi; ++j) {
    const uint32_t key = order_key(pv[j]);
    bool take = key > tau;
    uint32_t eq_taken = min(eq, need_eq);
    if (key == tau) {
      take = eq < need_eq;
      eq_taken = eq;
      ++eq;
    }
    if (take) {
      const uint32_t pos = gt + eq_taken;
      if ((int)pos < k_pref) {
        kept[pos] = j;
        if (kept2) kept2[pos] = j;
      }
    }
    if (key > tau) ++gt;
  }
  for (int w = tid; w < a.W; w += kSelT) {
    kept[k_pref + w] = L + w;
    if (kept2) kept2[k_pref + w] = L + w;
  }
  if (g == 0 && tid == 0) a.n_out[b] = a.keep;
}

// copy the kept tokens into the destination cache; one workgroup per 16 kept tokens.  K rows move
// as 256-byte rows.  The V values of the 16 tokens are staged in LDS as [channel][token] whatever the
// source layout, then leave as one contiguous channel-major tile (page size 16) or as token rows.
__global__ __launch_bounds__(256) void snap_gather_kernel(CacheView src, CacheView dst, SnapArgs a) {
  __shared__ int s_tok[kAttnPage];
  __shared__ bf16_t s_v[kHeadDim * kAttnPage];
  const int tid = threadIdx.x;
  const int unit = blockIdx.y, blk = blockIdx.x;
  const int b = unit / src.n_kv_heads, g = unit % src.n_kv_heads;
  const int S = src.seq_lens[b];
  const int cnt = S > src.pages_cap * kAttnPage ? 0 : min(S, a.keep);
  if (blk * kAttnPage >= cnt) return;
  if (tid < kAttnPage) {
    const int t = blk * kAttnPage + tid;
    s_tok[tid] = t < cnt ? a.kept[(int64_t)unit * a.keep + t] : -1;
  }
  __syncthreads();
  const int dps = dst.page_size;
  const int64_t dhead = (int64_t)g * dst.stride_head, shead = (int64_t)g * src.stride_head;
  // K: 16 rows of 256 B; thread -> (row = tid/16, 16-byte piece = tid%16)
  const int row = tid / 16, piece = tid % 16;
  const int tok = s_tok[row];
  const int dt = blk * kAttnPage + row;  // destination position of this thread's row
  const int64_t spp = tok >= 0 ? phys_page(src, b, tok / kAttnPage) : -1;
  const int64_t dpp = dt / dps < dst.pages_cap ? phys_page(dst, b, dt / dps) : -1;
  const bool row_live = tok >= 0 && spp >= 0;
  {
    uint4 val = make_uint4(0, 0, 0, 0);
    if (row_live)
      val = ld16<false>(src.k_pool + spp * src.stride_page + shead + (tok % kAttnPage) * kHeadDim + piece * 8);
    // a channel-major destination gets whole tiles (zero rows past the end); a token-major one only
    // the rows that exist, as later pages may belong to something else
    if (dpp >= 0 && (tok >= 0 || !dst.v_token_major))
      *reinterpret_cast<uint4*>(dst.k_pool + dpp * dst.stride_page + dhead + (dt % dps) * kHeadDim +
                                piece * 8) = val;
  }
  if (src.v_token_major && dst.v_token_major) {
    if (row_live && dpp >= 0)
      *reinterpret_cast<uint4*>(dst.v_pool + dpp * dst.stride_page + dhead + (dt % dps) * kHeadDim +
                                piece * 8) =
          ld16<false>(src.v_pool + spp * src.stride_page + shead + (tok % kAttnPage) * kHeadDim + piece * 8);
    return;
  }
  // stage V as s_v[channel][token]
  if (src.v_token_major) {
    uint4 val = make_uint4(0, 0, 0, 0);
    if (row_live)
      val = ld16<false>(src.v_pool + spp * src.stride_page + shead + (tok % kAttnPage) * kHeadDim + piece * 8);
    const uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s_v[(piece * 8 + 2 * i) * kAttnPage + row] = (bf16_t)(w[i] & 0xffffu);
      s_v[(piece * 8 + 2 * i + 1) * kAttnPage + row] = (bf16_t)(w[i] >> 16);
    }
  } else {
    for (int idx = tid; idx < kHeadDim * kAttnPage; idx += 256) {
      const int slot = idx % kAttnPage, ch = idx / kAttnPage;
      const int tk = s_tok[slot];
      bf16_t val = 0;
      if (tk >= 0) {
        const int64_t sp2 = phys_page(src, b, tk / kAttnPage);
        if (sp2 >= 0)
          val = src.v_pool[sp2 * src.stride_page + shead + ch * kAttnPage + tk % kAttnPage];
      }
      s_v[idx] = val;
    }
  }
  __syncthreads();
  if (!dst.v_token_major) {
    // page size 16: the staged block is the destination tile
    if (dpp >= 0)
      reinterpret_cast<uint4*>(dst.v_pool + dpp * dst.stride_page + dhead)[tid] =
          reinterpret_cast<const uint4*>(s_v)[tid];
  } else if (tok >= 0 && dpp >= 0) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = (uint32_t)s_v[(piece * 8 + 2 * i) * kAttnPage + row] |
             ((uint32_t)s_v[(piece * 8 + 2 * i + 1) * kAttnPage + row] << 16);
    *reinterpret_cast<uint4*>(dst.v_pool + dpp * dst.stride_page + dhead + (dt % dps) * kHeadDim +
                              piece * 8) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

SnapPlan plan_snapkv(const CacheView& src, int window, int keep) {
  SnapPlan p;
  const size_t units = (size_t)src.batch * src.n_kv_heads;
  const int NC = src.group * window;
  // Pages per workgroup in the score passes.  Every wavefront loads the whole observation-window
  // query block before its first page, so long chunks amortise that; short ones keep the chip full
  // when there are few (sequence, KV head) units.  Aim for about 2048 workgroups.
  int chunk_pages = 32;
  while (chunk_pages < 256 && units * ((src.pages_cap + chunk_pages - 1) / chunk_pages) > 2048) chunk_pages *= 2;
  p.chunk_pages = chunk_pages;
  p.n_chunks = (src.pages_cap + chunk_pages - 1) / chunk_pages;
  const size_t s_cap = (size_t)src.pages_cap * kAttnPage;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t off = 0;
  p.stats_off = off;
  off += up(units * p.n_chunks * NC * 2 * sizeof(float)) + up(units * NC * 2 * sizeof(float));
  p.votes_off = off;
  off += up(units * s_cap * sizeof(float));
  p.pooled_off = off;
  off += up(units * s_cap * sizeof(float));
  p.kept_off = off;
  off += up(units * (size_t)keep * sizeof(int32_t));
  p.total_bytes = off;
  return p;
}

hipError_t launch_snapkv(const bf16_t* q_obs, const CacheView& src, int window, int pool_kernel,
                         int keep, const CacheView* dst, int32_t* kept_idx, int kept_stride,
                         int32_t* n_out, void* ws, const SnapPlan& plan, hipStream_t st) {
  const int units = src.batch * src.n_kv_heads;
  char* base = static_cast<char*>(ws);
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  SnapArgs a;
  a.qobs = q_obs;
  a.W = window;
  a.NC = src.group * window;
  a.CG = a.NC > kSnapColBlocks * 16 ? 2 : 1;
  a.n_chunks = plan.n_chunks;
  a.chunk_pages = plan.chunk_pages;
  a.keep = keep;
  a.s_cap = src.pages_cap * kAttnPage;
  a.pool_r = (pool_kernel - 1) / 2;
  a.stats_part = reinterpret_cast<float*>(base + plan.stats_off);
  a.stats = reinterpret_cast<float*>(base + plan.stats_off +
                                     up((size_t)units * plan.n_chunks * a.NC * 2 * sizeof(float)));
  a.votes = reinterpret_cast<float*>(base + plan.votes_off);
  a.pooled = reinterpret_cast<float*>(base + plan.pooled_off);
  a.kept = reinterpret_cast<int32_t*>(base + plan.kept_off);
  a.kept_user = kept_idx;
  a.kept_stride = kept_stride;
  a.n_out = n_out;

  const dim3 sgrid(plan.n_chunks, units);
  hipLaunchKernelGGL(snap_score_kernel<false>, sgrid, dim3(256), 0, st, src, a);
  hipLaunchKernelGGL(snap_stats_kernel, dim3(units), dim3(256), 0, st, src, a);
  hipLaunchKernelGGL(snap_score_kernel<true>, sgrid, dim3(256), 0, st, src, a);
  const dim3 pgrid((a.s_cap + kPoolTile - 1) / kPoolTile, units);
  hipLaunchKernelGGL(snap_pool_kernel, pgrid, dim3(256), (kPoolTile + 2 * a.pool_r) * sizeof(float), st,
                     src, a);
  hipLaunchKernelGGL(snap_select_kernel, dim3(units), dim3(kSelT), 0, st, src, a);
  if (!dst) return hipGetLastError();  // filter only: the indices are the result
  const dim3 ggrid((keep + kAttnPage - 1) / kAttnPage, units);
  hipLaunchKernelGGL(snap_gather_kernel, ggrid, dim3(256), 0, st, src, *dst, a);
  return hipGetLastError();
}

}  // namespace rkv
