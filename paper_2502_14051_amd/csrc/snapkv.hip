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
#include "select_core.h"


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
  uint32_t* sel_hist; // split select: [units][4][256] digit counts, then [units][sel_split][2] slice counts
  int sel_split;
};

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// sum over the 16 lanes of a DPP row (the lanes that hold the 16 columns of one token group); every
// lane of the row ends up with the total
__device__ __forceinline__ float row16_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, true));   // quad_perm 1,0,3,2
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, true));   // quad_perm 2,3,0,1
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, true));  // row_half_mirror
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, true));  // row_mirror
  return v;
}

// max of three without the input canonicalisation fmaxf() brings along (three extra instructions
// per call here); the inputs are matrix-core outputs and running maxima, never signalling NaNs
__device__ __forceinline__ float max3_raw(float x, float y, float w) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(x), "v"(y), "v"(w));
  return d;
}

__device__ __forceinline__ float max2_raw(float x, float y) {
  float d;
  asm("v_max_f32 %0, %1, %2" : "=v"(d) : "v"(x), "v"(y));
  return d;
}

__device__ __forceinline__ int64_t readlane64(int64_t v, int l) {
  return ((int64_t)__builtin_amdgcn_readlane((int)(v >> 32), l) << 32) |
         (uint32_t)__builtin_amdgcn_readlane((int)(v & 0xffffffff), l);
}

constexpr int kSnapMaxIters = 2 * kWave;  // pages one wavefront walks in a chunk, at most
constexpr int kSnapRing = 3;              // key tiles a wavefront keeps in flight (4 KiB of LDS each)
constexpr size_t kSnapRingBytes = (size_t)4 * kSnapRing * 4 * kWave * 16;  // four wavefronts
constexpr int kSnapMaxChunkPages = 128;  // pages per workgroup; pass 2 stages their votes in LDS (8 KiB per column group)

// QD: groups of four column blocks every wavefront works through (2 when some wavefront owns more
// than four blocks with real softmax rows; blocks without any hold zero queries and are discarded).
template <bool PASS2, int QD>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void snap_score_kernel(CacheView c, SnapArgs a) {
  __shared__ float sM[4][kSnapColBlocks * 16], sZ[4][kSnapColBlocks * 16];
  const int tid = threadIdx.x, lane = tid % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // scalar: page indices stay in SGPRs
  const int hn = lane % 16, kg = lane / 16;
  const int unit = blockIdx.y, chunk = blockIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int L = S - a.W;
  const int cgi = wave % a.CG, pw = wave / a.CG, npw = 4 / a.CG;
  const int p_begin = chunk * a.chunk_pages;
  const int p_limit = PASS2 ? (L + kAttnPage - 1) / kAttnPage : (S + kAttnPage - 1) / kAttnPage;
  const int p_end = min(p_begin + a.chunk_pages, p_limit);
  const int n_it = p_end > p_begin ? (p_end - p_begin + npw - 1) / npw : 0;  // <= kSnapMaxIters (host)

  // Where this wavefront's pages live: lane i looks up iterations i and i + 64 once, up front, and
  // the loop hands the tile offsets out by readlane, so it contains no table lookups and no waits
  // on them.  -1 marks an absent page.
  int64_t off_lo = -1, off_hi = -1;
  {
    const int p0 = p_begin + lane * npw + pw, p1 = p0 + kWave * npw;
    if (lane < n_it && p0 < p_end) {
      const int64_t pp = phys_page(c, b, p0);
      if (pp >= 0) off_lo = pp * c.stride_page;
    }
    if (lane + kWave < n_it && p1 < p_end) {
      const int64_t pp = phys_page(c, b, p1);
      if (pp >= 0) off_hi = pp * c.stride_page;
    }
  }

  constexpr int NCB = 4 * QD;
  FragS qf[NCB][4];
  int limit[NCB];
  float M2[NCB], invZ[NCB];
  float m[NCB], z[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) { m[cb] = kNegBigS; z[cb] = 0.f; }
  const float sc = kLog2eS * 0.08838834764831845f;
  const int64_t head_off = (int64_t)g * c.stride_head;

  // Key tiles travel through a ring of kSnapRing slots of LDS per wavefront, filled by loads that
  // write LDS directly (no registers are held for tiles in flight, so three of them fit where two
  // register buffers used to): the tile for iteration it + kSnapRing is requested as soon as the
  // products of iteration it have consumed the slot.  An absent or out-of-range page reads tile 0
  // of the pool and is masked below; those loads are issued all the same, which keeps the number
  // of loads younger than the tile being waited for constant.
  typedef uint32_t ring_u32x4 __attribute__((ext_vector_type(4)));
  extern __shared__ __align__(16) unsigned char snap_dyn[];
  ring_u32x4* ring = reinterpret_cast<ring_u32x4*>(snap_dyn) + wave * (kSnapRing * 4 * kWave);
  float* s_votes = reinterpret_cast<float*>(snap_dyn + kSnapRingBytes);  // pass 2: [column group][chunk_pages][16]
  const auto tile_off = [&](int it) -> int64_t {  // `it` is wave-uniform; branch-free
    const int l = it & (kWave - 1);
    const int64_t lo = readlane64(off_lo, l), hi = readlane64(off_hi, l);
    return it >= n_it ? -1 : (it < kWave ? lo : hi);
  };
  // Pass 1 loads the keys with the streaming hint (a fifth faster here); pass 2 without, so that the
  // part of the keys it reads last stays in the last-level cache for the gather that follows (which
  // measures 20 us slower otherwise, more than the hint gains pass 2).
  constexpr int kPolicyStream = 2;  // the "nt" bit of the load's cache policy
  // Load instruction j of a tile brings in token rows 4j .. 4j+3 (1 KiB, whole cache lines); lane l
  // lands at 16 l bytes into the instruction's KiB of the slot, and fetches the 16-byte chunk that
  // belongs there: the chunks of a row are stored XOR-swizzled by the row number, so that the reads
  // below (16 rows at one chunk position) spread over all LDS banks.
  const int dma_row = lane >> 4;                 // + 4 j
  const auto issue = [&](int it, int slot) {
    const int64_t off = tile_off(it);
    const bf16_t* kt = c.k_pool + (off >= 0 ? off : 0) + head_off;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = 4 * j + dma_row;
      const int chunk = (lane & 15) ^ row;
      __builtin_amdgcn_global_load_lds(reinterpret_cast<const ring_u32x4*>(kt + row * kHeadDim + chunk * 8),
                                       ring + (slot * 4 + j) * kWave, 16, 0, PASS2 ? 0 : kPolicyStream);
    }
  };
  const auto read_tile = [&](int slot, bf16x8* kf) {
    // everything but the kSnapRing - 1 younger tiles (four loads each) has landed
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kSnapRing - 1) * 4) : "memory");
#pragma unroll
    for (int j = 0; j < 4; ++j)  // token hn, channels 32 j + 8 kg ..: chunk 4 j + kg of row hn
      kf[j] = __builtin_bit_cast(bf16x8, ring[slot * 4 * kWave + hn * 16 + ((4 * j + kg) ^ hn)]);
  };
  const auto products = [&](const bf16x8* kf, int qd, f32x4* acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j], qf[qd * 4 + i][j].v, acc[i], 0, 0, 0);
  };
  // MASKED = false is the hot case, a page that is present and lies wholly inside the prefix, so
  // every window row sees all of it; it is written for the fewest vector instructions: the softmax
  // scale goes into the exponent's multiply-add, and the page maximum is taken on the raw products
  // (the scale is positive).
  const auto update = [&](auto masked_tag, const f32x4* acc, int qd, bool present, int tok0, float* v) {
    constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int cb = qd * 4 + i;
      float s[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        s[r] = acc[i][r];
        if (MASKED) s[r] = (present && tok0 + r <= limit[cb]) ? s[r] : -INFINITY;
      }
      if (!PASS2) {
        // m[] is the running maximum in the log2 domain; an unchanged maximum rescales by exactly 1
        const float mn = max2_raw(m[cb], max2_raw(max3_raw(s[0], s[1], s[2]), s[3]) * sc);
        const float e01 = exp2_fast(fmaf(s[0], sc, -mn)) + exp2_fast(fmaf(s[1], sc, -mn));
        const float e23 = exp2_fast(fmaf(s[2], sc, -mn)) + exp2_fast(fmaf(s[3], sc, -mn));
        z[cb] = fmaf(z[cb], exp2_fast(m[cb] - mn), e01 + e23);
        m[cb] = mn;
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = fmaf(exp2_fast(fmaf(s[r], sc, -M2[cb])), invZ[cb], v[r]);
      }
    }
  };
  // votes of one page (already summed over the 16 columns a token group's lanes hold): staged in LDS,
  // one copy per column group, and written out once per chunk (a global store per page would sit among
  // the tile loads the wait above counts, and make it wait for more of them than it needs; adding the
  // column groups per page would cost two workgroup barriers per page)
  const int chunk_tokens = a.chunk_pages * kAttnPage;
  const auto emit_votes = [&](float* v, bool live, int tok0) {
    if (live && hn == 0)
      *reinterpret_cast<float4*>(s_votes + cgi * chunk_tokens + (tok0 - p_begin * kAttnPage)) =
          make_float4(v[0], v[1], v[2], v[3]);
  };
  int slot = 0;
  // One page: its tile out of the ring, then per group of four column blocks the products and the
  // update; the slot is refilled once the last products have read it.
  const auto page = [&](auto masked_tag, int it) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int p = p_begin + it * npw + pw;
    const bool present = MASKED ? tile_off(it) >= 0 : true;
    const int tok0 = p * kAttnPage + kg * 4;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    bf16x8 kf[4];
    read_tile(slot, kf);
#pragma unroll
    for (int qd = 0; qd < QD; ++qd) {
      f32x4 acc[4];
      products(kf, qd, acc);
      if (qd == QD - 1) {
        // the tile is in registers (the products had to wait for the LDS reads): refill its slot
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        issue(it + kSnapRing, slot);
      }
      // keep the groups in program order: products of a later group hoisted above this group's
      // update would need a second set of accumulators the register file has no room for
      __builtin_amdgcn_sched_barrier(0);
      update(masked_tag, acc, qd, present, tok0, v);
    }
    if (PASS2) {
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = row16_sum(v[r]);
    }
    __builtin_amdgcn_sched_barrier(0);
    slot = slot + 1 == kSnapRing ? 0 : slot + 1;
    if (PASS2) emit_votes(v, p < p_end, tok0);
  };
  // The leading run of pages that need no mask takes the hot variant: none of the wavefront's pages
  // absent, and the page's last token inside the prefix.
  const bool any_absent =
      __ballot((lane < n_it && off_lo < 0) || (lane + kWave < n_it && off_hi < 0)) != 0ull;
  int n_fast = 0;
  if (!any_absent) {
    // pages p_begin + it * npw + pw with p * 16 + 15 <= L, i.e. p <= (L - 15) / 16, also below p_end
    const int p_last = min(p_end - 1, (L - (kAttnPage - 1)) >= 0 ? (L - (kAttnPage - 1)) / kAttnPage : -1);
    if (p_last >= p_begin + pw) n_fast = (p_last - p_begin - pw) / npw + 1;
    n_fast = min(n_fast, n_it);
  }
#pragma unroll
  for (int t = 0; t < kSnapRing; ++t) issue(t, t);
  // the queries (and pass 2's row statistics) come in behind the first tiles rather than before them
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int col = (cgi * kSnapColBlocks + cb) * 16 + hn;
    if (col < a.NC) {
      const int h = col / a.W, w = col % a.W;
      const bf16_t* qp =
          a.qobs + (((int64_t)b * c.n_q_heads + (int64_t)g * c.group + h) * a.W + w) * kHeadDim + kg * 8;
#pragma unroll
      for (int j = 0; j < 4; ++j) qf[cb][j].u = *reinterpret_cast<const uint4*>(qp + j * 32);
      limit[cb] = L + w;
      if (PASS2) {
        const float2 st2 = *reinterpret_cast<const float2*>(a.stats + ((int64_t)unit * a.NC + col) * 2);
        M2[cb] = st2.x;
        invZ[cb] = st2.y;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) qf[cb][j].u = make_uint4(0, 0, 0, 0);
      limit[cb] = -1;
      M2[cb] = 0.f;
      invZ[cb] = 0.f;
    }
  }
  int it = 0;
  for (; it < n_fast; ++it) page(std::false_type{}, it);
  for (; it < n_it; ++it) page(std::true_type{}, it);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the last refills (unused) land before LDS is reused
  if (PASS2) {
    __syncthreads();
    const int tok_begin = p_begin * kAttnPage;
    const int n_tok = min(p_end * kAttnPage, L) - tok_begin;
    for (int i = tid; i < n_tok; i += 256)
      a.votes[(int64_t)unit * a.s_cap + tok_begin + i] = a.CG == 2 ? s_votes[i] + s_votes[chunk_tokens + i] : s_votes[i];
    return;
  }
  // ---- pass 1: merge statistics over token groups, waves, and hand the chunk's partial out -------
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
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

// merge the per-chunk statistics of one unit.  A long prompt has hundreds of chunks: the chunks of a
// softmax row are dealt to 1024 / ncp threads (ncp = the row count rounded up to a power of two),
// each merges its share with eight loads in flight, and one thread per row merges the partial
// results in a fixed order.
constexpr int kStatsT = 1024;
__global__ __launch_bounds__(kStatsT) void snap_stats_kernel(CacheView c, SnapArgs a) {
  __shared__ float pm[kStatsT], pz[kStatsT];
  const int tid = threadIdx.x;
  const int unit = blockIdx.x;
  const int b = unit / c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int chunks = ((S + kAttnPage - 1) / kAttnPage + a.chunk_pages - 1) / a.chunk_pages;
  int ncp = 64;
  while (ncp < a.NC) ncp <<= 1;  // NC <= 256 (host)
  const int col = tid % ncp, part = tid / ncp, parts = kStatsT / ncp;
  const auto merge = [](float& mm, float& zz, float mo, float zo) {
    const float mn = fmaxf(mm, mo);
    zz = zz * exp2_fast(mm - mn) + zo * exp2_fast(mo - mn);
    mm = mn;
  };
  float mm = kNegBigS, zz = 0.f;
  if (col < a.NC) {
    const float2* row = reinterpret_cast<const float2*>(a.stats_part) + (int64_t)unit * a.n_chunks * a.NC + col;
    for (int ch0 = part; ch0 < chunks; ch0 += parts * 8) {
      float2 o[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int ch = ch0 + u * parts;
        o[u] = ch < chunks ? row[(int64_t)ch * a.NC] : make_float2(kNegBigS, 0.f);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) merge(mm, zz, o[u].x, o[u].y);
    }
  }
  pm[tid] = mm;
  pz[tid] = zz;
  __syncthreads();
  if (tid < a.NC) {
    mm = kNegBigS;
    zz = 0.f;
    for (int p = 0; p < parts; ++p) merge(mm, zz, pm[p * ncp + tid], pz[p * ncp + tid]);
    a.stats[((int64_t)unit * a.NC + tid) * 2] = mm;
    a.stats[((int64_t)unit * a.NC + tid) * 2 + 1] = zz > 0.f ? 1.f / zz : 0.f;
  }
}

// stride-1 max-pool over the prefix votes, window [j-r, j+r] clipped to [0, L).  Window maxima by
// doubling in LDS: M_1 = the votes, M_2w[i] = max(M_w[i], M_w[i+w]) up to the largest power of two
// p <= 2r+1, then two overlapping windows of p cover the 2r+1 (a maximum is exact, so the order of
// taking it does not matter): 3 log2(p) + 2 LDS accesses per vote instead of 2r+1.
constexpr int kPoolTile = 1024;
__global__ __launch_bounds__(256) void snap_pool_kernel(CacheView c, SnapArgs a) {
  extern __shared__ float tile[];  // two arrays of kPoolTile + 2r
  const int unit = blockIdx.y;
  const int b = unit / c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int L = S - a.W, r = a.pool_r;
  const int j0 = blockIdx.x * kPoolTile;
  if (j0 >= L) return;
  const int n = kPoolTile + 2 * r;
  float* cur = tile;
  float* nxt = tile + n;
  const float* v = a.votes + (int64_t)unit * a.s_cap;
  for (int i = threadIdx.x; i < n; i += 256) {
    const int j = j0 - r + i;
    cur[i] = (j >= 0 && j < L) ? v[j] : -INFINITY;
  }
  __syncthreads();
  int p = 1;
  while (2 * p <= 2 * r + 1) {
    for (int i = threadIdx.x; i < n; i += 256) nxt[i] = fmaxf(cur[i], i + p < n ? cur[i + p] : -INFINITY);
    __syncthreads();
    float* t = cur;
    cur = nxt;
    nxt = t;
    p *= 2;
  }
  const int second = 2 * r + 1 - p;  // tile index i holds position j0 - r + i: output i spans [i, i + 2r]
  for (int i = threadIdx.x; i < kPoolTile; i += 256) {
    const int j = j0 + i;
    if (j >= L) break;
    a.pooled[(int64_t)unit * a.s_cap + j] = fmaxf(cur[i], cur[i + second]);
  }
}

__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exact top-(keep-W) of pooled[0, L) + the window, ascending; one 1024-thread workgroup per unit.
// Six passes over the row (four radix digits, a count, the ordered emission), all of them as
// coalesced 16-byte loads with eight in flight per thread; the top digit (sign and exponent, which
// votes share) is counted once per group of lanes that hold the same one.  For the emission a
// wavefront owns a contiguous stretch of the row and walks it in 256-position steps, with a prefix
// sum over its lanes per step.
constexpr int kSelT = 1024;
constexpr int kSelBatch = 8;
__global__ __launch_bounds__(kSelT) void snap_select_kernel(CacheView c, SnapArgs a) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t wsum[kSelT / kWave], wsum_eq[kSelT / kWave];
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
  // the row holds s_cap >= L + W floats and starts 16-byte aligned: the last group of four is in bounds
  const float4* pv4 = reinterpret_cast<const float4*>(a.pooled + (int64_t)unit * a.s_cap);
  const int n4 = (L + 3) / 4;

  uint32_t prefix = 0, mask = 0, k = (uint32_t)k_pref;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int base = 0; base < n4; base += kSelT * kSelBatch) {  // the same trip count for every thread
      float4 v[kSelBatch];
#pragma unroll
      for (int u = 0; u < kSelBatch; ++u) {
        const int q = base + u * kSelT + tid;
        v[u] = q < n4 ? pv4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < kSelBatch; ++u) {
        const int q = base + u * kSelT + tid;
        const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
        bool on[4];
        uint32_t digit[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t key = order_key(x[e]);
          on[e] = q < n4 && 4 * q + e < L && (key & mask) == prefix;
          digit[e] = (key >> shift) & 255u;
        }
        // the top digit: four neighbours mostly share it (pooling repeats a maximum 2r+1 times), and
        // so do most lanes; such a group of four is counted in one step for all lanes that agree
        const bool four = pass == 0 && on[0] && on[1] && on[2] && on[3] && digit[0] == digit[1] &&
                          digit[1] == digit[2] && digit[2] == digit[3];
        if (pass == 0) hist_add_grouped(hist, digit[0], four, 4u);
        if (!four) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (on[e]) atomicAdd(&hist[digit[e]], 1u);
        }
      }
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

  // ordered emission: wavefront w owns groups [w * gpw, (w + 1) * gpw), gpw a multiple of 64
  const int gpw = ((n4 + kSelT / kWave - 1) / (kSelT / kWave) + kWave - 1) / kWave * kWave;
  const int wbeg = wave * gpw, wend = min(wbeg + gpw, n4);
  uint32_t cgt = 0, ceq = 0;
  for (int base = wbeg; base < wend; base += kWave * kSelBatch) {
    float4 v[kSelBatch];
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) {
      const int q = base + u * kWave + lane;
      v[u] = q < wend ? pv4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) {
      const int q = base + u * kWave + lane;
      const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t key = order_key(x[e]);
        const bool in = q < wend && 4 * q + e < L;
        cgt += in && key > tau;
        ceq += in && key == tau;
      }
    }
  }
  // keys above / equal to the threshold in the wavefronts before this one
  {
    const uint32_t tg = wave_incl_scan(cgt), te = wave_incl_scan(ceq);
    if (lane == kWave - 1) {
      wsum[wave] = tg;
      wsum_eq[wave] = te;
    }
  }
  __syncthreads();
  uint32_t gt = 0, eq = 0;  // the same for every lane of the wavefront
  for (int w = 0; w < wave; ++w) {
    gt += wsum[w];
    eq += wsum_eq[w];
  }
  for (int base = wbeg; base < wend; base += kWave * kSelBatch) {
    float4 v[kSelBatch];
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) {
      const int q = base + u * kWave + lane;
      v[u] = q < wend ? pv4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < kSelBatch; ++u) {
      const int q = base + u * kWave + lane;
      const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
      uint32_t key[4];
      uint32_t ng = 0, ne = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        key[e] = order_key(x[e]);
        const bool in = q < wend && 4 * q + e < L;
        if (!in) key[e] = 0;  // below every threshold that is reached here (kp < L)
        ng += in && key[e] > tau;
        ne += in && key[e] == tau;
      }
      const uint32_t sg = wave_incl_scan(ng), se = wave_incl_scan(ne);
      uint32_t mgt = gt + sg - ng, meq = eq + se - ne;  // before this lane's four positions
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool in = q < wend && 4 * q + e < L;
        bool take = in && key[e] > tau;
        uint32_t eq_taken = min(meq, need_eq);
        if (in && key[e] == tau) {
          take = meq < need_eq;
          eq_taken = meq;
          ++meq;
        }
        if (take) {
          const uint32_t pos = mgt + eq_taken;
          if ((int)pos < k_pref) {
            kept[pos] = 4 * q + e;
            if (kept2) kept2[pos] = 4 * q + e;
          }
        }
        if (in && key[e] > tau) ++mgt;
      }
      gt += (uint32_t)__builtin_amdgcn_readlane((int)sg, kWave - 1);
      eq += (uint32_t)__builtin_amdgcn_readlane((int)se, kWave - 1);
    }
  }
  for (int w = tid; w < a.W; w += kSelT) {
    kept[k_pref + w] = L + w;
    if (kept2) kept2[k_pref + w] = L + w;
  }
  if (g == 0 && tid == 0) a.n_out[b] = a.keep;
}

// ---- the same selection with several workgroups per unit ------------------------------------------
// One long prompt is eight units: one workgroup each leaves the chip idle for the six passes above.
// Here a unit's row is cut into `sel_split` slices, and every pass is a launch of its own: four
// launches add their slice's digit counts to the unit's histograms in memory (each workgroup first
// re-derives the digits fixed so far from the earlier histograms, which is 256 counters per digit),
// one counts the keys above / equal to the threshold per slice, and the last emits in order from the
// slice counts before it.  Same result as the single-launch kernel.
constexpr int kSplitT = 256;

// (prefix, remaining k) after the first `passes` radix digits, from the unit's histograms; every
// wavefront computes it for itself
__device__ __forceinline__ void split_threshold(const uint32_t* ghist, int passes, uint32_t k_pref,
                                                uint32_t& prefix, uint32_t& mask, uint32_t& k) {
  const int lane = threadIdx.x % kWave;
  prefix = 0;
  mask = 0;
  k = k_pref;
  for (int pass = 0; pass < passes; ++pass) {
    const int shift = 24 - 8 * pass;
    const int b0 = 4 * (kWave - 1 - lane);  // lane 0 owns the four highest bins
    const uint4 h = *reinterpret_cast<const uint4*>(ghist + pass * 256 + b0);
    const uint32_t s3 = h.w, s2 = h.z + s3, s1 = h.y + s2, s0 = h.x + s1;
    const uint32_t above = wave_incl_scan(s0) - s0;
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
}

// the slice of float4 groups of workgroup `wg`: a multiple of 64 groups, so wavefront steps stay whole
__device__ __forceinline__ void split_slice(int n4, int split, int wg, int& gbeg, int& gend) {
  const int per = ((n4 + split - 1) / split + kWave - 1) / kWave * kWave;
  gbeg = min(wg * per, n4);
  gend = min(gbeg + per, n4);
}

__global__ __launch_bounds__(kSplitT) void snap_split_hist_kernel(CacheView c, SnapArgs a, int pass) {
  __shared__ uint32_t hist[256];
  const int tid = threadIdx.x;
  const int unit = blockIdx.y, wg = blockIdx.x;
  const int b = unit / c.n_kv_heads;
  const int S = c.seq_lens[b];
  if (S <= a.keep || S > c.pages_cap * kAttnPage) return;
  const int L = S - a.W;
  const float4* pv4 = reinterpret_cast<const float4*>(a.pooled + (int64_t)unit * a.s_cap);
  const int n4 = (L + 3) / 4;
  int gbeg, gend;
  split_slice(n4, a.sel_split, wg, gbeg, gend);
  uint32_t* ghist = a.sel_hist + (int64_t)unit * 4 * 256;
  uint32_t prefix, mask, k;
  split_threshold(ghist, pass, (uint32_t)(a.keep - a.W), prefix, mask, k);
  const int shift = 24 - 8 * pass;
  hist[tid] = 0;
  __syncthreads();
  for (int base = gbeg; base < gend; base += kSplitT * 4) {  // the same trip count for every thread
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = base + u * kSplitT + tid;
      v[u] = q < gend ? pv4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = base + u * kSplitT + tid;
      const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
      bool on[4];
      uint32_t digit[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t key = order_key(x[e]);
        on[e] = q < gend && 4 * q + e < L && (key & mask) == prefix;
        digit[e] = (key >> shift) & 255u;
      }
      const bool four = pass == 0 && on[0] && on[1] && on[2] && on[3] && digit[0] == digit[1] &&
                        digit[1] == digit[2] && digit[2] == digit[3];
      if (pass == 0) hist_add_grouped(hist, digit[0], four, 4u);
      if (!four) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (on[e]) atomicAdd(&hist[digit[e]], 1u);
      }
    }
  }
  __syncthreads();
  if (hist[tid] != 0) atomicAdd(&ghist[pass * 256 + tid], hist[tid]);
}

// EMIT = false: the slice's counts of keys above / equal to the threshold, to sel_hist's second part.
// EMIT = true: the ordered emission of the slice (and, by slice 0, the window and the short prompts).
template <bool EMIT>
__global__ __launch_bounds__(kSplitT) void snap_split_emit_kernel(CacheView c, SnapArgs a) {
  __shared__ uint32_t wsum[kSplitT / kWave], wsum_eq[kSplitT / kWave];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int unit = blockIdx.y, wg = blockIdx.x;
  const int units = gridDim.y;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int S = c.seq_lens[b];
  int32_t* kept = a.kept + (int64_t)unit * a.keep;
  int32_t* kept2 = a.kept_user ? a.kept_user + (int64_t)unit * a.kept_stride : nullptr;
  const bool small = S <= a.keep;
  const bool bad = S > c.pages_cap * kAttnPage;
  if (small || bad) {
    if (EMIT && wg == 0) {
      const int cnt = bad ? 0 : S;
      for (int i = tid; i < a.keep; i += kSplitT) {
        const int v = i < cnt ? i : -1;
        kept[i] = v;
        if (kept2) kept2[i] = v;
      }
      if (g == 0 && tid == 0) a.n_out[b] = cnt;
    }
    return;
  }
  const int L = S - a.W;
  const int k_pref = a.keep - a.W;
  const float4* pv4 = reinterpret_cast<const float4*>(a.pooled + (int64_t)unit * a.s_cap);
  const int n4 = (L + 3) / 4;
  int gbeg, gend;
  split_slice(n4, a.sel_split, wg, gbeg, gend);
  uint32_t tau, mask, need_eq;
  split_threshold(a.sel_hist + (int64_t)unit * 4 * 256, 4, (uint32_t)k_pref, tau, mask, need_eq);
  uint32_t* slice_cnt = a.sel_hist + (int64_t)units * 4 * 256 + (int64_t)unit * a.sel_split * 2;

  // wavefront w of the workgroup owns groups [wbeg, wend) of the slice, a multiple of 64 long
  const int gpw = ((gend - gbeg + kSplitT / kWave - 1) / (kSplitT / kWave) + kWave - 1) / kWave * kWave;
  const int wbeg = min(gbeg + wave * gpw, gend), wend = min(wbeg + gpw, gend);
  uint32_t cgt = 0, ceq = 0;
  for (int base = wbeg; base < wend; base += kWave * 4) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = base + u * kWave + lane;
      v[u] = q < wend ? pv4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = base + u * kWave + lane;
      const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t key = order_key(x[e]);
        const bool in = q < wend && 4 * q + e < L;
        cgt += in && key > tau;
        ceq += in && key == tau;
      }
    }
  }
  {
    const uint32_t tg = wave_incl_scan(cgt), te = wave_incl_scan(ceq);
    if (lane == kWave - 1) {
      wsum[wave] = tg;
      wsum_eq[wave] = te;
    }
  }
  __syncthreads();
  if (!EMIT) {
    if (tid == 0) {
      uint32_t tg = 0, te = 0;
      for (int w = 0; w < kSplitT / kWave; ++w) {
        tg += wsum[w];
        te += wsum_eq[w];
      }
      slice_cnt[wg * 2] = tg;
      slice_cnt[wg * 2 + 1] = te;
    }
    return;
  }
  // keys above / equal to the threshold before this wavefront: earlier slices, earlier wavefronts
  uint32_t gt = 0, eq = 0;
  {
    uint32_t pg = 0, pe = 0;
    if (lane < wg) {  // sel_split <= 64 (host)
      pg = slice_cnt[lane * 2];
      pe = slice_cnt[lane * 2 + 1];
    }
    gt = (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(pg), kWave - 1);
    eq = (uint32_t)__builtin_amdgcn_readlane((int)wave_incl_scan(pe), kWave - 1);
  }
  for (int w = 0; w < wave; ++w) {
    gt += wsum[w];
    eq += wsum_eq[w];
  }
  for (int base = wbeg; base < wend; base += kWave * 4) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = base + u * kWave + lane;
      v[u] = q < wend ? pv4[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = base + u * kWave + lane;
      const float x[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
      uint32_t key[4];
      uint32_t ng = 0, ne = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        key[e] = order_key(x[e]);
        const bool in = q < wend && 4 * q + e < L;
        ng += in && key[e] > tau;
        ne += in && key[e] == tau;
      }
      const uint32_t sg = wave_incl_scan(ng), se = wave_incl_scan(ne);
      uint32_t mgt = gt + sg - ng, meq = eq + se - ne;  // before this lane's four positions
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool in = q < wend && 4 * q + e < L;
        bool take = in && key[e] > tau;
        uint32_t eq_taken = min(meq, need_eq);
        if (in && key[e] == tau) {
          take = meq < need_eq;
          eq_taken = meq;
          ++meq;
        }
        if (take) {
          const uint32_t pos = mgt + eq_taken;
          if ((int)pos < k_pref) {
            kept[pos] = 4 * q + e;
            if (kept2) kept2[pos] = 4 * q + e;
          }
        }
        if (in && key[e] > tau) ++mgt;
      }
      gt += (uint32_t)__builtin_amdgcn_readlane((int)sg, kWave - 1);
      eq += (uint32_t)__builtin_amdgcn_readlane((int)se, kWave - 1);
    }
  }
  if (wg == 0) {
    for (int w = tid; w < a.W; w += kSplitT) {
      kept[k_pref + w] = L + w;
      if (kept2) kept2[k_pref + w] = L + w;
    }
    if (g == 0 && tid == 0) a.n_out[b] = a.keep;
  }
}

__global__ __launch_bounds__(256) void snap_split_zero_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// The same selection for prompts of up to ROCKETKV_MAX_PAGES tokens, through the register-resident
// top-k that Step 2 of the decode path uses for its page scores (one token = one page of size 1,
// budget = the prefix share of the keep budget): every pooled vote is read once and stays in
// registers, where the radix kernels above walk the row six times.  Same result: the k largest, ties
// to the lower position, ascending.
__global__ __launch_bounds__(kSelT) void snap_select_fast_kernel(CacheView c, SnapArgs a) {
  __shared__ PickShared<kSelT> sh;
  const int tid = threadIdx.x;
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
  for (int i = tid; i < 4 * 256; i += kSelT) (&sh.hist[0][0])[i] = 0;  // the pick expects clear counters
  __syncthreads();
  CacheView row = c;  // the pooled votes of this unit as one sequence of one-token pages
  row.page_size = 1;
  row.pages_cap = a.s_cap;
  SelectArgs pa = {};
  pa.in_scores = a.pooled + (int64_t)unit * a.s_cap;
  pa.T = k_pref;
  pa.n_recent = 0;
  pa.out_pages = kept;
  pa.row_len = k_pref;
  pa.out_pages2 = kept2;
  pa.row_len2 = k_pref;
  pick_from_scores<kSelT, false, true>(row, pa, 0, L, sh);
  for (int w = tid; w < a.W; w += kSelT) {
    kept[k_pref + w] = L + w;
    if (kept2) kept2[k_pref + w] = L + w;
  }
  if (g == 0 && tid == 0) a.n_out[b] = a.keep;
}

// copy the kept tokens into the destination cache; one workgroup per kGatherBlocks x 16 kept tokens
// (each workgroup is a chain of dependent round trips: index, rows, stores; several blocks per
// workgroup put several times the loads in flight behind one such chain).  K rows move as 256-byte
// rows.  The V values of 16 tokens are staged in LDS as [channel][token] whatever the source layout,
// then leave as one contiguous channel-major tile (page size 16) or as token rows.
constexpr int kGatherBlocks = 4;
__global__ __launch_bounds__(256) void snap_gather_kernel(CacheView src, CacheView dst, SnapArgs a) {
  constexpr int NB = kGatherBlocks, NTOK = NB * kAttnPage;
  __shared__ int s_tok[NTOK];
  __shared__ int64_t s_src[NTOK];  // element offset of the token's source tile (page and head), or -1
  __shared__ __align__(16) bf16_t s_v[NB][kHeadDim * kAttnPage];
  const int tid = threadIdx.x;
  const int unit = blockIdx.y, blk0 = blockIdx.x * NB;
  const int b = unit / src.n_kv_heads, g = unit % src.n_kv_heads;
  const int S = src.seq_lens[b];
  const int cnt = S > src.pages_cap * kAttnPage ? 0 : min(S, a.keep);
  if (blk0 * kAttnPage >= cnt) return;
  const int64_t dhead = (int64_t)g * dst.stride_head, shead = (int64_t)g * src.stride_head;
  if (tid < NTOK) {
    const int t = blk0 * kAttnPage + tid;
    const int tok = t < cnt ? a.kept[(int64_t)unit * a.keep + t] : -1;
    const int64_t spp = tok >= 0 ? phys_page(src, b, tok / kAttnPage) : -1;
    s_tok[tid] = spp >= 0 ? tok : -1;
    s_src[tid] = spp >= 0 ? spp * src.stride_page + shead : -1;
  }
  __syncthreads();
  const int dps = dst.page_size;
  // rows: thread -> (row = tid/16 of each block, 16-byte piece = tid%16)
  const int row = tid / 16, piece = tid % 16;
  int tok[NB];
  int64_t so[NB], dof[NB];  // source tile, destination row (-1: none)
  bool in_cnt[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    tok[i] = s_tok[i * kAttnPage + row];
    so[i] = s_src[i * kAttnPage + row];
    const int dt = (blk0 + i) * kAttnPage + row;  // destination position of this thread's row
    in_cnt[i] = (blk0 + i) * kAttnPage < cnt;     // the block exists at all
    const int64_t dpp = (in_cnt[i] && dt / dps < dst.pages_cap) ? phys_page(dst, b, dt / dps) : -1;
    dof[i] = dpp >= 0 ? dpp * dst.stride_page + dhead + (dt % dps) * kHeadDim + piece * 8 : -1;
  }
  // the K rows: loaded now, stored after the V loads have gone out as well (one wait for both)
  uint4 kval[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    kval[i] = make_uint4(0, 0, 0, 0);
    if (tok[i] >= 0) kval[i] = ld16<false>(src.k_pool + so[i] + (tok[i] % kAttnPage) * kHeadDim + piece * 8);
  }
  // a channel-major destination gets whole tiles (zero rows past the end); a token-major one only
  // the rows that exist, as later pages may belong to something else
  const auto store_k = [&]() {
#pragma unroll
    for (int i = 0; i < NB; ++i)
      if (dof[i] >= 0 && (tok[i] >= 0 || !dst.v_token_major)) *reinterpret_cast<uint4*>(dst.k_pool + dof[i]) = kval[i];
  };
  if (src.v_token_major && dst.v_token_major) {
    uint4 val[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
      if (tok[i] >= 0) val[i] = ld16<false>(src.v_pool + so[i] + (tok[i] % kAttnPage) * kHeadDim + piece * 8);
    store_k();
#pragma unroll
    for (int i = 0; i < NB; ++i)
      if (tok[i] >= 0 && dof[i] >= 0) *reinterpret_cast<uint4*>(dst.v_pool + dof[i]) = val[i];
    return;
  }
  // stage V as s_v[block][channel][token]
  if (src.v_token_major) {
    uint4 val[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      val[i] = make_uint4(0, 0, 0, 0);
      if (tok[i] >= 0) val[i] = ld16<false>(src.v_pool + so[i] + (tok[i] % kAttnPage) * kHeadDim + piece * 8);
    }
    store_k();
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const uint32_t w[4] = {val[i].x, val[i].y, val[i].z, val[i].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s_v[i][(piece * 8 + 2 * e) * kAttnPage + row] = (bf16_t)(w[e] & 0xffffu);
        s_v[i][(piece * 8 + 2 * e + 1) * kAttnPage + row] = (bf16_t)(w[e] >> 16);
      }
    }
  } else {
    // thread -> (slot = tid%16, channels tid/16 + 16 j): the loads of all blocks go out before the first LDS store
    const int slot = tid % kAttnPage, ch0 = tid / kAttnPage;
    bf16_t val[NB][8];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int tk = s_tok[i * kAttnPage + slot];
      const int64_t sv = s_src[i * kAttnPage + slot];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        val[i][j] = 0;
        if (tk >= 0) val[i][j] = src.v_pool[sv + (ch0 + 16 * j) * kAttnPage + tk % kAttnPage];
      }
    }
    store_k();
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) s_v[i][(ch0 + 16 * j) * kAttnPage + slot] = val[i][j];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    if (!dst.v_token_major) {
      // page size 16: the staged block is the destination tile
      const int dt0 = (blk0 + i) * kAttnPage;
      const int64_t dpp = (in_cnt[i] && dt0 / kAttnPage < dst.pages_cap) ? phys_page(dst, b, dt0 / kAttnPage) : -1;
      if (dpp >= 0)
        reinterpret_cast<uint4*>(dst.v_pool + dpp * dst.stride_page + dhead)[tid] =
            reinterpret_cast<const uint4*>(s_v[i])[tid];
    } else if (tok[i] >= 0 && dof[i] >= 0) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        w[e] = (uint32_t)s_v[i][(piece * 8 + 2 * e) * kAttnPage + row] |
               ((uint32_t)s_v[i][(piece * 8 + 2 * e + 1) * kAttnPage + row] << 16);
      *reinterpret_cast<uint4*>(dst.v_pool + dof[i]) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

SnapPlan plan_snapkv(const CacheView& src, int window, int keep) {
  SnapPlan p;
  const size_t units = (size_t)src.batch * src.n_kv_heads;
  const int NC = src.group * window;
  // Pages per workgroup in the score passes.  Every wavefront loads the whole observation-window
  // query block before its first page, so long chunks amortise that; short ones keep the chip full
  // when there are few (sequence, KV head) units.  Aim for 512 workgroups or more (two per compute
  // unit): eight units of a 131072-token prompt ran a third slower in chunks of 32 pages than of 128.
  static_assert(kSnapMaxChunkPages / 2 <= kSnapMaxIters, "a wavefront's share of the longest chunk must fit its page-offset lanes");
  int chunk_pages = 32;
  while (chunk_pages < kSnapMaxChunkPages && units * ((src.pages_cap + chunk_pages - 1) / chunk_pages) > 512) chunk_pages *= 2;
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
  // long prompts of few units: the select runs as several workgroups per unit over several launches
  p.sel_split = 0;
  if (s_cap > ROCKETKV_MAX_PAGES && units <= 64) {
    int split = (int)(256 / units);
    p.sel_split = split > 32 ? 32 : split;
  }
  p.sel_off = off;
  off += up(units * (size_t)(4 * 256 + 2 * 64) * sizeof(uint32_t));
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
  a.sel_hist = reinterpret_cast<uint32_t*>(base + plan.sel_off);
  a.sel_split = plan.sel_split;

  const dim3 sgrid(plan.n_chunks, units);
  const size_t vote_bytes = (size_t)a.CG * a.chunk_pages * kAttnPage * sizeof(float);
  const bool two_groups = a.NC > 4 * 16;  // some wavefront owns more than four blocks of real rows
  if (two_groups)
    hipLaunchKernelGGL((snap_score_kernel<false, 2>), sgrid, dim3(256), kSnapRingBytes, st, src, a);
  else
    hipLaunchKernelGGL((snap_score_kernel<false, 1>), sgrid, dim3(256), kSnapRingBytes, st, src, a);
  hipLaunchKernelGGL(snap_stats_kernel, dim3(units), dim3(kStatsT), 0, st, src, a);

  if (two_groups)
    hipLaunchKernelGGL((snap_score_kernel<true, 2>), sgrid, dim3(256), kSnapRingBytes + vote_bytes, st, src, a);
  else
    hipLaunchKernelGGL((snap_score_kernel<true, 1>), sgrid, dim3(256), kSnapRingBytes + vote_bytes, st, src, a);
  const dim3 pgrid((a.s_cap + kPoolTile - 1) / kPoolTile, units);
  hipLaunchKernelGGL(snap_pool_kernel, pgrid, dim3(256), 2 * (kPoolTile + 2 * a.pool_r) * sizeof(float), st,
                     src, a);
  if (a.s_cap <= ROCKETKV_MAX_PAGES) {
    hipLaunchKernelGGL(snap_select_fast_kernel, dim3(units), dim3(kSelT), 0, st, src, a);
  } else if (plan.sel_split > 0) {
    const int n_clear = units * (4 * 256 + 2 * plan.sel_split);
    hipLaunchKernelGGL(snap_split_zero_kernel, dim3((n_clear + 255) / 256), dim3(256), 0, st, a.sel_hist, n_clear);
    const dim3 hgrid(plan.sel_split, units);
    for (int pass = 0; pass < 4; ++pass)
      hipLaunchKernelGGL(snap_split_hist_kernel, hgrid, dim3(kSplitT), 0, st, src, a, pass);
    hipLaunchKernelGGL(snap_split_emit_kernel<false>, hgrid, dim3(kSplitT), 0, st, src, a);
    hipLaunchKernelGGL(snap_split_emit_kernel<true>, hgrid, dim3(kSplitT), 0, st, src, a);
  } else {
    hipLaunchKernelGGL(snap_select_kernel, dim3(units), dim3(kSelT), 0, st, src, a);
  }
  if (!dst) return hipGetLastError();  // filter only: the indices are the result
  const dim3 ggrid((keep + kGatherBlocks * kAttnPage - 1) / (kGatherBlocks * kAttnPage), units);
  hipLaunchKernelGGL(snap_gather_kernel, ggrid, dim3(256), 0, st, src, *dst, a);
  return hipGetLastError();
}

}  // namespace rkv
