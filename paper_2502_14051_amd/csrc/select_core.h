// HSA Step 2 (Algorithm 1 of arXiv 2502.14051, assignments i1, g, P, s1, i2) as a workgroup-level
// routine: one workgroup of NT threads handles one (sequence, KV head).  It picks the top-k1
// channels of the group-summed |q|, streams only those rows of the channel-major page summaries
// (K_max where the group-summed q is >= 0, K_min otherwise), forms one fp32 score per page in LDS
// and keeps the top-kp pages with an exact 4-pass radix select.  Ties go to the lower index in both
// picks; the page list comes out ascending.
//
// Traffic: k1 rows of P bf16 values, read as 16-byte runs of eight pages; everything else lives in
// LDS.  Summation order is fixed, so results are bit-reproducible run to run.  The routine is
// latency-bound (a chain of a few dependent memory and LDS round trips), hence the batched loads,
// the one-barrier radix passes and the lane-shift scans.
#pragma once

#include "common.h"

namespace rkv {

__device__ __forceinline__ uint32_t f32_order_key(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // larger float <=> larger unsigned key
}

template <int NT>
struct SelectShared {
  __align__(16) float s_abs[kHeadDim];
  float s_sum[kHeadDim];
  int s_chan[kHeadDim];
  float s_wgt[kHeadDim];
  int s_rank[NT];
  float partial[NT * 8];
  __align__(16) uint32_t hist[4][256];  // one histogram per radix pass
  uint32_t wsum[NT / kWave];
  uint32_t cnt0;
};

// exclusive prefix sum of one uint32 per thread over the NT-thread workgroup.  REUSE = false leaves
// out the trailing barrier, for a caller that does not touch `wsum` again before its next barrier.
template <int NT, bool REUSE = true>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wsum) {
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const uint32_t inc = wave_incl_scan(v);
  if (lane == kWave - 1) wsum[wave] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += wsum[w];
  if (REUSE) __syncthreads();
  return base + inc - v;
}

// accumulate eight rows' worth of eight-page runs.  The rows are j0 + t * jstep, t = 0..7, with
// `jbase` the smallest j0 of the workgroup in this batch: whether batch slot t holds a row at all is
// then the same for every thread (a scalar branch), and a thread whose own row falls beyond k1 reads
// the last picked row with weight zero.  The channel / weight lookups (LDS) all come first and the
// eight 16-byte loads go out back to back, so the batch costs one LDS and one memory round trip.
// (In the general routine the page that is receiving a token in the same launch gets its score from
// the tail-page routines below instead.)
template <bool STREAM = false>
__device__ __forceinline__ void score_rows8(const SelectArgs& a, const int* s_chan, const float* s_wgt,
                                            int64_t rows, int pages_cap, int o, int j0, int jbase, int jstep,
                                            float (&acc)[8]) {
  uint4 v[8];
  float w[8];
  int ch[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int j = j0 + t * jstep;
    const int jj = j < a.k1 ? j : a.k1 - 1;
    ch[t] = s_chan[jj];
    w[t] = s_wgt[jj];
    if (j >= a.k1) w[t] = 0.f;
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    v[t] = make_uint4(0, 0, 0, 0);
    if (jbase + t * jstep < a.k1) {  // uniform over the workgroup
      const bf16_t* row = (w[t] >= 0.f ? a.kmax : a.kmin) + (rows + ch[t]) * pages_cap + o * 8;
      v[t] = ld16<STREAM>(row);
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

// The score of the page that is receiving a token (tp.page) is computed on its own by the first two
// wavefronts from the page's old bounds and the new key, one picked channel per thread: the bound of
// a channel is the old one folded with the new key's value, or the new value alone when the token
// opens the page (whatever memory holds for that column is then not looked at).  Cheaper than
// patching the packed rows in every wavefront that scores them.  In two parts, so that the lookup of
// the old bound goes out before the caller's row loads and is used after them (one memory round trip
// for both): tail_page_load returns the old bound's bits, tail_page_finish leaves the two wavefronts'
// partial sums in out2[0..1]; the caller adds them (fixed order) after a barrier.
template <int NT>
__device__ __forceinline__ uint32_t tail_page_load(const SelectArgs& a, const int* s_chan, const float* s_wgt,
                                                 int64_t rows, int pages_cap, const TailPatch& tp) {
  const int tid = threadIdx.x;
  uint32_t old = 0;
  if (tp.page >= 0 && tp.slot != 0 && tid < a.k1)
    old = ((s_wgt[tid] >= 0.f) ? a.kmax : a.kmin)[(rows + s_chan[tid]) * pages_cap + tp.page];
  return old;
}
template <int NT>
__device__ __forceinline__ void tail_page_finish(const SelectArgs& a, const int* s_chan, const float* s_wgt,
                                                 const TailPatch& tp, uint32_t old, float* out2) {
  const int tid = threadIdx.x;
  if (tp.page < 0 || tid >= 2 * kWave) return;
  float contrib = 0.f;
  if (tid < a.k1) {
    const float w = s_wgt[tid];
    float f = bf16_to_f32(tp.knew[s_chan[tid]]);
    if (tp.slot != 0) {
      const float fo = bf16_to_f32((bf16_t)use_late(old));
      f = (w >= 0.f) ? fmaxf(fo, f) : fminf(fo, f);
    }
    contrib = w * f;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) contrib += __shfl_xor(contrib, off);
  if (tid % kWave == 0) out2[tid / kWave] = contrib;
}

// `weight` counts into `hist[bin]` for every lane with `on`, where many lanes of a wavefront may
// share a bin: up to two steps in which the first pending lane's bin is counted once for all lanes
// that hold it, then plain atomics for whatever is left.
__device__ __forceinline__ void hist_add_grouped(uint32_t* hist, uint32_t bin, bool on, uint32_t weight = 1u) {
  const int lane = threadIdx.x % kWave;
  unsigned long long todo = __ballot(on);
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    if (todo == 0) break;  // the same for the whole wavefront
    const int leader = __ffsll((long long)todo) - 1;
    const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);
    const unsigned long long same = __ballot(on && bin == b);
    if (lane == leader) atomicAdd(&hist[b], weight * (uint32_t)__popcll(same));
    on = on && bin != b;
    todo &= ~same;
  }
  if (on) atomicAdd(&hist[bin], weight);
}

// The unit's q at channel `tid` for every head of the group (threads below 128), requested but not
// used here: a caller can put its own loads behind these before anything waits, so that all of them
// share one memory round trip.  Heads beyond the group re-read head 0 (and are ignored later); the
// blocks of heads are skipped by branches that are the same for the whole workgroup.
__device__ __forceinline__ void load_q_column(const CacheView& c, const SelectArgs& a, int unit,
                                              uint32_t (&qv)[kMaxGroup]) {
  const int tid = threadIdx.x;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int G = c.group;
#pragma unroll
  for (int h = 0; h < kMaxGroup; ++h) qv[h] = 0;
  if (tid < kHeadDim) {
    const bf16_t* qp = a.q + ((int64_t)b * c.n_q_heads + (int64_t)g * G) * kHeadDim + tid;
#pragma unroll
    for (int h = 0; h < 4; ++h) qv[h] = qp[(h < G ? h : 0) * kHeadDim];
    if (G > 4) {
#pragma unroll
      for (int h = 4; h < 8; ++h) qv[h] = qp[(h < G ? h : 0) * kHeadDim];
    }
    if (G > 8) {
#pragma unroll
      for (int h = 8; h < kMaxGroup; ++h) qv[h] = qp[(h < G ? h : 0) * kHeadDim];
    }
  }
}

// Step 2, first half (needs only q): a = sum_h |q|, s = sum_h q, i1 = top-k1 channels of a, left in
// sh.s_chan / sh.s_wgt.  `qv` comes from load_q_column.  All NT threads of the workgroup take part;
// ends with a barrier.
template <int NT>
__device__ __forceinline__ void select_channels(const CacheView& c, const SelectArgs& a, int unit,
                                                SelectShared<NT>& sh, bool write_global,
                                                const uint32_t (&qv)[kMaxGroup]) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int G = c.group;

#pragma unroll
  for (int i = 0; i < 4 * 256 / NT; ++i) (&sh.hist[0][0])[tid + i * NT] = 0;

  // ---- a[c] = sum_h |q|, s[c] = sum_h q (fp32, head order) -----------------------------------
  if (tid < kHeadDim) {
    float sa = 0.f, ss = 0.f;
#pragma unroll
    for (int h = 0; h < kMaxGroup; ++h) {
      const float x = h < G ? bf16_to_f32((bf16_t)qv[h]) : 0.f;
      sa += fabsf(x);
      ss += x;
    }
    sh.s_abs[tid] = sa;
    sh.s_sum[tid] = ss;
  }
  __syncthreads();
  // ---- i1: rank by counting ---------------------------------------------------------------------
  // kParts neighbouring lanes rank one channel against a slice of the channels each (4 LDS values per
  // read) and add up; ranks are unique (ties go to the lower channel), so the k1 picked channels go
  // straight to slot `rank`: no compaction, and the order of the score sums stays fixed.
  constexpr int kParts = NT / kHeadDim, kSlice = kHeadDim / kParts;
  {
    const int ch = tid / kParts, part = tid % kParts;
    const float mine = sh.s_abs[ch];
    const float4* v4 = reinterpret_cast<const float4*>(sh.s_abs + part * kSlice);
    int rank = 0;
#pragma unroll
    for (int i = 0; i < kSlice / 4; ++i) {
      const float4 v = v4[i];
      const int o = part * kSlice + 4 * i;
      rank += (v.x > mine) || (v.x == mine && o + 0 < ch);
      rank += (v.y > mine) || (v.y == mine && o + 1 < ch);
      rank += (v.z > mine) || (v.z == mine && o + 2 < ch);
      rank += (v.w > mine) || (v.w == mine && o + 3 < ch);
    }
#pragma unroll
    for (int off = 1; off < kParts; off <<= 1) rank += __shfl_xor(rank, off);
    if (part == 0) {
      sh.s_rank[ch] = rank;
      if (rank < a.k1) {
        sh.s_chan[rank] = ch;
        sh.s_wgt[rank] = sh.s_sum[ch];
      }
    }
  }
  __syncthreads();
  // the caller's copy of i1 is ascending by channel: compacted here, only when it is asked for
  if (write_global && a.out_channels) {
    bool sel = false;
    if (tid < kHeadDim) sel = sh.s_rank[tid] < a.k1;
    const unsigned long long bal = __ballot(sel);
    if (tid == 0) sh.cnt0 = (uint32_t)__popcll(bal);
    __syncthreads();
    if (sel) {
      const int pos = __popcll(bal & ((1ull << lane) - 1ull)) + (wave == 1 ? (int)sh.cnt0 : 0);
      a.out_channels[(int64_t)unit * a.k1 + pos] = tid;
    }
  }
}

// The kp-th largest of the P order keys in `keys` (LDS) by four 8-bit radix passes, as (tau, need_eq):
// the selection is every key above tau plus the first need_eq keys equal to it.  Needs kp < P and
// `hist` (LDS, 4 x 256 counters, 16-byte aligned) zeroed; every thread gets the result.
// FIRST_DONE: the caller has already counted every key's top digit into hist[0] (and synchronised).
template <int NT, bool FIRST_DONE = false>
__device__ __forceinline__ void radix_threshold(const uint32_t* keys, int P, int kp, uint32_t (*hist)[256],
                                                uint32_t& tau, uint32_t& need_eq) {
  const int tid = threadIdx.x, lane = tid % kWave;
  uint32_t prefix = 0, mask = 0, k = (uint32_t)kp;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (!(FIRST_DONE && pass == 0)) {
      for (int p = tid; p < P; p += NT) {
        const uint32_t key = keys[p];
        if ((key & mask) == prefix) atomicAdd(&hist[pass][(key >> shift) & 255u], 1u);
      }
      __syncthreads();
    }
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

template <int NT, int ROUNDS>
__device__ __forceinline__ int select_pages_small(const CacheView& c, const SelectArgs& a, int unit, int n,
                                                  SelectShared<NT>& sh, uint32_t* keys, int32_t* list_lds,
                                                  bool write_global, const TailPatch& tp);

// Step 2, second half for a sequence of n tokens: page scores from the picked summary rows, exact
// top-kp pages.  `keys` is LDS scratch of ceil8(pages_cap) words.  The ascending list goes to
// `list_lds` (if not null, kp entries) and, when `write_global`, to a.out_pages / a.out_pages2 (-1
// padded) and the optional score output.  Returns kp.  Ends WITHOUT a final barrier: the caller
// synchronises before reading `list_lds`.
template <int NT>
__device__ __forceinline__ int select_pages(const CacheView& c, const SelectArgs& a, int unit, int n,
                                            SelectShared<NT>& sh, uint32_t* keys, int32_t* list_lds,
                                            bool write_global, const TailPatch& tp) {
  // (the same for the whole launch)
  if (c.pages_cap <= 2 * NT) return select_pages_small<NT, 2>(c, a, unit, n, sh, keys, list_lds, write_global, tp);
  if (c.pages_cap <= 5 * NT) return select_pages_small<NT, 5>(c, a, unit, n, sh, keys, list_lds, write_global, tp);
  const int tid = threadIdx.x;
  const int ps = c.page_size;
  int P = (n + ps - 1) / ps;
  if (P > c.pages_cap) P = c.pages_cap;
  int kp = pages_to_pick(n, ps, a.T);
  if (kp > P) kp = P;
  if (kp > a.row_len) kp = a.row_len;
  if (write_global) {
    // -1 padding of the list rows beyond kp
    if (a.out_pages)
      for (int i = kp + tid; i < a.row_len; i += NT) a.out_pages[(int64_t)unit * a.row_len + i] = -1;
    if (a.out_pages2)
      for (int i = kp + tid; i < a.row_len2; i += NT) a.out_pages2[(int64_t)unit * a.row_len2 + i] = -1;
  }
  if (P == 0) return 0;
  const int n_rec = min(a.n_recent, kp);  // no more forced pages than pages picked: the newest ones win

  // ---- s1: page scores ---------------------------------------------------------------------------
  const int n_oct = (P + 7) / 8;
  const int64_t rows = (int64_t)unit * kHeadDim;
  float* out_scores = write_global ? a.out_scores : nullptr;
  float* tail2 = sh.s_abs;  // free since the channel pick ended; [0..1]: the two halves of tp.page's score
  // the old bounds of tp.page: requested ahead of the row loads, used after them
  const uint32_t tail_old = tail_page_load<NT>(a, sh.s_chan, sh.s_wgt, rows, c.pages_cap, tp);
  if (n_oct < NT) {
    int npow = 1;
    while (npow < n_oct) npow <<= 1;
    const int R = NT / npow;  // row groups summed separately, then in order
    const int r = tid / npow, o = tid % npow;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    if (o < n_oct)
      for (int jb = 0; jb < a.k1; jb += 8 * R)
        score_rows8(a, sh.s_chan, sh.s_wgt, rows, c.pages_cap, o, jb + r, jb, R, acc);
    tail_page_finish<NT>(a, sh.s_chan, sh.s_wgt, tp, tail_old, tail2);
    RKV_STAMP(2);
#pragma unroll
    for (int i = 0; i < 8; ++i) sh.partial[(r * npow + o) * 8 + i] = acc[i];
    __syncthreads();
    for (int p = tid; p < npow * 8; p += NT) {
      float s = 0.f;
      for (int rr = 0; rr < R; ++rr) s += sh.partial[rr * npow * 8 + p];
      if (p == tp.page) s = tail2[0] + tail2[1];
      if (p < n_oct * 8) {
        if (p < P && out_scores) out_scores[(int64_t)unit * c.pages_cap + p] = s;
        if (p >= P) s = -INFINITY;
        else if (p >= P - n_rec) s = INFINITY;
        const uint32_t key = f32_order_key(s);
        keys[p] = key;
        if (p < P) atomicAdd(&sh.hist[0][key >> 24], 1u);  // the first radix pass, counted on the way
      }
    }
  } else {
    tail_page_finish<NT>(a, sh.s_chan, sh.s_wgt, tp, tail_old, tail2);
    __syncthreads();  // tail2 is read below
    for (int o = tid; o < n_oct; o += NT) {
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
      for (int j0 = 0; j0 < a.k1; j0 += 8)
        score_rows8(a, sh.s_chan, sh.s_wgt, rows, c.pages_cap, o, j0, j0, 1, acc);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int p = o * 8 + i;
        float s = acc[i];
        if (p == tp.page) s = tail2[0] + tail2[1];
        if (p < P && out_scores) out_scores[(int64_t)unit * c.pages_cap + p] = s;
        if (p >= P) s = -INFINITY;
        else if (p >= P - n_rec) s = INFINITY;
        const uint32_t key = f32_order_key(s);
        keys[p] = key;
        if (p < P) atomicAdd(&sh.hist[0][key >> 24], 1u);  // the first radix pass, counted on the way
      }
    }
  }
  __syncthreads();

  // ---- i2: exact kp-th largest key by 4 x 8-bit radix passes -------------------------------------
  RKV_STAMP(3);
  uint32_t tau = 0, need_eq = (uint32_t)P;  // defaults select everything (kp == P)
  if (kp < P) radix_threshold<NT, true>(keys, P, kp, sh.hist, tau, need_eq);
  RKV_STAMP(4);

  // ---- emit ascending: every key > tau, plus the first need_eq keys == tau -----------------------
  const int ipt = (P + NT - 1) / NT;
  const int lo = min(P, tid * ipt), hi = min(P, lo + ipt);
  uint32_t cnt = 0;  // low 16 bits: keys > tau, high 16 bits: keys == tau
  for (int p = lo; p < hi; ++p) {
    const uint32_t key = keys[p];
    cnt += (key > tau) ? 1u : 0u;
    cnt += (key == tau) ? 0x10000u : 0u;
  }
  const uint32_t before = block_excl_scan<NT, false>(cnt, sh.wsum);  // the caller's barrier follows
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
        if (list_lds) list_lds[pos] = p;
        if (write_global) {
          if (a.out_pages) a.out_pages[(int64_t)unit * a.row_len + pos] = p;
          if (a.out_pages2 && (int)pos < a.row_len2) a.out_pages2[(int64_t)unit * a.row_len2 + pos] = p;
        }
      }
    }
    if (key > tau) ++gt;
  }
  return kp;
}

// Step 2, second half, for caches of at most ROUNDS * NT pages (every fused decode launch of the usual
// shapes): the same result as select_pages, arranged for latency.  The routine sits in front of the
// K/V stream with HBM idle, so what counts is the number of dependent steps, not the work:
//   - eight neighbouring lanes share an eight-page run and split the picked rows between them; the
//     row sums meet in three lane-exchange steps (no LDS, no barrier) and lane r keeps page r of the
//     run, so thread t holds the scores of pages t, NT + t, ... (one per round); the stale
//     bound of a page that is receiving a token is patched in the loaded rows, no extra loads;
//   - the kp-th largest score is found by counting into 1024 equal-width value bins between the
//     smallest and the largest finite score (the forced recent pages, +inf, in the top bin): one
//     histogram, scanned by every wavefront for itself.  Binning is monotone, so every page above the
//     threshold's bin is in, every page below is out, and only the few pages sharing that bin are
//     ranked exactly (by order key, ties to the lower page).  Page scores of one cache differ in
//     their mantissas, not their exponents: radix digits pile them onto a few counters (hundreds of
//     LDS atomics on one address), value bins spread them;
//   - scores without a finite range, or more than 64 pages in the threshold's bin, go through the
//     radix passes of the general routine instead.
// Ends WITHOUT a final barrier, like select_pages.
template <int NT, int ROUNDS>
__device__ __forceinline__ int select_pages_small(const CacheView& c, const SelectArgs& a, int unit, int n,
                                                  SelectShared<NT>& sh, uint32_t* keys, int32_t* list_lds,
                                                  bool write_global, const TailPatch& tp) {
  constexpr int kRuns = NT / 8;   // eight-page runs per round
  constexpr int kRounds = ROUNDS;
  constexpr int kWaves = NT / kWave;
  constexpr int kCandMax = 64;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int ps = c.page_size;
  int P = (n + ps - 1) / ps;
  if (P > c.pages_cap) P = c.pages_cap;
  int kp = pages_to_pick(n, ps, a.T);
  if (kp > P) kp = P;
  if (kp > a.row_len) kp = a.row_len;
  if (write_global) {
    if (a.out_pages)
      for (int i = kp + tid; i < a.row_len; i += NT) a.out_pages[(int64_t)unit * a.row_len + i] = -1;
    if (a.out_pages2)
      for (int i = kp + tid; i < a.row_len2; i += NT) a.out_pages2[(int64_t)unit * a.row_len2 + i] = -1;
  }
  if (P == 0) return 0;
  const int n_rec = min(a.n_recent, kp);  // no more forced pages than pages picked: the newest ones win
  const int n_oct = (P + 7) / 8;
  const int64_t rows = (int64_t)unit * kHeadDim;
  const int o = tid / 8, r = tid % 8;
  // scratch words in sh.partial (unused by the channel pick): candidate keys, their counter, the
  // wavefronts' score ranges and emission counts
  uint32_t* scr = reinterpret_cast<uint32_t*>(sh.partial);
  uint32_t* cand = scr;                                         // [kCandMax]
  uint32_t* cand_n = scr + kCandMax;                            // [1]
  float* wlo = reinterpret_cast<float*>(scr + kCandMax + 8);    // [kWaves]
  float* whi = wlo + kWaves;                                    // [kWaves]
  uint32_t* wcnt = scr + kCandMax + 8 + 2 * kWaves;             // [kRounds][kWaves]

  // ---- s1: page scores.  Thread (o, r) = (tid / 8, tid % 8) takes the rows r, r + 8, ... of the picked
  // channels for the runs o, o + kRuns, ... (one per round); the loads of every round go out before the
  // first is used, so the rounds share one memory round trip.
  float score[kRounds];
  {
    constexpr int kBatch = 4;  // rows of a thread whose loads are in flight together, for every round (registers)
    float acc[kRounds][8];
    float tail_acc = 0.f;  // the score of the page that is receiving a token, if this thread's run holds it
#pragma unroll
    for (int i = 0; i < kRounds; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[i][e] = 0.f;
    const int patch_round = tp.page >= 0 ? (tp.page / 8) / kRuns : -1;
    const int patch_col = (tp.page >= 0 && (tp.page / 8) % kRuns == o) ? tp.page % 8 : -1;  // in round patch_round
    for (int jb = 0; jb < a.k1; jb += 8 * kBatch) {
      float w[kBatch];
      int ch[kBatch];
      uint32_t knew[kBatch];  // the new key at the rows' channels (only with a token being appended)
#pragma unroll
      for (int t = 0; t < kBatch; ++t) {
        const int j = jb + r + t * 8;
        const int jj = j < a.k1 ? j : a.k1 - 1;  // a row beyond k1: the last picked row again, weight zero
        ch[t] = sh.s_chan[jj];
        w[t] = sh.s_wgt[jj];
        if (j >= a.k1) w[t] = 0.f;
      }
#pragma unroll
      for (int t = 0; t < kBatch; ++t) knew[t] = tp.page >= 0 ? (uint32_t)tp.knew[ch[t]] : 0u;
      const bf16_t* row[kBatch];
#pragma unroll
      for (int t = 0; t < kBatch; ++t) row[t] = (w[t] >= 0.f ? a.kmax : a.kmin) + (rows + ch[t]) * c.pages_cap + o * 8;
      uint4 v[kRounds][kBatch];
#pragma unroll
      for (int i = 0; i < kRounds; ++i)
#pragma unroll
        for (int t = 0; t < kBatch; ++t) {
          v[i][t] = make_uint4(0, 0, 0, 0);
          // (the first two conditions are the same for the whole workgroup)
          if (i * kRuns < n_oct && jb + t * 8 < a.k1 && i * kRuns + o < n_oct) v[i][t] = ld16<false>(row[t] + i * NT);
        }
      // The bound the rows hold for a page that is receiving a token is stale: the threads whose run
      // holds it also fetch that one bound of each of their rows on its own (a 2-byte load out of a
      // line the row load brings in anyway) and sum up the page's score from the bounds folded with the
      // new key, or from the new key alone when the token opens the page (slot 0: what memory holds
      // for that column is not looked at).  Only the wavefront that holds the page takes the branch.
      if (tp.page >= 0 && __any(patch_col >= 0)) {
        uint32_t old[kBatch];
#pragma unroll
        for (int t = 0; t < kBatch; ++t) {
          old[t] = 0;
          if (patch_col >= 0 && tp.slot != 0 && jb + t * 8 < a.k1) old[t] = row[t][patch_round * NT + patch_col];
        }
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < kBatch; ++t) {
          const float fn = bf16_to_f32((bf16_t)knew[t]);
          float f = fn;
          if (tp.slot != 0) {
            const float fo = bf16_to_f32((bf16_t)old[t]);
            f = w[t] >= 0.f ? fmaxf(fo, fn) : fminf(fo, fn);
          }
          sum = fmaf(w[t], f, sum);
        }
        if (patch_col >= 0) tail_acc += sum;
      }
#pragma unroll
      for (int i = 0; i < kRounds; ++i)
#pragma unroll
        for (int t = 0; t < kBatch; ++t) {
          const uint32_t x[4] = {v[i][t].x, v[i][t].y, v[i][t].z, v[i][t].w};
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            acc[i][2 * q4] = fmaf(w[t], bf16lo_to_f32(x[q4]), acc[i][2 * q4]);
            acc[i][2 * q4 + 1] = fmaf(w[t], bf16hi_to_f32(x[q4]), acc[i][2 * q4 + 1]);
          }
        }
    }
    // the eight lanes of a run add up their row groups: lane pairs, quads, then the two quads; every
    // lane ends with the same sums, formed in the same order; lane r keeps page r of the run
    const auto lanes8 = [](float x) {
      x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, false));   // quad_perm 1,0,3,2
      x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, false));   // quad_perm 2,3,0,1
      x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, false));  // row_half_mirror
      return x;
    };
    if (tp.page >= 0) tail_acc = lanes8(tail_acc);  // (the same for the whole workgroup)
#pragma unroll
    for (int i = 0; i < kRounds; ++i) {
      score[i] = 0.f;
      if (i * kRuns < n_oct) {  // the same for the whole workgroup
        float mine = lanes8(acc[i][0]);
#pragma unroll
        for (int e = 1; e < 8; ++e) {
          const float x = lanes8(acc[i][e]);
          mine = r == e ? x : mine;
        }
        if (i == patch_round && patch_col == r) mine = tail_acc;
        score[i] = mine;
      }
    }
  }
  RKV_STAMP(2);

  // ---- order keys, and the range of the finite scores ---------------------------------------------
  float* out_scores = write_global ? a.out_scores : nullptr;
  uint32_t key[kRounds];
  float val[kRounds];
  bool live[kRounds];
  float lo = INFINITY, hi = -INFINITY;
#pragma unroll
  for (int i = 0; i < kRounds; ++i) {
    const int p = i * NT + tid;
    live[i] = p < P;
    float sc = score[i];
    if (live[i] && out_scores) out_scores[(int64_t)unit * c.pages_cap + p] = sc;
    if (live[i] && p >= P - n_rec) sc = INFINITY;
    val[i] = sc;
    key[i] = live[i] ? f32_order_key(sc) : 0u;
    if (live[i] && fabsf(sc) < INFINITY) {
      lo = fminf(lo, sc);
      hi = fmaxf(hi, sc);
    }
  }
  uint32_t tau = 0, need_eq = (uint32_t)P;  // defaults select everything (kp == P)
  bool by_bin = false;                     // picked by bin alone: every page of the threshold's bin is in
  int bstar = 0;
  int bin[kRounds];
#pragma unroll
  for (int i = 0; i < kRounds; ++i) bin[i] = 0;
  if (kp < P) {
    lo = wave_min_f32(lo);
    hi = wave_max_f32(hi);
    if (lane == 0) {
      wlo[wave] = lo;
      whi[wave] = hi;
    }
    if (tid == 0) *cand_n = 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      lo = fminf(lo, wlo[w]);
      hi = fmaxf(hi, whi[w]);
    }
    // bins, and bins per lane of a scanning wavefront.  Every wavefront walks its lanes' bins one after
    // the other, so fewer bins make a shorter scan and more pages per bin a longer exact rank; with at
    // most two pages per thread 256 bins measured 0.4 us ahead of 1024 at the benchmark shape.
    constexpr int NB = ROUNDS <= 2 ? 256 : 1024, BPL = NB / kWave;
    const float scale = (float)(NB - 2) / (hi - lo);
    bool decided = (hi > lo) && (scale < 3.0e38f);  // the same for every thread
    if (decided) {
      uint32_t* hist = &sh.hist[0][0];  // 4 x 256 counters, all zero since the channel pick
#pragma unroll
      for (int i = 0; i < kRounds; ++i) {
        // clamped as a float, so that -inf, +inf and NaN never reach the conversion
        int b = (int)fminf(fmaxf((val[i] - lo) * scale, 0.f), (float)(NB - 2));
        if (val[i] == INFINITY) b = NB - 1;
        bin[i] = b;
        if (live[i]) atomicAdd(&hist[b], 1u);
      }
      __syncthreads();
      // every wavefront finds the bin of the kp-th largest for itself: lane L owns the BPL bins below
      // NB - L * BPL, so a prefix sum over the lanes counts the pages in higher bins
      const int btop = NB - 1 - lane * BPL;  // the lane's highest bin
      uint32_t hc[BPL], total = 0;
#pragma unroll
      for (int v = 0; v < BPL / 4; ++v) {
        const uint4 h = *reinterpret_cast<const uint4*>(&hist[btop - 4 * v - 3]);
        hc[4 * v + 0] = h.w;
        hc[4 * v + 1] = h.z;
        hc[4 * v + 2] = h.y;
        hc[4 * v + 3] = h.x;
        total += h.x + h.y + h.z + h.w;
      }
      uint32_t above = wave_incl_scan(total) - total;
      int found = -1;
      uint32_t need = 0, cnum = 0;
#pragma unroll
      for (int j = 0; j < BPL; ++j) {  // j = 0: the lane's highest bin
        if (above < (uint32_t)kp && (uint32_t)kp <= above + hc[j]) {
          found = btop - j;
          need = (uint32_t)kp - above;
          cnum = hc[j];
        }
        above += hc[j];
      }
      const int src = __ffsll((long long)__ballot(found >= 0)) - 1;
      bstar = __builtin_amdgcn_readlane(found, src);
      need = (uint32_t)__builtin_amdgcn_readlane((int)need, src);
      cnum = (uint32_t)__builtin_amdgcn_readlane((int)cnum, src);
      if (cnum == need) {
        by_bin = true;
      } else if (cnum <= (uint32_t)kCandMax) {
        // exact rank among the pages of the threshold's bin
#pragma unroll
        for (int i = 0; i < kRounds; ++i)
          if (live[i] && bin[i] == bstar) cand[atomicAdd(cand_n, 1u)] = key[i];
        __syncthreads();
        const uint32_t ki = lane < (int)cnum ? cand[lane] : 0u;
        uint32_t gt = 0, ge = 0;
        for (uint32_t j = 0; j < cnum; ++j) {
          const uint32_t kj = cand[j];
          gt += kj > ki;
          ge += kj >= ki;
        }
        const bool is_tau = lane < (int)cnum && gt < need && need <= ge;  // equal keys give the same pair
        const int who = __ffsll((long long)__ballot(is_tau)) - 1;
        tau = (uint32_t)__builtin_amdgcn_readlane((int)ki, who);
        need_eq = need - (uint32_t)__builtin_amdgcn_readlane((int)gt, who);
      } else {
        decided = false;
      }
    }
    if (!decided) {
      // the general routine's radix passes, on the keys in LDS
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kRounds; ++i)
        if (live[i]) keys[i * NT + tid] = key[i];
      for (int i = tid; i < 4 * 256; i += NT) (&sh.hist[0][0])[i] = 0;
      __syncthreads();
      radix_threshold<NT, false>(keys, P, kp, sh.hist, tau, need_eq);
      bstar = -1;  // every live page is ranked by its key
    }
  }
  RKV_STAMP(3);

  // ---- emit ascending.  Page order is (round, thread) order: a prefix sum over the threads per round.
  // In: every page above the threshold (by bin, then by key), plus the first need_eq pages equal to it.
  uint32_t cnt[kRounds];  // low 16 bits: pages above the threshold, high 16 bits: pages equal to it
  bool above_t[kRounds], equal_t[kRounds];
#pragma unroll
  for (int i = 0; i < kRounds; ++i) {
    if (kp >= P) {
      above_t[i] = false;
      equal_t[i] = live[i];  // key == tau is not needed: need_eq == P takes every live page
    } else if (by_bin) {
      above_t[i] = live[i] && bin[i] >= bstar;
      equal_t[i] = false;
    } else if (bstar >= 0) {
      above_t[i] = live[i] && (bin[i] > bstar || (bin[i] == bstar && key[i] > tau));
      equal_t[i] = live[i] && bin[i] == bstar && key[i] == tau;
    } else {
      above_t[i] = live[i] && key[i] > tau;
      equal_t[i] = live[i] && key[i] == tau;
    }
    cnt[i] = (above_t[i] ? 1u : 0u) + (equal_t[i] ? 0x10000u : 0u);
  }
  if (by_bin) need_eq = 0;
  uint32_t inc[kRounds];
#pragma unroll
  for (int i = 0; i < kRounds; ++i) {
    inc[i] = 0;
    if (i * NT < P) {  // the same for the whole workgroup
      inc[i] = wave_incl_scan(cnt[i]);
      if (lane == kWave - 1) wcnt[i * kWaves + wave] = inc[i];
    }
  }
  __syncthreads();
  uint32_t base = 0;  // counts of everything in front of this thread's page of the round at hand
#pragma unroll
  for (int i = 0; i < kRounds; ++i) {
    if (i * NT >= P) break;
    uint32_t before = base;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t x = wcnt[i * kWaves + w];
      if (w < wave) before += x;
      base += x;
    }
    before += inc[i] - cnt[i];
    const uint32_t gt = before & 0xffffu, eq = before >> 16;
    const bool take = above_t[i] || (equal_t[i] && eq < need_eq);
    if (take) {
      const uint32_t pos = gt + (equal_t[i] ? eq : min(eq, need_eq));
      const int p = i * NT + tid;
      if ((int)pos < kp) {
        if (list_lds) list_lds[pos] = p;
        if (write_global) {
          if (a.out_pages) a.out_pages[(int64_t)unit * a.row_len + pos] = p;
          if (a.out_pages2 && (int)pos < a.row_len2) a.out_pages2[(int64_t)unit * a.row_len2 + pos] = p;
        }
      }
    }
  }
  RKV_STAMP(4);
  return kp;
}

__device__ __forceinline__ float f32_from_order_key(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// Step 2's top-k (Algorithm 1, i2) on page scores that an earlier launch left in a.in_scores: the
// pick of the large-summary path.  A thread keeps its contiguous run of a few scores in registers
// from the one batch of loads to the ordered emission, so no pass waits on LDS reads.
//
// The kp-th largest score is found by counting, not by radix digits: one pass over 1023 equal-width
// value bins between the smallest and the largest finite score (+inf, the forced recent pages, has a
// bin of its own), a scan over the bins, then an exact rank among the few scores that share the bin
// of the kp-th.  Page scores differ in their low mantissa bits rather than in their exponents, so
// value bins spread them where the leading radix digits would pile them into one or two counters.
// Binning is monotone, hence the result is exactly the radix select's, ties to the lower page
// included.  Scores without a finite range, or more than 1024 of them in that one bin, fall back to
// radix passes over the same registers.  Up to ROCKETKV_MAX_PAGES pages.
template <int NT>
struct PickShared {
  __align__(16) uint32_t hist[4][256];  // 1024 value bins, or the four radix histograms of the fallback
  uint32_t cand[1024];
  float wmin[NT / kWave], wmax[NT / kWave];
  uint32_t wsum[NT / kWave];
  int found[6];
  uint32_t cnt0;
};

// COHERENT: the scores were written earlier in the SAME launch by other workgroups (with device-scope
// write-through stores): they are read with device-scope loads, which do not trust this XCD's L2.
// kVec: float4 loads per thread, i.e. NT * kVec * 4 >= pages_cap (the wrapper below picks it).
// sh.hist must be all zero on entry (the caller clears it, and synchronises, before the call).
// SKEWED: for values that pile up in a few exponents with a long tail above them (attention votes),
// where equal-width value bins would put nearly everything into the lowest one: the bins are laid
// on the ordered bit pattern instead, and the radix fallback counts with hist_add_grouped.
template <int NT, bool COHERENT, int kVec, bool SKEWED = false>
__device__ __forceinline__ void pick_from_scores_n(const CacheView& c, const SelectArgs& a, int unit, int n,
                                                   PickShared<NT>& sh) {
  constexpr int NB = 1024, BPT = NB / NT, CAP = 1024;
  static_assert(kVec >= 1 && NB % NT == 0, "thread count does not fit the pick");
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  // ---- this thread's run of pages, [4 * v_begin, 4 * v_begin + 4 * per), laid out on pages_cap so
  // that the loads go out before the sequence length is known ---------------------------------------
  const int per = (c.pages_cap / 4 + NT - 1) / NT;  // rows hold pages_cap (a multiple of 8) floats
  const int v_begin = tid * per;
  const float4* in4 = reinterpret_cast<const float4*>(a.in_scores + (int64_t)unit * c.pages_cap);
  float4 v[kVec];
#pragma unroll
  for (int i = 0; i < kVec; ++i) {
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < per && (v_begin + i) * 4 < c.pages_cap) {
      if (COHERENT) {
        const float* f = reinterpret_cast<const float*>(in4 + v_begin + i);
        v[i] = make_float4(__hip_atomic_load(f + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                           __hip_atomic_load(f + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                           __hip_atomic_load(f + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                           __hip_atomic_load(f + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      } else {
        v[i] = in4[v_begin + i];
      }
    }
  }
  const int ps = c.page_size;
  int P = (n + ps - 1) / ps;
  if (P > c.pages_cap) P = c.pages_cap;
  int kp = pages_to_pick(n, ps, a.T);
  if (kp > P) kp = P;
  if (kp > a.row_len) kp = a.row_len;
  if (a.out_pages)
    for (int i = kp + tid; i < a.row_len; i += NT) a.out_pages[(int64_t)unit * a.row_len + i] = -1;
  if (a.out_pages2)
    for (int i = kp + tid; i < a.row_len2; i += NT) a.out_pages2[(int64_t)unit * a.row_len2 + i] = -1;
  if (P == 0) return;
  const int n_rec = min(a.n_recent, kp);  // no more forced pages than pages picked: the newest ones win
  uint32_t key[kVec * 4];
  float lo = INFINITY, hi = -INFINITY;
#pragma unroll
  for (int i = 0; i < kVec; ++i) {
    const float x[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int pg = (v_begin + i) * 4 + e;
      const bool live = i < per && pg < P;
      float sc = live ? x[e] : -INFINITY;
      if (live && pg >= P - n_rec) sc = INFINITY;
      key[i * 4 + e] = f32_order_key(sc);
      if (live) {
        if (fabsf(sc) < INFINITY) {
          lo = fminf(lo, sc);
          hi = fmaxf(hi, sc);
        }
      }
    }
  }
  // `live` again, as a test on the register index alone
  const auto is_live = [&](int r) { return r / 4 < per && (v_begin + r / 4) * 4 + (r & 3) < P; };

  uint32_t tau = 0, need_eq = (uint32_t)P;  // defaults select everything (kp == P)
  if (kp < P) {
    uint32_t* hist = &sh.hist[0][0];
    uint32_t* cand = sh.cand;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      lo = fminf(lo, __shfl_xor(lo, off));
      hi = fmaxf(hi, __shfl_xor(hi, off));
    }
    if (lane == 0) {
      sh.wmin[wave] = lo;
      sh.wmax[wave] = hi;
    }
    if (tid == 0) sh.cnt0 = 0;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NT / kWave; ++w) {
      lo = fminf(lo, sh.wmin[w]);
      hi = fmaxf(hi, sh.wmax[w]);
    }
    // SKEWED: equal-width bins on the ordered bit pattern instead of the value, i.e. roughly on its
    // logarithm, which is just as monotone
    const uint32_t klo = f32_order_key(lo);
    const float scale = SKEWED ? (float)(NB - 1) / (float)(f32_order_key(hi) - klo) : (float)(NB - 1) / (hi - lo);
    bool decided = (hi > lo) && (scale < 3.0e38f);  // same for every thread
    if (decided) {
      const auto bin_of = [&](uint32_t k) -> int {
        const float f = f32_from_order_key(k);
        if (f == INFINITY) return NB - 1;
        // (a masked-out entry lies below klo: the difference wraps, the clamp catches it)
        const int b = SKEWED ? (int)fminf((float)(k - klo) * scale, (float)(NB - 2)) : (int)((f - lo) * scale);
        return min(max(b, 0), NB - 2);
      };
      int bin[kVec * 4];
#pragma unroll
      for (int r = 0; r < kVec * 4; ++r) {
        bin[r] = bin_of(key[r]);
        if (is_live(r)) atomicAdd(&hist[bin[r]], 1u);
      }
      __syncthreads();
      // thread t owns the BPT bins below NB - t*BPT: a prefix sum over threads counts the bins above
      uint32_t h[BPT], total = 0;
#pragma unroll
      for (int j = 0; j < BPT; ++j) {
        h[j] = hist[NB - 1 - tid * BPT - j];  // j = 0: the thread's highest bin
        total += h[j];
      }
      uint32_t above = block_excl_scan<NT>(total, sh.wsum);
#pragma unroll
      for (int j = 0; j < BPT; ++j) {
        if (above < (uint32_t)kp && (uint32_t)kp <= above + h[j]) {
          sh.found[0] = NB - 1 - tid * BPT - j;
          sh.found[1] = (int)((uint32_t)kp - above);
          sh.found[2] = (int)h[j];
        }
        above += h[j];
      }
      __syncthreads();
      const int bstar = sh.found[0], need = sh.found[1], cnum = sh.found[2];
      decided = cnum <= CAP;
      if (decided) {
#pragma unroll
        for (int r = 0; r < kVec * 4; ++r)
          if (is_live(r) && bin[r] == bstar) cand[atomicAdd(&sh.cnt0, 1u)] = key[r];
        __syncthreads();
        for (int i = tid; i < cnum; i += NT) {
          const uint32_t ki = cand[i];
          int gt = 0, ge = 0;
          for (int j = 0; j < cnum; ++j) {
            const uint32_t kj = cand[j];
            gt += kj > ki;
            ge += kj >= ki;
          }
          if (gt < need && need <= ge) {  // ki is the need-th largest; equal keys write the same pair
            sh.found[4] = (int)ki;
            sh.found[5] = need - gt;
          }
        }
        __syncthreads();
        tau = (uint32_t)sh.found[4];
        need_eq = (uint32_t)sh.found[5];
      }
    }
    if (!decided) {
      // four 8-bit radix passes over the keys in registers (same scan as radix_threshold)
      __syncthreads();
      for (int i = tid; i < 4 * 256; i += NT) hist[i] = 0;
      __syncthreads();
      uint32_t prefix = 0, mask = 0, k = (uint32_t)kp;
      for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
#pragma unroll
        for (int r = 0; r < kVec * 4; ++r) {
          const bool on = is_live(r) && (key[r] & mask) == prefix;
          const uint32_t digit = (key[r] >> shift) & 255u;
          if (SKEWED) hist_add_grouped(sh.hist[pass], digit, on);
          else if (on) atomicAdd(&sh.hist[pass][digit], 1u);
        }
        __syncthreads();
        const int b0 = 4 * (kWave - 1 - lane);
        const uint4 h = *reinterpret_cast<const uint4*>(&sh.hist[pass][b0]);
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
      tau = prefix;
      need_eq = k;
      __syncthreads();
    }
  }

  // ---- emit ascending: every key > tau, plus the first need_eq keys == tau -----------------------
  uint32_t cnt = 0;  // low 16 bits: keys > tau, high 16 bits: keys == tau
#pragma unroll
  for (int r = 0; r < kVec * 4; ++r) {
    if (is_live(r)) {
      cnt += (key[r] > tau) ? 1u : 0u;
      cnt += (key[r] == tau) ? 0x10000u : 0u;
    }
  }
  const uint32_t before = block_excl_scan<NT>(cnt, sh.wsum);
  uint32_t gt = before & 0xffffu, eq = before >> 16;
#pragma unroll
  for (int r = 0; r < kVec * 4; ++r) {
    if (is_live(r)) {
      const int pg = (v_begin + r / 4) * 4 + (r & 3);
      bool take = key[r] > tau;
      if (key[r] == tau) {
        take = eq < need_eq;
        ++eq;
      }
      if (take) {
        const uint32_t eq_taken = (key[r] == tau) ? eq - 1 : min(eq, need_eq);
        const uint32_t pos = gt + eq_taken;
        if ((int)pos < kp) {
          if (a.out_pages) a.out_pages[(int64_t)unit * a.row_len + pos] = pg;
          if (a.out_pages2 && (int)pos < a.row_len2) a.out_pages2[(int64_t)unit * a.row_len2 + pos] = pg;
        }
      }
      if (key[r] > tau) ++gt;
    }
  }
}

// The pick with the per-thread run sized to the cache (instruction count follows the unrolled run
// length, so a short cache must not pay for the longest one).
template <int NT, bool COHERENT = false, bool SKEWED = false>
__device__ __forceinline__ void pick_from_scores(const CacheView& c, const SelectArgs& a, int unit, int n,
                                                 PickShared<NT>& sh) {
  constexpr int kMaxVec = ROCKETKV_MAX_PAGES / 4 / NT;
  static_assert(kMaxVec >= 1, "thread count does not fit the pick");
  const int per = (c.pages_cap / 4 + NT - 1) / NT;  // same for every thread
  if (per <= 1) pick_from_scores_n<NT, COHERENT, 1, SKEWED>(c, a, unit, n, sh);
  else if (per <= 2 || kMaxVec < 4) pick_from_scores_n<NT, COHERENT, (kMaxVec < 2 ? kMaxVec : 2), SKEWED>(c, a, unit, n, sh);
  else if (per <= 4 || kMaxVec < 8) pick_from_scores_n<NT, COHERENT, (kMaxVec < 4 ? kMaxVec : 4), SKEWED>(c, a, unit, n, sh);
  else pick_from_scores_n<NT, COHERENT, kMaxVec, SKEWED>(c, a, unit, n, sh);
}

// Page scores of the eight-page runs [o_begin, o_begin + n_runs) of one unit, n_runs <= NT, written as
// raw fp32 sums to `scores_row[page]` for page < P.  For summaries too large for one workgroup to
// stream at a useful rate: several workgroups take a slice each (every one repeats the cheap channel
// pick), and the top-k runs afterwards on the scores.  Needs sh.s_chan / sh.s_wgt; ends with a barrier.
template <int NT, bool COHERENT = false>
__device__ __forceinline__ void score_chunk(const CacheView& c, const SelectArgs& a, int unit, int P,
                                            SelectShared<NT>& sh, int o_begin, int n_runs,
                                            float* scores_row, const TailPatch& tp) {
  const int tid = threadIdx.x;
  const int64_t rows = (int64_t)unit * kHeadDim;
  int npow = 1;
  while (npow < n_runs) npow <<= 1;
  const int R = NT / npow;  // row groups summed separately, then in order
  const int r = tid / npow, o = tid % npow;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  // the page that is receiving a token, if it lies in this slice: scored on its own (see tail_page_load)
  float* tail2 = sh.s_abs;  // free since the channel pick ended
  const int tail_local = tp.page >= 0 ? tp.page - o_begin * 8 : -1;
  const bool owns_tail = tail_local >= 0 && tail_local < n_runs * 8;  // same for the whole workgroup
  TailPatch mine = tp;
  if (!owns_tail) mine.page = -1;
  const uint32_t tail_old = tail_page_load<NT>(a, sh.s_chan, sh.s_wgt, rows, c.pages_cap, mine);
  if (o < n_runs)
    for (int jb = 0; jb < a.k1; jb += 8 * R)  // each slice of the rows has this one reader: streamed
      score_rows8<true>(a, sh.s_chan, sh.s_wgt, rows, c.pages_cap, o_begin + o, jb + r, jb, R, acc);
  tail_page_finish<NT>(a, sh.s_chan, sh.s_wgt, mine, tail_old, tail2);
#pragma unroll
  for (int i = 0; i < 8; ++i) sh.partial[(r * npow + o) * 8 + i] = acc[i];
  __syncthreads();
  for (int p = tid; p < n_runs * 8; p += NT) {
    float s = 0.f;
    for (int rr = 0; rr < R; ++rr) s += sh.partial[rr * npow * 8 + p];
    if (owns_tail && p == tail_local) s = tail2[0] + tail2[1];
    const int page = o_begin * 8 + p;
    if (page < P) {
      if (COHERENT)  // read back by another workgroup of this launch: write through, device scope
        __hip_atomic_store(&scores_row[page], s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else
        scores_row[page] = s;
    }
  }
  if (COHERENT) drain_stores();  // the scores are acknowledged before the barrier that the caller's report follows
  __syncthreads();
}

// Both halves back to back.
template <int NT>
__device__ __forceinline__ int select_block(const CacheView& c, const SelectArgs& a, int unit, int n,
                                            SelectShared<NT>& sh, uint32_t* keys, int32_t* list_lds,
                                            bool write_global, const TailPatch& tp) {
  uint32_t qv[kMaxGroup];  // one bf16 each, kept in a register of its own (no packing, hence no early use)
  load_q_column(c, a, unit, qv);
  select_channels<NT>(c, a, unit, sh, write_global, qv);
  return select_pages<NT>(c, a, unit, n, sh, keys, list_lds, write_global, tp);
}

}  // namespace rkv
