// HSA Step 3 (Algorithm 1 of arXiv 2502.14051, y = attn(q, K[i2], V[i2])) and the Full-KV baseline for
// caches whose V tiles are token-major, at any page size: the operating points Section 3.6 derives
// (pages of 2-4 tokens), the Exact-TopK setting of Section 4.1 (pages of one token) and everything in
// between.
//
// The selected pages are flattened into a run of token slots; a wavefront takes 32 consecutive slots
// per step as two 16-row tiles.  Every lane addresses its own token row (256 contiguous bytes in K and
// in V), so a page of any size costs exactly its own bytes.  The first product is the one of the
// 16-token-page kernel, S[token][head] = K[token][:] . Q[head][:].  The second one contracts over
// tokens, and a matrix-core operand must hold its contraction index contiguously per lane, which a
// token-major V row does not.  Instead of a detour through LDS the tile is transposed on the matrix
// cores themselves: V[16 tokens][32 channels] times a 0/1 selector matrix gives
// D[token][channel] with tokens along the accumulator registers, exact in fp32, and packing D back to
// bf16 (exact again) yields the operand layout the second product wants.  That costs 16 extra
// matrix instructions per 32 tokens on a pipe that is otherwise mostly idle in this HBM-bound kernel.
#include "attend_core.h"

namespace rkv {

struct TokenRun {
  int ps;      // tokens per list entry
  int tokens;  // list entries x ps: token slots per (sequence, KV head)
  // RocketKV-MT (Section 3.5): the list addresses pages of a logical sequence, whose token j sits at
  // position index[unit][j] of the cache; null = the cache's own order
  const int32_t* index;
  int index_stride;          // entries per (sequence, KV head) row of `index`
  const int32_t* n_logical;  // [batch] logical lengths
  int logical_pages_cap;
};

// One step over two 16-token tiles.  `row_ok[x]`: this lane's row (token hn of tile x) is real;
// `tok_ok`: bit 4x+r set when token 4kg+r of tile x is real.
template <bool MASK>
__device__ __forceinline__ void token_round(u32x4 (&kf)[2][4], u32x4 (&vr)[2][4], const u32x4 (&qf)[4],
                                            const u32x4 (&sel)[2], f32x4 (&O)[8], float& m, float& l,
                                            bool have_acc, bool row_ok0, bool row_ok1, uint32_t tok_ok,
                                            float sc) {
  if (MASK) {
    // A slot without a token reads some other row; its probability is zero, but 0 x NaN is not, so
    // the value row is cleared before it enters the products.
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!row_ok0) vr[0][j] = (u32x4){0u, 0u, 0u, 0u};
      if (!row_ok1) vr[1][j] = (u32x4){0u, 0u, 0u, 0u};
    }
  }
  f32x4 acc[1][2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    acc[0][x] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc[0][x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[x][j]), as_bf16x8(qf[j]), acc[0][x],
                                                          0, 0, 0);
  }
  // transpose V: slab j holds channels 32j..32j+31 of the 16 rows; selector h keeps 16 of them
  u32x2 vf[1][2][8];
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const f32x4 d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vr[x][j]), as_bf16x8(sel[h]),
                                                                (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        vf[0][x][2 * j + h] = (u32x2){pack_bf16x2(d[0], d[1]), pack_bf16x2(d[2], d[3])};
      }
  if (MASK) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (!((tok_ok >> (4 * x + r)) & 1u)) acc[0][x][r] = -INFINITY;
  }
  softmax_pv<1>(acc, vf, O, m, l, have_acc, sc);
}

template <int WAVES, bool INDEXED>
__global__ __launch_bounds__(WAVES* kWave) __attribute__((amdgpu_waves_per_eu(2)))
void attend_tokens_kernel(CacheView c, AttendArgs a, TokenRun t) {
  extern __shared__ float smem[];  // sO[WAVES][G][128], sM[WAVES][G], sL[WAVES][G]
  __shared__ int s_last;
  const int unit = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int G = c.group;
  const int ps = t.ps;
  const int cap_pages = INDEXED ? t.logical_pages_cap : c.pages_cap;
  int n = INDEXED ? t.n_logical[b] : c.seq_lens[b];
  if (n > cap_pages * ps) n = cap_pages * ps;
  const int32_t* list = a.pages ? a.pages + (int64_t)unit * a.row_len : nullptr;

  // this wave's share of the token slots (chunk and per_wave are multiples of 32).  The plan is laid
  // out on whole 16-slot entries; the last wavefront of the last workgroup also takes the few slots
  // left over when pages do not fill the last entry, rather than a workgroup being launched for them.
  const int e_begin = split * a.chunk;
  const int e_end = split == a.n_split - 1 ? t.tokens : min(e_begin + a.chunk, t.tokens);
  const int wb = min(e_begin + wave * a.per_wave, e_end);
  const int we = wave == WAVES - 1 ? e_end : min(wb + a.per_wave, e_end);

  u32x4 qf[4];
  {
    const bf16_t* qp = a.q + ((int64_t)b * c.n_q_heads + (int64_t)g * G + (hn < G ? hn : 0)) * kHeadDim + kg * 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      qf[j] = *reinterpret_cast<const u32x4*>(qp + j * 32);
      if (hn >= G) qf[j] = (u32x4){0u, 0u, 0u, 0u};
    }
  }
  // selector operands: lane (column hn, rows 8kg..8kg+7) of the 32x16 matrix with ones at
  // row == column + 16h
  u32x4 sel[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = hn + 16 * h, i = row % 8;
    const uint32_t one = row / 8 != kg ? 0u : (i & 1) ? 0x3f800000u : 0x00003f80u;  // bf16 1.0, placed
    sel[h] = (u32x4){i / 2 == 0 ? one : 0u, i / 2 == 1 ? one : 0u, i / 2 == 2 ? one : 0u, i / 2 == 3 ? one : 0u};
  }

  f32x4 O[8];
#pragma unroll
  for (int cb = 0; cb < 8; ++cb) O[cb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = kNegBig, l = 0.f;
  bool have_acc = false;
  const float sc = kLog2e * 0.08838834764831845f;  // log2(e) / sqrt(128)
  const int64_t lane_off = (int64_t)g * c.stride_head + kg * 8;

  for (int base = wb; base < we; base += kWave) {
    // lane -> token slot base+lane: its list entry, position, and the offset of its row
    const int f = base + lane;
    bool ok = f < we;
    const int e = f / ps, slot = f - e * ps;
    int page = -1;
    if (ok) page = list ? list[e] : e;
    ok = ok && page >= 0 && page < cap_pages;
    int64_t off = 0;
    unsigned long long live;
    if (INDEXED) {
      // logical token -> position in the cache -> page and slot of the cache's own paging
      const int j = page * ps + slot;
      ok = ok && j < n;
      const int pos = ok ? t.index[(int64_t)unit * t.index_stride + j] : 0;
      const int sp = pos / c.page_size, ss = pos - sp * c.page_size;
      ok = ok && pos >= 0 && sp < c.pages_cap;
      const int64_t pp = ok ? phys_page(c, b, sp) : -1;
      ok = ok && pp >= 0;
      if (ok) off = pp * c.stride_page + ss * kHeadDim;
      live = __ballot(ok);
    } else {
      // the row address needs only a page inside the table; the sequence length (possibly still on
      // its way from memory) enters the mask alone
      const int64_t pp = ok ? phys_page(c, b, page) : -1;
      ok = ok && pp >= 0;
      if (ok) off = pp * c.stride_page + slot * kHeadDim;
      live = __ballot(ok && page * ps + slot < n);
    }
    const int cnt = min(kWave, we - base);
    for (int i = 0; i * 32 < cnt; ++i) {
      u32x4 kf[2][4], vr[2][4];
      const bf16_t* vt[2];
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const int src = 32 * i + 16 * x + hn;
        const int64_t ofx = ((int64_t)__shfl((int)(off >> 32), src) << 32) |
                            (uint32_t)__shfl((int)(off & 0xffffffff), src);
        const bf16_t* kt = c.k_pool + lane_off + ofx;
        vt[x] = c.v_pool + lane_off + ofx;
#pragma unroll
        for (int j = 0; j < 4; ++j) kf[x][j] = *reinterpret_cast<const u32x4*>(kt + j * 32);
      }
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int j = 0; j < 4; ++j) vr[x][j] = *reinterpret_cast<const u32x4*>(vt[x] + j * 32);
      const uint32_t bits = (uint32_t)(live >> (32 * i));
      if (bits == 0xffffffffu) {
        token_round<false>(kf, vr, qf, sel, O, m, l, have_acc, true, true, 0xffu, sc);
      } else {
        const uint32_t tok_ok = ((bits >> (4 * kg)) & 0xfu) | (((bits >> (16 + 4 * kg)) & 0xfu) << 4);
        token_round<true>(kf, vr, qf, sel, O, m, l, have_acc, (bits >> hn) & 1u, (bits >> (16 + hn)) & 1u,
                          tok_ok, sc);
      }
      have_acc = true;
    }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  attend_merge<WAVES>(c, a, unit, split, O, m, l, smem, &s_last, b, g);
}

hipError_t launch_attend_tokens(const CacheView& c, const bf16_t* q, const int32_t* pages, int row_len,
                                bf16_t* out, float* out_lse, void* ws, const AttendPlan& plan,
                                const LogicalView* lv, hipStream_t st) {
  const int units = c.batch * c.n_kv_heads;
  AttendArgs a;
  a.q = q;
  a.pages = pages;
  a.row_len = row_len;
  a.out = out;
  a.out_lse = out_lse;
  a.partial = reinterpret_cast<float*>(static_cast<char*>(ws) + plan.partial_off);
  a.counters = attend_counters(ws, plan);
  a.n_split = plan.n_split;
  a.chunk = plan.chunk * kAttnPage;        // the plan counts 16-token entries
  a.per_wave = plan.per_wave * kAttnPage;  // even number of entries: a multiple of 32 slots
  TokenRun t;
  t.ps = lv ? lv->page_size : c.page_size;
  t.tokens = row_len * t.ps;
  t.index = lv ? lv->token_index : nullptr;
  t.index_stride = lv ? lv->pages_cap * lv->page_size : 0;
  t.n_logical = lv ? lv->n_indexed : nullptr;
  t.logical_pages_cap = lv ? lv->pages_cap : 0;
  const size_t smem = (size_t)plan.waves * c.group * (kHeadDim + 2) * sizeof(float);
  const dim3 grid(plan.n_split, units);
  if (plan.waves == 8) {
    if (lv)
      hipLaunchKernelGGL((attend_tokens_kernel<8, true>), grid, dim3(8 * kWave), smem, st, c, a, t);
    else
      hipLaunchKernelGGL((attend_tokens_kernel<8, false>), grid, dim3(8 * kWave), smem, st, c, a, t);
  } else {
    if (lv)
      hipLaunchKernelGGL((attend_tokens_kernel<4, true>), grid, dim3(4 * kWave), smem, st, c, a, t);
    else
      hipLaunchKernelGGL((attend_tokens_kernel<4, false>), grid, dim3(4 * kWave), smem, st, c, a, t);
  }
  return hipGetLastError();
}

}  // namespace rkv
