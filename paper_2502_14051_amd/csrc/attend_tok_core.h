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
#pragma once

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

// A token that is being appended in the same launch that attends to it: (logical) token `j_new` of
// the unit, whose key / value rows every reader takes from these LDS copies rather than from memory,
// so it does not matter whether the workgroup that stores them has got there yet.  j_new < 0: none.
struct TokenPatch {
  int j_new;
  const bf16_t* knew;  // LDS, [128]
  const bf16_t* vnew;  // LDS, [128]
};

// One step over two 16-token tiles.  `row_ok[x]`: this lane's row (token hn of tile x) is real;
// `tok_ok`: bit 4x+r set when token 4kg+r of tile x is real; `row_new[x]`: this lane's row is the
// token being appended (looked at by the MASK variant only).
template <bool MASK, bool PATCH>
__device__ __forceinline__ void token_round(u32x4 (&kf)[2][4], u32x4 (&vr)[2][4], const u32x4 (&qf)[4],
                                            const u32x4 (&sel)[2], f32x4 (&O)[8], float& m, float& l,
                                            bool have_acc, bool row_ok0, bool row_ok1, uint32_t tok_ok,
                                            float sc, bool row_new0, bool row_new1, const TokenPatch& tp,
                                            int kg) {
  if (MASK) {
    if (PATCH && (row_new0 || row_new1)) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32x4 kn = *reinterpret_cast<const u32x4*>(tp.knew + j * 32 + kg * 8);
        const u32x4 vn = *reinterpret_cast<const u32x4*>(tp.vnew + j * 32 + kg * 8);
        if (row_new0) { kf[0][j] = kn; vr[0][j] = vn; }
        if (row_new1) { kf[1][j] = kn; vr[1][j] = vn; }
      }
    }
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
  if (MASK) {
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (!((tok_ok >> (4 * x + r)) & 1u)) acc[0][x][r] = -INFINITY;
  }
  // online softmax of the 32 tokens (the one-pair case of softmax_pv)
  float mx = fmaxf(fmaxf(fmaxf(acc[0][0][0], acc[0][0][1]), fmaxf(acc[0][0][2], acc[0][0][3])),
                   fmaxf(fmaxf(acc[0][1][0], acc[0][1][1]), fmaxf(acc[0][1][2], acc[0][1][3])));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx * sc);  // running max in the scaled log2 domain
  if (have_acc) {
    const float alpha = fast_exp2(m - m_new);
    l *= alpha;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int cb = 0; cb < 8; ++cb) O[cb] *= alpha;
    }
  }
  m = m_new;
  float p[2][4], psum = 0.f;
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      p[x][r] = fast_exp2(fmaf(acc[0][x][r], sc, -m_new));
      psum += p[x][r];
    }
  l += psum;
  const u32x4 pf = {pack_bf16x2(p[0][0], p[0][1]), pack_bf16x2(p[0][2], p[0][3]),
                    pack_bf16x2(p[1][0], p[1][1]), pack_bf16x2(p[1][2], p[1][3])};
  // Second product, 16 channels at a time.  Slab j of a tile holds channels 32j..32j+31 of its 16
  // rows; selector h keeps 16 of them and hands them back with tokens along the registers, which
  // packed to bf16 is the operand the product wants.  Only one block's transposed values are alive
  // at a time.
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      const f32x4 d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vr[0][j]), as_bf16x8(sel[h]), zero, 0, 0, 0);
      const f32x4 d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vr[1][j]), as_bf16x8(sel[h]), zero, 0, 0, 0);
      const u32x4 vv = {pack_bf16x2(d0[0], d0[1]), pack_bf16x2(d0[2], d0[3]), pack_bf16x2(d1[0], d1[1]),
                        pack_bf16x2(d1[2], d1[3])};
      O[2 * j + h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vv), as_bf16x8(pf), O[2 * j + h], 0, 0, 0);
    }
}

// The attention of one workgroup over its share (`split`) of the token slots of `unit`, then the
// merges.  `n`: the unit's (logical) length, already counting a token being appended (which `tp`
// describes; compiled in with PATCH); `list`: the unit's page ids (global memory or LDS; null = identity); `smem`:
// WAVES*G*130 floats of LDS; `after_stream` runs once per thread after the last K/V row has been
// consumed, before the merges.
template <int WAVES, bool INDEXED, bool PATCH = false, typename Hook = NoHook>
__device__ __forceinline__ void attend_tokens_block(const CacheView& c, const AttendArgs& a, const TokenRun& t,
                                                    int unit, int split, int n, const int32_t* list,
                                                    float* smem, int* s_last, const TokenPatch& tp,
                                                    const Hook& after_stream = Hook()) {
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int hn = lane % 16, kg = lane / 16;
  const int b = unit / c.n_kv_heads, g = unit % c.n_kv_heads;
  const int G = c.group;
  const int ps = t.ps;
  const int cap_pages = INDEXED ? t.logical_pages_cap : c.pages_cap;
  if (n > cap_pages * ps) n = cap_pages * ps;

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
    // lane -> token slot base+lane: its list entry, (logical) position, and the offset of its row
    const int f = base + lane;
    bool ok = f < we;
    const int e = f / ps, slot = f - e * ps;
    int page = -1;
    if (ok) page = list ? list[e] : e;
    ok = ok && page >= 0 && page < cap_pages;
    const int j = page * ps + slot;
    // the token being appended comes from LDS and needs no address (its rows, and under an index its
    // index entry, may not have been written yet)
    const bool is_new = PATCH && ok && j == tp.j_new;
    bool valid;  // takes part in the softmax
    int64_t off = 0;
    if (INDEXED) {
      // logical token -> position in the cache -> page and slot of the cache's own paging
      ok = ok && j < n;
      const int pos = (ok && !is_new) ? t.index[(int64_t)unit * t.index_stride + j] : 0;
      const int sp = pos / c.page_size, ss = pos - sp * c.page_size;
      bool addr = ok && !is_new && pos >= 0 && sp < c.pages_cap;
      const int64_t pp = addr ? phys_page(c, b, sp) : -1;
      addr = addr && pp >= 0;
      if (addr) off = pp * c.stride_page + ss * kHeadDim;
      valid = addr || is_new;
    } else {
      // the row address needs only a page inside the table; the sequence length (possibly still on
      // its way from memory) enters the mask alone
      const int64_t pp = (ok && !is_new) ? phys_page(c, b, page) : -1;
      if (pp >= 0) off = pp * c.stride_page + slot * kHeadDim;
      valid = (pp >= 0 && j < n) || is_new;
    }
    const unsigned long long live = __ballot(valid);
    const unsigned long long fresh = PATCH ? __ballot(is_new) : 0ull;
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
        for (int jj = 0; jj < 4; ++jj) kf[x][jj] = ld_plain<u32x4>(kt + jj * 32);
      }
#pragma unroll
      for (int x = 0; x < 2; ++x)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) vr[x][jj] = ld_stream<u32x4>(vt[x] + jj * 32);
      const uint32_t bits = (uint32_t)(live >> (32 * i));
      const uint32_t nbits = (uint32_t)(fresh >> (32 * i));
      if (bits == 0xffffffffu && nbits == 0u) {
        token_round<false, PATCH>(kf, vr, qf, sel, O, m, l, have_acc, true, true, 0xffu, sc, false, false, tp, kg);
      } else {
        const uint32_t tok_ok = ((bits >> (4 * kg)) & 0xfu) | (((bits >> (16 + 4 * kg)) & 0xfu) << 4);
        token_round<true, PATCH>(kf, vr, qf, sel, O, m, l, have_acc, (bits >> hn) & 1u, (bits >> (16 + hn)) & 1u,
                          tok_ok, sc, (nbits >> hn) & 1u, (nbits >> (16 + hn)) & 1u, tp, kg);
      }
      have_acc = true;
    }
  }
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  after_stream();
  attend_merge<WAVES, 8>(c, a, unit, split, 0, O, m, l, smem, s_last, b, g);
}

}  // namespace rkv
