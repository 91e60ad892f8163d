// Stand-alone HSA Step 3 kernel and the Full-KV baseline (Algorithm 1 of arXiv 2502.14051,
// y = attn(q, K[i2], V[i2]); Table 1, first row): the workgroup-level attention routine driven by a
// page list in global memory (or the identity list), plus the launch geometry shared with the
// fused decode kernel.
#include "attend_core.h"

namespace rkv {

// CB: channel blocks of the output this workgroup computes (8: all 128 channels; 4: the unit's channels
// are divided between two workgroups, which the grid then lists as (unit, split x share) with the
// unit as the fast dimension, so that the two land on one XCD and share its L2 for the K tiles).
template <int WAVES, int NP, bool STREAM_K, int CB>
__global__ __launch_bounds__(WAVES* kWave) __attribute__((amdgpu_waves_per_eu(2)))
void attend_mfma_kernel(CacheView c, AttendArgs a) {
  extern __shared__ float smem[];  // sO[WAVES][G][CB*16], sM[WAVES][G], sL[WAVES][G]
  __shared__ int s_last;
  const int unit = CB == 8 ? blockIdx.y : blockIdx.x;
  const int y = CB == 8 ? blockIdx.x : blockIdx.y;
  const int split = y / a.n_csplit, cs = y % a.n_csplit;
  const int n = c.seq_lens[unit / c.n_kv_heads];
  const int32_t* list = a.pages ? a.pages + (int64_t)unit * a.row_len : nullptr;
  const TailPatch none = {-1, 0, nullptr, nullptr};
  attend_block<WAVES, NP, STREAM_K, CB>(c, a, unit, split, cs, n, list, smem, &s_last, none);
}

__global__ void zero_u32_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ---- launch geometry ---------------------------------------------------------------------------------
constexpr int kComputeUnits = 256;  // MI355X
constexpr int kPairsPerWave = 2;    // page pairs a wavefront aims to own
constexpr int kMaxWorkgroups = 2048;  // cap on workgroups per launch (keeps the dense case from over-splitting)

// `gather`: the launch follows a page list (Step 3 proper), as opposed to the identity list of the
// Full-KV baseline.
AttendPlan plan_attend(const CacheView& c, int row_len, bool gather) {
  AttendPlan p;
  const int units = c.batch * c.n_kv_heads;
  // Up to one (sequence, KV head) unit per compute unit: workgroups of eight wavefronts, one per
  // compute unit, dividing a unit's work between them if that fills the chip.  More units than
  // compute units: workgroups of four wavefronts, two of which share a compute unit and drift apart,
  // so that one's selection phase runs under the other's K/V stream (batch 64 of the benchmark shape:
  // 61 against 71 us per layer-step; at exactly 256 units the eight-wavefront form is still ahead).
  const bool many_units = units > kComputeUnits;
  int waves = many_units ? 4 : 8;
  // the LDS merge buffer must fit 64 KiB: waves * G * 130 floats
  while (waves > 4 && (size_t)waves * c.group * (kHeadDim + 2) * sizeof(float) > 60 * 1024) waves /= 2;
  p.waves = waves;
  // entries the smallest sensible workgroup takes: normally kPairsPerWave page pairs per wavefront,
  // one pair when even that leaves compute units idle (few units: shorter streams beat fewer merges)
  int pairs = many_units ? 2 * kPairsPerWave : kPairsPerWave;  // half the wavefronts, the same share per workgroup
  if ((int64_t)units * ((row_len + 2 * waves - 1) / (2 * waves)) <= kComputeUnits) pairs = 1;
  const int per_wg = 2 * pairs * waves;
  int n_wg = (row_len + per_wg - 1) / per_wg;  // workgroups per unit
  const int max_wg = kMaxWorkgroups / units > 1 ? kMaxWorkgroups / units : 1;
  // More work than one round of workgroups over the chip: twice the smallest share per workgroup
  // (a second round of short workgroups costs more than it hides), but never fewer workgroups than
  // compute units.
  const int fill = (kComputeUnits + units - 1) / units;
  if (n_wg > fill) n_wg = n_wg / 2 > fill ? n_wg / 2 : fill;
  if (n_wg > max_wg) n_wg = max_wg;
  if (n_wg < 1) n_wg = 1;
  // A gather over 16-token pages that leaves compute units idle divides every unit's output channels
  // two ways on top of its list: twice the workgroups, each with all of the K tiles of its pages (the
  // second reader finds them in L2) and half of the V bytes.  With the chip already full the same
  // division in place of a list split (two workgroups per unit that never meet) was measured as well:
  // it trades the hand-over of partials (2.6 us) for a longer stream (both workgroups run every
  // softmax step of the unit), 22.1 against 22.3 us without and 24.6 against 23.8 us with the token
  // append at the benchmark shape, and is not used.
  p.n_csplit = 1;
  if (gather && !c.v_token_major && waves == 8 && (int64_t)units * n_wg * 2 <= kComputeUnits) p.n_csplit = 2;
  int chunk = (row_len + n_wg - 1) / n_wg;
  int per_wave = (chunk + waves - 1) / waves;
  per_wave = (per_wave + 1) / 2 * 2;  // whole pairs
  chunk = per_wave * waves;
  p.chunk = chunk;
  p.per_wave = per_wave;
  p.n_split = (row_len + chunk - 1) / chunk;
  if (p.n_split < 1) p.n_split = 1;
  size_t off = 0;
  p.counter_off = off;  // always first: the part rocketkv_workspace_init clears
  off += ROCKETKV_WS_HEADER_BYTES;
  p.partial_off = off;
  off += ((size_t)units * p.n_csplit * p.n_split * c.group * kPartialStride * sizeof(float) + 255) / 256 * 256;
  p.total_bytes = off;
  return p;
}

uint32_t* attend_counters(void* ws, const AttendPlan& plan) {
  return reinterpret_cast<uint32_t*>(static_cast<char*>(ws) + plan.counter_off);
}

hipError_t launch_zero(void* p, size_t bytes, hipStream_t st) {
  const int n = (int)(bytes / sizeof(uint32_t));
  if (n > 0) hipLaunchKernelGGL(zero_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, static_cast<uint32_t*>(p), n);
  return hipGetLastError();
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
  a.counters = attend_counters(ws, plan);
  a.n_split = plan.n_split;
  a.chunk = plan.chunk;
  a.per_wave = plan.per_wave;
  a.n_csplit = plan.n_csplit;
  if (plan.n_csplit == 2) {
    // K tiles are read by both workgroups of a share pair: plain loads, so that the second finds them in L2
    const size_t smem = (size_t)plan.waves * c.group * (kHeadDim / 2 + 2) * sizeof(float);
    hipLaunchKernelGGL((attend_mfma_kernel<8, 1, false, 4>), dim3(units, plan.n_split * 2), dim3(8 * kWave), smem, st, c, a);
    return hipGetLastError();
  }
  const size_t smem = (size_t)plan.waves * c.group * (kHeadDim + 2) * sizeof(float);
  const dim3 grid(plan.n_split, units);
  const bool stream_k = pages != nullptr && wants_stream_k(c, row_len);  // a large gather, not the dense read
#define RKV_LAUNCH_ATTEND(W, S) \
  hipLaunchKernelGGL((attend_mfma_kernel<W, 1, S, 8>), grid, dim3(W * kWave), smem, st, c, a)
  if (plan.waves == 8) {
    if (stream_k) RKV_LAUNCH_ATTEND(8, true); else RKV_LAUNCH_ATTEND(8, false);
  } else {
    if (stream_k) RKV_LAUNCH_ATTEND(4, true); else RKV_LAUNCH_ATTEND(4, false);
  }
#undef RKV_LAUNCH_ATTEND
  return hipGetLastError();
}

}  // namespace rkv
