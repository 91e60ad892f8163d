/*
 * rocketkv.h -- C ABI of the MI355X (gfx950) RocketKV hot path.
 *
 * RocketKV (arXiv 2502.14051) compresses the KV cache of a decoder LLM in two
 * stages: a one-time, GQA-aware SnapKV eviction of prompt tokens (Section 3.3)
 * and, at every decode step, hybrid sparse attention (HSA, Section 3.4 and
 * Algorithm 1): page-wise min/max key summaries, a top-k1 channel pick per GQA
 * group, approximate page scores, a top-k page pick and exact attention over
 * the picked pages only.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers unless marked "host".  The struct
 *    `rocketkv_cache_t` itself lives in host memory and is read during the
 *    call only.
 *  - bf16 tensors are passed as `void*` / `const void*` (2 bytes per element,
 *    upper half of an IEEE binary32).
 *  - `stream` is a `hipStream_t` passed as `void*` (NULL = the null stream).
 *    Work is enqueued on it and the call returns without synchronising.  No
 *    entry point allocates or frees device memory; scratch comes from the
 *    caller's `workspace` (size from rocketkv_workspace_bytes, 256-byte
 *    aligned).  A workspace must be passed once through
 *    rocketkv_workspace_init after it is allocated, and again whenever it is
 *    reused for a cache of a different shape; every call leaves it ready for
 *    the next.  Two calls that overlap in time must not share one.
 *  - Return value: ROCKETKV_OK (0) or a negative rocketkv_status_t.  Argument
 *    validation runs on the host before anything is launched; on error
 *    nothing has been enqueued and rocketkv_last_error() describes the
 *    reason (thread-local, valid until the next call on the same thread).
 *  - The caller owns every buffer.  The library keeps no state between calls.
 *
 * Cache layout (chosen for CDNA4 matrix-core operand order)
 * ---------------------------------------------------------
 * A cache is a pool of physical pages of `page_size` tokens.  For a physical
 * page `pp` and KV head `g` the tile starts at element
 *        pp * stride_page + g * stride_head
 * of the pool and holds `page_size * head_dim` contiguous bf16 values:
 *        K tile: [page_size][head_dim]   (token-major, channels contiguous)
 *        V tile: [head_dim][page_size]   (channel-major, tokens contiguous) when
 *                v_layout == ROCKETKV_V_CHANNEL_MAJOR, else [page_size][head_dim]
 * The channel-major V tile with page_size 16 is the layout the fused decode
 * kernel is built for (the token index is the contraction index of its second
 * matrix product).  The token-major V tile keeps every token's value row
 * contiguous, which is what page sizes other than 16 (Section 3.6 derives 2-4
 * for the usual budgets) and token-granular gathers need.
 * Sequence b's logical page p (tokens p*page_size ...) is physical page
 * `block_table[b*pages_cap + p]`, or `b*pages_cap + p` when block_table is
 * NULL.  `seq_lens[b]` is the number of valid tokens of sequence b (all KV
 * heads of a sequence hold the same number of tokens).  Entries of the block
 * table outside [0, n_phys_pages) are treated as absent pages.
 *
 * Page summaries (Section 3.4 Step 1) are two bf16 tensors
 *        kmax, kmin: [batch][n_kv_heads][head_dim][pages_cap]
 * i.e. channel-major with the page index contiguous, so that each channel
 * picked in Step 2 is one contiguous row.  Columns >= ceil(seq_len/page_size)
 * are never read.
 *
 * Limits of this build: head_dim == 128; n_q_heads a multiple of n_kv_heads
 * with group size <= 16; page_size 1..64, and 16 where V is channel-major and
 * attention or SnapKV is involved; pages_cap a multiple of 8 and at most
 * ROCKETKV_MAX_PAGES for selection.
 */
#ifndef ROCKETKV_H
#define ROCKETKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROCKETKV_MAX_PAGES 32768

typedef enum {
  ROCKETKV_OK = 0,
  ROCKETKV_INVALID_ARG = -1,         /* NULL pointer, bad shape, bad budget ...      */
  ROCKETKV_UNSUPPORTED = -2,         /* valid request outside this build's limits    */
  ROCKETKV_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes < rocketkv_workspace_bytes() */
  ROCKETKV_HIP_ERROR = -4            /* a HIP runtime call failed                    */
} rocketkv_status_t;

typedef enum {
  ROCKETKV_OP_HSA_DECODE = 0,   /* a = token_budget                       */
  ROCKETKV_OP_DENSE_DECODE = 1, /* no extra arguments                     */
  ROCKETKV_OP_SNAPKV = 2,       /* a = window, b = keep_budget            */
  ROCKETKV_OP_ATTEND = 3        /* a = pages_row_len (0 = every page)     */
} rocketkv_op_t;

typedef enum {
  ROCKETKV_V_CHANNEL_MAJOR = 0, /* V tile [head_dim][page_size] */
  ROCKETKV_V_TOKEN_MAJOR = 1    /* V tile [page_size][head_dim] */
} rocketkv_v_layout_t;

typedef struct rocketkv_cache {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t page_size;
  int32_t pages_cap;          /* logical pages per sequence: row length of block_table / summaries */
  int64_t n_phys_pages;       /* pages in the pools */
  int64_t stride_page;        /* elements between physical pages (same for K and V pools) */
  int64_t stride_head;        /* elements between KV heads inside a page, >= page_size*head_dim */
  int32_t* seq_lens;          /* device [batch]; written by snapkv_compress (dst) and append_kv */
  const int32_t* block_table; /* device [batch][pages_cap] or NULL (identity) */
  void* k_pool;               /* device bf16 */
  void* v_pool;               /* device bf16 */
  int32_t v_layout;           /* rocketkv_v_layout_t */
} rocketkv_cache_t;

#define ROCKETKV_WS_HEADER_BYTES 65536 /* leading part of a workspace that workspace_init clears */

/* Scratch bytes needed by an operation on `cache` (host struct; device
 * pointers inside it are not dereferenced).  Returns 0 for an invalid
 * request (see rocketkv_last_error). */
size_t rocketkv_workspace_bytes(int32_t op, const rocketkv_cache_t* cache, int32_t a, int32_t b);

/*
 * Prepares a freshly allocated workspace: clears its first
 * min(workspace_bytes, ROCKETKV_WS_HEADER_BYTES) bytes (the arrival counters of the
 * split attention merge) on `stream`.  The attention entry points restore that
 * state themselves at the end of every call.
 */
int32_t rocketkv_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * HSA Step 1 (Section 3.4): element-wise max and min of the keys of each page,
 * over the valid tokens of the page only, for logical pages
 * [first_page, first_page + n_pages) of every (sequence, KV head); n_pages < 0
 * means "through the last page".  Pages at or beyond ceil(seq_len/page_size)
 * are skipped.  Exact: results are bf16 values present in K.
 * kmax, kmin: device bf16 [batch][n_kv_heads][head_dim][pages_cap], written.
 */
int32_t rocketkv_build_page_summaries(const rocketkv_cache_t* cache, void* kmax, void* kmin,
                                      int32_t first_page, int32_t n_pages, void* stream);

/*
 * HSA Step 2 (Algorithm 1, i1 / g / P / s1 / i2): per (sequence, KV head)
 *   a[c] = sum over the group's heads of |q[h][c]|,  s[c] = sum of q[h][c]  (fp32, head order)
 *   i1   = the channel_budget channels with the largest a (ties: lower channel)
 *   score[p] = sum over c in i1 of s[c] * (s[c] >= 0 ? kmax[c][p] : kmin[c][p])   (fp32)
 *   i2   = the kp pages with the largest score (ties: lower page), where
 *          kp = P if token_budget >= seq_len, else max(1, min(P, token_budget / page_size)),
 *          P = ceil(seq_len / page_size); the last min(n_recent_pages, kp) pages are always in.
 * q: bf16 [batch][n_q_heads][head_dim].
 * out_pages: int32 [batch][n_kv_heads][pages_row_len], ascending page ids, -1 padded;
 *            pages_row_len must be >= min(pages_cap, ceil(token_budget / page_size)).
 * out_channels: optional int32 [batch][n_kv_heads][channel_budget], ascending.
 * out_scores: optional fp32 [batch][n_kv_heads][pages_cap] (first P entries written); required
 *             when pages_cap exceeds 8192 (the selection then runs as a score launch and a top-k
 *             launch with the scores in between; the decode entry points keep them in the workspace).
 */
int32_t rocketkv_hsa_select(const rocketkv_cache_t* cache, const void* q, const void* kmax,
                            const void* kmin, int32_t channel_budget, int32_t token_budget,
                            int32_t n_recent_pages, int32_t* out_pages, int32_t pages_row_len,
                            int32_t* out_channels, float* out_scores, void* stream);

/*
 * HSA Step 3 (Algorithm 1, y = attn(q, K[i2], V[i2])): exact softmax attention
 * (scale 1/sqrt(head_dim)) of every query head over the valid tokens of the
 * listed pages of its KV head; bf16 operands, fp32 accumulation, bf16 result
 * rounded to nearest even.
 * pages: int32 [batch][n_kv_heads][pages_row_len] logical page ids; entries
 *        < 0 or >= ceil(seq_len/page_size) are ignored.  NULL = every page of
 *        the sequence (full-KV attention, the Full-KV row of Table 1).
 * out: bf16 [batch][n_q_heads][head_dim]; a sequence with no attended token
 *      gets zeros.  out_lse: optional fp32 [batch][n_q_heads], natural-log
 *      sum-exp of the scaled logits (-inf when nothing was attended).
 * workspace: rocketkv_workspace_bytes(ROCKETKV_OP_ATTEND, cache, pages_row_len, 0).
 */
int32_t rocketkv_attend(const rocketkv_cache_t* cache, const void* q, const int32_t* pages,
                        int32_t pages_row_len, void* out, float* out_lse, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * One HSA decode step over a cache whose summaries are current: Step 2 then
 * Step 3 (Algorithm 1 end to end).  Arguments as in rocketkv_hsa_select and
 * rocketkv_attend; out_pages (row length min(pages_cap, ceil(token_budget /
 * page_size))), out_channels and out_lse are optional.
 * workspace: rocketkv_workspace_bytes(ROCKETKV_OP_HSA_DECODE, cache, token_budget, 0).
 */
int32_t rocketkv_hsa_decode(const rocketkv_cache_t* cache, const void* q, const void* kmax,
                            const void* kmin, int32_t channel_budget, int32_t token_budget,
                            int32_t n_recent_pages, void* out, float* out_lse,
                            int32_t* out_pages, int32_t* out_channels, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * rocketkv_hsa_decode for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same
 * kernels and the same results as rocketkv_hsa_decode, minus the workspace: the scratch memory (arrival
 * counters, split partials, the page list and page scores of the multi-launch paths) is a buffer of
 * ROCKETKV_NOALLOC_SCRATCH_BYTES that is part of the library's device code, one copy per GPU, held
 * until the process ends.  The call allocates and frees nothing.  It clears the buffer's counter
 * header with a small fill kernel on `stream` first, so it costs one short launch more than
 * rocketkv_hsa_decode.  A shape whose scratch need (rocketkv_workspace_bytes(ROCKETKV_OP_HSA_DECODE,
 * ...)) exceeds the buffer is refused with ROCKETKV_UNSUPPORTED.  Every call on a GPU uses that GPU's
 * one buffer: calls that overlap in time on one GPU (two streams, two threads) race and must be
 * serialised by the caller; calls on different GPUs are independent.  The device current at the call
 * must be the one `stream` and the buffers belong to.
 */
#define ROCKETKV_NOALLOC_SCRATCH_BYTES (4u << 20)
int32_t rocketkv_hsa_decode_noalloc(const rocketkv_cache_t* cache, const void* q, const void* kmax,
                                    const void* kmin, int32_t channel_budget, int32_t token_budget,
                                    int32_t n_recent_pages, void* out, float* out_lse,
                                    int32_t* out_pages, int32_t* out_channels, void* stream);

/*
 * One decode step including the token generated at it (Section 3.4 Step 1, last
 * sentence, then Algorithm 1): the result, the caches, the summaries and
 * seq_lens end up exactly as after rocketkv_append_kv(k_new, v_new) followed by
 * rocketkv_hsa_decode, in one launch where the shapes allow.  kmax / kmin are
 * read and written.  k_new, v_new: bf16 [batch][n_kv_heads][head_dim].
 * workspace: as for rocketkv_hsa_decode (same size, same initialisation).
 */
int32_t rocketkv_hsa_decode_append(const rocketkv_cache_t* cache, const void* q, const void* k_new,
                                   const void* v_new, void* kmax, void* kmin, int32_t channel_budget,
                                   int32_t token_budget, int32_t n_recent_pages, void* out,
                                   float* out_lse, int32_t* out_pages, int32_t* out_channels,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Full-KV decode attention (Table 1, first row; the baseline every figure of
 * Section 4.3 is normalised to): rocketkv_attend with every page.
 * workspace: rocketkv_workspace_bytes(ROCKETKV_OP_DENSE_DECODE, cache, 0, 0).
 */
int32_t rocketkv_dense_decode(const rocketkv_cache_t* cache, const void* q, void* out,
                              float* out_lse, void* workspace, size_t workspace_bytes,
                              void* stream);

/*
 * Appending one generated token per sequence (Section 3.4 Step 1, last
 * sentence: the summaries follow every new key): writes k_new / v_new
 * (bf16 [batch][n_kv_heads][head_dim]) at position seq_lens[b], folds the key
 * into the tail page's kmax / kmin, then increments seq_lens[b].  A sequence
 * already holding pages_cap * page_size tokens is left unchanged.
 */
int32_t rocketkv_append_kv(const rocketkv_cache_t* cache, const void* k_new, const void* v_new,
                           void* kmax, void* kmin, void* stream);

/*
 * Stage 1 (Section 3.3; window and kernel sizes from Appendix A.3): GQA-aware
 * SnapKV.  Per (sequence, KV head) with prompt length S = src->seq_lens[b]:
 *   if S <= keep_budget every token is kept; otherwise
 *   A[h][w][j] = causal softmax over j <= S-window+w of q_obs[h][w] . K[j] / sqrt(head_dim)
 *   vote[j] = sum over heads of the group and window rows of A[h][w][j],  j < S-window
 *   pooled  = stride-1 max-pool of vote with odd kernel pool_kernel, clipped at the ends
 *   kept    = top-(keep_budget - window) of pooled (ties: lower position) plus the window
 * and K/V of the kept tokens are copied, in ascending position, into `dst`
 * (same head counts and head_dim; dst->pages_cap*page_size >= keep_budget),
 * dst->seq_lens[b] = min(S, keep_budget).
 * q_obs: bf16 [batch][n_q_heads][window][head_dim], queries of the last
 *        `window` prompt positions.
 * src needs page_size 16; dst may have any page size when its V is token-major.
 * kept_idx: optional int32 [batch][n_kv_heads][keep_budget], -1 padded.
 * workspace: rocketkv_workspace_bytes(ROCKETKV_OP_SNAPKV, src, window, keep_budget).
 */
int32_t rocketkv_snapkv_compress(const void* q_obs, const rocketkv_cache_t* src, int32_t window,
                                 int32_t pool_kernel, int32_t keep_budget,
                                 const rocketkv_cache_t* dst, int32_t* kept_idx, void* workspace,
                                 size_t workspace_bytes, void* stream);

/*
 * RocketKV-MT (Section 3.5): the multi-turn variant.  Stage 1 evicts nothing: the cache keeps every
 * token of the conversation, and Stage 2 runs over the subset Stage 1 filtered for the current turn
 * plus the tokens generated since, reached through an index.  At the next turn the filter runs
 * again over the whole cache, so a token passed over in one turn can come back in a later one.
 *
 * rocketkv_index_t describes that subset, the "logical sequence" of a (sequence, KV head):
 *   token_index[b][g][j] = position in the cache of logical token j, ascending in j;
 *   n_indexed[b]         = number of logical tokens (the same for every KV head of a sequence);
 *   page_size, pages_cap = page size and page capacity of Stage 2 over the logical order: page p
 *                          holds logical tokens p*page_size ..; summaries are
 *                          [batch][n_kv_heads][head_dim][pages_cap].
 * token_index rows have pages_cap * page_size entries.  The struct lives in host memory; its
 * pointers are device pointers, written by rocketkv_snapkv_filter and the *_append calls.
 * The cache itself must have token-major V (a token's row is what is gathered); its own page size
 * is free.  A logical sequence is exactly what rocketkv_snapkv_compress would have copied out, so
 * every mt call computes what its counterpart computes on that compacted cache.
 */
typedef struct rocketkv_index {
  int32_t* token_index;
  int32_t* n_indexed;
  int32_t page_size;
  int32_t pages_cap;
} rocketkv_index_t;

/*
 * Stage 1 as a filter (Section 3.5): the selection of rocketkv_snapkv_compress on `src` (all of its
 * rules, arguments and limits apply) written to index->token_index / index->n_indexed instead of a
 * compacted copy; src is left untouched.  Needs index->pages_cap * index->page_size >= keep_budget.
 * workspace: rocketkv_workspace_bytes(ROCKETKV_OP_SNAPKV, src, window, keep_budget).
 */
int32_t rocketkv_snapkv_filter(const void* q_obs, const rocketkv_cache_t* src, int32_t window,
                               int32_t pool_kernel, int32_t keep_budget, const rocketkv_index_t* index,
                               void* workspace, size_t workspace_bytes, void* stream);

/* rocketkv_build_page_summaries over the logical order of `index` (Section 3.4 Step 1 on the
 * filtered subset). */
int32_t rocketkv_mt_build_page_summaries(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                                         void* kmax, void* kmin, int32_t first_page, int32_t n_pages,
                                         void* stream);

/* Scratch bytes of rocketkv_mt_hsa_decode / rocketkv_mt_hsa_decode_append (0 on an invalid request). */
size_t rocketkv_mt_workspace_bytes(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                                   int32_t token_budget);

/*
 * rocketkv_hsa_decode over the logical sequence (Algorithm 1 restricted to the filtered subset):
 * selection on the logical pages, exact attention over the cache rows the picked logical tokens
 * point at.  out_pages holds logical page ids (row length min(index->pages_cap,
 * ceil(token_budget / index->page_size))).
 */
int32_t rocketkv_mt_hsa_decode(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                               const void* q, const void* kmax, const void* kmin,
                               int32_t channel_budget, int32_t token_budget, int32_t n_recent_pages,
                               void* out, float* out_lse, int32_t* out_pages, int32_t* out_channels,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * A generated token enters both the cache (position cache->seq_lens[b], as rocketkv_append_kv does)
 * and the logical sequence (entry index->n_indexed[b] of every KV head's index row, and the logical
 * tail page's kmax / kmin); both lengths grow by one.  A sequence whose cache or index is full is
 * left unchanged.
 */
int32_t rocketkv_mt_append_kv(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                              const void* k_new, const void* v_new, void* kmax, void* kmin,
                              void* stream);

/* rocketkv_mt_append_kv followed by rocketkv_mt_hsa_decode: one decode step of RocketKV-MT. */
int32_t rocketkv_mt_hsa_decode_append(const rocketkv_cache_t* cache, const rocketkv_index_t* index,
                                      const void* q, const void* k_new, const void* v_new, void* kmax,
                                      void* kmin, int32_t channel_budget, int32_t token_budget,
                                      int32_t n_recent_pages, void* out, float* out_lse,
                                      int32_t* out_pages, int32_t* out_channels, void* workspace,
                                      size_t workspace_bytes, void* stream);

/*
 * Adaptive compression decomposition (Section 3.6): for a sequence of seq_len
 * tokens and a total token budget t (memory traffic of one attention call in
 * key/value pairs, Step 2 and Step 3 together), c = seq_len / t (at least 1),
 *   r = min(0.2 + 0.06 log2 c, 0.8),  stage1 = c^r,  stage2 = c^(1-r),
 *   page_size = ceil(c^((1-r)/2)),  head_ratio = stage2 / page_size,
 * and, with the budget split evenly between Step 2 and Step 3 (Appendix A.3),
 *   keep_budget    = round(seq_len / stage1)          tokens Stage 1 keeps,
 *   channel_budget = round(head_dim / head_ratio)     in [1, head_dim],
 *   attend_tokens  = max(1, t / 2)                    the token_budget argument
 *                                                     of the decode entry points.
 * storage, storage_mt and traffic are the RocketKV and RocketKV-MT rows of Table 1 as printed:
 *   storage = 1/c^r + 2/c^((1+r)/2),  storage_mt = 1 + 2/c^((1+r)/2),  traffic = 1/c,
 * relative to the full KV cache; they bound what the buffers of this library need (the K_max /
 * K_min pair of a page size ps costs 1/ps of the kept K/V, half of Table 1's auxiliary term).
 * Host arithmetic only (double precision); `out` is a host struct.
 */
typedef struct rocketkv_split {
  double c, r, stage1, stage2, head_ratio;
  int32_t page_size, keep_budget, channel_budget, attend_tokens;
  double storage, storage_mt, traffic;
} rocketkv_split_t;
int32_t rocketkv_decompose(int64_t seq_len, int32_t token_budget, int32_t head_dim,
                           rocketkv_split_t* out);

/*
 * Measurement aid (no step of the method): read `bytes` (a multiple of 16) of device memory at
 * `src` (16-byte aligned) once, front to back, with plain streaming loads, and write one checksum
 * word per wavefront to `sink` (device, at least rocketkv_stream_read_sink_bytes() bytes).  Timed
 * over a buffer much larger than the 256 MB last-level cache it gives the read bandwidth this GPU
 * actually reaches, which the benchmark prints beside the published peak.  Asynchronous on `stream`.
 */
int32_t rocketkv_stream_read(const void* src, size_t bytes, void* sink, void* stream);
size_t rocketkv_stream_read_sink_bytes(void);

/*
 * Measurement aid (no step of the method): read the K and V tiles of the listed pages (the list
 * rocketkv_hsa_select writes: int32 [batch][n_kv_heads][pages_row_len], entries < 0 skipped) with the
 * work split and the load pattern of the attention kernels, and compute nothing: no logits, no
 * softmax, no merge.  Timed beside rocketkv_attend on the same list it gives the floor this GPU puts
 * under Step 3 (Algorithm 1, y = attn(q, K[i2], V[i2])) for that list: the gather of 4 KiB tiles
 * itself, plus one launch.  Channel-major V, 16-token pages.  `sink`: device, at least
 * rocketkv_stream_gather_sink_bytes(cache, pages_row_len) bytes, one checksum word per wavefront.
 * Asynchronous on `stream`.
 */
int32_t rocketkv_stream_gather(const rocketkv_cache_t* cache, const int32_t* pages, int32_t pages_row_len,
                               void* sink, void* stream);
size_t rocketkv_stream_gather_sink_bytes(const rocketkv_cache_t* cache, int32_t pages_row_len);

/* Thread-local description of the last error returned on this thread ("" if none). */
const char* rocketkv_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int32_t rocketkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ROCKETKV_H */
