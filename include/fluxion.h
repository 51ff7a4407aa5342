/* fluxion.h -- C ABI of the MI355X block-sparse decode-attention library (libfluxion.so).
 *
 * The library implements, as HIP kernels for gfx950, the per-step hot path of block-sparse attention
 * over a long KV cache as the paper states it (Sec. 2.1): the cache of every KV head is cut into
 * logical blocks, each block is represented by the per-channel minimum and maximum of its keys, a
 * decode query is compared with that metadata to rank the blocks, the top-k blocks are chosen, and
 * attention runs over the tokens of the chosen blocks only.  The first tokens (sink) and the most
 * recent tokens (local window) are always attended to, and their contribution is fused with that of
 * the chosen blocks (Sec. 2.2, Sec. 3.2, Sec. 4 step 4).  Under GQA all query heads of a group share
 * the block size of their KV head while every query head has its own budget (Sec. 5.3).
 *
 * Conventions
 *   - Plain C types only.  bf16 tensors are passed as `const void*` / `void*` to 2-byte elements;
 *     `stream` is a hipStream_t passed as `void*` (NULL = the default stream).
 *   - Unless a parameter says HOST, every pointer is a DEVICE pointer owned by the caller.  The
 *     library allocates nothing, frees nothing and never synchronises: every call only enqueues
 *     kernels on `stream` and returns.  Buffers must stay valid until that work has finished.
 *   - All arguments that can be checked without touching the device are checked before the first HIP
 *     call; a failed check returns an error code and enqueues nothing.  No call aborts or throws.
 *   - Inputs are assumed finite.
 *
 * Geometry of one (sequence b, KV head j) with N = seq_len[b] tokens and block size g = gran[j]:
 *   blocks            i = 0 .. ceil(N / g) - 1, block i holds tokens [i*g, min((i+1)*g, N))
 *   sink blocks       i <  n_sink = ceil(sink_tokens / g)
 *   window blocks     i >= w0     = floor(max(N - window_tokens, 0) / g)
 *   candidate blocks  n_sink <= i < w0   (n_cand = max(w0 - n_sink, 0)); only these are ranked.
 */
#ifndef FLUXION_H
#define FLUXION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum fx_status {
  FX_OK = 0,
  FX_ERR_INVALID_ARG = 1,         /* null pointer, inconsistent sizes, misaligned pointer or stride      */
  FX_ERR_UNSUPPORTED = 2,         /* head_dim, group size, block size or context outside the built range */
  FX_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes below what fx_*_workspace_bytes reports              */
  FX_ERR_HIP = 4,                 /* a HIP launch failed; hipGetLastError() has the cause                 */
  FX_ERR_SCRATCH_LIMIT = 5        /* fx_sparse_decode_static: the problem needs more than the built-in scratch */
} fx_status;

/* Static, never-NULL description of a status code. */
const char* fx_status_string(fx_status status);

/* Placement of one layer's KV cache.  Element (b, j, t, c) of K (and of V) is at
 *     K[seq_base[b] + j * kv_head_stride + t * token_stride + c],   0 <= c < head_dim,
 * so head-major, token-major and ragged (unpadded) batches are all expressible.  The summary of block
 * i of (b, j) is the pair of rows
 *     S[((sum_base[b * n_kv_heads + j] + i) * 2 + 0) * head_dim + c]   (minimum)
 *     S[((sum_base[b * n_kv_heads + j] + i) * 2 + 1) * head_dim + c]   (maximum).
 * Supported: head_dim 64 or 128; n_q_heads a multiple of n_kv_heads with group size <= 8;
 * n_kv_heads <= 64; gran[j] a multiple of 16 in [16, 128]; max_seq_len <= 2^19; batch * n_kv_heads <= 4096.
 * Alignment: K, V, S and q 16-byte aligned; token_stride, kv_head_stride and every seq_base[b]
 * multiples of 8 elements; token_stride >= head_dim.
 */
typedef struct fx_layout {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t max_seq_len;     /* HOST bound: seq_len[b] <= max_seq_len.  Longer entries are clamped to it.   */
  const int32_t* seq_len;  /* DEVICE [batch]              valid tokens per sequence                        */
  const int64_t* seq_base; /* DEVICE [batch]              element offset of sequence b in K and in V       */
  int64_t kv_head_stride;  /* elements                                                                     */
  int64_t token_stride;    /* elements                                                                     */
  const int64_t* sum_base; /* DEVICE [batch * n_kv_heads] block offset of (b, j) in the summaries          */
  const int32_t* gran;     /* HOST   [n_kv_heads]         logical block size g_j                           */
} fx_layout;

/* Block key summaries (Sec. 2.1: per block, the dimension-wise maxima and minima of its token keys).
 * Reads every valid key once and writes, for every block of every (b, j), the minimum row and the
 * maximum row over the block's valid tokens (a partial last block covers its valid tokens only).
 * The values written are elements of K, bit for bit (for +-0 either sign may be kept).
 *   K          bf16, placed as fx_layout says
 *   summaries  bf16, written; must hold max over (b, j) of sum_base + ceil(seq_len/g) blocks
 * Errors: INVALID_ARG (null/misaligned), UNSUPPORTED (layout outside the supported range), HIP. */
fx_status fx_summarize(const fx_layout* layout, const void* K, void* summaries, void* stream);

/* Incremental summaries for a cache that grew (Sec. 2.1: the metadata of a logical block is the per-channel
 * minimum and maximum of the keys it holds, so a block's summary changes only while tokens are appended to it;
 * decode appends tokens, blocks fill up and leave the local window, where selection starts to need them).  Recomputes, for every (b, j), only the blocks
 * that hold tokens at or after prev_len[b]; seq_len[b] is the length after the append.  The result equals
 * fx_summarize on the grown cache provided the summaries of the blocks before prev_len[b] were up to date.
 *   prev_len        DEVICE int32 [batch]: length of each sequence before the append (<= seq_len[b])
 *   max_new_tokens  HOST bound on seq_len[b] - prev_len[b]; blocks beyond ceil(max_new_tokens/16) + 1 per
 *                   (b, j), counted from the block holding token prev_len[b], are not revisited
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
fx_status fx_summarize_append(const fx_layout* layout, const void* K, void* summaries, const int32_t* prev_len,
                              int32_t max_new_tokens, void* stream);

/* Bytes of scratch fx_select needs for this layout (HOST computation, depends on batch, n_q_heads,
 * max_seq_len and gran only).  Returns 0 if the layout is invalid. */
size_t fx_select_workspace_bytes(const fx_layout* layout);

/* Block scoring and per-head top-k (Sec. 2.1: compare the query with the metadata of all key blocks,
 * then select the top-k blocks; Sec. 5.3: one block size per group, one budget per head).
 * For query head h of sequence b (KV head j = h / group) and every candidate block i
 *     score(i) = sum_c max(q[c] * min_i[c], q[c] * max_i[c])
 * and the k_h candidates that come first in the order (score descending, index ascending) are kept,
 * with k_h = budget_blocks[b][h] if given, else ceil(budget_frac[b][h] * n_cand) evaluated in double,
 * clamped to [0, min(n_cand, k_max)].
 * Contract on precision: the kept set is the one that order gives with every score evaluated from the exact
 * products summed in double precision.  (How: scores are first computed approximately with a proven error
 * bound; every candidate closer to the k-th score than that bound is re-scored in double before it is ranked.
 * Two candidates whose double-precision scores agree to ~1e-16 relative may be ordered by summation order.)
 * Budgets larger than k_max: budgets are device data, so this cannot be an argument error; such a head keeps
 * its best k_max candidates and cnt reports k_max.  Size idx with k_max >= the largest k_h to avoid it.
 *   q              bf16 [batch][n_q_heads][head_dim]
 *   summaries      bf16, as written by fx_summarize for the same layout
 *   budget_frac    float [batch][n_q_heads], or NULL   } exactly one of the two
 *   budget_blocks  int32 [batch][n_q_heads], or NULL   } is non-NULL
 *   idx            int32 [batch][n_q_heads][k_max], written: the kept block indices in ascending
 *                  order, then -1 up to k_max
 *   cnt            int32 [batch][n_q_heads], written: k_h
 *   workspace      >= fx_select_workspace_bytes(layout) bytes, 16-byte aligned; contents undefined after;
 *                  calls that may overlap in time (different streams) need a workspace each
 * A budget of 0 keeps nothing (streaming head: only sink and window are attended, Sec. 3.2); a budget
 * of 1.0 keeps every candidate, which makes the later attention dense.
 * Errors: INVALID_ARG (null/misaligned, both or neither budget, k_max < 1, negative sink/window),
 * UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP. */
fx_status fx_select(const fx_layout* layout, const void* q, const void* summaries, const float* budget_frac,
                    const int32_t* budget_blocks, int32_t sink_tokens, int32_t window_tokens, int32_t k_max,
                    int32_t* idx, int32_t* cnt, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of scratch fx_sparse_decode needs (HOST computation; depends on the layout's host fields,
 * k_max, sink_tokens and window_tokens).  Returns 0 if the arguments are invalid. */
size_t fx_decode_workspace_bytes(const fx_layout* layout, int32_t k_max, int32_t sink_tokens, int32_t window_tokens);

/* Split-K sparse decode attention with online-softmax merge (App. A.1: s = q K^T / sqrt(D),
 * O = softmax(s) V, restricted to the kept tokens; Sec. 2.2 / Sec. 4 step 4: the partial results
 * over the chosen blocks and over the retained sink and window tokens are fused into one output).
 * Query head h of sequence b attends to the valid tokens of: its own chosen blocks
 * idx[b][h][0 .. cnt[b][h]), every sink block and every window block.  The blocks the heads of one
 * group need are read from HBM once per group; partial (max, sum, accumulator) triples of the splits
 * are merged in a fixed order, so results are reproducible run to run.
 *   q          bf16 [batch][n_q_heads][head_dim]
 *   K, V       bf16, placed as fx_layout says
 *   idx, cnt   as produced by fx_select, or any list of block indices; entries outside
 *              [0, n_blocks) are ignored, duplicates and entries inside sink/window are harmless,
 *              cnt is clamped to [0, k_max]
 *   out        float [batch][n_q_heads][head_dim], written (zeros for a sequence of length 0)
 *   workspace  >= fx_decode_workspace_bytes(...) bytes, 16-byte aligned; contents undefined after;
 *              calls that may overlap in time (different streams) need a workspace each
 * Arithmetic: bf16 inputs, fp32 products, sums, exponentials and accumulators.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP. */
fx_status fx_sparse_decode(const fx_layout* layout, const void* q, const void* K, const void* V, const int32_t* idx,
                           const int32_t* cnt, int32_t k_max, int32_t sink_tokens, int32_t window_tokens, float* out,
                           void* workspace, size_t workspace_bytes, void* stream);

/* fx_sparse_decode for callers that cannot allocate device memory (code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc) and therefore cannot bring a workspace: the same computation,
 * the same kernels and the same result bits as fx_sparse_decode, with the scratch taken from a buffer of
 * FX_STATIC_SCRATCH_BYTES that is built into the library (each GPU the library runs on holds one copy of it
 * from the first call on that GPU until the process ends).  The call allocates and frees nothing.
 * Limit: the scratch the problem needs at this device's launch size -- union lists of
 * batch * n_kv_heads * min(blocks, sink + window blocks + group * k_max) * 4 bytes plus partial results of
 * (9 * launched workgroups + 2 * batch * n_kv_heads + 8) * group * (head_dim + 2) * 4 bytes -- must fit, else
 * FX_ERR_SCRATCH_LIMIT is returned and nothing is enqueued (on MI355X every named configuration of up to 8
 * heads per group at head_dim 128 fits).
 * All calls on one GPU share that GPU's buffer: calls that may overlap in time on one GPU (different streams
 * or threads) race; serialise them or use fx_sparse_decode with a workspace each.  Nothing in the buffer needs
 * clearing between calls (the one counter that must start at zero is reset by the call's first kernel).
 * The first call on a device looks up the buffer's device address and the kernel's occupancy (no allocation, but
 * runtime queries): make that first call outside stream capture; later calls only enqueue kernels.
 * Other arguments and errors as fx_sparse_decode. */
#define FX_STATIC_SCRATCH_BYTES (48u << 20)
fx_status fx_sparse_decode_static(const fx_layout* layout, const void* q, const void* K, const void* V,
                                  const int32_t* idx, const int32_t* cnt, int32_t k_max, int32_t sink_tokens,
                                  int32_t window_tokens, float* out, void* stream);

/* Group-union variant of fx_sparse_decode: every query head of a GQA group attends to the union of the blocks
 * chosen by the heads of its group (plus sink and window).  The group's blocks are in registers for all its
 * heads anyway (Sec. 5.3 bounds a group's data volume by the sum of its heads' budgets because the union is
 * what is actually moved), so the extra tokens cost arithmetic but no extra HBM traffic.  Same arguments,
 * workspace and errors as fx_sparse_decode. */
fx_status fx_sparse_decode_union(const fx_layout* layout, const void* q, const void* K, const void* V,
                                 const int32_t* idx, const int32_t* cnt, int32_t k_max, int32_t sink_tokens,
                                 int32_t window_tokens, float* out, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* Granularity-budget selector (Sec. 5.2 Eq. 1: bgt_h(blk) = bgt0_h + k_h * log2(blk); Sec. 5.3 Eq. 3: the data
 * volume of a GQA group at block size blk is V(blk) = 2 * L_cpu / blk + 2 * L_cpu * sum_h bgt_h(blk), metadata
 * plus selected KV, counted in keys).  HOST control logic, all pointers are HOST pointers.  For every KV head
 * the candidate block size with the smallest V is chosen (ties: the earlier candidate) and every head's budget
 * follows from Eq. 1 at that size, clipped to [0, 1].  Streaming heads (Sec. 3.2) get budget 0 and add nothing
 * to V; a group made of streaming heads only keeps candidates[0] and reports V = 0 (it is not scheduled).
 *   bgt0, slope   float [n_q_heads]: predicted head properties (budget at block size 1, growth per log2 block)
 *   streaming     uint8 [n_q_heads] or NULL (no streaming heads): non-zero marks a streaming head
 *   l_cpu         number of keys selection runs over (the candidate tokens)
 *   candidates    int32 [n_candidates], e.g. {16, 32, 64, 128}
 *   gran          int32 [n_kv_heads], written;  budget float [n_q_heads], written (feeds fx_select's budget_frac)
 *   volume        double [n_kv_heads] or NULL, written: V at the chosen size.  Informational: the paper orders its
 *                 CPU/GPU task queue by it (Sec. 6.2); this library balances by bytes inside one launch and
 *                 consumes no priority
 * Errors: INVALID_ARG. */
fx_status fx_choose_granularity(int32_t n_q_heads, int32_t n_kv_heads, const float* bgt0, const float* slope,
                                const uint8_t* streaming, int64_t l_cpu, const int32_t* candidates,
                                int32_t n_candidates, int32_t* gran, float* budget, double* volume);

/* Summary pyramid (Sec. 2.1: blocks are logical, so the same cache can be viewed at several block sizes; Sec. 5.3
 * picks the size per group and step): summaries of a coarser block size from finer ones, exactly (a block of r*g tokens is r
 * blocks of g tokens, so its minimum row is the minimum of their minimum rows and likewise for the maximum).
 * `fine` and `coarse` describe the same sequences (equal seq_len contents) and differ only in gran[] and
 * sum_base[]; coarse->gran[j] must be
 * a multiple of fine->gran[j] (both valid block sizes).  Reads 1/g of what fx_summarize reads.  The result is
 * identical to fx_summarize run with `coarse`.
 * Errors: INVALID_ARG (null/misaligned, layouts that differ in shape), UNSUPPORTED, HIP. */
fx_status fx_coarsen_summaries(const fx_layout* fine, const void* fine_summaries, const fx_layout* coarse,
                               void* coarse_summaries, void* stream);

/* Test aid (not part of the method; the layout it describes is an implementation detail that may change with
 * the kernels): where fx_select leaves its intermediate values inside the workspace after a call.  It exists so
 * that a test can check the error bound the selection contract above rests on against an independent fp64 score.  Candidates
 * are numbered c = i - n_sink (block index minus the number of sink blocks) and handled in tiles of 16.
 * With G = n_q_heads / n_kv_heads, j = h / G and r = h % G, the approximate score of candidate c for (b, h) is
 * the float at byte offset
 *     *approx_offset + 4 * ((((b * n_kv_heads + j) * (*mag_stride) + c / 16) * G + r) * 16 + c % 16)
 * and the largest magnitude sum (the bound of the rounding error) over the tile of c is the float at
 *     *mag_offset + 4 * ((b * n_q_heads + h) * (*mag_stride) + c / 16).
 * `*gamma` is the factor of the bound |approx - exact| <= gamma * magnitude that the selection relies on;
 * `*row_stride` is the row length of the per-(b, h) block arrays (fallback keys).
 * Returns INVALID_ARG/UNSUPPORTED for a bad layout. */
fx_status fx_select_workspace_view(const fx_layout* layout, size_t* approx_offset, size_t* mag_offset,
                                   int64_t* row_stride, int64_t* mag_stride, float* gamma);

/* Measurement aid (not part of the method).  While enabled, fx_select and fx_sparse_decode bracket every
 * kernel they launch with HIP events recorded on the caller's stream; fx_profile_read waits for the
 * events of the most recent call of each and returns the kernel durations in milliseconds:
 *   ms[0] block scoring, ms[1] top-k, ms[2] union-list planning, ms[3] split-K attention, ms[4] merge.
 * Enabling creates the events (the only place the library creates HIP objects); disabling destroys
 * them.  Entries of kernels that have not run since enabling are -1.  `n` must be 5.
 * Not thread-safe; meant for benchmarks.  Errors: INVALID_ARG, HIP. */
#define FX_PROFILE_SLOTS 5
fx_status fx_profile_enable(int enable);
fx_status fx_profile_read(float* ms, int n);

/* Measurement aids (not part of the method): a plain streaming read of `bytes` bytes at `src`
 * (nothing is written unless a data-dependent check that practically never holds fires; `sink` must
 * point to at least 4 writable bytes) and a plain copy.  Both run `wg_per_cu` (1..32) persistent
 * workgroups per compute unit with 16-byte loads.  `bytes` is rounded down to a multiple of 16.
 * Errors: INVALID_ARG (null, misaligned, bytes < 16), HIP. */
fx_status fx_probe_read(const void* src, size_t bytes, void* sink, int wg_per_cu, void* stream);
/* The same read with non-temporal loads (the kind the attention kernel uses for K and V rows, which are
 * read once per step): on MI355X it streams about 10% faster than the plain read.  Same arguments and errors. */
fx_status fx_probe_read_streaming(const void* src, size_t bytes, void* sink, int wg_per_cu, void* stream);
fx_status fx_probe_copy(void* dst, const void* src, size_t bytes, int wg_per_cu, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLUXION_H */
