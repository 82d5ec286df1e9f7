/*
 * powattn.h -- C ABI of the MI355X (gfx950) PowerAttention forward library.
 *
 * The library computes causal block-sparse attention under the static pattern
 * of the PowerAttention paper (arXiv 2503.03588): every query block attends a
 * local window of key blocks, the key blocks at power-of-two block distances,
 * and the first ("sink") blocks of the sequence.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary process memory.  The library never allocates,
 *     frees or keeps any pointer; the caller owns every buffer.
 *   - Device work is enqueued on `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and the call returns without waiting for it.
 *   - Tensors are contiguous, innermost stride 1, in the layouts stated below.
 *   - Every function returns a POWATTN_* status (or documents its own return
 *     value).  Argument errors are found on the host before anything is
 *     launched, so no kernel runs when the status is not POWATTN_OK.
 *     Nothing aborts or throws.
 */
#ifndef POWATTN_H
#define POWATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define POWATTN_OK                   0
#define POWATTN_INVALID_ARG          1  /* null pointer, non-positive size, Hq % Hkv != 0, length > capacity ... */
#define POWATTN_UNSUPPORTED          2  /* head_dim, block size or dtype the kernels are not built for */
#define POWATTN_WORKSPACE_TOO_SMALL  3  /* workspace_bytes or max_k below what the call needs */
#define POWATTN_HIP_ERROR            4  /* the HIP runtime refused a launch; see powattn_strerror */

/* powattn_pattern.flags */
#define POWATTN_POWER  1u  /* attend block distances that are zero or a power of two (the power term of Algorithm 1) */
#define POWATTN_DENSE  2u  /* full causal attention, A_i = {j <= i} (Section 3.1); other fields except block are ignored */

/* element types of Q/K/V/O */
#define POWATTN_BF16 0
#define POWATTN_F32  1

/*
 * The pattern's hyper-parameters, in the notation of Algorithm 1 (Section 3.3).
 * With d = floor(q/B) - floor(kv/B) the distance in blocks, query token q attends
 * key token kv when kv <= q and at least one of: d < W (local window), d is zero
 * or a power of two (POWATTN_POWER), kv lies in the first S blocks (sink).
 * Algorithm 1 has S = 1; Section 4.1 uses B = 256, W = 5, S = 1.  Because the
 * power term admits d == 0, the diagonal block is attended even when W == 0.
 * Without POWATTN_POWER (sliding window + sink, the first baseline of
 * Section 4.1) W must be >= 1.
 */
typedef struct {
  int32_t block;   /* B: tokens per block, >= 1 */
  int32_t window;  /* W: block distances 0..W-1 are attended, >= 0 */
  int32_t sink;    /* S: the first S key blocks are always attended, >= 0 */
  uint32_t flags;  /* POWATTN_POWER | POWATTN_DENSE */
} powattn_pattern;

/* Library version: major*10000 + minor*100 + patch. */
int powattn_version(void);

/* Static, human-readable text for a status code (never NULL). For
 * POWATTN_HIP_ERROR the text of the last HIP error seen by the calling thread
 * is appended. */
const char* powattn_strerror(int status);

/* Number of blocks nb = ceil(seq_len / B), or -POWATTN_INVALID_ARG. */
int64_t powattn_num_blocks(const powattn_pattern* pattern, int64_t seq_len);

/*
 * Row capacity: the largest number of key blocks any query block of a
 * seq_len-token sequence attends (O(log nb) for the power pattern: at most
 * W + S + the powers of two below nb; Theorem B.1 bounds the power part by
 * log n).  Host-only.  Returns the capacity (>= 1) or -status.
 */
int32_t powattn_max_k(const powattn_pattern* pattern, int64_t seq_len);

/*
 * Host-side enumeration of one row of the block-sparse pattern: writes the
 * ascending key-block indices attended by query block `q_block` to
 * `out` (host, `capacity` entries) and returns how many there are, or -status
 * (-POWATTN_WORKSPACE_TOO_SMALL when capacity is short; nothing is written
 * beyond `capacity`).  `out` may be NULL with capacity 0 to query the count.
 */
int32_t powattn_row_host(const powattn_pattern* pattern, int64_t q_block, int32_t* out, int32_t capacity);

/*
 * Step "block-index generation" (Algorithm 1 lifted to blocks, Sections 3.3
 * and 4.1): for each query block i in [0, nb) emit the ascending, duplicate-
 * free list of key blocks j <= i that some token of block i attends.
 *   d_kv_cnt     device int32 [nb]            out: list lengths
 *   d_kv_idx     device int32 [nb, max_k]     out: lists, padded with -1
 *   max_k        row capacity of d_kv_idx; must be >= powattn_max_k(...)
 *   d_block_mask device uint8 [nb, nb] or NULL  out: 1 where block j is in row i
 * Errors: INVALID_ARG (null pattern/outputs, seq_len <= 0, bad pattern),
 * WORKSPACE_TOO_SMALL (max_k short), HIP_ERROR.
 */
int powattn_mask_build(const powattn_pattern* pattern, int64_t seq_len,
                       int32_t* d_kv_cnt, int32_t* d_kv_idx, int32_t max_k,
                       uint8_t* d_block_mask, void* hip_stream);

/*
 * Prefill: Equation 1 (Section 3.1) for every query token, with A_i given by
 * the block lists: for query block i, every token of a listed block j < i is
 * attended, and inside the diagonal block j == i token q attends kv <= q.
 *   d_kv_cnt, d_kv_idx, max_k   lists as written by powattn_mask_build for the
 *                  same pattern.block and seq_len (any causal block list is
 *                  accepted: entries outside [0, i] are skipped).  Ignored,
 *                  and may be NULL, when pattern->flags has POWATTN_DENSE.
 *   q, o           device [batch, n_q_heads, seq_len, head_dim]
 *   k, v           device [batch, n_kv_heads, seq_len, head_dim]; query head h
 *                  reads KV head h / (n_q_heads / n_kv_heads)
 *   lse            device float [batch, n_q_heads, seq_len] or NULL:
 *                  natural-log sum of exp(scaled logits) over the attended keys
 *   dtype          POWATTN_BF16 (MFMA path, fp32 accumulation; head_dim 64 or 128,
 *                  block a multiple of 64, at most 1024) or POWATTN_F32 (plain FMA path;
 *                  head_dim 64 or 128, block 16..256 and a multiple of 16)
 *   softmax_scale  logit scale; <= 0 selects 1/sqrt(head_dim) (Equation 1)
 * seq_len need not be a multiple of the block size.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP_ERROR.
 */
int powattn_prefill(const powattn_pattern* pattern,
                    const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                    const void* q, const void* k, const void* v, void* o, float* lse,
                    int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                    int64_t seq_len, int32_t head_dim, int32_t dtype,
                    float softmax_scale, void* hip_stream);

/*
 * Chunked prefill against a KV cache (what serving needs between powattn_prefill
 * and powattn_decode: a long prompt processed in pieces, or a prompt appended to
 * a cached prefix).  The q_len query tokens sit at positions q_start ..
 * q_start + q_len - 1 of their sequences; the caches already hold the keys and
 * values of positions 0 .. q_start + q_len - 1.  The result equals rows
 * q_start .. q_start + q_len - 1 of powattn_prefill over those positions
 * (Equation 1 with the same A_i), bit for bit.
 *   d_kv_cnt, d_kv_idx, max_k   block lists indexed by the block number in the
 *                  whole sequence (as powattn_mask_build writes them for any
 *                  seq_len >= q_start + q_len, e.g. the cache capacity)
 *   q, o           device [batch, n_q_heads, q_len, head_dim]
 *   k_cache, v_cache  device [batch, n_kv_heads, cache_capacity, head_dim]
 *   lse            device float [batch, n_q_heads, q_len] or NULL
 *   q_start        any position >= 0 (a chunk may start and end inside a block);
 *                  q_start + q_len <= cache_capacity
 *   dtype          POWATTN_BF16 only; head_dim 64 or 128; block a multiple of 64, at most 1024
 * Errors: INVALID_ARG, UNSUPPORTED, HIP_ERROR.
 */
int powattn_prefill_chunk(const powattn_pattern* pattern,
                          const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                          const void* q, const void* k_cache, const void* v_cache, void* o, float* lse,
                          int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                          int64_t q_start, int64_t q_len, int64_t cache_capacity,
                          int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream);

/*
 * powattn_prefill_chunk over a paged KV cache (the layout of powattn_decode_paged):
 * a piece of a prompt is processed against keys and values that live in pages of
 * one block each, which is how a serving system that decodes from pages (Section
 * 4.3: prefill plus decode steps end to end) also has to prefill.  The result is,
 * bit for bit, that of powattn_prefill_chunk on the contiguous cache the pages
 * spell out.
 *   q, o              device [batch, n_q_heads, q_len, head_dim], rows = positions
 *                     q_start .. q_start+q_len-1 (q_start anywhere, also inside a block)
 *   lse               device [batch, n_q_heads, q_len] fp32, or null
 *   k_pages, v_pages  device [n_pages, n_kv_heads, block, head_dim]; positions
 *                     0 .. q_start+q_len-1 of every sequence must be filled in
 *   d_block_table     device int32 [batch, table_stride]: entry [b][j] is the page of
 *                     tokens j*block .. (j+1)*block-1 of sequence b; a page number
 *                     outside [0, n_pages) is clamped into the pool by the kernel
 *                     (wrong numbers, no stray access); q_start+q_len <= table_stride*block
 *   d_kv_cnt, d_kv_idx, max_k   the block lists, indexed by the block number in the
 *                     sequence (built for at least q_start+q_len tokens)
 *   dtype             POWATTN_BF16 only; head_dim 64 or 128; block a multiple of 64, at
 *                     most 1024; max_k <= 63 and max_k * block / 64 <= 1024;
 *                     n_pages * n_kv_heads * block < 2^31.  POWATTN_DENSE is not
 *                     supported here (UNSUPPORTED): copy the pages out, or decode.
 * One kernel launch; allocates nothing.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP_ERROR.
 */
int powattn_prefill_chunk_paged(const powattn_pattern* pattern,
                                const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* d_block_table, int32_t table_stride, int64_t n_pages,
                                void* o, float* lse,
                                int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                int64_t q_start, int64_t q_len,
                                int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream);

/*
 * A serving step's prefill work in one launch: for every sequence of the batch a
 * piece of its prompt (its own start and its own number of rows) against the
 * paged KV cache of powattn_prefill_chunk_paged.  Sequence b's rows are the
 * positions d_q_start[b] .. d_q_start[b]+d_q_len[b]-1; the result is, bit for
 * bit, that of powattn_prefill_chunk_paged called for each sequence alone
 * (Equation 1 over the blocks of Algorithm 1; Section 4.3 for the setting).
 *   q, o              device [batch, n_q_heads, q_rows, head_dim]: row r of sequence b is
 *                     position d_q_start[b] + r; rows r >= d_q_len[b] are neither read nor written
 *   lse               device [batch, n_q_heads, q_rows] fp32, or null
 *   d_q_start         device int32 [batch], >= 0 (clamped into [0, table_stride*block])
 *   d_q_len           device int32 [batch], 0 <= d_q_len[b] <= q_rows (clamped so that the context
 *                     d_q_start[b] + d_q_len[b] stays inside the table); 0: the sequence is skipped
 *   q_rows            rows per (sequence, head) slab of q/o/lse, 1 <= q_rows <= table_stride*block
 *   k_pages, v_pages, d_block_table, table_stride, n_pages   as for powattn_prefill_chunk_paged;
 *                     positions 0 .. d_q_start[b]+d_q_len[b]-1 of sequence b must be filled in
 *   d_kv_cnt, d_kv_idx, max_k   the block lists, built for at least table_stride*block tokens
 *                     (or for the longest context of the batch)
 * Limits as for powattn_prefill_chunk_paged.  The lengths are read by the kernel: no
 * host synchronisation, one launch whatever the mix of lengths; work is dealt by
 * position in the padded batch, so q_rows should not be much larger than the longest piece.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP_ERROR.
 */
int powattn_prefill_batch_paged(const powattn_pattern* pattern,
                                const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                                const void* q, const void* k_pages, const void* v_pages,
                                const int32_t* d_block_table, int32_t table_stride, int64_t n_pages,
                                const int32_t* d_q_start, const int32_t* d_q_len, int64_t q_rows,
                                void* o, float* lse,
                                int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                                int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream);

/*
 * powattn_prefill for a batch of sequences of different lengths (what a serving
 * batch of prompts looks like; Section 4.3 measures end-to-end generation), in
 * ONE launch, with the lengths in device memory (no host copy, no
 * synchronisation; they may be the output of an earlier kernel on the stream).
 * The tensors are padded to `padded_len` rows per head; sequence b uses rows
 * 0 .. seq_len[b]-1 and its other rows of o and lse are left untouched.  A row of
 * the block lists does not depend on the sequence length (Algorithm 1 looks at
 * positions only), so one pair of lists built for padded_len serves all.  The
 * result for each sequence equals powattn_prefill on that sequence alone, bit
 * for bit.
 *   q, o           device [batch, n_q_heads, padded_len, head_dim]
 *   k, v           device [batch, n_kv_heads, padded_len, head_dim]
 *   lse            device float [batch, n_q_heads, padded_len] or NULL
 *   d_seq_len      device int32 [batch], 0 <= seq_len[b] <= padded_len (0: nothing
 *                  to do; values outside that range are clamped into it by the kernel)
 *   d_kv_cnt, d_kv_idx, max_k   lists covering ceil(padded_len / block) rows
 *   dtype          POWATTN_BF16 only; head_dim 64 or 128; block a multiple of 64, at most 1024
 * Work is dealt to the compute units by position in the padded batch, not by
 * length, in an order that keeps them level for any mix of lengths when there
 * are 1, 2 or a multiple of 8 KV heads (every part of the chip then sees every
 * sequence); with other head counts a part sees some of the sequences, and a
 * batch whose long sequences sit next to one another is balanced less well
 * than a shuffled one.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP_ERROR.
 */
int powattn_prefill_varlen(const powattn_pattern* pattern,
                           const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                           const void* q, const void* k, const void* v, void* o, float* lse,
                           int32_t batch, int32_t n_q_heads, int32_t n_kv_heads,
                           const int32_t* d_seq_len, int64_t padded_len,
                           int32_t head_dim, int32_t dtype, float softmax_scale, void* hip_stream);

/*
 * Bytes of device workspace powattn_decode needs for caches of up to
 * `cache_capacity` tokens (0 on invalid arguments).  It holds the split-K
 * partial results when a (sequence, KV head) is spread over several workgroups.
 */
size_t powattn_decode_workspace_bytes(const powattn_pattern* pattern, int32_t batch,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                      int64_t cache_capacity);

/*
 * Decode: one new token per sequence attends its KV cache under the same
 * pattern as prefill (Section 4.1 keeps one pattern for both phases).  The
 * cache already holds the new token's key and value, so
 * the query of sequence b sits at position t = kv_len[b] - 1 and the result
 * equals row t of powattn_prefill over the first kv_len[b] cache positions.
 * The attended block list of row floor(t / B) is generated inside the kernel;
 * the work is split over the attended blocks and combined (split-K).
 *   q, o           device [batch, n_q_heads, head_dim]
 *   k_cache, v_cache  device [batch, n_kv_heads, cache_capacity, head_dim]
 *   d_kv_len       device int32 [batch], 1 <= kv_len[b] <= cache_capacity
 *                  (values outside that range are clamped into it by the kernel)
 *   lse            device float [batch, n_q_heads] or NULL
 *   dtype          POWATTN_BF16 only; head_dim 64 or 128; block a multiple of 64, at most 1024
 *   workspace      device, at least powattn_decode_workspace_bytes(...) bytes,
 *                  256-byte aligned; needs no initialisation.  It holds the
 *                  partial results of the workgroups that share a (sequence,
 *                  KV head), each value tagged with a generation number that is
 *                  also kept there and advanced by every call, so that a call
 *                  tells its own partials from whatever the memory held before.
 *                  Two calls that may run at the same time must not share a
 *                  workspace; there is no other limit on calls in flight.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR.
 */
int powattn_decode(const powattn_pattern* pattern,
                   const void* q, const void* k_cache, const void* v_cache,
                   const int32_t* d_kv_len, int64_t cache_capacity,
                   void* o, float* lse,
                   int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                   int32_t dtype, float softmax_scale,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * powattn_decode for callers that cannot allocate device memory for a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation).  Same arguments and result as powattn_decode, without the
 * workspace: the partial results go to a buffer of POWATTN_STATIC_SCRATCH_BYTES
 * bytes that the library holds in its own device memory on every GPU it runs on,
 * from the time it is loaded until the process ends.  The call allocates and
 * frees nothing.  A shape whose powattn_decode_workspace_bytes(...) exceeds that
 * size is refused with POWATTN_WORKSPACE_TOO_SMALL before anything is launched.
 * All calls on one GPU share the one buffer: calls that may overlap in time on
 * the same GPU (different streams) race and must be serialised by the caller.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR.
 */
#define POWATTN_STATIC_SCRATCH_BYTES (32u << 20)
int powattn_decode_static(const powattn_pattern* pattern,
                          const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* d_kv_len, int64_t cache_capacity,
                          void* o, float* lse,
                          int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                          int32_t dtype, float softmax_scale, void* hip_stream);

/*
 * powattn_decode over a paged KV cache, the form serving systems keep their
 * caches in (Section 4.3 measures prefill plus 1024 decode steps end to end).
 * A page holds one block of the pattern (pattern->block tokens) for every KV
 * head; a table per sequence says which page holds which block, so the attended
 * blocks of a row (Algorithm 1) are a dozen table look-ups.  The result equals
 * powattn_decode on the cache those pages spell out.
 *   k_pages, v_pages  device [n_pages, n_kv_heads, block, head_dim]
 *   d_block_table     device int32 [batch, table_stride]: entry [b][j] is the page of
 *                     tokens j*block .. (j+1)*block-1 of sequence b; entries of blocks
 *                     beyond the sequence are not read.  A page number outside
 *                     [0, n_pages) is clamped into the pool by the kernel (wrong
 *                     numbers, no stray access).
 *   d_kv_len          device int32 [batch], 1 <= kv_len[b] <= table_stride * block
 *                     (clamped into that range by the kernel)
 *   workspace         as for powattn_decode with cache_capacity = table_stride * block
 * Everything else as for powattn_decode.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR.
 */
int powattn_decode_paged(const powattn_pattern* pattern,
                         const void* q, const void* k_pages, const void* v_pages, int64_t n_pages,
                         const int32_t* d_block_table, int32_t table_stride,
                         const int32_t* d_kv_len,
                         void* o, float* lse,
                         int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         int32_t dtype, float softmax_scale,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Gradients of powattn_prefill (Equation 1, Section 3.1; the paper trains with
 * the pattern in place, Section 4.1): given dO, the inputs, the output and the
 * log-sum-exp of a whole-sequence powattn_prefill call, writes
 *   dQ = scale * dS K,  dK = scale * dS^T Q,  dV = P^T dO,
 *   P = exp(scale * Q K^T - lse) on attended pairs, dS = P * (dO V^T - rowsum(dO * O)),
 * the gradients of sum(O * dO).  dK and dV of a KV head sum over its query heads.
 *   d_kv_cnt, d_kv_idx, max_k   the lists powattn_mask_build wrote for this pattern and
 *                  seq_len (dQ walks the rows; dK/dV walk the columns, which are
 *                  generated from the pattern in closed form, so the lists must be
 *                  the pattern's own: max_k < powattn_max_k is refused)
 *   q, o, d_o, dq  device [batch, n_q_heads, seq_len, head_dim]
 *   k, v, dk, dv   device [batch, n_kv_heads, seq_len, head_dim]
 *   lse            device float [batch, n_q_heads, seq_len], as written by powattn_prefill
 *   dtype          POWATTN_BF16 only; head_dim 64 or 128; block 64, 128 or 256; not POWATTN_DENSE
 *   workspace      device, powattn_backward_workspace_bytes(...) bytes, 256-byte aligned,
 *                  contents on entry ignored (rowsum(dO * O), and fp32 sums for the sink
 *                  blocks, whose columns are cut into parts that add up with atomics:
 *                  the last bits of the sink rows of dK/dV depend on the order of arrival)
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR.
 */
size_t powattn_backward_workspace_bytes(const powattn_pattern* pattern, int32_t batch, int32_t n_q_heads,
                                        int32_t n_kv_heads, int64_t seq_len, int32_t head_dim);
int powattn_backward(const powattn_pattern* pattern,
                     const int32_t* d_kv_cnt, const int32_t* d_kv_idx, int32_t max_k,
                     const void* q, const void* k, const void* v, const void* o, const float* lse,
                     const void* d_o, void* dq, void* dk, void* dv,
                     int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int64_t seq_len,
                     int32_t head_dim, int32_t dtype, float softmax_scale,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* POWATTN_H */
