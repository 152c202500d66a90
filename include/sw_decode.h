/*
 * sw_decode.h -- C ABI of the MI355X (gfx950) decode-attention library.
 *
 * The operation is one token-generation step's attention, as the paper states
 * the step (section 2.2, "Generative LLM inference phases": the newest token
 * and the request's KV cache are the inputs of the forward pass; section 3.5,
 * "Memory utilization": each active token reads the cache of its entire
 * context), batched over requests (section 3.4, "Throughput": token phases of
 * up to 64 requests are batched), at one GPU's tensor-parallel share of the
 * heads (section 2.5, "Model parallelism": tensor parallelism over 8 GPUs).
 * The attention itself is the scaled dot-product attention the paper reaches
 * by citation in section 2.1:
 *
 *   for request r, query head h, key/value head g = h / (n_qh / n_kvh),
 *   L = clamp(seq_lens[r], 0, max_len):
 *     out[r,h,:] = sum_{t<L} softmax_t( q[r,h,:] . K[r,g,t,:] / sqrt(head_dim) ) * V[r,g,t,:]
 *     out[r,h,:] = +0 when L == 0.
 *
 * Inputs and output are IEEE binary16; products and sums are accumulated in
 * binary32; the output is rounded to binary16 with round-to-nearest-even.
 *
 * Every function returns an int: SW_OK (0) or a negative SW_ERR_* code.
 * Nothing here throws, aborts or prints.  All scalar and pointer validation
 * happens before the first HIP call, so bad arguments are reported even on a
 * machine with no GPU.
 */
#ifndef SW_DECODE_H
#define SW_DECODE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SW_OK               0
#define SW_ERR_NULL        -1  /* a required pointer is NULL while n_req > 0            */
#define SW_ERR_SHAPE       -2  /* n_req < 0, n_qh/n_kvh/max_len <= 0, n_qh % n_kvh != 0,
                                  or a size whose element count overflows the library's
                                  limits (see sw_decode_attn)                           */
#define SW_ERR_UNSUPPORTED -3  /* head_dim not in {64, 128}; n_qh / n_kvh > 64          */
#define SW_ERR_ALIGN       -4  /* q, k_cache, v_cache or out not 16-byte aligned,
                                  seq_lens not 4-byte aligned                            */
#define SW_ERR_HIP         -5  /* a HIP call failed (no device, allocation, launch);
                                  text in sw_last_error()                                */
#define SW_ERR_PARAM       -6  /* sw_set_param: unknown key or value out of range        */
#define SW_ERR_STATE       -7  /* sw_prof_*: called out of order                          */

#define SW_F16 1               /* sw_kv_layout_t.dtype: IEEE binary16                    */

/*
 * How the library wants the K and V caches laid out.  Strides are in ELEMENTS
 * (binary16 values), not bytes.  Element (r, g, t, j) of a cache -- request r,
 * key/value head g, token position t, dimension j -- lives at
 *     base + r*stride_req + g*stride_kvh + t*stride_tok + j*stride_dim.
 * The logical order is [req][kv_head][token][dim] with dim contiguous
 * (stride_dim == 1) and a token's row dense (stride_tok == head_dim); the
 * strides of the two outer axes may carry padding, so callers must index
 * through them and never assume a dense array.  Positions t >= seq_lens[r]
 * and all padding are never read into a result; their content is arbitrary.
 */
typedef struct sw_kv_layout_t {
    int32_t dtype;        /* SW_F16                                                    */
    int32_t elem_bytes;   /* 2                                                         */
    int64_t stride_req;   /* elements between consecutive requests                     */
    int64_t stride_kvh;   /* elements between consecutive key/value heads              */
    int64_t stride_tok;   /* elements between consecutive token positions (= head_dim) */
    int64_t stride_dim;   /* 1                                                         */
    int64_t total_elems;  /* elements to allocate for ONE cache buffer (K or V)         */
    int32_t base_align;   /* required alignment of each buffer's base address, bytes   */
    int32_t reserved;     /* 0                                                         */
} sw_kv_layout_t;

/*
 * sw_kv_layout -- layout query for the per-request KV state of the step
 * (section 2.2: the KV cache keeps the attention context of every earlier
 * token of a request; section 3.5: it grows with the tokens in the batch).
 * Pure host arithmetic, no HIP call.  `out` is host memory owned by the
 * caller.  Errors: SW_ERR_NULL (out), SW_ERR_SHAPE, SW_ERR_UNSUPPORTED.
 */
int sw_kv_layout(int n_req, int n_kvh, int head_dim, int max_len, sw_kv_layout_t *out);

/*
 * sw_decode_attn -- one decode step's attention for a batch of requests
 * (sections 2.2, 3.4 and 3.5 as cited at the top of this file).
 *
 *   q         DEVICE, binary16, dense [n_req][n_qh][head_dim]; the newest
 *             token's query vectors.  Read only.
 *   k_cache   DEVICE, binary16, laid out as sw_kv_layout(n_req, n_kvh,
 *             head_dim, max_len) says.  Read only.
 *   v_cache   DEVICE, same layout as k_cache, a separate buffer.  Read only.
 *   seq_lens  DEVICE, int32 [n_req]; the number of cached positions of each
 *             request, the newest token included.  Never read by the host.
 *             Values outside [0, max_len] are clamped on the device.
 *   out       DEVICE, binary16, dense [n_req][n_qh][head_dim].  Fully
 *             overwritten (rows of requests with length 0 become +0).
 *   n_req >= 0; n_qh, n_kvh > 0 with n_qh % n_kvh == 0 and n_qh / n_kvh <= 64;
 *   head_dim in {64, 128}; 0 < max_len <= 2^23; n_req * n_qh and
 *   n_req * n_kvh at most 2^20.
 *   stream    a hipStream_t passed as void*; NULL is the default stream.
 *
 * The call enqueues its kernels on `stream` and returns without waiting for
 * them.  All buffers stay owned by the caller, who must keep them alive and
 * unmodified until the enqueued work has finished; the library keeps no
 * pointer past that.  Between its kernels the call uses a workspace for
 * partial results that the library owns: one per (device, stream), grown on
 * demand (a growing call allocates, which synchronises the device), never
 * shrunk, released by sw_release() or at process exit.  Two calls on the SAME
 * stream are ordered; calls on different streams use different workspaces and
 * may overlap.  The call may be recorded into a HIP graph (stream capture)
 * once a call of the same or a larger shape has run on that stream outside
 * any capture: a call that has to grow the workspace allocates and
 * synchronises, which a capture does not allow (SW_ERR_HIP where the runtime
 * refuses it).  A recorded call holds the workspace's address in its kernel
 * arguments: a later call that grows the workspace takes a new block and leaves
 * the old one allocated until sw_release(), so graphs recorded earlier stay
 * valid -- until sw_release(), after which they must not be launched again.
 * The workspace belongs to the stream the call was RECORDED on: launch such a
 * graph on that stream, or make sure no other call that uses the same stream's
 * workspace (eager, or another graph recorded there) can run at the same time;
 * the library cannot order them.  The result of a request does not depend on which other
 * requests share the batch, and repeating a call gives the same bits.
 * n_req == 0 returns SW_OK without touching the device.
 * Errors: SW_ERR_NULL, SW_ERR_SHAPE, SW_ERR_UNSUPPORTED, SW_ERR_ALIGN (all
 * before any HIP call), SW_ERR_HIP.
 */
int sw_decode_attn(const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *seq_lens, void *out,
                   int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                   void *stream);

/*
 * Block-table ("paged") variant of the same step.  The paper's prototype keeps
 * the KV cache in fixed-size blocks and ships it block by block (section 5.1,
 * "KV-cache transfer" implementation), which is also what lets a token machine
 * batch until its memory is nearly full (section 4.2) instead of reserving
 * max_len positions per request.  Same attention, different addressing:
 * positions [i*block_size, (i+1)*block_size) of request r live in pool block
 * block_table[r*max_blocks + i], and element (b, g, t, j) of a pool -- block
 * b, key/value head g, position t inside the block, dimension j -- is at
 *     base + b*stride_block + g*stride_kvh + t*stride_tok + j*stride_dim
 * with the strides sw_kv_paged_layout returns (in elements).
 */
typedef struct sw_kv_paged_layout_t {
    int32_t dtype;         /* SW_F16                                              */
    int32_t elem_bytes;    /* 2                                                   */
    int64_t stride_block;  /* elements between consecutive pool blocks            */
    int64_t stride_kvh;    /* elements between key/value heads inside a block     */
    int64_t stride_tok;    /* elements between positions inside a block (= head_dim) */
    int64_t stride_dim;    /* 1                                                   */
    int64_t total_elems;   /* elements to allocate for ONE pool (K or V)          */
    int32_t base_align;    /* required alignment of each pool's base, bytes       */
    int32_t block_size;    /* positions per block, as passed in                   */
} sw_kv_paged_layout_t;

/*
 * sw_kv_paged_layout -- layout query for block pools.  Pure host arithmetic.
 * block_size must be a power of two in [4, 4096].  Errors: SW_ERR_NULL (out),
 * SW_ERR_SHAPE (n_blocks/n_kvh <= 0), SW_ERR_UNSUPPORTED (head_dim, block_size).
 */
int sw_kv_paged_layout(int n_blocks, int n_kvh, int head_dim, int block_size,
                       sw_kv_paged_layout_t *out);

/*
 * sw_decode_attn_paged -- sw_decode_attn over block pools.
 *   q, seq_lens, out, n_req, n_qh, n_kvh, head_dim, stream: as in sw_decode_attn.
 *   k_pool, v_pool  DEVICE, binary16, laid out as sw_kv_paged_layout(n_blocks,
 *                   n_kvh, head_dim, block_size) says; separate buffers.  Read only.
 *   block_table     DEVICE, int32 [n_req][max_blocks].  Only the first
 *                   ceil(L_r / block_size) entries of row r are read; ids outside
 *                   [0, n_blocks-1] are clamped into that range on the device.
 *   block_size      positions per block: a power of two in [4, 4096].
 *   max_blocks      table entries per request; lengths are clamped to
 *                   [0, max_blocks*block_size], which must not exceed 2^23.
 *   n_blocks        blocks in each pool (> 0).
 * Asynchrony, workspace, ownership and errors as for sw_decode_attn; in
 * addition block_table must be non-NULL and 4-byte aligned.  For the same
 * cached values the result has the same bits as sw_decode_attn's.
 */
int sw_decode_attn_paged(const void *q, const void *k_pool, const void *v_pool,
                         const int32_t *block_table, const int32_t *seq_lens, void *out,
                         int n_req, int n_qh, int n_kvh, int head_dim,
                         int block_size, int max_blocks, int n_blocks, void *stream);

/*
 * Append-then-attend variants: one layer's attention inside a running decode
 * loop.  Every token-phase iteration takes the last generated token and the KV
 * cache as inputs (section 2.2, "token phase"): the token's own key and value
 * rows join the cache of every layer, and the token attends over the cache
 * including itself.  These calls do both in one pass over the cache, so a
 * model step is n_layers such calls (one per layer cache, all sharing one
 * seq_lens array) followed by one sw_advance_lens.
 *
 *   k_new, v_new   DEVICE, binary16, dense [n_req][n_kvh][head_dim]: the newest
 *                  token's K and V rows for this layer.  Read only, 16-byte aligned.
 *   k_cache, v_cache (k_pool, v_pool)  as in sw_decode_attn (_paged), but
 *                  WRITTEN: with L0 = clamp(seq_lens[r], 0, max_len) the number
 *                  of positions cached BEFORE this token, a request with
 *                  L0 < max_len gets k_new[r] / v_new[r] stored, bit for bit, at
 *                  position L0 of every key/value head and attends over
 *                  positions [0, L0]; a request whose cache is full (L0 ==
 *                  max_len) stores nothing and attends over the max_len cached
 *                  positions without the new token.  Nothing else in the
 *                  caches is written.
 *   block_table    (paged) the entry for position L0, i.e. entry
 *                  L0 / block_size of row r, must name the block the caller
 *                  has allotted to it; an id outside the pool is clamped into
 *                  it like any other.  Two requests must not share the block
 *                  either of them appends to.
 *   seq_lens       read only here; every layer of a step sees the same values.
 * Everything else (arguments, asynchrony, workspace, errors) as in
 * sw_decode_attn / sw_decode_attn_paged.  `out` has the bits sw_decode_attn
 * gives on the cache after the append with lengths L0 + 1 (L0 when full).
 */
int sw_decode_attn_append(const void *q, const void *k_new, const void *v_new,
                          void *k_cache, void *v_cache,
                          const int32_t *seq_lens, void *out,
                          int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                          void *stream);
int sw_decode_attn_paged_append(const void *q, const void *k_new, const void *v_new,
                                void *k_pool, void *v_pool,
                                const int32_t *block_table, const int32_t *seq_lens, void *out,
                                int n_req, int n_qh, int n_kvh, int head_dim,
                                int block_size, int max_blocks, int n_blocks, void *stream);

/*
 * sw_advance_lens -- end of a model step: seq_lens[r] = min(clamp(seq_lens[r],
 * 0, max_len) + 1, max_len) for every request, on the device, enqueued on
 * `stream` after the step's layer calls.  seq_lens: DEVICE, int32 [n_req],
 * 4-byte aligned.  Errors: SW_ERR_NULL, SW_ERR_SHAPE (n_req < 0, max_len <= 0),
 * SW_ERR_ALIGN, SW_ERR_HIP.  n_req == 0 returns SW_OK.
 */
int sw_advance_lens(int32_t *seq_lens, int n_req, int max_len, void *stream);

/*
 * sw_prefill_attn -- the prompt phase's attention (section 2.2: all tokens of a
 * prompt are processed in one pass, which produces the KV cache; section 3.5,
 * Insight V: this phase is compute bound).  Prompt token i of request r attends
 * to cached positions 0..i of that request:
 *     out[s_r + i, h, :] = softmax_{t <= i}( q[s_r + i, h, :] . K[r, g, t, :] / sqrt(head_dim) ) . V[r, g, 0..i, :]
 * for i < L_r = clamp(seq_lens[r], 0, max_len), s_r = q_starts[r], g = h / (n_qh / n_kvh).
 *   q, out     DEVICE, binary16, [n_tokens][n_qh][head_dim]; 16-byte aligned.  Rows of
 *              `out` that belong to no prompt token are not written.
 *   k_cache, v_cache   as in sw_decode_attn: the prompt's K/V rows are already in place
 *              (positions 0 .. L_r - 1); read only.
 *   seq_lens   DEVICE int32 [n_req]: prompt lengths, clamped to [0, max_len].
 *   q_starts   DEVICE int32 [n_req]: row of each request's first prompt token.  Rows
 *              s_r .. s_r + L_r - 1 must lie in [0, n_tokens) and the requests' row
 *              ranges must not overlap; row indices outside [0, n_tokens) are never
 *              dereferenced (such rows are skipped).
 *   n_tokens   rows of q and out (0 returns SW_OK without touching the device).
 *   head_dim must be 128 (SW_ERR_UNSUPPORTED otherwise); n_qh / n_kvh at most 64.
 * One kernel, no workspace; asynchrony, ownership and the other errors as in
 * sw_decode_attn.  Which of the library's two prompt kernels runs depends on the call's
 * size (n_tokens, n_req, the head counts); they sum in different orders, so a prompt's
 * result may differ in the last bits between a small and a large batch.  Under either
 * kernel it does not depend on the other requests of the batch.  The launch is sized by the smaller of n_req * max_len and about
 * n_tokens + 64 * n_req query tokens, so a batch of a few long and many short prompts
 * costs what its tokens cost.  Weights enter the second matrix product rounded to binary16 (the
 * normaliser sums them in binary32 before that rounding); results differ from the fp64
 * definition by about 1e-3 absolute at most for values of order one.
 */
int sw_prefill_attn(const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *seq_lens, const int32_t *q_starts, void *out, long long n_tokens,
                    int n_req, int n_qh, int n_kvh, int head_dim, int max_len, void *stream);

/*
 * sw_mixed_attn -- attention of a mixed batch (section 2.4, "mixed batching": the
 * scheduler runs prompt and token phases together in one forward pass; the paper's
 * baseline and the mixed pool of section 4.1 work this way).  Request r contributes
 * its LAST nq_r cached tokens as queries, nq_r = clamp(q_lens[r], 0, min(L_r,
 * max_q_len)); query i (row q_starts[r] + i of q and out) is the token at position
 * L_r - nq_r + i and attends to positions 0 .. L_r - nq_r + i.  nq_r = L_r is a whole
 * prompt (sw_prefill_attn is this call with q_lens = all of them), nq_r = 1 a request in
 * its token phase, values between a prompt processed in pieces.  The K/V rows of the
 * query tokens are already in the cache, as in sw_prefill_attn.
 *   q_lens      DEVICE int32 [n_req], 4-byte aligned.
 *   max_q_len   bound on nq_r known to the host (> 0; values above max_len mean
 *               max_len).
 * Everything else as in sw_prefill_attn, including the rule that the requests' row
 * ranges must not overlap (the launch is sized by n_tokens and n_req on that
 * assumption; overlapping ranges leave rows of out undefined, nothing out of bounds).
 * Two families of kernels serve the call, enqueued one after the other: requests with
 * nq_r == 1 (token phase: memory bound) go through sw_decode_attn's kernels, reading
 * and writing row q_starts[r] -- their results are bit for bit those of sw_decode_attn
 * for the same max_len -- and the others through the prompt kernels.  Which family
 * serves a request depends on that request alone.  A request with nq_r == 1 whose row
 * lies outside [0, n_tokens) is skipped.  Uses sw_decode_attn's workspace.
 */
int sw_mixed_attn(const void *q, const void *k_cache, const void *v_cache,
                  const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                  void *out, long long n_tokens,
                  int n_req, int n_qh, int n_kvh, int head_dim, int max_len, int max_q_len,
                  void *stream);

/*
 * sw_prefill_attn_paged, sw_mixed_attn_paged -- the two calls above over block pools
 * (the layout of sw_decode_attn_paged: position t of request r is row t % block_size
 * of pool block block_table[r * max_blocks + t / block_size]; the paper's prototype
 * keeps the cache in such blocks, section 5.1).  max_len is max_blocks * block_size;
 * lengths clamp to it, block ids to [0, n_blocks - 1]; table entries past a request's
 * last block are never followed.  block_size: a power of two in [4, 4096]
 * (SW_ERR_UNSUPPORTED); max_blocks * block_size at most 2^23 (SW_ERR_SHAPE).
 * Token-phase requests of a mixed batch give the bits of sw_decode_attn_paged.
 * Everything else as in sw_prefill_attn / sw_mixed_attn.
 */
int sw_prefill_attn_paged(const void *q, const void *k_pool, const void *v_pool,
                          const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_starts,
                          void *out, long long n_tokens, int n_req, int n_qh, int n_kvh, int head_dim,
                          int block_size, int max_blocks, int n_blocks, void *stream);
int sw_mixed_attn_paged(const void *q, const void *k_pool, const void *v_pool,
                        const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_starts,
                        const int32_t *q_lens, void *out, long long n_tokens,
                        int n_req, int n_qh, int n_kvh, int head_dim,
                        int block_size, int max_blocks, int n_blocks, int max_q_len, void *stream);

/*
 * sw_kv_store, sw_kv_store_paged -- the cache side of a prompt or mixed pass (section
 * 2.2: the prompt phase processes all prompt tokens in one pass, which produces the KV
 * cache).  The pass has computed one K row and one V row per new token and key/value
 * head; this call puts them where they belong, after which sw_prefill_attn /
 * sw_mixed_attn (same seq_lens, q_starts, q_lens) attend over them.  With L_r =
 * clamp(seq_lens[r], 0, max_len) cached positions INCLUDING the new tokens and nq_r =
 * clamp(q_lens[r], 0, min(L_r, max_q_len)) of them new (q_lens == NULL: all L_r, a whole
 * prompt), rows k_rows[q_starts[r] + i, g, :] and v_rows[...] go, bit for bit, to
 * position L_r - nq_r + i of head g of request r, for i < nq_r.  Nothing else is written.
 *   k_rows, v_rows   DEVICE, binary16, [n_tokens][n_kvh][head_dim], 16-byte aligned; rows
 *                    outside [0, n_tokens) do not exist and are skipped; the requests'
 *                    row ranges must not overlap (as in sw_mixed_attn).
 *   k_cache, v_cache the dense caches of sw_kv_layout (sw_kv_store) or the block pools of
 *                    sw_kv_paged_layout with their table (sw_kv_store_paged, where max_len is
 *                    max_blocks * block_size); written.
 *   head_dim 64 or 128; n_kvh at most 65535.  n_req == 0 or n_tokens == 0 returns SW_OK.
 * One kernel, no workspace; asynchrony, ownership and the other errors as in sw_mixed_attn.
 */
int sw_kv_store(const void *k_rows, const void *v_rows, void *k_cache, void *v_cache,
                const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                long long n_tokens, int n_req, int n_kvh, int head_dim, int max_len, int max_q_len,
                void *stream);
int sw_kv_store_paged(const void *k_rows, const void *v_rows, void *k_pool, void *v_pool,
                      const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_starts,
                      const int32_t *q_lens, long long n_tokens, int n_req, int n_kvh, int head_dim,
                      int block_size, int max_blocks, int n_blocks, int max_q_len, void *stream);

/*
 * KV-cache hand-off, the part inside one GPU's memory.  A prompt machine ships
 * each layer's KV cache to a token machine block by block, merging blocks that
 * are contiguous so that fewer transfers are issued (section 4.3, "KV-cache
 * transfer"; section 5.1).  The transfer itself is outside this library.
 *
 * sw_kv_pack -- copies positions [0, L_r) of every request and key/value head
 * from block pools (sw_kv_paged_layout) into dense caches (sw_kv_layout(n_req,
 * n_kvh, head_dim, max_len)), where every (request, head) is one contiguous run
 * ready to be sent or attended over; sw_kv_unpack is the reverse (dense -> the
 * blocks the table names).  L_r = clamp(seq_lens[r], 0, min(max_len,
 * max_blocks*block_size)).  Rows are copied bit for bit; nothing else in the
 * destination is written.  All pointers DEVICE; pools and caches 16-byte
 * aligned, int32 arrays 4-byte aligned; block ids clamped into the pool.
 * Errors and asynchrony as in sw_decode_attn_paged (no workspace).
 *
 * sw_kv_span_plan -- the transfers one layer needs when runs of consecutive
 * pool block ids go out as one span.  For request r with nb = ceil(L_r /
 * block_size) blocks in use (L_r clamped to max_blocks*block_size), entry i of
 * its table row starts a span when i == 0 or id[i] != id[i-1] + 1.  Outputs
 * (DEVICE int32): n_spans[r]; span_first[r*max_blocks + k] = pool id of span
 * k's first block; span_blocks[r*max_blocks + k] = its length in blocks, for
 * k < n_spans[r]; later entries are not written.
 */
int sw_kv_pack(const void *k_pool, const void *v_pool, const int32_t *block_table,
               const int32_t *seq_lens, void *k_dense, void *v_dense,
               int n_req, int n_kvh, int head_dim, int max_len,
               int block_size, int max_blocks, int n_blocks, void *stream);
int sw_kv_unpack(const void *k_dense, const void *v_dense, const int32_t *block_table,
                 const int32_t *seq_lens, void *k_pool, void *v_pool,
                 int n_req, int n_kvh, int head_dim, int max_len,
                 int block_size, int max_blocks, int n_blocks, void *stream);
int sw_kv_span_plan(const int32_t *block_table, const int32_t *seq_lens,
                    int32_t *span_first, int32_t *span_blocks, int32_t *n_spans,
                    int n_req, int block_size, int max_blocks, int n_blocks, void *stream);

/*
 * sw_last_error -- text of the calling thread's most recent failure
 * (a static or thread-local string; never NULL; valid until the thread's next
 * failing call).  Support call, not part of the step.
 */
const char *sw_last_error(void);

/* sw_version -- library version as major*10000 + minor*100 + patch. */
int sw_version(void);

/*
 * sw_release -- frees every workspace the library holds (after synchronising
 * the devices they live on).  Optional; the caller must make sure that no
 * call is in flight.  Support call, not part of the step.
 */
int sw_release(void);

/*
 * sw_decode_attn_static -- sw_decode_attn for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * Same arguments, same result up to the rounding of the merge (it is the two-kernel form,
 * SW_PARAM_COMBINE = 1, bit for bit), but the partial results between its two kernels live
 * in a static device array of SW_STATIC_SCRATCH_BYTES inside the library instead of the
 * per-stream workspace: the call allocates and frees nothing, on the device or through any
 * library.  A shape whose partial results, n_req * n_qh * ceil(max_len / chunk) *
 * (head_dim + 2) * 4 bytes (chunk: SW_PARAM_CHUNK, by default 256 doubled until 16 chunks
 * cover max_len, at most 1024), exceed that size is refused with SW_ERR_UNSUPPORTED
 * before anything is launched.
 * Every GPU the library runs on holds its own copy of the array until the process ends.  All
 * calls on one GPU share it, whatever their stream: calls that overlap on one GPU race, so
 * order them (one stream, or events).  Nothing in it needs clearing between calls: a call
 * reads back only what it has written itself.  Not recorded by sw_prof_start/stop.
 */
#define SW_STATIC_SCRATCH_BYTES (32u << 20)
int sw_decode_attn_static(const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *seq_lens, void *out,
                          int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                          void *stream);

/*
 * sw_device_status -- support: waits for the current device to go idle and reports
 * whether any single-launch merge on it ever gave up waiting for another workgroup's
 * partial result (the wait inside the kernel is bounded so that a kernel always ends; a
 * give-up leaves the affected output rows wrong and sets a flag in the workspace).
 *   gave_up   HOST, written: 0 = never, 1 = at least once since the workspace was allocated.
 * Returns SW_OK, SW_ERR_NULL or SW_ERR_HIP.  Not part of a step; synchronises.
 */
int sw_device_status(int *gave_up);

/*
 * Tuning and test knobs (support calls, not part of the step).  They change
 * how the step is scheduled, never what it computes.  Process-wide; set them
 * while no call is in flight.
 *   SW_PARAM_CHUNK     context positions per workgroup of the partial kernel
 *                      (split over context length); 0 = library default;
 *                      otherwise a power of two in [64, 65536].
 *   SW_PARAM_KERNEL    0 = library default choice, 1 = force the vector-ALU
 *                      kernel, 2 = force the matrix-core (MFMA) kernel
 *                      (SW_ERR_UNSUPPORTED at call time if the shape has no such
 *                      kernel: it needs head_dim 128).
 *   SW_PARAM_COMBINE   how the chunks of a request are merged: 0 = library default
 *                      (the same launch where no request can have more than four
 *                      chunks, i.e. max_len <= 4 * chunk; a second kernel otherwise),
 *                      1 = a second (combine) kernel, 2 = in the same launch, by
 *                      one of the workgroups of the request's head group
 *                      (SW_ERR_UNSUPPORTED at call time above 4 GiB).
 *                      Each is deterministic; the two differ by rounding only.
 *   SW_PARAM_WAVES     waves per workgroup of the matrix-core partial kernel:
 *                      0 = library default (4), else 4 or 8.
 *   SW_PARAM_PREFILL_HEADS  prompt-phase kernel: query heads of a group that share a
 *                      workgroup (0 = library default; a value that does not divide
 *                      the group size is ignored).
 *   SW_PARAM_PREFILL_WAVES  prompt-phase kernel: waves (32 query positions each) per
 *                      head in a workgroup (0 = library default; ignored if heads *
 *                      waves would exceed 8).  For the key-split kernel: waves per
 *                      workgroup, 2, 4 or 8.
 *   SW_PARAM_PREFILL_KERNEL  0 = library default, 1 = the kernel that shares staged
 *                      K/V tiles among the waves of a workgroup (up to 8 heads of a group),
 *                      2 = the kernel that splits a query block's key range over the
 *                      waves of a workgroup.  The two differ by rounding only.
 *   SW_PARAM_MIXED_MERGE  mixed batches: where the chunks of the token-phase requests are
 *                      merged: 0 = library default, 1 = in a combine kernel of its own,
 *                      2 = by extra workgroups of the prompt kernel (one launch fewer;
 *                      only with the four-wave key-split prompt kernel).  Same bits.
 */
#define SW_PARAM_CHUNK   1
#define SW_PARAM_KERNEL  2
#define SW_PARAM_COMBINE 3
#define SW_PARAM_WAVES   4
#define SW_PARAM_PREFILL_HEADS 5
#define SW_PARAM_PREFILL_WAVES 6
#define SW_PARAM_PREFILL_KERNEL 7
#define SW_PARAM_MIXED_MERGE 8
int sw_set_param(int key, int value);
int sw_get_param(int key, int *value);

/*
 * Per-kernel timing for measurement (support calls, not part of the step).
 * Between sw_prof_start and sw_prof_stop every sw_decode_attn call attaches a
 * pair of HIP events to each kernel it launches (on the call's stream), for
 * up to `capacity` calls; further calls run untimed.  sw_prof_stop waits for
 * the recorded events and reports, in microseconds summed over the recorded
 * calls, the device time of the partial kernel and of the combine kernel
 * (0 when the chunks are merged in the same launch),
 * and how many calls were recorded.  Pointers are host memory.
 */
int sw_prof_start(int capacity);
int sw_prof_stop(double *partial_us_sum, double *combine_us_sum, int *n_calls);
/*
 * The time between the partial kernel's end event and the combine kernel's start
 * event, in microseconds summed over the calls the last sw_prof_stop reported (0
 * where no combine kernel ran; negative where the two overlapped).  Host pointer.
 */
int sw_prof_last_gap(double *gap_us_sum);

/*
 * sw_stream_read -- measurement support: one kernel that reads n_bytes of device
 * memory once and does nothing else worth mentioning, the practical ceiling to hold the
 * token-phase call against (that phase is bound by reading the KV cache, section 3.5,
 * Insight V).  Workgroup b XORs the 32-bit words it reads (a grid-stride walk, 16
 * bytes per lane) and stores the result in sink[b]; the XOR of sink[0 .. workgroups)
 * is the XOR of all words of src, which is what the test checks.
 *   src         DEVICE, 16-byte aligned, n_bytes a multiple of 16 (SW_ERR_ALIGN / SW_ERR_SHAPE).
 *   sink        DEVICE, uint32 [workgroups], 4-byte aligned, written.
 *   workgroups  1 .. 65536 workgroups of 256 threads; 0 = the library's choice (2048 below
 *               128 MB, 16384 from there), in which case sink needs 16384 entries.
 * Enqueues on `stream` and returns; recorded by sw_prof_start/stop as a "partial" time.
 */
int sw_stream_read(const void *src, long long n_bytes, void *sink, int workgroups, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SW_DECODE_H */
