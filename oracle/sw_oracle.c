/*
 * sw_oracle.c -- CPU reference ("oracle") for one decode-attention step.
 *
 * THIS FILE IS TEST INFRASTRUCTURE. It is a plain, slow, fp64 implementation
 * used only to check the GPU library and to time a CPU baseline next to it.
 * The GPU library never calls, links or includes anything from this directory,
 * and nothing here includes anything of the GPU library.
 *
 * What it computes.  The paper (section 2.2, "Generative LLM inference
 * phases") states the token-generation step: the forward pass of a request's
 * newest token takes that token and the request's whole KV cache as inputs,
 * and (section 3.5, "Memory utilization") every active token reads the cache
 * of its entire context.  The attention it refers to (section 2.1, by
 * citation) is scaled dot-product attention, so for every request r and
 * query head h, with g = h / (n_qh / n_kvh) the key/value head that serves h,
 * and L = clamp(seq_lens[r], 0, max_len):
 *
 *     s_t   = (sum_j q[r,h,j] * K[r,g,t,j]) / sqrt(head_dim),   t = 0..L-1
 *     m     = max_t s_t
 *     p_t   = exp(s_t - m)
 *     l     = sum_t p_t
 *     ref_j = (sum_t p_t * V[r,g,t,j]) / l
 *
 * and ref = 0 when L = 0.  It is the definition written out: two passes, no
 * running maximum, no chunking, no blocking.  Inputs are IEEE binary16 bit
 * patterns, widened exactly to double by the decoder below; everything after
 * that is double.  Each (r, h) unit is computed sequentially by one thread, so
 * the result does not depend on the thread count.
 *
 * sw_oracle_decode_attn_paged is the same step over a block-table cache
 * (pinned against the dense routine: identity and shuffled block tables must
 * give bit-equal results).  Further down: the cache side of an iteration
 * (sw_oracle_kv_append), the prompt phase and mixed batches (sw_oracle_mixed_attn,
 * of which sw_oracle_prefill_attn is the all-tokens case; _paged over block
 * pools), the cache side of such a pass (sw_oracle_kv_store) and the in-GPU part
 * of the KV hand-off (sw_oracle_kv_pack, sw_oracle_kv_span_plan); each states its
 * own definition and pins in the comment above it.
 *
 * Pins: closed forms (one token, identical keys, a dominant key), brute force
 * against a dense matrix formulation, shift / permutation invariance,
 * convexity, the chunk-merge identity, GQA-as-replicated-MHA and a one-hot-V
 * comparison against a library softmax (tests/test_oracle_pins.py).
 * The paper prints no worked numerical example of this step, so parity with
 * the paper's own numbers is unpinned; parity is against the definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Exact widening of an IEEE 754 binary16 bit pattern to double.
 * sign 1 bit, exponent 5 bits (bias 15), fraction 10 bits. */
static double half_bits_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int expo = (b >> 10) & 0x1f;
    int frac = b & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* Exposed so that the tests can pin the decoder against numpy's float16. */
double sw_oracle_half_to_double(uint16_t bits) { return half_bits_to_double(bits); }

static int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

/*
 * One (request, query head) unit.  kg / vg point at token 0 of the serving
 * key/value head; consecutive tokens are stride_tok elements apart.
 * scores is scratch of at least L doubles.
 */
static void attend_one(const uint16_t *qrow, const uint16_t *kg, const uint16_t *vg,
                       int L, int d, int64_t stride_tok, double *scores,
                       double *ref, double *m_out, double *l_out)
{
    if (L <= 0) {
        for (int j = 0; j < d; ++j) ref[j] = 0.0;
        if (m_out) *m_out = -INFINITY;
        if (l_out) *l_out = 0.0;
        return;
    }
    const double scale = 1.0 / sqrt((double)d);
    double m = -INFINITY;
    for (int t = 0; t < L; ++t) {
        const uint16_t *krow = kg + (int64_t)t * stride_tok;
        double acc = 0.0;
        for (int j = 0; j < d; ++j)
            acc += half_bits_to_double(qrow[j]) * half_bits_to_double(krow[j]);
        scores[t] = acc * scale;
        if (scores[t] > m) m = scores[t];
    }
    double l = 0.0;
    for (int t = 0; t < L; ++t) {
        scores[t] = exp(scores[t] - m);
        l += scores[t];
    }
    for (int j = 0; j < d; ++j) {
        double acc = 0.0;
        for (int t = 0; t < L; ++t)
            acc += scores[t] * half_bits_to_double(vg[(int64_t)t * stride_tok + j]);
        ref[j] = acc / l;
    }
    if (m_out) *m_out = m;
    if (l_out) *l_out = l;
}

/*
 * Whole batch.  All pointers are host memory.
 *   q        binary16 bits, dense [n_req][n_qh][head_dim]
 *   k, v     binary16 bits; element (r, g, t, j) is at
 *            r*stride_req + g*stride_kvh + t*stride_tok + j
 *   seq_lens int32 [n_req]; values outside [0, max_len] are clamped
 *   ref      double, dense [n_req][n_qh][head_dim]   (not rounded to binary16)
 *   m_out, l_out   optional (may be NULL) double [n_req][n_qh]: the score
 *            maximum and the sum of exp(s - m); used by the chunk-merge pin
 *   n_threads  <= 0 means "all the runtime offers"
 * Returns the number of threads used (>= 1), or a negative value on a bad
 * argument.
 */
int sw_oracle_decode_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                          const int32_t *seq_lens, double *ref,
                          double *m_out, double *l_out,
                          int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                          int64_t stride_req, int64_t stride_kvh, int64_t stride_tok,
                          int n_threads)
{
    if (n_req < 0 || n_qh <= 0 || n_kvh <= 0 || head_dim <= 0 || max_len <= 0) return -1;
    if (n_qh % n_kvh != 0) return -2;
    if (n_req == 0) return 1;
    if (!q || !k || !v || !seq_lens || !ref) return -3;

    const int group = n_qh / n_kvh;
    const int64_t units = (int64_t)n_req * n_qh;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    if ((int64_t)n_threads > units) n_threads = (int)units;
    used = n_threads;
#else
    (void)n_threads;
#endif
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads)
#endif
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_len);
        if (!scores) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t u = 0; u < units; ++u) {
            if (!scores) continue;
            int r = (int)(u / n_qh);
            int h = (int)(u % n_qh);
            int g = h / group;
            int L = clampi(seq_lens[r], 0, max_len);
            const uint16_t *qrow = q + ((int64_t)r * n_qh + h) * head_dim;
            const uint16_t *kg = k + (int64_t)r * stride_req + (int64_t)g * stride_kvh;
            const uint16_t *vg = v + (int64_t)r * stride_req + (int64_t)g * stride_kvh;
            attend_one(qrow, kg, vg, L, head_dim, stride_tok, scores,
                       ref + u * head_dim,
                       m_out ? m_out + u : NULL, l_out ? l_out + u : NULL);
        }
        free(scores);
    }
    return failed ? -4 : used;
}

/*
 * Block-table ("paged") variant.  The paper's prototype keeps the KV cache in
 * fixed-size blocks (section 5.1: the cache is shipped block by block); the
 * step is the same attention, only the addressing differs: positions
 * [i*block_size, (i+1)*block_size) of request r live in pool block
 * block_table[r*max_blocks + i], and element (b, g, t, j) of a pool -- block
 * b, key/value head g, position t inside the block, dimension j -- is at
 *     b*stride_block + g*stride_kvh + t*stride_tok + j.
 * Lengths are clamped to [0, max_blocks*block_size]; block ids are clamped to
 * [0, n_blocks-1].  Each (request, head) unit gathers its rows into a dense
 * temporary and runs the same two-pass routine as above.
 */
int sw_oracle_decode_attn_paged(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                                const int32_t *block_table, const int32_t *seq_lens, double *ref,
                                int n_req, int n_qh, int n_kvh, int head_dim,
                                int block_size, int max_blocks, int n_blocks,
                                int64_t stride_block, int64_t stride_kvh, int64_t stride_tok,
                                int n_threads)
{
    if (n_req < 0 || n_qh <= 0 || n_kvh <= 0 || head_dim <= 0 || block_size <= 0 ||
        max_blocks <= 0 || n_blocks <= 0) return -1;
    if (n_qh % n_kvh != 0) return -2;
    if (n_req == 0) return 1;
    if (!q || !k_pool || !v_pool || !block_table || !seq_lens || !ref) return -3;

    const int group = n_qh / n_kvh;
    const int64_t max_len = (int64_t)max_blocks * block_size;
    const int64_t units = (int64_t)n_req * n_qh;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    if ((int64_t)n_threads > units) n_threads = (int)units;
    used = n_threads;
#else
    (void)n_threads;
#endif
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads)
#endif
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_len);
        uint16_t *kd = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)max_len * (size_t)head_dim);
        uint16_t *vd = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)max_len * (size_t)head_dim);
        if (!scores || !kd || !vd) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int64_t u = 0; u < units; ++u) {
            if (!scores || !kd || !vd) continue;
            int r = (int)(u / n_qh);
            int h = (int)(u % n_qh);
            int g = h / group;
            int64_t L64 = seq_lens[r];
            int L = (int)(L64 < 0 ? 0 : (L64 > max_len ? max_len : L64));
            for (int t = 0; t < L; ++t) {
                int b = clampi(block_table[(int64_t)r * max_blocks + t / block_size], 0, n_blocks - 1);
                int64_t off = (int64_t)b * stride_block + (int64_t)g * stride_kvh +
                              (int64_t)(t % block_size) * stride_tok;
                memcpy(kd + (size_t)t * head_dim, k_pool + off, sizeof(uint16_t) * (size_t)head_dim);
                memcpy(vd + (size_t)t * head_dim, v_pool + off, sizeof(uint16_t) * (size_t)head_dim);
            }
            attend_one(q + ((int64_t)r * n_qh + h) * head_dim, kd, vd, L, head_dim, head_dim, scores,
                       ref + u * head_dim, NULL, NULL);
        }
        free(scores);
        free(kd);
        free(vd);
    }
    return failed ? -4 : used;
}

/*
 * The cache side of one token-phase iteration (section 2.2: each iteration's
 * inputs are the last generated token and the KV cache, so that token's key and
 * value rows join the cache before it attends).  For every request r with
 * L0 = clamp(seq_lens[r], 0, max_len) < max_len, rows k_new[r, g, :] and
 * v_new[r, g, :] are copied, bit for bit, to position L0 of every key/value
 * head g, and lens_out[r] = L0 + 1; a request whose cache is full keeps its
 * cache and gets lens_out[r] = max_len.  k_new, v_new: dense
 * [n_req][n_kvh][head_dim].  A step of the append-then-attend variant is this
 * routine followed by sw_oracle_decode_attn with lens_out.
 * Pinned by brute force against array slicing (tests/test_oracle_pins.py).
 */
int sw_oracle_kv_append(const uint16_t *k_new, const uint16_t *v_new, uint16_t *k, uint16_t *v,
                        const int32_t *seq_lens, int32_t *lens_out,
                        int n_req, int n_kvh, int head_dim, int max_len,
                        int64_t stride_req, int64_t stride_kvh, int64_t stride_tok)
{
    if (n_req < 0 || n_kvh <= 0 || head_dim <= 0 || max_len <= 0) return -1;
    if (n_req == 0) return 0;
    if (!k_new || !v_new || !k || !v || !seq_lens || !lens_out) return -3;
    for (int r = 0; r < n_req; ++r) {
        int L0 = clampi(seq_lens[r], 0, max_len);
        if (L0 == max_len) {
            lens_out[r] = max_len;
            continue;
        }
        for (int g = 0; g < n_kvh; ++g) {
            int64_t dst = (int64_t)r * stride_req + (int64_t)g * stride_kvh + (int64_t)L0 * stride_tok;
            int64_t src = ((int64_t)r * n_kvh + g) * head_dim;
            for (int j = 0; j < head_dim; ++j) {
                k[dst + j] = k_new[src + j];
                v[dst + j] = v_new[src + j];
            }
        }
        lens_out[r] = L0 + 1;
    }
    return 0;
}

/* The same over block pools: position L0 of request r is row L0 % block_size of
 * pool block clamp(block_table[r*max_blocks + L0 / block_size], 0, n_blocks-1). */
int sw_oracle_kv_append_paged(const uint16_t *k_new, const uint16_t *v_new,
                              uint16_t *k_pool, uint16_t *v_pool,
                              const int32_t *block_table, const int32_t *seq_lens, int32_t *lens_out,
                              int n_req, int n_kvh, int head_dim,
                              int block_size, int max_blocks, int n_blocks,
                              int64_t stride_block, int64_t stride_kvh, int64_t stride_tok)
{
    if (n_req < 0 || n_kvh <= 0 || head_dim <= 0 || block_size <= 0 || max_blocks <= 0 ||
        n_blocks <= 0) return -1;
    if (n_req == 0) return 0;
    if (!k_new || !v_new || !k_pool || !v_pool || !block_table || !seq_lens || !lens_out) return -3;
    const int64_t max_len = (int64_t)max_blocks * block_size;
    for (int r = 0; r < n_req; ++r) {
        int64_t L0 = seq_lens[r];
        L0 = L0 < 0 ? 0 : (L0 > max_len ? max_len : L0);
        if (L0 == max_len) {
            lens_out[r] = (int32_t)max_len;
            continue;
        }
        int b = clampi(block_table[(int64_t)r * max_blocks + L0 / block_size], 0, n_blocks - 1);
        for (int g = 0; g < n_kvh; ++g) {
            int64_t dst = (int64_t)b * stride_block + (int64_t)g * stride_kvh +
                          (L0 % block_size) * stride_tok;
            int64_t src = ((int64_t)r * n_kvh + g) * head_dim;
            for (int j = 0; j < head_dim; ++j) {
                k_pool[dst + j] = k_new[src + j];
                v_pool[dst + j] = v_new[src + j];
            }
        }
        lens_out[r] = (int32_t)(L0 + 1);
    }
    return 0;
}

/*
 * Mixed batch (section 2.4, "mixed batching": prompt and token phases run together in
 * one forward pass): request r contributes its LAST nq_r tokens as queries,
 * nq_r = clamp(q_lens[r], 0, min(L_r, max_q_len)); query i is the token at position
 * L_r - nq_r + i and sees cached positions 0 .. L_r - nq_r + i.  nq_r = L_r is a whole
 * prompt, nq_r = 1 a token-phase request, anything between a prompt processed in pieces.
 * q_lens == NULL means nq_r = L_r for every request (the prompt phase,
 * sw_oracle_prefill_attn below).
 * Still one attend_one per (request, head, query token).
 * Pins: nq = L is the prompt routine; nq = 1 is sw_oracle_decode_attn; a prompt in two
 * pieces gives the rows of the prompt in one piece, bit for bit (tests/test_oracle_pins.py).
 */
int sw_oracle_mixed_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                         const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                         double *ref,
                         int n_req, int n_qh, int n_kvh, int head_dim, int max_len, int max_q_len,
                         int64_t n_tokens,
                         int64_t stride_req, int64_t stride_kvh, int64_t stride_tok,
                         int n_threads)
{
    if (n_req < 0 || n_qh <= 0 || n_kvh <= 0 || head_dim <= 0 || max_len <= 0 || max_q_len <= 0 ||
        n_tokens < 0) return -1;
    if (n_qh % n_kvh != 0) return -2;
    if (n_req == 0) return 1;
    if (!q || !k || !v || !seq_lens || !q_starts || !ref) return -3;
    for (int r = 0; r < n_req; ++r) {
        int L = clampi(seq_lens[r], 0, max_len);
        int nq = q_lens ? clampi(q_lens[r], 0, L < max_q_len ? L : max_q_len) : L;
        if (nq > 0 && (q_starts[r] < 0 || (int64_t)q_starts[r] + nq > n_tokens)) return -5;
    }
    const int group = n_qh / n_kvh;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads;
#else
    (void)n_threads;
#endif
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads)
#endif
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_len);
        if (!scores) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
        for (int r = 0; r < n_req; ++r) {
            int L = clampi(seq_lens[r], 0, max_len);
            int nq = q_lens ? clampi(q_lens[r], 0, L < max_q_len ? L : max_q_len) : L;
            int p0 = L - nq;                                 /* position of the first query token */
            for (int h = 0; h < n_qh; ++h) {
                int g = h / group;
                const uint16_t *kg = k + (int64_t)r * stride_req + (int64_t)g * stride_kvh;
                const uint16_t *vg = v + (int64_t)r * stride_req + (int64_t)g * stride_kvh;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 4) nowait
#endif
                for (int i = 0; i < nq; ++i) {
                    if (!scores) continue;
                    int64_t row = ((int64_t)q_starts[r] + i) * n_qh + h;
                    attend_one(q + row * head_dim, kg, vg, p0 + i + 1, head_dim, stride_tok, scores,
                               ref + row * head_dim, NULL, NULL);
                }
            }
        }
        free(scores);
    }
    return failed ? -4 : used;
}

/*
 * Prompt phase (section 2.2: all tokens of the prompt are processed in parallel
 * in one forward pass, which also produces the KV cache; section 3.5, Insight V:
 * this phase is compute bound).  Its attention is the causal form of the same
 * definition: prompt token i of request r sees cached positions 0..i, so row i is
 * exactly the token-phase routine run with length i + 1.  It is written that way:
 * the mixed routine above with every cached token a query, i.e. one attend_one per
 * (request, head, token).
 *   q         binary16 bits, [n_tokens][n_qh][head_dim]; token i of request r is
 *             row q_starts[r] + i
 *   q_starts  int32 [n_req]; rows q_starts[r] .. q_starts[r] + L_r - 1 must lie in
 *             [0, n_tokens) (checked: a request that would leave it returns -5)
 *   ref       double [n_tokens][n_qh][head_dim]; rows of no request are left as
 *             they were
 * Everything else as in sw_oracle_decode_attn.
 * Pins: row i equals sw_oracle_decode_attn at length i + 1; brute force against a
 * masked dense matrix formulation; rows do not depend on later positions
 * (tests/test_oracle_pins.py).
 */
int sw_oracle_prefill_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                           const int32_t *seq_lens, const int32_t *q_starts, double *ref,
                           int n_req, int n_qh, int n_kvh, int head_dim, int max_len, int64_t n_tokens,
                           int64_t stride_req, int64_t stride_kvh, int64_t stride_tok,
                           int n_threads)
{
    return sw_oracle_mixed_attn(q, k, v, seq_lens, q_starts, NULL, ref, n_req, n_qh, n_kvh, head_dim,
                                max_len, max_len, n_tokens, stride_req, stride_kvh, stride_tok,
                                n_threads);
}

/*
 * Mixed-batch attention over a block-table cache: sw_oracle_mixed_attn with the
 * addressing of sw_oracle_decode_attn_paged (positions [i*block_size, (i+1)*block_size)
 * of request r live in pool block block_table[r*max_blocks + i]; lengths clamp to
 * [0, max_blocks*block_size], block ids to [0, n_blocks-1]).  q_lens == NULL makes
 * every cached token a query (the prompt phase).  Each (request, key/value head)
 * gathers its rows into a dense temporary and the rows of its queries go through the
 * same two-pass routine.  Pinned: equal, bit for bit, to sw_oracle_mixed_attn on the
 * dense cache of the same batch (tests/test_oracle_pins.py).
 */
int sw_oracle_mixed_attn_paged(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                               const int32_t *block_table, const int32_t *seq_lens,
                               const int32_t *q_starts, const int32_t *q_lens, double *ref,
                               int n_req, int n_qh, int n_kvh, int head_dim,
                               int block_size, int max_blocks, int n_blocks, int max_q_len,
                               int64_t n_tokens,
                               int64_t stride_block, int64_t stride_kvh, int64_t stride_tok,
                               int n_threads)
{
    if (n_req < 0 || n_qh <= 0 || n_kvh <= 0 || head_dim <= 0 || block_size <= 0 ||
        max_blocks <= 0 || n_blocks <= 0 || max_q_len <= 0 || n_tokens < 0) return -1;
    if (n_qh % n_kvh != 0) return -2;
    if (n_req == 0) return 1;
    if (!q || !k_pool || !v_pool || !block_table || !seq_lens || !q_starts || !ref) return -3;
    const int64_t max_len = (int64_t)max_blocks * block_size;
    for (int r = 0; r < n_req; ++r) {
        int64_t L64 = seq_lens[r];
        int L = (int)(L64 < 0 ? 0 : (L64 > max_len ? max_len : L64));
        int nq = q_lens ? clampi(q_lens[r], 0, L < max_q_len ? L : max_q_len) : L;
        if (nq > 0 && (q_starts[r] < 0 || (int64_t)q_starts[r] + nq > n_tokens)) return -5;
    }
    const int group = n_qh / n_kvh;
    const int64_t units = (int64_t)n_req * n_kvh;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads;
#else
    (void)n_threads;
#endif
    /* one dense temporary per call, filled for one (request, key/value head) at a time;
       the threads share the gather and then the unit's (head, query) rows */
    uint16_t *kd = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)max_len * (size_t)head_dim);
    uint16_t *vd = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)max_len * (size_t)head_dim);
    if (!kd || !vd) {
        free(kd);
        free(vd);
        return -4;
    }
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads)
#endif
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)max_len);
        if (!scores) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
        for (int64_t u = 0; u < units; ++u) {
            int r = (int)(u / n_kvh);
            int g = (int)(u % n_kvh);
            int64_t L64 = seq_lens[r];
            int L = (int)(L64 < 0 ? 0 : (L64 > max_len ? max_len : L64));
            int nq = q_lens ? clampi(q_lens[r], 0, L < max_q_len ? L : max_q_len) : L;
            int p0 = L - nq;                                 /* position of the first query token */
            if (nq == 0) continue;                           /* the same decision in every thread */
#ifdef _OPENMP
#pragma omp for schedule(static)
#endif
            for (int t = 0; t < L; ++t) {
                int b = clampi(block_table[(int64_t)r * max_blocks + t / block_size], 0, n_blocks - 1);
                int64_t off = (int64_t)b * stride_block + (int64_t)g * stride_kvh +
                              (int64_t)(t % block_size) * stride_tok;
                memcpy(kd + (size_t)t * head_dim, k_pool + off, sizeof(uint16_t) * (size_t)head_dim);
                memcpy(vd + (size_t)t * head_dim, v_pool + off, sizeof(uint16_t) * (size_t)head_dim);
            }
            /* (the loop above ends with a barrier: the temporary is complete) */
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 4)
#endif
            for (int64_t w = 0; w < (int64_t)group * nq; ++w) {
                if (!scores) continue;
                int h = g * group + (int)(w / nq);
                int i = (int)(w % nq);
                int64_t row = ((int64_t)q_starts[r] + i) * n_qh + h;
                attend_one(q + row * head_dim, kd, vd, p0 + i + 1, head_dim, head_dim, scores,
                           ref + row * head_dim, NULL, NULL);
            }
            /* (and so does this one: nobody refills the temporary while it is read) */
        }
        free(scores);
    }
    free(kd);
    free(vd);
    return failed ? -4 : used;
}

/*
 * The cache side of a prompt or mixed pass (section 2.2: the prompt phase processes all
 * prompt tokens in one forward pass, which produces the KV cache; section 2.4: mixed
 * batches).  The pass computes one K row and one V row per query token and key/value
 * head; they belong at the positions of those tokens.  With L = clamp(seq_lens[r], 0,
 * max_len) cached positions INCLUDING the new tokens and nq = clamp(q_lens[r], 0,
 * min(L, max_q_len)) of them new (q_lens == NULL: all L), rows
 * k_rows[q_starts[r] + i, g, :] and v_rows[...] are copied, bit for bit, to position
 * L - nq + i of head g, i < nq.  k_rows, v_rows: dense [n_tokens][n_kvh][head_dim]; a
 * request whose rows would leave [0, n_tokens) returns -5.  Nothing else is written.
 * block_table == NULL: dense caches addressed by (stride_req, stride_kvh, stride_tok);
 * else block pools: position t of request r is row t % block_size of pool block
 * clamp(block_table[r*max_blocks + t/block_size], 0, n_blocks-1), max_len =
 * max_blocks*block_size, and stride_req is the pools' block stride.
 * With nq = 1 this is sw_oracle_kv_append seen from the lengths after the append.
 * Pinned by array slicing, by that equivalence, by paged = dense and by "store a prompt,
 * then attend = attend over a cache that was built directly" (tests/test_oracle_pins.py).
 */
int sw_oracle_kv_store(const uint16_t *k_rows, const uint16_t *v_rows, uint16_t *k, uint16_t *v,
                       const int32_t *block_table, const int32_t *seq_lens,
                       const int32_t *q_starts, const int32_t *q_lens,
                       int n_req, int n_kvh, int head_dim, int max_len, int max_q_len,
                       int64_t n_tokens,
                       int block_size, int max_blocks, int n_blocks,
                       int64_t stride_req, int64_t stride_kvh, int64_t stride_tok)
{
    if (n_req < 0 || n_kvh <= 0 || head_dim <= 0 || max_q_len <= 0 || n_tokens < 0) return -1;
    if (block_table) {
        if (block_size <= 0 || max_blocks <= 0 || n_blocks <= 0) return -1;
        max_len = (int)((int64_t)max_blocks * block_size);
    }
    if (max_len <= 0) return -1;
    if (n_req == 0) return 0;
    if (!k_rows || !v_rows || !k || !v || !seq_lens || !q_starts) return -3;
    for (int r = 0; r < n_req; ++r) {
        int L = clampi(seq_lens[r], 0, max_len);
        int nq = q_lens ? clampi(q_lens[r], 0, L < max_q_len ? L : max_q_len) : L;
        if (nq > 0 && (q_starts[r] < 0 || (int64_t)q_starts[r] + nq > n_tokens)) return -5;
    }
    for (int r = 0; r < n_req; ++r) {
        int L = clampi(seq_lens[r], 0, max_len);
        int nq = q_lens ? clampi(q_lens[r], 0, L < max_q_len ? L : max_q_len) : L;
        for (int i = 0; i < nq; ++i) {
            int64_t t = (int64_t)L - nq + i;                 /* position of query token i */
            for (int g = 0; g < n_kvh; ++g) {
                int64_t dst;
                if (block_table) {
                    int b = clampi(block_table[(int64_t)r * max_blocks + t / block_size], 0, n_blocks - 1);
                    dst = (int64_t)b * stride_req + (int64_t)g * stride_kvh + (t % block_size) * stride_tok;
                } else {
                    dst = (int64_t)r * stride_req + (int64_t)g * stride_kvh + t * stride_tok;
                }
                int64_t src = (((int64_t)q_starts[r] + i) * n_kvh + g) * head_dim;
                for (int j = 0; j < head_dim; ++j) {
                    k[dst + j] = k_rows[src + j];
                    v[dst + j] = v_rows[src + j];
                }
            }
        }
    }
    return 0;
}

/*
 * KV-cache hand-off (sections 4.3 and 5.1: the prompt machine ships each layer's
 * KV cache to the token machine, block by block, merging blocks that are contiguous
 * so that fewer transfers are issued).  Three plain routines cover the part of it
 * that happens inside one GPU's memory:
 *
 * sw_oracle_kv_pack: block pools -> the dense layout, i.e. every (request, head)
 * becomes one contiguous run of L rows (dir = 0), or the reverse (dir = 1).
 * Position t of request r, head g is
 *     pool:  clamp(block_table[r*max_blocks + t/block_size]) * stride_block
 *            + g*p_stride_kvh + (t % block_size)*stride_tok
 *     dense: r*d_stride_req + g*d_stride_kvh + t*stride_tok
 * for t < L = clamp(seq_lens[r], 0, min(max_len, max_blocks*block_size)).
 * Nothing else is written.
 * Pinned: packing pools built from a batch gives the dense buffer built from the
 * same batch; unpack(pack(x)) = x (tests/test_oracle_pins.py).
 */
int sw_oracle_kv_pack(uint16_t *k_pool, uint16_t *v_pool, const int32_t *block_table,
                      const int32_t *seq_lens, uint16_t *k_dense, uint16_t *v_dense, int dir,
                      int n_req, int n_kvh, int head_dim, int max_len,
                      int block_size, int max_blocks, int n_blocks,
                      int64_t stride_block, int64_t p_stride_kvh,
                      int64_t d_stride_req, int64_t d_stride_kvh, int64_t stride_tok)
{
    if (n_req < 0 || n_kvh <= 0 || head_dim <= 0 || max_len <= 0 || block_size <= 0 ||
        max_blocks <= 0 || n_blocks <= 0) return -1;
    if (n_req == 0) return 0;
    if (!k_pool || !v_pool || !block_table || !seq_lens || !k_dense || !v_dense) return -3;
    int64_t cap = (int64_t)max_blocks * block_size;
    if (cap > max_len) cap = max_len;
    for (int r = 0; r < n_req; ++r) {
        int64_t L = seq_lens[r];
        L = L < 0 ? 0 : (L > cap ? cap : L);
        for (int g = 0; g < n_kvh; ++g)
            for (int64_t t = 0; t < L; ++t) {
                int b = clampi(block_table[(int64_t)r * max_blocks + t / block_size], 0, n_blocks - 1);
                int64_t po = (int64_t)b * stride_block + (int64_t)g * p_stride_kvh + (t % block_size) * stride_tok;
                int64_t dn = (int64_t)r * d_stride_req + (int64_t)g * d_stride_kvh + t * stride_tok;
                for (int j = 0; j < head_dim; ++j) {
                    if (dir == 0) {
                        k_dense[dn + j] = k_pool[po + j];
                        v_dense[dn + j] = v_pool[po + j];
                    } else {
                        k_pool[po + j] = k_dense[dn + j];
                        v_pool[po + j] = v_dense[dn + j];
                    }
                }
            }
    }
    return 0;
}

/*
 * sw_oracle_kv_span_plan: the transfers one layer of one request needs when blocks
 * with consecutive pool ids are shipped as one span.  For request r with
 * nb = ceil(L / block_size) blocks in use, entry i starts a new span when i == 0
 * or id[i] != id[i-1] + 1 (ids clamped into the pool).  Outputs, per request:
 * n_spans[r]; span_first[r*max_blocks + k] = pool id of the k-th span's first
 * block; span_blocks[r*max_blocks + k] = its number of blocks.  Entries past
 * n_spans[r] are left as they were.
 */
int sw_oracle_kv_span_plan(const int32_t *block_table, const int32_t *seq_lens,
                           int32_t *span_first, int32_t *span_blocks, int32_t *n_spans,
                           int n_req, int block_size, int max_blocks, int n_blocks)
{
    if (n_req < 0 || block_size <= 0 || max_blocks <= 0 || n_blocks <= 0) return -1;
    if (n_req == 0) return 0;
    if (!block_table || !seq_lens || !span_first || !span_blocks || !n_spans) return -3;
    const int64_t cap = (int64_t)max_blocks * block_size;
    for (int r = 0; r < n_req; ++r) {
        int64_t L = seq_lens[r];
        L = L < 0 ? 0 : (L > cap ? cap : L);
        int nb = (int)((L + block_size - 1) / block_size);
        int k = -1;
        int prev = 0;
        for (int i = 0; i < nb; ++i) {
            int id = clampi(block_table[(int64_t)r * max_blocks + i], 0, n_blocks - 1);
            if (i == 0 || id != prev + 1) {
                ++k;
                span_first[(int64_t)r * max_blocks + k] = id;
                span_blocks[(int64_t)r * max_blocks + k] = 0;
            }
            span_blocks[(int64_t)r * max_blocks + k] += 1;
            prev = id;
        }
        n_spans[r] = k + 1;
    }
    return 0;
}

int sw_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
