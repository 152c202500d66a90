// Internal interface between the host dispatcher (sw_api.hip) and the kernel
// translation units.  Not installed; the public ABI is include/sw_decode.h.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

// State of one (request, key/value head, head tile) unit of the single-launch variant,
// kept between calls: the ticket counter is zero outside a launch, the epoch counts the
// calls in which the unit merged.
struct SwUnitState {
    unsigned ticket;
    unsigned epoch;
};

// Everything a kernel needs, passed by value.
//
// Split over context length: positions [0, L) of a request are cut into
// chunks of `chunk` positions; a workgroup of the partial kernel handles chunk
// c of key/value head g of request r for the query heads that head serves,
// and leaves per query head an unnormalised partial result in the workspace.
// The workspace is item-major, so that one workgroup writes one contiguous
// block: with slot(r, g, c, hh) = ((r*n_kvh + g)*n_chunks + c)*group + hh for
// the hh-th head of the group,
//   ws_o [slot*head_dim + j] = sum_t 2^(s2_t - m2) * V[t][j]
//   ws_ml[slot*2 + {0,1}]    = m2, sum_t 2^(s2_t - m2)
// where s2 = score * log2(e) (so that the exponentials are exp2) and m2 is
// the chunk's maximum of s2.  Chunks at or past L are never written nor read.
struct SwArgs {
    const uint16_t *q;
    const uint16_t *k;
    const uint16_t *v;
    const int32_t  *seq_lens;
    uint16_t       *out;
    float          *ws_o;
    float          *ws_ml;
    // single-launch variant (else units is null): per-unit ticket and epoch, the tagged
    // 16-byte pieces (see sw_fused.h), and a word the device sets if a merge gave up
    // waiting for a piece
    SwUnitState    *units;
    void           *ws_tag;
    unsigned        ws_tag_bytes;
    unsigned       *dev_err;
    const uint16_t *k_new;              // append variant: the newest token's K rows [n_req][n_kvh][head_dim], else null
    const uint16_t *v_new;              //                 and V rows
    const int32_t  *block_table;        // block-table variant: [n_req][max_blocks] pool block ids, else null
    // Token-phase part of a mixed batch (all null / 0 otherwise): request r takes part only
    // if exactly one of its tokens is a query (q_lens[r] clamped to [0, min(L, max_q)] is 1)
    // and q_rows[r] is a row of q and out ([n_rows][n_qh][head_dim]); its query and result
    // are that row instead of row r.  The other requests are neither read nor written.
    const int32_t  *q_rows;
    const int32_t  *q_lens;
    long long       n_rows;
    int             max_q;
    int   n_req, n_qh, n_kvh, group;   // group = n_qh / n_kvh
    int   head_dim, max_len;
    int   chunk, chunk_shift, n_chunks; // chunk = 1 << chunk_shift; n_chunks = ceil(max_len / chunk)
    int   waves;                        // waves per workgroup of the matrix-core partial kernel (4 or 8)
    long long stride_req, stride_kvh;  // elements; the token stride is head_dim
    // block-table variant: k, v are pools; row t of request r is row t % block_size of pool
    // block block_table[r*max_blocks + t / block_size]; stride_req is unused
    long long stride_block;
    int   block_shift, max_blocks, n_blocks;   // block_size = 1 << block_shift
    float scale_log2e;                 // log2(e) / sqrt(head_dim)
};

// Arguments of the prompt-phase (causal) kernel.
struct SwPrefillArgs {
    const uint16_t *q;                  // [n_tokens][n_qh][head_dim]
    const uint16_t *k;                  // caches in the dense layout
    const uint16_t *v;
    const int32_t  *seq_lens;           // prompt lengths
    const int32_t  *q_starts;           // row of each request's first query token
    const int32_t  *q_lens;             // query tokens per request (the last ones), or null: all of them
    uint16_t       *out;                // [n_tokens][n_qh][head_dim]
    long long n_tokens;
    int   n_req, n_qh, n_kvh, group;
    int   head_dim, max_len;
    int   max_q;                        // bound on the query tokens of a request (sizes the grid)
    int   skip_single;                  // non-zero: requests with exactly one query token are left out
    int   compact;                      // non-zero: workgroups find their (request, query block) by a scan of the lengths
    int   hp;                           // query heads (of one group) per workgroup
    int   qw;                           // waves per query head in a workgroup
    int   n_qblocks;                    // query blocks (of 32 * qw positions) that cover max_len
    long long stride_req, stride_kvh;   // in elements
    // block-table variant: k, v are pools, row t of request r is row
    // t % block_size of pool block block_table[r*max_blocks + t / block_size]; stride_req unused
    const int32_t *block_table;         // null for the dense layout
    long long stride_block;
    int   block_shift, max_blocks, n_blocks;
    float scale_log2e;
};

// Arguments of the pools <-> dense copy of the KV hand-off.
struct SwHandoffArgs {
    uint16_t *k_pool, *v_pool;          // block pools
    uint16_t *k_dense, *v_dense;        // dense caches
    const int32_t *block_table;
    const int32_t *seq_lens;
    int   n_req, n_kvh, head_dim;
    int   cap;                          // positions copied at most: min(max_len, max_blocks * block_size)
    int   n_tiles;                      // workgroups per (request, head)
    int   block_shift, max_blocks, n_blocks;
    long long stride_block, p_stride_kvh;       // pools, in elements
    long long d_stride_req, d_stride_kvh;       // dense, in elements
};

// Number of cached positions request r attends over, with a flag.  seq_lens[r]
// is clamped to [0, max_len]; in the append variant it counts the positions
// cached BEFORE the newest token, whose K/V rows this call stores at that
// position (and attends over) unless the cache is already full.  Bit
// kSwAppendedBit of the result says that the rows are stored, i.e. that
// position L - 1 is the new one; the bits below it hold L (max_len <= 2^23).
// kSwSkip (negative, length bits 0) marks a request that takes no part in the call:
// it has no work item and its output row is left alone.
constexpr int kSwAppendedBit = 30;
constexpr int kSwLenMask     = (1 << kSwAppendedBit) - 1;
constexpr int kSwSkip        = (int)0x80000000u;

// (sw_flag_len: the same from a seq_lens[r] value that has already been read)
__device__ inline int sw_flag_len(const SwArgs &a, int r, int L)
{
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    if (a.q_lens) {
        const int cap = L < a.max_q ? L : a.max_q;
        const int nq = a.q_lens[r] < cap ? a.q_lens[r] : cap;
        const long long row = a.q_rows[r];
        if (nq != 1 || row < 0 || row >= a.n_rows) return kSwSkip;
    }
    if (a.k_new && L < a.max_len) L += 1 + (1 << kSwAppendedBit);
    return L;
}

__device__ inline int sw_request_len_flagged(const SwArgs &a, int r)
{
    return sw_flag_len(a, r, a.seq_lens[r]);
}

// Row of q and out that belongs to request r (valid for requests that take part).
__device__ inline long long sw_q_row(const SwArgs &a, int r)
{
    return a.q_rows ? (long long)a.q_rows[r] : (long long)r;
}

__device__ inline int sw_request_len(const SwArgs &a, int r)
{
    return sw_request_len_flagged(a, r) & kSwLenMask;
}

__host__ __device__ inline long long sw_ws_slot(const SwArgs &a, int r, int g, int c, int hh)
{
    return (((long long)r * a.n_kvh + g) * a.n_chunks + c) * a.group + hh;
}

// Optional per-kernel timing: when both are non-null the launch attaches them
// to the dispatch so that their difference is the kernel's device time.
struct SwLaunchEvents {
    hipEvent_t start;
    hipEvent_t stop;
};

// Vector-ALU partial kernel: any group size (looped in tiles of up to 8 heads).
hipError_t sw_launch_partial_valu(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev);
// Matrix-core kernel, K and V staged through LDS (head_dim 128, groups up to 64, 4 or 8 waves).
bool       sw_decode_split_supported(const SwArgs &a);
hipError_t sw_launch_decode_split(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev);
// Merge of the chunks' partial results, normalisation and rounding to binary16.
hipError_t sw_launch_combine(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev);
// Bound on the (request, block of q_block query tokens) items of a prompt-phase call, which
// sizes its grid: no request has more than n_qblocks of them, and requests whose rows of q
// and out do not overlap have at most n_tokens / q_block + 2 per request between them.
static inline long long sw_prefill_items(const SwPrefillArgs &a, int q_block, bool *compact)
{
    const long long by_shape = (long long)a.n_req * a.n_qblocks;
    const long long by_rows = a.n_tokens / q_block + 2LL * a.n_req;
    // the scan costs every workgroup a little (every wave reads all the lengths, ceil(n_req / 64)
    // per lane): it pays once it removes a good part of the grid, and never for huge batches
    *compact = by_rows * 4 < by_shape * 3 && a.n_req <= 4096;
    return *compact ? by_rows : by_shape;
}
bool       sw_prefill_mfma_supported(const SwPrefillArgs &a);
void       sw_prefill_shape(int n_req, int n_kvh, int group, int max_len, int *hp, int *qw);
// merge != null (mixed batches, four waves): extra workgroups merge the token-phase chunks that the
// partial kernel launched before on the same stream left in the workspace (instead of the combine kernel)
hipError_t sw_launch_prefill_split(const SwPrefillArgs &a, int waves, hipStream_t stream, const SwLaunchEvents *ev,
                                   const SwArgs *merge = nullptr);
hipError_t sw_launch_prefill_mfma(const SwPrefillArgs &a, hipStream_t stream, const SwLaunchEvents *ev);
int        sw_kv_copy_rows_per_group();
hipError_t sw_launch_kv_copy(const SwHandoffArgs &a, bool to_dense, hipStream_t stream, const SwLaunchEvents *ev);
hipError_t sw_launch_kv_span_plan(const int32_t *block_table, const int32_t *seq_lens,
                                  int32_t *span_first, int32_t *span_blocks, int32_t *n_spans,
                                  int n_req, int block_shift, int max_blocks, int n_blocks,
                                  hipStream_t stream);
hipError_t sw_launch_kv_store(const SwPrefillArgs &a, const uint16_t *k_rows, const uint16_t *v_rows,
                              uint16_t *k_out, uint16_t *v_out, hipStream_t stream, const SwLaunchEvents *ev);
hipError_t sw_launch_stream_read(const void *src, unsigned long long n_bytes, unsigned *sink,
                                 int workgroups, hipStream_t stream, const SwLaunchEvents *ev);
hipError_t sw_launch_advance_lens(int32_t *seq_lens, int n_req, int max_len, hipStream_t stream);

// Granularity the chunk length must be a multiple of (all kernels).
constexpr int SW_CHUNK_QUANTUM = 64;

template <typename... KArgs, typename... Args>
static inline hipError_t sw_launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds,
                                   hipStream_t stream, const SwLaunchEvents *ev, Args... args)
{
    if (ev && ev->start && ev->stop) {
        hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ev->start, ev->stop, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, args...);
    }
    return hipGetLastError();
}
