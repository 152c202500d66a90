// KV-cache hand-off inside one GPU's memory (gfx950).
//
// The paper's prompt machine ships each layer's KV cache to the token machine
// block by block and merges blocks that are contiguous, so that fewer transfers
// are issued (sections 4.3 and 5.1).  The part of that which runs on one GPU:
//   * copy a batch's valid rows between block pools and the dense layout, where
//     every (request, head) is one contiguous run (either direction);
//   * plan the spans: runs of consecutive pool block ids per request.
// Both are pure data movement / index work; the copy is bound by HBM bandwidth
// (every byte is read once and written once).
#include "sw_internal.h"

namespace {

typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

constexpr int kCopyThreads = 256;
constexpr int kCopyRows    = 32;     // positions per workgroup (small groups measured fastest: 16 KB each way)

template <int D, bool TO_DENSE>
__global__ __launch_bounds__(kCopyThreads)
void sw_kv_copy_kernel(SwHandoffArgs a)
{
    constexpr int LPR = D / 8;                      // lanes per row (16 bytes each)
    constexpr int RPP = kCopyThreads / LPR;         // rows per pass
    constexpr int PASSES = kCopyRows / RPP;
    static_assert(PASSES >= 1 && PASSES * RPP == kCopyRows, "a workgroup's rows must be whole passes");
    const unsigned unit = blockIdx.x / (unsigned)a.n_tiles;
    const int tile = (int)(blockIdx.x - unit * (unsigned)a.n_tiles);
    const int r = (int)(unit / (unsigned)a.n_kvh);
    const int g = (int)(unit - (unsigned)r * (unsigned)a.n_kvh);
    int L = a.seq_lens[r];
    L = L < 0 ? 0 : (L > a.cap ? a.cap : L);
    const int t0 = tile * kCopyRows;
    if (t0 >= L) return;

    const int sub = threadIdx.x % LPR;
    const int row = threadIdx.x / LPR;
    const int32_t *table = a.block_table + (long long)r * a.max_blocks;
    const long long dense0 = (long long)r * a.d_stride_req + (long long)g * a.d_stride_kvh + sub * 8;
    const long long pool0  = (long long)g * a.p_stride_kvh + sub * 8;

    // Three phases, each with all of a thread's requests in flight together: block ids,
    // rows in, rows out.  Rows past the length re-read the last valid row (in bounds) and
    // are not stored.
    int id[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int t = min(t0 + p * RPP + row, L - 1);
        id[p] = table[t >> a.block_shift];
    }
    uint4_t kx[PASSES], vx[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int t = min(t0 + p * RPP + row, L - 1);
        const int b = id[p] < 0 ? 0 : (id[p] >= a.n_blocks ? a.n_blocks - 1 : id[p]);
        const long long po = pool0 + (long long)b * a.stride_block + (long long)(t & ((1 << a.block_shift) - 1)) * D;
        const long long dn = dense0 + (long long)t * D;
        const long long src = TO_DENSE ? po : dn;
        // read once: keep the stream out of the way of whatever else lives in L2
        kx[p] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>((TO_DENSE ? a.k_pool : a.k_dense) + src));
        vx[p] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>((TO_DENSE ? a.v_pool : a.v_dense) + src));
    }
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int t = t0 + p * RPP + row;
        if (t < L) {
            const int b = id[p] < 0 ? 0 : (id[p] >= a.n_blocks ? a.n_blocks - 1 : id[p]);
            const long long po = pool0 + (long long)b * a.stride_block + (long long)(t & ((1 << a.block_shift) - 1)) * D;
            const long long dn = dense0 + (long long)t * D;
            const long long dst = TO_DENSE ? dn : po;
            *reinterpret_cast<uint4_t *>((TO_DENSE ? a.k_dense : a.k_pool) + dst) = kx[p];
            *reinterpret_cast<uint4_t *>((TO_DENSE ? a.v_dense : a.v_pool) + dst) = vx[p];
        }
    }
}

// One wave per request walks the request's table entries 64 at a time.
__global__ __launch_bounds__(64)
void sw_kv_span_plan_kernel(const int32_t *block_table, const int32_t *seq_lens,
                            int32_t *span_first, int32_t *span_blocks, int32_t *n_spans,
                            int n_req, int block_shift, int max_blocks, int n_blocks)
{
    const int r = blockIdx.x;
    if (r >= n_req) return;
    const int lane = threadIdx.x;
    const long long cap = (long long)max_blocks << block_shift;
    long long L = seq_lens[r];
    L = L < 0 ? 0 : (L > cap ? cap : L);
    const int nb = (int)((L + (1 << block_shift) - 1) >> block_shift);
    const int32_t *table = block_table + (long long)r * max_blocks;
    int32_t *first = span_first + (long long)r * max_blocks;
    int32_t *count = span_blocks + (long long)r * max_blocks;

    int n = 0;              // spans started so far (wave-uniform)
    int open_start = 0;     // entry index where the last started span begins
    for (int base = 0; base < nb; base += 64) {
        const int i = base + lane;
        bool start = false;
        int id = 0;
        if (i < nb) {
            id = table[i];
            id = id < 0 ? 0 : (id >= n_blocks ? n_blocks - 1 : id);
            if (i == 0) {
                start = true;
            } else {
                int prev = table[i - 1];
                prev = prev < 0 ? 0 : (prev >= n_blocks ? n_blocks - 1 : prev);
                start = id != prev + 1;
            }
        }
        const unsigned long long mask = __ballot(start);
        if (mask == 0) continue;
        const int before = __popcll(mask & ((1ull << lane) - 1ull));     // starts in lower lanes
        const int first_lane = __builtin_ctzll(mask);
        if (start) {
            const int k = n + before;
            first[k] = id;
            // a later start in this chunk closes this span at once
            const unsigned long long later = lane == 63 ? 0ull : (mask >> (lane + 1));
            if (later) count[k] = __builtin_ctzll(later) + 1;
            // the first start of the chunk closes the span left open by earlier chunks
            if (lane == first_lane && n > 0) count[n - 1] = i - open_start;
        }
        const int last_lane = 63 - __builtin_clzll(mask);
        open_start = base + last_lane;
        n += __popcll(mask);
    }
    if (lane == 0) {
        if (n > 0) count[n - 1] = nb - open_start;
        n_spans[r] = n;
    }
}

}  // namespace

int sw_kv_copy_rows_per_group() { return kCopyRows; }

hipError_t sw_launch_kv_copy(const SwHandoffArgs &a, bool to_dense, hipStream_t stream, const SwLaunchEvents *ev)
{
    const long long units = (long long)a.n_req * a.n_kvh;
    if (a.n_tiles <= 0 || units <= 0 || units * a.n_tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(units * a.n_tiles)), block(kCopyThreads);
    if (a.head_dim == 128)
        return to_dense ? sw_launch(sw_kv_copy_kernel<128, true>, grid, block, 0, stream, ev, a)
                        : sw_launch(sw_kv_copy_kernel<128, false>, grid, block, 0, stream, ev, a);
    return to_dense ? sw_launch(sw_kv_copy_kernel<64, true>, grid, block, 0, stream, ev, a)
                    : sw_launch(sw_kv_copy_kernel<64, false>, grid, block, 0, stream, ev, a);
}

hipError_t sw_launch_kv_span_plan(const int32_t *block_table, const int32_t *seq_lens,
                                  int32_t *span_first, int32_t *span_blocks, int32_t *n_spans,
                                  int n_req, int block_shift, int max_blocks, int n_blocks,
                                  hipStream_t stream)
{
    hipLaunchKernelGGL(sw_kv_span_plan_kernel, dim3((unsigned)n_req), dim3(64), 0, stream,
                       block_table, seq_lens, span_first, span_blocks, n_spans,
                       n_req, block_shift, max_blocks, n_blocks);
    return hipGetLastError();
}
