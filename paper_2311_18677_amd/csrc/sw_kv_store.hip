// The cache side of a prompt or mixed pass: the K and V rows a forward pass has just
// computed for the new tokens go to their positions in the KV cache (paper section
// 2.2: the prompt phase processes all prompt tokens in one pass, which produces the
// cache; section 2.4: mixed batches).  Request r's last NQ cached positions are the new
// ones; token i of them (row q_starts[r] + i of the packed [n_tokens][n_kvh][D] inputs)
// belongs at position L - NQ + i.  A plain copy, bound by HBM: one workgroup moves the
// rows of 32 tokens of one (request, key/value head), eight lanes per row, 16 bytes per
// lane and step.  Workgroups find their (request, block of 32 tokens) the way the
// prompt kernels do, so a batch of one long prompt and many single tokens costs what its
// tokens cost.
#include "sw_prefill_common.h"

namespace {

using namespace sw_prefill;

constexpr int kStoreTokens = 32;       // tokens per workgroup
constexpr int kStoreThreads = 256;     // 8 lanes per token row

typedef const __attribute__((address_space(4))) int32_t *const_table_t;

template <int D>
__global__ __launch_bounds__(kStoreThreads)
void sw_kv_store_kernel(SwPrefillArgs a, const uint16_t *k_rows, const uint16_t *v_rows,
                        uint16_t *k_out, uint16_t *v_out)
{
    const QItem it = find_item(a, blockIdx.x, kStoreTokens);
    if (!it.valid) return;
    const int g = (int)blockIdx.y;
    const int qi = it.qb * kStoreTokens + (int)(threadIdx.x >> 3);       // index among the request's new tokens
    if (qi >= it.NQ) return;
    const long long row = it.q_first + qi;
    if (row < 0 || row >= a.n_tokens) return;                            // such rows do not exist: skipped
    const int pos = it.L - it.NQ + qi;                                   // in [0, L)
    long long dst;
    if (a.block_table) {
        int id = a.block_table[(long long)it.r * a.max_blocks + (pos >> a.block_shift)];
        id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
        dst = (long long)id * a.stride_block + (long long)g * a.stride_kvh +
              (long long)(pos & ((1 << a.block_shift) - 1)) * D;
    } else {
        dst = (long long)it.r * a.stride_req + (long long)g * a.stride_kvh + (long long)pos * D;
    }
    const long long src = (row * a.n_kvh + g) * D;
    const int lane8 = (int)(threadIdx.x & 7);
    uint4_t kk[D / 64], vv[D / 64];
#pragma unroll
    for (int p = 0; p < D / 64; ++p) {
        kk[p] = *reinterpret_cast<const uint4_t *>(k_rows + src + 8 * (lane8 + 8 * p));
        vv[p] = *reinterpret_cast<const uint4_t *>(v_rows + src + 8 * (lane8 + 8 * p));
    }
#pragma unroll
    for (int p = 0; p < D / 64; ++p) {
        *reinterpret_cast<uint4_t *>(k_out + dst + 8 * (lane8 + 8 * p)) = kk[p];
        *reinterpret_cast<uint4_t *>(v_out + dst + 8 * (lane8 + 8 * p)) = vv[p];
    }
}

}  // namespace

hipError_t sw_launch_kv_store(const SwPrefillArgs &a_in, const uint16_t *k_rows, const uint16_t *v_rows,
                              uint16_t *k_out, uint16_t *v_out, hipStream_t stream, const SwLaunchEvents *ev)
{
    SwPrefillArgs a = a_in;
    if (a.head_dim != 64 && a.head_dim != 128) return hipErrorNotSupported;
    if (a.n_kvh < 1 || a.n_kvh > 65535) return hipErrorInvalidValue;
    bool compact;
    const long long items = sw_prefill_items(a, kStoreTokens, &compact);
    if (items <= 0 || items > 0x7fffffffLL) return hipErrorInvalidValue;
    a.compact = compact;
    const dim3 grid((unsigned)items, (unsigned)a.n_kvh);
    if (a.head_dim == 128)
        return sw_launch(sw_kv_store_kernel<128>, grid, dim3(kStoreThreads), 0, stream, ev, a, k_rows, v_rows, k_out, v_out);
    return sw_launch(sw_kv_store_kernel<64>, grid, dim3(kStoreThreads), 0, stream, ev, a, k_rows, v_rows, k_out, v_out);
}
