// End of a model step: every request's cached length grows by the token the
// step appended (paper section 2.2: each token-phase iteration adds one position
// to the KV cache), saturating at max_len.
#include "sw_internal.h"

namespace {

__global__ __launch_bounds__(256)
void sw_advance_lens_kernel(int32_t *seq_lens, int n_req, int max_len)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= n_req) return;
    int L = seq_lens[r];
    L = L < 0 ? 0 : (L > max_len ? max_len : L);
    seq_lens[r] = L < max_len ? L + 1 : max_len;
}

}  // namespace

hipError_t sw_launch_advance_lens(int32_t *seq_lens, int n_req, int max_len, hipStream_t stream)
{
    const dim3 grid((unsigned)((n_req + 255) / 256));
    hipLaunchKernelGGL(sw_advance_lens_kernel, grid, dim3(256), 0, stream, seq_lens, n_req, max_len);
    return hipGetLastError();
}
