// Second kernel of the split over context length: merges the chunks' partial
// results of each (request, query head), normalises and rounds to binary16.
//   m = max_c m_c;  out = sum_c 2^(m_c - m) o_c / sum_c 2^(m_c - m) l_c
// The chunks are visited in index order, so the result's bits depend only on
// the request's own length.
#include "sw_internal.h"

namespace {

template <int D>
__global__ __launch_bounds__(D)
void sw_combine_kernel(SwArgs a)
{
    const int rh = blockIdx.x;                 // r * n_qh + h
    const int r  = rh / a.n_qh;
    const int j  = threadIdx.x;
    int L = a.seq_lens[r];
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    const int nc = (L + a.chunk - 1) >> a.chunk_shift;
    _Float16 *out = reinterpret_cast<_Float16 *>(a.out) + (long long)rh * D + j;
    if (nc == 0) {
        *out = (_Float16)0.f;
        return;
    }
    const float *ml = a.ws_ml + (long long)rh * a.n_chunks * 2;
    const float *po = a.ws_o + (long long)rh * a.n_chunks * D + j;
    float mx = ml[0];
    for (int c = 1; c < nc; ++c) mx = fmaxf(mx, ml[2 * c]);
    float num = 0.f, den = 0.f;
    int c = 0;
    for (; c + 4 <= nc; c += 4) {
        float f[4], x[4], lc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[i]  = ml[2 * (c + i)];
            lc[i] = ml[2 * (c + i) + 1];
            x[i]  = po[(long long)(c + i) * D];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float w = __builtin_amdgcn_exp2f(f[i] - mx);
            num = fmaf(w, x[i], num);
            den = fmaf(w, lc[i], den);
        }
    }
    for (; c < nc; ++c) {
        const float w = __builtin_amdgcn_exp2f(ml[2 * c] - mx);
        num = fmaf(w, po[(long long)c * D], num);
        den = fmaf(w, ml[2 * c + 1], den);
    }
    *out = (_Float16)(num / den);              // round to nearest even
}

}  // namespace

hipError_t sw_launch_combine(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    dim3 grid((unsigned)(a.n_req * a.n_qh));
    if (a.head_dim == 128)
        return sw_launch(sw_combine_kernel<128>, grid, dim3(128), 0, stream, ev, a);
    return sw_launch(sw_combine_kernel<64>, grid, dim3(64), 0, stream, ev, a);
}
