// Second kernel of the split over context length: merges the chunks' partial
// results of each (request, query head), normalises and rounds to binary16.
//   m = max_c m_c;  out = sum_c 2^(m_c - m) o_c / sum_c 2^(m_c - m) l_c
//
// One workgroup of 256 threads per output row: 8 chunk groups x (D/4) lanes.
// Group k walks chunks k, k+8, k+16, ... with a running maximum (all of a
// thread's loads for up to four chunks are in flight together), then the 8
// groups merge through LDS in group order.  The summation order depends only
// on the request's own chunk count, so its bits do not depend on the batch.
#include "sw_internal.h"
#include "sw_merge.h"

namespace {

using namespace sw_merge;

template <int D>
__global__ __launch_bounds__(kGroups * (D / 4))
void sw_combine_kernel(SwArgs a)
{
    constexpr int V4 = D / 4;
    __shared__ float4_t sm_num[kGroups][V4];
    __shared__ float2_t sm_md[kGroups][V4];      // (running max, denominator) per group and lane

    const int rh = blockIdx.x;                   // r * n_qh + h
    const int r  = rh / a.n_qh;
    const int k  = threadIdx.x / V4;             // chunk group
    const int j4 = threadIdx.x - k * V4;
    const int h = rh - r * a.n_qh;
    const int g = h / a.group;
    const long long slot0 = sw_ws_slot(a, r, g, 0, h - g * a.group);   // chunk c is at slot0 + c*group
    const float2_t *ml = reinterpret_cast<const float2_t *>(a.ws_ml) + slot0;
    const float4_t *po = reinterpret_cast<const float4_t *>(a.ws_o + slot0 * D) + j4;
    const long long cs = a.group;                                     // slots between consecutive chunks

    // Partial results are requested once the length is known, so that slots nobody wrote are
    // never fetched.  (Asking for the first chunks together with the length was measured on the
    // five benchmark workloads: no faster on any, and it fetched up to five times the bytes
    // that were written.)
    float2_t mlc[4];
    float4_t x[4];
    const int lf = sw_request_len_flagged(a, r);
    if (lf == kSwSkip) return;                   // the request takes no part in this call
    const int L = lf & kSwLenMask;
    const int nc = (L + a.chunk - 1) >> a.chunk_shift;
    half4_t *out = reinterpret_cast<half4_t *>(reinterpret_cast<_Float16 *>(a.out) + (sw_q_row(a, r) * a.n_qh + h) * D) + j4;
    if (nc == 0) {
        if (k == 0) *out = half4_t{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
        return;
    }

    Group mine = empty_group();
    for (int c0 = k; c0 < nc; c0 += 4 * kGroups) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * kGroups;
            if (c < nc) {
                mlc[u] = ml[c * cs];
                x[u]   = po[c * cs * V4];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (c0 + u * kGroups < nc) add_chunk(mine, mlc[u][0], mlc[u][1], x[u]);
        }
    }
    sm_num[k][j4] = mine.num;
    sm_md[k][j4]  = float2_t{mine.m, mine.den};
    __syncthreads();
    if (k != 0) return;
    *out = finish([&](int g) {
        Group s;
        s.m = sm_md[g][j4][0];
        s.den = sm_md[g][j4][1];
        s.num = sm_num[g][j4];
        return s;
    });
}

}  // namespace

hipError_t sw_launch_combine(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    dim3 grid((unsigned)(a.n_req * a.n_qh));
    if (a.head_dim == 128)
        return sw_launch(sw_combine_kernel<128>, grid, dim3(kGroups * 32), 0, stream, ev, a);
    return sw_launch(sw_combine_kernel<64>, grid, dim3(kGroups * 16), 0, stream, ev, a);
}
