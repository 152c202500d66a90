// Merge of the chunks' partial results of one output row, the arithmetic of the second
// kernel of the split over context length:
//   m = max_c m_c;  out = sum_c 2^(m_c - m) o_c / sum_c 2^(m_c - m) l_c
// Eight chunk groups: group k walks chunks k, k+8, k+16, ... with a running maximum, then
// the groups are merged in group order.  Two users -- the combine kernel, where a group is
// a set of lanes and the groups meet in LDS, and the prompt kernel of a mixed batch, whose
// spare workgroups merge the token-phase rows with one thread per (row, four dims) walking
// all eight groups itself.  Both go through the functions below, operation for operation,
// so a row has the same bits whichever kernel merged it.
#pragma once
#include "sw_internal.h"

namespace sw_merge {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));

constexpr int   kGroups = 8;
constexpr float kNegBig = -1.0e30f;

// State of one chunk group for four output dims.
struct Group {
    float    m;      // running maximum (base-2 exponent units)
    float    den;
    float4_t num;
};

__device__ __forceinline__ Group empty_group()
{
    Group g;
    g.m = kNegBig;
    g.den = 0.f;
    g.num = float4_t{0.f, 0.f, 0.f, 0.f};
    return g;
}

// One more chunk into its group: (mc, lc) = the chunk's maximum and sum, x = its four dims.
__device__ __forceinline__ void add_chunk(Group &g, float mc, float lc, float4_t x)
{
    const float m_new = fmaxf(g.m, mc);
    const float f_old = __builtin_amdgcn_exp2f(g.m - m_new);
    const float f_new = __builtin_amdgcn_exp2f(mc - m_new);
#pragma unroll
    for (int t = 0; t < 4; ++t) g.num[t] = fmaf(f_new, x[t], g.num[t] * f_old);
    g.den = fmaf(f_new, lc, g.den * f_old);
    g.m = m_new;
}

// The eight groups into the row's four binary16 values (round to nearest even).
// Empty groups contribute 2^(-1e30 - mx) = 0.
template <typename GetGroup>
__device__ __forceinline__ half4_t finish(GetGroup get)
{
    float mx = get(0).m;
#pragma unroll
    for (int g = 1; g < kGroups; ++g) mx = fmaxf(mx, get(g).m);
    float4_t tot = float4_t{0.f, 0.f, 0.f, 0.f};
    float dtot = 0.f;
#pragma unroll
    for (int g = 0; g < kGroups; ++g) {
        const Group s = get(g);
        const float f = __builtin_amdgcn_exp2f(s.m - mx);
#pragma unroll
        for (int t = 0; t < 4; ++t) tot[t] = fmaf(f, s.num[t], tot[t]);
        dtot = fmaf(f, s.den, dtot);
    }
    half4_t res;
#pragma unroll
    for (int t = 0; t < 4; ++t) res[t] = (_Float16)(tot[t] / dtot);
    return res;
}

// The whole merge of output row rh = r * n_qh + h by one thread per four dims (j4 = which
// four): used where no workgroup-wide cooperation is available.  Up to 16 chunks' loads
// are in flight at a time.
template <int D>
__device__ __forceinline__ void merge_row_serial(const SwArgs &a, int rh, int j4)
{
    constexpr int V4 = D / 4;
    constexpr int kRound = 2 * kGroups;
    const int r = rh / a.n_qh;
    const int h = rh - r * a.n_qh;
    const int g = h / a.group;
    const int lf = sw_request_len_flagged(a, r);
    if (lf == kSwSkip) return;                   // the request takes no part in this call
    const int L = lf & kSwLenMask;
    const int nc = (L + a.chunk - 1) >> a.chunk_shift;
    half4_t *out = reinterpret_cast<half4_t *>(reinterpret_cast<_Float16 *>(a.out) + (sw_q_row(a, r) * a.n_qh + h) * D) + j4;
    if (nc == 0) {
        *out = half4_t{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
        return;
    }
    const long long slot0 = sw_ws_slot(a, r, g, 0, h - g * a.group);   // chunk c is at slot0 + c*group
    const float2_t *ml = reinterpret_cast<const float2_t *>(a.ws_ml) + slot0;
    const float4_t *po = reinterpret_cast<const float4_t *>(a.ws_o + slot0 * D) + j4;
    const long long cs = a.group;
    Group grp[kGroups];
#pragma unroll
    for (int k = 0; k < kGroups; ++k) grp[k] = empty_group();
    for (int c0 = 0; c0 < nc; c0 += kRound) {
        float2_t mlc[kRound];
        float4_t x[kRound];
#pragma unroll
        for (int u = 0; u < kRound; ++u) {
            const int c = min(c0 + u, nc - 1);       // clamped: in bounds, unused past nc
            mlc[u] = ml[c * cs];
            x[u]   = po[c * cs * V4];
        }
        // chunk c0 + u belongs to group u % 8; within a group in rising chunk order
#pragma unroll
        for (int u = 0; u < kRound; ++u)
            if (c0 + u < nc) add_chunk(grp[u % kGroups], mlc[u][0], mlc[u][1], x[u]);
    }
    *out = finish([&](int k) { return grp[k]; });
}

}  // namespace sw_merge
