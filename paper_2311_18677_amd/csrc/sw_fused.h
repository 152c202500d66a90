// Single-launch variant of the split over context length: the workgroup that
// finishes a (request, key/value head, head tile) last merges that unit's
// chunks itself, so no second kernel is needed.
//
// The partial results cross workgroups on different XCDs, whose L2 caches are
// not coherent with each other.  Device-wide release/acquire fences would make
// them coherent by writing back and invalidating a whole L2 per workgroup, which
// costs far more than the kernel itself; instead every access to a shared
// location is a relaxed device-scope atomic (compiled to a load/store that is
// served at the device's coherence point, no cache maintenance), and ordering
// comes from completion: a workgroup waits until its partial stores have been
// acknowledged (s_waitcnt vmcnt(0), then the workgroup barrier) before one of
// its threads takes a ticket from the unit's counter, and the holder of the last
// ticket (nc - 1) reads the partial results only after it has seen its ticket.
// It merges chunks 0 .. nc-1 in index order (a fixed order, so repeated calls
// give the same bits), writes the binary16 output rows and puts the counter back to zero for the next call
// on the stream.  Counters start at zero (cleared when the library allocates
// them) and every launch leaves them zero.
#pragma once
#include "sw_internal.h"

typedef float sw_float4_t __attribute__((ext_vector_type(4)));
typedef float sw_float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 sw_half4_t __attribute__((ext_vector_type(4)));

// Device-coherent 8-byte accesses (p is 8-byte aligned).
__device__ __forceinline__ void sw_coherent_store2(float *p, float x, float y)
{
    union { sw_float2_t f; unsigned long long u; } v;
    v.f = sw_float2_t{x, y};
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), v.u, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ sw_float2_t sw_coherent_load2(const float *p)
{
    union { sw_float2_t f; unsigned long long u; } v;
    v.u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                            __HIP_MEMORY_SCOPE_AGENT);
    return v.f;
}

// Store four consecutive partial-result floats (p is 16-byte aligned); coherent
// across the device when the single-launch variant will read them back.
__device__ __forceinline__ void sw_store_partial4(float *p, sw_float4_t x, bool coherent)
{
    if (coherent) {
        sw_coherent_store2(p, x[0], x[1]);
        sw_coherent_store2(p + 2, x[2], x[3]);
    } else {
        *reinterpret_cast<sw_float4_t *>(p) = x;
    }
}

__device__ __forceinline__ void sw_store_partial2(float *p, float x, float y, bool coherent)
{
    if (coherent) sw_coherent_store2(p, x, y);
    else *reinterpret_cast<sw_float2_t *>(p) = sw_float2_t{x, y};
}

// A request with a single chunk needs no merge at all: in the single-launch variant its
// workgroup normalises and writes the output rows itself (the same arithmetic the merge
// would do with one chunk, so the same bits), and takes no ticket.
template <int D>
__device__ __forceinline__ void sw_store_final4(const SwArgs &a, long long rh, int j4, sw_float4_t num, float den)
{
    sw_half4_t res;
#pragma unroll
    for (int t = 0; t < 4; ++t) res[t] = (_Float16)(num[t] / den);   // round to nearest even
    *reinterpret_cast<sw_half4_t *>(reinterpret_cast<_Float16 *>(a.out) + rh * D + 4 * j4) = res;
}

// Called by every thread of the workgroup after its partial-result stores.
//   r, g, hh_first, n_heads : heads hh_first .. hh_first + n_heads - 1 of the group of
//                         key/value head g of request r
//   nc                  : number of chunks of request r (>= 1)
//   counter             : this unit's ticket counter
//   sm_flag             : one int of LDS
template <int D>
__device__ __forceinline__ void sw_fused_tail(const SwArgs &a, int r, int g, int hh_first, int n_heads,
                                              int nc, unsigned *counter, int *sm_flag)
{
    __builtin_amdgcn_s_waitcnt(0);         // this thread's partial stores are acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
        const int last = ticket == (unsigned)(nc - 1);
        if (last)   // everyone has arrived; ready for the next call
            __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *sm_flag = last;
    }
    __syncthreads();
    if (!*sm_flag) return;

    constexpr int V4 = D / 4;
    constexpr int kBatch = 8;
    for (int idx = threadIdx.x; idx < n_heads * V4; idx += blockDim.x) {
        const int hh = idx / V4;
        const int j4 = idx - hh * V4;
        const long long rh = sw_q_row(a, r) * a.n_qh + g * a.group + hh_first + hh;
        const long long slot0 = sw_ws_slot(a, r, g, 0, hh_first + hh);
        const long long cs = a.group;                     // slots between consecutive chunks
        const float *ml = a.ws_ml + slot0 * 2;
        const float *po = a.ws_o + slot0 * D + 4 * j4;
        // running-maximum merge, kBatch chunks' loads in flight at a time
        float m = -1.0e30f, den = 0.f;
        sw_float4_t num = sw_float4_t{0.f, 0.f, 0.f, 0.f};
        for (int c0 = 0; c0 < nc; c0 += kBatch) {
            sw_float2_t mlc[kBatch], x01[kBatch], x23[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int c = min(c0 + u, nc - 1);       // clamped: in bounds, masked below
                mlc[u] = sw_coherent_load2(ml + 2 * c * cs);
                x01[u] = sw_coherent_load2(po + c * cs * D);
                x23[u] = sw_coherent_load2(po + c * cs * D + 2);
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                if (c0 + u < nc) {
                    const float m_new = fmaxf(m, mlc[u][0]);
                    const float f_old = __builtin_amdgcn_exp2f(m - m_new);
                    const float f_new = __builtin_amdgcn_exp2f(mlc[u][0] - m_new);
                    num[0] = fmaf(f_new, x01[u][0], num[0] * f_old);
                    num[1] = fmaf(f_new, x01[u][1], num[1] * f_old);
                    num[2] = fmaf(f_new, x23[u][0], num[2] * f_old);
                    num[3] = fmaf(f_new, x23[u][1], num[3] * f_old);
                    den = fmaf(f_new, mlc[u][1], den * f_old);
                    m = m_new;
                }
            }
        }
        sw_half4_t res;
#pragma unroll
        for (int t = 0; t < 4; ++t) res[t] = (_Float16)(num[t] / den);   // round to nearest even
        *reinterpret_cast<sw_half4_t *>(reinterpret_cast<_Float16 *>(a.out) + rh * D + 4 * j4) = res;
    }
}

// Rows of requests with no cached position get +0; no chunk workgroup exists for
// them, so workgroup b < n_req looks after request b.  Called by every thread
// of such a workgroup before it looks for its own work item.
template <int D>
__device__ __forceinline__ void sw_fused_zero_rows(const SwArgs &a, int req)
{
    if (sw_request_len_flagged(a, req) != 0) return;      // has positions, or takes no part in the call
    sw_half4_t z = sw_half4_t{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    _Float16 *row = reinterpret_cast<_Float16 *>(a.out) + sw_q_row(a, req) * a.n_qh * D;
    for (int idx = threadIdx.x; idx < a.n_qh * (D / 4); idx += blockDim.x)
        *reinterpret_cast<sw_half4_t *>(row + 4 * idx) = z;
}
