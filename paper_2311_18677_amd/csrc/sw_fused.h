// Single-launch form of the split over context length: one of the workgroups of a
// (request, key/value head, head tile) unit merges the unit's chunks itself, so the
// token-phase step (paper sections 2.2 and 3.5) is one kernel, not two.
//
// The chunks' partial results cross workgroups that sit on different XCDs, whose L2
// caches are not coherent with each other.  No fence and no store acknowledgement is
// waited for.  Instead the data validates itself: a partial result travels as 16-byte
// pieces, each holding two floats and a 64-bit tag, written with one device-coherent
// 16-byte store and read back with device-coherent 16-byte loads (both served at the
// memory side, past the L2s).  A piece is taken only when its tag is the one this call
// of this unit uses; anything else is a piece of an earlier call whose replacement has
// not landed yet, and the reader asks again.
//
//   tag = geometry id (20 bits) | the unit's epoch + 1 (44 bits)
//
// The epoch is a per-unit counter in device memory that the merging workgroup advances
// at the end of every call, so tags written by one unit under one geometry grow from call
// to call (a HIP graph replays the same kernel arguments, hence the counter lives on the
// device); the geometry id changes whenever a call lays the workspace out differently
// from the call before it, so pieces left by another shape never carry a live tag.
// The workspace starts zeroed and no tag is zero.
//
// Who merges: every workgroup of a unit with more than one chunk takes a ticket from the
// unit's counter when its last tile is under way; the holder of the last ticket merges.
// All other workgroups of the unit have then taken theirs, i.e. are inside their last
// tile or past it: they store their pieces without waiting for anything, so the merging
// workgroup waits for stores that are already on their way (the wait is bounded anyway,
// and a device-side flag records a give-up).  It folds chunks 0 .. nc-1 in index order
// with a running maximum -- its own chunk from registers -- so the bits of a row do not
// depend on which workgroup merged, and writes the binary16 rows.
#pragma once
#include "sw_internal.h"

typedef float sw_float4_t __attribute__((ext_vector_type(4)));
typedef float sw_float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 sw_half4_t __attribute__((ext_vector_type(4)));
typedef unsigned int sw_uint4_t __attribute__((ext_vector_type(4)));

constexpr int kSwEpochBits = 44;
constexpr int kSwFusedBatch = 4;              // chunks whose pieces a thread requests together
constexpr int kSwSpinMax = 1 << 20;           // re-reads of a batch before the merge gives up

// What a workgroup knows about its part in the single-launch merge.
struct SwFused {
    __amdgpu_buffer_rsrc_t ws;                // the tagged workspace as a raw buffer
    unsigned tag_lo, tag_hi;                  // this call's tag of this unit
    int  nc;                                  // chunks of the unit
    int  c;                                   // this workgroup's chunk
    bool merger;                              // this workgroup folds the chunks
};

// Pieces of one (chunk, head) slot: D/2 pieces of two output dims, then (m, l).
template <int D>
__device__ __forceinline__ unsigned sw_piece_offset(const SwArgs &a, int r, int g, int c, int hh, int p)
{
    return (unsigned)((sw_ws_slot(a, r, g, c, hh) * (D / 2 + 1) + p) * 16);
}

// Device-coherent 16-byte accesses (cache policy sc1: served past the L2s).
__device__ __forceinline__ void sw_piece_store(const SwFused &f, unsigned off, float x, float y)
{
    __builtin_amdgcn_raw_buffer_store_b128(
        sw_uint4_t{__float_as_uint(x), __float_as_uint(y), f.tag_lo, f.tag_hi}, f.ws, off, 0, 16);
}

__device__ __forceinline__ sw_uint4_t sw_piece_load(const SwFused &f, unsigned off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(f.ws, off, 0, 16);
}

// The tag a unit uses in this call, from its epoch (read through the constant address
// space: the word was last written before this kernel started).
__device__ __forceinline__ void sw_fused_begin(const SwArgs &a, SwFused &f, long long unit)
{
    typedef const __attribute__((address_space(4))) unsigned long long *const_u64_t;
    const unsigned long long epoch = *(const_u64_t)(&a.units[unit].epoch);
    const unsigned long long tag = ((unsigned long long)a.geometry << kSwEpochBits) |
                                   ((epoch + 1) & ((1ull << kSwEpochBits) - 1));
    f.tag_lo = (unsigned)tag;
    f.tag_hi = (unsigned)(tag >> 32);
    // the epoch has been read by here, i.e. before this workgroup can take its ticket: the
    // merging workgroup advances it once every ticket of the unit is taken
    asm volatile("" : "+s"(f.tag_lo), "+s"(f.tag_hi));
    f.ws = __builtin_amdgcn_make_buffer_rsrc(a.ws_tag, 0, (int)a.ws_tag_bytes, 0x00020000);
}

// One lane takes the unit's ticket (the answer may be left in flight) ...
__device__ __forceinline__ unsigned sw_fused_ticket(const SwArgs &a, long long unit)
{
    return __hip_atomic_fetch_add(&a.units[unit].ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ... and the same lane reads it later: true for the workgroup that merges, which also
// leaves the counter at zero and the epoch advanced for the next call.  (Both are read
// again only by the next kernel on the stream.)
__device__ __forceinline__ bool sw_fused_is_merger(const SwArgs &a, long long unit, unsigned ticket, int nc)
{
    if (ticket != (unsigned)(nc - 1)) return false;
    __hip_atomic_store(&a.units[unit].ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_fetch_add(&a.units[unit].epoch, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// Binary16 output of four dims (round to nearest even).
template <int D>
__device__ __forceinline__ void sw_store_final4(const SwArgs &a, long long rh, int j4, sw_float4_t num, float den)
{
    sw_half4_t res;
#pragma unroll
    for (int t = 0; t < 4; ++t) res[t] = (_Float16)(num[t] / den);   // round to nearest even
    *reinterpret_cast<sw_half4_t *>(reinterpret_cast<_Float16 *>(a.out) + rh * D + 4 * j4) = res;
}

// Called by the thread that holds dims 4*j4 .. 4*j4+3 of head hh (within the group) of
// this workgroup's chunk: num = sum_t 2^(s_t - mx) V_t over the chunk, den the sum of the
// weights, mx the chunk's maximum (base-2 exponent units).
//   not the merging workgroup: stores its pieces and is done;
//   the merging workgroup: folds the unit's chunks and stores the output row's four dims.
template <int D>
__device__ __forceinline__ void sw_fused_finish(const SwArgs &a, const SwFused &f, int r, int g, int hh, int j4,
                                                sw_float4_t num, float den, float mx)
{
    constexpr int P = D / 2;                  // index of the (m, l) piece
    if (!f.merger) {
        const unsigned off = sw_piece_offset<D>(a, r, g, f.c, hh, 2 * j4);
        sw_piece_store(f, off, num[0], num[1]);
        sw_piece_store(f, off + 16, num[2], num[3]);
        if (j4 == 0) sw_piece_store(f, sw_piece_offset<D>(a, r, g, f.c, hh, P), mx, den);
        return;
    }
    float m_run = -1.0e30f, d_run = 0.f;
    sw_float4_t n_run = sw_float4_t{0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < f.nc; c0 += kSwFusedBatch) {
        sw_uint4_t lo[kSwFusedBatch], hi[kSwFusedBatch], ml[kSwFusedBatch];
        bool ok = false;
        for (int spin = 0; spin < kSwSpinMax && !ok; ++spin) {
#pragma unroll
            for (int u = 0; u < kSwFusedBatch; ++u) {
                const int c = min(c0 + u, f.nc - 1);     // clamped: in bounds, unused past nc
                const unsigned off = sw_piece_offset<D>(a, r, g, c, hh, 2 * j4);
                lo[u] = sw_piece_load(f, off);
                hi[u] = sw_piece_load(f, off + 16);
                ml[u] = sw_piece_load(f, sw_piece_offset<D>(a, r, g, c, hh, P));
            }
            asm volatile("" ::: "memory");               // every round reads memory again
            ok = true;
#pragma unroll
            for (int u = 0; u < kSwFusedBatch; ++u) {
                if (c0 + u >= f.nc || c0 + u == f.c) continue;
                ok = ok && lo[u][2] == f.tag_lo && lo[u][3] == f.tag_hi &&
                           hi[u][2] == f.tag_lo && hi[u][3] == f.tag_hi &&
                           ml[u][2] == f.tag_lo && ml[u][3] == f.tag_hi;
            }
        }
        if (!ok) *a.dev_err = 1u;                        // gave up on a piece: the row is wrong, the kernel ends
#pragma unroll
        for (int u = 0; u < kSwFusedBatch; ++u) {
            if (c0 + u >= f.nc) continue;
            const bool own = c0 + u == f.c;
            const float mc = own ? mx : __uint_as_float(ml[u][0]);
            const float lc = own ? den : __uint_as_float(ml[u][1]);
            const sw_float4_t x = own ? num
                                      : sw_float4_t{__uint_as_float(lo[u][0]), __uint_as_float(lo[u][1]),
                                                    __uint_as_float(hi[u][0]), __uint_as_float(hi[u][1])};
            const float m_new = fmaxf(m_run, mc);
            const float f_old = __builtin_amdgcn_exp2f(m_run - m_new);
            const float f_new = __builtin_amdgcn_exp2f(mc - m_new);
#pragma unroll
            for (int t = 0; t < 4; ++t) n_run[t] = fmaf(f_new, x[t], n_run[t] * f_old);
            d_run = fmaf(f_new, lc, d_run * f_old);
            m_run = m_new;
        }
    }
    sw_store_final4<D>(a, sw_q_row(a, r) * a.n_qh + g * a.group + hh, j4, n_run, d_run);
}

// A row of +0 for every query head of a request with no cached position (no item exists
// for such a request).  Called by every thread of the workgroup that looks after it.
template <int D>
__device__ __forceinline__ void sw_zero_rows(const SwArgs &a, int req)
{
    sw_half4_t z = sw_half4_t{(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
    _Float16 *row = reinterpret_cast<_Float16 *>(a.out) + sw_q_row(a, req) * a.n_qh * D;
    for (int idx = threadIdx.x; idx < a.n_qh * (D / 4); idx += blockDim.x)
        *reinterpret_cast<sw_half4_t *>(row + 4 * idx) = z;
}
