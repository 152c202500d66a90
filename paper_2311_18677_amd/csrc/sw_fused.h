// Single-launch form of the split over context length: one of the workgroups of a
// (request, key/value head, head tile) unit merges the unit's chunks itself, so the
// token-phase step (paper sections 2.2 and 3.5) is one kernel, not two.
//
// The chunks' partial results cross workgroups that sit on different XCDs, whose L2
// caches are not coherent with each other.  No fence and no store acknowledgement is
// waited for.  Instead the data validates itself: a partial result travels as 16-byte
// pieces, each holding three floats and a 32-bit tag, written with one device-coherent
// 16-byte store and read back with device-coherent 16-byte loads (both served at the
// memory side, past the L2s).  A piece is taken only when its tag is the one this call
// of this unit uses; anything else is a piece of an earlier call whose replacement has
// not landed yet, and the reader asks again.
//
//   tag = the unit's epoch + 1
//
// The epoch is a per-unit counter in device memory that the merging workgroup advances
// at the end of every call, so the tags a unit writes grow from call to call (a HIP graph
// replays the same kernel arguments, hence the counter lives on the device).  Every
// workspace geometry -- (n_kvh, group, n_chunks, head_dim, kernel) decide where a slot lies
// and which unit owns it -- has a block of unit states and pieces of its own, so a piece is only ever overwritten by the
// same unit's same chunk and head.  Blocks start zeroed and no tag is zero.  (The tag wraps
// after 2^32 merges of one unit; a stale piece could only pass for a fresh one if it had
// been written exactly a multiple of 2^32 merges earlier and not since.)
//
// The thread that owns dims 4*j4 .. 4*j4+3 of a head writes two pieces per chunk:
//   piece A (index j4)      = { o[4*j4], o[4*j4+1], o[4*j4+2], tag }
//   piece B (index 32 + j4) = { o[4*j4+3], m, l, tag }        (D = 128; 16 + j4 for D = 64)
// so the chunk's (m, l) ride along with every thread's own data, each store instruction of a
// wave covers whole 128-byte lines, and a (chunk, head) slot is D / 2 pieces = 8 * D bytes.
//
// Who merges: every workgroup of a unit with more than one chunk takes a ticket from the
// unit's counter once its tiles are done, and sends its pieces while the answer travels; the
// holder of the last ticket merges.  All other workgroups of the unit have then taken
// theirs and sent their pieces, without waiting for anything, so the merging workgroup waits
// for stores that are already on their way (the wait is bounded anyway, and a device-side
// flag records a give-up).  It requests the pieces of up to 16 chunks at
// once (one round trip to the memory side), folds chunks 0 .. nc-1 in index order with a
// running maximum -- its own chunk from registers -- so the bits of a row do not depend on
// which workgroup merged, and writes the binary16 rows.
#pragma once
#include "sw_internal.h"

typedef float sw_float4_t __attribute__((ext_vector_type(4)));
typedef float sw_float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 sw_half4_t __attribute__((ext_vector_type(4)));
typedef unsigned int sw_uint4_t __attribute__((ext_vector_type(4)));

constexpr int kSwSpinMax = 1 << 20;           // re-reads of a batch before the merge gives up

// What a workgroup knows about its part in the single-launch merge.
struct SwFused {
    __amdgpu_buffer_rsrc_t ws;                // the pieces as a raw buffer
    unsigned tag;                             // this call's tag of this unit
    int  nc;                                  // chunks of the unit
    int  c;                                   // this workgroup's chunk
    bool merger;                              // this workgroup folds the chunks
};

// Byte offset of piece p of the (chunk, head) slot; consecutive chunks of a unit are
// group slots apart.
template <int D>
__device__ __forceinline__ unsigned sw_piece_offset(const SwArgs &a, int r, int g, int c, int hh, int p)
{
    return (unsigned)((sw_ws_slot(a, r, g, c, hh) * (D / 2) + p) * 16);
}

// Device-coherent 16-byte accesses (cache policy sc1: served past the L2s).
__device__ __forceinline__ void sw_piece_store(const SwFused &f, unsigned off, float x, float y, float z)
{
    __builtin_amdgcn_raw_buffer_store_b128(
        sw_uint4_t{__float_as_uint(x), __float_as_uint(y), __float_as_uint(z), f.tag}, f.ws, off, 0, 16);
}

// (soff: a wave-uniform byte offset added to off)
__device__ __forceinline__ sw_uint4_t sw_piece_load(const SwFused &f, unsigned off, unsigned soff)
{
    return __builtin_amdgcn_raw_buffer_load_b128(f.ws, off, soff, 16);
}

// The tag a unit uses in this call, from its epoch (read through the constant address
// space: the word was last written before this kernel started).
__device__ __forceinline__ void sw_fused_begin(const SwArgs &a, SwFused &f, long long unit)
{
    typedef const __attribute__((address_space(4))) unsigned *const_u32_t;
    f.tag = *(const_u32_t)(&a.units[unit].epoch) + 1u;
    if (f.tag == 0u) f.tag = 1u;              // zero marks a piece that was never written
    // the epoch has been read by here, i.e. before this workgroup can take its ticket: the
    // merging workgroup advances it once every ticket of the unit is taken
    asm volatile("" : "+s"(f.tag));
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
    __hip_atomic_fetch_add(&a.units[unit].epoch, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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

// Running-maximum state of one thread's four dims while it folds the chunks.
struct SwFold {
    float m, den;
    sw_float4_t num;
};

// Chunks c0 .. c0+B-1 (as far as they exist) into the fold: their pieces are requested
// together and asked for again until every one carries the tag; the thread's own chunk
// comes from its registers.
template <int D, int B>
__device__ __forceinline__ void sw_fold_chunks(const SwArgs &a, const SwFused &f, SwFold &s, int c0,
                                               unsigned off_a, unsigned off_b, unsigned chunk_stride,
                                               sw_float4_t num, float den, float mx)
{
    sw_uint4_t pa[B], pb[B];
    bool ok = false;
    for (int spin = 0; spin < kSwSpinMax && !ok; ++spin) {
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const unsigned soff = (unsigned)min(c0 + u, f.nc - 1) * chunk_stride;   // clamped: in bounds, unused past nc
            pa[u] = sw_piece_load(f, off_a, soff);
            pb[u] = sw_piece_load(f, off_b, soff);
        }
        asm volatile("" ::: "memory");               // every round reads memory again
        if (spin) __builtin_amdgcn_s_sleep(4);       // a piece was late: do not crowd the memory side
        ok = true;
#pragma unroll
        for (int u = 0; u < B; ++u)
            if (c0 + u < f.nc && c0 + u != f.c) ok = ok && pa[u][3] == f.tag && pb[u][3] == f.tag;
    }
    if (!ok) *a.dev_err = 1u;                        // gave up on a piece: the row is wrong, the kernel ends
#pragma unroll
    for (int u = 0; u < B; ++u) {
        if (c0 + u >= f.nc) continue;
        const bool own = c0 + u == f.c;
        const float mc = own ? mx : __uint_as_float(pb[u][1]);
        const float lc = own ? den : __uint_as_float(pb[u][2]);
        const sw_float4_t x = own ? num
                                  : sw_float4_t{__uint_as_float(pa[u][0]), __uint_as_float(pa[u][1]),
                                                __uint_as_float(pa[u][2]), __uint_as_float(pb[u][0])};
        const float m_new = fmaxf(s.m, mc);
        const float f_old = __builtin_amdgcn_exp2f(s.m - m_new);
        const float f_new = __builtin_amdgcn_exp2f(mc - m_new);
#pragma unroll
        for (int t = 0; t < 4; ++t) s.num[t] = fmaf(f_new, x[t], s.num[t] * f_old);
        s.den = fmaf(f_new, lc, s.den * f_old);
        s.m = m_new;
    }
}

// Called by the thread that holds dims 4*j4 .. 4*j4+3 of head hh (within the group) of
// this workgroup's chunk: num = sum_t 2^(s_t - mx) V_t over the chunk, den the sum of the
// weights, mx the chunk's maximum (base-2 exponent units).  Sends the thread's two pieces.
template <int D>
__device__ __forceinline__ void sw_fused_send(const SwArgs &a, const SwFused &f, int r, int g, int hh, int j4,
                                              sw_float4_t num, float den, float mx)
{
    const unsigned off = sw_piece_offset<D>(a, r, g, f.c, hh, j4);
    sw_piece_store(f, off, num[0], num[1], num[2]);
    sw_piece_store(f, off + (D / 4) * 16, num[3], mx, den);
}

// The merging workgroup's thread for the same dims: folds the unit's chunks (its own from
// the values it sent) and stores the output row's four dims.
template <int D>
__device__ __forceinline__ void sw_fused_fold(const SwArgs &a, const SwFused &f, int r, int g, int hh, int j4,
                                              sw_float4_t num, float den, float mx)
{
    const unsigned off_a = sw_piece_offset<D>(a, r, g, 0, hh, j4);
    const unsigned off_b = off_a + (D / 4) * 16;
    const unsigned chunk_stride = (unsigned)a.group * (D / 2) * 16;
    SwFold s;
    s.m = -1.0e30f;
    s.den = 0.f;
    s.num = sw_float4_t{0.f, 0.f, 0.f, 0.f};
    if (f.nc <= 4) {
        sw_fold_chunks<D, 4>(a, f, s, 0, off_a, off_b, chunk_stride, num, den, mx);
    } else if (f.nc <= 8) {
        sw_fold_chunks<D, 8>(a, f, s, 0, off_a, off_b, chunk_stride, num, den, mx);
    } else {
        for (int c0 = 0; c0 < f.nc; c0 += 16)
            sw_fold_chunks<D, 16>(a, f, s, c0, off_a, off_b, chunk_stride, num, den, mx);
    }
    sw_store_final4<D>(a, sw_q_row(a, r) * a.n_qh + g * a.group + hh, j4, s.num, s.den);
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
