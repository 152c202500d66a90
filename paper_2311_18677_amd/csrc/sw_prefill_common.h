// Pieces shared by the two prompt-phase (causal attention) kernels: operand
// types, the per-query online softmax and the second matrix product, both for a
// wave that owns 32 query positions (two 16-wide MFMA column blocks) of one head
// and works on tiles of 32 cached positions.  Lane (n16 = lane % 16, gq = lane / 16)
// owns query 16*nb + n16 of block nb and, of a tile's scores, positions
// 16*tb + 4*gq + i.
#pragma once
#include "sw_internal.h"
#include "sw_lane_ops.h"
#include "sw_worklist.h"

namespace sw_prefill {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int   kD         = 128;
constexpr int   kTile      = 32;             // cached positions per tile
constexpr int   kRowBytes  = 256;
constexpr int   kTileBytes = kTile * kRowBytes;       // 8192: one K or one V tile
constexpr int   kQPerWave  = 32;             // query positions per wave
constexpr float kNegBig    = -1.0e30f;

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (n < 64),
// leaving the other counters unconstrained; & 0xc07f adds "no LDS operation outstanding".
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

union Frag {
    uint4_t u;
    half8_t h;
};

// The running maximum of a query is only raised when a score exceeds it by more than
// this many binary orders of magnitude, and the accumulators are rescaled rarely instead
// of every tile.  Whether a raise is due is read off the sum of a lane's eight weights of
// a tile (no per-tile maximum): a sum of at most kSumBound = 8 * 2^kLazyBits changes
// nothing, so weights stay below 2^11 (exact enough in binary16, whose precision is
// relative); a larger sum means some score lies more than 2^kLazyBits above the maximum.
constexpr float kLazyBits = 8.0f;
constexpr float kSumBound = 8.0f * 256.0f;

// Query tokens of a request: with L cached positions and nq of them queries (the last
// nq; nq = L when no q_lens array is given), query index i is the token at position
// L - nq + i.
__device__ __forceinline__ int request_queries(const SwPrefillArgs &a, int r, int L)
{
    if (!a.q_lens) return L;
    const int cap = L < a.max_q ? L : a.max_q;
    int nq = a.q_lens[r];
    nq = nq < 0 ? 0 : (nq > cap ? cap : nq);
    // a request with a single query token is a token-phase request: when the call runs
    // those through the token-phase kernels, it is none of this kernel's business
    return (a.skip_single && nq == 1) ? 0 : nq;
}

// ---- workgroup -> (request, query block).  How many query blocks a request has depends
// on lengths only the device knows, so the grid is sized by a host-side bound and every
// wave finds its workgroup's item itself (no LDS, no barrier): items are numbered request
// by request, a request's late blocks (which see the most positions) first.  (When the
// bound is no smaller than requests x blocks-per-request anyway, the host asks for the
// direct mapping instead, which puts the late blocks of ALL requests first.)  A request
// owns one item per block of q_block query indices that holds a query whose row exists
// (rows outside [0, n_tokens) are never stored, so blocks of only such rows are no items).
struct QItem {
    int  r;            // request
    int  qb;           // query block: query indices qb * q_block ...
    int  L;            // cached positions of the request
    int  NQ;           // its query tokens (the last NQ positions)
    long long q_first; // row of its query index 0
    bool valid;        // false: nothing to do for this workgroup
};

__device__ __forceinline__ void request_span(const SwPrefillArgs &a, int r, int q_block, int &L, int &NQ,
                                             long long &q_first, int &qb_lo, int &cnt)
{
    L = a.seq_lens[r];
    q_first = a.q_starts[r];
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    NQ = request_queries(a, r, L);
    const long long lo = q_first < 0 ? -q_first : 0;                       // first query index with a row
    const long long room = a.n_tokens - q_first;
    const long long hi = room < (long long)NQ ? room : (long long)NQ;      // one past the last
    qb_lo = cnt = 0;
    if (hi > lo) {
        qb_lo = (int)(lo / q_block);
        cnt = (int)((hi - 1) / q_block) - qb_lo + 1;
    }
}

// Called by all 64 lanes of a wave; every wave of a workgroup gets the same answer.
__device__ __forceinline__ QItem find_item(const SwPrefillArgs &a, unsigned item, int q_block)
{
    QItem it;
    it.r = it.qb = it.L = it.NQ = 0;
    it.q_first = 0;
    it.valid = false;
    if (!a.compact) {
        // direct mapping: item = (n_qblocks - 1 - qb) * n_req + r, late blocks of all requests first
        const int r = (int)(item % (unsigned)a.n_req);
        int L = a.seq_lens[r];
        it.q_first = a.q_starts[r];          // read together with the length: one wait for both
        L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
        it.r = r;
        it.qb = a.n_qblocks - 1 - (int)(item / (unsigned)a.n_req);
        it.L = L;
        it.NQ = request_queries(a, r, L);
        it.valid = it.qb >= 0;
        return it;
    }
    const int lane = threadIdx.x & 63;
    const int per = (a.n_req + 63) >> 6;            // consecutive requests per lane
    int L = 0, NQ = 0, qb_lo = 0, cnt = 0, mine = 0;
    long long qf = 0;
    for (int j = 0; j < per; ++j) {
        const int r = lane * per + j;
        if (r < a.n_req) {
            request_span(a, r, q_block, L, NQ, qf, qb_lo, cnt);
            mine += cnt;
        }
    }
    const int incl = sw_wave_inclusive_scan(mine);
    const unsigned long long hit = __ballot((unsigned)incl > item);
    if (hit == 0) return it;                        // past the last item
    const int owner = __builtin_ctzll(hit);         // first lane whose requests reach the item
    unsigned before = (unsigned)__builtin_amdgcn_readlane(incl - mine, owner);
    int r = owner;
    if (per == 1) {
        L = __builtin_amdgcn_readlane(L, owner);
        NQ = __builtin_amdgcn_readlane(NQ, owner);
        qb_lo = __builtin_amdgcn_readlane(qb_lo, owner);
        cnt = __builtin_amdgcn_readlane(cnt, owner);
        const unsigned lo32 = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(unsigned long long)qf, owner);
        const unsigned hi32 = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)qf >> 32), owner);
        qf = (long long)(((unsigned long long)hi32 << 32) | lo32);
    } else {
        // walk the owner lane's requests again (wave-uniform loads, served from cache)
        cnt = 0;
        for (int j = 0; j < per; ++j) {
            before += (unsigned)cnt;
            r = min(owner * per + j, a.n_req - 1);
            request_span(a, r, q_block, L, NQ, qf, qb_lo, cnt);
            if (before + (unsigned)cnt > item) break;
        }
    }
    const unsigned local = item - before;
    if (local >= (unsigned)cnt) return it;          // cannot happen when the scan is right
    // wave-uniform by construction; say so, so that everything derived stays in scalar registers
    it.r = __builtin_amdgcn_readfirstlane(r);
    it.qb = __builtin_amdgcn_readfirstlane(qb_lo + cnt - 1 - (int)local);
    it.L = __builtin_amdgcn_readfirstlane(L);
    it.NQ = __builtin_amdgcn_readfirstlane(NQ);
    const unsigned lo32 = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(unsigned long long)qf);
    const unsigned hi32 = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)qf >> 32));
    it.q_first = (long long)(((unsigned long long)hi32 << 32) | lo32);
    it.valid = true;
    return it;
}

// Q^T operands of a wave: lane (n16, gq) holds dims 32kk + 8gq .. +7 of the query with
// index q0 + 16nb + n16 (of nq).  Indices past the last query repeat it (never stored);
// row indices are clamped into [0, n_tokens).
__device__ __forceinline__ void load_q(const SwPrefillArgs &a, long long q_first, int q0, int nq, int h,
                                       int n16, int gq, Frag (&qreg)[2][4])
{
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        int qpos = q0 + 16 * nb + n16;
        qpos = qpos < nq ? qpos : nq - 1;
        long long row = q_first + qpos;
        row = row < 0 ? 0 : (row >= a.n_tokens ? a.n_tokens - 1 : row);
        const uint16_t *src = a.q + (row * a.n_qh + h) * kD + 8 * gq;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qreg[nb][kk].u = *reinterpret_cast<const uint4_t *>(src + 32 * kk);
    }
}

// S^T = K Q^T for one tile staged at kb (rows XOR-swizzled by 16-byte piece):
// two 16-position blocks x two 16-query blocks, four 32-dim steps.
__device__ __forceinline__ void qk_tile(const unsigned char *kb, const Frag (&qreg)[2][4], int n16, int gq,
                                        float4_t (&sacc)[2][2])
{
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int tb = 0; tb < 2; ++tb) sacc[nb][tb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int off = n16 * kRowBytes + (((4 * kk + gq) ^ n16) << 4);   // row n16, piece 4kk+gq
        Frag k0, k1;
        k0.u = *reinterpret_cast<const uint4_t *>(kb + off);
        k1.u = *reinterpret_cast<const uint4_t *>(kb + 16 * kRowBytes + off);
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            sacc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k0.h, qreg[nb][kk].h, sacc[nb][0], 0, 0, 0);
            sacc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k1.h, qreg[nb][kk].h, sacc[nb][1], 0, 0, 0);
        }
    }
}

// The same product in two steps, so that work of the two query blocks can be interleaved:
// the K operands of a tile (both 16-position blocks, four 32-dim steps) ...
__device__ __forceinline__ void load_k_ops(const unsigned char *kb, int n16, int gq, Frag (&kop)[2][4])
{
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int off = n16 * kRowBytes + (((4 * kk + gq) ^ n16) << 4);
        kop[0][kk].u = *reinterpret_cast<const uint4_t *>(kb + off);
        kop[1][kk].u = *reinterpret_cast<const uint4_t *>(kb + 16 * kRowBytes + off);
    }
}

// ... and S^T of one query block from them.
__device__ __forceinline__ void qk_block(int nb, const Frag (&kop)[2][4], const Frag (&qreg)[2][4],
                                         float4_t (&sacc)[2][2])
{
    sacc[nb][0] = float4_t{0.f, 0.f, 0.f, 0.f};
    sacc[nb][1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        sacc[nb][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kop[0][kk].h, qreg[nb][kk].h, sacc[nb][0], 0, 0, 0);
        sacc[nb][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kop[1][kk].h, qreg[nb][kk].h, sacc[nb][1], 0, 0, 0);
    }
}

typedef short short4_t __attribute__((ext_vector_type(4)));
typedef short4_t __attribute__((address_space(3))) *lds_short4_ptr;

// A staged V row keeps its sixteen 16-byte pieces XOR-swizzled by row, in pairs:
// piece p of row rho sits in slot p ^ v_swizzle(rho).  (Pairs, because the transposing
// read below takes 8 bytes per lane and two neighbouring lanes share a piece.)
__device__ __forceinline__ int v_swizzle(int rho) { return (rho & 7) << 1; }

// Byte offsets, inside a staged V tile, of this lane's sixteen transposing reads: entry
// [hk][e] serves keys 16hk + 4gq .. +3 and dims 16e .. 16e+15.  They depend on the lane
// only, so a kernel computes them once.
__device__ __forceinline__ void vt_offsets(int n16, int gq, unsigned (&off)[8])
{
    // rows 4gq + n16/4 (keys 0..15 of the tile); the rows 16 further on (keys 16..31) share
    // the swizzle and lie exactly 16 rows = 4096 bytes behind: an immediate offset of the read
    const int rho = 4 * gq + (n16 >> 2);                      // the row whose 8 bytes this lane addresses
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int piece = 2 * e + ((n16 >> 1) & 1);           // dims 16e + 4(n16 % 4) .. +3 live in this piece
        off[e] = (unsigned)(rho * kRowBytes + ((piece ^ v_swizzle(rho)) << 4) + 8 * (n16 & 1));
    }
}

// V^T operands of the second product straight from LDS with the transposing read of
// gfx950 (ds_read_b64_tr_b16).  Within 16 lanes, result j of lane l is element l % 4 of
// the 8 bytes that lane 4j + l / 4 addresses; with the addresses of vt_offsets lane
// (n16, gq) therefore receives V[key 16hk + 4gq + j][dim 16e + n16], j = 0..3 -- exactly
// the A operand (row = dim 16e + n16, k-slots = the keys this lane group's P operand
// holds).  Block e covers dims 16e .. 16e+15 (row = MFMA row).
__device__ __forceinline__ void load_vt(const unsigned char *vb, const unsigned (&off)[8], Frag (&va)[8])
{
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int hk = 0; hk < 2; ++hk) {
            union { short4_t s; unsigned int u[2]; } x;
            x.s = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(vb + off[e] + hk * 16 * kRowBytes));
            va[e].u[2 * hk] = x.u[0];
            va[e].u[2 * hk + 1] = x.u[1];
        }
}

// Online softmax of one tile, base 2, for both query blocks.  m[] is kept in raw score
// units; the scale enters through one fused multiply-add.  `diagonal`: some position of
// the tile is later than some query of the wave (q0 = the wave's first query, t0 = the
// tile's first position).
__device__ __forceinline__ void softmax_block(int nb, const float4_t (&sacc)[2][2], bool diagonal, int q0, int t0,
                                              int n16, int gq, float scale_log2e, float lazy_raw,
                                              float (&m)[2], float4_t (&l)[2], float4_t (&o)[2][8], Frag (&p)[2])
{
    {
        float s[8];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 4; ++i) s[4 * tb + i] = sacc[nb][tb][i];
        if (diagonal) {
            const int qpos = q0 + 16 * nb + n16;
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (t0 + 16 * tb + 4 * gq + i > qpos) s[4 * tb + i] = -INFINITY;
        }
        // Optimistic pass: weights against the running maximum as it stands.  While every
        // lane's eight weights sum to at most 8 * 2^kLazyBits nothing has to change -- no
        // weight exceeds that bound (fine for binary16, whose precision is relative) and the
        // tile's own maximum is never needed.  A larger (or infinite, or NaN) sum in any
        // lane sends the whole wave through the exact pass below; sums above the bound
        // imply a score more than 2^kLazyBits above the maximum, so that pass raises it.
        float neg_m = -m[nb] * scale_log2e;
        float pj[8];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            pj[j] = __builtin_amdgcn_exp2f(fmaf(s[j], scale_log2e, neg_m));
            psum += pj[j];
        }
        if (__builtin_amdgcn_ballot_w64(!(psum <= kSumBound)) != 0) {       // rare after the first tiles
            float mt = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                             fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
            mt = quad_rows_max(mt);
            const bool raise = mt > m[nb] + lazy_raw;
            const float m_new = raise ? mt : m[nb];
            const float alpha = __builtin_amdgcn_exp2f((m[nb] - m_new) * scale_log2e);
            m[nb] = m_new;
            l[nb] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[nb][e] *= alpha;
            neg_m = -m[nb] * scale_log2e;
            psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pj[j] = __builtin_amdgcn_exp2f(fmaf(s[j], scale_log2e, neg_m));
                psum += pj[j];
            }
        }
        // (psum only decides whether the maximum must be raised; the sum that normalises the
        // row is taken from the rounded weights, by the matrix cores, in pv_block)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const half2_t h2 = __builtin_convertvector((float2_t){pj[2 * j], pj[2 * j + 1]}, half2_t);
            p[nb].h[2 * j] = h2[0];
            p[nb].h[2 * j + 1] = h2[1];
        }
    }
}

__device__ __forceinline__ void softmax_tile(const float4_t (&sacc)[2][2], bool diagonal, int q0, int t0,
                                             int n16, int gq, float scale_log2e, float lazy_raw,
                                             float (&m)[2], float4_t (&l)[2], float4_t (&o)[2][8], Frag (&p)[2])
{
    softmax_block(0, sacc, diagonal, q0, t0, n16, gq, scale_log2e, lazy_raw, m, l, o, p);
    softmax_block(1, sacc, diagonal, q0, t0, n16, gq, scale_log2e, lazy_raw, m, l, o, p);
}

// O^T += V^T P^T for one query block, and the sum of the same weights: one more product with
// an all-ones operand leaves, in every element of l[nb], the tile's sum over ALL 32 keys of
// the binary16 weights of query n16.  Numerator and denominator of a row are thus built from
// the same rounded weights, w~_i = w_i (1 + d_i): the row's error is sum_i w_i d_i (v_i - out),
// which vanishes where one key dominates (its v is the row) -- with the exact sum as
// denominator it would be sum_i w_i d_i v_i, up to 2^-11 |v| for such a row, which alone
// exceeds the error bound once |v| reaches 4.
__device__ __forceinline__ void pv_block(int nb, const Frag (&va)[8], const Frag (&p)[2], float4_t (&o)[2][8],
                                         float4_t (&l)[2])
{
    Frag ones;
    ones.u = uint4_t{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};      // eight binary16 ones
#pragma unroll
    for (int e = 0; e < 8; ++e)
        o[nb][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va[e].h, p[nb].h, o[nb][e], 0, 0, 0);
    l[nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones.h, p[nb].h, l[nb], 0, 0, 0);
}

}  // namespace sw_prefill
