// Prompt-phase (causal) attention on the matrix cores (gfx950, wave64),
// head_dim 128, up to 8 query heads per key/value head.
//
// The prompt phase processes all tokens of a prompt in one pass (paper section
// 2.2) and is compute bound (section 3.5, Insight V): prompt token i attends to
// cached positions 0..i.  One workgroup takes one (request, key/value head) and a
// block of query positions; every wave owns 32 query positions of one query
// head, so no result is ever merged across waves.  K and V tiles of 32 positions
// travel global->LDS once per workgroup (three buffers, two tiles in flight) and
// are shared by all waves; the contractions are the ones of the token-phase
// kernel with the query position, not the head, on the 16-wide N axis:
//
//   S^T = K Q^T   A = K rows from LDS (swizzled), B = Q^T kept in registers
//   O^T += V^T P^T   A = V^T built in registers from V rows, B = P^T (binary16)
//
// Each lane therefore owns one query position: its running maximum, its sum and
// its causal bound are per-lane scalars, and its output row is stored straight
// from the accumulators.
#include "sw_internal.h"

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

constexpr int   kD         = 128;
constexpr int   kTile      = 32;             // cached positions per tile
constexpr int   kRowBytes  = 256;
constexpr int   kTileBytes = kTile * kRowBytes;       // 8192: one K or one V tile
constexpr int   kBufBytes  = 2 * kTileBytes;          // K tile, then V tile
constexpr int   kBufs      = 3;
constexpr int   kQPerWave  = 32;             // query positions per wave (two MFMA column blocks)
constexpr float kNegBig    = -1.0e30f;

constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

union Frag {
    uint4_t u;
    half8_t h;
};

typedef float float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// Lanes n16, n16+16, n16+32, n16+48 hold parts of one query's row.  Two swap
// instructions give every one of them the maximum (or the sum) over the four:
// the first exchanges odd rows of 16 lanes with even ones, the second the upper
// 32 lanes with the lower.
__device__ __forceinline__ float quad_rows_max(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float quad_rows_sum(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// The running maximum of a query is only raised when a score exceeds it by more than
// this many binary orders of magnitude: weights then stay below 2^kLazyBits (exact
// enough in binary16, whose precision is relative) and the accumulators are rescaled
// rarely instead of every tile.
constexpr float kLazyBits = 8.0f;

// NW = waves per workgroup = (query heads per workgroup) * (waves per head).
template <int NW>
__global__ __launch_bounds__(64 * NW, 1)
void sw_prefill_mfma_kernel(SwPrefillArgs a)
{
    // a tile's 16 one-kilobyte load instructions are dealt round-robin to the waves;
    // every wave issues C of them per tile (the last may repeat instruction 15)
    constexpr int C = (16 + NW - 1) / NW;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kBufs * kBufBytes];

    // blockIdx -> (query block, request, key/value head, block of hp query heads)
    const unsigned n_hb = (unsigned)(a.group / a.hp);
    const unsigned hb = blockIdx.x % n_hb;
    const unsigned rest = blockIdx.x / n_hb;
    const unsigned n_units = (unsigned)a.n_req * (unsigned)a.n_kvh;
    const unsigned unit = rest % n_units;
    // late query blocks see the most positions: they come first in dispatch order
    const int qb = a.n_qblocks - 1 - (int)(rest / n_units);
    const int r = (int)(unit / (unsigned)a.n_kvh);
    const int g = (int)(unit - (unsigned)r * (unsigned)a.n_kvh);
    int L = a.seq_lens[r];
    const long long q_first = a.q_starts[r];     // read together with the length: one wait for both
    L = L < 0 ? 0 : (L > a.max_len ? a.max_len : L);
    const int q_block = kQPerWave * a.qw;        // query positions per workgroup
    const int Q0 = qb * q_block;
    if (Q0 >= L) return;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n16  = lane & 15;
    const int gq   = lane >> 4;
    const int hh   = (int)hb * a.hp + wave % a.hp;   // query head within the group
    const int sb   = wave / a.hp;                // which 32 query positions of the block
    const int qw0  = Q0 + kQPerWave * sb;
    const int h    = g * a.group + hh;

    // The staging area is filled by global->LDS loads only; one ordinary store keeps
    // the compiler from treating it as never written.
    *reinterpret_cast<uint4_t *>(lds + threadIdx.x * 16) = uint4_t{0u, 0u, 0u, 0u};
    __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0): the store is done before any load lands
    __builtin_amdgcn_s_barrier();

    const char *kslab = reinterpret_cast<const char *>(a.k) + 2 * ((long long)r * a.stride_req + (long long)g * a.stride_kvh);
    const char *vslab = reinterpret_cast<const char *>(a.v) + 2 * ((long long)r * a.stride_req + (long long)g * a.stride_kvh);

    // tiles the workgroup walks: up to its last query position, within the prompt
    const int last_q = min(Q0 + q_block, L) - 1;
    const int n_tiles = last_q / kTile + 1;
    // tiles this wave computes on: up to its own last query position
    const int my_tiles = qw0 < L ? qw0 / kTile + 1 : 0;

    // this wave's share of tile ti's loads -> buffer ti % 3.  Instruction j < 8 is K rows
    // 4j .. 4j+3 (16-byte pieces XOR-swizzled by row), j >= 8 is V rows 4(j-8) .. +3.
    auto issue_tile = [&](int ti) {
        unsigned char *buf = lds + (ti % kBufs) * kBufBytes;
        const int t0 = ti * kTile;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            int j = wave + NW * c;
            j = j < 16 ? j : 15;
            const int n = j & 7;
            const bool is_v = j >= 8;
            const int rho = 4 * n + gq;
            const int t = min(t0 + rho, L - 1);                      // rows past the prompt repeat its last row
            const int piece = is_v ? n16 : (n16 ^ (rho & 15));
            const char *src = (is_v ? vslab : kslab) + (((unsigned)t << 8) | (unsigned)(piece << 4));
            __builtin_amdgcn_global_load_lds(src, buf + (is_v ? kTileBytes : 0) + n * 1024, 16, 0, 0);
        }
    };

    float m[2] = {kNegBig, kNegBig}, l[2] = {0.f, 0.f};
    const float lazy_raw = kLazyBits / a.scale_log2e;      // the threshold in raw score units
    float4_t o[2][8];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[nb][e] = float4_t{0.f, 0.f, 0.f, 0.f};

    issue_tile(0);
    if (n_tiles > 1) issue_tile(1);

    // ---- Q^T operands: lane (n16, gq) holds dims 32kk + 8gq .. +7 of query qw0 + 16nb + n16.
    // Requested after the first tiles so that both latencies overlap; awaited here, once,
    // so that no wait inside the loop has to cover them.
    Frag qreg[2][4];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        int qpos = qw0 + 16 * nb + n16;
        qpos = qpos < L ? qpos : L - 1;          // rows past the prompt repeat its last row (never stored)
        long long row = q_first + qpos;
        row = row < 0 ? 0 : (row >= a.n_tokens ? a.n_tokens - 1 : row);
        const uint16_t *src = a.q + (row * a.n_qh + h) * kD + 8 * gq;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qreg[nb][kk].u = *reinterpret_cast<const uint4_t *>(src + 32 * kk);
    }

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

    for (int ti = 0; ti < n_tiles; ++ti) {
        // this wave's loads of tile ti have landed (those of tile ti + 1 may be in flight) ...
        if (ti + 1 < n_tiles) __builtin_amdgcn_s_waitcnt(vmcnt_imm(C) & 0xc07f);
        else                  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0) & 0xc07f);
        // ... and so have everyone's; every wave has also finished reading tile ti - 1,
        // whose buffer tile ti + 2 may now overwrite
        __builtin_amdgcn_s_barrier();
        if (ti + 2 < n_tiles) issue_tile(ti + 2);
        if (ti >= my_tiles) continue;

        const unsigned char *kb = lds + (ti % kBufs) * kBufBytes;
        const unsigned char *vb = kb + kTileBytes;
        const int t0 = ti * kTile;

        // ---- S^T = K Q^T : two 16-position blocks x two 16-query blocks, four 32-dim steps
        float4_t sacc[2][2];
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

        // ---- V rows: lane group gq takes the 8 positions its P operand holds
        uint4_t vreg[8];
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int row = n < 4 ? 4 * gq + n : 16 + 4 * gq + (n - 4);
            vreg[n] = *reinterpret_cast<const uint4_t *>(vb + row * kRowBytes + n16 * 16);
        }

        // ---- online softmax, base 2; this lane: query qw0 + 16nb + n16, positions t0 + 16tb + 4gq + i.
        // m[] is kept in raw score units; the scale enters through one fused multiply-add.
        const bool diagonal = t0 + kTile > qw0;      // some position of the tile is later than some query
        Frag p[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            float s[8];
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 4; ++i) s[4 * tb + i] = sacc[nb][tb][i];
            if (diagonal) {
                const int qpos = qw0 + 16 * nb + n16;
#pragma unroll
                for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (t0 + 16 * tb + 4 * gq + i > qpos) s[4 * tb + i] = -INFINITY;
            }
            float mt = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                             fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
            mt = quad_rows_max(mt);
            const bool raise = mt > m[nb] + lazy_raw;
            if (__builtin_amdgcn_ballot_w64(raise) != 0) {       // rare after the first tiles
                const float m_new = raise ? mt : m[nb];
                const float alpha = __builtin_amdgcn_exp2f((m[nb] - m_new) * a.scale_log2e);
                m[nb] = m_new;
                l[nb] *= alpha;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[nb][e] *= alpha;
            }
            const float neg_m = -m[nb] * a.scale_log2e;
            float pj[8];
            float psum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pj[j] = __builtin_amdgcn_exp2f(fmaf(s[j], a.scale_log2e, neg_m));
                psum += pj[j];
            }
            l[nb] += psum;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const half2_t h2 = __builtin_convertvector((float2_t){pj[2 * j], pj[2 * j + 1]}, half2_t);
                p[nb].h[2 * j] = h2[0];
                p[nb].h[2 * j + 1] = h2[1];
            }
        }

        // ---- O^T += V^T P^T : block e covers dims 8*row + e (row = MFMA row)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int w2 = e >> 1;
            const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
            Frag va;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                va.u[j] = __builtin_amdgcn_perm(vreg[2 * j + 1][w2], vreg[2 * j][w2], sel);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                o[nb][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, p[nb].h, o[nb][e], 0, 0, 0);
        }
    }

    // ---- this lane's query rows: dims 32gq + 8i + e
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float ls = quad_rows_sum(l[nb]);
        const int qpos = qw0 + 16 * nb + n16;
        const long long row = q_first + qpos;
        if (qpos < L && row >= 0 && row < a.n_tokens) {
            const float inv = 1.0f / ls;
            _Float16 *dst = reinterpret_cast<_Float16 *>(a.out) + (row * a.n_qh + h) * kD + 32 * gq;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                Frag x;
#pragma unroll
                for (int e = 0; e < 8; ++e) x.h[e] = (_Float16)(o[nb][e][i] * inv);
                *reinterpret_cast<uint4_t *>(dst + 8 * i) = x.u;
            }
        }
    }
}

}  // namespace

bool sw_prefill_mfma_supported(const SwPrefillArgs &a)
{
    return a.head_dim == kD && a.group >= 1 && a.group <= 8;
}

// How a workgroup is shaped: hp query heads of one group, qw waves (32 query positions
// each) per head.  Large problems share each staged K/V tile among all heads of the group
// (8 waves); small ones are cut into more, smaller workgroups so that the chip fills.
void sw_prefill_shape(int n_req, int n_kvh, int group, int max_len, int *hp, int *qw)
{
    int h = group, w = group >= 8 ? 1 : 8 / group;
    auto groups = [&](int hh, int ww) {
        return (long long)n_req * n_kvh * (group / hh) * ((max_len + 32 * ww - 1) / (32 * ww));
    };
    // first fewer positions per workgroup, then fewer heads
    while (w > 1 && groups(h, w) < 512) w /= 2;
    while (h > 1 && h % 2 == 0 && groups(h, w) < 512) h /= 2;
    *hp = h;
    *qw = w;
}

hipError_t sw_launch_prefill_mfma(const SwPrefillArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    if (!sw_prefill_mfma_supported(a)) return hipErrorNotSupported;
    if (a.hp < 1 || a.group % a.hp != 0 || a.qw < 1) return hipErrorInvalidValue;
    const long long blocks = (long long)a.n_req * a.n_kvh * a.n_qblocks * (a.group / a.hp);
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    const int nw = a.hp * a.qw;
#define SW_PREFILL_CASE(W) \
    if (nw == W) return sw_launch(sw_prefill_mfma_kernel<W>, grid, dim3(64 * W), 0, stream, ev, a);
    SW_PREFILL_CASE(8) SW_PREFILL_CASE(7) SW_PREFILL_CASE(6) SW_PREFILL_CASE(5)
    SW_PREFILL_CASE(4) SW_PREFILL_CASE(3) SW_PREFILL_CASE(2) SW_PREFILL_CASE(1)
#undef SW_PREFILL_CASE
    return hipErrorInvalidValue;
}
