// Partial decode attention on the matrix cores (gfx950, wave64), head_dim 128,
// up to 16 query heads per key/value head.
//
// Under grouped-query attention the group's heads share every K and V row, so
// scores and the weighted sum are small dense contractions:
//     S^T[token][head] = K[token][:] . Q[head][:]        (contraction over head_dim)
//     O^T[dim][head]   = V^T[dim][token] . P^T[token][head]   (contraction over tokens)
// Both run as v_mfma_f32_16x16x32_f16 with the heads on the 16-wide N axis
// (unused heads are zero columns), which leaves the vector ALUs to the softmax
// only and keeps the kernel bound by the K/V stream from HBM -- the read of
// each request's whole cached context that the token phase consists of
// (paper sections 2.2 and 3.5).
//
// One workgroup = WAVES waves = one chunk of one (request, key/value head).
// Each wave owns 32-token tiles of the chunk and keeps its own running
// softmax state; the waves merge through LDS at the end.
//
// Per tile and wave:
//   K  : 8 wave-wide 16-byte global->LDS loads (no registers held while the
//        data is in flight), each fetching 4 whole 256-byte rows.  Lane i
//        always lands at LDS byte 16*i of the instruction's 1 KB block, so the
//        bank-conflict-free layout is made on the GLOBAL side: the lane that
//        lands in slot s of row r fetches chunk s ^ (r % 16) of that row.
//        The MFMA A operand (lane = token, 8 consecutive dims) then reads
//        chunk c of row r from slot c ^ (r % 16): 16 tokens, 16 distinct slots.
//   V  : 8 wave-wide loads of whole rows into registers, ordered so that each
//        lane ends up with the same 8 tokens its P operand holds; an
//        in-register 8x8 16-bit transpose (v_perm_b32) turns them into A
//        operands (lane = dim, 8 tokens).
//   S^T: the MFMA output puts head = lane%16 and 8 tokens in each lane, which
//        is exactly the B-operand layout P^T needs -- no data movement between
//        the two contractions, and every per-head scalar (max, sum, rescale)
//        lives in the lane that owns the head.
//   P  : fed to the matrix core as a binary16 pair (hi + lo), so the weights
//        keep fp32-level precision.
// The next tile's K is requested as soon as the current K has been consumed,
// the next V as soon as the current V has; registers stay at 128 so that four
// workgroups (16 waves) per compute unit keep ~256 KB of loads in flight.
#include "sw_internal.h"
#include "sw_worklist.h"
#include "sw_fused.h"

#include <type_traits>

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

constexpr int   kD        = 128;
constexpr int   kTile     = 32;            // tokens per wave per iteration
constexpr int   kRowBytes = 256;           // a staged K row (chunks XOR-swizzled, no padding)
constexpr int   kHeadStride = 132;         // floats; merge buffer row = head, 128 dims + 4 of padding
constexpr int   kWaveLds  = 16 * kHeadStride * 4;   // 8448 B per wave: K tile (8192) or merge buffer
constexpr float kNegBig   = -1.0e30f;
// Cache policy of the K/V stream: non-temporal (read once; must not push the
// partial results, which are written and read back, out of L2).
constexpr int   kStream   = 2;

static_assert(kTile * kRowBytes <= kWaveLds, "K tile must fit in the wave's LDS area");

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (n < 64),
// leaving the other counters unconstrained.
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

union Frag {
    uint4_t u;
    half8_t h;
};

template <int WAVES, int PER, bool FUSED>
__global__ __launch_bounds__(64 * WAVES, 4)
void sw_partial_mfma_kernel(SwArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[WAVES * kWaveLds];
    __shared__ __attribute__((aligned(16))) unsigned char sm_q[16 * kRowBytes];
    __shared__ float sm_m[WAVES][16];
    __shared__ float sm_l[WAVES][16];
    __shared__ int sm_flag;

    if (FUSED && blockIdx.x < (unsigned)a.n_req) sw_fused_zero_rows<kD>(a, (int)blockIdx.x);

    const SwWork w = sw_find_work<PER>(a, blockIdx.x);
    if (!w.valid) return;
    const int r = w.r, g = w.g, c = w.c;
    const int t_begin = c << a.chunk_shift;
    const int t_end = min(w.L, t_begin + a.chunk);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
    const int n16  = lane & 15;     // head (B operand / output column), token (A operand of QK), dim chunk (A operand of PV)
    const int gq   = lane >> 4;     // k-slot group

    // ---- Q^T for the B operands goes to LDS once per workgroup (row = head, chunks
    // swizzled like K's; heads past the group are zero columns).  Wave w covers
    // rows 4w .. 4w+3 with one global->LDS load: lane i lands in slot i%16 of row
    // 4w + i/16 and therefore fetches chunk slot ^ row.
    {
        const int row = 4 * wave + gq;
        // zero rows first, loads second: no LDS store follows a pending global->LDS load
        if (row < 16 && row >= a.group)
            *reinterpret_cast<uint4_t *>(sm_q + row * kRowBytes + n16 * 16) = uint4_t{0u, 0u, 0u, 0u};
        if (row < a.group) {       // group <= 16: waves past the fourth stage nothing
            const uint16_t *src = a.q + (sw_q_row(a, r) * a.n_qh + g * a.group + row) * kD + 8 * (n16 ^ row);
            __builtin_amdgcn_global_load_lds(src, sm_q + wave * 1024, 16, 0, 0);
        }
    }

    float m = kNegBig, l = 0.f;
    float4_t o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = float4_t{0.f, 0.f, 0.f, 0.f};

    // slab bases are wave-uniform; rows are addressed with 32-bit byte offsets from
    // them (a slab is below 4 GiB: max_len <= 2^23 rows of 256 bytes)
    const char *kbase = reinterpret_cast<const char *>(a.k + (long long)r * a.stride_req + (long long)g * a.stride_kvh);
    const char *vbase = reinterpret_cast<const char *>(a.v + (long long)r * a.stride_req + (long long)g * a.stride_kvh);
    unsigned char *wlds = lds + wave * kWaveLds;

    const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;

    // K tile -> LDS, asynchronously.  Rows past the chunk's end re-read its last
    // row (in bounds, result masked below).
    auto issue_k = [&](int t0) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int rho = 4 * n + gq;
            const int tk  = min(t0 + rho, t_end - 1);
            const char *src = kbase + (((unsigned)tk << 8) | (unsigned)((n16 ^ (rho & 15)) << 4));
            __builtin_amdgcn_global_load_lds(src, wlds + n * 1024, 16, 0, kStream);
        }
    };
    // V tile -> registers: lane group gq takes the 8 tokens its P operand will
    // hold, 4gq .. 4gq+3 and 16+4gq .. 16+4gq+3.
    uint4_t vreg[8];
    auto issue_v = [&](int t0) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int tv = min(t0 + (n < 4 ? 4 * gq + n : 16 + 4 * gq + (n - 4)), t_end - 1);
            vreg[n] = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>(vbase + (((unsigned)tv << 8) | (unsigned)(n16 << 4))));
        }
    };

    // One tile: the wave's loads for this tile are in flight on entry (K first,
    // then V).  MORE says whether the wave has a further tile, whose loads are
    // then issued from here; it is a compile-time flag so that the waits in
    // between can count exactly which loads are still outstanding.
    auto process_tile = [&](int t0, int t0_next, auto more_c) {
        constexpr bool MORE = decltype(more_c)::value;

        // ---- S^T = K Q^T : two 16-token blocks, four 32-dim steps.
        // Both K(t0) (in LDS) and V(t0) (in registers) are awaited here: the
        // compiler counts global->LDS loads and register loads as different
        // kinds of operation and would not wait for one without the other, and
        // with V known complete the next K request below stays in flight all the
        // way to the next tile.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        float4_t sacc[2];
        sacc[0] = float4_t{0.f, 0.f, 0.f, 0.f};
        sacc[1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int off = n16 * kRowBytes + (((4 * kk + gq) ^ n16) << 4);   // row n16, chunk 4kk+gq
            Frag qb, k0, k1;
            qb.u = *reinterpret_cast<const uint4_t *>(sm_q + off);
            k0.u = *reinterpret_cast<const uint4_t *>(wlds + off);
            k1.u = *reinterpret_cast<const uint4_t *>(wlds + 16 * kRowBytes + off);
            sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k0.h, qb.h, sacc[0], 0, 0, 0);
            sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k1.h, qb.h, sacc[1], 0, 0, 0);
        }
        // the K tile has been read into registers: its LDS area may be refilled
        if (MORE) {
            // every read of the K tile must have RETURNED before its area is refilled:
            // global->LDS writes arrive outside the LDS instruction queue
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
            issue_k(t0_next);
        }

        // ---- online softmax, base 2; this lane: head n16, tokens t0 + 16tb + 4gq + i
        float s[8];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 4; ++i) s[4 * tb + i] = sacc[tb][i] * a.scale_log2e;
        // only a wave's last tile can reach past the chunk's end
        const bool ragged = !MORE && t0 + kTile > t_end;
        if (ragged) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (t0 + 16 * tb + 4 * gq + i >= t_end) s[4 * tb + i] = -INFINITY;
        }
        float mt = s[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) mt = fmaxf(mt, s[j]);
        mt = fmaxf(mt, __shfl_xor(mt, 16));
        mt = fmaxf(mt, __shfl_xor(mt, 32));
        const float m_new = fmaxf(m, mt);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        float p[8];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            p[j] = __builtin_amdgcn_exp2f(s[j] - m_new);
            psum += p[j];
        }
        l = l * alpha + psum;
        Frag phi, plo;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const _Float16 hi = (_Float16)p[j];
            phi.h[j] = hi;
            plo.h[j] = (_Float16)(p[j] - (float)hi);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= alpha;

        // ---- O^T += V^T P^T : block e covers dims 8*row + e (row = MFMA row)
        if (ragged) {
            // weights of the re-read rows are exactly 0; clear the rows too so that
            // a non-finite value in the last valid row cannot turn 0 * x into NaN
#pragma unroll
            for (int n = 0; n < 8; ++n)
                if (t0 + (n < 4 ? 4 * gq + n : 16 + 4 * gq + (n - 4)) >= t_end) vreg[n] = uint4_t{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int w = e >> 1;
            const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;
            Frag va;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                va.u[j] = __builtin_amdgcn_perm(vreg[2 * j + 1][w], vreg[2 * j][w], sel);
            o[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, phi.h, o[e], 0, 0, 0);
            o[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, plo.h, o[e], 0, 0, 0);
        }
        if (MORE) issue_v(t0_next);
    };

    int ti = wave;
    if (ti < n_tiles) {
        issue_k(t_begin + ti * kTile);
        issue_v(t_begin + ti * kTile);
    }
    // Q must be in LDS before any wave goes on; the tile loads stay in flight
    // across the barrier.  Vector-memory operations complete in issue order, so
    // "at most the 16 tile loads outstanding" means this wave's Q load is done.
    if (ti < n_tiles) __builtin_amdgcn_s_waitcnt(vmcnt_imm(16) & 0xc07f);   // vmcnt(16), lgkmcnt(0)
    else              __builtin_amdgcn_s_waitcnt(vmcnt_imm(0) & 0xc07f);    // vmcnt(0),  lgkmcnt(0)
    __builtin_amdgcn_s_barrier();

    if (ti < n_tiles) {
        while (ti + WAVES < n_tiles) {
            process_tile(t_begin + ti * kTile, t_begin + (ti + WAVES) * kTile, std::true_type{});
            ti += WAVES;
        }
        process_tile(t_begin + ti * kTile, 0, std::false_type{});
    }

    // ---- the lane groups summed disjoint tokens into l
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);

    // ---- merge the waves through LDS (each wave reuses its own K staging area):
    // row = head (stride 132 floats), column = dim; this lane owns dims
    // 32gq + 8i + e, i.e. for each i two aligned groups of four consecutive dims
    float *mo = reinterpret_cast<float *>(wlds);
    if (n16 < a.group) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                *reinterpret_cast<float4_t *>(mo + n16 * kHeadStride + 32 * gq + 8 * i + 4 * hf) =
                    float4_t{o[4 * hf][i], o[4 * hf + 1][i], o[4 * hf + 2][i], o[4 * hf + 3][i]};
        if (gq == 0) {
            sm_m[wave][n16] = m;
            sm_l[wave][n16] = l;
        }
    }
    __syncthreads();
    // single-launch variant: a request of one chunk is finished here
    const bool alone = FUSED && w.L <= a.chunk;
    for (int idx = threadIdx.x; idx < a.group * (kD / 4); idx += 64 * WAVES) {
        const int hh = idx >> 5;
        const int j4 = idx & 31;
        float mx = sm_m[0][hh];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) mx = fmaxf(mx, sm_m[w][hh]);
        float4_t num = float4_t{0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float f = __builtin_amdgcn_exp2f(sm_m[w][hh] - mx);
            const float4_t x = *reinterpret_cast<const float4_t *>(
                reinterpret_cast<const float *>(lds + w * kWaveLds) + hh * kHeadStride + 4 * j4);
#pragma unroll
            for (int t = 0; t < 4; ++t) num[t] = fmaf(f, x[t], num[t]);
            den = fmaf(f, sm_l[w][hh], den);
        }
        if (alone) {
            sw_store_final4<kD>(a, sw_q_row(a, r) * a.n_qh + g * a.group + hh, j4, num, den);
            continue;
        }
        const long long slot = sw_ws_slot(a, r, g, c, hh);
        sw_store_partial4(a.ws_o + slot * kD + 4 * j4, num, FUSED);
        if (j4 == 0) sw_store_partial2(a.ws_ml + slot * 2, mx, den, FUSED);
    }
    if (FUSED && !alone)
        sw_fused_tail<kD>(a, r, g, 0, a.group, (w.L + a.chunk - 1) >> a.chunk_shift,
                          a.counters + (r * a.n_kvh + g), &sm_flag);
}

}  // namespace

bool sw_partial_mfma_supported(const SwArgs &a)
{
    return a.head_dim == kD && a.group <= 16;
}

hipError_t sw_launch_partial_mfma(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    if (!sw_partial_mfma_supported(a)) return hipErrorNotSupported;
    const long long blocks = (long long)a.n_req * a.n_kvh * a.n_chunks;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    const int per = sw_worklist_per(a.n_req);
#define SW_MFMA_CASE(W, P)                                                                            \
    if (a.waves == W && per == P)                                                                     \
        return a.counters                                                                             \
            ? sw_launch(sw_partial_mfma_kernel<W, P, true>, grid, dim3(64 * W), 0, stream, ev, a)     \
            : sw_launch(sw_partial_mfma_kernel<W, P, false>, grid, dim3(64 * W), 0, stream, ev, a);
#define SW_MFMA_WAVES(W) SW_MFMA_CASE(W, 1) SW_MFMA_CASE(W, 4) SW_MFMA_CASE(W, 16) SW_MFMA_CASE(W, 0)
    SW_MFMA_WAVES(4)
    SW_MFMA_WAVES(8)
    SW_MFMA_WAVES(16)
#undef SW_MFMA_WAVES
#undef SW_MFMA_CASE
    return hipErrorInvalidValue;
}
