// Prompt-phase (causal) attention on the matrix cores (gfx950, wave64),
// head_dim 128, any number of query heads per key/value head (up to 8 of them share a workgroup).
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
#include "sw_prefill_common.h"

#include <type_traits>

namespace {

using namespace sw_prefill;

constexpr int kBufBytes = 2 * kTileBytes;          // K tile, then V tile
constexpr int kBufs     = 3;

// The block table is read-only for the whole launch; reading it through the constant
// address space lets wave-uniform entries come in over the scalar path.
typedef const __attribute__((address_space(4))) int32_t *const_table_t;

// NW = waves per workgroup = (query heads per workgroup) * (waves per head).
// PAGED: K and V are block pools addressed through the request's row of the block table
// (position t = row t % block_size of pool block table[t / block_size]).
template <int NW, bool PAGED>
__global__ __launch_bounds__(64 * NW, 1)
void sw_prefill_mfma_kernel(SwPrefillArgs a)
{
    // a tile's 16 one-kilobyte load instructions are dealt round-robin to the waves;
    // every wave issues C of them per tile (the last may repeat instruction 15)
    constexpr int C = (16 + NW - 1) / NW;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kBufs * kBufBytes];

    // blockIdx -> (item = (request, query block), key/value head, block of hp query heads)
    const int q_block = kQPerWave * a.qw;        // query tokens per workgroup
    const unsigned n_hb = (unsigned)(a.group / a.hp);
    const unsigned hb = blockIdx.x % n_hb;
    const unsigned rest = blockIdx.x / n_hb;
    const int g = (int)(rest % (unsigned)a.n_kvh);
    const QItem it = find_item(a, rest / (unsigned)a.n_kvh, q_block);
    if (!it.valid) return;
    const int r = it.r, qb = it.qb, L = it.L, NQ = it.NQ;   // NQ: the request's last NQ tokens are its queries
    const long long q_first = it.q_first;
    const int P0 = L - NQ;                       // position of query index 0
    const int Q0 = qb * q_block;                 // first query index of the workgroup
    if (Q0 >= NQ) return;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n16  = lane & 15;
    const int gq   = lane >> 4;
    const int hh   = (int)hb * a.hp + wave % a.hp;   // query head within the group
    const int sb   = wave / a.hp;                // which 32 query positions of the block
    const int qw0  = Q0 + kQPerWave * sb;        // first query index of the wave ...
    const int aw0  = P0 + qw0;                   // ... and its position
    const int h    = g * a.group + hh;

    // The staging area is filled by global->LDS loads only; one ordinary store keeps
    // the compiler from treating it as never written.
    *reinterpret_cast<uint4_t *>(lds + threadIdx.x * 16) = uint4_t{0u, 0u, 0u, 0u};
    __builtin_amdgcn_s_waitcnt(0xc07f);          // lgkmcnt(0): the store is done before any load lands
    __builtin_amdgcn_s_barrier();

    // dense: the (request, head) slab; block table: the head's rows inside pool block 0
    const long long slab = PAGED ? (long long)g * a.stride_kvh : (long long)r * a.stride_req + (long long)g * a.stride_kvh;
    const char *kslab = reinterpret_cast<const char *>(a.k) + 2 * slab;
    const char *vslab = reinterpret_cast<const char *>(a.v) + 2 * slab;
    const_table_t table = PAGED ? (const_table_t)(a.block_table + (long long)r * a.max_blocks) : nullptr;
    const int in_block = PAGED ? (1 << a.block_shift) - 1 : ~0;

    // tiles the workgroup walks: up to the position of its last query
    const int last_pos = P0 + min(Q0 + q_block, NQ) - 1;
    const int n_tiles = last_pos / kTile + 1;
    // tiles this wave computes on: up to the position of its own last query
    const int my_tiles = qw0 < NQ ? min(aw0 + kQPerWave - 1, L - 1) / kTile + 1 : 0;

    // this wave's share of tile ti's loads -> buffer ti % 3.  Instruction j < 8 is K rows
    // 4j .. 4j+3 (16-byte pieces XOR-swizzled by row), j >= 8 is V rows 4(j-8) .. +3.
    // (the buffer index is a compile-time constant everywhere: LDS addresses are then a
    // per-lane value computed once plus an immediate offset, instead of two vector
    // instructions per LDS read to add the rotating buffer's offset)
    auto issue_tile = [&](int ti, auto buf_c) {
        constexpr int B = decltype(buf_c)::value;
        static_assert(B >= 0 && B < kBufs, "buffer index");
        unsigned char *buf = lds + B * kBufBytes;
        const int t0 = ti * kTile;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            int j = wave + NW * c;
            j = j < 16 ? j : 15;
            const int n = j & 7;
            const bool is_v = j >= 8;
            const int rho = 4 * n + gq;
            const int t = min(t0 + rho, L - 1);                      // rows past the prompt repeat its last row
            const int piece = is_v ? (n16 ^ v_swizzle(rho)) : (n16 ^ (rho & 15));
            // block table: the four rows of an instruction share a pool block (blocks hold a
            // multiple of four positions, tiles start at multiples of 32): one wave-uniform
            // table read, the id clamped into the pool
            long long block_off = 0;
            if (PAGED) {
                const int tu = min(t0 + 4 * n, L - 1);
                int id = table[tu >> a.block_shift];
                id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
                block_off = 2 * (long long)id * a.stride_block;
            }
            const char *src = (is_v ? vslab : kslab) + block_off +
                              ((((unsigned)t & (unsigned)in_block) << 8) | (unsigned)(piece << 4));
            __builtin_amdgcn_global_load_lds(src, buf + (is_v ? kTileBytes : 0) + n * 1024, 16, 0, 0);
        }
    };

    unsigned vt_off[8];
    vt_offsets(n16, gq, vt_off);
    float m[2] = {kNegBig, kNegBig};
    float4_t l[2] = {float4_t{0.f, 0.f, 0.f, 0.f}, float4_t{0.f, 0.f, 0.f, 0.f}};   // sums of the weights (every element the same)
    const float lazy_raw = kLazyBits / a.scale_log2e;      // the threshold in raw score units
    float4_t o[2][8];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[nb][e] = float4_t{0.f, 0.f, 0.f, 0.f};

    issue_tile(0, std::integral_constant<int, 0>{});
    if (n_tiles > 1) issue_tile(1, std::integral_constant<int, 1>{});

    // ---- Q^T operands.  Requested after the first tiles so that both latencies overlap;
    // awaited here, once, so that no wait inside the loop has to cover them.
    Frag qreg[2][4];
    load_q(a, q_first, qw0, NQ, h, n16, gq, qreg);

    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

    // One tile, staged in buffer B (= ti % kBufs, as a compile-time constant).
    auto step = [&](int ti, auto buf_c) {
        constexpr int B = decltype(buf_c)::value;
        // this wave's loads of tile ti have landed (those of tile ti + 1 may be in flight) ...
        if (ti + 1 < n_tiles) __builtin_amdgcn_s_waitcnt(vmcnt_imm(C) & 0xc07f);
        else                  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0) & 0xc07f);
        // ... and so have everyone's; every wave has also finished reading tile ti - 1,
        // whose buffer tile ti + 2 may now overwrite
        __builtin_amdgcn_s_barrier();
        if (ti + 2 < n_tiles) issue_tile(ti + 2, std::integral_constant<int, (B + 2) % kBufs>{});
        if (ti >= my_tiles) return;

        const unsigned char *kb = lds + B * kBufBytes;
        const unsigned char *vb = kb + kTileBytes;
        const int t0 = ti * kTile;

        // The two query blocks are independent: the second block's vector work is placed
        // behind the first block's matrix work so that the two units overlap within the wave.
        float4_t sacc[2][2];
        qk_tile(kb, qreg, n16, gq, sacc);
        const bool diagonal = t0 + kTile > aw0;
        Frag p[2];
        softmax_block(0, sacc, diagonal, aw0, t0, n16, gq, a.scale_log2e, lazy_raw, m, l, o, p);
        Frag va[8];
        load_vt(vb, vt_off, va);
        pv_block(0, va, p, o, l);
        softmax_block(1, sacc, diagonal, aw0, t0, n16, gq, a.scale_log2e, lazy_raw, m, l, o, p);
        pv_block(1, va, p, o, l);
    };
    static_assert(kBufs == 3, "the loop below is unrolled by the number of buffers");
    for (int ti = 0; ti < n_tiles; ti += kBufs) {
        step(ti, std::integral_constant<int, 0>{});
        if (ti + 1 < n_tiles) step(ti + 1, std::integral_constant<int, 1>{});
        if (ti + 2 < n_tiles) step(ti + 2, std::integral_constant<int, 2>{});
    }

    // ---- this lane's query rows: dims 16e + 4gq + i
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float ls = l[nb][0];                    // already summed over the tile's 32 keys
        const int qpos = qw0 + 16 * nb + n16;        // query index
        const long long row = q_first + qpos;
        if (qpos < NQ && row >= 0 && row < a.n_tokens) {
            const float inv = 1.0f / ls;
            _Float16 *dst = reinterpret_cast<_Float16 *>(a.out) + (row * a.n_qh + h) * kD + 4 * gq;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const half2_t lo = __builtin_convertvector((float2_t){o[nb][e][0] * inv, o[nb][e][1] * inv}, half2_t);
                const half2_t hi = __builtin_convertvector((float2_t){o[nb][e][2] * inv, o[nb][e][3] * inv}, half2_t);
                union { half2_t h[2]; unsigned long long u; } pk;
                pk.h[0] = lo;
                pk.h[1] = hi;
                *reinterpret_cast<unsigned long long *>(dst + 16 * e) = pk.u;
            }
        }
    }
}

}  // namespace

bool sw_prefill_mfma_supported(const SwPrefillArgs &a)
{
    return a.head_dim == kD && a.group >= 1 && a.hp >= 1 && a.hp <= 8 && a.group % a.hp == 0;
}

// How a workgroup is shaped: hp query heads of one group, qw waves (32 query positions
// each) per head, eight waves in all where the group size allows: hp is the largest
// divisor of the group size that is at most 8.  (Cutting small problems into smaller
// workgroups was tried and measured slower: half the waves per staged tile, same chain of
// dependent tiles.)
void sw_prefill_shape(int n_req, int n_kvh, int group, int max_len, int *hp, int *qw)
{
    (void)n_req; (void)n_kvh; (void)max_len;
    int h = group < 8 ? group : 8;
    while (h > 1 && group % h != 0) --h;
    *hp = h;
    *qw = 8 / h > 0 ? 8 / h : 1;
}

hipError_t sw_launch_prefill_mfma(const SwPrefillArgs &a_in, hipStream_t stream, const SwLaunchEvents *ev)
{
    SwPrefillArgs a = a_in;
    if (!sw_prefill_mfma_supported(a)) return hipErrorNotSupported;
    if (a.hp < 1 || a.group % a.hp != 0 || a.qw < 1) return hipErrorInvalidValue;
    bool compact;
    const long long blocks = sw_prefill_items(a, kQPerWave * a.qw, &compact) * a.n_kvh * (a.group / a.hp);
    a.compact = compact;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    const int nw = a.hp * a.qw;
#define SW_PREFILL_CASE(W) \
    if (nw == W) return a.block_table ? sw_launch(sw_prefill_mfma_kernel<W, true>, grid, dim3(64 * W), 0, stream, ev, a) \
                                      : sw_launch(sw_prefill_mfma_kernel<W, false>, grid, dim3(64 * W), 0, stream, ev, a);
    SW_PREFILL_CASE(8) SW_PREFILL_CASE(7) SW_PREFILL_CASE(6) SW_PREFILL_CASE(5)
    SW_PREFILL_CASE(4) SW_PREFILL_CASE(3) SW_PREFILL_CASE(2) SW_PREFILL_CASE(1)
#undef SW_PREFILL_CASE
    return hipErrorInvalidValue;
}
