// Prompt-phase (causal) attention, key-split form for short and medium prompts
// (gfx950, wave64), head_dim 128.
//
// A prompt batch on a prompt machine is capped at about two thousand tokens
// (paper section 4.2), which at one GPU's share of the heads is only a few
// hundred (query block, head) pairs: with one wave per pair the chip is mostly
// idle and every wave walks a long chain of key tiles.  Here the waves of a
// workgroup share ONE pair -- 32 query positions of one head -- and split its
// key range instead: wave w takes tiles w, w + W, ...  Each wave stages its own
// K and V tiles global->LDS and waits on its own counters (no barrier in the
// loop), exactly like the token-phase kernel; at the end the waves' partial
// (maximum, sum, accumulator) triples are merged through LDS and the rows are
// normalised and stored.  The arithmetic per tile is the one of
// sw_prefill_mfma.hip (shared code in sw_prefill_common.h).
#include "sw_prefill_common.h"
#include "sw_merge.h"

#include <type_traits>

namespace {

using namespace sw_prefill;

constexpr int kWaveLds = 2 * kTileBytes;     // K tile + V tile; reused for the merge (32 rows x 128 floats)

// Block-table variant: byte offset of the pool block behind each of a tile's 8 load instructions.
struct TileBlocks { long long off[8]; };

// The block table is read-only for the whole launch; reading it through the constant
// address space lets wave-uniform entries come in over the scalar path.
typedef const __attribute__((address_space(4))) int32_t *const_table_t;

// PAGED: K and V are block pools addressed through the request's row of the block table
// (position t = row t % block_size of pool block table[t / block_size]).
// MERGE (mixed batches): the workgroups from number n_prompt on do not belong to the prompt
// phase at all.  They merge the chunks of the token-phase requests that the partial kernel
// of the same call, launched just before on the same stream, has left in the workspace
// (arguments d) -- the work of the combine kernel, riding along here so that the call is
// two launches instead of three.  Eight output rows per workgroup, one thread per four dims.
template <int WAVES, bool PAGED, bool MERGE>
__global__ __launch_bounds__(64 * WAVES, WAVES >= 4 ? 8 / WAVES : 2)
void sw_prefill_split_kernel(SwPrefillArgs a, SwArgs d, unsigned n_prompt)
{
    if (MERGE && blockIdx.x >= n_prompt) {
        const long long rh = (long long)(blockIdx.x - n_prompt) * (64 * WAVES / (kD / 4)) + (threadIdx.x / (kD / 4));
        if (rh < (long long)d.n_req * d.n_qh) sw_merge::merge_row_serial<kD>(d, (int)rh, (int)(threadIdx.x % (kD / 4)));
        return;
    }
    __shared__ __attribute__((aligned(16))) unsigned char lds[WAVES * kWaveLds];
    // the block's 32 query rows
    __shared__ __attribute__((aligned(16))) unsigned char sm_q[kQPerWave * kRowBytes];
    __shared__ float sm_m[WAVES][kQPerWave];
    __shared__ float sm_l[WAVES][kQPerWave];

    // blockIdx -> (item = (request, query block), key/value head, query head of the group).
    // The heads of a group walk the same K/V tiles; consecutive workgroup numbers go to
    // different XCDs (eight L2s), so the heads of one (item, key/value head) are numbered
    // eight apart and meet behind the same L2.  With x = id % 8, y = id / 8: head y % group
    // of pair (y / group) * 8 + x (the host rounds the pairs up to a multiple of eight;
    // numbers past the last pair find no item).
    const unsigned x8 = blockIdx.x & 7u, y8 = blockIdx.x >> 3;
    const unsigned hh = y8 % (unsigned)a.group;
    const unsigned rest = (y8 / (unsigned)a.group) * 8u + x8;
    const int g = (int)(rest % (unsigned)a.n_kvh);
    const QItem it = find_item(a, rest / (unsigned)a.n_kvh, kQPerWave);
    if (!it.valid) return;
    const int r = it.r, qb = it.qb, L = it.L, NQ = it.NQ;   // NQ: the request's last NQ tokens are its queries
    const long long q_first = it.q_first;
    const int Q0 = qb * kQPerWave;               // first query index of the block ...
    if (Q0 >= NQ) return;
    const int A0 = L - NQ + Q0;                  // ... and its position

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n16  = lane & 15;
    const int gq   = lane >> 4;
    const int h    = g * a.group + (int)hh;
    unsigned char *wlds = lds + wave * kWaveLds;
    unsigned char *vlds = wlds + kTileBytes;

    // ---- the block's query rows go global->LDS (pieces XOR-swizzled by row like K's), each
    // wave fetching its share; every load of the kernel is then of one kind and the waits
    // below count exactly.  Rows past the prompt repeat its last row (never stored).
    // (sm_q is filled by global->LDS loads only; one ordinary store keeps the compiler
    // from treating it as never written)
    if (threadIdx.x < 16) *reinterpret_cast<uint4_t *>(sm_q + threadIdx.x * 16) = uint4_t{0u, 0u, 0u, 0u};
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int c = 0; c < 8 / WAVES; ++c) {
        const int j = wave + WAVES * c;                   // rows 4j .. 4j+3
        const int qi = 4 * j + gq;
        const int qpos = min(Q0 + qi, NQ - 1);
        long long row = q_first + qpos;
        row = row < 0 ? 0 : (row >= a.n_tokens ? a.n_tokens - 1 : row);
        const uint16_t *src = a.q + (row * a.n_qh + h) * kD + 8 * (n16 ^ (qi & 15));
        __builtin_amdgcn_global_load_lds(src, sm_q + j * 1024, 16, 0, 0);
    }

    // dense: the (request, head) slab; block table: the head's rows inside pool block 0
    const long long slab = PAGED ? (long long)g * a.stride_kvh : (long long)r * a.stride_req + (long long)g * a.stride_kvh;
    const char *kslab = reinterpret_cast<const char *>(a.k) + 2 * slab;
    const char *vslab = reinterpret_cast<const char *>(a.v) + 2 * slab;
    const_table_t table = PAGED ? (const_table_t)(a.block_table + (long long)r * a.max_blocks) : nullptr;
    const int in_block = PAGED ? (1 << a.block_shift) - 1 : ~0;

    // the tiles that hold every position the block's queries may see (all start inside the context)
    const int n_tiles = min(A0 + kQPerWave - 1, L - 1) / kTile + 1;

    // Per-lane byte offsets of a tile's load instructions relative to the tile's first row,
    // computed once: instruction n brings rows 4n .. 4n+3 (lane group gq row 4n+gq, lane n16
    // one 16-byte piece; K pieces XOR-swizzled by row).  A tile that lies wholly inside a
    // dense context then needs one 32-bit add per instruction in the vector unit: a
    // wave-uniform slab base plus (tile offset + these offsets).  Only a tile that reaches
    // past the context's end (the last one) takes the slow path that clamps every row.
    // (Keeping the whole uniform part in scalar registers was tried: the compiler then
    // builds 64-bit per-lane pointers and the loads lose their scalar-base form; no gain.)
    unsigned koff[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const int rho = 4 * n + gq;
        koff[n] = (unsigned)(rho * kRowBytes + ((n16 ^ (rho & 15)) << 4));     // rows 16..31: + 4096
    }
    // V pieces are swizzled too (v_swizzle); rows 4n+gq and 4(n+2)+gq share a swizzle
    unsigned voff[2];
#pragma unroll
    for (int n = 0; n < 2; ++n) {
        const int rho = 4 * n + gq;
        voff[n] = (unsigned)(rho * kRowBytes + ((n16 ^ v_swizzle(rho)) << 4));   // rows +8, +16, +24: + 2048 each
    }
    // Block table: the same per-lane offsets inside a pool block, for tiles that lie wholly
    // inside the context (no row to clamp).  Row 4n + gq of a tile is row
    // (t0 + 4n + gq) % block_size of its block; tiles start at multiples of 32 and blocks hold
    // a power of two of positions, so that is (t0 % block_size) + ((4n + gq) % block_size)
    // with a wave-uniform first term, which goes into the scalar base of the load.
    unsigned pk_off[8], pv_off[8];
    if (PAGED) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int rho = 4 * n + gq;
            const unsigned row = ((unsigned)rho & (unsigned)in_block) << 8;
            pk_off[n] = row | (unsigned)((n16 ^ (rho & 15)) << 4);
            pv_off[n] = row | (unsigned)((n16 ^ v_swizzle(rho)) << 4);
        }
    }
    unsigned vt_off[8];
    vt_offsets(n16, gq, vt_off);

    // Block table: byte offset of the pool block that holds row 4n of tile t0 (clamped like
    // the rows themselves).  The four rows of one load instruction always share a block:
    // blocks hold a multiple of four positions and tiles start at multiples of 32.  One
    // wave-uniform table read per instruction; ids are clamped into the pool.
    auto find_blocks = [&](int t0) {
        TileBlocks tb;
        if (PAGED && a.block_shift >= 5) {
            // blocks of 32 positions or more hold the whole tile: one table read
            int id = table[min(t0, L - 1) >> a.block_shift];
            id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
            const long long off = 2 * (long long)id * a.stride_block;
#pragma unroll
            for (int n = 0; n < 8; ++n) tb.off[n] = off;
            return tb;
        }
        if (PAGED && a.block_shift == 4) {
            // blocks of 16 positions: one read per half tile
            int id0 = table[min(t0, L - 1) >> 4];
            int id1 = table[min(t0 + 16, L - 1) >> 4];
            id0 = id0 < 0 ? 0 : (id0 >= a.n_blocks ? a.n_blocks - 1 : id0);
            id1 = id1 < 0 ? 0 : (id1 >= a.n_blocks ? a.n_blocks - 1 : id1);
            const long long off0 = 2 * (long long)id0 * a.stride_block;
            const long long off1 = 2 * (long long)id1 * a.stride_block;
#pragma unroll
            for (int n = 0; n < 8; ++n) tb.off[n] = n < 4 ? off0 : off1;
            return tb;
        }
        // (all eight table reads first, then the arithmetic: one wait instead of eight)
        int id[8];
#pragma unroll
        for (int n = 0; n < 8; ++n) id[n] = PAGED ? table[min(t0 + 4 * n, L - 1) >> a.block_shift] : 0;   // wave-uniform
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int c = id[n] < 0 ? 0 : (id[n] >= a.n_blocks ? a.n_blocks - 1 : id[n]);
            tb.off[n] = PAGED ? 2 * (long long)c * a.stride_block : 0;
        }
        return tb;
    };

    auto issue_k = [&](int t0, const TileBlocks &tb) {
        if (!PAGED && t0 + kTile <= L) {
            // slab base (scalar) + one 32-bit add per instruction (a slab is below 4 GiB)
            const unsigned tile = (unsigned)t0 << 8;
#pragma unroll
            for (int n = 0; n < 8; ++n)
                __builtin_amdgcn_global_load_lds(kslab + (tile + (n >> 2) * 4096 + koff[n & 3]), wlds + n * 1024, 16, 0, 0);
        } else if (PAGED && t0 + kTile <= L) {
            const long long in_blk = (long long)(((unsigned)t0 & (unsigned)in_block) << 8);
#pragma unroll
            for (int n = 0; n < 8; ++n)
                __builtin_amdgcn_global_load_lds(kslab + (tb.off[n] + in_blk) + pk_off[n], wlds + n * 1024, 16, 0, 0);
        } else {
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const int rho = 4 * n + gq;
                const int t = min(t0 + rho, L - 1);      // rows past the context repeat its last row (masked)
                const char *src = kslab + tb.off[n] + ((((unsigned)t & (unsigned)in_block) << 8) | (unsigned)((n16 ^ (rho & 15)) << 4));
                __builtin_amdgcn_global_load_lds(src, wlds + n * 1024, 16, 0, 0);
            }
        }
    };
    auto issue_v = [&](int t0, const TileBlocks &tb) {
        if (!PAGED && t0 + kTile <= L) {
            const unsigned tile = (unsigned)t0 << 8;
#pragma unroll
            for (int n = 0; n < 8; ++n)
                __builtin_amdgcn_global_load_lds(vslab + (tile + (n >> 1) * 2048 + voff[n & 1]), vlds + n * 1024, 16, 0, 0);
        } else if (PAGED && t0 + kTile <= L) {
            const long long in_blk = (long long)(((unsigned)t0 & (unsigned)in_block) << 8);
#pragma unroll
            for (int n = 0; n < 8; ++n)
                __builtin_amdgcn_global_load_lds(vslab + (tb.off[n] + in_blk) + pv_off[n], vlds + n * 1024, 16, 0, 0);
        } else {
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const int rho = 4 * n + gq;
                const int t = min(t0 + rho, L - 1);
                __builtin_amdgcn_global_load_lds(vslab + tb.off[n] + ((((unsigned)t & (unsigned)in_block) << 8) | (unsigned)((n16 ^ v_swizzle(rho)) << 4)),
                                                 vlds + n * 1024, 16, 0, 0);
            }
        }
    };

    Frag qreg[2][4];
    float m[2] = {kNegBig, kNegBig};
    float4_t l[2] = {float4_t{0.f, 0.f, 0.f, 0.f}, float4_t{0.f, 0.f, 0.f, 0.f}};   // sums of the weights (every element the same)
    const float lazy_raw = kLazyBits / a.scale_log2e;
    float4_t o[2][8];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[nb][e] = float4_t{0.f, 0.f, 0.f, 0.f};

    // One tile: its loads are in flight on entry (K first, then V).  MORE (compile time)
    // says whether the wave has a further tile, whose loads are then issued from here,
    // so that every wait counts exactly which loads are still outstanding.
    auto process_tile = [&](int t0, int t0_next, auto more_c) {
        constexpr bool MORE = decltype(more_c)::value;
        // block ids of the next tile: requested first, needed only after the first product
        TileBlocks nb;
        if (MORE) nb = find_blocks(t0_next);
        // outstanding, oldest first: K(t0) x8, V(t0) x8
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
        // The two query blocks are independent: the vector-unit work of one is placed
        // next to the matrix-core work of the other so that the two units overlap.
        Frag kop[2][4];
        load_k_ops(wlds, n16, gq, kop);
        float4_t sacc[2][2];
        qk_block(0, kop, qreg, sacc);
        qk_block(1, kop, qreg, sacc);
        if (MORE) {
            // every read of the K tile has returned before its area is refilled
            __builtin_amdgcn_s_waitcnt(0xc07f);
            issue_k(t0_next, nb);
        }
        const bool diagonal = t0 + kTile > A0;
        Frag p[2];
        softmax_block(0, sacc, diagonal, A0, t0, n16, gq, a.scale_log2e, lazy_raw, m, l, o, p);
        // outstanding, oldest first: V(t0) x8, then K(next) x8 if there is a next tile
        if (MORE) __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
        else      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        Frag va[8];
        load_vt(vlds, vt_off, va);
        if (MORE) {
            __builtin_amdgcn_s_waitcnt(0xc07f);
            issue_v(t0_next, nb);
        }
        pv_block(0, va, p, o, l);
        softmax_block(1, sacc, diagonal, A0, t0, n16, gq, a.scale_log2e, lazy_raw, m, l, o, p);
        pv_block(1, va, p, o, l);
    };

    int ti = wave;
    if (ti < n_tiles) {
        const TileBlocks tb = find_blocks(ti * kTile);
        issue_k(ti * kTile, tb);
        issue_v(ti * kTile, tb);
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(16));      // this wave's query rows have landed
    } else {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    }
    __builtin_amdgcn_s_barrier();                       // ... and so have the other waves'

    if (ti < n_tiles) {
        // Q^T operands: lane (n16, gq) holds dims 32kk + 8gq .. +7 of query 16nb + n16
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                qreg[nb][kk].u = *reinterpret_cast<const uint4_t *>(
                    sm_q + (16 * nb + n16) * kRowBytes + (((4 * kk + gq) ^ n16) << 4));
        while (ti + WAVES < n_tiles) {
            process_tile(ti * kTile, (ti + WAVES) * kTile, std::true_type{});
            ti += WAVES;
        }
        process_tile(ti * kTile, 0, std::false_type{});
    }

    // ---- merge the waves through LDS.  Each wave writes its accumulators over its own
    // staging area as [query 0..31][dim 0..127] floats (16-byte pieces XOR-swizzled by
    // query); this lane owns query 16nb + n16, dims 16e + 4gq + i.
    float *mo = reinterpret_cast<float *>(wlds);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int qi = 16 * nb + n16;
        const float ls = l[nb][0];                    // already summed over the tile's 32 keys
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int piece = 4 * e + gq;                                 // dims 4*piece .. 4*piece+3
            *reinterpret_cast<float4_t *>(mo + qi * kD + 4 * (piece ^ qi)) = o[nb][e];
        }
        if (gq == 0) {
            sm_m[wave][qi] = m[nb];
            sm_l[wave][qi] = ls;
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kQPerWave * (kD / 4); idx += 64 * WAVES) {
        const int qi = idx >> 5;
        const int piece = idx & 31;
        const int qpos = Q0 + qi;                   // query index
        const long long row = q_first + qpos;
        if (qpos >= NQ || row < 0 || row >= a.n_tokens) continue;
        float mx = sm_m[0][qi];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) mx = fmaxf(mx, sm_m[w][qi]);
        float4_t num = float4_t{0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float f = __builtin_amdgcn_exp2f((sm_m[w][qi] - mx) * a.scale_log2e);
            const float4_t x = *reinterpret_cast<const float4_t *>(
                reinterpret_cast<const float *>(lds + w * kWaveLds) + qi * kD + 4 * (piece ^ qi));
#pragma unroll
            for (int t = 0; t < 4; ++t) num[t] = fmaf(f, x[t], num[t]);
            den = fmaf(f, sm_l[w][qi], den);
        }
        const float inv = 1.0f / den;
        const half2_t lo = __builtin_convertvector((float2_t){num[0] * inv, num[1] * inv}, half2_t);
        const half2_t hi = __builtin_convertvector((float2_t){num[2] * inv, num[3] * inv}, half2_t);
        union { half2_t h[2]; unsigned long long u; } pk;
        pk.h[0] = lo;
        pk.h[1] = hi;
        *reinterpret_cast<unsigned long long *>(reinterpret_cast<_Float16 *>(a.out) + (row * a.n_qh + h) * kD + 4 * piece) = pk.u;
    }
}

}  // namespace

hipError_t sw_launch_prefill_split(const SwPrefillArgs &a_in, int waves, hipStream_t stream, const SwLaunchEvents *ev,
                                   const SwArgs *merge)
{
    if (a_in.head_dim != kD) return hipErrorNotSupported;
    SwPrefillArgs a = a_in;
    bool compact;
    const long long pairs = sw_prefill_items(a, kQPerWave, &compact) * a.n_kvh;
    const long long n_prompt = (pairs + 7) / 8 * 8 * a.group;      // see the kernel's numbering of the heads
    if (n_prompt <= 0 || n_prompt > 0x7fffffffLL) return hipErrorInvalidValue;
    a.compact = compact;
    if (merge) {
        // the token-phase rows to merge: 256 threads = 8 rows of 32 four-dim pieces
        if (waves != 4 || merge->head_dim != kD) return hipErrorInvalidValue;
        const long long rows = (long long)merge->n_req * merge->n_qh;
        const long long blocks = n_prompt + (rows + 7) / 8;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        const dim3 grid((unsigned)blocks);
        return a.block_table
            ? sw_launch(sw_prefill_split_kernel<4, true, true>, grid, dim3(256), 0, stream, ev, a, *merge, (unsigned)n_prompt)
            : sw_launch(sw_prefill_split_kernel<4, false, true>, grid, dim3(256), 0, stream, ev, a, *merge, (unsigned)n_prompt);
    }
    const dim3 grid((unsigned)n_prompt);
    const SwArgs none = {};
    const unsigned np = (unsigned)n_prompt;
    if (a.block_table) {
        if (waves == 8) return sw_launch(sw_prefill_split_kernel<8, true, false>, grid, dim3(512), 0, stream, ev, a, none, np);
        if (waves == 4) return sw_launch(sw_prefill_split_kernel<4, true, false>, grid, dim3(256), 0, stream, ev, a, none, np);
        if (waves == 2) return sw_launch(sw_prefill_split_kernel<2, true, false>, grid, dim3(128), 0, stream, ev, a, none, np);
        return hipErrorInvalidValue;
    }
    if (waves == 8) return sw_launch(sw_prefill_split_kernel<8, false, false>, grid, dim3(512), 0, stream, ev, a, none, np);
    if (waves == 4) return sw_launch(sw_prefill_split_kernel<4, false, false>, grid, dim3(256), 0, stream, ev, a, none, np);
    if (waves == 2) return sw_launch(sw_prefill_split_kernel<2, false, false>, grid, dim3(128), 0, stream, ev, a, none, np);
    return hipErrorInvalidValue;
}
