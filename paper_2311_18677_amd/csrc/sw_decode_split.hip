// Token-phase (decode) attention on the matrix cores, split over context length, one launch
// (gfx950, wave64), head_dim 128, 16 query heads of a key/value head per workgroup
// (larger groups, up to 64 heads, in head tiles of 16).
//
// The step the paper's token machines run for every generated token (sections 2.2 and
// 3.5): the newest token's query attends over the whole cached context, which is read
// exactly once.  S^T = K Q^T and O^T = V^T P^T run on v_mfma_f32_16x16x32_f16 with the
// group's heads on the 16-wide N axis (head = lane % 16), so the first product's output
// layout is the second product's B-operand layout, P never moves between lanes and every
// softmax scalar lives in the lane that owns the head.
//
// A workgroup handles one item: one chunk of one (request, key/value head), found from a
// scan of the lengths (sw_worklist.h).  A request of L positions is cut into
// nc = ceil(L / chunk) items of (nearly) equal numbers of 32-position tiles.  K and V tiles
// go global->LDS directly (no registers held while data is in flight, all of a wave's
// loads of one kind, so the waits count exactly); a wave keeps the next tile's K and V
// requests in flight while it computes the current tile:
//
//   wait K(i) | QK(i) from LDS | request K(i+1) | softmax(i) |
//   wait V(i) | V(i) LDS->registers | request V(i+1) | transpose, PV(i)
//
// The item's result is merged with the request's other items in the same launch
// (sw_fused.h), or -- FUSED = false -- left in the workspace for a merge kernel.
//
// Append variant (the newest token's rows join the cache in the same pass): the one wave
// whose tile holds the new position overwrites that row of its staged K and V tiles with
// the new rows (brought into LDS once per workgroup) and stores them to the cache in
// global memory; no other wave or workgroup reads that position.
//
// Each wave owns 16 KB of LDS (K tile + V tile), so two 4-wave workgroups fit a compute unit.
//
// The kernel's leading arguments repeat what the length scan needs: they arrive in
// registers with the wave (kernel-argument preload), so the lengths are requested before
// the rest of the arguments has been fetched.
#include "sw_internal.h"
#include "sw_worklist.h"
#include "sw_fused.h"
#include "sw_lane_ops.h"

#include <type_traits>

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

constexpr int   kD        = 128;
constexpr int   kTile     = 32;            // tokens per wave per iteration
constexpr int   kRowBytes = 256;           // a staged K row (chunks XOR-swizzled, no padding)
constexpr int   kHeadStride = 132;         // floats; merge buffer row = head, 128 dims + 4 of padding
constexpr int   kTileBytes = kTile * kRowBytes;         // 8192
constexpr int   kWaveLds  = 2 * kTileBytes;             // K tile + V tile; the merge buffer reuses it
constexpr float kNegBig   = -1.0e30f;
// A running maximum is raised only when a score exceeds it by more than this many
// binary orders of magnitude: weights then stay below 2^kLazyBits.
constexpr float kLazyBits = 8.0f;

typedef float float2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
// Cache policy of the K/V stream: non-temporal (read once; must not push the
// partial results, which are written and read back, out of L2).
constexpr int   kStream   = 2;

static_assert(16 * kHeadStride * 4 <= kWaveLds, "merge buffer must fit in the wave's LDS area");

// s_waitcnt immediate for "at most n vector-memory operations outstanding" (n < 64),
// leaving the other counters unconstrained.
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// Block-table variant: byte offset of the pool block behind each of a tile's 8 load instructions.
struct TileBlocks { long long off[8]; };

// The block table is read-only for the whole launch; reading it through the constant
// address space lets wave-uniform entries come in over the scalar path.
typedef const __attribute__((address_space(4))) int32_t *const_table_t;

union Frag {
    uint4_t u;
    half8_t h;
};

// Keeps a wave-uniform value in scalar registers from here on: whatever it is computed or
// loaded from has been waited for at this point.
template <typename T>
__device__ __forceinline__ void sw_pin(T &x)
{
    asm volatile("" : "+s"(x));
}

template <int WAVES, int PER, bool FUSED, bool PAGED>
__global__ __launch_bounds__(64 * WAVES, 2)
void sw_decode_split_kernel(const int32_t *seq_lens, int n_req, int max_len, int chunk_shift, int n_kvh, SwArgs a_rest)
{
    SwArgs a = a_rest;
    a.seq_lens = seq_lens;
    a.n_req = n_req;
    a.max_len = max_len;
    a.chunk_shift = chunk_shift;
    a.chunk = 1 << chunk_shift;
    a.n_kvh = n_kvh;

    __shared__ __attribute__((aligned(16))) unsigned char lds[WAVES * kWaveLds];
    // Q rows, then (append variant) the new K row and the new V row.  One array: the
    // compiler sees no ordinary store into the new rows' part -- they arrive by
    // global->LDS load only -- and must not take it for never written.
    __shared__ __attribute__((aligned(16))) unsigned char sm_q[16 * kRowBytes + 1024];
    __shared__ float sm_m[WAVES][16];
    __shared__ float sm_l[WAVES][16];
    __shared__ int sm_flag;

    // -- phase: workgroup started
    // First of all the lengths: asking for them needs nothing but the leading arguments, which
    // arrive in registers.  While they travel, every other argument the workgroup will need is
    // read from the argument block in one go: left to itself the compiler reads each one where
    // it is first used, past the early exit below, which puts several scalar-memory round trips
    // in a row between knowing the item and asking for its first tile.
    const SwRawLens<PER> raw_lens = sw_scan_issue<PER>(a);
    sw_pin(a.q);
    sw_pin(a.k);
    sw_pin(a.v);
    sw_pin(a.q_rows);
    sw_pin(a.k_new);
    sw_pin(a.stride_req);
    sw_pin(a.stride_kvh);
    sw_pin(a.group);
    sw_pin(a.n_qh);
    sw_pin(a.n_chunks);
    sw_pin(a.scale_log2e);
    if (FUSED) {
        sw_pin(a.out);
        sw_pin(a.units);
        sw_pin(a.ws_tag);
        sw_pin(a.ws_tag_bytes);
    } else {
        sw_pin(a.ws_o);
        sw_pin(a.ws_ml);
    }
    if (PAGED) {
        sw_pin(a.block_table);
        sw_pin(a.stride_block);
        sw_pin(a.block_shift);
        sw_pin(a.max_blocks);
        sw_pin(a.n_blocks);
    }

    // ... and everything that does not depend on the item is done now, under the lengths' latency.
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
    const int n16  = lane & 15;     // head (B operand / output column), token (A operand of QK), dim chunk (A operand of PV)
    const int gq   = lane >> 4;     // k-slot group
    unsigned char *wlds = lds + wave * kWaveLds;

    // A group of more than 16 query heads is served in head tiles of 16, one workgroup per
    // tile and chunk.  Consecutive workgroups go to different XCDs (eight L2s), so the tiles
    // of one chunk are numbered eight apart: they start almost together behind the SAME L2,
    // where the second and later readers of the chunk find it.  With x = id % 8, y = id / 8:
    // tile y % n_ht of item (y / n_ht) * 8 + x (the host rounds the items up to a multiple
    // of eight; numbers past the last item find no work).
    // h0 = the tile's first head within the group, gn = how many it has.
    const unsigned n_ht = (unsigned)(a.group + 15) >> 4;
    unsigned item = blockIdx.x;
    int ht = 0;
    if (n_ht > 1) {
        const unsigned x = blockIdx.x & 7u, y = blockIdx.x >> 3;
        ht = (int)(y % n_ht);
        item = (y / n_ht) * 8u + x;
    }
    const int h0 = 16 * ht;
    const int gn = min(16, a.group - h0);
    // Q^T rows of heads past the group are zero columns of the B operands.  Stored before any
    // global->LDS load is issued: no LDS store may follow a pending one.
    {
        const int row = 4 * wave + gq;
        if (row < 16 && row >= gn)
            *reinterpret_cast<uint4_t *>(sm_q + row * kRowBytes + n16 * 16) = uint4_t{0u, 0u, 0u, 0u};
    }
    float m = kNegBig, l = 0.f;                        // m in raw score units
    const float lazy_raw = kLazyBits / a.scale_log2e;  // the raise threshold in raw score units
    float4_t o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = float4_t{0.f, 0.f, 0.f, 0.f};

    const SwScan<PER> scan = sw_scan_finish<PER>(a, raw_lens);

    // Rows of requests with no cached position get +0; no item exists for them, so
    // workgroup b < n_req looks after request b.
    if (FUSED && blockIdx.x < (unsigned)a.n_req && sw_scanned_len<PER>(a, scan, (int)blockIdx.x) == 0)
        sw_zero_rows<kD>(a, (int)blockIdx.x);
    const SwWork w = sw_lookup<PER>(a, scan, item);
    // -- phase: item known
    if (!w.valid) return;
    const int r = w.r, g = w.g, c = w.c;
    // the request's tiles of 32 positions, dealt evenly to its nc items: n_all = q * nc + rem
    // tiles, the first rem items take q + 1 of them.  (One division; both numbers are below
    // 2^24, so the single-precision quotient is off by at most one and one look at the
    // remainder settles it.)
    const unsigned n_all = (unsigned)(w.L + kTile - 1) / kTile;
    const unsigned nc = (unsigned)(w.L + a.chunk - 1) >> a.chunk_shift;
    unsigned quot = (unsigned)((float)n_all * __builtin_amdgcn_rcpf((float)nc));
    quot = __builtin_amdgcn_readfirstlane(quot);
    if (quot * nc > n_all) --quot;
    if ((quot + 1) * nc <= n_all) ++quot;
    const unsigned rem = n_all - quot * nc;
    const unsigned tile_begin = (unsigned)c * quot + min((unsigned)c, rem);
    const unsigned tile_count = quot + ((unsigned)c < rem ? 1u : 0u);
    const int t_begin = (int)(tile_begin * kTile);
    const int t_end = min(w.L, (int)((tile_begin + tile_count) * kTile));
    const bool alone = FUSED && nc == 1;            // the whole request: finished here, no merge
    const long long unit = ((long long)r * a.n_kvh + g) * n_ht + ht;
    SwFused fz;
    if (FUSED) {
        sw_fused_begin(a, fz, unit);
        fz.nc = (int)nc;
        fz.c = c;
        fz.merger = false;
    }

    // ---- Q^T for the B operands goes to LDS once per workgroup (row = head, chunks
    // swizzled like K's).  Wave w covers rows 4w .. 4w+3 with one global->LDS load: lane i
    // lands in slot i%16 of row 4w + i/16 and therefore fetches chunk slot ^ row.
    {
        const int row = 4 * wave + gq;
        if (row < gn) {            // at most 16 rows: waves past the fourth stage nothing
            const uint16_t *src = a.q + (sw_q_row(a, r) * a.n_qh + g * a.group + h0 + row) * kD + 8 * (n16 ^ row);
            __builtin_amdgcn_global_load_lds(src, sm_q + wave * 1024, 16, 0, 0);
        }
    }

    // Append variant: position the new rows go to if it lies in this chunk, else -1
    // (workgroup-uniform).  Wave 0 brings both rows into LDS with one load: lanes
    // 0-15 the K row's 16-byte pieces, lanes 16-31 the V row's (lanes 32-63 repeat them).
    unsigned char *sm_new = sm_q + 16 * kRowBytes;
    const int new_pos = (w.new_pos >= t_begin && w.new_pos < t_end) ? w.new_pos : -1;
    if (new_pos >= 0 && wave == 0) {
        const uint16_t *src = ((gq & 1) ? a.v_new : a.k_new) + ((long long)r * a.n_kvh + g) * kD + 8 * n16;
        __builtin_amdgcn_global_load_lds(src, sm_new, 16, 0, 0);
    }

    // Row addressing: a wave-uniform 64-bit base plus a 32-bit byte offset per lane.
    // Dense layout: the base is the (request, head) slab (below 4 GiB: max_len <= 2^23
    // rows of 256 bytes).  Block-table layout: the base is the pool block of the
    // instruction's four rows -- they always share one block (blocks hold a multiple of
    // four positions and tiles start at multiples of 32), so the block id is one scalar
    // table read per instruction; ids are clamped into the pool.
    const char *kslab = reinterpret_cast<const char *>(a.k) + 2 * ((long long)r * a.stride_req + (long long)g * a.stride_kvh);
    const char *vslab = reinterpret_cast<const char *>(a.v) + 2 * ((long long)r * a.stride_req + (long long)g * a.stride_kvh);
    // the table is read-only for the whole launch: read it through the constant address
    // space so that wave-uniform entries come in over the scalar path
    const_table_t table = PAGED ? (const_table_t)(a.block_table + (long long)r * a.max_blocks) : nullptr;
    const int in_block = PAGED ? (1 << a.block_shift) - 1 : ~0;
    const int n_tiles = (int)((unsigned)(t_end - t_begin + kTile - 1) / (unsigned)kTile);   // t_end > t_begin

    // byte offset, from the block-table base, of the block that holds row 4n of tile t0
    // (clamped like the rows themselves); unused in the dense layout
    auto find_blocks = [&](int t0) {
        TileBlocks tb;
        if (PAGED && a.block_shift >= 5) {
            // blocks of 32 positions or more hold the whole tile: one table read
            int id = table[min(t0, t_end - 1) >> a.block_shift];
            id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
            const long long off = 2 * (long long)id * a.stride_block;
#pragma unroll
            for (int n = 0; n < 8; ++n) tb.off[n] = off;
            return tb;
        }
        if (PAGED && a.block_shift == 4) {
            // blocks of 16 positions: one read per half tile
            int id0 = table[min(t0, t_end - 1) >> 4];
            int id1 = table[min(t0 + 16, t_end - 1) >> 4];
            id0 = id0 < 0 ? 0 : (id0 >= a.n_blocks ? a.n_blocks - 1 : id0);
            id1 = id1 < 0 ? 0 : (id1 >= a.n_blocks ? a.n_blocks - 1 : id1);
            const long long off0 = 2 * (long long)id0 * a.stride_block;
            const long long off1 = 2 * (long long)id1 * a.stride_block;
#pragma unroll
            for (int n = 0; n < 8; ++n) tb.off[n] = n < 4 ? off0 : off1;
            return tb;
        }
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            tb.off[n] = 0;
            if (PAGED) {
                const int tu = min(t0 + 4 * n, t_end - 1);            // wave-uniform
                int id = table[tu >> a.block_shift];
                id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
                tb.off[n] = 2 * (long long)id * a.stride_block;
            }
        }
        return tb;
    };

    // K tile -> LDS, asynchronously.  Rows past the chunk's end re-read its last
    // row (in bounds, result masked below).
    auto issue_k = [&](int t0, const TileBlocks &tb) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int rho = 4 * n + gq;
            const int tk  = min(t0 + rho, t_end - 1);
            const char *src = kslab + tb.off[n] + ((((unsigned)tk & (unsigned)in_block) << 8) | (unsigned)((n16 ^ (rho & 15)) << 4));
            __builtin_amdgcn_global_load_lds(src, wlds + n * 1024, 16, 0, kStream);
        }
    };
    // V tile -> LDS, asynchronously, whole rows in token order (row t0 + 4n + gq by
    // instruction n).
    unsigned char *vlds = wlds + kTileBytes;
    auto issue_v = [&](int t0, const TileBlocks &tb) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int tv = min(t0 + 4 * n + gq, t_end - 1);
            __builtin_amdgcn_global_load_lds(vslab + tb.off[n] + ((((unsigned)tv & (unsigned)in_block) << 8) | (unsigned)(n16 << 4)),
                                             vlds + n * 1024, 16, 0, kStream);
        }
    };

    // One tile: the wave's loads for this tile are in flight on entry (K first,
    // then V).  MORE says whether the wave has a further tile, whose loads are
    // then issued from here; it is a compile-time flag so that the waits in
    // between can count exactly which loads are still outstanding.
    auto process_tile = [&](int t0, int t0_next, auto more_c) {
        constexpr bool MORE = decltype(more_c)::value;
        // block ids of the next tile: requested first, needed only after QK
        TileBlocks nb;
        if (MORE) nb = find_blocks(t0_next);

        // ---- S^T = K Q^T : two 16-token blocks, four 32-dim steps.
        // Outstanding, oldest first: K(t0) x8, V(t0) x8.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
        // -- phase: K tile landed
        // the new position lies in the chunk's last tile, which is some wave's last tile
        const bool has_new = !MORE && new_pos >= t0 && new_pos < t0 + kTile;     // wave-uniform
        if (has_new && gq == 0) {
            const int rho = new_pos - t0;
            *reinterpret_cast<uint4_t *>(wlds + rho * kRowBytes + ((n16 ^ (rho & 15)) << 4)) =
                *reinterpret_cast<const uint4_t *>(sm_new + n16 * 16);
        }
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
        // The K tile's LDS area is refilled only once every read of it has RETURNED:
        // the global->LDS writes arrive outside the LDS instruction queue, so a
        // refill requested while reads are still queued can overtake them when the
        // rows come back quickly (cache-resident data).
        if (MORE) {
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
            issue_k(t0_next, nb);
        }

        // ---- online softmax, base 2; this lane: head n16, tokens t0 + 16tb + 4gq + i.
        // m is kept in raw score units (the scale enters through one fused multiply-add) and
        // is only raised when a score exceeds it by more than kLazyBits binary orders of
        // magnitude, so the accumulators are rescaled rarely instead of every tile.
        float s[8];
#pragma unroll
        for (int tb = 0; tb < 2; ++tb)
#pragma unroll
            for (int i = 0; i < 4; ++i) s[4 * tb + i] = sacc[tb][i];
        // only a wave's last tile can reach past the chunk's end
        const bool ragged = !MORE && t0 + kTile > t_end;
        if (ragged) {
#pragma unroll
            for (int tb = 0; tb < 2; ++tb)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (t0 + 16 * tb + 4 * gq + i >= t_end) s[4 * tb + i] = -INFINITY;
        }
        float mt = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])),
                         fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
        mt = quad_rows_max(mt);
        const bool raise = mt > m + lazy_raw;
        if (__builtin_amdgcn_ballot_w64(raise) != 0) {
            const float m_new = raise ? mt : m;
            const float alpha = __builtin_amdgcn_exp2f((m - m_new) * a.scale_log2e);
            m = m_new;
            l *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] *= alpha;
        }
        const float neg_m = -m * a.scale_log2e;
        float p[8];
        float psum = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            p[j] = __builtin_amdgcn_exp2f(fmaf(s[j], a.scale_log2e, neg_m));
            psum += p[j];
        }
        l += psum;
        // weights as a binary16 pair hi + lo (together ~22 bits)
        Frag phi, plo;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const half2_t hi = __builtin_convertvector((float2_t){p[2 * j], p[2 * j + 1]}, half2_t);
            const half2_t lo = __builtin_convertvector(
                (float2_t){p[2 * j] - (float)hi[0], p[2 * j + 1] - (float)hi[1]}, half2_t);
            phi.h[2 * j] = hi[0];
            phi.h[2 * j + 1] = hi[1];
            plo.h[2 * j] = lo[0];
            plo.h[2 * j + 1] = lo[1];
        }

        // ---- V(t0): LDS -> registers.  Lane group gq takes the 8 tokens its P operand
        // holds, 4gq .. 4gq+3 and 16+4gq .. 16+4gq+3.
        // Outstanding, oldest first: V(t0) x8, then K(next) x8 if there is a next tile.
        if (MORE) __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));
        else      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        // -- phase: V tile landed
        if (has_new) {
            // all of the wave's loads have landed: patch the staged V row, then store
            // both rows to the cache (lanes 0-15 the K row, lanes 16-31 the V row)
            if (gq == 0)
                *reinterpret_cast<uint4_t *>(vlds + (new_pos - t0) * kRowBytes + n16 * 16) =
                    *reinterpret_cast<const uint4_t *>(sm_new + 256 + n16 * 16);
            if (gq < 2 && ht == 0) {       // every head tile patches its staged rows, the first one stores
                long long boff = 0;
                if (PAGED) {
                    int id = table[new_pos >> a.block_shift];
                    id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
                    boff = 2 * (long long)id * a.stride_block;
                }
                char *dst = const_cast<char *>(gq ? vslab : kslab) + boff +
                            ((((unsigned)new_pos & (unsigned)in_block) << 8) | (unsigned)(n16 << 4));
                *reinterpret_cast<uint4_t *>(dst) = *reinterpret_cast<const uint4_t *>(sm_new + gq * 256 + n16 * 16);
            }
        }
        uint4_t vreg[8];
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int row = n < 4 ? 4 * gq + n : 16 + 4 * gq + (n - 4);
            vreg[n] = *reinterpret_cast<const uint4_t *>(vlds + row * kRowBytes + n16 * 16);
        }
        if (ragged) {
            // weights of the re-read rows are exactly 0; clear the rows too so that
            // a non-finite value in the last valid row cannot turn 0 * x into NaN
#pragma unroll
            for (int n = 0; n < 8; ++n)
                if (t0 + (n < 4 ? 4 * gq + n : 16 + 4 * gq + (n - 4)) >= t_end) vreg[n] = uint4_t{0u, 0u, 0u, 0u};
        }
        // the V tile is in registers: its LDS area may be refilled
        if (MORE) {
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the LDS reads above have returned
            issue_v(t0_next, nb);
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
            o[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, phi.h, o[e], 0, 0, 0);
            o[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va.h, plo.h, o[e], 0, 0, 0);
        }
    };


    int ti = wave;
    if (ti < n_tiles) {
        const TileBlocks fb = find_blocks(t_begin + ti * kTile);
        issue_k(t_begin + ti * kTile, fb);
        issue_v(t_begin + ti * kTile, fb);
    }
    // -- phase: first loads issued
    // Q (and the new rows) must be in LDS before any wave goes on; the tile loads stay in flight
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

    // -- phase: tiles done
    // ---- the lane groups summed disjoint tokens into l
    l = quad_rows_sum(l);

    // ---- merge the waves through LDS (each wave reuses its own K staging area):
    // row = head (stride 132 floats), column = dim; this lane owns dims
    // 32gq + 8i + e, i.e. for each i two aligned groups of four consecutive dims
    float *mo = reinterpret_cast<float *>(wlds);
    if (n16 < gn) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                *reinterpret_cast<float4_t *>(mo + n16 * kHeadStride + 32 * gq + 8 * i + 4 * hf) =
                    float4_t{o[4 * hf][i], o[4 * hf + 1][i], o[4 * hf + 2][i], o[4 * hf + 3][i]};
        if (gq == 0) {
            sm_m[wave][n16] = m * a.scale_log2e;       // from here on in scaled (base-2 exponent) units
            sm_l[wave][n16] = l;
        }
    }
    __syncthreads();
    // Single launch: every wave's tiles are done.  One lane takes the unit's ticket; while the
    // answer travels, the threads merge the waves and send the chunk's pieces off.
    unsigned ticket = 0;
    if (FUSED && !alone && threadIdx.x == 0) ticket = sw_fused_ticket(a, unit);
    // (a group of more than 8 heads gives a thread two rows' worth of dims)
    constexpr int kMine = (16 * (kD / 4) + 64 * WAVES - 1) / (64 * WAVES);
    float4_t my_num[kMine];
    float my_den[kMine], my_mx[kMine];
#pragma unroll
    for (int k = 0; k < kMine; ++k) {
        const int idx = threadIdx.x + k * 64 * WAVES;
        if (idx >= gn * (kD / 4)) break;
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
            sw_store_final4<kD>(a, sw_q_row(a, r) * a.n_qh + g * a.group + h0 + hh, j4, num, den);
            continue;
        }
        if (FUSED) {
            sw_fused_send<kD>(a, fz, r, g, h0 + hh, j4, num, den, mx);
            my_num[k] = num;
            my_den[k] = den;
            my_mx[k] = mx;
            continue;
        }
        const long long slot = sw_ws_slot(a, r, g, c, h0 + hh);
        *reinterpret_cast<float4_t *>(a.ws_o + slot * kD + 4 * j4) = num;
        if (j4 == 0) *reinterpret_cast<float2_t *>(a.ws_ml + slot * 2) = float2_t{mx, den};
    }
    // -- phase: results stored
    if (FUSED && !alone) {
        // the workgroup that drew the unit's last ticket folds the chunks: every other one has
        // sent its pieces before it drew its own
        if (threadIdx.x == 0) sm_flag = sw_fused_is_merger(a, unit, ticket, (int)nc) ? 1 : 0;
        __syncthreads();
        if (sm_flag == 0) return;
#pragma unroll
        for (int k = 0; k < kMine; ++k) {
            const int idx = threadIdx.x + k * 64 * WAVES;
            if (idx < gn * (kD / 4))
                sw_fused_fold<kD>(a, fz, r, g, h0 + (idx >> 5), idx & 31, my_num[k], my_den[k], my_mx[k]);
        }
    }
    // -- phase: merged
}

}  // namespace

bool sw_decode_split_supported(const SwArgs &a)
{
    return a.head_dim == kD && a.group <= 64 && (a.waves == 4 || a.waves == 8);
}

hipError_t sw_launch_decode_split(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    if (!sw_decode_split_supported(a)) return hipErrorNotSupported;
    long long blocks = (long long)a.n_req * a.n_kvh * a.n_chunks;
    const int n_ht = (a.group + 15) / 16;
    if (n_ht > 1) blocks = (blocks + 7) / 8 * 8 * n_ht;      // see the kernel's numbering of head tiles
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    const int per = sw_worklist_per(a.n_req);
    const bool paged = a.block_table != nullptr;
#define SW_MFMA2_CASE(W, P, B)                                                                           \
    if (a.waves == W && per == P && paged == B)                                                                   \
        return a.units                                                                                \
            ? sw_launch(sw_decode_split_kernel<W, P, true, B>, grid, dim3(64 * W), 0, stream, ev,        \
                        a.seq_lens, a.n_req, a.max_len, a.chunk_shift, a.n_kvh, a)                        \
            : sw_launch(sw_decode_split_kernel<W, P, false, B>, grid, dim3(64 * W), 0, stream, ev,       \
                        a.seq_lens, a.n_req, a.max_len, a.chunk_shift, a.n_kvh, a);
#define SW_MFMA2_WAVES(W)                                                                             \
    SW_MFMA2_CASE(W, 1, false) SW_MFMA2_CASE(W, 4, false) SW_MFMA2_CASE(W, 16, false) SW_MFMA2_CASE(W, 0, false) \
    SW_MFMA2_CASE(W, 1, true) SW_MFMA2_CASE(W, 4, true) SW_MFMA2_CASE(W, 16, true) SW_MFMA2_CASE(W, 0, true)
    SW_MFMA2_WAVES(4)
    SW_MFMA2_WAVES(8)
#undef SW_MFMA2_WAVES
#undef SW_MFMA2_CASE
    return hipErrorInvalidValue;
}
