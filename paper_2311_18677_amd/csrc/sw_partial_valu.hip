// Partial decode attention on the vector ALUs (gfx950, wave64).
//
// One workgroup (4 waves) handles one chunk of one (request, key/value head)
// for a tile of up to GT query heads of that head's group.  A K or V row of D
// binary16 values is read by D/8 neighbouring lanes, 16 bytes each, so one
// wave-wide load instruction fetches 64/(D/8) whole rows as one contiguous
// kilobyte.  Scores are formed with the packed binary16 dot product
// (fp32 accumulate) and summed across the row's lanes with DPP; the softmax
// runs online per 16-token tile in base 2; P.V accumulates in fp32.
// The step is the token-phase attention of the paper (section 2.2; every
// cached position is read once, section 3.5).
#include "sw_internal.h"
#include "sw_worklist.h"
#include "sw_fused.h"

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
struct __attribute__((aligned(16))) Row8 { half2_t h[4]; };

typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));

// 16-byte load with the non-temporal hint
__device__ __forceinline__ Row8 stream_load(const uint16_t *p)
{
    union { uint4_t u; Row8 r; } x;
    x.u = __builtin_nontemporal_load(reinterpret_cast<const uint4_t *>(p));
    return x.r;
}

constexpr float kNegBig = -1.0e30f;   // below any reachable score; stays finite under subtraction
constexpr int   kWaves  = 4;

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over the LPR (8 or 16) neighbouring lanes that share a row; every lane gets the total.
template <int LPR>
__device__ __forceinline__ float row_allreduce_sum(float x)
{
    x += dpp_mov<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp_mov<0x141>(x);   // row_half_mirror: lane i <-> 7-i within 8
    if (LPR == 16) x += dpp_mov<0x140>(x);   // row_mirror: lane i <-> 15-i within 16
    return x;
}

template <int D, int GT, int PER>
__global__ __launch_bounds__(64 * kWaves)
void sw_partial_valu_kernel(SwArgs a)
{
    constexpr int LPR = D / 8;        // lanes per row
    constexpr int RPW = 64 / LPR;     // rows per wave-wide load
    constexpr int U   = 16 / RPW;     // loads per 16-token tile
    constexpr int TPW = 16;           // tokens per wave per iteration

    const bool fused = a.units != nullptr;
    const SwScan<PER> scan = sw_scan_lens<PER>(a);
    if (fused && blockIdx.y == 0 && blockIdx.x < (unsigned)a.n_req &&
        sw_scanned_len<PER>(a, scan, (int)blockIdx.x) == 0)
        sw_zero_rows<D>(a, (int)blockIdx.x);

    const SwWork w = sw_lookup<PER>(a, scan, blockIdx.x);
    if (!w.valid) return;
    const int r = w.r, g = w.g, c = w.c;
    const int ht = blockIdx.y;
    const int t_begin = c << a.chunk_shift;
    const int t_end = min(w.L, t_begin + a.chunk);

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int sub  = lane % LPR;      // which 8 dims of the row
    const int row  = lane / LPR;      // which row of a wave-wide load

    const int h0 = g * a.group + ht * GT;         // first query head of this tile
    const int n_valid = min(GT, a.group - ht * GT);

    half2_t qv[GT][4];
#pragma unroll
    for (int hh = 0; hh < GT; ++hh) {
        Row8 x = {};
        if (hh < n_valid)
            x = *reinterpret_cast<const Row8 *>(a.q + (sw_q_row(a, r) * a.n_qh + h0 + hh) * D + sub * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) qv[hh][i] = x.h[i];
    }

    float m[GT], l[GT], o[GT][8];
#pragma unroll
    for (int hh = 0; hh < GT; ++hh) {
        m[hh] = kNegBig;
        l[hh] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[hh][j] = 0.f;
    }

    const bool paged = a.block_table != nullptr;     // then stride_req is 0 and k, v are block pools
    // Append variant (paper section 2.2: the newest token's rows join the cache): the
    // position the new rows go to if it lies in this chunk, else -1.  The lanes that
    // would load that row take the new row instead, and the first head tile stores
    // it to the cache.
    const int new_pos = (w.new_pos >= t_begin && w.new_pos < t_end) ? w.new_pos : -1;
    const uint16_t *kbase = a.k + (long long)r * a.stride_req + (long long)g * a.stride_kvh + sub * 8;
    const uint16_t *vbase = a.v + (long long)r * a.stride_req + (long long)g * a.stride_kvh + sub * 8;

    for (int tile = t_begin + wave * TPW; tile < t_end; tile += kWaves * TPW) {
        Row8 kk[U], vv[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = tile + u * RPW + row;
            ok[u] = t < t_end;
            kk[u] = Row8{};
            vv[u] = Row8{};
            if (ok[u]) {
                // non-temporal: read once, must not push the partial results out of L2
                long long row = (long long)t * D;            // dense: row t of the slab
                if (paged) {
                    // block-table layout: row t % block_size of the pool block the table names
                    int id = a.block_table[(long long)r * a.max_blocks + (t >> a.block_shift)];
                    id = id < 0 ? 0 : (id >= a.n_blocks ? a.n_blocks - 1 : id);
                    row = (long long)id * a.stride_block + (long long)(t & ((1 << a.block_shift) - 1)) * D;
                }
                if (t == new_pos) {
                    const long long src = ((long long)r * a.n_kvh + g) * D + sub * 8;
                    kk[u] = *reinterpret_cast<const Row8 *>(a.k_new + src);
                    vv[u] = *reinterpret_cast<const Row8 *>(a.v_new + src);
                    if (ht == 0) {
                        *reinterpret_cast<Row8 *>(const_cast<uint16_t *>(kbase + row)) = kk[u];
                        *reinterpret_cast<Row8 *>(const_cast<uint16_t *>(vbase + row)) = vv[u];
                    }
                } else {
                    kk[u] = stream_load(kbase + row);
                    vv[u] = stream_load(vbase + row);
                }
            }
        }
#pragma unroll
        for (int hh = 0; hh < GT; ++hh) {
            float s[U];
            float mt = -INFINITY;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float acc = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc = __builtin_amdgcn_fdot2(qv[hh][i], kk[u].h[i], acc, false);
                acc = row_allreduce_sum<LPR>(acc);
                s[u] = ok[u] ? acc * a.scale_log2e : -INFINITY;
                mt = fmaxf(mt, s[u]);
            }
            const float m_new = fmaxf(m[hh], mt);
            const float alpha = __builtin_amdgcn_exp2f(m[hh] - m_new);
            m[hh] = m_new;
            float p[U];
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                p[u] = __builtin_amdgcn_exp2f(s[u] - m_new);
                psum += p[u];
            }
            l[hh] = l[hh] * alpha + psum;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float o0 = o[hh][2 * i] * alpha;
                float o1 = o[hh][2 * i + 1] * alpha;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    o0 = fmaf(p[u], (float)vv[u].h[i].x, o0);
                    o1 = fmaf(p[u], (float)vv[u].h[i].y, o1);
                }
                o[hh][2 * i]     = o0;
                o[hh][2 * i + 1] = o1;
            }
        }
    }

    // ---- merge the RPW row groups of each wave (they saw disjoint tokens) ----
#pragma unroll
    for (int hh = 0; hh < GT; ++hh) {
        float mw = m[hh];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
        const float f = __builtin_amdgcn_exp2f(m[hh] - mw);
        float lw = l[hh] * f;
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) lw += __shfl_xor(lw, off);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float x = o[hh][j] * f;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
            o[hh][j] = x;
        }
        m[hh] = mw;
        l[hh] = lw;
    }

    // ---- merge the waves through LDS, write the chunk's partial result ----
    __shared__ float sm_o[kWaves][GT][D];
    __shared__ float sm_m[kWaves][GT];
    __shared__ float sm_l[kWaves][GT];
    __shared__ int sm_flag;
    if (row == 0) {
#pragma unroll
        for (int hh = 0; hh < GT; ++hh) {
#pragma unroll
            for (int j = 0; j < 8; ++j) sm_o[wave][hh][sub * 8 + j] = o[hh][j];
            if (sub == 0) {
                sm_m[wave][hh] = m[hh];
                sm_l[wave][hh] = l[hh];
            }
        }
    }
    // single-launch variant: a request of one chunk is finished here; otherwise one thread
    // takes the unit's ticket (see sw_fused.h) once every wave is done, the threads send the
    // chunk's pieces, and the workgroup that drew the last ticket folds the unit's chunks
    const int nc = (w.L + a.chunk - 1) >> a.chunk_shift;
    const bool alone = fused && nc == 1;
    const long long unit = ((long long)r * a.n_kvh + g) * gridDim.y + ht;
    SwFused fz;
    if (fused) {
        sw_fused_begin(a, fz, unit);
        fz.nc = nc;
        fz.c = c;
        fz.merger = false;
    }
    __syncthreads();
    unsigned ticket = 0;
    if (fused && !alone && threadIdx.x == 0) ticket = sw_fused_ticket(a, unit);
    // at most GT * D / 4 <= 256 (head, four dims) pairs: one per thread
    sw_float4_t my_num = sw_float4_t{0.f, 0.f, 0.f, 0.f};
    float my_den = 0.f, my_mx = 0.f;
    for (int idx = threadIdx.x; idx < n_valid * (D / 4); idx += 64 * kWaves) {
        const int hh = idx / (D / 4);
        const int j4 = idx - hh * (D / 4);
        float mx = sm_m[0][hh];
#pragma unroll
        for (int w2 = 1; w2 < kWaves; ++w2) mx = fmaxf(mx, sm_m[w2][hh]);
        sw_float4_t num = sw_float4_t{0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < kWaves; ++w2) {
            const float f = __builtin_amdgcn_exp2f(sm_m[w2][hh] - mx);
#pragma unroll
            for (int t = 0; t < 4; ++t) num[t] = fmaf(f, sm_o[w2][hh][4 * j4 + t], num[t]);
            den = fmaf(f, sm_l[w2][hh], den);
        }
        if (alone) {
            sw_store_final4<D>(a, sw_q_row(a, r) * a.n_qh + h0 + hh, j4, num, den);
            continue;
        }
        if (fused) {
            sw_fused_send<D>(a, fz, r, g, ht * GT + hh, j4, num, den, mx);
            my_num = num;
            my_den = den;
            my_mx = mx;
            continue;
        }
        const long long slot = sw_ws_slot(a, r, g, c, ht * GT + hh);
        *reinterpret_cast<sw_float4_t *>(a.ws_o + slot * D + 4 * j4) = num;
        if (j4 == 0) *reinterpret_cast<sw_float2_t *>(a.ws_ml + slot * 2) = sw_float2_t{mx, den};
    }
    if (fused && !alone) {
        if (threadIdx.x == 0) sm_flag = sw_fused_is_merger(a, unit, ticket, nc) ? 1 : 0;
        __syncthreads();
        if (sm_flag == 0) return;
        const int idx = threadIdx.x;
        if (idx < n_valid * (D / 4))
            sw_fused_fold<D>(a, fz, r, g, ht * GT + idx / (D / 4), idx % (D / 4), my_num, my_den, my_mx);
    }
}

template <int D, int GT>
hipError_t launch(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    const int tiles = (a.group + GT - 1) / GT;
    dim3 grid((unsigned)((long long)a.n_req * a.n_kvh * a.n_chunks), (unsigned)tiles, 1);
    const dim3 block(64 * kWaves);
    switch (sw_worklist_per(a.n_req)) {
    case 1:  return sw_launch(sw_partial_valu_kernel<D, GT, 1>, grid, block, 0, stream, ev, a);
    case 4:  return sw_launch(sw_partial_valu_kernel<D, GT, 4>, grid, block, 0, stream, ev, a);
    case 16: return sw_launch(sw_partial_valu_kernel<D, GT, 16>, grid, block, 0, stream, ev, a);
    default: return sw_launch(sw_partial_valu_kernel<D, GT, 0>, grid, block, 0, stream, ev, a);
    }
}

template <int D>
hipError_t launch_d(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    if (a.group == 1) return launch<D, 1>(a, stream, ev);
    if (a.group == 2) return launch<D, 2>(a, stream, ev);
    if (a.group <= 4) return launch<D, 4>(a, stream, ev);
    return launch<D, 8>(a, stream, ev);
}

}  // namespace

hipError_t sw_launch_partial_valu(const SwArgs &a, hipStream_t stream, const SwLaunchEvents *ev)
{
    if ((long long)a.n_req * a.n_kvh * a.n_chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    return a.head_dim == 128 ? launch_d<128>(a, stream, ev) : launch_d<64>(a, stream, ev);
}
