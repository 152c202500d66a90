// Host side of the C ABI declared in include/sw_decode.h: argument checks,
// layout arithmetic, the per-(device, stream) workspace, kernel choice and
// launch.  No torch, no oracle, no CPU fallback: without a GPU sw_decode_attn
// reports SW_ERR_HIP.
#include "sw_decode.h"
#include "sw_internal.h"

#include <algorithm>
#include <array>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

namespace {

constexpr int kVersion = 200;   // 0.2.0

// Workgroups of eight waves from which the shared-tile prompt kernel is the faster of the
// two on long prompts (batches of short prompts switch earlier, see causal_attn).
constexpr long long kPrefillSharedMinGroups = 300;

thread_local std::string t_last_error = "";

int fail(int code, const std::string &msg)
{
    t_last_error = msg;
    return code;
}

int fail_hip(hipError_t e, const char *what)
{
    (void)hipGetLastError();   // clear the sticky error so that later calls start clean
    return fail(SW_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Library-owned device memory of one (device, stream).
//   plain : partial results of the two-kernel form, (head_dim + 2) floats per slot.
//   fused : single-launch form, one block per workspace geometry -- (n_kvh, group, n_chunks,
//           head_dim, kernel) decide where a slot lies and which unit owns it, and a piece must
//           only ever be overwritten by the same unit's same chunk and head (see sw_fused.h).  A block is a 256-byte
//           header (word 0: set by the device if a merge gave up), the unit states, then the
//           tagged pieces, sized for a number of requests and zeroed when allocated.
// A block that is outgrown is not freed: a HIP graph captured earlier on the stream still
// holds its address.  It goes to `retired` and is freed by sw_release().
struct FusedBlock {
    char *base = nullptr;
    int n_req_cap = 0;              // requests the block is sized for
    size_t tag_bytes = 0;
};
struct Workspace {
    float *plain = nullptr;
    size_t plain_bytes = 0;
    std::map<std::array<int, 5>, FusedBlock> fused;
    std::vector<void *> retired;
};
constexpr size_t kFusedHeader = 256;

// Workspace of sw_decode_attn_static: partial results of the two-kernel form, for callers
// that cannot allocate.  Every GPU the library runs on holds its own copy of the array, at
// its own address, until the process ends; host code never uses the array's name as a
// pointer (it is a host-side stand-in), only the address hipGetSymbolAddress returns for it
// on the device that is current at the time, looked up once per device.
constexpr size_t kStaticScratchBytes = SW_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};      // per device, null until looked up (guarded by g_scratch_mu)
std::mutex g_scratch_mu;

int static_scratch(int dev, float **ptr)
{
    if (dev < 0 || dev >= kMaxDevices) return fail(SW_ERR_UNSUPPORTED, "device index above 63");
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));     // the current device is `dev`
        if (e != hipSuccess || !p) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *ptr = static_cast<float *>(g_scratch_ptr[dev]);
    return SW_OK;
}

std::mutex g_mu;
std::map<std::pair<int, hipStream_t>, Workspace> g_ws;

// tuning knobs (0 = default)
int g_chunk = 0;
int g_kernel = 0;
int g_combine = 0;
int g_waves = 0;
int g_prefill_hp = 0;   // prompt-phase kernel: query heads per workgroup
int g_prefill_qw = 0;   //                      waves per query head (key-split kernel: waves per workgroup)
int g_prefill_kernel = 0;   // 0 = default, 1 = shared-tile kernel, 2 = key-split kernel
int g_mixed_merge = 0;      // mixed batches: 0 = default, 1 = combine kernel of its own, 2 = inside the prompt kernel

// per-kernel timing
struct ProfRec { hipEvent_t ev[4]; bool has_combine; };
bool g_prof_on = false;
int g_prof_cap = 0;
std::vector<ProfRec> g_prof;
double g_prof_gap_us = 0.0;            // partial kernel's end to combine kernel's start, summed by the last sw_prof_stop
std::vector<hipEvent_t> g_event_pool;   // created by sw_prof_start so that profiled calls stay cheap on the host
constexpr int kEventPoolRecords = 8192;

// Per-kernel timing of one call.  prof_begin decides whether this call is recorded and, if
// so, hands out its four events (from the pool while it lasts); after the launches the
// record is either kept (prof_commit) or its events are destroyed (prof_abort).
int prof_begin(ProfRec &rec, bool has_combine, bool *active)
{
    rec.has_combine = has_combine;
    *active = false;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_prof_on || (int)g_prof.size() >= g_prof_cap) return SW_OK;
    for (int i = 0; i < 4; ++i) {
        if (!g_event_pool.empty()) {
            rec.ev[i] = g_event_pool.back();
            g_event_pool.pop_back();
            continue;
        }
        hipError_t e = hipEventCreate(&rec.ev[i]);
        if (e != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(rec.ev[j]);
            return fail_hip(e, "hipEventCreate");
        }
    }
    *active = true;
    return SW_OK;
}

void prof_abort(ProfRec &rec)
{
    for (hipEvent_t x : rec.ev) (void)hipEventDestroy(x);
}

void prof_commit(ProfRec &rec)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_prof_on && (int)g_prof.size() < g_prof_cap) g_prof.push_back(rec);
    else for (hipEvent_t x : rec.ev) (void)hipEventDestroy(x);
}

int check_shape(int n_req, int n_kvh, int head_dim, int max_len)
{
    if (n_req < 0 || n_kvh <= 0 || max_len <= 0)
        return fail(SW_ERR_SHAPE, "n_req must be >= 0, n_kvh and max_len > 0");
    if (head_dim != 64 && head_dim != 128)
        return fail(SW_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if (max_len > (1 << 23))
        return fail(SW_ERR_SHAPE, "max_len above 2^23");
    if ((long long)n_req * n_kvh > (1LL << 20))
        return fail(SW_ERR_SHAPE, "n_req * n_kvh above 2^20");
    return SW_OK;
}

// Slab of one (request, key/value head): max_len dense rows plus 8 rows of
// padding, so that the slabs of a batch do not all start a large power of two
// apart (workgroups stream many slabs at the same offset at the same time).
long long slab_elems(int head_dim, int max_len)
{
    return (long long)(max_len + 8) * head_dim;
}

// Default positions per workgroup of the partial kernel: a request at max_len
// is cut into at most 16 chunks, within [256, 1024].  Short chunks give the
// parallelism that small batches need, long chunks amortise each workgroup's
// partial-result traffic; measured best on all five reference shapes.  The
// choice depends on max_len alone, so a request's bits never depend on the
// other requests of its batch.
int default_chunk(int n_req, int n_kvh, int max_len)
{
    (void)n_req; (void)n_kvh;
    int chunk = 256;
    while (chunk < 1024 && chunk * 16 < max_len) chunk *= 2;
    return chunk;
}

// Which partial kernel serves a shape when the caller has not forced one.
int default_kernel(const SwArgs &a)
{
    return sw_decode_split_supported(a) ? 2 : 1;
}

// One launch (a workgroup of each unit merges the unit's chunks, sw_fused.h) or two (a merge
// kernel).  Measured over batches of 4 to 128 requests (8 query heads on one key/value head):
// one launch wins while a request has at most 4 chunks -- 30 % where every request is a single
// chunk and no merge happens at all, 4-7 % at 2 to 4 chunks -- and loses beyond (3 % at 8
// chunks, 10-25 % at 14 to 28): the one workgroup that merges a unit walks its chunks on one
// compute unit, where the merge kernel spreads every output row over lanes of its own all
// over the chip.  The choice looks at max_len alone (through the chunk length), never at the
// batch's lengths.
bool default_fused(int n_chunks, size_t slots, int head_dim)
{
    return n_chunks <= 4 && slots * (size_t)head_dim * 8 < 0xffffff00ull;
}

// The single-launch form's pieces are addressed with 32-bit offsets.
bool fused_fits(size_t slots, int head_dim)
{
    return slots * (size_t)head_dim * 8 < 0xffffff00ull;
}

// Everything one step needs, dense or block-table.
struct StepIn {
    const void *q, *k, *v;
    const void *k_new, *v_new;      // append variant: the newest token's rows (then k, v are written), else null
    const int32_t *seq_lens;
    void *out;
    int n_req, n_qh, n_kvh, head_dim, max_len;
    const int32_t *block_table;     // null for the dense layout
    int block_size, max_blocks, n_blocks;
    hipStream_t stream;
    // token-phase part of a mixed batch: see SwArgs (null / 0 otherwise)
    const int32_t *q_rows = nullptr, *q_lens = nullptr;
    long long n_rows = 0;
    int max_q = 0;
    // mixed batches: if non-null and the step would launch the combine kernel, it does not;
    // the kernel's arguments go here instead and the caller sees to the merge
    SwArgs *defer_merge = nullptr;
    // sw_decode_attn_static: two kernels over the library's static scratch array; no
    // allocation, no per-kernel timing
    bool static_ws = false;
};

// Two-kernel form: slots of (head_dim + 2) floats per (request, query head, chunk).
int workspace_plain(Workspace &ws, SwArgs &a, size_t slots, hipStream_t stream)
{
    (void)stream;
    const size_t need = slots * (size_t)(a.head_dim + 2) * sizeof(float);
    if (ws.plain_bytes < need) {
        if (ws.plain) ws.retired.push_back(ws.plain);
        ws.plain = nullptr;
        ws.plain_bytes = 0;
        const size_t grow = need + need / 4;
        hipError_t e = hipMalloc((void **)&ws.plain, grow);
        if (e != hipSuccess) {
            ws.plain = nullptr;
            return fail_hip(e, "hipMalloc(workspace)");
        }
        ws.plain_bytes = grow;
    }
    a.ws_o = ws.plain;
    a.ws_ml = ws.plain + slots * a.head_dim;
    return SW_OK;
}

// Single-launch form: the block of this call's geometry (header, unit states, tagged pieces),
// allocated and zeroed -- in stream order, before the kernel that uses it -- when the geometry
// is new or the batch has outgrown it.
int workspace_fused(Workspace &ws, SwArgs &a, int which, hipStream_t stream)
{
    // (the two kernels cut a group into head tiles, i.e. units, differently)
    const std::array<int, 5> key = {a.n_kvh, a.group, a.n_chunks, a.head_dim, which};
    FusedBlock &blk = ws.fused[key];
    if (blk.n_req_cap < a.n_req) {
        // pieces of one (chunk, head) slot: head_dim / 2 of 16 bytes
        auto pieces_bytes = [&](int n) { return (size_t)n * a.n_qh * a.n_chunks * (size_t)a.head_dim * 8; };
        int cap = std::max(a.n_req, blk.n_req_cap * 2);
        if (pieces_bytes(cap) >= 0xffffff00ull) cap = a.n_req;      // the caller has checked that n_req fits
        const size_t tag_bytes = pieces_bytes(cap);
        const size_t units_bytes = ((size_t)cap * a.n_qh * sizeof(SwUnitState) + 255) & ~(size_t)255;
        const size_t total = kFusedHeader + units_bytes + tag_bytes;
        char *base = nullptr;
        hipError_t e = hipMalloc((void **)&base, total);
        if (e == hipSuccess) {
            e = hipMemsetAsync(base, 0, total, stream);
            if (e != hipSuccess) (void)hipFree(base);
        }
        if (e != hipSuccess) return fail_hip(e, "hipMalloc(workspace)");
        if (blk.base) ws.retired.push_back(blk.base);
        blk.base = base;
        blk.n_req_cap = cap;
        blk.tag_bytes = tag_bytes;
    }
    const size_t units_bytes = ((size_t)blk.n_req_cap * a.n_qh * sizeof(SwUnitState) + 255) & ~(size_t)255;
    a.dev_err = reinterpret_cast<unsigned *>(blk.base);
    a.units = reinterpret_cast<SwUnitState *>(blk.base + kFusedHeader);
    a.ws_tag = blk.base + kFusedHeader + units_bytes;
    a.ws_tag_bytes = (unsigned)blk.tag_bytes;
    return SW_OK;
}

// Policy, workspace and launches; the arguments have been validated.
int run_step(const StepIn &in)
{
    const void *q = in.q, *k_cache = in.k, *v_cache = in.v;
    const int32_t *seq_lens = in.seq_lens;
    void *out = in.out;
    const int n_req = in.n_req, n_qh = in.n_qh, n_kvh = in.n_kvh, head_dim = in.head_dim, max_len = in.max_len;
    const int group = n_qh / n_kvh;
    hipStream_t stream = in.stream;

    int chunk, kernel, combine, waves;
    bool prof;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        chunk = g_chunk;
        kernel = g_kernel;
        combine = g_combine;
        waves = g_waves;
        prof = false;
    }
    if (chunk == 0) chunk = default_chunk(n_req, n_kvh, max_len);
    // keep the partial kernel's grid below 2^31 workgroups
    // (a group of more than 16 heads takes one workgroup per 16 heads and chunk)
    while ((((long long)(max_len + chunk - 1) / chunk) * n_req * n_kvh + 7) * ((group + 15) / 16) > 0x7fffffffLL) chunk *= 2;
    const int n_chunks = (max_len + chunk - 1) / chunk;

    SwArgs a;
    a.q = (const uint16_t *)q;
    a.k = (const uint16_t *)k_cache;
    a.v = (const uint16_t *)v_cache;
    a.k_new = (const uint16_t *)in.k_new;
    a.v_new = (const uint16_t *)in.v_new;
    a.seq_lens = seq_lens;
    a.out = (uint16_t *)out;
    a.n_req = n_req;
    a.n_qh = n_qh;
    a.n_kvh = n_kvh;
    a.group = group;
    a.head_dim = head_dim;
    a.max_len = max_len;
    a.chunk = chunk;
    a.chunk_shift = 0;
    while ((1 << a.chunk_shift) < chunk) ++a.chunk_shift;
    a.n_chunks = n_chunks;
    // four waves per workgroup measured best at every chunk length; a wave walks
    // chunk / 128 tiles of 32 positions
    a.waves = waves ? waves : 4;
    if (a.waves * 32 > chunk) a.waves = 4;      // a chunk of 64 still runs 4 waves (2 idle)
    a.q_rows = in.q_rows;
    a.q_lens = in.q_lens;
    a.n_rows = in.n_rows;
    a.max_q = in.max_q;
    a.block_table = in.block_table;
    if (in.block_table) {
        a.block_shift = 0;
        while ((1 << a.block_shift) < in.block_size) ++a.block_shift;
        a.max_blocks = in.max_blocks;
        a.n_blocks = in.n_blocks;
        a.stride_kvh = (long long)in.block_size * head_dim;
        a.stride_block = a.stride_kvh * n_kvh;
        a.stride_req = 0;
    } else {
        a.block_shift = a.max_blocks = a.n_blocks = 0;
        a.stride_block = 0;
        a.stride_kvh = slab_elems(head_dim, max_len);
        a.stride_req = a.stride_kvh * n_kvh;
    }
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)head_dim));

    // 1 = vector ALU, 2 = matrix cores
    int which = kernel;
    if (which == 0) which = default_kernel(a);
    if (which == 2 && !sw_decode_split_supported(a))
        return fail(SW_ERR_UNSUPPORTED, "the matrix-core kernel does not cover this shape");

    const size_t slots = (size_t)n_req * n_qh * n_chunks;
    if (combine == 2 && !fused_fits(slots, head_dim))
        return fail(SW_ERR_UNSUPPORTED, "the single-launch workspace would exceed 4 GiB");
    const bool fused = in.static_ws ? false : (combine == 0 ? default_fused(n_chunks, slots, head_dim) : combine == 2);
    if (in.static_ws && slots * (size_t)(head_dim + 2) * sizeof(float) > kStaticScratchBytes)
        return fail(SW_ERR_UNSUPPORTED, "the partial results of this shape (n_req * n_qh * ceil(max_len / chunk) * "
                                        "(head_dim + 2) * 4 bytes) exceed the static scratch of "
                                        + std::to_string(kStaticScratchBytes) + " bytes");

    // ---- workspace ----
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    a.ws_o = a.ws_ml = nullptr;
    a.units = nullptr;
    a.ws_tag = nullptr;
    a.ws_tag_bytes = 0;
    a.dev_err = nullptr;
    if (in.static_ws) {
        float *base = nullptr;
        int rc = static_scratch(dev, &base);
        if (rc != SW_OK) return rc;
        a.ws_o = base;
        a.ws_ml = base + slots * head_dim;
    } else {
        std::lock_guard<std::mutex> lk(g_mu);
        Workspace &ws = g_ws[std::make_pair(dev, stream)];
        int rc = fused ? workspace_fused(ws, a, which, stream) : workspace_plain(ws, a, slots, stream);
        if (rc != SW_OK) return rc;
    }

    const bool defer = in.defer_merge && !fused;
    SwLaunchEvents ev_p = {nullptr, nullptr}, ev_c = {nullptr, nullptr};
    ProfRec rec;
    int prc = in.static_ws ? SW_OK : prof_begin(rec, !fused && !defer, &prof);
    if (prc != SW_OK) return prc;
    if (prof) {
        ev_p = {rec.ev[0], rec.ev[1]};
        ev_c = {rec.ev[2], rec.ev[3]};
    }

    e = which == 2 ? sw_launch_decode_split(a, stream, prof ? &ev_p : nullptr)
                   : sw_launch_partial_valu(a, stream, prof ? &ev_p : nullptr);
    if (e == hipSuccess && !fused && !defer) e = sw_launch_combine(a, stream, prof ? &ev_c : nullptr);
    if (e == hipSuccess && defer) *in.defer_merge = a;
    if (e != hipSuccess) {
        if (prof) prof_abort(rec);
        return fail_hip(e, "kernel launch");
    }
    if (prof) prof_commit(rec);
    return SW_OK;
}

}  // namespace

extern "C" {

int sw_version(void) { return kVersion; }

const char *sw_last_error(void) { return t_last_error.c_str(); }

int sw_kv_layout(int n_req, int n_kvh, int head_dim, int max_len, sw_kv_layout_t *out)
{
    if (!out) return fail(SW_ERR_NULL, "out is NULL");
    int rc = check_shape(n_req, n_kvh, head_dim, max_len);
    if (rc != SW_OK) return rc;
    const long long slab = slab_elems(head_dim, max_len);
    out->dtype = SW_F16;
    out->elem_bytes = 2;
    out->stride_dim = 1;
    out->stride_tok = head_dim;
    out->stride_kvh = slab;
    out->stride_req = slab * n_kvh;
    out->total_elems = slab * n_kvh * (long long)n_req;
    out->base_align = 256;
    out->reserved = 0;
    return SW_OK;
}

int sw_set_param(int key, int value)
{
    std::lock_guard<std::mutex> lk(g_mu);
    switch (key) {
    case SW_PARAM_CHUNK:
        if (value != 0 && (value < 64 || value > 65536 || (value & (value - 1))))
            return fail(SW_ERR_PARAM, "chunk must be 0 or a power of two in [64, 65536]");
        g_chunk = value;
        return SW_OK;
    case SW_PARAM_KERNEL:
        if (value < 0 || value > 2) return fail(SW_ERR_PARAM, "kernel must be 0, 1 or 2");
        g_kernel = value;
        return SW_OK;
    case SW_PARAM_COMBINE:
        if (value < 0 || value > 2) return fail(SW_ERR_PARAM, "combine must be 0, 1 or 2");
        g_combine = value;
        return SW_OK;
    case SW_PARAM_WAVES:
        if (value != 0 && value != 4 && value != 8)
            return fail(SW_ERR_PARAM, "waves must be 0, 4 or 8");
        g_waves = value;
        return SW_OK;
    case SW_PARAM_PREFILL_HEADS:
        if (value < 0 || value > 8) return fail(SW_ERR_PARAM, "prefill heads must be in [0, 8]");
        g_prefill_hp = value;
        return SW_OK;
    case SW_PARAM_PREFILL_WAVES:
        if (value < 0 || value > 8) return fail(SW_ERR_PARAM, "prefill waves per head must be in [0, 8]");
        g_prefill_qw = value;
        return SW_OK;
    case SW_PARAM_PREFILL_KERNEL:
        if (value < 0 || value > 2) return fail(SW_ERR_PARAM, "prefill kernel must be 0, 1 or 2");
        g_prefill_kernel = value;
        return SW_OK;
    case SW_PARAM_MIXED_MERGE:
        if (value < 0 || value > 2) return fail(SW_ERR_PARAM, "mixed merge must be 0, 1 or 2");
        g_mixed_merge = value;
        return SW_OK;
    default:
        return fail(SW_ERR_PARAM, "unknown parameter key");
    }
}

int sw_get_param(int key, int *value)
{
    if (!value) return fail(SW_ERR_NULL, "value is NULL");
    std::lock_guard<std::mutex> lk(g_mu);
    switch (key) {
    case SW_PARAM_CHUNK:  *value = g_chunk;  return SW_OK;
    case SW_PARAM_KERNEL: *value = g_kernel; return SW_OK;
    case SW_PARAM_COMBINE: *value = g_combine; return SW_OK;
    case SW_PARAM_WAVES: *value = g_waves; return SW_OK;
    case SW_PARAM_PREFILL_HEADS: *value = g_prefill_hp; return SW_OK;
    case SW_PARAM_PREFILL_WAVES: *value = g_prefill_qw; return SW_OK;
    case SW_PARAM_PREFILL_KERNEL: *value = g_prefill_kernel; return SW_OK;
    case SW_PARAM_MIXED_MERGE: *value = g_mixed_merge; return SW_OK;
    default: return fail(SW_ERR_PARAM, "unknown parameter key");
    }
}

int sw_prof_start(int capacity)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_prof_on) return fail(SW_ERR_STATE, "sw_prof_start called twice");
    if (capacity <= 0 || capacity > (1 << 20)) return fail(SW_ERR_PARAM, "capacity out of range");
    g_prof.clear();
    g_prof.reserve((size_t)capacity);
    // events for the first records up front: creating them inside a profiled call would
    // leave the GPU idle between kernels and distort what is being measured
    const int pooled = 4 * (capacity < kEventPoolRecords ? capacity : kEventPoolRecords);
    for (int i = 0; i < pooled; ++i) {
        hipEvent_t ev;
        if (hipEventCreate(&ev) != hipSuccess) {
            (void)hipGetLastError();
            break;                      // calls fall back to creating their own
        }
        g_event_pool.push_back(ev);
    }
    g_prof_cap = capacity;
    g_prof_on = true;
    return SW_OK;
}

int sw_prof_stop(double *partial_us_sum, double *combine_us_sum, int *n_calls)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_prof_on) return fail(SW_ERR_STATE, "sw_prof_stop without sw_prof_start");
    g_prof_on = false;
    double p = 0.0, c = 0.0, gap = 0.0;
    int n = 0, rc = SW_OK;
    for (ProfRec &rec : g_prof) {
        float ms0 = 0.f, ms1 = 0.f, ms_gap = 0.f;
        hipError_t e = hipEventSynchronize(rec.has_combine ? rec.ev[3] : rec.ev[1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms0, rec.ev[0], rec.ev[1]);
        if (e == hipSuccess && rec.has_combine) e = hipEventElapsedTime(&ms1, rec.ev[2], rec.ev[3]);
        if (e == hipSuccess && rec.has_combine) e = hipEventElapsedTime(&ms_gap, rec.ev[1], rec.ev[2]);
        if (e == hipSuccess) {
            p += 1e3 * ms0;
            c += 1e3 * ms1;
            gap += 1e3 * ms_gap;
            ++n;
        } else if (rc == SW_OK) {
            rc = fail_hip(e, "reading profile events");
        }
        for (hipEvent_t ev : rec.ev) (void)hipEventDestroy(ev);
    }
    g_prof.clear();
    for (hipEvent_t ev : g_event_pool) (void)hipEventDestroy(ev);
    g_event_pool.clear();
    g_prof_gap_us = gap;
    if (partial_us_sum) *partial_us_sum = p;
    if (combine_us_sum) *combine_us_sum = c;
    if (n_calls) *n_calls = n;
    return rc;
}

int sw_prof_last_gap(double *gap_us_sum)
{
    std::lock_guard<std::mutex> lk(g_mu);
    if (!gap_us_sum) return fail(SW_ERR_PARAM, "null pointer");
    *gap_us_sum = g_prof_gap_us;
    return SW_OK;
}

int sw_release(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    int rc = SW_OK;
    int cur = 0;
    if (g_ws.empty()) return SW_OK;
    if (hipGetDevice(&cur) != hipSuccess) cur = 0;
    for (auto &kv : g_ws) {
        hipError_t e = hipSetDevice(kv.first.first);
        if (e == hipSuccess) e = hipDeviceSynchronize();
        if (e == hipSuccess && kv.second.plain) e = hipFree(kv.second.plain);
        for (auto &fb : kv.second.fused)
            if (e == hipSuccess && fb.second.base) e = hipFree(fb.second.base);
        for (void *old : kv.second.retired)
            if (e == hipSuccess) e = hipFree(old);
        if (e != hipSuccess && rc == SW_OK) rc = fail_hip(e, "sw_release");
    }
    g_ws.clear();
    (void)hipSetDevice(cur);
    return rc;
}

int sw_device_status(int *gave_up)
{
    if (!gave_up) return fail(SW_ERR_NULL, "gave_up is NULL");
    *gave_up = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail_hip(e, "sw_device_status");
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto &kv : g_ws) {
        if (kv.first.first != dev) continue;
        for (auto &fb : kv.second.fused) {
            if (!fb.second.base) continue;
            unsigned word = 0;
            e = hipMemcpy(&word, fb.second.base, sizeof(word), hipMemcpyDeviceToHost);
            if (e != hipSuccess) return fail_hip(e, "sw_device_status");
            if (word) *gave_up = 1;
        }
    }
    return SW_OK;
}

// sw_decode_attn and sw_decode_attn_append; k_new == v_new == NULL selects the former.
static int decode_dense(const void *q, const void *k_new, const void *v_new, bool append,
                        const void *k_cache, const void *v_cache,
                        const int32_t *seq_lens, void *out,
                        int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                        void *stream_v, bool static_ws = false)
{
    // ---- validation: nothing below this block runs on bad arguments, and
    // nothing in it touches HIP ----
    if (n_qh <= 0) return fail(SW_ERR_SHAPE, "n_qh must be > 0");
    if (n_kvh <= 0 || n_qh % n_kvh != 0)
        return fail(SW_ERR_SHAPE, "n_kvh must be > 0 and divide n_qh");
    int rc = check_shape(n_req, n_kvh, head_dim, max_len);
    if (rc != SW_OK) return rc;
    const int group = n_qh / n_kvh;
    if (group > 64) return fail(SW_ERR_UNSUPPORTED, "more than 64 query heads per key/value head");
    if ((long long)n_req * n_qh > (1LL << 20)) return fail(SW_ERR_SHAPE, "n_req * n_qh above 2^20");
    if (n_req == 0) return SW_OK;
    if (!q || !k_cache || !v_cache || !seq_lens || !out)
        return fail(SW_ERR_NULL, "q, k_cache, v_cache, seq_lens and out must be non-NULL");
    if (append && (!k_new || !v_new)) return fail(SW_ERR_NULL, "k_new and v_new must be non-NULL");
    if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out |
         (uintptr_t)k_new | (uintptr_t)v_new) & 15u)
        return fail(SW_ERR_ALIGN, "q, k_new, v_new, k_cache, v_cache and out must be 16-byte aligned");
    if ((uintptr_t)seq_lens & 3u) return fail(SW_ERR_ALIGN, "seq_lens must be 4-byte aligned");

    StepIn in;
    in.q = q; in.k = k_cache; in.v = v_cache; in.seq_lens = seq_lens; in.out = out;
    in.k_new = k_new; in.v_new = v_new;
    in.n_req = n_req; in.n_qh = n_qh; in.n_kvh = n_kvh; in.head_dim = head_dim; in.max_len = max_len;
    in.block_table = nullptr; in.block_size = in.max_blocks = in.n_blocks = 0;
    in.stream = (hipStream_t)stream_v;
    in.static_ws = static_ws;
    return run_step(in);
}

int sw_decode_attn_static(const void *q, const void *k_cache, const void *v_cache,
                          const int32_t *seq_lens, void *out,
                          int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                          void *stream)
{
    return decode_dense(q, nullptr, nullptr, false, k_cache, v_cache, seq_lens, out,
                        n_req, n_qh, n_kvh, head_dim, max_len, stream, true);
}

int sw_decode_attn(const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *seq_lens, void *out,
                   int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                   void *stream)
{
    return decode_dense(q, nullptr, nullptr, false, k_cache, v_cache, seq_lens, out,
                        n_req, n_qh, n_kvh, head_dim, max_len, stream);
}

int sw_decode_attn_append(const void *q, const void *k_new, const void *v_new,
                          void *k_cache, void *v_cache,
                          const int32_t *seq_lens, void *out,
                          int n_req, int n_qh, int n_kvh, int head_dim, int max_len,
                          void *stream)
{
    return decode_dense(q, k_new, v_new, true, k_cache, v_cache, seq_lens, out,
                        n_req, n_qh, n_kvh, head_dim, max_len, stream);
}

// Block-table geometry of the paged entry points (block_table == NULL: dense layout).
struct PagedGeom {
    const int32_t *block_table;
    int block_size, max_blocks, n_blocks;
};

// sw_prefill_attn (q_lens == NULL: every cached token is a query) and sw_mixed_attn, dense
// (pg == NULL) or over block pools (then max_len is max_blocks * block_size)
static int causal_attn(const void *q, const void *k_cache, const void *v_cache, const PagedGeom *pg,
                       const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                       bool mixed, void *out, long long n_tokens,
                       int n_req, int n_qh, int n_kvh, int head_dim, int max_len, int max_q_len,
                       void *stream_v)
{
    // ---- validation, before any HIP call ----
    if (n_qh <= 0) return fail(SW_ERR_SHAPE, "n_qh must be > 0");
    if (n_kvh <= 0 || n_qh % n_kvh != 0)
        return fail(SW_ERR_SHAPE, "n_kvh must be > 0 and divide n_qh");
    if (pg) {
        if (pg->block_size < 4 || pg->block_size > 4096 || (pg->block_size & (pg->block_size - 1)))
            return fail(SW_ERR_UNSUPPORTED, "block_size must be a power of two in [4, 4096]");
        if (pg->max_blocks <= 0 || pg->n_blocks <= 0)
            return fail(SW_ERR_SHAPE, "max_blocks and n_blocks must be > 0");
        if ((long long)pg->max_blocks * pg->block_size > (1 << 23))
            return fail(SW_ERR_SHAPE, "max_blocks * block_size above 2^23");
        max_len = pg->max_blocks * pg->block_size;
        if (!mixed) max_q_len = max_len;
    }
    int rc = check_shape(n_req, n_kvh, head_dim, max_len);
    if (rc != SW_OK) return rc;
    if (n_tokens < 0 || n_tokens > (1LL << 31)) return fail(SW_ERR_SHAPE, "n_tokens must be in [0, 2^31]");
    if (max_q_len <= 0) return fail(SW_ERR_SHAPE, "max_q_len must be > 0");
    if (max_q_len > max_len) max_q_len = max_len;
    if (head_dim != 128) return fail(SW_ERR_UNSUPPORTED, "the prompt-phase kernels need head_dim 128");
    if (n_qh / n_kvh > 64) return fail(SW_ERR_UNSUPPORTED, "more than 64 query heads per key/value head");
    if (n_req == 0 || n_tokens == 0) return SW_OK;
    if (!q || !k_cache || !v_cache || !seq_lens || !q_starts || !out || (mixed && !q_lens))
        return fail(SW_ERR_NULL, "q, k_cache, v_cache, seq_lens, q_starts, q_lens and out must be non-NULL");
    if (pg && !pg->block_table) return fail(SW_ERR_NULL, "block_table must be non-NULL");
    if (pg && ((uintptr_t)pg->block_table & 3u)) return fail(SW_ERR_ALIGN, "block_table must be 4-byte aligned");
    if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15u)
        return fail(SW_ERR_ALIGN, "q, k_cache, v_cache and out must be 16-byte aligned");
    if (((uintptr_t)seq_lens | (uintptr_t)q_starts | (uintptr_t)q_lens) & 3u)
        return fail(SW_ERR_ALIGN, "seq_lens, q_starts and q_lens must be 4-byte aligned");

    SwPrefillArgs a;
    a.q = (const uint16_t *)q;
    a.k = (const uint16_t *)k_cache;
    a.v = (const uint16_t *)v_cache;
    a.seq_lens = seq_lens;
    a.q_starts = q_starts;
    a.q_lens = q_lens;
    a.max_q = max_q_len;
    a.skip_single = 0;
    a.compact = 0;                  // the launchers decide
    a.out = (uint16_t *)out;
    a.n_tokens = n_tokens;
    a.n_req = n_req;
    a.n_qh = n_qh;
    a.n_kvh = n_kvh;
    a.group = n_qh / n_kvh;
    a.head_dim = head_dim;
    a.max_len = max_len;
    // Two kernels.  The shared-tile kernel stages every K/V tile once for the eight waves of
    // a workgroup (the heads of a group, or more query positions of one head) and runs at a
    // steady 41-45 % of the matrix peak once its workgroups fill the chip more than once;
    // with fewer its time is that of the longest prompt's last block.  The key-split kernel
    // gives every (32 queries, head) pair a workgroup of its own and splits its keys among
    // the waves: four times the workgroups, each a quarter as long, but no tile is shared.
    // Measured crossover: about 300 eight-wave workgroups, i.e. query tokens x heads of
    // about 77000 (one 12288-token prompt or ten 1024-token prompts at 8 heads); less for
    // batches of short prompts.  The choice
    // looks at the call's number of query tokens, which the host knows; inside either kernel
    // a request's result does not depend on the rest of its batch.
    int shared_hp, shared_qw;
    sw_prefill_shape(n_req, n_kvh, a.group, max_q_len, &shared_hp, &shared_qw);
    int which, knob_hp, knob_qw, knob_merge;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        which = g_prefill_kernel;
        knob_hp = g_prefill_hp;
        knob_qw = g_prefill_qw;
        knob_merge = g_mixed_merge;
    }
    if (which == 0) {
        // (in a mixed batch most requests are usually token-phase requests, one row each,
        // which the prompt kernel never sees: leave one row per request out of the estimate)
        long long q_bound = std::min<long long>(n_tokens, (long long)n_req * max_q_len);
        if (mixed) q_bound = std::max<long long>(0, q_bound - n_req);
        const long long groups = (q_bound / (32 * shared_qw)) * n_kvh * (a.group / shared_hp);
        // short prompts make short chains of tiles, so fewer workgroups already suffice
        // (measured: 24 x 256 and 16 x 512 tokens gain 17-25 % from the shared-tile kernel)
        const long long avg_q = q_bound / (n_req > 0 ? n_req : 1);
        const long long need = avg_q <= 256 ? 192 : (avg_q <= 1024 ? 256 : kPrefillSharedMinGroups);
        which = groups >= need ? 1 : 2;
    }
    int split_waves = 4;
    if (which == 2) {
        a.hp = 1;
        a.qw = 1;
        if (knob_qw == 2 || knob_qw == 4 || knob_qw == 8) split_waves = knob_qw;
    } else {
        a.hp = shared_hp;
        a.qw = shared_qw;
        if (knob_hp > 0 && a.group % knob_hp == 0) {
            a.hp = knob_hp;
            a.qw = 8 / a.hp > 0 ? 8 / a.hp : 1;
        }
        if (knob_qw > 0 && a.hp * knob_qw <= 8) a.qw = knob_qw;
    }
    a.n_qblocks = (max_q_len + 32 * a.qw - 1) / (32 * a.qw);      // the grid covers max_q_len query tokens
    if (pg) {
        a.block_table = pg->block_table;
        a.block_shift = 0;
        while ((1 << a.block_shift) < pg->block_size) ++a.block_shift;
        a.max_blocks = pg->max_blocks;
        a.n_blocks = pg->n_blocks;
        a.stride_kvh = (long long)pg->block_size * head_dim;
        a.stride_block = a.stride_kvh * n_kvh;
        a.stride_req = 0;
    } else {
        a.block_table = nullptr;
        a.block_shift = a.max_blocks = a.n_blocks = 0;
        a.stride_block = 0;
        a.stride_kvh = slab_elems(head_dim, max_len);
        a.stride_req = a.stride_kvh * n_kvh;
    }
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)head_dim));
    if ((long long)n_req * n_qh * a.n_qblocks > 0x7fffffffLL)
        return fail(SW_ERR_SHAPE, "too many workgroups");

    // A mixed batch is served by both families of kernels: requests with exactly one query
    // token are token-phase requests (memory bound, one pass over their cache: the
    // split-over-context kernels, reading and writing row q_starts[r]); the prompt kernel
    // takes the others.  Which family serves a request depends on that request alone.
    // (Running the two parts side by side on two streams was tried in both orders, the
    // token-phase kernels first and the prompt kernel first: 33.4 us against 32.1 us on one
    // stream for 63 token-phase requests beside a 1500-token prompt -- no gain.)
    SwArgs merge_args = {};             // ws_o stays null unless the merge was left to the prompt kernel
    if (mixed) {
        StepIn in{};
        in.q = q; in.k = k_cache; in.v = v_cache;
        in.k_new = in.v_new = nullptr;
        in.seq_lens = seq_lens;
        in.out = out;
        in.n_req = n_req; in.n_qh = n_qh; in.n_kvh = n_kvh; in.head_dim = head_dim; in.max_len = max_len;
        in.block_table = pg ? pg->block_table : nullptr;
        in.block_size = pg ? pg->block_size : 0;
        in.max_blocks = pg ? pg->max_blocks : 0;
        in.n_blocks = pg ? pg->n_blocks : 0;
        in.stream = (hipStream_t)stream_v;
        in.q_rows = q_starts; in.q_lens = q_lens; in.n_rows = n_tokens; in.max_q = max_q_len;
        // With the four-wave key-split kernel to follow, the chunks of the token-phase requests
        // are merged by extra workgroups of that kernel: two launches instead of three.
        if (which == 2 && split_waves == 4 && max_q_len > 1 && knob_merge != 1) in.defer_merge = &merge_args;
        rc = run_step(in);
        if (rc != SW_OK) return rc;
        a.skip_single = 1;
        if (max_q_len == 1) return SW_OK;          // no request can have more than one query
    }

    bool prof = false;
    SwLaunchEvents ev = {nullptr, nullptr};
    ProfRec rec;
    int prc = prof_begin(rec, false, &prof);
    if (prc != SW_OK) return prc;
    if (prof) ev = {rec.ev[0], rec.ev[1]};
    hipError_t e;
    e = which == 2 ? sw_launch_prefill_split(a, split_waves, (hipStream_t)stream_v, prof ? &ev : nullptr,
                                             merge_args.ws_o ? &merge_args : nullptr)
                   : sw_launch_prefill_mfma(a, (hipStream_t)stream_v, prof ? &ev : nullptr);
    if (e != hipSuccess) {
        if (prof) prof_abort(rec);
        return fail_hip(e, "kernel launch");
    }
    if (prof) prof_commit(rec);
    return SW_OK;
}

int sw_prefill_attn(const void *q, const void *k_cache, const void *v_cache,
                    const int32_t *seq_lens, const int32_t *q_starts, void *out, long long n_tokens,
                    int n_req, int n_qh, int n_kvh, int head_dim, int max_len, void *stream)
{
    return causal_attn(q, k_cache, v_cache, nullptr, seq_lens, q_starts, nullptr, false, out, n_tokens,
                       n_req, n_qh, n_kvh, head_dim, max_len, max_len > 0 ? max_len : 1, stream);
}

int sw_prefill_attn_paged(const void *q, const void *k_pool, const void *v_pool,
                          const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_starts,
                          void *out, long long n_tokens, int n_req, int n_qh, int n_kvh, int head_dim,
                          int block_size, int max_blocks, int n_blocks, void *stream)
{
    const PagedGeom pg = {block_table, block_size, max_blocks, n_blocks};
    return causal_attn(q, k_pool, v_pool, &pg, seq_lens, q_starts, nullptr, false, out, n_tokens,
                       n_req, n_qh, n_kvh, head_dim, 1, 1, stream);
}

int sw_mixed_attn_paged(const void *q, const void *k_pool, const void *v_pool,
                        const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_starts,
                        const int32_t *q_lens, void *out, long long n_tokens,
                        int n_req, int n_qh, int n_kvh, int head_dim,
                        int block_size, int max_blocks, int n_blocks, int max_q_len, void *stream)
{
    const PagedGeom pg = {block_table, block_size, max_blocks, n_blocks};
    return causal_attn(q, k_pool, v_pool, &pg, seq_lens, q_starts, q_lens, true, out, n_tokens,
                       n_req, n_qh, n_kvh, head_dim, 1, max_q_len, stream);
}

int sw_mixed_attn(const void *q, const void *k_cache, const void *v_cache,
                  const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                  void *out, long long n_tokens,
                  int n_req, int n_qh, int n_kvh, int head_dim, int max_len, int max_q_len,
                  void *stream)
{
    return causal_attn(q, k_cache, v_cache, nullptr, seq_lens, q_starts, q_lens, true, out, n_tokens,
                       n_req, n_qh, n_kvh, head_dim, max_len, max_q_len, stream);
}

// sw_kv_store / sw_kv_store_paged
static int kv_store(const void *k_rows, const void *v_rows, void *k_cache, void *v_cache, const PagedGeom *pg,
                    const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                    long long n_tokens, int n_req, int n_kvh, int head_dim, int max_len, int max_q_len,
                    void *stream_v)
{
    if (pg) {
        if (pg->block_size < 4 || pg->block_size > 4096 || (pg->block_size & (pg->block_size - 1)))
            return fail(SW_ERR_UNSUPPORTED, "block_size must be a power of two in [4, 4096]");
        if (pg->max_blocks <= 0 || pg->n_blocks <= 0)
            return fail(SW_ERR_SHAPE, "max_blocks and n_blocks must be > 0");
        if ((long long)pg->max_blocks * pg->block_size > (1 << 23))
            return fail(SW_ERR_SHAPE, "max_blocks * block_size above 2^23");
        max_len = pg->max_blocks * pg->block_size;
    }
    int rc = check_shape(n_req, n_kvh, head_dim, max_len);
    if (rc != SW_OK) return rc;
    if (n_kvh > 65535) return fail(SW_ERR_SHAPE, "n_kvh above 65535");
    if (n_tokens < 0 || n_tokens > (1LL << 31)) return fail(SW_ERR_SHAPE, "n_tokens must be in [0, 2^31]");
    if (max_q_len <= 0) return fail(SW_ERR_SHAPE, "max_q_len must be > 0");
    if (max_q_len > max_len) max_q_len = max_len;
    if (n_req == 0 || n_tokens == 0) return SW_OK;
    if (!k_rows || !v_rows || !k_cache || !v_cache || !seq_lens || !q_starts)
        return fail(SW_ERR_NULL, "k_rows, v_rows, the caches, seq_lens and q_starts must be non-NULL");
    if (pg && !pg->block_table) return fail(SW_ERR_NULL, "block_table must be non-NULL");
    if (((uintptr_t)k_rows | (uintptr_t)v_rows | (uintptr_t)k_cache | (uintptr_t)v_cache) & 15u)
        return fail(SW_ERR_ALIGN, "k_rows, v_rows and the caches must be 16-byte aligned");
    if (((uintptr_t)seq_lens | (uintptr_t)q_starts | (uintptr_t)q_lens | (uintptr_t)(pg ? pg->block_table : nullptr)) & 3u)
        return fail(SW_ERR_ALIGN, "seq_lens, q_starts, q_lens and block_table must be 4-byte aligned");

    SwPrefillArgs a;
    a.q = nullptr;
    a.k = (const uint16_t *)k_cache;
    a.v = (const uint16_t *)v_cache;
    a.seq_lens = seq_lens;
    a.q_starts = q_starts;
    a.q_lens = q_lens;
    a.out = nullptr;
    a.n_tokens = n_tokens;
    a.n_req = n_req;
    a.n_qh = n_kvh;
    a.n_kvh = n_kvh;
    a.group = 1;
    a.head_dim = head_dim;
    a.max_len = max_len;
    a.max_q = max_q_len;
    a.skip_single = 0;
    a.compact = 0;
    a.hp = a.qw = 1;
    a.n_qblocks = (max_q_len + 31) / 32;
    if (pg) {
        a.block_table = pg->block_table;
        a.block_shift = 0;
        while ((1 << a.block_shift) < pg->block_size) ++a.block_shift;
        a.max_blocks = pg->max_blocks;
        a.n_blocks = pg->n_blocks;
        a.stride_kvh = (long long)pg->block_size * head_dim;
        a.stride_block = a.stride_kvh * n_kvh;
        a.stride_req = 0;
    } else {
        a.block_table = nullptr;
        a.block_shift = a.max_blocks = a.n_blocks = 0;
        a.stride_block = 0;
        a.stride_kvh = slab_elems(head_dim, max_len);
        a.stride_req = a.stride_kvh * n_kvh;
    }
    a.scale_log2e = 0.f;
    if ((long long)n_req * a.n_qblocks > 0x7fffffffLL) return fail(SW_ERR_SHAPE, "too many workgroups");

    bool prof = false;
    SwLaunchEvents ev = {nullptr, nullptr};
    ProfRec rec;
    int prc = prof_begin(rec, false, &prof);
    if (prc != SW_OK) return prc;
    if (prof) ev = {rec.ev[0], rec.ev[1]};
    hipError_t e = sw_launch_kv_store(a, (const uint16_t *)k_rows, (const uint16_t *)v_rows,
                                      (uint16_t *)k_cache, (uint16_t *)v_cache, (hipStream_t)stream_v,
                                      prof ? &ev : nullptr);
    if (e != hipSuccess) {
        if (prof) prof_abort(rec);
        return fail_hip(e, "kernel launch");
    }
    if (prof) prof_commit(rec);
    return SW_OK;
}

int sw_kv_store(const void *k_rows, const void *v_rows, void *k_cache, void *v_cache,
                const int32_t *seq_lens, const int32_t *q_starts, const int32_t *q_lens,
                long long n_tokens, int n_req, int n_kvh, int head_dim, int max_len, int max_q_len,
                void *stream)
{
    return kv_store(k_rows, v_rows, k_cache, v_cache, nullptr, seq_lens, q_starts, q_lens, n_tokens,
                    n_req, n_kvh, head_dim, max_len, max_q_len, stream);
}

int sw_kv_store_paged(const void *k_rows, const void *v_rows, void *k_pool, void *v_pool,
                      const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_starts,
                      const int32_t *q_lens, long long n_tokens, int n_req, int n_kvh, int head_dim,
                      int block_size, int max_blocks, int n_blocks, int max_q_len, void *stream)
{
    const PagedGeom pg = {block_table, block_size, max_blocks, n_blocks};
    return kv_store(k_rows, v_rows, k_pool, v_pool, &pg, seq_lens, q_starts, q_lens, n_tokens,
                    n_req, n_kvh, head_dim, 1, max_q_len, stream);
}

// sw_kv_pack / sw_kv_unpack
static int kv_copy(void *k_pool, void *v_pool, const int32_t *block_table, const int32_t *seq_lens,
                   void *k_dense, void *v_dense, bool to_dense,
                   int n_req, int n_kvh, int head_dim, int max_len,
                   int block_size, int max_blocks, int n_blocks, void *stream_v)
{
    if (block_size < 4 || block_size > 4096 || (block_size & (block_size - 1)))
        return fail(SW_ERR_UNSUPPORTED, "block_size must be a power of two in [4, 4096]");
    if (max_blocks <= 0 || n_blocks <= 0) return fail(SW_ERR_SHAPE, "max_blocks and n_blocks must be > 0");
    if ((long long)max_blocks * block_size > (1 << 23))
        return fail(SW_ERR_SHAPE, "max_blocks * block_size above 2^23");
    int rc = check_shape(n_req, n_kvh, head_dim, max_len);
    if (rc != SW_OK) return rc;
    if (n_req == 0) return SW_OK;
    if (!k_pool || !v_pool || !block_table || !seq_lens || !k_dense || !v_dense)
        return fail(SW_ERR_NULL, "pools, block_table, seq_lens and dense caches must be non-NULL");
    if (((uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)k_dense | (uintptr_t)v_dense) & 15u)
        return fail(SW_ERR_ALIGN, "pools and dense caches must be 16-byte aligned");
    if (((uintptr_t)seq_lens | (uintptr_t)block_table) & 3u)
        return fail(SW_ERR_ALIGN, "seq_lens and block_table must be 4-byte aligned");

    SwHandoffArgs a;
    a.k_pool = (uint16_t *)k_pool;
    a.v_pool = (uint16_t *)v_pool;
    a.k_dense = (uint16_t *)k_dense;
    a.v_dense = (uint16_t *)v_dense;
    a.block_table = block_table;
    a.seq_lens = seq_lens;
    a.n_req = n_req;
    a.n_kvh = n_kvh;
    a.head_dim = head_dim;
    const long long cap = (long long)max_blocks * block_size;
    a.cap = (int)(cap < max_len ? cap : max_len);
    const int rows = sw_kv_copy_rows_per_group();
    a.n_tiles = (a.cap + rows - 1) / rows;
    a.block_shift = 0;
    while ((1 << a.block_shift) < block_size) ++a.block_shift;
    a.max_blocks = max_blocks;
    a.n_blocks = n_blocks;
    a.p_stride_kvh = (long long)block_size * head_dim;
    a.stride_block = a.p_stride_kvh * n_kvh;
    a.d_stride_kvh = slab_elems(head_dim, max_len);
    a.d_stride_req = a.d_stride_kvh * n_kvh;
    if ((long long)n_req * n_kvh * a.n_tiles > 0x7fffffffLL) return fail(SW_ERR_SHAPE, "too many workgroups");

    bool prof = false;
    SwLaunchEvents ev = {nullptr, nullptr};
    ProfRec rec;
    int prc = prof_begin(rec, false, &prof);
    if (prc != SW_OK) return prc;
    if (prof) ev = {rec.ev[0], rec.ev[1]};
    hipError_t e;
    e = sw_launch_kv_copy(a, to_dense, (hipStream_t)stream_v, prof ? &ev : nullptr);
    if (e != hipSuccess) {
        if (prof) prof_abort(rec);
        return fail_hip(e, "kernel launch");
    }
    if (prof) prof_commit(rec);
    return SW_OK;
}

int sw_kv_pack(const void *k_pool, const void *v_pool, const int32_t *block_table,
               const int32_t *seq_lens, void *k_dense, void *v_dense,
               int n_req, int n_kvh, int head_dim, int max_len,
               int block_size, int max_blocks, int n_blocks, void *stream)
{
    return kv_copy(const_cast<void *>(k_pool), const_cast<void *>(v_pool), block_table, seq_lens,
                   k_dense, v_dense, true, n_req, n_kvh, head_dim, max_len,
                   block_size, max_blocks, n_blocks, stream);
}

int sw_kv_unpack(const void *k_dense, const void *v_dense, const int32_t *block_table,
                 const int32_t *seq_lens, void *k_pool, void *v_pool,
                 int n_req, int n_kvh, int head_dim, int max_len,
                 int block_size, int max_blocks, int n_blocks, void *stream)
{
    return kv_copy(k_pool, v_pool, block_table, seq_lens, const_cast<void *>(k_dense),
                   const_cast<void *>(v_dense), false, n_req, n_kvh, head_dim, max_len,
                   block_size, max_blocks, n_blocks, stream);
}

int sw_kv_span_plan(const int32_t *block_table, const int32_t *seq_lens,
                    int32_t *span_first, int32_t *span_blocks, int32_t *n_spans,
                    int n_req, int block_size, int max_blocks, int n_blocks, void *stream)
{
    if (n_req < 0 || n_req > (1 << 20)) return fail(SW_ERR_SHAPE, "n_req must be in [0, 2^20]");
    if (block_size < 4 || block_size > 4096 || (block_size & (block_size - 1)))
        return fail(SW_ERR_UNSUPPORTED, "block_size must be a power of two in [4, 4096]");
    if (max_blocks <= 0 || n_blocks <= 0) return fail(SW_ERR_SHAPE, "max_blocks and n_blocks must be > 0");
    if ((long long)max_blocks * block_size > (1 << 23))
        return fail(SW_ERR_SHAPE, "max_blocks * block_size above 2^23");
    if (n_req == 0) return SW_OK;
    if (!block_table || !seq_lens || !span_first || !span_blocks || !n_spans)
        return fail(SW_ERR_NULL, "block_table, seq_lens, span_first, span_blocks and n_spans must be non-NULL");
    if (((uintptr_t)block_table | (uintptr_t)seq_lens | (uintptr_t)span_first |
         (uintptr_t)span_blocks | (uintptr_t)n_spans) & 3u)
        return fail(SW_ERR_ALIGN, "int32 arrays must be 4-byte aligned");
    int shift = 0;
    while ((1 << shift) < block_size) ++shift;
    hipError_t e = sw_launch_kv_span_plan(block_table, seq_lens, span_first, span_blocks, n_spans,
                                          n_req, shift, max_blocks, n_blocks, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return SW_OK;
}

int sw_advance_lens(int32_t *seq_lens, int n_req, int max_len, void *stream)
{
    if (n_req < 0 || max_len <= 0) return fail(SW_ERR_SHAPE, "n_req must be >= 0 and max_len > 0");
    if (n_req == 0) return SW_OK;
    if (!seq_lens) return fail(SW_ERR_NULL, "seq_lens is NULL");
    if ((uintptr_t)seq_lens & 3u) return fail(SW_ERR_ALIGN, "seq_lens must be 4-byte aligned");
    hipError_t e = sw_launch_advance_lens(seq_lens, n_req, max_len, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "kernel launch");
    return SW_OK;
}

int sw_stream_read(const void *src, long long n_bytes, void *sink, int workgroups, void *stream)
{
    if (n_bytes < 0 || (n_bytes & 15)) return fail(SW_ERR_SHAPE, "n_bytes must be a non-negative multiple of 16");
    if (workgroups < 0 || workgroups > 65536) return fail(SW_ERR_SHAPE, "workgroups must be in [0, 65536]");
    // measured best: eight workgroups per compute unit up to about 128 MB, 64 beyond
    if (workgroups == 0) workgroups = n_bytes < (128LL << 20) ? 2048 : 16384;
    if (!src || !sink) return fail(SW_ERR_NULL, "src and sink must be non-NULL");
    if ((uintptr_t)src & 15u) return fail(SW_ERR_ALIGN, "src must be 16-byte aligned");
    if ((uintptr_t)sink & 3u) return fail(SW_ERR_ALIGN, "sink must be 4-byte aligned");
    bool prof = false;
    SwLaunchEvents ev = {nullptr, nullptr};
    ProfRec rec;
    int prc = prof_begin(rec, false, &prof);
    if (prc != SW_OK) return prc;
    if (prof) ev = {rec.ev[0], rec.ev[1]};
    hipError_t e = sw_launch_stream_read(src, (unsigned long long)n_bytes, (unsigned *)sink, workgroups,
                                         (hipStream_t)stream, prof ? &ev : nullptr);
    if (e != hipSuccess) {
        if (prof) prof_abort(rec);
        return fail_hip(e, "kernel launch");
    }
    if (prof) prof_commit(rec);
    return SW_OK;
}

int sw_kv_paged_layout(int n_blocks, int n_kvh, int head_dim, int block_size,
                       sw_kv_paged_layout_t *out)
{
    if (!out) return fail(SW_ERR_NULL, "out is NULL");
    if (n_blocks <= 0 || n_kvh <= 0) return fail(SW_ERR_SHAPE, "n_blocks and n_kvh must be > 0");
    if (head_dim != 64 && head_dim != 128) return fail(SW_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if (block_size < 4 || block_size > 4096 || (block_size & (block_size - 1)))
        return fail(SW_ERR_UNSUPPORTED, "block_size must be a power of two in [4, 4096]");
    out->dtype = SW_F16;
    out->elem_bytes = 2;
    out->stride_dim = 1;
    out->stride_tok = head_dim;
    out->stride_kvh = (long long)block_size * head_dim;
    out->stride_block = out->stride_kvh * n_kvh;
    out->total_elems = out->stride_block * (long long)n_blocks;
    out->base_align = 256;
    out->block_size = block_size;
    return SW_OK;
}

static int decode_paged(const void *q, const void *k_new, const void *v_new, bool append,
                        const void *k_pool, const void *v_pool,
                        const int32_t *block_table, const int32_t *seq_lens, void *out,
                        int n_req, int n_qh, int n_kvh, int head_dim,
                        int block_size, int max_blocks, int n_blocks, void *stream_v)
{
    // ---- validation, before any HIP call ----
    if (n_qh <= 0) return fail(SW_ERR_SHAPE, "n_qh must be > 0");
    if (n_kvh <= 0 || n_qh % n_kvh != 0)
        return fail(SW_ERR_SHAPE, "n_kvh must be > 0 and divide n_qh");
    if (block_size < 4 || block_size > 4096 || (block_size & (block_size - 1)))
        return fail(SW_ERR_UNSUPPORTED, "block_size must be a power of two in [4, 4096]");
    if (max_blocks <= 0 || n_blocks <= 0) return fail(SW_ERR_SHAPE, "max_blocks and n_blocks must be > 0");
    if ((long long)max_blocks * block_size > (1 << 23))
        return fail(SW_ERR_SHAPE, "max_blocks * block_size above 2^23");
    const int max_len = max_blocks * block_size;
    int rc = check_shape(n_req, n_kvh, head_dim, max_len);
    if (rc != SW_OK) return rc;
    if (n_qh / n_kvh > 64) return fail(SW_ERR_UNSUPPORTED, "more than 64 query heads per key/value head");
    if ((long long)n_req * n_qh > (1LL << 20)) return fail(SW_ERR_SHAPE, "n_req * n_qh above 2^20");
    if (n_req == 0) return SW_OK;
    if (!q || !k_pool || !v_pool || !block_table || !seq_lens || !out)
        return fail(SW_ERR_NULL, "q, k_pool, v_pool, block_table, seq_lens and out must be non-NULL");
    if (append && (!k_new || !v_new)) return fail(SW_ERR_NULL, "k_new and v_new must be non-NULL");
    if (((uintptr_t)q | (uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)out |
         (uintptr_t)k_new | (uintptr_t)v_new) & 15u)
        return fail(SW_ERR_ALIGN, "q, k_new, v_new, k_pool, v_pool and out must be 16-byte aligned");
    if (((uintptr_t)seq_lens | (uintptr_t)block_table) & 3u)
        return fail(SW_ERR_ALIGN, "seq_lens and block_table must be 4-byte aligned");

    StepIn in;
    in.q = q; in.k = k_pool; in.v = v_pool; in.seq_lens = seq_lens; in.out = out;
    in.k_new = k_new; in.v_new = v_new;
    in.n_req = n_req; in.n_qh = n_qh; in.n_kvh = n_kvh; in.head_dim = head_dim; in.max_len = max_len;
    in.block_table = block_table; in.block_size = block_size; in.max_blocks = max_blocks; in.n_blocks = n_blocks;
    in.stream = (hipStream_t)stream_v;
    return run_step(in);
}

int sw_decode_attn_paged(const void *q, const void *k_pool, const void *v_pool,
                         const int32_t *block_table, const int32_t *seq_lens, void *out,
                         int n_req, int n_qh, int n_kvh, int head_dim,
                         int block_size, int max_blocks, int n_blocks, void *stream)
{
    return decode_paged(q, nullptr, nullptr, false, k_pool, v_pool, block_table, seq_lens, out,
                        n_req, n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks, stream);
}

int sw_decode_attn_paged_append(const void *q, const void *k_new, const void *v_new,
                                void *k_pool, void *v_pool,
                                const int32_t *block_table, const int32_t *seq_lens, void *out,
                                int n_req, int n_qh, int n_kvh, int head_dim,
                                int block_size, int max_blocks, int n_blocks, void *stream)
{
    return decode_paged(q, k_new, v_new, true, k_pool, v_pool, block_table, seq_lens, out,
                        n_req, n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks, stream);
}

}  // extern "C"
