// Workgroup -> work item mapping of the partial kernels.
//
// A work item is one chunk of one (request, key/value head).  How many items a
// request has depends on its length, which only the device knows, so the grid
// workgroups find their items themselves: the items are numbered request by
// request (request r owns n_kvh * ceil(L_r / chunk) consecutive numbers,
// key/value head major, chunk minor), and workgroup b takes items b,
// b + gridDim.x, ... up to the last one.  Compared with mapping blockIdx
// straight onto (request, head, chunk) no launched workgroup is empty once the
// grid is no larger than what the device holds at a time.
//
// Every wave computes the mapping on its own (no LDS, no barrier): a lane
// holds up to kMaxPerLane consecutive requests, the per-lane counts are
// prefix-summed across the wave with DPP, and a ballot finds the owning lane.
// Batches of more than 64 * kMaxPerLane requests use the direct mapping.
#pragma once
#include "sw_internal.h"

struct SwWork {
    int  r;       // request
    int  g;       // key/value head
    int  c;       // chunk index
    int  L;       // number of positions request r attends over
    int  new_pos; // append variant: position this call stores the newest rows at, else -1
    bool valid;   // false: this workgroup has nothing to do
};

constexpr int kSwMaxPerLane   = 16;
constexpr int kSwMaxScanReqs  = 64 * kSwMaxPerLane;

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ int sw_wave_inclusive_scan(int x)
{
    // within rows of 16 lanes: lanes shifted in from outside the row read 0
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);   // row_shr:1
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);   // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);   // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);   // row_shr:8
    // across rows: lane 15 of a row into rows 1 and 3, then lane 31 into rows 2 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);  // row_bcast:15
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);  // row_bcast:31
    return x;
}

// PER = requests held per lane (1, 4 or 16; 0 selects the direct mapping).
// The chunk length is a power of two, and the host keeps
// n_req * n_kvh * n_chunks below 2^31, so item numbers fit 32 bits.
//
// The lookup is split in two so that a workgroup that walks several items
// (item b, b + gridDim.x, ...) reads the lengths only once: sw_scan_lens leaves
// each lane with its requests' lengths and chunk counts and the wave-wide prefix
// sum, sw_lookup finds an item from that state with a ballot and lane reads.
// Both must be called by all 64 lanes of a wave.
template <int PER>
struct SwScan {
    int len[PER > 0 ? PER : 1];
    int cnt[PER > 0 ? PER : 1];
    int mine;          // chunks of this lane's requests
    int incl;          // chunks of all requests up to this lane's last
    unsigned total;    // number of item slots to walk (for PER > 0: exactly the real items)
};

// The lane's lengths as they lie in memory: sw_scan_issue requests them (all of them before
// anything else is looked at) and sw_scan_finish turns them into the scan state, so a caller
// can put work that does not depend on the lengths between the two.
template <int PER>
struct SwRawLens {
    int v[PER > 0 ? PER : 1];
};

template <int PER>
__device__ __forceinline__ SwRawLens<PER> sw_scan_issue(const SwArgs &a)
{
    SwRawLens<PER> raw;
    raw.v[0] = 0;
    if constexpr (PER > 0) {
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int r = lane * PER + j;
            raw.v[j] = r < a.n_req ? a.seq_lens[r] : 0;
        }
    }
    return raw;
}

template <int PER>
__device__ __forceinline__ SwScan<PER> sw_scan_finish(const SwArgs &a, const SwRawLens<PER> &raw)
{
    SwScan<PER> s;
    if constexpr (PER == 0) {
        s.len[0] = s.cnt[0] = s.mine = s.incl = 0;
        s.total = (unsigned)a.n_req * (unsigned)a.n_kvh * (unsigned)a.n_chunks;
    } else {
        const int lane = threadIdx.x & 63;
        s.mine = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int r = lane * PER + j;
            s.len[j] = r < a.n_req ? sw_flag_len(a, r, raw.v[j]) : 0;
            s.cnt[j] = ((s.len[j] & kSwLenMask) + a.chunk - 1) >> a.chunk_shift;
            s.mine += s.cnt[j];
        }
        s.incl = sw_wave_inclusive_scan(s.mine);
        s.total = (unsigned)__builtin_amdgcn_readlane(s.incl, 63) * (unsigned)a.n_kvh;
    }
    return s;
}

template <int PER>
__device__ __forceinline__ SwScan<PER> sw_scan_lens(const SwArgs &a)
{
    const SwRawLens<PER> raw = sw_scan_issue<PER>(a);
    return sw_scan_finish<PER>(a, raw);
}

template <int PER>
__device__ __forceinline__ SwWork sw_lookup(const SwArgs &a, const SwScan<PER> &s, unsigned b)
{
    SwWork w;
    w.valid = false;
    w.r = w.g = w.c = w.L = 0;
    w.new_pos = -1;
    if constexpr (PER == 0) {
        // direct mapping: b = c * n_units + unit
        const unsigned n_units = (unsigned)a.n_req * (unsigned)a.n_kvh;
        const unsigned c = b / n_units, unit = b - c * n_units;
        w.r = (int)(unit / (unsigned)a.n_kvh);
        w.g = (int)(unit - (unsigned)w.r * (unsigned)a.n_kvh);
        w.c = (int)c;
        const int lf = sw_request_len_flagged(a, w.r);
        w.L = lf & kSwLenMask;
        if ((lf >> kSwAppendedBit) & 1) w.new_pos = w.L - 1;
        w.valid = ((long long)w.c << a.chunk_shift) < w.L;
        return w;
    } else {
        const unsigned long long hit = __ballot((unsigned)s.incl * (unsigned)a.n_kvh > b);
        if (hit == 0) return w;                          // past the last item
        const int owner = __builtin_ctzll(hit);          // first lane whose range reaches item b
        unsigned before = (unsigned)__builtin_amdgcn_readlane(s.incl - s.mine, owner);   // chunks before the owner's requests
        bool found = false;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const unsigned cj = (unsigned)__builtin_amdgcn_readlane(s.cnt[j], owner);
            const int lj = __builtin_amdgcn_readlane(s.len[j], owner);
            if (!found && (before + cj) * (unsigned)a.n_kvh > b) {
                const unsigned rem = b - before * (unsigned)a.n_kvh;   // < cj * n_kvh
                // the clamps below change nothing when the scan is right; they keep
                // every later address in bounds whatever the lanes delivered
                const unsigned gg = a.n_kvh == 1 ? 0u : rem / (cj ? cj : 1u);
                w.r = max(0, min(owner * PER + j, a.n_req - 1));
                w.g = (int)min(gg, (unsigned)(a.n_kvh - 1));
                w.c = (int)(rem - (unsigned)w.g * cj) & 0x7fffffff;
                w.L = min(lj & kSwLenMask, a.max_len);
                if (((lj >> kSwAppendedBit) & 1) && w.L > 0) w.new_pos = w.L - 1;
                w.valid = ((long long)w.c << a.chunk_shift) < w.L;
                found = true;
            }
            before += cj;
        }
        return w;
    }
}

// Flagged length of request req (see sw_request_len_flagged) from a finished scan; all 64
// lanes of the wave must call it.  The direct mapping keeps no lengths and reads memory.
template <int PER>
__device__ __forceinline__ int sw_scanned_len(const SwArgs &a, const SwScan<PER> &s, int req)
{
    if constexpr (PER == 0) {
        return sw_request_len_flagged(a, req);
    } else {
        const int owner = req / PER, j = req - owner * PER;
        int v = s.len[0];
#pragma unroll
        for (int k = 1; k < PER; ++k) v = j == k ? s.len[k] : v;
        return __builtin_amdgcn_readlane(v, owner);
    }
}

// One-item form: workgroup b handles item b only.
template <int PER>
__device__ __forceinline__ SwWork sw_find_work(const SwArgs &a, unsigned b)
{
    const SwScan<PER> s = sw_scan_lens<PER>(a);
    return sw_lookup<PER>(a, s, b);
}

// Which mapping the host picks for a batch size.
static inline int sw_worklist_per(int n_req)
{
    return n_req <= 64 ? 1 : (n_req <= 256 ? 4 : (n_req <= kSwMaxScanReqs ? kSwMaxPerLane : 0));
}
