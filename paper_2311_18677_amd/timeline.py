"""Per-workgroup phase timeline of the token-phase kernel (a measurement aid).

    python -m paper_2311_18677_amd.timeline --build            # here or on the GPU machine (hipcc)
    python -m paper_2311_18677_amd.timeline --workload NAME    # on the GPU machine

--build makes an instrumented copy of csrc/sw_decode_split.hip: every line of the form
`// -- phase: <name>` in that file becomes a time stamp (the 100 MHz wall clock all XCDs
share, read by the workgroup's first lane and stored to a table indexed by blockIdx.x and
phase), and links it with the library's other objects into libsw_decode_timeline.so.  The
product library is not touched and never contains the stamps.

Without --build the module loads that library, runs the plain decode call on a rotation
of cache sets (as bench.py does, so that the rows come from HBM), and prints, for every
phase, when the workgroups that have work pass it: microseconds after the first
workgroup's start, minimum / 10th percentile / median / 90th percentile / maximum over
the workgroups of several launches, and the same for the time a workgroup spends between
phases.  Each stamp costs the wave a scalar-memory round trip, so intervals are a little
longer than in the product kernel; the picture of who waits where is what it is for.
"""
import argparse
import ctypes
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsw_decode_timeline.so")

# phase comment in the kernel source -> code put in its place (slot = column of the table)
STAMPS = [
    ("workgroup started", "bool tl_once = false; SW_STAMP(0);"),
    ("item known", "SW_STAMP(1);"),
    ("first loads issued", "SW_STAMP(2);"),
    ("K tile landed", "SW_STAMP_ONCE(3); if (!MORE) SW_STAMP(4);"),
    ("V tile landed", "if (!MORE) SW_STAMP(5);"),
    ("tiles done", "SW_STAMP(6);"),
    ("results stored", "__builtin_amdgcn_s_waitcnt(0); SW_STAMP(7);"),
    ("merged", "SW_STAMP(8);"),
]
COLUMNS = ["workgroup started", "item known", "first tile's loads issued", "first K tile landed",
           "last K tile landed", "last V tile landed", "tiles done", "results stored", "end"]
SLOTS = 16
MAX_BLOCKS = 1 << 16

PREAMBLE = r'''
#include <hip/hip_runtime.h>
__device__ unsigned long long *g_sw_tl = nullptr;
extern "C" int sw_tl_set(void *p) { return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_sw_tl), &p, sizeof(p)); }
#define SW_TL_BLOCKS %d
#define SW_STAMP(i) do { const unsigned long long t_ = wall_clock64(); \
    if (threadIdx.x == 0 && g_sw_tl && blockIdx.x < SW_TL_BLOCKS) g_sw_tl[(size_t)blockIdx.x * %d + (i)] = t_; } while (0)
#define SW_STAMP_ONCE(i) do { if (!tl_once) { SW_STAMP(i); tl_once = true; } } while (0)
''' % (MAX_BLOCKS, SLOTS)


def build():
    from . import build as b
    src = open(os.path.join(b.CSRC, "sw_decode_split.hip")).read()
    anchor = '#include "sw_internal.h"'
    src = src.replace(anchor, PREAMBLE + anchor, 1)
    for name, code in STAMPS:
        tag = "// -- phase: " + name
        if src.count(tag) != 1:
            raise RuntimeError("phase comment %r not found exactly once in sw_decode_split.hip" % name)
        src = src.replace(tag, code)
    os.makedirs(b.OBJ_DIR, exist_ok=True)
    gen = os.path.join(b.OBJ_DIR, "sw_decode_split_timeline.hip")
    open(gen, "w").write(src)
    objs = []
    for s in b.SOURCES:
        obj = os.path.join(b.OBJ_DIR, os.path.splitext(s)[0] + (".timeline.o" if s == "sw_decode_split.hip" else ".o"))
        path = gen if s == "sw_decode_split.hip" else os.path.join(b.CSRC, s)
        if s == "sw_decode_split.hip" or not os.path.exists(obj):
            res = subprocess.run([b.HIPCC] + b.FLAGS + ["-c", path, "-o", obj], capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc failed on %s:\n%s" % (s, res.stderr))
        objs.append(obj)
    res = subprocess.run([b.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs,
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    print("built", LIB)


def run(args):
    import numpy as np
    import torch
    from . import binding as sw
    from . import workloads as wl
    if not os.path.exists(LIB):
        raise SystemExit("%s is not built; run `python -m paper_2311_18677_amd.timeline --build`" % LIB)
    sw.LIB_PATH = LIB
    lib = sw.load()
    lib.sw_tl_set.argtypes = [ctypes.c_void_p]
    sw.sw_set_param(sw.SW_PARAM_COMBINE, args.combine)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, args.chunk)
    sw.sw_set_param(sw.SW_PARAM_WAVES, args.waves)
    cfg = wl.CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    lay = sw.sw_kv_layout(cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    sys.path.insert(0, ROOT)
    import bench
    sets = [bench.make_device_set(cfg, lay, wl.BASE_SEED + 77 + i, torch, np, wl, dev) for i in range(args.sets)]
    stream = torch.cuda.Stream()

    def call(s):
        sw.sw_decode_attn(s["q"], s["k_cache"], s["v_cache"], s["seq_lens"], s["out"], cfg.n_req, cfg.n_qh,
                          cfg.n_kvh, cfg.head_dim, cfg.max_len, stream)

    for s in sets:
        call(s)
    stream.synchronize()
    table = torch.zeros(MAX_BLOCKS * SLOTS, dtype=torch.int64, device=dev)
    rows = []
    for rep in range(args.launches + 1):
        s = sets[(rep + 1) % len(sets)]
        call(sets[rep % len(sets)])          # calls right before, as in a running loop
        call(sets[(rep + 2) % len(sets)])
        table.zero_()
        torch.cuda.synchronize()
        assert lib.sw_tl_set(table.data_ptr()) == 0
        call(s)
        stream.synchronize()
        assert lib.sw_tl_set(None) == 0
        t = table.cpu().numpy().reshape(MAX_BLOCKS, SLOTS)
        started = t[:, 0] != 0
        worked = t[:, 6] != 0
        a = (t[worked][:, :len(COLUMNS)] - t[started, 0].min()) * 0.01     # 100 MHz ticks -> microseconds
        if rep == 0:
            print("workload %s: %d workgroups launched, %d with work, K/V bytes %d" %
                  (args.workload, int(started.sum()), int(worked.sum()), s["kv_bytes"]))
            continue                          # the first instrumented launch is warm-up
        rows.append(a)
        print("launch %d: last workgroup ends %.2f us after the first one starts" % (rep, a[:, 8].max()))
    a = np.concatenate(rows)
    print("when the workgroups that have work pass each phase (stamp of the workgroup's first wave), microseconds "
          "after the launch's first workgroup starts; %d launches, n = %d" % (args.launches, len(a)))
    print("  %-28s %7s %7s %7s %7s %7s" % ("phase", "min", "p10", "median", "p90", "max"))
    for i, n in enumerate(COLUMNS):
        v = a[:, i]
        print("  %-28s %7.2f %7.2f %7.2f %7.2f %7.2f" % (n, v.min(), np.percentile(v, 10), np.median(v),
                                                         np.percentile(v, 90), v.max()))
    print("time a workgroup spends between phases, microseconds")
    for (i, j) in ((0, 1), (1, 2), (2, 3), (3, 5), (4, 5), (5, 6), (6, 7), (7, 8), (5, 8), (0, 8)):
        v = a[:, j] - a[:, i]
        print("  %-28s -> %-28s %7.2f %7.2f %7.2f %7.2f %7.2f" % (COLUMNS[i], COLUMNS[j], v.min(), np.percentile(v, 10),
                                                                  np.median(v), np.percentile(v, 90), v.max()))


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--build", action="store_true")
    ap.add_argument("--workload", default="llama70b_tp8")
    ap.add_argument("--combine", type=int, default=1, help="SW_PARAM_COMBINE (1 = two kernels, 2 = single launch)")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--sets", type=int, default=6)
    ap.add_argument("--launches", type=int, default=10)
    args = ap.parse_args()
    if args.build:
        return build()
    run(args)


if __name__ == "__main__":
    main()
