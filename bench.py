#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

A "step" is one sw_decode_attn call: one layer's decode attention for the whole
batch (both kernels).  Inputs are resident in HBM before the timed region; the
calls rotate over several distinct cache sets so that the K/V rows come from
HBM, not from the last-level cache.  One JSON line is printed.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

The K steps are launched as HIP-graph replays (whole rotations, plus one graph for
a remainder) and timed with HIP events recorded on the stream they run on; they
are run --repeats times and the median repeat is reported (minimum beside it).
After the headline workload the other workloads are run briefly the same way and
reported in the line's `configs` array.

--append times the append-then-attend entry point instead (same rotation, the
newest rows rewritten in place every call).  --decode-loop runs whole model
steps: one append-then-attend call per layer over that many per-layer caches
sharing one length array, then sw_advance_lens; a "step" is still one layer call.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
LLC_BYTES = 256 << 20           # last-level (Infinity) cache the rotation must exceed 4x


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--workload", default="llama70b_tp8")
    ap.add_argument("--sets", type=int, default=0, help="distinct cache sets (0 = enough for 4x the LLC)")
    ap.add_argument("--mode", default="graph", choices=["graph", "eager"],
                    help="graph: replay a HIP graph of one rotation; eager: one host call per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-read-ceiling", action="store_true",
                    help="skip the plain streaming-read kernel timed beside the call (same byte count)")
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--combine", type=int, default=0)
    ap.add_argument("--paged", type=int, default=0, metavar="BLOCK",
                    help="run the block-table variant with this block size (0 = dense layout)")
    ap.add_argument("--append", action="store_true",
                    help="time sw_decode_attn_append / sw_decode_attn_paged_append")
    ap.add_argument("--decode-loop", action="store_true",
                    help="whole model steps: the workload's layer count of per-layer caches, one "
                         "append-then-attend call each, lengths advanced on the device per step")
    ap.add_argument("--prefill", action="store_true",
                    help="time the prompt-phase (causal) attention instead; workloads prefill_*")
    ap.add_argument("--handoff", action="store_true",
                    help="time the KV hand-off copy (block pools -> dense) instead; uses --paged "
                         "BLOCK (default 16)")
    ap.add_argument("--prefill-heads", type=int, default=0)
    ap.add_argument("--prefill-waves", type=int, default=0)
    ap.add_argument("--prefill-kernel", type=int, default=0)
    ap.add_argument("--repeats", type=int, default=5,
                    help="the K timed steps are run this many times; ms_per_step is the median")
    ap.add_argument("--no-configs", action="store_true",
                    help="leave out the short runs of the other workloads (the `configs` array)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also launch plain device copies of this size (for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings); 0 = none")
    return ap.parse_args()


def add_new_rows(bufs, cfg, g, torch, dev):
    """The newest token's K and V rows for the append variants, N(0,1) like the cache."""
    for name in ("k_new", "v_new"):
        t = torch.empty(cfg.n_req * cfg.n_kvh * cfg.head_dim, dtype=torch.float16, device=dev)
        t.normal_(0.0, 1.0, generator=g)
        bufs[name] = t


def make_device_set(cfg, lay, seed, torch, np, wl, dev, lens=None):
    """A cache set generated on the device: same shapes, lengths from the config's
    recipe (or the ones given), values N(0,1) in binary16 (every position, so padding
    is arbitrary data)."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence(int(seed))))
    if lens is None:
        lens = wl.draw_seq_lens(cfg, rng)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    bufs = {}
    for name in ("k_cache", "v_cache"):
        t = torch.empty(lay.total_elems, dtype=torch.float16, device=dev)
        t.normal_(0.0, 1.0, generator=g)
        bufs[name] = t
    if cfg.k_row_scale:
        prob, factor = cfg.k_row_scale
        rows = bufs["k_cache"].view(-1, cfg.head_dim)
        hit = torch.rand(rows.shape[0], device=dev, generator=g) < prob
        rows[hit] *= factor
    q = torch.empty(cfg.n_req * cfg.n_qh * cfg.head_dim, dtype=torch.float16, device=dev)
    q.normal_(0.0, 1.0, generator=g)
    bufs["q"] = q
    bufs["seq_lens"] = torch.from_numpy(lens).to(dev)
    bufs["out"] = torch.zeros((cfg.n_req, cfg.n_qh, cfg.head_dim), dtype=torch.float16, device=dev)
    valid = np.clip(lens, 0, cfg.max_len).astype(np.int64)
    bufs["kv_bytes"] = int(valid.sum()) * cfg.n_kvh * cfg.head_dim * 4
    add_new_rows(bufs, cfg, g, torch, dev)
    return bufs


def make_paged_set(cfg, block_size, seed, torch, np, wl, sw, dev, lens=None, room=0):
    """A block-table cache set generated on the device: pools of exactly the blocks the
    lengths (plus `room` further positions) need, plus 3, values N(0,1), a seeded random
    block assignment."""
    rng = np.random.Generator(np.random.Philox(np.random.SeedSequence(int(seed))))
    if lens is None:
        lens = wl.draw_seq_lens(cfg, rng)
    valid = np.clip(lens, 0, cfg.max_len).astype(np.int64)
    per_req = -(-np.minimum(valid + room, cfg.max_len) // block_size)
    n_blocks = int(per_req.sum()) + 3
    max_blocks = -(-cfg.max_len // block_size)
    lay = sw.sw_kv_paged_layout(n_blocks, cfg.n_kvh, cfg.head_dim, block_size)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    bufs = {"block_size": block_size, "max_blocks": max_blocks, "n_blocks": n_blocks}
    for name in ("k_pool", "v_pool"):
        t = torch.empty(lay.total_elems, dtype=torch.float16, device=dev)
        t.normal_(0.0, 1.0, generator=g)
        bufs[name] = t
    if cfg.k_row_scale:
        prob, factor = cfg.k_row_scale
        rows = bufs["k_pool"].view(-1, cfg.head_dim)
        hit = torch.rand(rows.shape[0], device=dev, generator=g) < prob
        rows[hit] *= factor
    order = rng.permutation(n_blocks)
    table = np.full((cfg.n_req, max_blocks), 0x3FFFFFF0, dtype=np.int32)
    nxt = 0
    for r in range(cfg.n_req):
        table[r, :per_req[r]] = order[nxt:nxt + per_req[r]]
        nxt += int(per_req[r])
    q = torch.empty(cfg.n_req * cfg.n_qh * cfg.head_dim, dtype=torch.float16, device=dev)
    q.normal_(0.0, 1.0, generator=g)
    bufs["q"] = q
    bufs["block_table"] = torch.from_numpy(table).to(dev)
    bufs["seq_lens"] = torch.from_numpy(lens).to(dev)
    bufs["out"] = torch.zeros((cfg.n_req, cfg.n_qh, cfg.head_dim), dtype=torch.float16, device=dev)
    bufs["kv_bytes"] = int(valid.sum()) * cfg.n_kvh * cfg.head_dim * 4
    add_new_rows(bufs, cfg, g, torch, dev)
    return bufs


def read_traffic(workload, summary=None):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc
    summary for this workload (profiles/pmc_<workload>.txt, or a line naming the workload
    in the summary file given), or None."""
    path = os.path.join(ROOT, "profiles", summary or "pmc_%s.txt" % workload)
    key = "hbm_bytes_per_launch %s:" % workload if summary else "hbm_bytes_per_launch:"
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 matrix peak


def stream_read_ceiling(sw, torch, n_bytes, dev, launches=400):
    """What a kernel that only reads n_bytes from HBM achieves on this machine: the practical
    ceiling for a call bound by such a read.  Rotates over buffers worth four times the
    last-level cache, as the timed path does; returns per-launch figures (HIP-graph replays
    for the call time, HIP events on the dispatch for the kernel time)."""
    n_bytes = max(16, int(n_bytes) // 16 * 16)
    n_bufs = int(max(2, min(64, -(-4 * LLC_BYTES // n_bytes))))
    bufs = [torch.empty(n_bytes // 4, dtype=torch.int32, device=dev).random_() for _ in range(n_bufs)]
    sink = torch.zeros(16384, dtype=torch.int32, device=dev)
    stream = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    sw.sw_stream_read(bufs[0], n_bytes, sink, 0, stream)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for b in bufs:
            sw.sw_stream_read(b, n_bytes, sink, 0, torch.cuda.current_stream())
    torch.cuda.synchronize()
    reps = max(2, launches // n_bufs)
    with torch.cuda.stream(stream):
        graph.replay()

    def replays():
        with torch.cuda.stream(stream):
            for _ in range(reps):
                graph.replay()

    call_us = min(time_on_stream(torch, stream, replays)[0] for _ in range(3)) / (reps * n_bufs) * 1e3
    n_prof = min(launches, 4 * n_bufs)
    sw.sw_prof_start(n_prof)
    for i in range(n_prof):
        sw.sw_stream_read(bufs[i % n_bufs], n_bytes, sink, 0, stream)
    k_us, _, n_rec = sw.sw_prof_stop()
    kernel_us = k_us / max(n_rec, 1)
    del bufs
    # the same kernel over one 2 GiB buffer: what streaming reads reach when launch and tail
    # no longer count
    big_bytes = 2 << 30
    big = torch.empty(big_bytes // 4, dtype=torch.int32, device=dev).random_()
    sw.sw_stream_read(big, big_bytes, sink, 0, stream)
    stream.synchronize()
    sw.sw_prof_start(5)
    for _ in range(5):
        sw.sw_stream_read(big, big_bytes, sink, 0, stream)
    b_us, _, b_rec = sw.sw_prof_stop()
    big_us = b_us / max(b_rec, 1)
    del big
    torch.cuda.empty_cache()
    return {"bytes": n_bytes, "buffers": n_bufs, "call_us": call_us, "call_GBps": n_bytes / call_us / 1e3,
            "kernel_us": kernel_us, "kernel_GBps": n_bytes / kernel_us / 1e3 if kernel_us > 0 else 0.0,
            "large_read_bytes": big_bytes, "large_read_us": big_us,
            "large_read_GBps": big_bytes / big_us / 1e3 if big_us > 0 else 0.0,
            "what": "sw_stream_read: one plain kernel that reads this many bytes once (grid-stride, "
                    "16 B per lane, 8 loads in flight); a reference point, not a proven ceiling. "
                    "large_read: the same kernel over one 2 GiB buffer"}


def main_prefill(args):
    """Prompt-phase attention: a step is one sw_prefill_attn call (one layer, one prompt batch)."""
    import numpy as np
    import torch
    from paper_2311_18677_amd import binding as sw
    from paper_2311_18677_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    sw.load()
    sw.sw_set_param(sw.SW_PARAM_PREFILL_HEADS, args.prefill_heads)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, args.prefill_waves)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, args.prefill_kernel)
    mixed = args.workload.startswith("mixed_")
    if mixed:
        # prompt and token phases of different requests in one call (sw_mixed_attn)
        name = args.workload
        cfg = wl.MIXED_CONFIGS[name][0]
        batch0, qlens0 = wl.make_mixed_batch(name)
        qt0, starts0, qlens0 = wl.make_mixed_queries(batch0, qlens0)
        flops = wl.mixed_flops(cfg, batch0.seq_lens, qlens0)
        max_q = int(qlens0.max())
    else:
        name = args.workload if args.workload.startswith("prefill_") else "prefill_llama70b_tp8"
        cfg = wl.PREFILL_CONFIGS[name]
        batch0 = wl.make_batch(cfg)
        qt0, starts0 = wl.make_prefill_queries(batch0)
        flops = wl.prefill_flops(cfg, batch0.seq_lens)
    n_tokens = qt0.shape[0]
    n_sets = args.sets or 4
    sets = []
    for i in range(n_sets):
        # the other sets: the same lengths (so that one q_starts array serves all), other values
        b = batch0 if i == 0 else wl.make_batch(cfg, seed=batch0.seed + 100 + i,
                                                seq_lens=list(batch0.seq_lens) if mixed else None)
        if mixed:
            qt = qt0 if i == 0 else wl.make_mixed_queries(b, qlens0)[0]
        else:
            qt = qt0 if i == 0 else wl.make_prefill_queries(b)[0]
        if args.paged:
            bufs = sw.upload_paged_batch(b, args.paged, device="cuda:0", pad_bits=0, seed=i)
        else:
            bufs = sw.upload_batch(b, device="cuda:0", pad_bits=0)
        bufs["qt"] = torch.from_numpy(qt.view(np.int16).reshape(-1)).to(dev).view(torch.float16)
        bufs["starts"] = torch.from_numpy(starts0).to(dev)
        if mixed:
            bufs["qlens"] = torch.from_numpy(qlens0).to(dev)
        bufs["pout"] = torch.zeros((n_tokens, cfg.n_qh, cfg.head_dim), dtype=torch.float16, device=dev)
        if i:
            bufs.pop("k_host"), bufs.pop("v_host")
        sets.append(bufs)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        if args.paged and mixed:
            sw.sw_mixed_attn_paged(s["qt"], s["k_pool"], s["v_pool"], s["block_table"], s["seq_lens"],
                                   s["starts"], s["qlens"], s["pout"], n_tokens, cfg.n_req, cfg.n_qh,
                                   cfg.n_kvh, cfg.head_dim, s["block_size"], s["max_blocks"],
                                   s["n_blocks"], max_q, st)
        elif args.paged:
            sw.sw_prefill_attn_paged(s["qt"], s["k_pool"], s["v_pool"], s["block_table"], s["seq_lens"],
                                     s["starts"], s["pout"], n_tokens, cfg.n_req, cfg.n_qh, cfg.n_kvh,
                                     cfg.head_dim, s["block_size"], s["max_blocks"], s["n_blocks"], st)
        elif mixed:
            sw.sw_mixed_attn(s["qt"], s["k_cache"], s["v_cache"], s["seq_lens"], s["starts"], s["qlens"],
                             s["pout"], n_tokens, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim,
                             cfg.max_len, max_q, st)
        else:
            sw.sw_prefill_attn(s["qt"], s["k_cache"], s["v_cache"], s["seq_lens"], s["starts"], s["pout"],
                               n_tokens, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, st)

    call(sets[0], stream)
    stream.synchronize()
    steps, warmup = args.steps, args.warmup
    graph = None
    mode = args.mode
    if mode == "graph":
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for s in sets:
                    call(s, torch.cuda.current_stream())
            torch.cuda.synchronize()
        except Exception as e:      # noqa: BLE001
            print("bench.py: graph capture failed (%s); using eager launches" % e, file=sys.stderr)
            graph, mode = None, "eager"

    def run_steps(n):
        if graph is not None:
            full, rem = divmod(n, n_sets)
            with torch.cuda.stream(stream):
                for _ in range(full):
                    graph.replay()
            for i in range(rem):
                call(sets[i], stream)
            return
        for i in range(n):
            call(sets[i % n_sets], stream)

    run_steps(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    prof_calls = min(steps, 200)
    sw.sw_prof_start(prof_calls * (2 if mixed else 1))
    for i in range(prof_calls):
        call(sets[i % n_sets], stream)
    k_us_sum, c_us_sum, n_rec = sw.sw_prof_stop()
    if mixed:
        # two records per call: the token-phase kernels (partial + merge), then the prompt kernel
        kernel_us = (k_us_sum + c_us_sum) / prof_calls
        n_rec = prof_calls
    else:
        kernel_us = k_us_sum / max(n_rec, 1)
    achieved = flops / (kernel_us * 1e-6) / 1e12 if kernel_us > 0 else 0.0

    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        lay = sets[0]["layout"]
        # A bounded sample of the same workload: the last S query tokens of every request
        # (the expensive ones), S the largest that keeps the oracle near twenty seconds.
        nq_all = np.asarray(qlens0 if mixed else np.clip(batch0.seq_lens, 0, cfg.max_len), dtype=np.int64)
        budget = 2.5e10
        lo_s, hi_s = 1, int(max(nq_all.max(), 1))
        while lo_s < hi_s:
            mid = (lo_s + hi_s + 1) // 2
            if wl.mixed_flops(cfg, batch0.seq_lens, np.minimum(nq_all, mid)) <= budget:
                lo_s = mid
            else:
                hi_s = mid - 1
        nq_s = np.minimum(nq_all, lo_s).astype(np.int32)
        starts_s = (np.asarray(starts0, dtype=np.int64) + nq_all - nq_s).astype(np.int32)
        flops_s = wl.mixed_flops(cfg, batch0.seq_lens, nq_s)
        c0 = time.perf_counter()
        if args.paged:
            s0 = sets[0]
            pl = s0["layout"]
            ref = oracle.mixed_attn_paged(qt0, s0["k_host"], s0["v_host"], s0["table_host"],
                                          batch0.seq_lens, starts_s, nq_s, cfg.n_req,
                                          cfg.n_qh, cfg.n_kvh, cfg.head_dim, s0["block_size"],
                                          s0["max_blocks"], s0["n_blocks"], cfg.max_len,
                                          pl.stride_block, pl.stride_kvh, pl.stride_tok)
            used = oracle.max_threads()
        else:
            ref, used = oracle.mixed_attn(qt0, sets[0]["k_host"], sets[0]["v_host"], batch0.seq_lens,
                                          starts_s, nq_s, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim,
                                          cfg.max_len, cfg.max_len, lay.stride_req, lay.stride_kvh,
                                          lay.stride_tok, return_threads=True)
        t_cpu = time.perf_counter() - c0
        rows = np.zeros(n_tokens, dtype=bool)
        for r in range(cfg.n_req):
            rows[starts_s[r]:starts_s[r] + nq_s[r]] = True
        whole = bool((nq_s == nq_all).all())
        cpu_baseline = {"value": flops_s / t_cpu / 1e12, "unit": "TFLOP/s", "cores": int(used),
                        "kind": "oracle",
                        "sample": "set 0 of %s, %s (%d of %d query tokens, %.2f of %.2f GFLOP), once, %.1f s"
                                  % (cfg.name, "the whole batch" if whole else
                                     "the last %d query tokens of every request" % lo_s,
                                     int(rows.sum()), n_tokens, flops_s / 1e9, flops / 1e9, t_cpu)}
        call(sets[0], stream)
        stream.synchronize()
        out = sets[0]["pout"].cpu().numpy().astype(np.float64)[rows]
        ref = ref[rows]
        diff = out - ref
        den = np.sqrt((ref ** 2).sum(-1))
        rel = np.sqrt((diff ** 2).sum(-1)) / np.where(den == 0, 1.0, den)
        parity = {"max_abs": float(np.abs(diff).max()), "max_row_rel_l2": float(rel.max()),
                  "rows_checked": int(rows.sum())}

    tflops = flops * steps / elapsed / 1e12
    line = {
        "metric": "prompt-phase attention TFLOP/s (causal pairs only; % of MI355X fp16 matrix peak)",
        "value": tflops, "unit": "TFLOP/s", "pct_of_peak": 100.0 * tflops / MFMA_F16_PEAK_TFLOPS,
        "prompt_tokens_per_s_attention_only": n_tokens * steps / elapsed / cfg.n_layers,
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * elapsed / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "accumulate": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "n_req": cfg.n_req, "n_qh": cfg.n_qh, "n_kvh": cfg.n_kvh,
                   "head_dim": cfg.head_dim, "max_len": cfg.max_len, "lens": str(cfg.lens),
                   "prompt_tokens": n_tokens, "flops_per_step": flops, "cache_sets": n_sets,
                   "launch": mode, "entry_point": "sw_prefill_attn" + ("_paged" if args.paged else ""),
                   "kv_layout": ("block pools, block_size %d" % args.paged) if args.paged
                   else "dense, padded to max_len"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_F16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_F16_PEAK_TFLOPS,
                     "traffic": None if args.paged else read_traffic(cfg.name, "pmc_prefill.txt"),
                     "kernel": "prompt kernel (sw_prefill_split_kernel below about 77000 query tokens x heads, "
                               "sw_prefill_mfma_kernel from there)", "kernel_us": kernel_us,
                     "flops_per_launch": flops, "launches_timed": n_rec},
        "cpu_baseline": cpu_baseline,
        "parity_set0": parity,
    }
    if mixed:
        # The token-phase requests dominate the bytes, the prompt the flops: the call is
        # priced against the HBM roofline on the K/V rows every request reads once (+ q, out),
        # and the flops are reported beside it.
        kv = int(batch0.kv_bytes) + 2 * 2 * n_tokens * cfg.n_qh * cfg.head_dim
        gbps = kv / (kernel_us * 1e-6) / 1e9 if kernel_us > 0 else 0.0
        line["metric"] = "mixed-batch attention calls per second (one layer; prompt and token phases in one call)"
        line["value"] = steps / elapsed
        line["unit"] = "calls/s"
        line.pop("pct_of_peak")
        line.pop("prompt_tokens_per_s_attention_only")
        line["config"]["entry_point"] = "sw_mixed_attn" + ("_paged" if args.paged else "")
        line["config"]["query_tokens"] = n_tokens
        line["config"]["prompt_requests"] = int((qlens0 > 1).sum())
        line["config"]["algorithmic_bytes_per_step"] = kv
        line["roofline"] = {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                            "frac": gbps / HBM_PEAK_GBPS, "traffic": None,
                            "kernel": "token-phase partial kernel, then the prompt kernel with the merge of the token-phase "
                                      "chunks riding along (sum of the kernels' times)",
                            "kernel_us": kernel_us, "bytes_per_launch": kv, "launches_timed": n_rec,
                            "tflops": achieved}
        if cpu_baseline:
            cpu_baseline["value"] = flops_s / flops / t_cpu
            cpu_baseline["unit"] = "calls/s (sample time scaled by its share of the flops)"
    print(json.dumps(line))


def main_handoff(args):
    """KV hand-off packing: a step is one sw_kv_pack call (one layer of one batch, pools -> dense)."""
    import numpy as np
    import torch
    from paper_2311_18677_amd import binding as sw
    from paper_2311_18677_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    sw.load()
    cfg = wl.CONFIGS[args.workload]
    bs = args.paged or 16
    lay = sw.sw_kv_layout(cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    batch0 = wl.make_batch(cfg)
    set0 = sw.upload_paged_batch(batch0, bs, device="cuda:0", pad_bits=0)
    set0["kv_bytes"] = batch0.kv_bytes
    # the copy reads and writes every byte: the rotation must exceed the LLC on both sides
    n_sets = args.sets or max(2, -(-4 * LLC_BYTES // max(2 * batch0.kv_bytes, 1)))
    sets = [set0]
    for i in range(1, n_sets):
        sets.append(make_paged_set(cfg, bs, wl.BASE_SEED + 1000 * cfg.seed_index + i, torch, np, wl, sw, dev))
    for s in sets:
        s["k_dense"] = torch.zeros(lay.total_elems, dtype=torch.float16, device=dev)
        s["v_dense"] = torch.zeros(lay.total_elems, dtype=torch.float16, device=dev)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        sw.sw_kv_pack(s["k_pool"], s["v_pool"], s["block_table"], s["seq_lens"], s["k_dense"],
                      s["v_dense"], cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len, bs,
                      s["max_blocks"], s["n_blocks"], st)

    call(sets[0], stream)
    stream.synchronize()
    steps, warmup = args.steps, args.warmup
    graph, mode = None, args.mode
    if mode == "graph":
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for s in sets:
                    call(s, torch.cuda.current_stream())
            torch.cuda.synchronize()
        except Exception as e:      # noqa: BLE001
            print("bench.py: graph capture failed (%s); using eager launches" % e, file=sys.stderr)
            graph, mode = None, "eager"

    def run_steps(n):
        if graph is not None:
            full, rem = divmod(n, n_sets)
            with torch.cuda.stream(stream):
                for _ in range(full):
                    graph.replay()
            for i in range(rem):
                call(sets[i], stream)
            return
        for i in range(n):
            call(sets[i % n_sets], stream)

    run_steps(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    moved = 2 * sum(sets[i % n_sets]["kv_bytes"] for i in range(steps))      # read + written

    prof_calls = 50 * n_sets                 # whatever K is: a series long enough to be back to back
    sw.sw_prof_start(prof_calls)
    for i in range(prof_calls):
        call(sets[i % n_sets], stream)
    k_us_sum, _, n_rec = sw.sw_prof_stop()
    kernel_us = k_us_sum / max(n_rec, 1)
    prof_bytes = 2 * sum(sets[i % n_sets]["kv_bytes"] for i in range(n_rec)) / max(n_rec, 1)
    achieved = prof_bytes / (kernel_us * 1e-6) / 1e9 if kernel_us > 0 else 0.0

    cpu_baseline, parity = None, None
    if not args.no_cpu_baseline:
        import oracle
        pl = set0["layout"]
        kd = np.zeros(lay.total_elems, np.uint16)
        vd = np.zeros(lay.total_elems, np.uint16)
        reps, t_cpu = 0, 0.0
        while t_cpu < 10.0 and reps < 200:
            c0 = time.perf_counter()
            oracle.kv_pack(set0["k_host"], set0["v_host"], set0["table_host"], batch0.seq_lens, kd, vd,
                           True, cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len, bs, set0["max_blocks"],
                           set0["n_blocks"], pl.stride_block, pl.stride_kvh, lay.stride_req,
                           lay.stride_kvh, lay.stride_tok)
            t_cpu += time.perf_counter() - c0
            reps += 1
        cpu_baseline = {"value": 2 * batch0.kv_bytes * reps / t_cpu / 1e9, "unit": "GB/s", "cores": 1,
                        "kind": "oracle",
                        "sample": "set 0 of %s (whole batch), %d repetitions, %.1f s" % (cfg.name, reps, t_cpu)}
        set0["k_dense"].zero_(), set0["v_dense"].zero_()
        torch.cuda.synchronize()          # the fills ran on another stream than the call below
        call(set0, stream)
        stream.synchronize()
        same = (np.array_equal(set0["k_dense"].cpu().numpy().view(np.uint16), kd)
                and np.array_equal(set0["v_dense"].cpu().numpy().view(np.uint16), vd))
        parity = {"bit_exact": bool(same)}

    gbps = moved / elapsed / 1e9
    line = {
        "metric": "KV hand-off packing GB/s (bytes read + bytes written; % of MI355X HBM peak)",
        "value": gbps, "unit": "GB/s", "pct_of_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": 1e3 * elapsed / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": cfg.name, "n_req": cfg.n_req, "n_kvh": cfg.n_kvh,
                   "head_dim": cfg.head_dim, "max_len": cfg.max_len, "lens": str(cfg.lens),
                   "block_size": bs, "bytes_moved_per_step": moved / steps, "cache_sets": n_sets,
                   "launch": mode, "entry_point": "sw_kv_pack"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "kernel": "sw_kv_copy_kernel", "kernel_us": kernel_us,
                     "bytes_per_launch": prof_bytes, "launches_timed": n_rec},
        "cpu_baseline": cpu_baseline,
        "parity_set0": parity,
    }
    print(json.dumps(line))


class GraphSteps:
    """Runs exactly n steps as HIP-graph launches on one stream.  A short run (up to
    kOneGraph steps) is ONE graph of exactly n calls walking the rotation; a longer one replays
    a graph of one whole rotation over the cache sets and, for a remainder, a second graph of
    the rotation's first sets.  Nothing is launched eagerly, so every step of a timed region
    is launched the same way.  record(k, stream) enqueues the rotation's first k calls (and
    what follows a whole rotation when k is the number of sets)."""

    kOneGraph = 256

    def __init__(self, torch, stream, n_sets, record):
        self.torch, self.stream, self.n_sets, self.record = torch, stream, n_sets, record
        self.graphs = {}

    def _parts(self, n):
        """(key of the graph, how many replays) in launch order."""
        full, rem = divmod(n, self.n_sets)
        if n <= self.kOneGraph:
            return [(("run", n), 1)] if n else []
        return [(("rot", self.n_sets), full)] + ([(("rot", rem), 1)] if rem else [])

    def graph(self, key):
        if key not in self.graphs:
            kind, n = key
            g = self.torch.cuda.CUDAGraph()
            with self.torch.cuda.graph(g, stream=self.stream):
                st = self.torch.cuda.current_stream()
                if kind == "rot":
                    self.record(n, st)
                else:
                    full, rem = divmod(n, self.n_sets)
                    for _ in range(full):
                        self.record(self.n_sets, st)
                    if rem:
                        self.record(rem, st)
            self.torch.cuda.synchronize()
            self.graphs[key] = g
        return self.graphs[key]

    def prepare(self, *counts):
        for n in counts:
            for key, _ in self._parts(n):
                self.graph(key)

    def run(self, n):
        with self.torch.cuda.stream(self.stream):
            for key, times in self._parts(n):
                g = self.graph(key)
                for _ in range(times):
                    g.replay()


def time_on_stream(torch, stream, launch, lead_in=None):
    """Milliseconds between two HIP events recorded on `stream` right before and right after
    what launch() enqueues there, and the host's wall-clock time around the bracket (with a
    device synchronisation on both sides).  lead_in(), if given, enqueues untimed work (the
    warm-up steps) on the stream right before the first event, so that the timed work is already
    queued when the GPU gets to it and the events see the steps, not the host's launch latency;
    the host's wall-clock time then covers the lead-in as well."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if lead_in is not None:
        lead_in()
    e0.record(stream)
    launch()
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return e0.elapsed_time(e1), 1e3 * (t1 - t0)


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def parity_vs_oracle(np, out, ref):
    diff = out - ref
    den = np.sqrt((ref ** 2).sum(-1))
    rel = np.sqrt((diff ** 2).sum(-1)) / np.where(den == 0, 1.0, den)
    return {"max_abs": float(np.abs(diff).max()), "max_row_rel_l2": float(rel.max())}


def measure_other_config(name, torch, np, sw, wl, dev, steps, warmup, repeats, with_oracle):
    """A short run of another workload on the plain entry point, library defaults: the same
    rotation over cache sets, the same event timing, the same per-dispatch kernel times, and
    set 0 against the oracle."""
    cfg = wl.CONFIGS[name]
    lay = sw.sw_kv_layout(cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    batch0 = wl.make_batch(cfg)
    set0 = sw.upload_batch(batch0, device="cuda:0", pad_bits=0)
    set0["kv_bytes"] = batch0.kv_bytes
    want = -(-4 * LLC_BYTES // max(batch0.kv_bytes, 1))
    n_sets = int(max(2, min(want, 32)))
    sets = [set0]
    for i in range(1, n_sets):
        sets.append(make_device_set(cfg, lay, wl.BASE_SEED + 1000 * cfg.seed_index + i, torch, np, wl, dev))
    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        sw.sw_decode_attn(s["q"], s["k_cache"], s["v_cache"], s["seq_lens"], s["out"],
                          cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, st)

    call(set0, stream)
    stream.synchronize()
    runner = GraphSteps(torch, stream, n_sets, lambda k, st: [call(s, st) for s in sets[:k]])
    runner.prepare(steps, warmup)
    ev_ms = [time_on_stream(torch, stream, lambda: runner.run(steps), lambda: runner.run(warmup))[0]
             for _ in range(repeats)]
    mean_bytes = sum(sets[i % n_sets]["kv_bytes"] for i in range(steps)) / steps
    n_prof = 20 * n_sets
    sw.sw_prof_start(n_prof)
    for i in range(n_prof):
        call(sets[i % n_sets], stream)
    p_us, c_us, n_rec = sw.sw_prof_stop()
    prof_bytes = sum(sets[i % n_sets]["kv_bytes"] for i in range(n_rec)) / max(n_rec, 1)
    partial_us, combine_us = p_us / max(n_rec, 1), c_us / max(n_rec, 1)
    res = {"workload": cfg.name, "steps": steps, "warmup": warmup, "repeats": repeats,
           "cache_sets": n_sets, "llc_resident": bool(want > n_sets),
           "kv_bytes_per_step": mean_bytes,
           "call_us": 1e3 * median(ev_ms) / steps, "call_us_min": 1e3 * min(ev_ms) / steps,
           "GBps": mean_bytes * steps / (median(ev_ms) * 1e-3) / 1e9,
           "kernel_us": partial_us, "combine_us": combine_us,
           "kernel_GBps": prof_bytes / partial_us / 1e3 if partial_us > 0 else 0.0}
    res["kernel_frac"] = res["kernel_GBps"] / HBM_PEAK_GBPS
    res["traffic"] = read_traffic(cfg.name)
    if with_oracle:
        import oracle
        call(set0, stream)
        stream.synchronize()
        out = set0["out"].cpu().numpy().astype(np.float64)
        c0 = time.perf_counter()
        ref = oracle.decode_attn(batch0.q, set0["k_host"], set0["v_host"], batch0.seq_lens, cfg.n_req,
                                 cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, lay.stride_req,
                                 lay.stride_kvh, lay.stride_tok)
        res["oracle_s"] = time.perf_counter() - c0
        res["parity_set0"] = parity_vs_oracle(np, out, ref)
    del sets, set0, runner
    torch.cuda.empty_cache()
    return res


def oracle_single_thread(np, wl, sw, name="tiny_mha", budget_s=2.0):
    """The oracle on one host thread over the small workload: time per decode step."""
    import oracle
    cfg = wl.CONFIGS[name]
    lay = sw.sw_kv_layout(cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    b = wl.make_batch(cfg)
    k = wl.pack_cache(b.k_rows, cfg, lay.stride_req, lay.stride_kvh, lay.stride_tok, lay.total_elems)
    v = wl.pack_cache(b.v_rows, cfg, lay.stride_req, lay.stride_kvh, lay.stride_tok, lay.total_elems)
    reps, t = 0, 0.0
    while t < budget_s and reps < 20000:
        c0 = time.perf_counter()
        oracle.decode_attn(b.q, k, v, b.seq_lens, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim,
                           cfg.max_len, lay.stride_req, lay.stride_kvh, lay.stride_tok, n_threads=1)
        t += time.perf_counter() - c0
        reps += 1
    return {"workload": cfg.name, "threads": 1, "us_per_step": 1e6 * t / reps,
            "value": b.kv_bytes * reps / t / 1e9, "unit": "GB/s", "repetitions": reps}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.prefill:
        return main_prefill(args)
    if args.handoff:
        return main_handoff(args)

    import numpy as np
    import torch
    from paper_2311_18677_amd import binding as sw
    from paper_2311_18677_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    sw.load()
    sw.sw_set_param(sw.SW_PARAM_CHUNK, args.chunk)
    sw.sw_set_param(sw.SW_PARAM_KERNEL, args.kernel)
    sw.sw_set_param(sw.SW_PARAM_WAVES, args.waves)
    sw.sw_set_param(sw.SW_PARAM_COMBINE, args.combine)

    cfg = wl.CONFIGS[args.workload]
    lay = sw.sw_kv_layout(cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len)

    # ---- inputs: set 0 from the host recipe (also the oracle's input), the rest on device
    append = args.append or args.decode_loop
    loop = args.decode_loop
    room = (max(1, args.repeats) * (args.steps + args.warmup) + args.warmup) // cfg.n_layers + 60 if loop else (1 if append else 0)
    batch0 = wl.make_batch(cfg)
    if args.paged:
        set0 = sw.upload_paged_batch(batch0, args.paged, device="cuda:0", pad_bits=0, room=room)
    else:
        set0 = sw.upload_batch(batch0, device="cuda:0", pad_bits=0)
    set0["kv_bytes"] = batch0.kv_bytes
    kn0, vn0 = wl.make_new_rows(cfg, batch0.seed)
    for name, rows in (("k_new", kn0), ("v_new", vn0)):
        set0[name] = torch.from_numpy(rows.view(np.int16).reshape(-1)).to(dev).view(torch.float16)
    if loop:
        n_sets = cfg.n_layers        # one cache per layer, all with the batch's lengths
    else:
        n_sets = args.sets or max(2, -(-4 * LLC_BYTES // max(batch0.kv_bytes, 1)))
    sets = [set0]
    for i in range(1, n_sets):
        seed_i = wl.BASE_SEED + 1000 * cfg.seed_index + i
        lens_i = batch0.seq_lens if loop else None
        if args.paged:
            sets.append(make_paged_set(cfg, args.paged, seed_i, torch, np, wl, sw, dev, lens_i, room))
        else:
            sets.append(make_device_set(cfg, lay, seed_i, torch, np, wl, dev, lens_i))
    if loop:
        for s in sets[1:]:
            s["seq_lens"] = set0["seq_lens"]      # the layers of a model share one length array
    torch.cuda.synchronize()

    if args.copy_calibration:
        # a plain copy of known size: reads N bytes and writes N bytes per launch
        n = args.copy_calibration << 20
        src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        if append and args.paged:
            sw.sw_decode_attn_paged_append(s["q"], s["k_new"], s["v_new"], s["k_pool"], s["v_pool"],
                                           s["block_table"], s["seq_lens"], s["out"], cfg.n_req,
                                           cfg.n_qh, cfg.n_kvh, cfg.head_dim, s["block_size"],
                                           s["max_blocks"], s["n_blocks"], st)
        elif append:
            sw.sw_decode_attn_append(s["q"], s["k_new"], s["v_new"], s["k_cache"], s["v_cache"],
                                     s["seq_lens"], s["out"], cfg.n_req, cfg.n_qh, cfg.n_kvh,
                                     cfg.head_dim, cfg.max_len, st)
        elif args.paged:
            sw.sw_decode_attn_paged(s["q"], s["k_pool"], s["v_pool"], s["block_table"], s["seq_lens"],
                                    s["out"], cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim,
                                    s["block_size"], s["max_blocks"], s["n_blocks"], st)
        else:
            sw.sw_decode_attn(s["q"], s["k_cache"], s["v_cache"], s["seq_lens"], s["out"],
                              cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, st)

    def end_of_model_step(st):
        if loop:
            sw.sw_advance_lens(set0["seq_lens"], cfg.n_req, cfg.max_len, st)

    def attended_bytes():
        """K/V bytes one layer call reads at the lengths now on the device."""
        lens_now = np.clip(set0["seq_lens"].cpu().numpy().astype(np.int64), 0, cfg.max_len)
        if append:
            lens_now = np.minimum(lens_now + 1, cfg.max_len)
        return int(lens_now.sum()) * cfg.n_kvh * cfg.head_dim * 4

    # first call on the stream sizes the workspace (allocates); keep it out of everything timed
    call(sets[0], stream)
    stream.synchronize()

    # ---- append variants: parity of set 0 now, while its lengths are the recipe's (the
    # call above stored the new rows; storing them again changes nothing)
    parity = None
    host0 = None
    if append and not args.no_cpu_baseline:
        import oracle
        k0, v0 = set0["k_host"].copy(), set0["v_host"].copy()
        if args.paged:
            pl = set0["layout"]
            geom = (set0["block_size"], set0["max_blocks"], set0["n_blocks"],
                    pl.stride_block, pl.stride_kvh, pl.stride_tok)
            lens1 = oracle.kv_append_paged(kn0, vn0, k0, v0, set0["table_host"], batch0.seq_lens,
                                           cfg.n_req, cfg.n_kvh, cfg.head_dim, *geom)
            ref = oracle.decode_attn_paged(batch0.q, k0, v0, set0["table_host"], lens1, cfg.n_req,
                                           cfg.n_qh, cfg.n_kvh, cfg.head_dim, *geom)
        else:
            lens1 = oracle.kv_append(kn0, vn0, k0, v0, batch0.seq_lens, cfg.n_req, cfg.n_kvh,
                                     cfg.head_dim, cfg.max_len, lay.stride_req, lay.stride_kvh,
                                     lay.stride_tok)
            ref = oracle.decode_attn(batch0.q, k0, v0, lens1, cfg.n_req, cfg.n_qh, cfg.n_kvh,
                                     cfg.head_dim, cfg.max_len, lay.stride_req, lay.stride_kvh,
                                     lay.stride_tok)
        host0 = (k0, v0, lens1)
        out = set0["out"].cpu().numpy().astype(np.float64)
        parity = parity_vs_oracle(np, out, ref)

    steps, warmup = args.steps, args.warmup
    mode = args.mode
    repeats = max(1, args.repeats)

    def record(k, st):
        for s in sets[:k]:
            call(s, st)
        if k == n_sets:
            end_of_model_step(st)

    runner = None
    if mode == "graph":
        try:
            runner = GraphSteps(torch, stream, n_sets, record)
            runner.prepare(steps, warmup)
        except Exception as e:      # noqa: BLE001 -- report and fall back to eager launches
            print("bench.py: graph capture failed (%s); using eager launches" % e, file=sys.stderr)
            runner = None
            mode = "eager"

    def run_steps(n):
        """Exactly n steps on the bench stream."""
        if runner is not None:
            runner.run(n)
            return
        for i in range(n):
            call(sets[i % n_sets], stream)
            if i % n_sets == n_sets - 1:
                end_of_model_step(stream)

    run_steps(warmup)
    torch.cuda.synchronize()
    # the W warm-up steps and the K timed steps, back to back, `repeats` times over; the K steps
    # of each repeat timed with HIP events recorded on the bench stream itself, and the whole
    # bracket (W + K steps) with the host clock around a synchronised region beside it
    ev_ms, wall_ms, rep_bytes = [], [], []
    for _ in range(repeats):
        bytes_before = attended_bytes()
        if loop:
            # the warm-up steps that lead into the timed ones advance the lengths as well
            bytes_before += (warmup // n_sets) * cfg.n_req * cfg.n_kvh * cfg.head_dim * 4
        e_ms, w_ms = time_on_stream(torch, stream, lambda: run_steps(steps), lambda: run_steps(warmup))
        if loop:
            # every layer call of a model step reads the same lengths, which grow by one per
            # model step: the mean of the first and the last step's bytes, times the calls
            full_steps = steps // n_sets
            bytes_last = attended_bytes() - (cfg.n_req * cfg.n_kvh * cfg.head_dim * 4 if full_steps else 0)
            bytes_done = 0.5 * (bytes_before + bytes_last) * steps
        elif append:
            bytes_done = bytes_before / sets[0]["kv_bytes"] * sum(sets[i % n_sets]["kv_bytes"] for i in range(steps))
        else:
            bytes_done = sum(sets[i % n_sets]["kv_bytes"] for i in range(steps))
        ev_ms.append(e_ms)
        wall_ms.append(w_ms)
        rep_bytes.append(bytes_done)
    order = sorted(range(repeats), key=lambda i: ev_ms[i])
    mid = order[(repeats - 1) // 2]                  # the median repeat (lower one if even)
    elapsed = ev_ms[mid] * 1e-3
    bytes_done = rep_bytes[mid]
    mean_bytes = bytes_done / steps
    gbps = bytes_done / elapsed / 1e9
    steps_per_s = steps / elapsed
    timing = {"method": "HIP events recorded on the bench stream around the K graph-launched steps; "
                        "value and ms_per_step are the median repeat",
              "repeats": repeats,
              "ms_per_step_median": 1e3 * elapsed / steps,
              "ms_per_step_min": min(ev_ms) / steps,
              "ms_per_step_max": max(ev_ms) / steps,
              "host_clock_ms_per_step_median": median(wall_ms) / (steps + warmup),
              "host_clock_covers": "warm-up and timed steps of a repeat, launch and synchronisation included"}

    # ---- single calls with a synchronisation between them (host clock): launch + tail overhead
    single = []
    for i in range(40):
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        call(sets[i % n_sets], stream)
        stream.synchronize()
        single.append(1e6 * (time.perf_counter() - c0))
    timing["single_call_synchronised_us_median"] = median(single[8:])

    # ---- per-kernel device time (HIP events attached to each dispatch, same stream, eager)
    prof_calls = min(steps, 50 * n_sets)
    sw.sw_prof_start(prof_calls)
    for i in range(prof_calls):
        call(sets[i % n_sets], stream)
    p_us, c_us, n_rec = sw.sw_prof_stop()
    if loop:
        prof_bytes = attended_bytes()
    else:
        prof_bytes = sum(sets[i % n_sets]["kv_bytes"] for i in range(n_rec)) / max(n_rec, 1)
        if append:
            prof_bytes *= bytes_before / sets[0]["kv_bytes"]
    partial_us = p_us / max(n_rec, 1)
    combine_us = c_us / max(n_rec, 1)
    eager_gap_us = sw.sw_prof_last_gap() / max(n_rec, 1)
    achieved = prof_bytes / (partial_us * 1e-6) / 1e9 if partial_us > 0 else 0.0

    # ---- the plain streaming read of the same byte count, timed the same way and at the same
    # point of the run as the kernel above (single launches time differently once the host
    # has been busy with the CPU baseline)
    ceiling = None if args.no_read_ceiling else stream_read_ceiling(sw, torch, mean_bytes, dev)

    # ---- parity of set 0 and the CPU baseline (the oracle as it stands, on the host cores)
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        if not append:
            call(sets[0], stream)
            stream.synchronize()
            out = set0["out"].cpu().numpy().astype(np.float64)
        reps, t_cpu, ref, used = 0, 0.0, None, 0
        while t_cpu < 10.0 and reps < 500:
            c0 = time.perf_counter()
            if append:
                # the oracle's step: store the rows (again: same rows, same place), then attend
                k0, v0, _ = host0
                if args.paged:
                    lens1 = oracle.kv_append_paged(kn0, vn0, k0, v0, set0["table_host"],
                                                   batch0.seq_lens, cfg.n_req, cfg.n_kvh,
                                                   cfg.head_dim, *geom)
                    oracle.decode_attn_paged(batch0.q, k0, v0, set0["table_host"], lens1, cfg.n_req,
                                             cfg.n_qh, cfg.n_kvh, cfg.head_dim, *geom)
                    used = oracle.max_threads()
                else:
                    lens1 = oracle.kv_append(kn0, vn0, k0, v0, batch0.seq_lens, cfg.n_req, cfg.n_kvh,
                                             cfg.head_dim, cfg.max_len, lay.stride_req,
                                             lay.stride_kvh, lay.stride_tok)
                    _, _, _, used = oracle.decode_attn(
                        batch0.q, k0, v0, lens1, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim,
                        cfg.max_len, lay.stride_req, lay.stride_kvh, lay.stride_tok,
                        return_stats=True)
            elif args.paged:
                pl = set0["layout"]
                ref = oracle.decode_attn_paged(
                    batch0.q, set0["k_host"], set0["v_host"], set0["table_host"], batch0.seq_lens,
                    cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, set0["block_size"],
                    set0["max_blocks"], set0["n_blocks"], pl.stride_block, pl.stride_kvh, pl.stride_tok)
                used = oracle.max_threads()
            else:
                ref, _, _, used = oracle.decode_attn(
                    batch0.q, set0["k_host"], set0["v_host"], batch0.seq_lens, cfg.n_req, cfg.n_qh,
                    cfg.n_kvh, cfg.head_dim, cfg.max_len, lay.stride_req, lay.stride_kvh,
                    lay.stride_tok, return_stats=True)
            t_cpu += time.perf_counter() - c0
            reps += 1
        cpu_gbps = batch0.kv_bytes * reps / t_cpu / 1e9
        cpu_baseline = {"value": cpu_gbps, "unit": "GB/s", "cores": int(used), "kind": "oracle",
                        "sample": "set 0 of %s (whole batch, %d K/V bytes), %d repetitions, %.1f s"
                                  % (cfg.name, batch0.kv_bytes, reps, t_cpu),
                        "decode_steps_per_s": reps / t_cpu}
        if not append:
            parity = parity_vs_oracle(np, out, ref)
        cpu_baseline["cpu_model"] = cpu_model()
        cpu_baseline["single_thread"] = oracle_single_thread(np, wl, sw)

    # ---- the other workloads, briefly (library defaults, plain entry point)
    others = None
    plain = not (args.paged or append or args.chunk or args.kernel or args.waves or args.combine)
    if plain and not args.no_configs:
        others = []
        for name in wl.CONFIGS:
            if name == cfg.name:
                continue
            others.append(measure_other_config(name, torch, np, sw, wl, dev,
                                               steps=min(steps, 1000), warmup=min(warmup, 200),
                                               repeats=repeats, with_oracle=not args.no_cpu_baseline))

    line = {
        "metric": "achieved HBM GB/s on K/V reads (% of MI355X peak) + decode steps/sec",
        "value": gbps,
        "unit": "GB/s",
        "pct_of_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "decode_steps_per_s": steps_per_s,
        "model_steps_per_s_attention_only": steps_per_s / cfg.n_layers,
        "tokens_per_s_attention_only": steps_per_s / cfg.n_layers * cfg.n_req,
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": 1e3 * elapsed / steps,
        "timing": timing,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16", "accumulate": "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "n_req": cfg.n_req, "n_qh": cfg.n_qh, "n_kvh": cfg.n_kvh,
                   "head_dim": cfg.head_dim, "max_len": cfg.max_len, "lens": str(cfg.lens),
                   "kv_bytes_per_step": mean_bytes, "cache_sets": n_sets, "launch": mode,
                   "kv_layout": ("block table, %d positions per block" % args.paged) if args.paged
                   else "dense, padded to max_len",
                   "entry_point": ("sw_decode_attn" + ("_paged" if args.paged else "")
                                   + ("_append" if append else "")),
                   "decode_loop": ("%d layer caches, lengths advanced per model step" % n_sets)
                   if loop else None,
                   "chunk": sw.sw_get_param(sw.SW_PARAM_CHUNK),
                   "kernel": sw.sw_get_param(sw.SW_PARAM_KERNEL)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": None if (args.paged or append) else read_traffic(cfg.name),
                     "kernel": "partial (dominant)", "kernel_us": partial_us,
                     "combine_us": combine_us, "bytes_per_launch": prof_bytes,
                     "launches_timed": n_rec,
                     "call_us": 1e6 * elapsed / steps,
                     "inter_kernel_gap_us": 1e6 * elapsed / steps - partial_us - combine_us,
                     "eager_inter_kernel_gap_us": eager_gap_us,
                     "note": "kernel_us and combine_us are HIP events attached to each dispatch of eager "
                             "launches, eager_inter_kernel_gap_us the time from the first kernel's end "
                             "event to the second's start event in those launches; call_us is the whole "
                             "call in the graph-launched timed steps and inter_kernel_gap_us = call_us - "
                             "kernel_us - combine_us (negative: graph-launched neighbours overlap part of "
                             "what the per-dispatch events count for each kernel)"},
        "cpu_baseline": cpu_baseline,
        "parity_set0": parity,
        "configs": others,
    }
    if ceiling is not None:
        line["roofline"]["stream_read_ceiling"] = ceiling
        if ceiling["kernel_GBps"] > 0:
            line["roofline"]["frac_of_stream_read"] = achieved / ceiling["kernel_GBps"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
