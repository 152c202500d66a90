"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Floating point within max-abs 2e-3 / row rel-L2
1e-3; length and index handling bit-exact."""
import numpy as np
import pytest

from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity, oracle_on_packed

pytestmark = pytest.mark.gpu

# mode -> (SW_PARAM_KERNEL, SW_PARAM_COMBINE)
MODES = {"default": (0, 0), "valu": (1, 1), "mfma": (2, 1), "valu_fused": (1, 2), "mfma_fused": (2, 2)}
ALL_MODES = ["valu", "mfma", "valu_fused", "mfma_fused"]


def set_mode(which):
    k, c = MODES[which]
    sw.sw_set_param(sw.SW_PARAM_KERNEL, k)
    sw.sw_set_param(sw.SW_PARAM_COMBINE, c)


@pytest.fixture(autouse=True)
def _defaults():
    def reset():
        sw.sw_set_param(sw.SW_PARAM_CHUNK, 0)
        sw.sw_set_param(sw.SW_PARAM_KERNEL, 0)
        sw.sw_set_param(sw.SW_PARAM_COMBINE, 0)
        sw.sw_set_param(sw.SW_PARAM_WAVES, 0)
    reset()
    yield
    reset()


def gpu_out(batch, pad_bits=0, stream=None, bufs=None):
    import torch
    if bufs is None:
        bufs = sw.upload_batch(batch, pad_bits=pad_bits)
    print("run", batch.cfg.name, "seed", batch.seed, "n_req", batch.cfg.n_req,
          "chunk", sw.sw_get_param(sw.SW_PARAM_CHUNK), "kernel", sw.sw_get_param(sw.SW_PARAM_KERNEL),
          "combine", sw.sw_get_param(sw.SW_PARAM_COMBINE),
          flush=True)
    sw.run_batch(bufs, batch.cfg, stream)
    torch.cuda.synchronize()
    return bufs["out"].cpu().numpy(), bufs




@pytest.mark.parametrize("which", ["default"] + ALL_MODES)
@pytest.mark.parametrize("name", ["tiny_mha", "llama70b_tp8", "bloom176b_tp8", "skewed_256",
                                  "longctx_8x32k"])
def test_configs_match_oracle(name, which):
    batch = wl.make_batch(name)
    set_mode(which)
    try:
        out, bufs = gpu_out(batch, pad_bits=0x7E00)
    except sw.SwError as e:
        if e.code == sw.SW_ERR_UNSUPPORTED and which.startswith("mfma"):
            pytest.skip("no matrix-core kernel for this shape")
        raise
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    errs = assert_parity(out, ref, name)
    print(name, which, "max_abs %.3e row_rel_l2 %.3e whole_rel_l2 %.3e" % errs)


GROUP_SHAPES = [  # (n_qh, n_kvh, head_dim)
    (1, 1, 64), (2, 1, 64), (3, 3, 128), (4, 2, 128), (6, 2, 64), (3, 1, 128), (5, 1, 128),
    (7, 1, 64), (8, 1, 64), (16, 2, 128), (14, 1, 128), (16, 1, 128), (24, 1, 128), (64, 1, 64),
    (12, 4, 128), (40, 1, 128), (64, 1, 128), (66, 2, 128),      # groups above 16: head tiles of 16, 16, 1
]


@pytest.mark.parametrize("which", ALL_MODES)
@pytest.mark.parametrize("n_qh,n_kvh,d", GROUP_SHAPES)
def test_group_sizes_and_ragged_lengths(n_qh, n_kvh, d, which):
    lens = [0, 1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 255, 256, 257, 300, 511, 513, 700]
    cfg = wl.custom_config("g%d_%d_%d" % (n_qh, n_kvh, d), len(lens), n_qh, n_kvh, d, 704)
    batch = wl.make_batch(cfg, seed=1000 + n_qh * 7 + n_kvh + d, seq_lens=lens)
    set_mode(which)
    try:
        out, bufs = gpu_out(batch, pad_bits=0x7E00)
    except sw.SwError as e:
        if e.code == sw.SW_ERR_UNSUPPORTED and which.startswith("mfma"):
            pytest.skip("no matrix-core kernel for this shape")
        raise
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, cfg.name)


@pytest.mark.parametrize("which", ALL_MODES)
@pytest.mark.parametrize("chunk", [64, 128, 256, 512, 1024])
def test_chunk_boundaries(chunk, which):
    lens = [chunk - 1, chunk, chunk + 1, 2 * chunk - 1, 2 * chunk, 2 * chunk + 1, 3 * chunk + 7, 1]
    cfg = wl.custom_config("cb%d" % chunk, len(lens), 8, 1, 128, 3 * chunk + 64)
    batch = wl.make_batch(cfg, seed=2000 + chunk, seq_lens=lens)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, chunk)
    set_mode(which)
    try:
        out, bufs = gpu_out(batch, pad_bits=0x7BFF)
    except sw.SwError as e:
        if e.code == sw.SW_ERR_UNSUPPORTED and which.startswith("mfma"):
            pytest.skip("no matrix-core kernel for this shape")
        raise
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, cfg.name)


@pytest.mark.parametrize("which", ALL_MODES)
@pytest.mark.parametrize("n_qh,n_kvh,d", [(8, 8, 64), (8, 1, 128), (14, 14, 128)])
def test_padding_never_reaches_the_result(n_qh, n_kvh, d, which):
    lens = [1, 5, 64, 100, 257, 0, 300]
    cfg = wl.custom_config("pad", len(lens), n_qh, n_kvh, d, 320)
    batch = wl.make_batch(cfg, seed=3000 + d, seq_lens=lens)
    set_mode(which)
    try:
        base, _ = gpu_out(batch, pad_bits=0)
    except sw.SwError as e:
        if e.code == sw.SW_ERR_UNSUPPORTED and which.startswith("mfma"):
            pytest.skip("no matrix-core kernel for this shape")
        raise
    for pad in (0x7E00, 0x7BFF, 0xFC00):        # NaN, 65504, -inf
        out, _ = gpu_out(batch, pad_bits=pad)
        assert np.array_equal(out.view(np.uint16), base.view(np.uint16)), hex(pad)


@pytest.mark.parametrize("which", ALL_MODES)
def test_length_edge_cases_bit_exact(which):
    # length 1 returns the V row bit for bit; length 0 and negative give +0;
    # lengths above max_len are clamped to max_len
    M = 96
    lens = [1, 0, -3, M + 50, M, 1]
    cfg = wl.custom_config("edge", len(lens), 8, 2, 128, M)
    batch = wl.make_batch(cfg, seed=4000, seq_lens=lens)
    set_mode(which)
    try:
        out, bufs = gpu_out(batch, pad_bits=0x7E00)
    except sw.SwError as e:
        if e.code == sw.SW_ERR_UNSUPPORTED and which.startswith("mfma"):
            pytest.skip("no matrix-core kernel for this shape")
        raise
    bits = out.view(np.uint16)
    for r in (0, 5):
        for h in range(8):
            assert np.array_equal(bits[r, h], batch.v_rows[r][h // 4, 0].view(np.uint16))
    assert np.all(bits[1] == 0) and np.all(bits[2] == 0)
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, "edge")
    # the clamped request equals the same request with length M
    batch2 = wl.make_batch(cfg, seed=4000, seq_lens=[1, 0, -3, M, M, 1])
    out2, _ = gpu_out(batch2, pad_bits=0x7E00)
    assert np.array_equal(out2.view(np.uint16), bits)


@pytest.mark.parametrize("which", ALL_MODES)
def test_permutation_batch_independence_and_repeatability(which):
    import torch
    lens = [700, 3, 256, 1023, 64, 511, 90, 1]
    cfg = wl.custom_config("perm", len(lens), 8, 1, 128, 1024)
    batch = wl.make_batch(cfg, seed=5000, seq_lens=lens)
    set_mode(which)
    try:
        out, bufs = gpu_out(batch)
    except sw.SwError as e:
        if e.code == sw.SW_ERR_UNSUPPORTED and which.startswith("mfma"):
            pytest.skip("no matrix-core kernel for this shape")
        raise
    # same call again: same bits
    out_again, _ = gpu_out(batch, bufs=bufs)
    assert np.array_equal(out.view(np.uint16), out_again.view(np.uint16))
    # permuted requests: permuted rows, same bits
    perm = [5, 2, 7, 0, 3, 6, 1, 4]
    pb = wl.Batch(cfg, batch.seed, batch.seq_lens[perm], batch.q[perm],
                  [batch.k_rows[i] for i in perm], [batch.v_rows[i] for i in perm])
    out_p, _ = gpu_out(pb)
    assert np.array_equal(out_p.view(np.uint16), out.view(np.uint16)[perm])
    # a request alone in its batch: same bits as inside the batch
    for r in (0, 3):
        c1 = wl.custom_config("solo", 1, 8, 1, 128, 1024)
        sb = wl.Batch(c1, batch.seed, batch.seq_lens[r:r + 1], batch.q[r:r + 1],
                      [batch.k_rows[r]], [batch.v_rows[r]])
        out_s, _ = gpu_out(sb)
        assert np.array_equal(out_s.view(np.uint16)[0], out.view(np.uint16)[r])


@pytest.mark.parametrize("kernel", [1, 2])
def test_single_launch_variant_is_repeatable_and_agrees_with_two_kernels(kernel):
    lens = [700, 3, 256, 1023, 64, 511, 90, 1, 0, 129]
    cfg = wl.custom_config("fz", len(lens), 8, 1, 128, 1024)
    batch = wl.make_batch(cfg, seed=5100, seq_lens=lens)
    sw.sw_set_param(sw.SW_PARAM_KERNEL, kernel)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, 128)
    sw.sw_set_param(sw.SW_PARAM_COMBINE, 1)
    two, bufs = gpu_out(batch, pad_bits=0x7E00)
    sw.sw_set_param(sw.SW_PARAM_COMBINE, 2)
    first = None
    for _ in range(3):       # repeated calls: the ticket counters must come back to zero
        bufs["out"].fill_(float("nan"))
        one, _ = gpu_out(batch, bufs=bufs)
        if first is None:
            first = one.copy()
        assert np.array_equal(one.view(np.uint16), first.view(np.uint16))
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(first, ref, "single launch")
    assert np.max(np.abs(first.astype(np.float64) - two.astype(np.float64))) <= 2e-3


@pytest.mark.parametrize("name,chunk", [("llama70b_tp8", 512), ("bloom176b_tp8", 1024), ("skewed_256", 1024)])
def test_single_launch_variant_at_bench_size_over_many_rotations(name, chunk):
    # The single-launch merge passes partial results between workgroups on different XCDs
    # through tagged 16-byte pieces, with no fence; what guards it is that every piece read
    # carries this call's tag.  Here it runs the way bench.py runs the step -- full-size
    # batches, three cache sets rotated in one replayed graph, many replays, at most eight
    # chunks per request -- and after every rotation each set's rows must be, bit for bit,
    # what the first single-launch call gave for that set (the sets share one workspace, so
    # a piece of an earlier call accepted by mistake would carry another set's values), which
    # in turn agrees with the two-kernel form (whose merge rounds differently: all chunks
    # against the overall maximum there, a running maximum here).  Stops at the first mismatch.
    import torch
    cfg = wl.CONFIGS[name]
    sw.sw_set_param(sw.SW_PARAM_CHUNK, chunk)
    sets, two = [], []
    sw.sw_set_param(sw.SW_PARAM_COMBINE, 1)
    for i in range(3):
        batch = wl.make_batch(cfg, seed=7300 + 10 * cfg.seed_index + i)
        out, bufs = gpu_out(batch, pad_bits=0x7E00)
        if i == 0:
            assert_parity(out, oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"]), name)
        del bufs["k_host"], bufs["v_host"]
        sets.append(bufs)
        two.append(out.astype(np.float64))
    sw.sw_set_param(sw.SW_PARAM_COMBINE, 2)
    stream = torch.cuda.Stream()
    want = []
    for i, b in enumerate(sets):         # the first call sizes the workspace, outside any capture
        b["out"].fill_(float("nan"))
        sw.run_batch(b, cfg, stream)
        stream.synchronize()
        one = b["out"].cpu().numpy()
        assert np.max(np.abs(one.astype(np.float64) - two[i])) <= 1e-3, (name, i)
        want.append(one.view(np.uint16).copy())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for b in sets:
            sw.run_batch(b, cfg, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(40):
        if rep % 8 == 0:
            print("rotation", rep, name, flush=True)
            for b in sets:
                b["out"].fill_(float("nan"))
        with torch.cuda.stream(stream):
            for _ in range(5):
                graph.replay()
        stream.synchronize()
        for i, b in enumerate(sets):
            got = b["out"].cpu().numpy().view(np.uint16)
            assert np.array_equal(got, want[i]), (name, "rotation", rep, "set", i,
                                                   int((got != want[i]).sum()), "elements differ")
    assert sw.sw_device_status() == 0


@pytest.mark.parametrize("combine", [1, 2])
def test_decode_call_in_a_replayed_graph(combine):
    # the way bench.py launches the step: captured once, replayed with eager work and
    # synchronisation in between; every replay must give the eager call's bits (for the
    # single-launch variant that also means its ticket counters are back at zero each time)
    import torch
    lens = [700, 3, 256, 1023, 64, 511, 90, 1, 0, 129]
    cfg = wl.custom_config("gr", len(lens), 8, 1, 128, 1024)
    batch = wl.make_batch(cfg, seed=5150, seq_lens=lens)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, 128)
    sw.sw_set_param(sw.SW_PARAM_COMBINE, combine)
    bufs = sw.upload_batch(batch, pad_bits=0x7E00)
    stream = torch.cuda.Stream()
    sw.run_batch(bufs, cfg, stream)      # the first call allocates the workspace, outside any capture
    stream.synchronize()
    want = bufs["out"].cpu().numpy().copy()
    assert_parity(want, oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"]), "eager")
    eager_out = bufs["out"]
    graph_out = torch.full_like(eager_out, float("nan"))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        sw.sw_decode_attn(bufs["q"], bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], graph_out,
                          cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        graph_out.fill_(float("nan"))
        torch.cuda.synchronize()
        print("replay", rep, "combine", combine, flush=True)
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(graph_out.cpu().numpy().view(np.uint16), want.view(np.uint16)), rep
        eager_out.fill_(float("nan"))
        sw.run_batch(bufs, cfg, stream)  # eager work between the replays
        stream.synchronize()
        assert np.array_equal(eager_out.cpu().numpy().view(np.uint16), want.view(np.uint16)), rep


@pytest.mark.parametrize("which", ["valu", "mfma", "valu_fused", "mfma_fused"])
@pytest.mark.parametrize("n_req", [65, 300, 1100])
def test_many_requests_exercise_every_work_map(n_req, which):
    # 65 / 300 / 1100 requests select the 4-per-lane scan, the 16-per-lane scan and
    # the direct block -> (request, chunk) mapping of the partial kernels
    rng = np.random.Generator(np.random.Philox(6000 + n_req))
    lens = rng.integers(0, 200, size=n_req).astype(np.int32)
    lens[::17] = 0
    lens[5] = 192
    cfg = wl.custom_config("many%d" % n_req, n_req, 8, 2, 128, 192)
    batch = wl.make_batch(cfg, seed=6000 + n_req, seq_lens=lens)
    set_mode(which)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, 64)
    out, bufs = gpu_out(batch, pad_bits=0x7E00)
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, cfg.name)


@pytest.mark.parametrize("waves", [4, 8])
@pytest.mark.parametrize("kernel", [2])
def test_waves_per_workgroup(kernel, waves):
    lens = [1000, 37, 512, 513, 0, 256]
    cfg = wl.custom_config("w%d" % waves, len(lens), 8, 1, 128, 1024)
    batch = wl.make_batch(cfg, seed=7000 + waves, seq_lens=lens)
    sw.sw_set_param(sw.SW_PARAM_KERNEL, kernel)
    sw.sw_set_param(sw.SW_PARAM_WAVES, waves)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, 512)
    out, bufs = gpu_out(batch, pad_bits=0x7E00)
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, cfg.name)


def test_non_default_stream_and_two_streams():
    import torch
    batch = wl.make_batch("tiny_mha")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    o0, bufs = gpu_out(batch)
    with torch.cuda.stream(s1):
        b1 = sw.upload_batch(batch)
    with torch.cuda.stream(s2):
        b2 = sw.upload_batch(batch)
    torch.cuda.synchronize()
    sw.run_batch(b1, batch.cfg, s1)
    sw.run_batch(b2, batch.cfg, s2)
    torch.cuda.synchronize()
    assert np.array_equal(b1["out"].cpu().numpy().view(np.uint16), o0.view(np.uint16))
    assert np.array_equal(b2["out"].cpu().numpy().view(np.uint16), o0.view(np.uint16))


def test_prof_reports_kernel_times():
    import torch
    batch = wl.make_batch("tiny_mha")
    bufs = sw.upload_batch(batch)
    sw.run_batch(bufs, batch.cfg)
    torch.cuda.synchronize()
    sw.sw_set_param(sw.SW_PARAM_COMBINE, 1)          # two kernels: both are timed
    sw.sw_prof_start(3)
    for _ in range(5):
        sw.run_batch(bufs, batch.cfg)
    p, c, n = sw.sw_prof_stop()
    assert n == 3 and 0 < p < 1e5 and 0 < c < 1e5
    sw.sw_set_param(sw.SW_PARAM_COMBINE, 2)          # single launch: there is no second kernel
    sw.sw_prof_start(4)
    for _ in range(4):
        sw.run_batch(bufs, batch.cfg)
    p, c, n = sw.sw_prof_stop()
    assert n == 4 and 0 < p < 1e5 and c == 0


def test_sampled_outputs_at_full_size_in_bench_configuration():
    """Config 2 exactly as bench.py launches it (default chunk and kernel):
    every row against the oracle, plus the properties that hold at any size."""
    batch = wl.make_batch("llama70b_tp8")
    out, bufs = gpu_out(batch, pad_bits=0x7E00)
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, "llama70b_tp8")
    o = out.astype(np.float64)
    for r in range(batch.cfg.n_req):
        v = batch.v_rows[r][0].astype(np.float64)
        assert np.all(o[r] <= v.max(axis=0) + 2e-3) and np.all(o[r] >= v.min(axis=0) - 2e-3)


@pytest.mark.parametrize("n_qh,n_kvh", [(14, 14), (8, 1)])
def test_repeated_calls_on_cache_resident_data_are_stable(n_qh, n_kvh):
    """A small batch stays in the on-chip caches across calls, so a tile's rows come back
    fast; every call must still give the first call's bits (a wave refills its staging
    area only after its reads of the previous tile have returned)."""
    import torch
    lens = [129, 255, 256, 400, 511, 512, 700, 766, 767, 768] * 2
    cfg = wl.custom_config("hot%d" % n_kvh, len(lens), n_qh, n_kvh, 128, 768)
    batch = wl.make_batch(cfg, seed=7700 + n_kvh, seq_lens=lens)
    bufs = sw.upload_batch(batch, pad_bits=0x7E00)
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    first = None
    for rep in range(40):
        out = torch.full_like(bufs["out"], float("nan"))
        sw.sw_decode_attn(bufs["q"], bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], out,
                          cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        if first is None:
            first = got
            assert_parity(got, ref, cfg.name)
        assert np.array_equal(got.view(np.uint16), first.view(np.uint16)), rep


@pytest.mark.parametrize("kernel", [0, 1])
def test_maximum_context_length(kernel):
    """max_len at the documented limit of 2^23 positions (a 2 GiB slab per head): one key, placed
    at the very end / in the middle, is aligned with the query so strongly that every other
    weight vanishes below binary32 resolution -- the result must be that position's V row."""
    import torch
    max_len = 1 << 23
    lay = sw.sw_kv_layout(1, 1, 128, max_len)
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    k = torch.zeros(lay.total_elems, dtype=torch.float16, device=dev)
    v = torch.empty(lay.total_elems, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
    q1 = torch.empty(128, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
    q = q1.repeat(8)                                   # the same query in all 8 heads
    out = torch.full((1, 8, 128), float("nan"), dtype=torch.float16, device=dev)
    sw.sw_set_param(sw.SW_PARAM_KERNEL, kernel)
    for L, pos in ((max_len, max_len - 1), (max_len, 4_194_305), (max_len - 5, max_len - 6)):
        k.zero_()
        k[pos * 128:(pos + 1) * 128] = 4.0 * q1
        lens = torch.tensor([L], dtype=torch.int32, device=dev)
        print("max context: L", L, "key at", pos, "kernel", kernel, flush=True)
        sw.sw_decode_attn(q, k, v, lens, out, 1, 8, 1, 128, max_len)
        torch.cuda.synchronize()
        want = v[pos * 128:(pos + 1) * 128].cpu().numpy().view(np.uint16)
        got = out.cpu().numpy().view(np.uint16)
        for h in range(8):
            assert np.array_equal(got[0, h], want), (L, pos, h)
    del k, v
    torch.cuda.empty_cache()


def test_maximum_number_of_rows():
    """n_req * n_qh at the documented limit of 2^20 (direct work mapping, a grid of 131072 groups)."""
    n_req = 1 << 17
    rng = np.random.Generator(np.random.Philox(7800))
    lens = rng.integers(0, 5, size=n_req).astype(np.int32)
    cfg = wl.custom_config("rows", n_req, 8, 1, 128, 4)
    batch = wl.make_batch(cfg, seed=7800, seq_lens=lens)
    out, bufs = gpu_out(batch, pad_bits=0x7E00)
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    assert_parity(out, ref, cfg.name)
    assert not out[lens == 0].any()
