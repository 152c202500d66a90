"""GPU parity of the mixed-batch attention (prompt and token phases in one call)."""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity

pytestmark = pytest.mark.gpu

NAN_BITS = 0x7E00


@pytest.fixture(autouse=True, params=["default", "shared", "split4", "split4_own_combine", "split8"])
def _kernel(request):
    # split4: the chunks of the token-phase requests are merged inside the prompt kernel
    # (the default wherever that kernel runs); split4_own_combine: by the combine kernel
    which, waves, merge = {"default": (0, 0, 0), "shared": (1, 0, 0), "split4": (2, 4, 2),
                           "split4_own_combine": (2, 4, 1), "split8": (2, 8, 0)}[request.param]
    sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, which)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, waves)
    sw.sw_set_param(sw.SW_PARAM_MIXED_MERGE, merge)
    yield request.param
    sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, 0)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, 0)
    sw.sw_set_param(sw.SW_PARAM_MIXED_MERGE, 0)


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).reshape(-1)).to("cuda:0").view(torch.float16)


def run_mixed(batch, qt, starts, q_lens, max_q_len, bufs=None, tag=""):
    import torch
    cfg = batch.cfg
    if bufs is None:
        bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    lay = bufs["layout"]
    ref = oracle.mixed_attn(qt, bufs["k_host"], bufs["v_host"], batch.seq_lens, starts, q_lens, cfg.n_req,
                            cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, max_q_len, lay.stride_req,
                            lay.stride_kvh, lay.stride_tok)
    out = torch.full((qt.shape[0], cfg.n_qh, cfg.head_dim), float("nan"), dtype=torch.float16, device="cuda:0")
    print("mixed run", tag, cfg.name, "q_lens", list(q_lens)[:10], "max_q", max_q_len, flush=True)
    sw.sw_mixed_attn(to_dev(qt), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"],
                     torch.from_numpy(np.ascontiguousarray(starts, dtype=np.int32)).to("cuda:0"),
                     torch.from_numpy(np.ascontiguousarray(q_lens, dtype=np.int32)).to("cuda:0"),
                     out, qt.shape[0], cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, max_q_len)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ref, bufs


@pytest.mark.parametrize("n_qh,n_kvh", [(8, 1), (4, 4), (6, 2)])
def test_mixed_batch_matches_oracle(n_qh, n_kvh):
    lens = [300, 300, 257, 64, 33, 1, 0, 200, 129, 300, 96, 250]
    qls = [300, 1, 100, 64, 1, 1, 5, 31, 33, 0, 32, 77]          # whole prompts, token phases, pieces
    cfg = wl.custom_config("mx%d_%d" % (n_qh, n_kvh), len(lens), n_qh, n_kvh, 128, 300)
    batch = wl.make_batch(cfg, seed=4000 + n_qh, seq_lens=lens)
    qt, starts, nq = wl.make_mixed_queries(batch, qls)
    assert nq.tolist() == [300, 1, 100, 64, 1, 1, 0, 31, 33, 0, 32, 77]
    out, ref, _ = run_mixed(batch, qt, starts, qls, 300, tag="pattern")
    assert not np.isnan(out.astype(np.float32)).any()
    assert_parity(out, ref, cfg.name)


def test_mixed_batch_with_key_rows_scaled_by_8():
    # prompts, prompt pieces and token-phase requests over caches in which a tenth of the key
    # rows is scaled by 8 (single keys dominate a row, whose value is then one V row)
    import dataclasses
    lens = [1500, 1800, 2048, 900, 1, 2048, 64, 1200]
    qls = [1500, 1, 300, 1, 1, 2048, 64, 1]
    cfg = dataclasses.replace(wl.custom_config("mxx8", len(lens), 8, 1, 128, 2048), k_row_scale=(0.1, 8.0))
    batch = wl.make_batch(cfg, seed=8850, seq_lens=lens)
    qt, starts, nq = wl.make_mixed_queries(batch, qls)
    out, ref, _ = run_mixed(batch, qt, starts, qls, 2048, tag="x8")
    assert not np.isnan(out.astype(np.float32)).any()
    assert np.abs(ref).max() > 3.5
    assert_parity(out, ref, cfg.name)


def test_all_tokens_as_queries_is_the_prompt_call_bit_for_bit():
    import torch
    lens = [200, 77, 130]
    cfg = wl.custom_config("mxp", len(lens), 8, 2, 128, 256)
    batch = wl.make_batch(cfg, seed=4100, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    out, ref, bufs = run_mixed(batch, qt, starts, lens, 256, tag="all")
    assert_parity(out, ref, cfg.name)
    pre = torch.full_like(to_dev(qt).view(qt.shape), float("nan"))
    sw.sw_prefill_attn(to_dev(qt), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"],
                       torch.from_numpy(starts).to("cuda:0"), pre, qt.shape[0], cfg.n_req, 8, 2, 128, 256)
    torch.cuda.synchronize()
    assert np.array_equal(pre.cpu().numpy().view(np.uint16), out.view(np.uint16))


def test_one_query_per_request_agrees_with_the_token_phase_call():
    import torch
    lens = [257, 64, 1, 300, 31, 150]
    cfg = wl.custom_config("mxd", len(lens), 8, 1, 128, 320)
    batch = wl.make_batch(cfg, seed=4200, seq_lens=lens)
    out, ref, bufs = run_mixed(batch, batch.q, np.arange(len(lens), dtype=np.int32), [1] * len(lens), 1, tag="decode")
    assert_parity(out, ref, cfg.name)
    sw.run_batch(bufs, cfg)
    torch.cuda.synchronize()
    # a request with one query token is served by the token-phase kernels: the same bits
    dec = bufs["out"].cpu().numpy().reshape(out.shape)
    assert np.array_equal(dec.view(np.uint16), out.view(np.uint16))


def test_a_prompt_in_pieces_and_the_query_bound():
    lens = [300, 180]
    cfg = wl.custom_config("mxc", 2, 8, 1, 128, 320)
    batch = wl.make_batch(cfg, seed=4300, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    whole, ref_whole, bufs = run_mixed(batch, qt, starts, lens, 320, tag="whole")
    # the last 100 / 37 tokens as a second piece: the same rows, up to rounding order
    q2 = np.concatenate([qt[200:300], qt[300 + 143:300 + 180]])
    piece, ref_piece, _ = run_mixed(batch, q2, np.array([0, 100], np.int32), [100, 37], 128, bufs=bufs, tag="piece")
    assert_parity(piece, ref_piece, cfg.name)
    assert np.array_equal(ref_piece[:100], ref_whole[200:300])
    assert np.abs(piece[:100].astype(np.float64) - whole[200:300].astype(np.float64)).max() <= 2e-3
    # q_lens above max_q_len: only the last max_q_len tokens are queries
    q3 = np.concatenate([qt[236:300], qt[300 + 116:300 + 180]])
    clamped, ref_c, _ = run_mixed(batch, q3, np.array([0, 64], np.int32), [1000, 90], 64, bufs=bufs, tag="bound")
    assert_parity(clamped, ref_c, cfg.name)
    assert np.array_equal(ref_c[:64], ref_whole[236:300]) and np.array_equal(ref_c[64:], ref_whole[300 + 116:300 + 180])


def test_mixed_rows_of_no_query_are_untouched():
    lens = [90, 40, 64]
    cfg = wl.custom_config("mxu", 3, 4, 2, 128, 96)
    batch = wl.make_batch(cfg, seed=4400, seq_lens=lens)
    qt, starts, nq = wl.make_mixed_queries(batch, [10, 0, 33])
    q2 = np.zeros((80, 4, 128), np.float16)
    new_starts = np.array([50, 0, 5], np.int32)
    q2[50:60] = qt[0:10]
    q2[5:38] = qt[10:43]
    out, ref, _ = run_mixed(batch, q2, new_starts, [10, 0, 33], 96, tag="gaps")
    mask = np.zeros(80, bool)
    mask[50:60] = True
    mask[5:38] = True
    assert np.isnan(out[~mask].astype(np.float32)).all()
    assert_parity(out[mask], ref[mask], cfg.name)


@pytest.mark.parametrize("kernel,combine", [(0, 0), (1, 1), (1, 2), (2, 1), (2, 2)])
def test_token_phase_requests_through_every_decode_variant(kernel, combine, _kernel):
    if _kernel not in ("default", "shared"):
        pytest.skip("the prompt kernel is not what varies here")
    lens = [2600, 1, 700, 0, 3000, 513, 64, 1200]
    qls = [1, 1, 90, 1, 1, 1, 0, 1]
    cfg = wl.custom_config("mxv", len(lens), 8, 1, 128, 4096)
    batch = wl.make_batch(cfg, seed=4500, seq_lens=lens)
    qt, starts, nq = wl.make_mixed_queries(batch, qls)
    assert nq.tolist() == [1, 1, 90, 0, 1, 1, 0, 1]
    # rows in a shuffled order with a gap, so that row != request everywhere
    order = [5, 0, 3, 6, 1, 7, 2, 4]
    new_starts = np.zeros(len(lens), np.int32)
    q2 = np.zeros((qt.shape[0] + 7, 8, 128), np.float16)
    at = 7
    for r in order:
        new_starts[r] = at
        q2[at:at + nq[r]] = qt[starts[r]:starts[r] + nq[r]]
        at += int(nq[r])
    sw.sw_set_param(sw.SW_PARAM_KERNEL, kernel)
    sw.sw_set_param(sw.SW_PARAM_COMBINE, combine)
    try:
        out, ref, _ = run_mixed(batch, q2, new_starts, qls, 128, tag="decode variant %d/%d" % (kernel, combine))
    finally:
        sw.sw_set_param(sw.SW_PARAM_KERNEL, 0)
        sw.sw_set_param(sw.SW_PARAM_COMBINE, 0)
    assert np.isnan(out[:7].astype(np.float32)).all()
    assert not np.isnan(out[7:].astype(np.float32)).any()
    assert_parity(out[7:], ref[7:], cfg.name)


@pytest.mark.parametrize("n_req", [65, 150, 300, 5000])
def test_many_requests_few_prompts(n_req):
    # more requests than lanes of a wave: every lane of the length scan holds several
    # (5000: beyond what the scans take on, both kernel families map workgroups directly)
    rng = np.random.Generator(np.random.Philox(4600 + n_req))
    lens = rng.integers(0, 201, n_req)
    kind = rng.integers(0, 8, n_req)
    qls = np.where(kind == 0, lens, np.where(kind == 1, rng.integers(0, 70, n_req), np.where(kind == 2, 0, 1)))
    cfg = wl.custom_config("mxm%d" % n_req, n_req, 2, 1, 128, 200)
    batch = wl.make_batch(cfg, seed=4600 + n_req, seq_lens=lens.tolist())
    qt, starts, nq = wl.make_mixed_queries(batch, qls.tolist())
    out, ref, _ = run_mixed(batch, qt, starts, qls.tolist(), 200, tag="many")
    assert not np.isnan(out.astype(np.float32)).any()
    assert_parity(out, ref, cfg.name)


def test_a_request_keeps_its_bits_whatever_its_batch():
    # alone (direct workgroup mapping) and inside larger batches (mapping by a scan of the
    # lengths, one and several requests per lane): the same tiles in the same order
    import torch
    L, nq = 250, 200
    outs = []
    for n_req, where in ((1, 0), (9, 4), (140, 77)):
        lens = [64] * n_req
        qls = [1] * n_req
        lens[where], qls[where] = L, nq
        if n_req > 2:
            lens[0], qls[0] = 200, 200
        cfg = wl.custom_config("mxb%d" % n_req, n_req, 8, 1, 128, 256)
        batch = wl.make_batch(cfg, seed=4700 + n_req, seq_lens=lens)
        # the request under test gets the same rows in every batch
        ref_cfg = wl.custom_config("mxb_ref", 1, 8, 1, 128, 256)
        ref_batch = wl.make_batch(ref_cfg, seed=4700, seq_lens=[L])
        batch.k_rows[where] = ref_batch.k_rows[0]
        batch.v_rows[where] = ref_batch.v_rows[0]
        qt, starts, nqs = wl.make_mixed_queries(batch, qls)
        q_ref = wl.make_mixed_queries(ref_batch, [nq])[0]
        qt[starts[where]:starts[where] + nq] = q_ref
        out, ref, _ = run_mixed(batch, qt, starts, qls, 256, tag="batch of %d" % n_req)
        assert_parity(out, ref, cfg.name)
        outs.append(out[starts[where]:starts[where] + nq].copy())
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))
    assert np.array_equal(outs[0].view(np.uint16), outs[2].view(np.uint16))


def test_mixed_call_in_a_replayed_graph():
    # the call enqueues several kernels; captured in a graph and replayed with eager work in
    # between, every replay must give the eager result
    import torch
    lens = [300, 257, 64, 200, 129, 300, 96, 250]
    qls = [300, 1, 1, 31, 1, 1, 32, 1]
    cfg = wl.custom_config("mxg", len(lens), 8, 1, 128, 320)
    batch = wl.make_batch(cfg, seed=4800, seq_lens=lens)
    qt, starts, nq = wl.make_mixed_queries(batch, qls)
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    q_dev, s_dev, l_dev = to_dev(qt), None, None
    s_dev = torch.from_numpy(starts).to("cuda:0")
    l_dev = torch.from_numpy(np.asarray(qls, np.int32)).to("cuda:0")
    n_tok = qt.shape[0]

    def call(out, stream):
        sw.sw_mixed_attn(q_dev, bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], s_dev, l_dev, out,
                         n_tok, cfg.n_req, 8, 1, 128, 320, 300, stream)

    eager = torch.full((n_tok, 8, 128), float("nan"), dtype=torch.float16, device="cuda:0")
    stream = torch.cuda.Stream()
    call(eager, stream)              # the first call allocates the workspace, outside any capture
    stream.synchronize()
    want = eager.cpu().numpy().view(np.uint16)
    assert not np.isnan(eager.cpu().numpy().astype(np.float32)).any()
    out = torch.full_like(eager, float("nan"))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call(out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep in range(4):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        print("replay", rep, flush=True)
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), want), rep
        call(eager, stream)          # eager work between the replays
        stream.synchronize()
        assert np.array_equal(eager.cpu().numpy().view(np.uint16), want)


def test_merge_inside_the_prompt_kernel_gives_the_combine_kernels_bits(_kernel):
    # token-phase requests long enough for many chunks (two-kernel form of the token phase),
    # beside prompts: the rows are the same bits whichever kernel merges the chunks, and
    # the token-phase rows are sw_decode_attn's
    if _kernel != "default":
        pytest.skip("sets the merge itself")
    import torch
    lens = [2300, 40, 900, 2304, 1, 513, 2000, 0, 1500, 257, 300]
    qls = [1, 40, 1, 1, 1, 13, 1, 1, 700, 1, 0]
    cfg = wl.custom_config("mxmerge", len(lens), 8, 1, 128, 2304)
    batch = wl.make_batch(cfg, seed=4900, seq_lens=lens)
    qt, starts, nq = wl.make_mixed_queries(batch, qls)
    sw.sw_set_param(sw.SW_PARAM_CHUNK, 128)          # 18 chunks per long request: the two-kernel form
    sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, 2)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, 4)
    outs = {}
    try:
        for merge in (1, 2):
            sw.sw_set_param(sw.SW_PARAM_MIXED_MERGE, merge)
            out, ref, bufs = run_mixed(batch, qt, starts, qls, 2304, tag="merge %d" % merge)
            assert_parity(out, ref, cfg.name)
            outs[merge] = out.copy()
        assert np.array_equal(outs[1].view(np.uint16), outs[2].view(np.uint16))
        # the token-phase rows against the plain decode call on the same cache
        dq = np.stack([qt[min(int(starts[r]), qt.shape[0] - 1)] for r in range(len(lens))])
        d_out = torch.zeros((len(lens), 8, 128), dtype=torch.float16, device="cuda:0")
        sw.sw_decode_attn(to_dev(dq), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], d_out, len(lens), 8, 1, 128, 2304)
        torch.cuda.synchronize()
        d_np = d_out.cpu().numpy()
        for r, (L, q) in enumerate(zip(lens, qls)):
            if q == 1 and L > 0:
                assert np.array_equal(outs[2][starts[r]].view(np.uint16), d_np[r].view(np.uint16)), r
    finally:
        sw.sw_set_param(sw.SW_PARAM_CHUNK, 0)
        sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, 0)
        sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, 0)
        sw.sw_set_param(sw.SW_PARAM_MIXED_MERGE, 0)
