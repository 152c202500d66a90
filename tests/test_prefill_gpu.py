"""GPU parity of the prompt-phase (causal) attention against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity

pytestmark = pytest.mark.gpu

NAN_BITS = 0x7E00


@pytest.fixture(autouse=True, params=["default", "shared", "split4", "split8", "split2"])
def _kernel(request):
    """Every test runs with the library's own choice and with each prompt kernel forced."""
    which, waves = {"default": (0, 0), "shared": (1, 0), "split4": (2, 4), "split8": (2, 8),
                    "split2": (2, 2)}[request.param]
    sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, which)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, waves)
    yield request.param
    sw.sw_set_param(sw.SW_PARAM_PREFILL_KERNEL, 0)
    sw.sw_set_param(sw.SW_PARAM_PREFILL_WAVES, 0)


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).reshape(-1)).to("cuda:0").view(torch.float16)


def run_prefill(batch, qt, starts, n_tokens=None, pad_bits=NAN_BITS, tag=""):
    """Returns (out float16 [n_tokens, n_qh, d] with untouched rows still NaN, ref float64)."""
    import torch
    cfg = batch.cfg
    bufs = sw.upload_batch(batch, pad_bits=pad_bits)
    lay = bufs["layout"]
    n_tokens = qt.shape[0] if n_tokens is None else n_tokens
    ref = oracle.prefill_attn(qt, bufs["k_host"], bufs["v_host"], batch.seq_lens, starts, cfg.n_req,
                              cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, lay.stride_req,
                              lay.stride_kvh, lay.stride_tok)
    out = torch.full((n_tokens, cfg.n_qh, cfg.head_dim), float("nan"), dtype=torch.float16, device="cuda:0")
    starts_d = torch.from_numpy(np.ascontiguousarray(starts, dtype=np.int32)).to("cuda:0")
    print("prefill run", tag, cfg.name, "lens", list(batch.seq_lens)[:8], "n_tokens", n_tokens, flush=True)
    sw.sw_prefill_attn(to_dev(qt), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], starts_d, out,
                       n_tokens, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    torch.cuda.synchronize()
    return out.cpu().numpy(), ref


def covered_rows(batch, starts, n_tokens):
    mask = np.zeros(n_tokens, bool)
    for r, L in enumerate(batch.valid_lens):
        mask[starts[r]:starts[r] + int(L)] = True
    return mask


@pytest.mark.parametrize("n_qh,n_kvh", [(8, 1), (1, 1), (2, 2), (4, 1), (6, 2), (5, 1), (12, 2), (7, 1),
                                         (14, 14), (16, 2), (12, 1), (64, 2)])
def test_prefill_group_sizes_and_ragged_lengths(n_qh, n_kvh):
    lens = [0, 1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 255, 256, 257, 300, -4, 999]
    cfg = wl.custom_config("pf%d_%d" % (n_qh, n_kvh), len(lens), n_qh, n_kvh, 128, 300)
    batch = wl.make_batch(cfg, seed=6000 + n_qh, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    out, ref = run_prefill(batch, qt, starts, tag="groups")
    assert not np.isnan(out.astype(np.float32)).any()          # packed rows: every row belongs to a token
    assert_parity(out, ref, cfg.name)
    # a prompt's first token sees itself only: its row is V[0], exactly
    g = np.repeat(np.arange(n_kvh), n_qh // n_kvh)
    for r, L in enumerate(batch.valid_lens):
        if L > 0:
            assert np.array_equal(out[starts[r]].view(np.uint16), batch.v_rows[r][g, 0, :].view(np.uint16))


def test_prefill_key_rows_scaled_by_8_stress_the_softmax_range():
    # a tenth of the key rows scaled by 8, as in the skewed token-phase workload: single keys
    # dominate a row, whose value is then one V row -- up to 4.7 in magnitude here, where the
    # binary16 result alone rounds by up to 1.95e-3.  The bound only holds because numerator and
    # denominator of a row are built from the same rounded weights.
    import dataclasses
    lens = [2048, 700, 1500, 33, 1024]
    cfg = dataclasses.replace(wl.custom_config("pfx8", len(lens), 8, 1, 128, 2048), k_row_scale=(0.1, 8.0))
    batch = wl.make_batch(cfg, seed=8800, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    out, ref = run_prefill(batch, qt, starts, tag="x8")
    assert np.abs(ref).max() > 4.0
    assert_parity(out, ref, cfg.name)


def test_prefill_last_row_matches_the_decode_step():
    # the last prompt token's row is the token-phase step over the whole prompt
    import torch
    lens = [257, 64, 1, 300, 31]
    cfg = wl.custom_config("pfd", len(lens), 8, 1, 128, 320)
    batch = wl.make_batch(cfg, seed=6100, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    out, ref = run_prefill(batch, qt, starts, tag="last row")
    assert_parity(out, ref, cfg.name)
    last = np.stack([qt[starts[r] + L - 1] for r, L in enumerate(lens)])
    batch.q = last
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    sw.run_batch(bufs, cfg)
    torch.cuda.synchronize()
    dec = bufs["out"].cpu().numpy().astype(np.float64)
    pre = np.stack([out[starts[r] + L - 1] for r, L in enumerate(lens)]).astype(np.float64)
    assert np.abs(dec - pre).max() <= 2e-3


def test_prefill_unpacked_rows_and_untouched_padding():
    # rows with gaps and in reversed request order; rows of no token keep their content
    lens = [70, 33, 0, 129]
    cfg = wl.custom_config("pfg", len(lens), 4, 2, 128, 160)
    batch = wl.make_batch(cfg, seed=6200, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    new_starts = np.array([200, 150, 7, 3], np.int32)
    q2 = np.zeros((300, 4, 128), np.float16)
    for r, L in enumerate(lens):
        q2[new_starts[r]:new_starts[r] + L] = qt[starts[r]:starts[r] + L]
    out, ref = run_prefill(batch, q2, new_starts, tag="gaps")
    mask = covered_rows(batch, new_starts, 300)
    assert np.isnan(out[~mask].astype(np.float32)).all()       # not written
    assert_parity(out[mask], ref[mask], cfg.name)
    # and the rows equal the packed run's rows bit for bit
    out_p, _ = run_prefill(batch, qt, starts, tag="packed twin")
    for r, L in enumerate(lens):
        assert np.array_equal(out[new_starts[r]:new_starts[r] + L].view(np.uint16),
                              out_p[starts[r]:starts[r] + L].view(np.uint16))


def test_prefill_padding_values_never_reach_a_result():
    lens = [45, 128, 97]
    cfg = wl.custom_config("pfp", len(lens), 8, 2, 128, 160)
    batch = wl.make_batch(cfg, seed=6300, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    base, ref = run_prefill(batch, qt, starts, pad_bits=0, tag="pad 0")
    assert_parity(base, ref, cfg.name)
    for pad in (0x7E00, 0x7BFF, 0xFC00):                        # NaN, 65504, -inf
        out, _ = run_prefill(batch, qt, starts, pad_bits=pad, tag="pad %x" % pad)
        assert np.array_equal(out.view(np.uint16), base.view(np.uint16)), hex(pad)


def test_prefill_repeatable_and_batch_independent():
    lens = [200, 77, 130]
    cfg = wl.custom_config("pfr", len(lens), 8, 1, 128, 256)
    batch = wl.make_batch(cfg, seed=6400, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    a, ref = run_prefill(batch, qt, starts, tag="rep a")
    b, _ = run_prefill(batch, qt, starts, tag="rep b")
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    # request 1 alone gives the same rows
    cfg1 = wl.custom_config("pfr1", 1, 8, 1, 128, 256)
    b1 = wl.make_batch(cfg1, seed=1, seq_lens=[77])
    b1.k_rows, b1.v_rows = [batch.k_rows[1]], [batch.v_rows[1]]
    solo, _ = run_prefill(b1, qt[starts[1]:starts[1] + 77], np.array([0], np.int32), tag="solo")
    assert np.array_equal(solo.view(np.uint16), a[starts[1]:starts[1] + 77].view(np.uint16))


@pytest.mark.parametrize("name", ["prefill_tiny", "prefill_llama70b_tp8", "prefill_bloom176b_tp8"])
def test_prefill_configs_match_oracle(name):
    batch = wl.make_batch(wl.PREFILL_CONFIGS[name])
    qt, starts = wl.make_prefill_queries(batch)
    out, ref = run_prefill(batch, qt, starts, tag=name)
    errs = assert_parity(out, ref, name)
    print(name, "prefill max_abs %.3e row_rel_l2 %.3e whole_rel_l2 %.3e" % errs)


def test_prefill_unsupported_shapes_are_refused():
    assert sw.sw_prefill_attn(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 10, 1, 8, 8, 64, 128,
                              check=False) == sw.SW_ERR_UNSUPPORTED
    assert sw.sw_prefill_attn(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 10, 1, 130, 2, 128, 128,
                              check=False) == sw.SW_ERR_UNSUPPORTED


def test_prefill_repeated_calls_on_cache_resident_data_are_stable():
    """A small prompt batch stays in the on-chip caches, so staged tiles come back fast; every
    call must still give the first call's bits (staging areas are refilled only after the reads
    of the previous tile have returned)."""
    import torch
    lens = [300, 200, 257, 33]
    cfg = wl.custom_config("pfhot", len(lens), 8, 2, 128, 320)
    batch = wl.make_batch(cfg, seed=6500, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(batch)
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    q_d = to_dev(qt)
    starts_d = torch.from_numpy(starts).to("cuda:0")
    first = None
    for rep in range(40):
        out = torch.full((qt.shape[0], cfg.n_qh, cfg.head_dim), float("nan"), dtype=torch.float16, device="cuda:0")
        sw.sw_prefill_attn(q_d, bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], starts_d, out,
                           qt.shape[0], cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        if first is None:
            first = got
            assert not np.isnan(got.astype(np.float32)).any()
        assert np.array_equal(got.view(np.uint16), first.view(np.uint16)), rep
