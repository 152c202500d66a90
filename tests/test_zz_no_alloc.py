"""sw_decode_attn_static, the entry point that allocates nothing: through the C ABI, against
sw_decode_attn and the CPU oracle, on two calls in a row of which the second is smaller."""
import numpy as np
import pytest

from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity, oracle_on_packed

pytestmark = pytest.mark.gpu


def _both(batch, stream=None):
    """(static entry point, sw_decode_attn two-kernel form, sw_decode_attn default) on one batch."""
    import torch
    cfg = batch.cfg
    bufs = sw.upload_batch(batch, pad_bits=0x7E00)
    outs = []
    for which in ("static", "two", "default"):
        bufs["out"].fill_(float("nan"))
        print("no-alloc case", cfg.name, "n_req", cfg.n_req, "max_len", cfg.max_len, "entry", which, flush=True)
        if which == "static":
            sw.sw_decode_attn_static(bufs["q"], bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], bufs["out"],
                                     cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, stream)
        else:
            sw.sw_set_param(sw.SW_PARAM_COMBINE, 1 if which == "two" else 0)
            try:
                sw.run_batch(bufs, cfg, stream)
            finally:
                sw.sw_set_param(sw.SW_PARAM_COMBINE, 0)
        torch.cuda.synchronize()
        outs.append(bufs["out"].cpu().numpy().copy())
    ref = oracle_on_packed(batch, bufs["k_host"], bufs["v_host"], bufs["layout"])
    return outs, ref


def test_static_entry_point_two_calls_in_a_row_the_second_smaller():
    big = wl.make_batch(wl.custom_config("na_big", 9, 8, 1, 128, 2048), seed=7301,
                        seq_lens=[2048, 1, 700, 0, 1290, 513, 64, 2047, 300])
    small = wl.make_batch(wl.custom_config("na_small", 3, 8, 1, 128, 2048), seed=7302,
                          seq_lens=[130, 1025, 17])
    for batch in (big, small):                       # the second call leaves most of the first's scratch untouched
        (static, two, default), ref = _both(batch)
        assert_parity(static, ref, batch.cfg.name)
        # same kernels as the two-kernel form of the existing entry point: same bits
        assert np.array_equal(static.view(np.uint16), two.view(np.uint16))
        # against the existing entry point as it runs by default: floating point, the bar of the parity tests
        assert np.max(np.abs(static.astype(np.float64) - default.astype(np.float64))) <= 2e-3
        assert_parity(default, ref, batch.cfg.name)


def test_static_entry_point_other_shapes_and_a_stream():
    import torch
    stream = torch.cuda.Stream()
    for cfg, lens, seed in ((wl.custom_config("na_mha", 4, 6, 6, 64, 300), [300, 1, 257, 64], 7303),
                            (wl.custom_config("na_g16", 3, 32, 2, 128, 1100), [1100, 5, 640], 7304)):
        batch = wl.make_batch(cfg, seed=seed, seq_lens=lens)
        (static, two, default), ref = _both(batch, stream)
        assert_parity(static, ref, cfg.name)
        assert np.array_equal(static.view(np.uint16), two.view(np.uint16))


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    # 4096 requests x 8 heads x 16 chunks x 520 bytes = 273 MB of partial results
    q = torch.zeros(16, dtype=torch.float16, device="cuda:0")
    lens = torch.zeros(4096, dtype=torch.int32, device="cuda:0")
    rc = sw.sw_decode_attn_static(q, q, q, lens, q, 4096, 8, 1, 128, 4096, None, check=False)
    assert rc == sw.SW_ERR_UNSUPPORTED
    assert "static scratch" in sw.sw_last_error()
