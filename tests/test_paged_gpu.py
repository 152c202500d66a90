"""GPU parity of the block-table (paged) variant: against the CPU oracle's paged
routine, and bit for bit against the dense entry point on the same cached values."""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _defaults():
    def reset():
        for key in (sw.SW_PARAM_CHUNK, sw.SW_PARAM_KERNEL, sw.SW_PARAM_COMBINE, sw.SW_PARAM_WAVES):
            sw.sw_set_param(key, 0)
    reset()
    yield
    reset()


def paged_out(batch, block_size, pad_bits=0x7E00, seed=0, table=None):
    import torch
    bufs = sw.upload_paged_batch(batch, block_size, seed=seed, pad_bits=pad_bits, table=table)
    print("paged run", batch.cfg.name, "block", block_size, "n_blocks", bufs["n_blocks"],
          "kernel", sw.sw_get_param(sw.SW_PARAM_KERNEL), flush=True)
    sw.run_paged_batch(bufs, batch.cfg)
    torch.cuda.synchronize()
    return bufs["out"].cpu().numpy(), bufs


def dense_out(batch, pad_bits=0x7E00):
    import torch
    bufs = sw.upload_batch(batch, pad_bits=pad_bits)
    sw.run_batch(bufs, batch.cfg)
    torch.cuda.synchronize()
    return bufs["out"].cpu().numpy()


def paged_ref(batch, bufs):
    cfg, lay = batch.cfg, bufs["layout"]
    return oracle.decode_attn_paged(batch.q, bufs["k_host"], bufs["v_host"], bufs["table_host"],
                                    batch.seq_lens, cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim,
                                    bufs["block_size"], bufs["max_blocks"], bufs["n_blocks"],
                                    lay.stride_block, lay.stride_kvh, lay.stride_tok)


SHAPES = [  # n_qh, n_kvh, d, kernel (0 = default)
    (8, 1, 128, 0), (8, 1, 128, 1), (14, 14, 128, 0), (8, 8, 64, 0), (24, 1, 128, 0), (16, 2, 128, 2),
    (6, 2, 64, 1), (40, 2, 128, 2),
]


@pytest.mark.parametrize("block_size", [4, 16, 32, 256])
@pytest.mark.parametrize("n_qh,n_kvh,d,kernel", SHAPES)
def test_paged_matches_oracle_and_dense_bits(n_qh, n_kvh, d, kernel, block_size):
    lens = [0, 1, 3, 4, 5, 15, 16, 17, 63, 64, 65, 255, 256, 257, 500, 700, 768]
    cfg = wl.custom_config("pg%d_%d_%d" % (n_qh, n_kvh, d), len(lens), n_qh, n_kvh, d, 768)
    batch = wl.make_batch(cfg, seed=8000 + n_qh + d + block_size, seq_lens=lens)
    sw.sw_set_param(sw.SW_PARAM_KERNEL, kernel)
    out, bufs = paged_out(batch, block_size)
    assert_parity(out, paged_ref(batch, bufs), cfg.name)
    assert np.array_equal(out.view(np.uint16), dense_out(batch).view(np.uint16))


@pytest.mark.parametrize("kernel", [0, 1])
def test_table_entries_past_the_length_are_never_followed_and_ids_are_clamped(kernel):
    lens = [40, 1, 0, 100, 64]
    cfg = wl.custom_config("pgc", len(lens), 8, 1, 128, 128)
    batch = wl.make_batch(cfg, seed=8100, seq_lens=lens)
    sw.sw_set_param(sw.SW_PARAM_KERNEL, kernel)
    base, bufs = paged_out(batch, 16)                 # spare entries hold a far out-of-range id
    for spare in (-1, 0, 2 ** 31 - 1, -2 ** 31):
        def with_spare(tab):
            t = tab.copy()
            for r, L in enumerate(batch.valid_lens):
                t[r, -(-int(L) // 16):] = spare
            return t
        out, _ = paged_out(batch, 16, table=with_spare)
        assert np.array_equal(out.view(np.uint16), base.view(np.uint16)), spare
    # ids outside the pool in USED entries behave like the clamped id
    n_blocks = bufs["n_blocks"]

    def out_of_range(tab):
        t = tab.copy()
        t[3, 0] = n_blocks + 5
        t[3, 1] = -9
        return t

    def clamped(tab):
        t = tab.copy()
        t[3, 0] = n_blocks - 1
        t[3, 1] = 0
        return t
    a, _ = paged_out(batch, 16, table=out_of_range)
    b, _ = paged_out(batch, 16, table=clamped)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert np.all(np.isfinite(a.astype(np.float32)[[0, 1, 2, 4]]))


@pytest.mark.parametrize("name,block_size", [("llama70b_tp8", 16), ("bloom176b_tp8", 16),
                                             ("longctx_8x32k", 32)])
def test_paged_full_size_configs(name, block_size):
    batch = wl.make_batch(name)
    out, bufs = paged_out(batch, block_size)
    errs = assert_parity(out, paged_ref(batch, bufs), name)
    print(name, "paged max_abs %.3e row_rel_l2 %.3e whole_rel_l2 %.3e" % errs)
