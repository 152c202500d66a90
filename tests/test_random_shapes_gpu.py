"""Seeded random shapes through every attention entry point, each against its oracle routine.

Shapes, lengths, block sizes and query counts are drawn from a counter-based generator, so a
failing case is named by its seed; every draw is a shape the entry points document as valid.
"""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity

pytestmark = pytest.mark.gpu

NAN_BITS = 0x7E00
HEADS = [(1, 1), (2, 1), (3, 1), (4, 2), (6, 2), (8, 1), (8, 8), (12, 4), (14, 14), (16, 1), (5, 5), (7, 1)]


def draw(seed, d_choices=(64, 128)):
    rng = np.random.Generator(np.random.Philox(seed))
    n_qh, n_kvh = HEADS[int(rng.integers(len(HEADS)))]
    d = int(rng.choice(d_choices))
    max_len = int(rng.choice([33, 64, 100, 257, 600, 1500, 3000]))
    n_req = int(rng.integers(1, 24))
    kind = rng.integers(0, 4, n_req)
    lens = np.where(kind == 0, max_len, np.where(kind == 1, rng.integers(0, 4, n_req),
                                                 rng.integers(0, max_len + 1, n_req)))
    return rng, n_qh, n_kvh, d, max_len, n_req, [int(x) for x in lens]


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).reshape(-1)).to("cuda:0").view(torch.float16)


def i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


@pytest.mark.parametrize("seed", range(9100, 9124))
def test_random_decode_dense_and_paged(seed):
    import torch
    rng, n_qh, n_kvh, d, max_len, n_req, lens = draw(seed)
    cfg = wl.custom_config("rnd%d" % seed, n_req, n_qh, n_kvh, d, max_len)
    batch = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    print("decode", seed, n_qh, n_kvh, d, max_len, n_req, lens[:8], flush=True)
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    lay = bufs["layout"]
    ref = oracle.decode_attn(batch.q, bufs["k_host"], bufs["v_host"], batch.seq_lens, n_req, n_qh, n_kvh, d,
                             max_len, lay.stride_req, lay.stride_kvh, lay.stride_tok)
    sw.run_batch(bufs, cfg)
    torch.cuda.synchronize()
    dense = bufs["out"].cpu().numpy()
    assert_parity(dense, ref, cfg.name)
    bs = int(rng.choice([4, 16, 64, 256]))
    pb = sw.upload_paged_batch(batch, bs, pad_bits=NAN_BITS, seed=seed)
    sw.run_paged_batch(pb, cfg)
    torch.cuda.synchronize()
    paged = pb["out"].cpu().numpy()
    assert_parity(paged, ref, cfg.name + " paged %d" % bs)


@pytest.mark.parametrize("seed", range(9200, 9216))
def test_random_append(seed):
    import torch
    rng, n_qh, n_kvh, d, max_len, n_req, lens = draw(seed)
    cfg = wl.custom_config("rna%d" % seed, n_req, n_qh, n_kvh, d, max_len)
    batch = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    k_new, v_new = wl.make_new_rows(cfg, seed)
    print("append", seed, n_qh, n_kvh, d, max_len, n_req, lens[:8], flush=True)
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    lay = bufs["layout"]
    k_ref, v_ref = bufs["k_host"].copy(), bufs["v_host"].copy()
    lens1 = oracle.kv_append(k_new, v_new, k_ref, v_ref, batch.seq_lens, n_req, n_kvh, d, max_len,
                             lay.stride_req, lay.stride_kvh, lay.stride_tok)
    ref = oracle.decode_attn(batch.q, k_ref, v_ref, lens1, n_req, n_qh, n_kvh, d, max_len,
                             lay.stride_req, lay.stride_kvh, lay.stride_tok)
    sw.sw_decode_attn_append(bufs["q"], to_dev(k_new), to_dev(v_new), bufs["k_cache"], bufs["v_cache"],
                             bufs["seq_lens"], bufs["out"], n_req, n_qh, n_kvh, d, max_len)
    torch.cuda.synchronize()
    assert_parity(bufs["out"].cpu().numpy(), ref, cfg.name)
    # the caches now hold the new rows, bit for bit, and nothing else changed
    assert np.array_equal(bufs["k_cache"].cpu().numpy().view(np.uint16), k_ref)
    assert np.array_equal(bufs["v_cache"].cpu().numpy().view(np.uint16), v_ref)


@pytest.mark.parametrize("seed", range(9300, 9320))
def test_random_mixed_dense_and_paged(seed):
    import torch
    rng, n_qh, n_kvh, d, max_len, n_req, lens = draw(seed, d_choices=(128,))
    cfg = wl.custom_config("rnm%d" % seed, n_req, n_qh, n_kvh, d, max_len)
    batch = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    kind = rng.integers(0, 4, n_req)
    qls = np.where(kind == 0, lens, np.where(kind == 1, 1, np.where(kind == 2, 0, rng.integers(0, max_len + 5, n_req))))
    qls = [int(x) for x in qls]
    max_q = int(rng.choice([1, 7, 64, max_len, max_len + 9]))
    eff = [min(max(q, 0), min(L, max_q)) for q, L in zip(qls, lens)]
    qt, starts, nq = wl.make_mixed_queries(batch, eff)
    if qt.shape[0] == 0:
        pytest.skip("no query token drawn")
    print("mixed", seed, n_qh, n_kvh, max_len, n_req, "q", qls[:8], "max_q", max_q, flush=True)
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)
    lay = bufs["layout"]
    ref = oracle.mixed_attn(qt, bufs["k_host"], bufs["v_host"], batch.seq_lens, starts, qls, n_req, n_qh, n_kvh,
                            d, max_len, max_q, lay.stride_req, lay.stride_kvh, lay.stride_tok)
    out = torch.full((qt.shape[0], n_qh, d), float("nan"), dtype=torch.float16, device="cuda:0")
    sw.sw_mixed_attn(to_dev(qt), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], i32(starts), i32(qls),
                     out, qt.shape[0], n_req, n_qh, n_kvh, d, max_len, max_q)
    torch.cuda.synchronize()
    dense = out.cpu().numpy()
    assert_parity(dense, ref, cfg.name)
    bs = int(rng.choice([4, 16, 32, 128]))
    pb = sw.upload_paged_batch(batch, bs, pad_bits=NAN_BITS, seed=seed)
    # the block-table form reaches max_blocks * block_size positions; queries are counted the same way
    out2 = torch.full_like(out, float("nan"))
    sw.sw_mixed_attn_paged(to_dev(qt), pb["k_pool"], pb["v_pool"], pb["block_table"], pb["seq_lens"],
                           i32(starts), i32(qls), out2, qt.shape[0], n_req, n_qh, n_kvh, d, bs,
                           pb["max_blocks"], pb["n_blocks"], max_q)
    torch.cuda.synchronize()
    assert_parity(out2.cpu().numpy(), ref, cfg.name + " paged %d" % bs)
