"""GPU checks of sw_kv_store / sw_kv_store_paged: bit-exact against the oracle's copies."""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import assert_parity

pytestmark = pytest.mark.gpu

NAN_BITS = 0x7E00
HEADS = [1, 2, 3, 8, 14]


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).reshape(-1)).to("cuda:0").view(torch.float16)


def i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


def bits(t):
    return t.cpu().numpy().view(np.uint16).reshape(-1)


def draw(seed):
    rng = np.random.Generator(np.random.Philox(seed))
    n_kvh = int(rng.choice(HEADS))
    d = int(rng.choice([64, 128]))
    max_len = int(rng.choice([33, 100, 257, 700]))
    n_req = int(rng.choice([1, 5, 70, 150]))
    lens = rng.integers(0, max_len + 1, n_req)
    kind = rng.integers(0, 4, n_req)
    qls = np.where(kind == 0, lens, np.where(kind == 1, 1, np.where(kind == 2, 0, rng.integers(0, max_len + 9, n_req))))
    max_q = int(rng.choice([1, 40, max_len, max_len + 3]))
    return rng, n_kvh, d, max_len, n_req, [int(x) for x in lens], [int(x) for x in qls], max_q


@pytest.mark.parametrize("seed", range(9400, 9420))
def test_store_dense_and_paged_against_the_oracle(seed):
    import torch
    rng, n_kvh, d, max_len, n_req, lens, qls, max_q = draw(seed)
    cfg = wl.custom_config("rs%d" % seed, n_req, n_kvh, n_kvh, d, max_len)
    batch = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    eff = [min(max(q, 0), min(L, max_q)) for q, L in zip(qls, lens)]
    k_tok, v_tok, starts, nq = wl.token_rows(batch, eff)
    if k_tok.shape[0] == 0:
        pytest.skip("no new token drawn")
    print("store", seed, n_kvh, d, max_len, n_req, "max_q", max_q, flush=True)
    # dense: caches full of NaN, the store writes the new rows and nothing else
    lay = sw.sw_kv_layout(n_req, n_kvh, d, max_len)
    k_ref = np.full(lay.total_elems, NAN_BITS, np.uint16)
    v_ref = np.full(lay.total_elems, NAN_BITS, np.uint16)
    oracle.kv_store(k_tok, v_tok, k_ref, v_ref, lens, starts, qls, n_req, n_kvh, d, max_len, max_q,
                    lay.stride_req, lay.stride_kvh, lay.stride_tok)
    k_dev = torch.from_numpy(np.full(lay.total_elems, NAN_BITS, np.uint16).view(np.int16)).to("cuda:0")
    v_dev = k_dev.clone()
    sw.sw_kv_store(to_dev(k_tok), to_dev(v_tok), k_dev, v_dev, i32(lens), i32(starts), i32(qls),
                   k_tok.shape[0], n_req, n_kvh, d, max_len, max_q)
    torch.cuda.synchronize()
    assert np.array_equal(bits(k_dev), k_ref) and np.array_equal(bits(v_dev), v_ref)
    # block pools
    bs = int(rng.choice([4, 16, 64]))
    pb = sw.upload_paged_batch(batch, bs, pad_bits=NAN_BITS, seed=seed)
    play = pb["layout"]
    kp_ref = np.full_like(pb["k_host"], NAN_BITS)
    vp_ref = np.full_like(pb["v_host"], NAN_BITS)
    oracle.kv_store(k_tok, v_tok, kp_ref, vp_ref, lens, starts, qls, n_req, n_kvh, d, max_len, max_q,
                    play.stride_block, play.stride_kvh, play.stride_tok, block_table=pb["table_host"],
                    block_size=bs, max_blocks=pb["max_blocks"], n_blocks=pb["n_blocks"])
    kp_dev = torch.from_numpy(np.full_like(pb["k_host"], NAN_BITS).view(np.int16)).to("cuda:0")
    vp_dev = kp_dev.clone()
    sw.sw_kv_store_paged(to_dev(k_tok), to_dev(v_tok), kp_dev, vp_dev, pb["block_table"], i32(lens),
                         i32(starts), i32(qls), k_tok.shape[0], n_req, n_kvh, d, bs, pb["max_blocks"],
                         pb["n_blocks"], max_q)
    torch.cuda.synchronize()
    assert np.array_equal(bits(kp_dev), kp_ref) and np.array_equal(bits(vp_dev), vp_ref)


def test_store_whole_prompts_then_attend():
    import torch
    lens = [300, 77, 1, 0, 130]
    cfg = wl.custom_config("sp", len(lens), 8, 2, 128, 320)
    batch = wl.make_batch(cfg, seed=9500, seq_lens=lens)
    qt, qs = wl.make_prefill_queries(batch)
    k_tok, v_tok, starts, nq = wl.token_rows(batch)
    bufs = sw.upload_batch(batch, pad_bits=NAN_BITS)          # what the store must reproduce
    lay = bufs["layout"]
    k_dev = torch.from_numpy(np.full(lay.total_elems, NAN_BITS, np.uint16).view(np.int16)).to("cuda:0")
    v_dev = k_dev.clone()
    sw.sw_kv_store(to_dev(k_tok), to_dev(v_tok), k_dev, v_dev, bufs["seq_lens"], i32(starts), None,
                   k_tok.shape[0], cfg.n_req, 2, 128, 320, 320)
    out = torch.full((qt.shape[0], 8, 128), float("nan"), dtype=torch.float16, device="cuda:0")
    sw.sw_prefill_attn(to_dev(qt), k_dev.view(torch.float16), v_dev.view(torch.float16), bufs["seq_lens"],
                       i32(qs), out, qt.shape[0], cfg.n_req, 8, 2, 128, 320)
    torch.cuda.synchronize()
    assert np.array_equal(bits(k_dev), bufs["k_host"]) and np.array_equal(bits(v_dev), bufs["v_host"])
    ref = oracle.prefill_attn(qt, bufs["k_host"], bufs["v_host"], batch.seq_lens, qs, cfg.n_req, 8, 2, 128, 320,
                              lay.stride_req, lay.stride_kvh, lay.stride_tok)
    assert_parity(out.cpu().numpy(), ref, cfg.name)


def test_store_skips_rows_that_do_not_exist():
    import torch
    lens = [40, 20]
    cfg = wl.custom_config("sk", 2, 2, 2, 128, 64)
    batch = wl.make_batch(cfg, seed=9600, seq_lens=lens)
    k_tok, v_tok, starts, nq = wl.token_rows(batch)
    lay = sw.sw_kv_layout(2, 2, 128, 64)
    k_dev = torch.from_numpy(np.full(lay.total_elems, NAN_BITS, np.uint16).view(np.int16)).to("cuda:0")
    v_dev = k_dev.clone()
    # request 0 starts 5 rows before the arrays, request 1 runs 8 rows past their end: those rows are skipped
    n_tok = 47
    k2 = np.zeros((n_tok, 2, 128), np.float16)
    v2 = np.zeros((n_tok, 2, 128), np.float16)
    k2[0:35], v2[0:35] = k_tok[5:40], v_tok[5:40]
    k2[35:47], v2[35:47] = k_tok[40:52], v_tok[40:52]
    sw.sw_kv_store(to_dev(k2), to_dev(v2), k_dev, v_dev, i32(lens), i32([-5, 35]), None, n_tok, 2, 2, 128, 64, 64)
    torch.cuda.synchronize()
    kv = bits(k_dev)
    view = np.lib.stride_tricks.as_strided(kv, shape=(2, 2, 64, 128),
                                           strides=(2 * lay.stride_req, 2 * lay.stride_kvh, 2 * lay.stride_tok, 2))
    assert (view[0, :, 0:5] == NAN_BITS).all() and (view[1, :, 12:20] == NAN_BITS).all()
    assert np.array_equal(view[0, :, 5:40], batch.k_rows[0][:, 5:40].view(np.uint16))
    assert np.array_equal(view[1, :, 0:12], batch.k_rows[1][:, 0:12].view(np.uint16))
