"""GPU checks of the KV hand-off kernels: bit-exact against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl

pytestmark = pytest.mark.gpu


def dev_u16(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to("cuda:0")


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def pack_case(n_qh, n_kvh, d, max_len, lens, bs, seed):
    """Pools built from a batch, dense buffers full of a marker; returns everything both sides need."""
    cfg = wl.custom_config("hk", len(lens), n_qh, n_kvh, d, max_len)
    batch = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    p = sw.upload_paged_batch(batch, bs, seed=seed, pad_bits=0x7E00)
    lay_d = sw.sw_kv_layout(cfg.n_req, n_kvh, d, max_len)
    return cfg, batch, p, lay_d


@pytest.mark.parametrize("bs", [4, 16, 128])
@pytest.mark.parametrize("n_kvh,d", [(1, 128), (3, 128), (2, 64)])
def test_pack_and_unpack_match_the_oracle_bit_for_bit(n_kvh, d, bs):
    import torch
    lens = [0, 1, 63, 64, 65, 127, 128, 129, 300, 511, 512, -2, 700]
    cfg, batch, p, lay_d = pack_case(n_kvh * 2, n_kvh, d, 512, lens, bs, 5000 + bs + d)
    lay_p = p["layout"]
    geom = (cfg.n_req, n_kvh, d, 512, bs, p["max_blocks"], p["n_blocks"], lay_p.stride_block,
            lay_p.stride_kvh, lay_d.stride_req, lay_d.stride_kvh, lay_d.stride_tok)
    # ---- pools -> dense
    kd_h = np.full(lay_d.total_elems, 0x1357, np.uint16)
    vd_h = np.full(lay_d.total_elems, 0x2468, np.uint16)
    kd, vd = dev_u16(kd_h), dev_u16(vd_h)
    oracle.kv_pack(p["k_host"], p["v_host"], p["table_host"], batch.seq_lens, kd_h, vd_h, True, *geom)
    print("pack", n_kvh, d, bs, flush=True)
    sw.sw_kv_pack(p["k_pool"], p["v_pool"], p["block_table"], p["seq_lens"], kd, vd, cfg.n_req, n_kvh, d,
                  512, bs, p["max_blocks"], p["n_blocks"])
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(kd), kd_h) and np.array_equal(host_u16(vd), vd_h)
    # the dense result is what building the dense cache from the batch gives (marker as padding)
    want = wl.pack_cache(batch.k_rows, cfg, lay_d.stride_req, lay_d.stride_kvh, lay_d.stride_tok,
                         lay_d.total_elems, 0x1357)
    assert np.array_equal(kd_h, want)
    # ---- dense -> fresh pools
    kp_h = np.full(p["k_host"].size, 0x0BAD, np.uint16)
    vp_h = np.full(p["v_host"].size, 0x0BAD, np.uint16)
    kp, vp = dev_u16(kp_h), dev_u16(vp_h)
    oracle.kv_pack(kp_h, vp_h, p["table_host"], batch.seq_lens, kd_h, vd_h, False, *geom)
    print("unpack", n_kvh, d, bs, flush=True)
    sw.sw_kv_unpack(kd, vd, p["block_table"], p["seq_lens"], kp, vp, cfg.n_req, n_kvh, d, 512, bs,
                    p["max_blocks"], p["n_blocks"])
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(kp), kp_h) and np.array_equal(host_u16(vp), vp_h)


def test_prompt_machine_to_token_machine_round_trip():
    """Prefill on a dense cache, unpack it into block pools, decode on the pools: the decode result
    has the bits of decoding on the dense cache directly."""
    import torch
    lens = [200, 77, 130, 1]
    cfg = wl.custom_config("rt", len(lens), 8, 1, 128, 256)
    batch = wl.make_batch(cfg, seed=5100, seq_lens=lens)
    dense = sw.upload_batch(batch, pad_bits=0x7E00)
    sw.run_batch(dense, cfg)
    torch.cuda.synchronize()
    direct = dense["out"].cpu().numpy()
    # an empty pool with a table that has room for every request
    p = sw.upload_paged_batch(batch, 16, seed=9, pad_bits=0x7E00)
    p["k_pool"].fill_(float("nan")), p["v_pool"].fill_(float("nan"))
    print("round trip", flush=True)
    sw.sw_kv_unpack(dense["k_cache"], dense["v_cache"], p["block_table"], p["seq_lens"], p["k_pool"],
                    p["v_pool"], cfg.n_req, 1, 128, 256, 16, p["max_blocks"], p["n_blocks"])
    sw.run_paged_batch(p, cfg)
    torch.cuda.synchronize()
    assert np.array_equal(p["out"].cpu().numpy().view(np.uint16), direct.view(np.uint16))


def test_span_plan_matches_the_oracle():
    import torch
    rng = np.random.Generator(np.random.Philox(5200))
    n_req, bs, mb, nb = 40, 16, 300, 5000
    lens = rng.integers(0, mb * bs + 50, size=n_req).astype(np.int32)
    lens[:4] = [0, 1, mb * bs, -7]
    table = np.zeros((n_req, mb), np.int32)
    for r in range(n_req):
        # runs of consecutive ids of random lengths, some crossing the 64-entry chunks
        i = 0
        while i < mb:
            run = int(rng.integers(1, 150 if r % 3 == 0 else 6))
            start = int(rng.integers(-3, nb + 3))
            for j in range(min(run, mb - i)):
                table[r, i + j] = start + j
            i += run
    table[5] = np.arange(100, 100 + mb)                 # a single span
    table[6] = 7                                        # every block its own span
    want_f, want_c, want_n = oracle.kv_span_plan(table, lens, n_req, bs, mb, nb, fill=-1)
    f = torch.full((n_req, mb), -1, dtype=torch.int32, device="cuda:0")
    c = torch.full((n_req, mb), -1, dtype=torch.int32, device="cuda:0")
    n = torch.full((n_req,), -1, dtype=torch.int32, device="cuda:0")
    print("span plan", flush=True)
    sw.sw_kv_span_plan(torch.from_numpy(table).to("cuda:0"), torch.from_numpy(lens).to("cuda:0"), f, c, n,
                       n_req, bs, mb, nb)
    torch.cuda.synchronize()
    assert np.array_equal(n.cpu().numpy(), want_n)
    assert np.array_equal(f.cpu().numpy(), want_f)
    assert np.array_equal(c.cpu().numpy(), want_c)
    assert want_n[5] == 1 and want_n[0] == 0
