"""Prompt-phase and mixed-batch attention at the sizes bench.py times, on sampled rows.

The oracle computes a sampled row on its own: row i of a request is the token-phase step at
length i + 1, so a sample costs O(i * head_dim), and a few hundred samples cover first and last
rows, block boundaries and random positions of every request.
"""
import numpy as np
import pytest

import oracle
from paper_2311_18677_amd import binding as sw
from paper_2311_18677_amd import workloads as wl
from helpers import parity_errors, MAX_ABS, MAX_REL_L2

pytestmark = pytest.mark.gpu


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16).reshape(-1)).to("cuda:0").view(torch.float16)


def i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to("cuda:0")


def sample_positions(rng, first, last, n_random):
    """Query positions in [first, last]: the ends, tile and block boundaries near them, random ones."""
    fixed = [first, first + 1, first + 31, first + 32, first + 33, last - 33, last - 32, last - 31, last - 1, last,
             (first + last) // 2, ((first + last) // 64) * 32 - 1, ((first + last) // 64) * 32]
    pos = [p for p in fixed if first <= p <= last]
    pos += [int(x) for x in rng.integers(first, last + 1, n_random)]
    return sorted(set(pos))


def check_sampled(batch, bufs, qt, starts, nq, out, rng, per_request):
    """Compare sampled rows of `out` with the oracle, one token-phase call per sample batch."""
    cfg = batch.cfg
    lay = bufs["layout"]
    worst_abs, worst_rel, checked = 0.0, 0.0, 0
    # samples are grouped into rounds: round j takes the j-th sample of every request, so each
    # oracle call is one token-phase step of the whole batch at per-request lengths
    samples = []
    for r in range(cfg.n_req):
        L, n = int(batch.valid_lens[r]), int(nq[r])
        samples.append(sample_positions(rng, L - n, L - 1, per_request) if n > 0 else [])
    for j in range(max(len(s) for s in samples)):
        lens_j = np.zeros(cfg.n_req, np.int32)
        q_j = np.zeros((cfg.n_req, cfg.n_qh, cfg.head_dim), np.float16)
        rows = {}
        for r, s in enumerate(samples):
            if j < len(s):
                pos = s[j]
                L, n = int(batch.valid_lens[r]), int(nq[r])
                row = int(starts[r]) + pos - (L - n)
                lens_j[r] = pos + 1
                q_j[r] = qt[row]
                rows[r] = row
        ref = oracle.decode_attn(q_j, bufs["k_host"], bufs["v_host"], lens_j, cfg.n_req, cfg.n_qh, cfg.n_kvh,
                                 cfg.head_dim, cfg.max_len, lay.stride_req, lay.stride_kvh, lay.stride_tok)
        for r, row in rows.items():
            a, rel, _ = parity_errors(out[row][None], ref[r][None])
            worst_abs, worst_rel, checked = max(worst_abs, a), max(worst_rel, rel), checked + 1
    assert worst_abs <= MAX_ABS and worst_rel <= MAX_REL_L2, (worst_abs, worst_rel)
    return worst_abs, worst_rel, checked


@pytest.mark.parametrize("name,shape", [
    ("prefill_long_8k", None),                   # key-split kernel
    ("prefill_long_32k", None),                  # shared-tile kernel
    ("prompts_16x1024", (16, 8, 1, 1024)),       # shared-tile kernel, many prompts
    ("prompts_12x1500_mha", (12, 14, 14, 1500)), # BLOOM-like heads, shared-tile kernel
])
def test_prompt_batches_at_bench_sizes_on_sampled_rows(name, shape):
    import torch
    if shape is None:
        cfg = wl.PREFILL_CONFIGS[name]
        batch = wl.make_batch(cfg)
    else:
        n_req, n_qh, n_kvh, plen = shape
        cfg = wl.custom_config(name, n_req, n_qh, n_kvh, 128, plen)
        batch = wl.make_batch(cfg, seed=7700 + n_req, seq_lens=[plen] * (n_req - 1) + [plen - 37])
    qt, starts = wl.make_prefill_queries(batch)
    bufs = sw.upload_batch(batch, pad_bits=0x7E00)
    out = torch.full((qt.shape[0], cfg.n_qh, cfg.head_dim), float("nan"), dtype=torch.float16, device="cuda:0")
    print("large prompt run", name, qt.shape, flush=True)
    sw.sw_prefill_attn(to_dev(qt), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], i32(starts), out,
                       qt.shape[0], cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not np.isnan(got.astype(np.float32)).any()          # every row was written
    rng = np.random.Generator(np.random.Philox(7700))
    per_request = 60 if cfg.n_req == 1 else 12
    worst = check_sampled(batch, bufs, qt, starts, batch.valid_lens, got, rng, per_request)
    print(name, "sampled rows: max_abs %.3e row_rel_l2 %.3e over %d rows" % worst)


def test_large_prompt_batch_over_block_pools_equals_the_dense_layout():
    # 16 prompts of 1024 tokens: the shared-tile kernel, with block-table addressing
    import torch
    cfg = wl.custom_config("paged_16x1024", 16, 8, 1, 128, 1024)
    batch = wl.make_batch(cfg, seed=7800, seq_lens=[1024] * 15 + [1000])
    qt, starts = wl.make_prefill_queries(batch)
    db = sw.upload_batch(batch, pad_bits=0x7E00)
    dense = torch.full((qt.shape[0], 8, 128), float("nan"), dtype=torch.float16, device="cuda:0")
    sw.sw_prefill_attn(to_dev(qt), db["k_cache"], db["v_cache"], db["seq_lens"], i32(starts), dense,
                       qt.shape[0], 16, 8, 1, 128, 1024)
    rng = np.random.Generator(np.random.Philox(7800))
    torch.cuda.synchronize()
    got = dense.cpu().numpy()
    worst = check_sampled(batch, db, qt, starts, batch.valid_lens, got, rng, 10)
    print("dense 16x1024 sampled rows: max_abs %.3e row_rel_l2 %.3e over %d rows" % worst)
    for bs in (16, 64):
        pb = sw.upload_paged_batch(batch, bs, pad_bits=0x7E00, seed=bs)
        out = torch.full_like(dense, float("nan"))
        print("paged large run, block", bs, flush=True)
        sw.sw_prefill_attn_paged(to_dev(qt), pb["k_pool"], pb["v_pool"], pb["block_table"], pb["seq_lens"],
                                 i32(starts), out, qt.shape[0], 16, 8, 1, 128, bs, pb["max_blocks"], pb["n_blocks"])
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), got.view(np.uint16))


@pytest.mark.parametrize("name", ["mixed_tiny", "mixed_llama70b_tp8"])
def test_mixed_configs_match_oracle(name):
    import torch
    from helpers import assert_parity
    batch, qls = wl.make_mixed_batch(name)
    cfg = batch.cfg
    qt, starts, nq = wl.make_mixed_queries(batch, qls)
    bufs = sw.upload_batch(batch, pad_bits=0x7E00)
    lay = bufs["layout"]
    max_q = int(nq.max())
    out = torch.full((qt.shape[0], cfg.n_qh, cfg.head_dim), float("nan"), dtype=torch.float16, device="cuda:0")
    print("mixed config run", name, qt.shape, flush=True)
    sw.sw_mixed_attn(to_dev(qt), bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"], i32(starts), i32(qls), out,
                     qt.shape[0], cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len, max_q)
    torch.cuda.synchronize()
    ref = oracle.mixed_attn(qt, bufs["k_host"], bufs["v_host"], batch.seq_lens, starts, qls, cfg.n_req, cfg.n_qh,
                            cfg.n_kvh, cfg.head_dim, cfg.max_len, max_q, lay.stride_req, lay.stride_kvh,
                            lay.stride_tok)
    errs = assert_parity(out.cpu().numpy(), ref, name)
    print(name, "mixed max_abs %.3e row_rel_l2 %.3e whole_rel_l2 %.3e" % errs)
