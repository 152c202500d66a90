"""Pins of the CPU oracle against what the definition and the mathematics fix.

None of these tests touches the GPU library.  Each pin is chosen so that a
plausible slip in oracle/sw_oracle.c (a dropped scale, a wrong head mapping, a
transposed index, a missing max subtraction, a wrong stride) fails at least
one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2311_18677_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def run_dense(q, k, v, lens, n_threads=0, stats=False):
    """q [R,Hq,d], k/v [R,Hk,M,d] float16 dense arrays."""
    R, Hq, d = q.shape
    _, Hk, M, _ = k.shape
    return oracle.decode_attn(
        np.ascontiguousarray(q), np.ascontiguousarray(k).reshape(-1),
        np.ascontiguousarray(v).reshape(-1), lens, R, Hq, Hk, d, M,
        Hk * M * d, M * d, d, n_threads=n_threads, return_stats=stats)


def brute(q, k, v, lens):
    """Dense matrix formulation written separately: softmax(Q K^T / sqrt(d)) V."""
    R, Hq, d = q.shape
    Hk = k.shape[1]
    G = Hq // Hk
    out = np.zeros((R, Hq, d))
    q64, k64, v64 = q.astype(np.float64), k.astype(np.float64), v.astype(np.float64)
    for r in range(R):
        L = int(lens[r])
        if L == 0:
            continue
        for h in range(Hq):
            Kmat = k64[r, h // G, :L, :]
            Vmat = v64[r, h // G, :L, :]
            w = scipy.special.softmax(Kmat @ q64[r, h] / math.sqrt(d))
            out[r, h] = w @ Vmat
    return out


def rnd(shape, seed, scale=1.0):
    g = np.random.Generator(np.random.Philox(seed))
    return (g.standard_normal(shape) * scale).astype(np.float16)


def test_half_decoder_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_golden_softmax_012():
    rows = {}
    with open(os.path.join(HERE, "golden", "softmax_012.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            rows[key] = [float(x) for x in vals]
    q = np.array(rows["q"], dtype=np.float16).reshape(1, 1, 4)
    k = np.array([rows["k0"], rows["k1"], rows["k2"]], dtype=np.float16).reshape(1, 1, 3, 4)
    v = np.array([rows["v0"], rows["v1"], rows["v2"]], dtype=np.float16).reshape(1, 1, 3, 4)
    ref = run_dense(q, k, v, [3])
    assert np.allclose(ref[0, 0], rows["out"], rtol=0, atol=1e-15)


def test_p1_single_token_returns_v_exactly():
    q, k, v = rnd((3, 4, 64), 1), rnd((3, 2, 5, 64), 2), rnd((3, 2, 5, 64), 3)
    ref = run_dense(q, k, v, [1, 1, 1])
    for r in range(3):
        for h in range(4):
            assert np.array_equal(ref[r, h], v[r, h // 2, 0].astype(np.float64))


def test_p2_identical_keys_give_mean_of_v():
    q, v = rnd((2, 2, 128), 4), rnd((2, 2, 37, 128), 5)
    k = np.repeat(rnd((2, 2, 1, 128), 6), 37, axis=2)
    ref = run_dense(q, k, v, [37, 20])
    assert np.allclose(ref[0], v[0, :, :37].astype(np.float64).mean(axis=1), rtol=1e-13, atol=1e-15)
    assert np.allclose(ref[1], v[1, :, :20].astype(np.float64).mean(axis=1), rtol=1e-13, atol=1e-15)
    # q = 0 is the same closed form
    ref0 = run_dense(np.zeros_like(q), rnd((2, 2, 37, 128), 7), v, [37, 37])
    assert np.allclose(ref0, v.astype(np.float64).mean(axis=2), rtol=1e-13, atol=1e-15)


def test_p3_dominant_key_returns_its_v():
    d, L, hot = 64, 50, 31
    q = np.zeros((1, 1, d), np.float16)
    q[0, 0, 0] = 16.0
    k = rnd((1, 1, L, d), 8, 0.01)
    k[0, 0, :, 0] = 0.0
    k[0, 0, hot, 0] = 40.0          # score 16*40/8 = 80, all others 0: margin 80 > 60
    v = rnd((1, 1, L, d), 9)
    ref = run_dense(q, k, v, [L])
    assert np.max(np.abs(ref[0, 0] - v[0, 0, hot].astype(np.float64))) <= 1e-20 * L * 10


@pytest.mark.parametrize("R,Hq,Hk,d,M", [(1, 1, 1, 2, 3), (3, 4, 2, 4, 9), (2, 4, 4, 64, 7),
                                           (2, 6, 2, 64, 9), (1, 8, 1, 128, 33)])
def test_p4_brute_force_matrix_formulation(R, Hq, Hk, d, M):
    q, k, v = rnd((R, Hq, d), 10), rnd((R, Hk, M, d), 11), rnd((R, Hk, M, d), 12)
    lens = [(M - 2 * r) if (M - 2 * r) > 0 else 1 for r in range(R)]
    ref = run_dense(q, k, v, lens)
    want = brute(q, k, v, lens)
    assert np.allclose(ref, want, rtol=1e-12, atol=1e-14)


def test_p5_key_shift_invariance():
    # adding a constant vector c to every key adds q.c/sqrt(d) to every score
    d, L = 64, 40
    q = rnd((1, 2, d), 13)
    # multiples of 2^-8 in [-0.4, 0.4], so that adding 0.5 is exact in binary16
    k_small = (np.clip(np.rint(rnd((1, 1, L, d), 14).astype(np.float32) * 32), -100, 100) / 256).astype(np.float16)
    c = np.zeros(d, np.float16)
    c[::3] = 0.5
    k_shift = (k_small.astype(np.float32) + c.astype(np.float32)).astype(np.float16)
    assert np.array_equal(k_shift.astype(np.float64), k_small.astype(np.float64) + c.astype(np.float64))
    v = rnd((1, 1, L, d), 15)
    a = run_dense(q, k_small, v, [L])
    b = run_dense(q, k_shift, v, [L])
    assert np.allclose(a, b, rtol=1e-10, atol=1e-13)


def test_p6_joint_permutation_of_keys_and_values():
    d, L = 128, 61
    q, k, v = rnd((1, 3, d), 16), rnd((1, 3, L, d), 17), rnd((1, 3, L, d), 18)
    perm = np.random.Generator(np.random.Philox(19)).permutation(L)
    a = run_dense(q, k, v, [L])
    b = run_dense(q, k[:, :, perm], v[:, :, perm], [L])
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)


def test_p7_convexity_and_weight_sum():
    d, L = 64, 90
    q, k, v = rnd((2, 2, d), 20), rnd((2, 2, L, d), 21), rnd((2, 2, L, d), 22)
    ref = run_dense(q, k, v, [L, L // 2])
    for r, Lr in enumerate([L, L // 2]):
        vv = v[r, :, :Lr].astype(np.float64)
        assert np.all(ref[r] >= vv.min(axis=1) - 1e-15)
        assert np.all(ref[r] <= vv.max(axis=1) + 1e-15)
    ones = np.ones_like(v)
    assert np.allclose(run_dense(q, k, ones, [L, L // 2]), 1.0, rtol=0, atol=1e-15)


@pytest.mark.parametrize("cuts", [(0, 13, 40), (0, 0, 40), (0, 1, 2, 39, 40), (0, 40, 40)])
def test_p8_chunk_merge_identity(cuts):
    # splitting [0, L) anywhere, running the oracle per piece and merging the
    # pieces' (o, m, l) gives the one-shot result; an empty piece has
    # m = -inf, l = 0 and contributes nothing.
    d, L, Hq, Hk = 64, 40, 4, 2
    q, k, v = rnd((1, Hq, d), 23), rnd((1, Hk, L, d), 24), rnd((1, Hk, L, d), 25)
    whole = run_dense(q, k, v, [L])
    parts = []
    for a, b in zip(cuts[:-1], cuts[1:]):
        n = b - a
        kk = np.ascontiguousarray(k[:, :, a:b]) if n else np.zeros((1, Hk, 1, d), np.float16)
        vv = np.ascontiguousarray(v[:, :, a:b]) if n else np.zeros((1, Hk, 1, d), np.float16)
        ref, m, l, _ = run_dense(q, kk, vv, [n], stats=True)
        parts.append((ref, m, l))
    m_all = np.max(np.stack([p[1] for p in parts]), axis=0)
    num = np.zeros_like(whole)
    den = np.zeros_like(m_all)
    for ref, m, l in parts:
        w = np.where(l > 0, np.exp(np.where(l > 0, m - m_all, 0.0)), 0.0)
        num += (w * l)[..., None] * ref
        den += w * l
    assert np.allclose(num / den[..., None], whole, rtol=1e-12, atol=1e-14)


def test_p9_gqa_equals_mha_with_replicated_kv_heads():
    d, L, Hq, Hk = 64, 23, 8, 2
    G = Hq // Hk
    q, k, v = rnd((2, Hq, d), 26), rnd((2, Hk, L, d), 27), rnd((2, Hk, L, d), 28)
    a = run_dense(q, k, v, [L, 5])
    b = run_dense(q, np.repeat(k, G, axis=1), np.repeat(v, G, axis=1), [L, 5])
    assert np.array_equal(a, b)
    # and the mapping is by contiguous groups: head h uses kv head h // G
    for h in range(Hq):
        one = run_dense(q[:, h:h + 1], k[:, h // G:h // G + 1], v[:, h // G:h // G + 1], [L, 5])
        assert np.array_equal(one[:, 0], a[:, h])


def test_p10_one_hot_values_expose_the_softmax():
    d, L = 64, 64
    q, k = rnd((1, 1, d), 29), rnd((1, 1, L, d), 30)
    v = np.zeros((1, 1, L, d), np.float16)
    v[0, 0, np.arange(L), np.arange(L)] = 1.0
    ref = run_dense(q, k, v, [L])
    s = k[0, 0].astype(np.float64) @ q[0, 0].astype(np.float64) / math.sqrt(d)
    assert np.allclose(ref[0, 0], scipy.special.softmax(s), rtol=1e-12, atol=1e-16)


def test_p11_large_scores_do_not_overflow():
    d, L = 4, 6
    q = np.full((1, 1, d), 65504.0, np.float16)
    k = np.zeros((1, 1, L, d), np.float16)
    k[0, 0, :, 0] = [65504, -65504, 65472, 100, 0, 65504]
    v = rnd((1, 1, L, d), 31)
    ref = run_dense(q, k, v, [L])
    assert np.all(np.isfinite(ref))
    # extended-precision rerun of the definition
    ld = np.longdouble
    s = (k[0, 0].astype(ld) @ q[0, 0].astype(ld)) / np.sqrt(ld(d))
    p = np.exp(s - s.max())
    want = (p[:, None] * v[0, 0].astype(ld)).sum(axis=0) / p.sum()
    assert np.allclose(ref[0, 0], want.astype(np.float64), rtol=1e-12, atol=1e-14)
    # config-4-style x8 key rows
    k2 = rnd((1, 1, 50, 64), 32)
    k2[0, 0, ::7] *= 8
    q2, v2 = rnd((1, 1, 64), 33), rnd((1, 1, 50, 64), 34)
    assert np.allclose(run_dense(q2, k2, v2, [50]), brute(q2, k2, v2, [50]), rtol=1e-12, atol=1e-14)


def test_length_clamp_and_zero_length():
    d, M = 64, 10
    q, k, v = rnd((4, 2, d), 35), rnd((4, 2, M, d), 36), rnd((4, 2, M, d), 37)
    ref, m, l, _ = run_dense(q, k, v, [0, -5, M + 7, 3], stats=True)
    assert np.array_equal(ref[0], np.zeros((2, d))) and not np.signbit(ref[0]).any()
    assert np.array_equal(ref[1], np.zeros((2, d)))
    assert np.all(l[:2] == 0) and np.all(np.isneginf(m[:2]))
    assert np.array_equal(ref[2], run_dense(q[2:3], k[2:3], v[2:3], [M])[0])
    assert np.allclose(ref[3], brute(q[3:4], k[3:4], v[3:4], [3])[0], rtol=1e-12, atol=1e-14)


def test_padding_is_never_read_and_strides_are_honoured():
    cfg = wl.custom_config("pad", 3, 4, 2, 64, 16)
    b = wl.make_batch(cfg, seed=77, seq_lens=[5, 16, 9])
    sr, sg, st, tot = wl.dense_layout(cfg)
    sg2 = sg + 3 * 64          # padded strides
    sr2 = cfg.n_kvh * sg2 + 64
    tot2 = cfg.n_req * sr2
    outs = []
    st3 = st + 8               # padded token rows as well
    sg3 = cfg.max_len * st3 + 24
    sr3 = cfg.n_kvh * sg3
    for (a, bb, c, t) in [(sr, sg, st, tot), (sr2, sg2, st, tot2), (sr3, sg3, st3, cfg.n_req * sr3)]:
        for pad in (0, 0x7E00, 0x7BFF):
            kb = wl.pack_cache(b.k_rows, cfg, a, bb, c, t, pad)
            vb = wl.pack_cache(b.v_rows, cfg, a, bb, c, t, pad)
            outs.append(oracle.decode_attn(b.q, kb, vb, b.seq_lens, 3, 4, 2, 64, 16, a, bb, c))
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    assert np.all(np.isfinite(outs[0]))


def test_thread_count_does_not_change_bits():
    q, k, v = rnd((5, 4, 64), 38), rnd((5, 2, 33, 64), 39), rnd((5, 2, 33, 64), 40)
    lens = [33, 1, 0, 17, 8]
    a = run_dense(q, k, v, lens, n_threads=1)
    b = run_dense(q, k, v, lens, n_threads=4)
    assert np.array_equal(a, b)


def test_tiny_config_matches_brute_force():
    b = wl.make_batch("tiny_mha")
    cfg = b.cfg
    assert list(b.seq_lens) == [1, 17, 64, 128]
    sr, sg, st, tot = wl.dense_layout(cfg)
    kb = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0x7E00)
    vb = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0x7E00)
    ref = oracle.decode_attn(b.q, kb, vb, b.seq_lens, 4, 8, 8, 64, 128, sr, sg, st)
    kd = np.zeros((4, 8, 128, 64), np.float16)
    vd = np.zeros((4, 8, 128, 64), np.float16)
    for r in range(4):
        L = b.seq_lens[r]
        kd[r, :, :L] = b.k_rows[r]
        vd[r, :, :L] = b.v_rows[r]
    assert np.allclose(ref, brute(b.q, kd, vd, b.seq_lens), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("block_size", [4, 16, 32])
def test_paged_oracle_equals_dense_oracle(block_size):
    # the block-table routine is pinned to the dense one: whatever the block size
    # and however the blocks are scattered, the result has the same bits
    cfg = wl.custom_config("pg", 5, 6, 2, 64, 96)
    b = wl.make_batch(cfg, seed=91, seq_lens=[96, 1, 0, 33, 64])
    sr, sg, st, tot = wl.dense_layout(cfg)
    kb = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0x7E00)
    vb = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0x7E00)
    dense = oracle.decode_attn(b.q, kb, vb, b.seq_lens, 5, 6, 2, 64, 96, sr, sg, st)
    sb, sgp, stp = wl.dense_paged_layout(cfg, block_size)
    sb += 64                                     # padded block stride
    n_blocks = 5 * (96 // block_size) + 3
    for seed in (0, 1):
        kp, vp, table = wl.pack_paged(b.k_rows, b.v_rows, cfg, block_size, sb, sgp, stp, n_blocks,
                                      seed=seed, pad_bits=0x7E00)
        paged = oracle.decode_attn_paged(b.q, kp, vp, table, b.seq_lens, 5, 6, 2, 64, block_size,
                                         96 // block_size, n_blocks, sb, sgp, stp)
        assert np.array_equal(paged, dense)
    assert np.all(np.isfinite(dense))


def test_paged_oracle_matches_brute_force_and_clamps():
    cfg = wl.custom_config("pg2", 3, 4, 4, 64, 32)
    b = wl.make_batch(cfg, seed=92, seq_lens=[7, 32, 19])
    sb, sg, st = wl.dense_paged_layout(cfg, 8)
    kp, vp, table = wl.pack_paged(b.k_rows, b.v_rows, cfg, 8, sb, sg, st, 12, seed=3)
    kd = np.zeros((3, 4, 32, 64), np.float16)
    vd = np.zeros((3, 4, 32, 64), np.float16)
    for r in range(3):
        L = b.seq_lens[r]
        kd[r, :, :L] = b.k_rows[r]
        vd[r, :, :L] = b.v_rows[r]
    got = oracle.decode_attn_paged(b.q, kp, vp, table, b.seq_lens, 3, 4, 4, 64, 8, 4, 12, sb, sg, st)
    assert np.allclose(got, brute(b.q, kd, vd, b.seq_lens), rtol=1e-12, atol=1e-14)
    # lengths above max_blocks*block_size clamp; length <= 0 gives zeros
    lens2 = np.array([-1, 99, 19], np.int32)
    got2 = oracle.decode_attn_paged(b.q, kp, vp, table, lens2, 3, 4, 4, 64, 8, 4, 12, sb, sg, st)
    assert np.array_equal(got2[0], np.zeros((4, 64))) and np.array_equal(got2[1], got[1])


# ---- append-then-attend (the cache side of one decode iteration) ----

def _dense_views(buf, cfg, sr, sg, st):
    return np.lib.stride_tricks.as_strided(
        buf, shape=(cfg.n_req, cfg.n_kvh, cfg.max_len, cfg.head_dim), strides=(2 * sr, 2 * sg, 2 * st, 2))


def test_kv_append_matches_array_slicing_and_touches_nothing_else():
    cfg = wl.custom_config("ap", 5, 6, 2, 64, 48)
    lens = np.array([0, 47, 48, 13, -3], np.int32)       # empty, last free slot, full, middle, negative
    b = wl.make_batch(cfg, seed=93, seq_lens=lens)
    kn, vn = wl.make_new_rows(cfg, 93)
    sr, sg, st, tot = wl.dense_layout(cfg)
    sg += 24; sr = 2 * sg + 40; tot = 5 * sr               # padded strides
    k = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0x7E00)
    v = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0x7E01)
    ek, ev = k.copy(), v.copy()
    ekv, evv = _dense_views(ek, cfg, sr, sg, st), _dense_views(ev, cfg, sr, sg, st)
    for r, pos in enumerate([0, 47, None, 13, 0]):
        if pos is not None:
            ekv[r, :, pos, :] = kn[r].view(np.uint16)
            evv[r, :, pos, :] = vn[r].view(np.uint16)
    out = oracle.kv_append(kn, vn, k, v, lens, 5, 2, 64, 48, sr, sg, st)
    assert out.tolist() == [1, 48, 48, 14, 1]
    assert np.array_equal(k, ek) and np.array_equal(v, ev)
    assert not np.array_equal(k, v)                       # K rows went to K, V rows to V


def test_append_then_attend_equals_attending_over_the_longer_context():
    # a step of the append variant = the plain step on a cache that already holds the token
    cfg = wl.custom_config("ap2", 4, 4, 2, 64, 40)
    lens = np.array([5, 39, 0, 40], np.int32)
    b = wl.make_batch(cfg, seed=94, seq_lens=lens)
    kn, vn = wl.make_new_rows(cfg, 94)
    sr, sg, st, tot = wl.dense_layout(cfg)
    k = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0x7E00)
    v = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0x7E00)
    new_lens = oracle.kv_append(kn, vn, k, v, lens, 4, 2, 64, 40, sr, sg, st)
    got = oracle.decode_attn(b.q, k, v, new_lens, 4, 4, 2, 64, 40, sr, sg, st)
    kd = np.zeros((4, 2, 40, 64), np.float16)
    vd = np.zeros((4, 2, 40, 64), np.float16)
    longer = []
    for r in range(4):
        L = int(lens[r])
        kr, vr = b.k_rows[r], b.v_rows[r]
        if L < 40:
            kr = np.concatenate([kr, kn[r][:, None, :]], axis=1)
            vr = np.concatenate([vr, vn[r][:, None, :]], axis=1)
        kd[r, :, :kr.shape[1]] = kr
        vd[r, :, :vr.shape[1]] = vr
        longer.append(kr.shape[1])
    assert new_lens.tolist() == longer == [6, 40, 1, 40]
    assert np.allclose(got, brute(b.q, kd, vd, np.array(longer, np.int32)), rtol=1e-12, atol=1e-14)
    # the request with an empty cache attends over its own token only: the result is v_new
    g = np.repeat(np.arange(2), 2)
    assert np.array_equal(got[2], vn[2][g].astype(np.float64))


@pytest.mark.parametrize("block_size", [4, 16])
def test_paged_kv_append_equals_dense_kv_append(block_size):
    cfg = wl.custom_config("ap3", 5, 4, 2, 64, 64)
    lens = np.array([0, 16, 63, 64, 21], np.int32)        # new block needed, last slot, full
    b = wl.make_batch(cfg, seed=95, seq_lens=lens)
    kn, vn = wl.make_new_rows(cfg, 95)
    sr, sg, st, tot = wl.dense_layout(cfg)
    k = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0)
    v = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0)
    new_lens = oracle.kv_append(kn, vn, k, v, lens, 5, 2, 64, 64, sr, sg, st)
    dense = oracle.decode_attn(b.q, k, v, new_lens, 5, 4, 2, 64, 64, sr, sg, st)
    sb, sgp, stp = wl.dense_paged_layout(cfg, block_size)
    mb = 64 // block_size
    n_blocks = 5 * mb + 2
    kp, vp, table = wl.pack_paged(b.k_rows, b.v_rows, cfg, block_size, sb, sgp, stp, n_blocks,
                                  seed=5, pad_bits=0x7E00, room=1)
    kp0 = kp.copy()
    lens_p = oracle.kv_append_paged(kn, vn, kp, vp, table, lens, 5, 2, 64, block_size, mb, n_blocks,
                                    sb, sgp, stp)
    assert np.array_equal(lens_p, new_lens)
    assert int((kp != kp0).any(axis=None)) and np.count_nonzero(kp != kp0) <= 4 * 2 * 64
    paged = oracle.decode_attn_paged(b.q, kp, vp, table, lens_p, 5, 4, 2, 64, block_size, mb, n_blocks,
                                     sb, sgp, stp)
    assert np.array_equal(paged, dense) and np.all(np.isfinite(paged))


# ---- prompt phase (causal) ----

def _prefill_case(n_qh, n_kvh, d, max_len, lens, seed):
    cfg = wl.custom_config("pf", len(lens), n_qh, n_kvh, d, max_len)
    b = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    qt, starts = wl.make_prefill_queries(b)
    sr, sg, st, tot = wl.dense_layout(cfg)
    k = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0x7E00)
    v = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0x7E00)
    ref = oracle.prefill_attn(qt, k, v, b.seq_lens, starts, cfg.n_req, n_qh, n_kvh, d, max_len, sr, sg, st)
    return cfg, b, qt, starts, k, v, (sr, sg, st), ref


def test_prefill_row_i_is_the_decode_step_at_length_i_plus_1():
    cfg, b, qt, starts, k, v, (sr, sg, st), ref = _prefill_case(4, 2, 64, 24, [24, 1, 0, 9], 96)
    assert ref.shape == (34, 4, 64)
    for r, L in enumerate([24, 1, 0, 9]):
        for i in range(L):
            q1 = np.zeros((cfg.n_req, 4, 64), np.float16)
            q1[r] = qt[starts[r] + i]
            lens1 = np.zeros(cfg.n_req, np.int32)
            lens1[r] = i + 1
            dec = oracle.decode_attn(q1, k, v, lens1, cfg.n_req, 4, 2, 64, 24, sr, sg, st)
            assert np.array_equal(ref[starts[r] + i], dec[r])
    # the first token of a prompt sees itself only: its row is V[0] exactly
    g = np.repeat(np.arange(2), 2)
    assert np.array_equal(ref[starts[0]], b.v_rows[0][g, 0, :].astype(np.float64))


def test_prefill_matches_masked_matrix_formulation():
    cfg, b, qt, starts, k, v, _, ref = _prefill_case(6, 3, 64, 40, [40, 17, 3], 97)
    for r, L in enumerate([40, 17, 3]):
        for h in range(6):
            g = h // 2
            q = qt[starts[r]:starts[r] + L, h].astype(np.float64)
            kk = b.k_rows[r][g].astype(np.float64)
            vv = b.v_rows[r][g].astype(np.float64)
            s = q @ kk.T / np.sqrt(64.0)
            s[np.triu_indices(L, 1)] = -np.inf          # token i does not see positions > i
            want = scipy.special.softmax(s, axis=1) @ vv
            assert np.allclose(ref[starts[r]:starts[r] + L, h], want, rtol=1e-12, atol=1e-14)


def test_prefill_rows_do_not_depend_on_later_positions_or_other_requests():
    cfg, b, qt, starts, k, v, (sr, sg, st), ref = _prefill_case(4, 4, 64, 32, [32, 20], 98)
    # scramble every cached position >= 12 of request 0: rows 0..11 keep their bits
    k2, v2 = k.copy(), v.copy()
    kv = np.lib.stride_tricks.as_strided(k2, shape=(2, 4, 32, 64), strides=(2 * sr, 2 * sg, 2 * st, 2))
    vv = np.lib.stride_tricks.as_strided(v2, shape=(2, 4, 32, 64), strides=(2 * sr, 2 * sg, 2 * st, 2))
    kv[0, :, 12:, :] = 0x7E00
    vv[0, :, 12:, :] = 0x7E00
    ref2 = oracle.prefill_attn(qt, k2, v2, b.seq_lens, starts, 2, 4, 4, 64, 32, sr, sg, st)
    assert np.array_equal(ref2[:12], ref[:12]) and np.array_equal(ref2[32:], ref[32:])
    assert not np.all(np.isfinite(ref2[12:32]))
    # unpacked query rows (a gap between the requests, reversed order) give the same rows
    qt3 = np.zeros((70, 4, 64), np.float16)
    qt3[40:60] = qt[32:52]
    qt3[3:35] = qt[0:32]
    ref3 = oracle.prefill_attn(qt3, k, v, b.seq_lens, [3, 40], 2, 4, 4, 64, 32, sr, sg, st)
    assert np.array_equal(ref3[3:35], ref[0:32]) and np.array_equal(ref3[40:60], ref[32:52])
    assert not ref3[:3].any() and not ref3[35:40].any() and not ref3[60:].any()
    with pytest.raises(ValueError):
        oracle.prefill_attn(qt, k, v, b.seq_lens, [0, 40], 2, 4, 4, 64, 32, sr, sg, st)


# ---- KV hand-off: pools <-> dense, transfer spans ----

def test_kv_pack_of_pools_equals_the_dense_buffer_of_the_same_batch_and_round_trips():
    cfg = wl.custom_config("pk", 5, 4, 2, 64, 64)
    lens = [0, 1, 17, 64, 40]
    b = wl.make_batch(cfg, seed=99, seq_lens=lens)
    sr, sg, st, tot = wl.dense_layout(cfg)
    sg += 64; sr = 2 * sg + 128; tot = 5 * sr
    want_k = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, 0x1234)
    want_v = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, 0x1234)
    for bs in (4, 16):
        sb, sgp, stp = wl.dense_paged_layout(cfg, bs)
        sb += 32
        mb, nb = 64 // bs, 5 * (64 // bs) + 2
        kp, vp, table = wl.pack_paged(b.k_rows, b.v_rows, cfg, bs, sb, sgp, stp, nb, seed=bs, pad_bits=0x7E00)
        kd = np.full(tot, 0x1234, np.uint16)
        vd = np.full(tot, 0x1234, np.uint16)
        geom = (5, 2, 64, 64, bs, mb, nb, sb, sgp, sr, sg, st)
        oracle.kv_pack(kp, vp, table, lens, kd, vd, True, *geom)
        assert np.array_equal(kd, want_k) and np.array_equal(vd, want_v)    # and padding untouched
        # back into fresh pools: the valid rows return, everything else keeps its fill
        kp2 = np.full(kp.size, 0x4321, np.uint16)
        vp2 = np.full(vp.size, 0x4321, np.uint16)
        oracle.kv_pack(kp2, vp2, table, lens, kd, vd, False, *geom)
        kp_ref, vp_ref, _ = wl.pack_paged(b.k_rows, b.v_rows, cfg, bs, sb, sgp, stp, nb, seed=bs, pad_bits=0x4321)
        assert np.array_equal(kp2, kp_ref) and np.array_equal(vp2, vp_ref)
        assert not np.array_equal(kd, vd)


def test_kv_span_plan_matches_brute_force():
    rng = np.random.Generator(np.random.Philox(100))
    n_req, bs, mb, nb = 7, 8, 12, 64
    lens = np.array([0, 1, 8, 9, 96, 50, 200], np.int32)          # 200 clamps to 96
    table = rng.integers(0, nb, size=(n_req, mb)).astype(np.int32)
    table[4] = np.arange(10, 22)                                   # one span
    table[5, :7] = [3, 4, 5, 9, 10, 2, 3]                          # 3 spans: [3,4,5] [9,10] [2,3]
    table[6, :4] = [70, 71, -5, 1]                                 # clamped ids: 63, 63, 0, 1
    first, count, n = oracle.kv_span_plan(table, lens, n_req, bs, mb, nb)
    for r in range(n_req):
        L = min(max(int(lens[r]), 0), mb * bs)
        ids = np.clip(table[r, :-(-L // bs)], 0, nb - 1).tolist()
        spans = []
        for i, b in enumerate(ids):
            if i and b == ids[i - 1] + 1:
                spans[-1][1] += 1
            else:
                spans.append([b, 1])
        assert n[r] == len(spans)
        assert first[r, :n[r]].tolist() == [s[0] for s in spans]
        assert count[r, :n[r]].tolist() == [s[1] for s in spans]
        assert (first[r, n[r]:] == -1).all() and (count[r, n[r]:] == -1).all()
        assert count[r, :n[r]].sum() == len(ids)
    assert n[4] == 1 and n[5] == 3 and n[0] == 0
    assert first[6, :3].tolist() == [63, 63, 0] and count[6, :3].tolist() == [1, 1, 2]


# ---- mixed batch: the last q_lens tokens of every request are queries ----

def test_mixed_batch_reduces_to_prompt_phase_and_to_token_phase():
    cfg, b, qt, starts, k, v, (sr, sg, st), ref = _prefill_case(4, 2, 64, 24, [24, 1, 0, 9], 101)
    lens = b.seq_lens
    # all tokens as queries: the prompt routine
    full = oracle.mixed_attn(qt, k, v, lens, starts, lens, 4, 4, 2, 64, 24, 24, sr, sg, st)
    assert np.array_equal(full, ref)
    # one query per request: the token-phase step on the same cache
    q1 = np.stack([qt[starts[r] + max(int(L) - 1, 0)] if L > 0 else np.zeros((4, 64), np.float16)
                   for r, L in enumerate(lens)])
    dec = oracle.decode_attn(q1, k, v, lens, 4, 4, 2, 64, 24, sr, sg, st)
    one = oracle.mixed_attn(q1, k, v, lens, [0, 1, 2, 3], [1, 1, 1, 1], 4, 4, 2, 64, 24, 24, sr, sg, st)
    assert np.array_equal(one[[0, 1, 3]], dec[[0, 1, 3]]) and not one[2].any()


def test_a_prompt_in_two_pieces_gives_the_rows_of_the_prompt_in_one_piece():
    cfg, b, qt, starts, k, v, (sr, sg, st), ref = _prefill_case(4, 4, 64, 40, [40, 23], 102)
    # piece 1: the first 17 (resp. 10) tokens; piece 2: the rest, with the whole prompt cached
    cut = np.array([17, 10], np.int32)
    q_a = np.concatenate([qt[0:17], qt[40:50]])
    a = oracle.mixed_attn(q_a, k, v, cut, [0, 17], cut, 2, 4, 4, 64, 40, 40, sr, sg, st)
    q_b = np.concatenate([qt[17:40], qt[50:63]])
    bq = np.array([23, 13], np.int32)
    bb = oracle.mixed_attn(q_b, k, v, b.seq_lens, [0, 23], bq, 2, 4, 4, 64, 40, 40, sr, sg, st)
    assert np.array_equal(a[:17], ref[0:17]) and np.array_equal(a[17:], ref[40:50])
    assert np.array_equal(bb[:23], ref[17:40]) and np.array_equal(bb[23:], ref[50:63])
    # q_lens above the length or above max_q_len are clamped; negative counts give no rows
    c = oracle.mixed_attn(qt[:8], k, v, [5, 3], [0, 5], [99, 3], 2, 4, 4, 64, 40, 40, sr, sg, st)
    d = oracle.mixed_attn(qt[:8], k, v, [5, 3], [0, 5], [5, 3], 2, 4, 4, 64, 40, 40, sr, sg, st)
    assert np.array_equal(c, d)
    e = oracle.mixed_attn(qt[:8], k, v, [5, 3], [0, 2], [99, -4], 2, 4, 4, 64, 40, 2, sr, sg, st)
    f = oracle.mixed_attn(qt[:8], k, v, [5, 3], [0, 2], [2, 0], 2, 4, 4, 64, 40, 40, sr, sg, st)
    assert np.array_equal(e, f) and not e[2:].any()


@pytest.mark.parametrize("block_size", [4, 8, 16])
def test_paged_mixed_batch_equals_the_dense_routine_bit_for_bit(block_size):
    lens = [40, 23, 1, 0, 17]
    cfg, b, qt, starts, k, v, (sr, sg, st), ref = _prefill_case(4, 2, 64, 40, lens, 110 + block_size)
    sb, sgp, stp = wl.dense_paged_layout(cfg, block_size)
    max_blocks = -(-40 // block_size)
    n_blocks = sum(-(-L // block_size) for L in lens) + 5
    kp, vp, table = wl.pack_paged(b.k_rows, b.v_rows, cfg, block_size, sb, sgp, stp, n_blocks,
                                  seed=block_size, pad_bits=0x7E00)
    # every cached token a query: the prompt phase
    full = oracle.mixed_attn_paged(qt, kp, vp, table, b.seq_lens, starts, None, 5, 4, 2, 64,
                                   block_size, max_blocks, n_blocks, 40, sb, sgp, stp)
    assert np.array_equal(full, ref)
    # a mixed batch: prompt, piece, token phase, nothing, token phase
    qls = [40, 9, 1, 0, 1]
    qm, sm, nq = wl.make_mixed_queries(b, qls)
    dense = oracle.mixed_attn(qm, k, v, b.seq_lens, sm, qls, 5, 4, 2, 64, 40, 40, sr, sg, st)
    paged = oracle.mixed_attn_paged(qm, kp, vp, table, b.seq_lens, sm, qls, 5, 4, 2, 64,
                                    block_size, max_blocks, n_blocks, 40, sb, sgp, stp)
    assert np.array_equal(paged, dense) and dense.any()
    # the bound on the queries of a request
    dense = oracle.mixed_attn(qm, k, v, b.seq_lens, sm, qls, 5, 4, 2, 64, 40, 7, sr, sg, st)
    paged = oracle.mixed_attn_paged(qm, kp, vp, table, b.seq_lens, sm, qls, 5, 4, 2, 64,
                                    block_size, max_blocks, n_blocks, 7, sb, sgp, stp)
    assert np.array_equal(paged, dense)
    # block ids out of range are clamped into the pool, lengths to the table's reach
    wild = table.copy()
    wild[0, 0] = n_blocks + 100
    ok = table.copy()
    ok[0, 0] = n_blocks - 1
    a = oracle.mixed_attn_paged(qm, kp, vp, wild, [99, 23, 1, 0, 17], sm, qls, 5, 4, 2, 64,
                                block_size, max_blocks, n_blocks, 40, sb, sgp, stp)
    c = oracle.mixed_attn_paged(qm, kp, vp, ok, [max_blocks * block_size, 23, 1, 0, 17], sm, qls, 5, 4, 2, 64,
                                block_size, max_blocks, n_blocks, 40, sb, sgp, stp)
    assert np.array_equal(a, c, equal_nan=True)


def _store_case(n_kvh, d, max_len, lens, seed, pad=0x7E00):
    cfg = wl.custom_config("st", len(lens), n_kvh, n_kvh, d, max_len)
    b = wl.make_batch(cfg, seed=seed, seq_lens=lens)
    sr, sg, st, tot = wl.dense_layout(cfg)
    full_k = wl.pack_cache(b.k_rows, cfg, sr, sg, st, tot, pad)
    full_v = wl.pack_cache(b.v_rows, cfg, sr, sg, st, tot, pad)
    return cfg, b, (sr, sg, st, tot), full_k, full_v


def test_store_of_whole_prompts_builds_the_cache_and_touches_nothing_else():
    lens = [24, 1, 0, 9, 17]
    cfg, b, (sr, sg, st, tot), full_k, full_v = _store_case(2, 64, 24, lens, 120)
    k_tok, v_tok, starts, nq = wl.token_rows(b)
    k = np.full(tot, 0x7E00, np.uint16)
    v = np.full(tot, 0x7E00, np.uint16)
    oracle.kv_store(k_tok, v_tok, k, v, b.seq_lens, starts, None, 5, 2, 64, 24, 24, sr, sg, st)
    assert np.array_equal(k, full_k) and np.array_equal(v, full_v)
    # by slicing, on strides with padding everywhere (token stride 80, head and request gaps)
    st2, sg2, sr2 = 80, 24 * 80 + 16, 2 * (24 * 80 + 16) + 48
    tot2 = 5 * sr2
    k2 = np.full(tot2, 0x1234, np.uint16)
    v2 = np.full(tot2, 0x4321, np.uint16)
    oracle.kv_store(k_tok, v_tok, k2, v2, b.seq_lens, starts, None, 5, 2, 64, 24, 24, sr2, sg2, st2)
    want_k = np.full(tot2, 0x1234, np.uint16)
    want_v = np.full(tot2, 0x4321, np.uint16)
    for r, L in enumerate(lens):
        for g in range(2):
            for t in range(L):
                o = r * sr2 + g * sg2 + t * st2
                want_k[o:o + 64] = b.k_rows[r][g, t].view(np.uint16)
                want_v[o:o + 64] = b.v_rows[r][g, t].view(np.uint16)
    assert np.array_equal(k2, want_k) and np.array_equal(v2, want_v)


def test_store_of_the_last_tokens_and_its_clamps():
    lens = [24, 5, 0, 9, 17]
    cfg, b, (sr, sg, st, tot), full_k, full_v = _store_case(2, 64, 24, lens, 121)
    qls = [7, 1, 3, 99, 0]                       # piece, token phase, nothing cached, more than cached, none
    k_tok, v_tok, starts, nq = wl.token_rows(b, qls)
    assert nq.tolist() == [7, 1, 0, 9, 0]
    # a cache that holds everything but the new rows (NaN there): the store completes it
    k, v = full_k.copy(), full_v.copy()
    kk = np.lib.stride_tricks.as_strided(k, shape=(5, 2, 24, 64), strides=(2 * sr, 2 * sg, 2 * st, 2), writeable=True)
    vv = np.lib.stride_tricks.as_strided(v, shape=(5, 2, 24, 64), strides=(2 * sr, 2 * sg, 2 * st, 2), writeable=True)
    for r, (L, n) in enumerate(zip(lens, nq)):
        kk[r, :, L - n:L, :] = 0x7E00
        vv[r, :, L - n:L, :] = 0x7E00
    before_k = k.copy()
    oracle.kv_store(k_tok, v_tok, k, v, b.seq_lens, starts, qls, 5, 2, 64, 24, 24, sr, sg, st)
    assert np.array_equal(k, full_k) and np.array_equal(v, full_v) and not np.array_equal(before_k, full_k)
    # the bound on new tokens per request: only the last max_q_len are stored
    k3, v3 = before_k.copy(), v.copy()
    kt3, vt3, s3, n3 = wl.token_rows(b, [3, 1, 0, 3, 0])
    oracle.kv_store(kt3, vt3, k3, v3, b.seq_lens, s3, qls, 5, 2, 64, 24, 3, sr, sg, st)
    k3v = np.lib.stride_tricks.as_strided(k3, shape=(5, 2, 24, 64), strides=(2 * sr, 2 * sg, 2 * st, 2))
    fkv = np.lib.stride_tricks.as_strided(full_k, shape=(5, 2, 24, 64), strides=(2 * sr, 2 * sg, 2 * st, 2))
    assert np.array_equal(k3v[0, :, 21:24], fkv[0, :, 21:24]) and (k3v[0, :, 17:21] == 0x7E00).all()
    # lengths above max_len count as max_len
    k4, v4 = before_k.copy(), v.copy()
    oracle.kv_store(k_tok, v_tok, k4, v4, [99, 5, 0, 9, 17], starts, qls, 5, 2, 64, 24, 24, sr, sg, st)
    assert np.array_equal(k4, full_k)
    # rows that would leave the token arrays are refused
    with pytest.raises(ValueError):
        oracle.kv_store(k_tok, v_tok, k4, v4, b.seq_lens, [0, 7, 8, 9, 17], qls, 5, 2, 64, 24, 24, sr, sg, st)


def test_store_of_one_token_is_the_append_routine():
    lens = [10, 1, 24, 7]
    cfg, b, (sr, sg, st, tot), full_k, full_v = _store_case(3, 64, 24, lens, 122)
    k_new, v_new = wl.make_new_rows(cfg, 122)
    before = np.array([9, 0, 23, 6], np.int32)
    ka, va = full_k.copy(), full_v.copy()
    after = oracle.kv_append(k_new, v_new, ka, va, before, 4, 3, 64, 24, sr, sg, st)
    assert after.tolist() == lens
    ks, vs = full_k.copy(), full_v.copy()
    oracle.kv_store(k_new, v_new, ks, vs, after, [0, 1, 2, 3], [1, 1, 1, 1], 4, 3, 64, 24, 1, sr, sg, st)
    assert np.array_equal(ka, ks) and np.array_equal(va, vs) and not np.array_equal(ks, full_k)


@pytest.mark.parametrize("block_size", [4, 16])
def test_store_into_block_pools_equals_the_dense_store(block_size):
    lens = [24, 5, 0, 9, 17]
    cfg, b, (sr, sg, st, tot), full_k, full_v = _store_case(2, 64, 24, lens, 123)
    qls = [7, 1, 3, 99, 17]
    k_tok, v_tok, starts, nq = wl.token_rows(b, qls)
    sb, sgp, stp = wl.dense_paged_layout(cfg, block_size)
    max_blocks = -(-24 // block_size)
    n_blocks = sum(-(-L // block_size) for L in lens) + 4
    # pools that hold the batch; wipe the new rows, store them again, compare with the pools as packed
    kp, vp, table = wl.pack_paged(b.k_rows, b.v_rows, cfg, block_size, sb, sgp, stp, n_blocks, seed=5, pad_bits=0x7E00)
    kp0, vp0 = kp.copy(), vp.copy()
    kv = np.lib.stride_tricks.as_strided(kp, shape=(n_blocks, 2, block_size, 64), strides=(2 * sb, 2 * sgp, 2 * stp, 2), writeable=True)
    vv = np.lib.stride_tricks.as_strided(vp, shape=(n_blocks, 2, block_size, 64), strides=(2 * sb, 2 * sgp, 2 * stp, 2), writeable=True)
    for r, (L, n) in enumerate(zip(lens, nq)):
        for t in range(L - n, L):
            kv[table[r, t // block_size], :, t % block_size, :] = 0
            vv[table[r, t // block_size], :, t % block_size, :] = 0
    assert not np.array_equal(kp, kp0)
    oracle.kv_store(k_tok, v_tok, kp, vp, b.seq_lens, starts, qls, 5, 2, 64, 24, 24, sb, sgp, stp,
                    block_table=table, block_size=block_size, max_blocks=max_blocks, n_blocks=n_blocks)
    assert np.array_equal(kp, kp0) and np.array_equal(vp, vp0)


def test_store_then_attend_is_attention_over_the_cache_built_directly():
    lens = [24, 9, 17]
    cfg, b, (sr, sg, st, tot), full_k, full_v = _store_case(2, 64, 24, lens, 124, pad=0)
    qt, qs = wl.make_prefill_queries(b)
    k_tok, v_tok, starts, nq = wl.token_rows(b)
    k = np.zeros(tot, np.uint16)
    v = np.zeros(tot, np.uint16)
    oracle.kv_store(k_tok, v_tok, k, v, b.seq_lens, starts, None, 3, 2, 64, 24, 24, sr, sg, st)
    a = oracle.prefill_attn(qt, k, v, b.seq_lens, qs, 3, 2, 2, 64, 24, sr, sg, st)
    c = oracle.prefill_attn(qt, full_k, full_v, b.seq_lens, qs, 3, 2, 2, 64, 24, sr, sg, st)
    assert np.array_equal(a, c) and a.any()
