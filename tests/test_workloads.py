"""The seeded input generators: determinism, shapes, length recipes."""
import numpy as np

from paper_2311_18677_amd import workloads as wl


def test_same_seed_same_bytes_and_different_seed_differs():
    a = wl.make_batch("tiny_mha")
    b = wl.make_batch("tiny_mha")
    c = wl.make_batch("tiny_mha", seed=5)
    assert np.array_equal(a.q.view(np.uint16), b.q.view(np.uint16))
    for x, y in zip(a.k_rows + a.v_rows, b.k_rows + b.v_rows):
        assert np.array_equal(x.view(np.uint16), y.view(np.uint16))
    assert not np.array_equal(a.q.view(np.uint16), c.q.view(np.uint16))


def test_config_shapes_and_lengths():
    b = wl.make_batch("tiny_mha")
    assert list(b.seq_lens) == [1, 17, 64, 128] and b.total_tokens == 210
    assert b.kv_bytes == 430080
    assert b.q.shape == (4, 8, 64) and b.k_rows[1].shape == (8, 17, 64)
    cfg = wl.CONFIGS["llama70b_tp8"]
    lens = wl.draw_seq_lens(cfg, np.random.Generator(np.random.Philox(1)))
    assert lens.shape == (64,) and lens.min() >= 1000 and lens.max() <= 2600
    for name in ("bloom176b_tp8", "skewed_256"):
        cfg = wl.CONFIGS[name]
        many = np.concatenate([wl.draw_seq_lens(cfg, np.random.Generator(np.random.Philox(s)))
                               for s in range(40)])
        assert many.min() >= 16 and many.max() <= 8192
        assert 0.8 * cfg.lens[1] < np.median(many) < 1.25 * cfg.lens[1]
    assert wl.CONFIGS["longctx_8x32k"].lens[1] == (32768,) * 8


def test_values_are_standard_normal_rounded_to_half():
    cfg = wl.custom_config("v", 2, 4, 2, 128, 4096)
    b = wl.make_batch(cfg, seed=3, seq_lens=[4096, 2000])
    x = np.concatenate([r.reshape(-1) for r in b.k_rows]).astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert b.k_rows[0].dtype == np.float16


def test_scaled_key_rows():
    cfg = wl.Config("s", 2, 8, 1, 128, 4096, ("fixed", (4096, 4096)), k_row_scale=(0.1, 8.0))
    b = wl.make_batch(cfg, seed=9)
    rms = np.sqrt((b.k_rows[0].astype(np.float64) ** 2).mean(axis=-1)).reshape(-1)
    frac = (rms > 4.0).mean()
    assert 0.07 < frac < 0.13
    assert np.all(np.isfinite(b.k_rows[0].astype(np.float32)))


def test_pack_cache_places_rows_and_padding():
    cfg = wl.custom_config("p", 2, 2, 2, 64, 8)
    b = wl.make_batch(cfg, seed=1, seq_lens=[3, 8])
    sg = 8 * 64 + 128
    sr = 2 * sg
    buf = wl.pack_cache(b.k_rows, cfg, sr, sg, 64, 2 * sr, pad_bits=0x7E00)
    assert buf.size == 2 * sr
    assert np.array_equal(buf[sr + sg + 5 * 64: sr + sg + 6 * 64], b.k_rows[1][1, 5].view(np.uint16))
    assert np.all(buf[3 * 64: 8 * 64] == 0x7E00)          # positions past the length
    assert np.all(buf[8 * 64: sg] == 0x7E00)              # stride padding


def test_out_of_range_lengths_are_kept_for_the_library_but_clamped_for_data():
    cfg = wl.custom_config("c", 3, 2, 2, 64, 8)
    b = wl.make_batch(cfg, seed=1, seq_lens=[-4, 100, 0])
    assert list(b.seq_lens) == [-4, 100, 0]
    assert [r.shape[1] for r in b.k_rows] == [0, 8, 0]
