"""CPU tests of the piece-wise linear performance model (host logic only)."""
import numpy as np
import pytest

from paper_2311_18677_amd import perf_model as pm


def test_hat_basis_partitions_unity_interpolates_and_clamps():
    knots = [0.0, 1.0, 3.0, 7.0]
    x = np.array([-5.0, 0.0, 0.25, 1.0, 2.0, 6.9, 7.0, 99.0])
    h = pm.hat_basis(x, knots)
    assert h.shape == (8, 4) and np.allclose(h.sum(1), 1.0) and (h >= 0).all()
    vals = np.array([10.0, 20.0, 0.0, 4.0])
    got = h @ vals
    want = np.interp(np.clip(x, 0, 7), knots, vals)
    assert np.allclose(got, want)
    with pytest.raises(ValueError):
        pm.hat_basis(x, [0.0, 0.0, 1.0])


def test_model_recovers_a_function_that_is_linear_in_every_cell():
    bk, ck = (1, 4, 16, 64), (128, 512, 2048)
    rng = np.random.Generator(np.random.Philox(1))
    node = rng.uniform(5.0, 50.0, size=(len(bk), len(ck)))

    def truth(b, c):
        hb = pm.hat_basis(np.log2(b), np.log2(bk))
        hc = pm.hat_basis(np.log2(c), np.log2(ck))
        return np.einsum("ni,nj,ij->n", hb, hc, node)
    b = 2.0 ** rng.uniform(0, 6, 400)
    c = 2.0 ** rng.uniform(7, 11, 400)
    t = truth(b, c)
    res = pm.evaluate(b, c, t, bk, ck, seed=3)
    assert res["n_train"] == 320 and res["n_test"] == 80
    assert res["train_mape"] < 1e-4 and res["test_mape"] < 1e-4
    assert np.allclose(res["model"].coef.reshape(len(bk), len(ck)), node, rtol=1e-5)
    # outside the knot range the model holds the edge value
    assert np.allclose(res["model"].predict([1000.0], [128.0]), truth(np.array([64.0]), np.array([128.0])))


def test_latency_floor_plus_bandwidth_shape_is_fitted_within_a_few_percent():
    # the shape the token phase has: a launch floor, then time proportional to the bytes read
    b, c = np.meshgrid(pm.BATCHES, pm.CONTEXTS, indexing="ij")
    b, c = b.ravel().astype(float), c.ravel().astype(float)
    t = np.maximum(6.0, 4.0 + b * c * 512 / 5.5e6)
    rng = np.random.Generator(np.random.Philox(2))
    t = t * (1.0 + 0.01 * rng.standard_normal(t.size))
    res = pm.evaluate(b, c, t, pm.BATCH_KNOTS, pm.CONTEXT_KNOTS, seed=0)
    assert res["test_mape"] < 12.0 and res["train_mape"] < 10.0


def test_split_is_seeded_and_disjoint_and_mape_is_a_percentage():
    tr, te = pm.split_80_20(50, seed=7)
    tr2, te2 = pm.split_80_20(50, seed=7)
    assert np.array_equal(tr, tr2) and np.array_equal(te, te2)
    assert len(te) == 10 and len(tr) == 40 and not set(tr) & set(te)
    assert set(tr) | set(te) == set(range(50))
    assert pm.mape([110.0, 90.0], [100.0, 100.0]) == pytest.approx(10.0)


def test_regime_model_fits_a_surface_with_steps_at_the_breaks():
    rng = np.random.Generator(np.random.Philox(5))
    b = 2.0 ** rng.uniform(0, 7, 600)
    c = 2.0 ** rng.uniform(7, 13, 600)

    def truth(b, c):
        base = 3.0 + 0.002 * b * np.log2(c)                      # smooth part
        return base + np.where(c > 256, 2.0, 0.0) + np.where(c > 1024, 1.5, 0.0)   # steps at the breaks
    t = truth(b, c)
    res = pm.evaluate(b, c, t, pm.REGIME_BATCH_KNOTS, None, seed=1, regimes=pm.REGIMES)
    one = pm.evaluate(b, c, t, pm.BATCH_KNOTS, pm.CONTEXT_KNOTS, seed=1)
    assert res["test_mape"] < 1.5 and res["test_mape"] < 0.5 * one["test_mape"]
    m = res["model"]
    lo, hi = m.predict([8.0, 8.0], [256.0, 257.0])
    assert hi - lo > 1.5                                          # the step is kept, not smeared


def test_power_law_cells_reproduce_a_power_law():
    # with log_time the model is a power law inside every cell: t = a * b^0.5 * c^2 is exact
    b, c = np.meshgrid([1, 2, 3, 4, 6, 8], [64, 96, 128, 192, 256, 384, 512], indexing="ij")
    b, c = b.ravel().astype(float), c.ravel().astype(float)
    t = 0.01 * np.sqrt(b) * c ** 2
    m = pm.PiecewiseLinearModel((1, 2, 4, 8), (64, 128, 256, 512), log_time=True).fit(b, c, t)
    assert pm.mape(m.predict(b, c), t) < 1e-6
    # the time-linear form cannot follow the quadratic half-way between knots
    lin = pm.PiecewiseLinearModel((1, 2, 4, 8), (64, 128, 256, 512)).fit(b, c, t)
    assert pm.mape(lin.predict(b, c), t) > 1.0
    res = pm.evaluate(b, c, t, (1, 2, 4, 8), (64, 128, 256, 512), log_time=True)
    assert res["test_mape"] < 1e-6
