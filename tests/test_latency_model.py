"""CPU tests of the Eq. 1 fit (paper Sec. 5.2): Lat(B, A) = (K4 B + K5)(K6 A + K7) with K7 fixed to 1."""
import numpy as np
import pytest

from paper_2602_24044_amd import latency_model as lm


def _grid():
    B, A = np.meshgrid([32, 64, 128, 256, 512], [0, 1, 2, 4, 8, 16, 32], indexing="ij")
    return B.ravel().astype(float), A.ravel().astype(float)


def test_fit_recovers_exact_constants():
    B, A = _grid()
    true = (0.31, 95.0, 0.012, 1.0)
    r = lm.fit(B, A, lm.predict(true, B, A))
    assert r["K4"] == pytest.approx(true[0], rel=1e-6)
    assert r["K5"] == pytest.approx(true[1], rel=1e-6)
    assert r["K6"] == pytest.approx(true[2], rel=1e-6)
    assert r["smape_percent"] < 1e-6 and r["max_rel_err"] < 1e-8


def test_fit_is_scale_invariant_in_the_product():
    # (K4, K5, K6, K7) and (c K4, c K5, K6 / c', K7 / c') describe the same law; with K7 = 1 the fit returns the
    # normalised constants whatever scale the data were generated with
    B, A = _grid()
    r = lm.fit(B, A, lm.predict((0.2, 50.0, 0.03, 2.0), B, A))
    assert r["K4"] == pytest.approx(0.4, rel=1e-6) and r["K5"] == pytest.approx(100.0, rel=1e-6)
    assert r["K6"] == pytest.approx(0.015, rel=1e-6)


def test_fit_with_noise_stays_close():
    rng = np.random.default_rng(0)
    B, A = _grid()
    true = (0.31, 95.0, 0.012, 1.0)
    y = lm.predict(true, B, A) * (1.0 + 0.02 * rng.standard_normal(B.shape))
    r = lm.fit(B, A, y)
    assert r["K4"] == pytest.approx(true[0], rel=0.1) and r["K5"] == pytest.approx(true[1], rel=0.1)
    assert r["K6"] == pytest.approx(true[2], rel=0.15)
    assert r["smape_percent"] < 3.0


def test_fit_rejects_bad_input():
    with pytest.raises(ValueError):
        lm.fit([1, 2], [0, 1], [1.0, 2.0])
    with pytest.raises(ValueError):
        lm.fit([1, 2, 3], [0, 1], [1.0, 2.0, 3.0])


def test_additive_fit_recovers_exact_constants():
    B, A = _grid()
    y = 0.3 * B + 150.0 + 0.5 * A + 20.0 * (A >= 1)
    r = lm.fit_additive(B, A, y)
    assert r["c_B"] == pytest.approx(0.3) and r["c_0"] == pytest.approx(150.0)
    assert r["c_A"] == pytest.approx(0.5) and r["c_step"] == pytest.approx(20.0)
    assert r["max_rel_err"] < 1e-9


def test_slot_region_bytes():
    # one rank unit of a two-layer model with projections (64 -> 128) and (128 -> 64): 2 layers x 384 elements x 2 bytes
    from paper_2602_24044_amd.model_step import slot_region_bytes
    r = slot_region_bytes([(64, 128), (128, 64)], 2, [8, 16, 32, 8], 32, 3)
    assert r["per_rank_unit"] == 2 * 2 * 384
    assert r["uniform"] == 3 * 32 * 1536                 # A_max slots of the largest rank
    assert r["packed"] == (8 + 16 + 32) * 1536           # the first A_max adapters at their own ranks
