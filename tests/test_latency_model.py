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


def test_load_law_table_and_line():
    # Lat_load(S), Sec. 5.2: a table over the measured sizes and the straight line through the points
    r = lm.fit_load([8, 16, 32, 64], [0.1 + 0.09 * s for s in (8, 16, 32, 64)])
    assert r["fixed_ms"] == pytest.approx(0.1) and r["per_rank_ms"] == pytest.approx(0.09)
    assert r["smape_percent"] < 1e-9
    assert r["table_ms"] == {8: pytest.approx(0.82), 16: pytest.approx(1.54), 32: pytest.approx(2.98), 64: pytest.approx(5.86)}
    # repeated sizes are averaged in the table; a size that was not measured is read off the line
    r = lm.fit_load([8, 8, 32, 32], [1.0, 1.2, 3.0, 3.4])
    assert r["table_ms"][8] == pytest.approx(1.1) and r["table_ms"][32] == pytest.approx(3.2)
    assert lm.predict_load(r, 8) == pytest.approx(1.1)
    assert lm.predict_load(r, 16) == pytest.approx(r["fixed_ms"] + 16 * r["per_rank_ms"])
    assert r["per_rank_ms"] == pytest.approx((3.2 - 1.1) / 24)
    with pytest.raises(ValueError):
        lm.fit_load([8, 8], [1.0, 1.1])           # one distinct size only
    with pytest.raises(ValueError):
        lm.fit_load([8, 16], [1.0])


def test_profile_round_trip(tmp_path):
    B, A = _grid()
    rows = [{"B": int(b), "A": int(a), "latency_us": float((0.3 * b + 140.0) * (0.005 * a + 1.0))} for b, a in zip(B, A)]
    with_ad = [r for r in rows if r["A"] > 0]
    col = lambda rs, k: [r[k] for r in rs]
    res = {"points": rows, "fit_all": lm.fit(col(rows, "B"), col(rows, "A"), col(rows, "latency_us")),
           "fit_A_ge_1": lm.fit(col(with_ad, "B"), col(with_ad, "A"), col(with_ad, "latency_us")),
           "fit_additive": lm.fit_additive(col(rows, "B"), col(rows, "A"), col(rows, "latency_us")),
           "load_points": [{"rank": 8, "ms": 0.9}, {"rank": 16, "ms": 1.6}, {"rank": 32, "ms": 3.0}],
           "load_layers": 32, "fit_load": lm.fit_load([8, 16, 32], [0.9, 1.6, 3.0]), "step_ms_all_layers": 7.9}
    path = tmp_path / "law.md"
    lm.write_profile(res, str(path))
    kv = lm.read_profile(str(path))
    assert kv["K4_us_per_token"] == pytest.approx(0.3, rel=1e-4) and kv["K5_us"] == pytest.approx(140.0, rel=1e-4)
    assert kv["K6_per_adapter"] == pytest.approx(0.005, rel=1e-4) and kv["K7"] == 1.0
    assert kv["load_table_ms"] == {8: pytest.approx(0.9), 16: pytest.approx(1.6), 32: pytest.approx(3.0)}
    from paper_2602_24044_amd.placement_model import ServingModel
    m = ServingModel.from_profile(str(path))
    assert m.k4 == pytest.approx(0.3, rel=1e-4) and m.load_ms(16) == pytest.approx(1.6)
    assert m.load_ms(24) == pytest.approx(kv["load_fixed_ms"] + 24 * kv["load_per_rank_ms"])


def test_committed_latency_law_is_readable():
    # what placement_model reads by default: the measurement committed under profiles/
    from paper_2602_24044_amd.placement_model import LATENCY_LAW, ServingModel
    m = ServingModel.from_profile()
    assert m.k4 > 0 and m.k5 > 0 and m.k6 >= 0 and m.k7 == 1.0
    assert m.load_ms_per_rank > 0 and m.load_ms(32) > m.load_ms(8) > 0
    assert lm.read_profile(LATENCY_LAW)["eq1_smape_percent"] < 15.0


@pytest.mark.gpu
def test_sweep_on_the_library_at_reduced_shapes():
    """A 3 x 2 sweep through the library (model dimensions divided by 8): finite, growing with the batch, and Eq. 1
    fits its own points to within 20 % (a timing on a shared machine: the bound is loose on purpose)."""
    rows = lm.sweep(batch_sizes=(64, 512, 1024), adapters_in_batch=(0, 8), rank=16, steps=40, warmup=10, shrink=8)
    assert [(r["B"], r["A"]) for r in rows] == [(64, 0), (64, 8), (512, 0), (512, 8), (1024, 0), (1024, 8)]
    lat = {(r["B"], r["A"]): r["latency_us"] for r in rows}
    assert all(np.isfinite(v) and 1.0 < v < 1e5 for v in lat.values())
    for a in (0, 8):
        assert lat[(1024, a)] > lat[(64, a)]                 # a larger batch is never cheaper
    f = lm.fit([r["B"] for r in rows], [r["A"] for r in rows], [r["latency_us"] for r in rows])
    assert f["K4"] > 0 and f["K5"] > 0
    assert f["max_rel_err"] < 0.20, f
