"""Pins for the projection oracle (CPU only): each check compares it with something that
does not depend on its own code."""
import os

import numpy as np
import pytest
import torch

import oracle
from conftest import GOLDEN, parse_fixture
from paper_2602_24044_amd import workloads as wl


def _bits(a):
    return wl.to_bf16_bits(np.asarray(a, dtype=np.float32))


def _small_workload(seed=7, T=9, d_in=48, d_out=40, ranks=(4, 8, 0, 16), with_base_only=True):
    rng = np.random.default_rng(seed)
    n_ad = len(ranks)
    ids = rng.integers(-1 if with_base_only else 0, n_ad, size=T).astype(np.int32)
    w = wl.custom("small", seed, [(d_in, d_out)], ["p"], n_ad, max(ranks), wl.BUCKET_SORTED, ids,
                  {i: r for i, r in enumerate(ranks)})
    return w


def test_hand_computed_fixture():
    # paper Sec. 2.2 definition, worked by hand in tests/golden/tiny_projection.txt
    fx = parse_fixture(os.path.join(GOLDEN, "tiny_projection.txt"))
    W = _bits(fx["W"])
    x = _bits(fx["x"])
    ids = np.array(fx["ids"][0], dtype=np.int32)
    adapters = {}
    for i in (0, 1):
        r = fx[f"a{i}_rank"][0][0]
        adapters[i] = (r, fx[f"a{i}_scale"][0][0], _bits(fx[f"a{i}_A"]).reshape(r, -1),
                       _bits(fx[f"a{i}_B"]).reshape(-1, r))
    y = oracle.project(x, W, ids, adapters)
    assert np.array_equal(y, np.array(fx["y"], dtype=np.float64))
    ts = np.array([0, 0, 1, 1, 2, 2], dtype=np.int32)
    ns = np.array([0, 1, 0, 1, 0, 1], dtype=np.int32)
    assert np.array_equal(oracle.project_at(x, W, ids, adapters, ts, ns), np.array(fx["y"]).reshape(-1))


def _tiny_fixture():
    fx = parse_fixture(os.path.join(GOLDEN, "tiny_projection.txt"))
    adapters = {}
    for i in (0, 1):
        r = fx[f"a{i}_rank"][0][0]
        adapters[i] = (r, fx[f"a{i}_scale"][0][0], _bits(fx[f"a{i}_A"]).reshape(r, -1),
                       _bits(fx[f"a{i}_B"]).reshape(-1, r))
    return _bits(fx["x"]), _bits(fx["W"]), np.array(fx["ids"][0], dtype=np.int32), adapters


def test_hand_computed_fixture_with_bias():
    # the backbone layer's output includes its bias; worked by hand in tests/golden/tiny_projection_bias.txt
    x, W, ids, adapters = _tiny_fixture()
    fb = parse_fixture(os.path.join(GOLDEN, "tiny_projection_bias.txt"))
    b = _bits(fb["bias"][0])
    y = oracle.project(x, W, ids, adapters, bias=b)
    assert np.array_equal(y, np.array(fb["y"], dtype=np.float64))
    ts = np.array([0, 0, 1, 1, 2, 2], dtype=np.int32)
    ns = np.array([0, 1, 0, 1, 0, 1], dtype=np.int32)
    assert np.array_equal(oracle.project_at(x, W, ids, adapters, ts, ns, bias=b), np.array(fb["y"]).reshape(-1))


def test_bias_properties():
    # T != d_out and a bias that differs in every column: a bias indexed by token, scaled by the adapter, or
    # added only to rows with (or without) an adapter fails one of these
    w = _small_workload(seed=31, T=7, d_in=32, d_out=24, ranks=(8, 0, 16))
    ad = oracle.adapters_of(w, 0)
    b = _bits(np.arange(24, dtype=np.float32) * 0.25 - 2.0)
    bd = wl.bf16_bits_to_f64(b)
    # x = 0: every row is the bias itself
    y0 = oracle.project(np.zeros_like(w.x[0]), w.W[0], w.token_ids, ad, bias=b)
    assert np.array_equal(y0, np.tile(bd, (w.T, 1)))
    # mixed batch: the bias shifts every row by b, whatever its adapter
    y = oracle.project(w.x[0], w.W[0], w.token_ids, ad)
    yb = oracle.project(w.x[0], w.W[0], w.token_ids, ad, bias=b)
    assert len(set(w.token_ids.tolist())) > 1
    assert np.max(np.abs((yb - y) - bd[None, :])) <= 1e-12 * np.max(np.abs(y))
    # backbone only: library matmul plus bias
    ids = np.full(w.T, -1, dtype=np.int32)
    ref = wl.bf16_bits_to_f64(w.x[0]) @ wl.bf16_bits_to_f64(w.W[0]).T + bd[None, :]
    assert np.max(np.abs(oracle.project(w.x[0], w.W[0], ids, ad, bias=b) - ref)) <= 1e-12 * np.max(np.abs(ref))
    # a zero bias is no bias, bitwise
    assert np.array_equal(oracle.project(w.x[0], w.W[0], w.token_ids, ad, bias=np.zeros(24, dtype=np.uint16)), y)
    # sampled evaluation agrees
    ts = np.array([0, 3, 6, 2], dtype=np.int32)
    ns = np.array([23, 0, 11, 5], dtype=np.int32)
    ys = oracle.project_at(w.x[0], w.W[0], w.token_ids, ad, ts, ns, bias=b)
    assert np.max(np.abs(ys - yb[ts, ns])) <= 1e-13 * np.max(np.abs(yb))


def test_backbone_only_equals_library_matmul():
    w = _small_workload(T=17, d_in=96, d_out=72)
    ids = np.full(w.T, -1, dtype=np.int32)
    y = oracle.project(w.x[0], w.W[0], ids, oracle.adapters_of(w, 0))
    ref = torch.matmul(torch.from_numpy(wl.bf16_bits_to_f64(w.x[0])),
                       torch.from_numpy(wl.bf16_bits_to_f64(w.W[0])).T).numpy()
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))


@pytest.mark.parametrize("maker", [
    lambda: _small_workload(seed=3, T=13, d_in=64, d_out=56, ranks=(8, 16, 4, 32)),
    lambda: wl.config1(),
    lambda: wl.config2(shrink=16, n_tokens=24),
    lambda: wl.config4(shrink=16, n_tokens=20, n_adapters=12),
])
def test_merged_weight_identity(maker):
    # y[t,:] = x[t,:] (W + s_i B_i A_i)^T with the merged matrix formed by a library matmul
    w = maker()
    for p, (d_in, d_out) in enumerate(w.proj):
        y = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p))
        Wd = wl.bf16_bits_to_f64(w.W[p])
        xd = wl.bf16_bits_to_f64(w.x[p])
        merged = {-1: Wd}
        for aid, a in w.adapters.items():
            if a.rank > 0:
                merged[aid] = Wd + float(np.float32(a.scale)) * (wl.bf16_bits_to_f64(a.B[p]) @ wl.bf16_bits_to_f64(a.A[p]))
            else:
                merged[aid] = Wd
        ref = np.stack([xd[t] @ merged[int(w.token_ids[t])].T for t in range(w.T)])
        assert np.max(np.abs(y - ref)) <= 1e-10 * np.max(np.abs(ref))


def test_zero_cases_reproduce_base_bitwise():
    w = _small_workload(seed=11, ranks=(8, 8, 8, 8), with_base_only=False)
    ad = oracle.adapters_of(w, 0)
    base = oracle.project(w.x[0], w.W[0], np.full(w.T, -1, dtype=np.int32), ad)
    # B = 0
    adB0 = {i: (r, s, A, np.zeros_like(B)) for i, (r, s, A, B) in ad.items()}
    yB0 = oracle.project(w.x[0], w.W[0], w.token_ids, adB0)
    assert np.array_equal(yB0, base)
    # scale = 0
    ads0 = {i: (r, 0.0, A, B) for i, (r, s, A, B) in ad.items()}
    assert np.array_equal(oracle.project(w.x[0], w.W[0], w.token_ids, ads0), base)
    # rank 0
    adr0 = {i: (0, s, None, None) for i, (r, s, A, B) in ad.items()}
    assert np.array_equal(oracle.project(w.x[0], w.W[0], w.token_ids, adr0), base)
    # and the adapters do matter otherwise
    assert not np.array_equal(oracle.project(w.x[0], w.W[0], w.token_ids, ad), base)


def test_one_hot_rows_read_columns_of_the_merged_matrix():
    # x[t,:] = e_k  =>  y[t,:] = W[:,k] + s (B A)[:,k], every term read straight from the inputs
    rng = np.random.default_rng(5)
    d_in, d_out, r = 12, 10, 2
    Wi = rng.integers(-3, 4, size=(d_out, d_in))
    Ai = rng.integers(-2, 3, size=(r, d_in))
    Bi = rng.integers(-2, 3, size=(d_out, r))
    ks = [0, 5, 11, 7]
    x = np.zeros((len(ks), d_in))
    for t, k in enumerate(ks):
        x[t, k] = 1.0
    ids = np.array([0, 0, -1, 0], dtype=np.int32)
    y = oracle.project(_bits(x), _bits(Wi), ids, {0: (r, 4.0, _bits(Ai), _bits(Bi))})
    for t, k in enumerate(ks):
        expect = Wi[:, k].astype(np.float64)
        if ids[t] == 0:
            expect = expect + 4.0 * sum(Bi[:, j] * Ai[j, k] for j in range(r))
        assert np.array_equal(y[t], expect)


def test_linearity_in_x_and_in_scale():
    rng = np.random.default_rng(9)
    d_in, d_out, r, T = 16, 12, 4, 5
    W = _bits(rng.integers(-2, 3, size=(d_out, d_in)))
    A = _bits(rng.integers(-2, 3, size=(r, d_in)))
    B = _bits(rng.integers(-2, 3, size=(d_out, r)))
    x1 = rng.integers(-2, 3, size=(T, d_in))
    x2 = rng.integers(-2, 3, size=(T, d_in))
    ids = np.array([0, -1, 0, 0, -1], dtype=np.int32)
    f = lambda x, s: oracle.project(_bits(x), W, ids, {0: (r, s, A, B)})
    assert np.array_equal(f(x1 + x2, 2.0), f(x1, 2.0) + f(x2, 2.0))
    base = oracle.project(_bits(x1), W, np.full(T, -1, dtype=np.int32), {0: (r, 2.0, A, B)})
    assert np.array_equal(f(x1, 4.0) - base, 2.0 * (f(x1, 2.0) - base))


def test_sampled_evaluation_matches_full():
    w = _small_workload(seed=21, T=11, d_in=80, d_out=33, ranks=(8, 0, 16))
    ad = oracle.adapters_of(w, 0)
    y = oracle.project(w.x[0], w.W[0], w.token_ids, ad)
    rng = np.random.default_rng(0)
    ts = rng.integers(0, w.T, size=50).astype(np.int32)
    ns = rng.integers(0, 33, size=50).astype(np.int32)
    ys = oracle.project_at(w.x[0], w.W[0], w.token_ids, ad, ts, ns)
    assert np.max(np.abs(ys - y[ts, ns])) <= 1e-13 * np.max(np.abs(y))


def test_unknown_adapter_is_rejected():
    w = _small_workload()
    ids = w.token_ids.copy()
    ids[0] = 99
    with pytest.raises(ValueError):
        oracle.project(w.x[0], w.W[0], ids, oracle.adapters_of(w, 0))


def test_bf16_rounding_of_inputs_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    vals = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.0, 3.0], dtype=np.float32)
    back = wl.bf16_bits_to_f32(wl.to_bf16_bits(vals))
    assert back.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -0.0, 3.0]


# ---- silu(gate) * up ----
def test_silu_against_the_library_routine_and_its_limits():
    import torch
    z = np.concatenate([np.linspace(-60, 60, 2001), [-745.0, -40.0, 0.0, 1e-300, 40.0, 800.0]])
    want = torch.nn.functional.silu(torch.from_numpy(z)).numpy()
    got = oracle.silu(z)
    assert np.allclose(got, want, rtol=1e-14, atol=1e-300)
    assert oracle.silu(np.array([0.0]))[0] == 0.0
    assert oracle.silu(np.array([800.0]))[0] == 800.0                  # sigmoid saturates, no overflow
    assert abs(oracle.silu(np.array([-800.0]))[0]) < 1e-300 and np.isfinite(oracle.silu(np.array([-800.0]))[0])
    # z * sigmoid(z) - (-z) * sigmoid(-z) = z  (sigmoid(z) + sigmoid(-z) = 1)
    zz = np.linspace(-30, 30, 601)
    assert np.allclose(oracle.silu(zz) - oracle.silu(-zz), zz, rtol=0, atol=1e-13)
    # minimum of z * sigmoid(z): about -0.27846 at z = -1.27846
    assert abs(oracle.silu(zz).min() + 0.2784645) < 1e-4


def test_gated_hand_case_and_reductions():
    bits = lambda a: wl.to_bf16_bits(np.asarray(a, dtype=np.float32))
    # one token, x = [1, 2]; gate row [1, -1] -> -1 + adapter 2 * (x . [1, 0]) * 0.5 = 0; up row [0.5, 0.25] -> 1
    x = bits([[1.0, 2.0]])
    Wg, Wu = bits([[1.0, -1.0], [0.0, 1.0]]), bits([[0.5, 0.25], [2.0, 0.0]])
    ids = np.array([0], dtype=np.int32)
    Ag, Bg = bits([[1.0, 0.0]]), bits([[0.5], [0.0]])
    ad_g = {0: (1, 2.0, Ag, Bg)}
    ad_u = {0: (0, 0.0, None, None)}
    h = oracle.gated(x, Wg, Wu, ids, ad_g, ad_u)
    # column 0: gate = -1 + 2 * 1 * 0.5 = 0 -> silu 0 -> h = 0;  column 1: gate = 2, up = 2 -> 2 / (1 + e^-2) * 2
    assert h[0, 0] == 0.0
    assert h[0, 1] == pytest.approx(4.0 / (1.0 + np.exp(-2.0)), rel=1e-15)
    # without adapters and with a huge gate the activation is the identity: h = gate * up
    rng = np.random.default_rng(3)
    x = bits(rng.standard_normal((5, 8)))
    Wg = bits(np.full((4, 8), 0.0))
    Wg_big = bits(np.tile(np.sign(wl.bf16_bits_to_f32(x))[0] * 64.0, (4, 1)))      # gate of token 0 is large and positive
    Wu = bits(rng.standard_normal((4, 8)))
    none = np.full(5, -1, dtype=np.int32)
    h0 = oracle.gated(x, Wg, Wu, none, {}, {})
    assert np.all(h0 == 0.0)                                                       # silu(0) = 0 whatever `up` is
    hb = oracle.gated(x, Wg_big, Wu, none, {}, {})
    g = oracle.project(x, Wg_big, none, {})
    u = oracle.project(x, Wu, none, {})
    assert g[0].min() > 50 and np.allclose(hb[0], g[0] * u[0], rtol=1e-15)
