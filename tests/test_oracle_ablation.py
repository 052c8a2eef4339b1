"""Pins of the quantization-error study (oracle/quant_error_study.py): its building blocks against the already pinned
oracle and the paper's printed values, the definition of stochastic rounding (App. D.3), and the qualitative claims
of Sec. 4.1 on a synthetic second moment."""
import numpy as np

import oracle
from oracle import quant_error_study as qs


def test_maps():
    de, de0, lin = qs.mapping("de"), qs.mapping("de0"), qs.mapping("linear")
    assert de.size == 16 and de[0] == 0.0 and de0.size == 15 and lin.size == 16
    assert abs(de0[0] - 0.0033) < 5e-5            # Sec. 4.1: "the smallest number representable by DE-0 is 0.0033"
    assert lin[0] == 0.0625 and lin[-1] == 1.0    # Sec. 4.1: smallest representable number of the Linear map
    assert de0[-1] == 1.0 and np.all(np.diff(de0) > 0)


def test_nearest_rounding_is_the_oracles_mapping():
    rng = np.random.default_rng(1)
    n = rng.random(20000).astype(np.float32)
    for name in ("linear", "de"):
        T = qs.mapping(name).astype(np.float32)
        np.testing.assert_array_equal(qs.quantize(n.astype(np.float64), T.astype(np.float64)), oracle.nearest_codes(T, n))


def test_scales_are_the_oracles_normalizations():
    rng = np.random.default_rng(2)
    x = (rng.standard_normal((24, 160)) ** 2).astype(np.float32)
    _, r, c = oracle.quant_v(x)
    np.testing.assert_array_equal(qs.scales(x.astype(np.float64), "rank1"), np.minimum(r[:, None], c[None, :]))
    _, s = oracle.quant_v_block(x.reshape(-1))
    np.testing.assert_array_equal(qs.scales(x.astype(np.float64), "b128").reshape(-1), np.repeat(s, 128)[:x.size])
    assert (qs.scales(x.astype(np.float64), "tensor") == x.max()).all()


def test_stochastic_rounding_definition():
    T = qs.mapping("de0")
    rng = np.random.default_rng(3)
    # an entry of the table, and values outside its range, have a single candidate whatever the random number
    for u in (0.0, 0.5, 0.999999):
        np.testing.assert_array_equal(qs.quantize(T.copy(), T, np.full(T.size, u)), np.arange(T.size))
        assert qs.quantize(np.array([T[0] / 2]), T, np.array([u]))[0] == 0
    # between two entries: the upper one exactly when u < (n - T[q1]) / (T[q2] - T[q1]); the expectation is n
    n = rng.uniform(T[0], T[-1], 2000)
    up = qs.quantize(n, T, np.zeros(n.size))           # u = 0: the upper candidate
    dn = qs.quantize(n, T, np.full(n.size, 1 - 1e-12))  # u -> 1: the lower one
    assert np.all(T[dn] <= n) and np.all(n <= T[up]) and np.all(up - dn <= 1)
    p = (n - T[dn]) / np.where(up > dn, T[up] - T[dn], 1.0)
    np.testing.assert_allclose(p * T[up] + (1 - p) * T[dn], n, rtol=1e-12)
    u = rng.random(n.size)
    np.testing.assert_array_equal(qs.quantize(n, T, u), np.where(u < p, up, dn))
    # Monte Carlo: the mean of many draws approaches n
    x = np.full(200000, 0.3)
    assert abs(T[qs.quantize(x, T, rng.random(x.size))].mean() - 0.3) < 1e-3


def test_zero_point_claims_on_a_synthetic_second_moment():
    rows = {(r["norm"], r["map"], r["rounding"]): r for r in qs.study(qs.synthetic_second_moment(256, 1024))}
    # a map that contains zero sends a large share of the entries to zero; neither a smaller block nor stochastic
    # rounding removes them (Sec. 4.1)
    assert rows[("b2048", "de", "nearest")]["zero_share"] > 0.3
    assert rows[("b2048", "de", "stochastic")]["zero_share"] > 0.3
    assert rows[("b128", "de", "nearest")]["zero_share"] > 0.03
    assert rows[("b128", "de", "stochastic")]["zero_share"] > 0.03
    # ... and their update direction is off by orders of magnitude
    assert rows[("b2048", "de", "nearest")]["median_h_factor"] > 50
    # without zero in the map nothing becomes zero
    for key, r in rows.items():
        if key[1] in ("de0", "linear"):
            assert r["zero_share"] == 0.0
    # the paper's choice, Rank-1 / Linear, has the smallest error of all and keeps h within 2x everywhere
    best = min(rows.values(), key=lambda r: r["rel_err_v"])
    assert (best["norm"], best["map"], best["rounding"]) == ("rank1", "linear", "nearest")
    assert rows[("rank1", "linear", "nearest")]["share_h_off_2x"] == 0.0
    # DE-0 rescues the large-block quantizer of the 8-bit optimizer (B2048/DE -> B2048/DE-0)
    assert rows[("b2048", "de0", "nearest")]["median_h_factor"] < 2 < rows[("b2048", "de", "nearest")]["median_h_factor"]
