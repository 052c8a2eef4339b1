"""Pins of the oracle's ablation quantizers (Sec. 4.1, Tab. 1: B2048 / B128 / rank-1 normalization x DE / DE-0 /
Linear map) and of stochastic rounding (App. D.3): the maps against the paper's printed value and a table worked by
hand, the quantizers against the separately pinned ones where they coincide and against numpy brute force elsewhere,
the generator against SplitMix64's published test vector, the rounding rule against its definition, and the
qualitative claims of Sec. 4.1 on a synthetic second moment."""
import numpy as np
import pytest

import oracle
from conftest import golden
from oracle import quant_error_study as qs


def test_maps_against_the_hand_table_and_the_printed_value():
    g = golden("de_unsigned_4bit_by_hand.txt")
    de, de0, lin = oracle.ablation_table("de"), oracle.ablation_table("de0"), oracle.ablation_table("linear")
    np.testing.assert_array_equal(de, np.array([float(x) for x in g["de_unsigned"]], np.float32))
    assert de0.size == int(g["de0_points"][0]) and np.array_equal(de0, de[1:])      # "simply remove zero"
    printed = float(golden("paper_printed_values.txt")["de0_unsigned_4bit_min"][0])
    assert abs(float(de0[0]) - printed) < 5e-5                                       # 0.0033 to two digits
    assert lin[0] == 0.0625 and lin[-1] == 1.0 and np.array_equal(lin, oracle.table_linear())
    np.testing.assert_array_equal(oracle.ablation_table("de", signed=True), oracle.step_table("de"))
    for bad in (("de0", True), ("linear", True)):
        with pytest.raises(ValueError):
            oracle.ablation_table(*bad)


def test_coincides_with_the_pinned_quantizers_of_the_step():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((37, 200)).astype(np.float32) * np.exp(rng.standard_normal((37, 200))).astype(np.float32)
    v = (x * x).astype(np.float32)
    codes, sa, _ = oracle.quant_ablation(x, "b128", "de", signed=True)
    want = oracle.quant_m(x)
    np.testing.assert_array_equal(codes, want[0]); np.testing.assert_array_equal(sa, want[1])
    codes, sa, _ = oracle.quant_ablation(v, "b128", "linear")
    want = oracle.quant_v_block(v)
    np.testing.assert_array_equal(codes, want[0]); np.testing.assert_array_equal(sa, want[1])
    codes, sa, sb = oracle.quant_ablation(v, "rank1", "linear")
    want = oracle.quant_v(v)
    for a, b in zip((codes, sa, sb), want):
        np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(oracle.dequant_ablation(codes, sa, sb, 37, 200, "rank1", "linear"),
                                  oracle.dequant_v(*want))


def _numpy_nearest(n32, T32):
    d = np.abs(n32.astype(np.float64)[:, None] - T32.astype(np.float64)[None, :])
    return np.argmin(d, axis=1)                       # first minimum: ties to the lower index


@pytest.mark.parametrize("norm,map_name,signed", [("b2048", "de", False), ("b2048", "de0", False), ("b2048", "de", True),
                                                  ("b128", "de", False), ("b128", "de0", False), ("rank1", "de0", False),
                                                  ("rank1", "de", False), ("b2048", "linear", False)])
def test_against_numpy_brute_force(norm, map_name, signed):
    rng = np.random.default_rng(2)
    rows, cols = 21, 300                               # 6300 elements: three blocks of 2048 and a ragged fourth
    x = (rng.standard_normal((rows, cols)) * np.exp(2 * rng.standard_normal((rows, cols)))).astype(np.float32)
    if not signed:
        x = (x * x).astype(np.float32)
    x[3, :] = 0.0                                      # a zero row, and below a whole zero block
    x.reshape(-1)[2048:4096] = 0.0
    T = oracle.ablation_table(map_name, signed)
    codes, sa, sb = oracle.quant_ablation(x, norm, map_name, signed)
    flat = x.reshape(-1)
    if norm == "rank1":
        np.testing.assert_array_equal(sa, x.max(axis=1)); np.testing.assert_array_equal(sb, x.max(axis=0))
        scale = np.minimum(sa[:, None], sb[None, :]).reshape(-1)
    else:
        B = oracle.NORM_BLOCK[norm]
        nb = -(-flat.size // B)
        pad = np.zeros(nb * B, np.float32); pad[:flat.size] = np.abs(flat)
        np.testing.assert_array_equal(sa, pad.reshape(nb, B).max(axis=1))
        scale = np.repeat(sa, B)[:flat.size]
    with np.errstate(invalid="ignore", divide="ignore"):
        n = np.where(scale > 0, flat / scale, np.float32(0)).astype(np.float32)
    assert np.all(np.abs(n) <= 1)
    got = oracle.unpack_codes(codes, flat.size)
    np.testing.assert_array_equal(got, _numpy_nearest(n, T))
    out = oracle.dequant_ablation(codes, sa, sb, rows, cols, norm, map_name, signed).reshape(-1)
    np.testing.assert_array_equal(out, T[got] * scale)
    if map_name == "de0":
        assert got.max() <= 14 and np.all(out[scale > 0] > 0)      # the zero point is gone
    if map_name == "de" and not signed:
        assert (out[scale > 0] == 0).any()                          # ... and here it is not


def test_invalid_combinations_are_refused():
    x = np.ones((4, 128), np.float32)
    for norm, map_name, signed in (("rank1", "de", True), ("b128", "de0", True), ("b2048", "linear", True)):
        with pytest.raises(ValueError):
            oracle.quant_ablation(x, norm, map_name, signed)


def test_generator_is_splitmix64():
    # published test vector of SplitMix64 for the state 1234567 (first five outputs)
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431, 16408922859458223821]
    assert [oracle.splitmix64_at(1234567, i) for i in range(5)] == want
    for i in range(5):
        assert oracle.uniform_at(1234567, i) == (want[i] >> 40) / 2.0 ** 24
    u = np.array([oracle.uniform_at(7, i) for i in range(20000)])
    assert 0 <= u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 0.01 and abs((u < 0.25).mean() - 0.25) < 0.01


def test_stochastic_rounding_rule():
    T = oracle.ablation_table("de0")
    # an entry of the table, and values outside its range, have a single candidate whatever the random number
    for u in (0.0, 0.5, 0.999999):
        assert [oracle.round_stochastic(T, float(t), u) for t in T] == list(range(T.size))
        assert oracle.round_stochastic(T, float(T[0]) / 2, u) == 0
        assert oracle.round_stochastic(T, 1.5, u) == T.size - 1
    rng = np.random.default_rng(3)
    for n in rng.uniform(T[0], T[-1], 300).astype(np.float32):
        up, dn = oracle.round_stochastic(T, float(n), 0.0), oracle.round_stochastic(T, float(n), 0.99999994)
        assert up - dn == 1 and T[dn] < n < T[up]                   # u = 0: upper candidate, u -> 1: lower one
        p = (float(n) - float(T[dn])) / (float(T[up]) - float(T[dn]))
        for u in (0.9 * p, 1.1 * p):
            if 0 < u < 1 and abs(u - p) > 1e-6:
                assert oracle.round_stochastic(T, float(n), u) == (up if u < p else dn)
        assert abs(p * T[up] + (1 - p) * T[dn] - n) < 1e-6          # the expectation of the rounded value is n


def test_stochastic_quantizer_composition_and_statistics():
    rng = np.random.default_rng(4)
    v = (rng.standard_normal((16, 384)) ** 2).astype(np.float32)
    T = oracle.ablation_table("de")
    codes, sa, _ = oracle.quant_ablation(v, "b128", "de", stochastic=True, seed=99)
    got = oracle.unpack_codes(codes, v.size)
    n = (v.reshape(-1) / np.repeat(sa, 128)).astype(np.float32)
    want = [oracle.round_stochastic(T, float(n[e]), oracle.uniform_at(99, e)) for e in range(v.size)]
    np.testing.assert_array_equal(got, want)                        # element e draws number e of the stream
    near = oracle.unpack_codes(oracle.quant_ablation(v, "b128", "de")[0], v.size)
    assert np.all(np.abs(got.astype(int) - near.astype(int)) <= 1) and (got != near).any()
    again = oracle.unpack_codes(oracle.quant_ablation(v, "b128", "de", stochastic=True, seed=99)[0], v.size)
    other = oracle.unpack_codes(oracle.quant_ablation(v, "b128", "de", stochastic=True, seed=100)[0], v.size)
    assert np.array_equal(got, again) and not np.array_equal(got, other)
    # Monte Carlo: many elements with the same normalized value 0.3 (each block holds one element equal to 1)
    x = np.full((2000, 128), 0.3, np.float32); x[:, 0] = 1.0
    c = oracle.unpack_codes(oracle.quant_ablation(x, "b128", "de0", stochastic=True, seed=5)[0], x.size).reshape(2000, 128)[:, 1:]
    T0 = oracle.ablation_table("de0")
    assert abs(float(T0[c].mean()) - 0.3) < 1e-3
    lo, hi = np.searchsorted(T0, 0.3) - 1, np.searchsorted(T0, 0.3)
    assert set(np.unique(c)) == {lo, hi}
    assert abs((c == hi).mean() - (0.3 - T0[lo]) / (T0[hi] - T0[lo])) < 5e-3


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
