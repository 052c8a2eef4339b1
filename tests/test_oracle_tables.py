"""Pins for the oracle's quantization mappings and nearest-entry search (CPU only).

Each check goes back to something the paper prints or to a property that follows from its text
(Sec. 2.2, Sec. 4.1, App. D.2), not to the oracle's own code.
"""
import numpy as np
import pytest

import oracle
from conftest import golden

PRINTED = golden("paper_printed_values.txt")
BY_HAND = golden("de_signed_4bit_by_hand.txt")


def test_linear_map_matches_paper():
    T = oracle.table_linear(4)
    assert T.size == int(PRINTED["n_points"][0])
    # App. D.2 gives it as linspace(0, 1, 2^b + 1) without the first point
    np.testing.assert_array_equal(T, np.linspace(0, 1, 17)[1:].astype(np.float32))
    assert T[0] == np.float32(PRINTED["linear_4bit_min"][0])      # Sec. 4.1: 0.0625
    assert 0.0 not in T and T[-1] == 1.0                          # zero point excluded
    assert np.all(np.diff(T) == np.float32(1 / 16))               # evenly spaced
    np.testing.assert_array_equal(oracle.step_table("linear"), T)


def test_linear_map_other_bitwidths():
    for b in (2, 3, 8):
        np.testing.assert_array_equal(oracle.table_linear(b),
                                      np.linspace(0, 1, 2 ** b + 1)[1:].astype(np.float32))


def test_de_unsigned_reproduces_printed_minimum():
    T = oracle.table_de(4, signed=False)
    nz = T[T > 0]
    # Sec. 4.1 prints 0.0033 for the smallest non-zero point of the 4-bit DE map
    assert f"{nz.min():.4f}" in ("0.0033", "0.0032")   # 0.00325 printed to 2 significant digits
    assert abs(nz.min() - float(PRINTED["de0_unsigned_4bit_min"][0])) < 1e-4
    assert T.size == 16 and T[0] == 0.0 and T[-1] == 1.0
    assert np.all(np.diff(T) > 0)
    np.testing.assert_allclose(T, np.array(BY_HAND["table_unsigned"], np.float64), rtol=1e-7)


def test_de_signed_structure():
    T = oracle.table_de(4, signed=True)
    assert T.size == 16
    assert np.all(np.diff(T) > 0)                      # Sec. 2.2: T is increasing
    for v in PRINTED["de_signed_has"]:
        assert np.float32(v) in T
    assert np.float32(PRINTED["de_signed_lacks"][0]) not in T
    assert T[7] == 0.0 and T[15] == 1.0                # rank of 0 and of +1
    # apart from +1 the table is symmetric about zero
    np.testing.assert_array_equal(T[:7], -T[8:15][::-1])
    np.testing.assert_array_equal(oracle.step_table("de"), T)


def test_de_signed_decades_and_even_fractions():
    """T(i) = 10^-E * fraction with the fraction spread evenly over (0.1, 1): entries of one E
    sit strictly inside one decade, are equally spaced, and are centred on the decade's
    arithmetic middle 0.55 * 10^-E (bin midpoints of an even partition)."""
    T = oracle.table_de_f64(4, signed=True)
    pos = T[(T > 0) & (T < 1)]
    for E, count in ((0, 4), (1, 2), (2, 1)):
        lo, hi = 0.1 * 10.0 ** -E, 1.0 * 10.0 ** -E
        dec = pos[(pos > lo) & (pos < hi)]
        assert dec.size == count                       # F = 2, 1, 0 fraction bits
        assert abs(dec.mean() - 0.55 * 10.0 ** -E) < 1e-12
        if count > 1:
            assert np.allclose(np.diff(dec), 0.9 * 10.0 ** -E / count, rtol=1e-12)
    assert pos.size == 7


def test_de_signed_equals_hand_derivation():
    T = oracle.table_de(4, signed=True)
    np.testing.assert_array_equal(T, np.array(BY_HAND["table"], np.float64).astype(np.float32))


def test_de_8bit_special_patterns():
    """App. D.2 states the special patterns for 8 bits; the construction is the same at any width."""
    Tu = oracle.table_de(8, signed=False)
    Ts = oracle.table_de(8, signed=True)
    assert Tu.size == 256 and Ts.size == 256
    assert Tu[0] == 0.0 and Tu[-1] == 1.0 and np.all(np.diff(Tu) > 0)
    assert 0.0 in Ts and Ts[-1] == 1.0 and -1.0 not in Ts and np.all(np.diff(Ts) > 0)
    # largest regular entry: E = 0, all fraction bits set -> last bin midpoint below 1
    assert Ts[-2] == np.float32(1.0 - 0.45 / 64)
    assert Tu[-2] == np.float32(1.0 - 0.45 / 128)


# ---- nearest-entry search -------------------------------------------------------------------------

def _argmin_def(T, n):
    d = np.abs(n.astype(np.float64)[:, None] - T.astype(np.float64)[None, :])
    return np.argmin(d, axis=1).astype(np.uint8)       # numpy's argmin returns the first minimum


@pytest.mark.parametrize("which", ["de", "linear"])
def test_nearest_is_identity_on_table_values(which):
    T = oracle.step_table(which)
    np.testing.assert_array_equal(oracle.nearest_codes(T, T), np.arange(16, dtype=np.uint8))


@pytest.mark.parametrize("which", ["de", "linear"])
def test_nearest_against_definition(which):
    T = oracle.step_table(which)
    rng = np.random.default_rng(7)
    lo = -1.0 if which == "de" else 0.0
    n = rng.uniform(lo, 1.0, 200000).astype(np.float32)
    # add points at and next to every midpoint, where a wrong comparison or tie rule shows
    mids = ((T[:-1].astype(np.float64) + T[1:].astype(np.float64)) / 2).astype(np.float32)
    near = np.concatenate([mids, np.nextafter(mids, np.float32(2)), np.nextafter(mids, np.float32(-2)),
                           np.array([lo, 1.0, 0.0, -0.0, 1e-30, -1e-30, 1.5, -1.5], np.float32)])
    n = np.concatenate([n, near]).astype(np.float32)
    np.testing.assert_array_equal(oracle.nearest_codes(T, n), _argmin_def(T, n))


def test_nearest_tie_goes_to_lower_index():
    T = oracle.step_table("linear")
    # 0.09375 is exactly half-way between 0.0625 (code 0) and 0.125 (code 1), and a float
    assert oracle.nearest_codes(T, np.array([0.09375], np.float32))[0] == 0
    assert oracle.nearest_codes(T, np.array([0.96875], np.float32))[0] == 14


def test_linear_nearest_has_closed_form():
    """On an even grid the nearest point with ties down is ceil(16 n - 1.5), clamped."""
    T = oracle.step_table("linear")
    rng = np.random.default_rng(3)
    n = np.concatenate([rng.uniform(0, 1, 100000), np.arange(0, 33) / 32.0]).astype(np.float32)
    want = np.clip(np.ceil(16.0 * n.astype(np.float64) - 1.5), 0, 15).astype(np.uint8)
    np.testing.assert_array_equal(oracle.nearest_codes(T, n), want)
