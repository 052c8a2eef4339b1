"""Pins for the oracle's two quantizers (CPU only): B128 + signed DE for the first moment
(Sec. 2.2, Sec. 3, App. D.1/D.2) and rank-1 + Linear for the second moment (Sec. 4.1, 4.2).

Checks are hand-worked examples, invariants that follow from the definitions, and independent
numpy formulations of the same definitions (block reshape + reduce, closed-form rounding).
"""
import numpy as np
import pytest

import oracle
from conftest import golden

HAND = golden("rank1_by_hand.txt")


def _arr(key, dtype=np.float32):
    return np.array(HAND[key], np.float64).astype(dtype)


# ---- first moment -----------------------------------------------------------------------------------

def test_m_hand_example_and_nibble_layout():
    x = _arr("m_x")
    codes, scales = oracle.quant_m(x)
    assert scales.tolist() == [1.0]
    np.testing.assert_array_equal(oracle.unpack_codes(codes, x.size), _arr("m_codes", np.uint8))
    # element 2k in the low nibble, 2k+1 in the high nibble; the unused last nibble is 0
    assert codes.tolist() == [15 | (0 << 4), 12 | (8 << 4), 7]
    np.testing.assert_array_equal(oracle.dequant_m(codes, scales, x.size), _arr("m_dequant"))


def test_m_scales_are_blockwise_absmax_of_flattened_tensor():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((37, 200)).astype(np.float32)      # 7400 = 57 blocks + 104 left over
    codes, scales = oracle.quant_m(x)
    flat = np.abs(x.reshape(-1))
    pad = np.zeros(oracle.n_blocks(x.size) * 128, np.float32)
    pad[:flat.size] = flat
    np.testing.assert_array_equal(scales, pad.reshape(-1, 128).max(axis=1))
    assert codes.size == x.size // 2


def test_m_codes_follow_definition():
    """q = argmin_i |x/s - T(i)| with s the block's absmax, via numpy."""
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(128 * 9 + 50) * np.exp(rng.standard_normal(128 * 9 + 50))).astype(np.float32)
    codes, scales = oracle.quant_m(x)
    T = oracle.table_de(4, True).astype(np.float64)
    s = np.repeat(scales, 128)[:x.size]
    n = (x / s).astype(np.float32)                             # fp32 division, as the oracle
    want = np.argmin(np.abs(n.astype(np.float64)[:, None] - T[None, :]), axis=1)
    np.testing.assert_array_equal(oracle.unpack_codes(codes, x.size), want)


def test_m_invariants():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(128 * 64).astype(np.float32) * np.float32(1e-3)
    x[5 * 128:6 * 128] = 0.0                                    # an all-zero block
    codes, scales = oracle.quant_m(x)
    deq = oracle.dequant_m(codes, scales, x.size)
    s = np.repeat(scales, 128)
    # signed unit interval: every reconstruction lies within [-0.8875 s, s]
    assert np.all(deq <= s) and np.all(deq >= np.float32(-0.8875) * s)
    # largest gap of the table is 0.2125 <-> 0.4375, and -1 maps to -0.8875: error <= 0.1125 s
    assert np.all(np.abs(deq.astype(np.float64) - x) <= 0.1125 * s.astype(np.float64) * (1 + 1e-6))
    # a block whose absmax element is positive reproduces it exactly (n = 1 -> T = 1)
    xb, db = x.reshape(-1, 128), deq.reshape(-1, 128)
    imax = np.abs(xb).argmax(axis=1)
    pos = xb[np.arange(64), imax] > 0
    assert pos.any() and (~pos).any()
    np.testing.assert_array_equal(db[pos, imax[pos]], xb[pos, imax[pos]])
    # ... and a negative one is shrunk to -0.8875 s because -1 is not in the table
    neg = ~pos & (scales > 0)
    np.testing.assert_array_equal(db[neg, imax[neg]], np.float32(-0.8875) * scales[neg])
    # zero block: scale 0, every code is the rank of 0.0, reconstruction is exactly 0
    assert scales[5] == 0 and np.all(oracle.unpack_codes(codes, x.size)[5 * 128:6 * 128] == 7)
    assert np.all(deq[5 * 128:6 * 128] == 0)
    # quantizing the reconstruction changes nothing when the block maximum is reproduced
    # exactly, i.e. for blocks whose largest element is positive
    c2, s2 = oracle.quant_m(deq)
    np.testing.assert_array_equal(s2[pos], scales[pos])
    np.testing.assert_array_equal(oracle.unpack_codes(c2, x.size).reshape(-1, 128)[pos],
                                  oracle.unpack_codes(codes, x.size).reshape(-1, 128)[pos])


# ---- second moment ----------------------------------------------------------------------------------

def test_v_hand_example():
    x = _arr("x").reshape(2, 2)
    codes, r, c = oracle.quant_v(x)
    np.testing.assert_array_equal(r, _arr("r"))
    np.testing.assert_array_equal(c, _arr("c"))
    np.testing.assert_array_equal(oracle.unpack_codes(codes, 4), _arr("codes", np.uint8))
    np.testing.assert_array_equal(oracle.dequant_v(codes, r, c).reshape(-1), _arr("dequant"))


def _lognormal_v(rng, rows, cols):
    row = np.exp(2.0 * rng.standard_normal(rows))[:, None]
    col = np.exp(2.0 * rng.standard_normal(cols))[None, :]
    return (rng.standard_normal((rows, cols)) ** 2 * row * col * 1e-8).astype(np.float32)


def test_v_statistics_and_axes():
    rng = np.random.default_rng(3)
    x = _lognormal_v(rng, 33, 70)                               # deliberately not square
    codes, r, c = oracle.quant_v(x)
    np.testing.assert_array_equal(r, x.max(axis=1))            # one per row, over dimension 1
    np.testing.assert_array_equal(c, x.max(axis=0))            # one per column, over dimension 0
    assert r.size == 33 and c.size == 70


def test_v_codes_follow_closed_form():
    """Nearest point of the even grid (i+1)/16 with ties down = ceil(16 n - 1.5) clamped."""
    rng = np.random.default_rng(4)
    x = _lognormal_v(rng, 50, 64)
    x[7, :] = 0.0                                               # a row that never saw a gradient
    x[:, 11] = 0.0
    codes, r, c = oracle.quant_v(x)
    sc = np.minimum(r[:, None], c[None, :])
    with np.errstate(invalid="ignore", divide="ignore"):
        n = np.where(sc > 0, x / sc, np.float32(0)).astype(np.float32)
    want = np.clip(np.ceil(16.0 * n.astype(np.float64) - 1.5), 0, 15).astype(np.uint8)
    np.testing.assert_array_equal(oracle.unpack_codes(codes, x.size).reshape(50, 64), want)
    assert n.max() <= 1.0 and n.min() >= 0.0


def test_v_invariants_zero_point_and_idempotence():
    rng = np.random.default_rng(5)
    x = _lognormal_v(rng, 96, 160)
    x[3, :] = 0.0
    codes, r, c = oracle.quant_v(x)
    deq = oracle.dequant_v(codes, r, c)
    sc = np.minimum(r[:, None], c[None, :]).astype(np.float64)
    # Sec. 4.1: zero is not representable -> wherever the scale is positive the reconstruction
    # is at least scale/16, however small the entry was
    assert np.all(deq[sc > 0] >= np.float32(0.0625) * sc[sc > 0].astype(np.float32))
    assert np.all(deq[sc == 0] == 0) and (sc == 0).sum() == 160
    # the row/column maximum has n = 1 and is reproduced exactly, so the statistics survive
    np.testing.assert_array_equal(deq.max(axis=1), r)
    np.testing.assert_array_equal(deq.max(axis=0), c)
    # error at most half a grid step above scale/16, and below scale/16 the entry moves up to it
    err = np.abs(deq.astype(np.float64) - x)
    assert np.all(err <= sc / 16 + 1e-30)
    big = x >= sc / 16
    assert np.all(err[big] <= sc[big] / 32 * (1 + 1e-6))
    # quantize o dequantize o quantize == quantize
    c2, r2, cc2 = oracle.quant_v(deq)
    np.testing.assert_array_equal(c2, codes)
    np.testing.assert_array_equal(r2, r)
    np.testing.assert_array_equal(cc2, c)


def test_v_rank1_beats_single_axis_scales():
    """Sec. 4.2: min(r_i, c_j) is a tighter bound than either statistic alone."""
    rng = np.random.default_rng(6)
    x = _lognormal_v(rng, 64, 64)
    _, r, c = oracle.quant_v(x)
    sc = np.minimum(r[:, None], c[None, :])
    assert np.all(x <= sc) and np.all(sc <= r[:, None]) and np.all(sc <= c[None, :])


def test_state_bytes_match_paper_ratio():
    """Sec. 5 (memory): 4-bit states are half of 8-bit states, i.e. about 8x below fp32 states."""
    rows = cols = 4096
    P = rows * cols
    st_bytes = 2 * oracle.codes_bytes(P) + 4 * oracle.n_blocks(P) + 4 * (rows + cols)
    assert abs(st_bytes / P - (1 + 4 / 128 + 8 / 4096)) < 1e-9
    assert 7.5 < 8.0 * P / st_bytes < 8.0
