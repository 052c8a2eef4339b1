"""Pins of the oracle's rank-1 normalization for tensors with more than two dimensions (App. F Alg. 4).

What fixes the expected values: a worked example (tests/golden/rank1_nd_by_hand.txt); numpy's axis maxima and
broadcasting for the statistics and the scale, with the already pinned closed form of the Linear map; the
already pinned 2-dimensional quantizer and step, which the general form must reproduce for p = 2 and for a
tensor with an extra dimension of size 1; invariants and the equivariance under a permutation of the axes.
"""
import itertools

import numpy as np
import pytest

import oracle
from conftest import golden

HAND = golden("rank1_nd_by_hand.txt")


def test_hand_example():
    shape = tuple(int(d) for d in HAND["shape"])
    x = np.array(HAND["x"], np.float64).astype(np.float32).reshape(shape)
    codes, stats = oracle.quant_v_nd(x)
    np.testing.assert_array_equal(stats, np.array(HAND["stats"], np.float32))
    np.testing.assert_array_equal(oracle.unpack_codes(codes, x.size), np.array(HAND["codes"], np.uint8))
    np.testing.assert_array_equal(oracle.dequant_v_nd(codes, stats, shape).reshape(-1),
                                  np.array(HAND["dequant"], np.float64).astype(np.float32))


def _numpy_scale(x):
    """statistics and element scales with numpy: maxima over all other axes, broadcast minimum"""
    p = x.ndim
    mus = [x.max(axis=tuple(a for a in range(p) if a != r)) for r in range(p)]
    M = None
    for r, mu in enumerate(mus):
        shape = [1] * p
        shape[r] = -1
        b = np.broadcast_to(mu.reshape(shape), x.shape)
        M = b if M is None else np.minimum(M, b)
    return mus, M


@pytest.mark.parametrize("shape", [(5, 7), (4, 3, 6), (3, 2, 5, 4), (2, 3, 1, 4, 3), (64, 3, 3, 3)])
def test_statistics_scales_and_codes_against_numpy(shape):
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(shape) * rng.lognormal(0, 1.5, (shape[0],) + (1,) * (len(shape) - 1))).astype(np.float32) ** 2
    x[0] = 0.0                                   # an index that never saw a value: statistic 0, scale 0, code 0
    codes, stats = oracle.quant_v_nd(x)
    mus, M = _numpy_scale(x)
    np.testing.assert_array_equal(stats, np.concatenate(mus))
    with np.errstate(divide="ignore", invalid="ignore"):
        n = np.where(M == 0, np.float32(0), x / M).astype(np.float32)
    want = np.clip(np.ceil(16.0 * n.astype(np.float64) - 1.5), 0, 15).astype(np.uint8)
    np.testing.assert_array_equal(oracle.unpack_codes(codes, x.size), want.reshape(-1))
    d = oracle.dequant_v_nd(codes, stats, shape)
    np.testing.assert_array_equal(d, ((want.astype(np.float32) + 1) / 16 * M).astype(np.float32))
    # invariants: every statistic survives the round trip; the zero point is absent where the scale is not 0
    mus_d, _ = _numpy_scale(d)
    np.testing.assert_array_equal(np.concatenate(mus_d), stats)
    assert (d[M > 0] > 0).all() and (d[M == 0] == 0).all()
    assert (np.abs(d - x) <= M / 16 + 1e-12).all()


def test_two_dimensions_is_the_matrix_form():
    rng = np.random.default_rng(12)
    x = (rng.standard_normal((37, 50)).astype(np.float32)) ** 2
    codes, stats = oracle.quant_v_nd(x)
    codes2, r, c = oracle.quant_v(x)
    np.testing.assert_array_equal(codes, codes2)
    np.testing.assert_array_equal(stats, np.concatenate([r, c]))


def test_axis_permutation_permutes_everything():
    rng = np.random.default_rng(13)
    x = (rng.standard_normal((4, 5, 6)).astype(np.float32)) ** 2
    codes, stats = oracle.quant_v_nd(x)
    q = oracle.unpack_codes(codes, x.size).reshape(x.shape)
    parts = np.split(stats, np.cumsum(x.shape)[:-1])
    for perm in itertools.permutations(range(3)):
        xp = np.ascontiguousarray(x.transpose(perm))
        cp, sp = oracle.quant_v_nd(xp)
        np.testing.assert_array_equal(oracle.unpack_codes(cp, x.size).reshape(xp.shape), q.transpose(perm))
        np.testing.assert_array_equal(sp, np.concatenate([parts[a] for a in perm]))


def test_step_with_two_dimensions_and_with_a_unit_dimension_is_the_matrix_step():
    rng = np.random.default_rng(14)
    rows, cols = 20, 200
    hp = oracle.Hyper()
    w0 = rng.standard_normal(rows * cols).astype(np.float32)
    wa, sa = w0.copy(), oracle.state_zero(rows, cols)
    wb, sb = w0.copy(), oracle.state_zero_nd((rows, cols))
    wc, sc = w0.copy(), oracle.state_zero_nd((rows, 1, cols))
    assert (sb.v_stats == 0).all()
    for t in (1, 2, 3):
        g = (rng.standard_normal((rows, cols)) * rng.lognormal(0, 1, (1, cols))).astype(np.float32).reshape(-1)
        oracle.adamw4_step(wa, g, sa, hp, t)
        oracle.adamw4_nd_step(wb, g, sb, hp, t)
        oracle.adamw4_nd_step(wc, g, sc, hp, t)
        for w, s in ((wb, sb), (wc, sc)):
            np.testing.assert_array_equal(w, wa)
            np.testing.assert_array_equal(s.m_codes, sa.m_codes)
            np.testing.assert_array_equal(s.v_codes, sa.v_codes)
        np.testing.assert_array_equal(sb.v_stats, np.concatenate([sa.v_r, sa.v_c]))
        # a dimension of size 1 holds the global maximum, which never is the minimum
        np.testing.assert_array_equal(sc.v_stats, np.concatenate([sa.v_r, [max(sa.v_r.max(), 0)], sa.v_c]).astype(np.float32))


def test_step_is_decompress_rule_compress_in_four_dimensions():
    # assembled from the separately pinned pieces: dequantizers, the fp32-state AdamW rule, quantizers
    rng = np.random.default_rng(15)
    shape = (6, 4, 3, 3)
    P = int(np.prod(shape))
    hp = oracle.Hyper(lr=2e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)
    w, st = rng.standard_normal(P).astype(np.float32), oracle.state_zero_nd(shape)
    w2 = w.copy()
    st2 = st.copy()
    for t in (1, 2, 3):
        g = rng.standard_normal(P).astype(np.float32)
        oracle.adamw4_nd_step(w, g, st, hp, t)
        m = oracle.dequant_m(st2.m_codes, st2.m_scales, P)
        v = oracle.dequant_v_nd(st2.v_codes, st2.v_stats, shape).reshape(-1)
        oracle.adamw32_step(w2, g, m, v, hp, t)
        st2.m_codes, st2.m_scales = oracle.quant_m(m)
        st2.v_codes, st2.v_stats = oracle.quant_v_nd(v.reshape(shape))
        np.testing.assert_array_equal(w, w2)
        np.testing.assert_array_equal(st.m_codes, st2.m_codes)
        np.testing.assert_array_equal(st.v_codes, st2.v_codes)
        np.testing.assert_array_equal(st.v_stats, st2.v_stats)
