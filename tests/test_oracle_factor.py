"""Pins of the oracle's "4-bit Factor" step (factorized second moment, Sec. 4.3).

What fixes the expected values: a worked example (tests/golden/factor_by_hand.txt); the defining property
of the factorization, that it is exact for a rank-one matrix, which turns the already pinned fp32-state
AdamW into the expected result; the marginals of the reconstructed matrix; closed forms for a constant
gradient and for the zero gradient; exact equivariances (scaling by a power of two, permuting rows); and
the already pinned first-moment path of the 4-bit AdamW step, which does not depend on the second moment.
"""
import numpy as np
import pytest

import oracle
from conftest import golden

HAND = golden("factor_by_hand.txt")


def _f(key):
    return np.array(HAND[key], np.float64)


def test_hand_example_two_steps():
    rows, cols = int(HAND["rows"][0]), int(HAND["cols"][0])
    hp = oracle.Hyper(lr=0.0, beta1=0.5, beta2=float(HAND["beta2"][0]), eps=0.0, weight_decay=0.0)
    g = _f("g").astype(np.float32)
    w = np.zeros(rows * cols, np.float32)
    st = oracle.state_zero_factor(rows, cols)
    assert (st.v_row == 0).all() and (st.v_col == 0).all()
    for t, (kr, kc, kv) in enumerate((("R1", "C1", "v1"), ("R2", "C2", "v2")), 1):
        _, vt = oracle.adamw4_factor_step(w, g, st, hp, t, want_moments=True)
        np.testing.assert_array_equal(st.v_row, _f(kr).astype(np.float32))
        np.testing.assert_array_equal(st.v_col, _f(kc).astype(np.float32))
        np.testing.assert_allclose(vt, _f(kv), rtol=2e-7)


def test_rank_one_squared_gradient_reproduces_adam():
    # |g_ij| = a_i b_j: row and column sums determine g^2 exactly, so the reconstructed second moment IS
    # Adam's, at every step as long as the gradient keeps that structure
    rng = np.random.default_rng(3)
    rows, cols = 37, 200
    a = rng.uniform(0.1, 3.0, rows)
    b = rng.uniform(0.01, 2.0, cols)
    sign = rng.choice([-1.0, 1.0], (rows, cols))
    hp = oracle.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    w0 = rng.standard_normal(rows * cols).astype(np.float32)
    w, st = w0.copy(), oracle.state_zero_factor(rows, cols)
    w32, m32, v32 = w0.copy(), np.zeros(w0.size, np.float32), np.zeros(w0.size, np.float32)
    for t in (1, 2, 3):
        g = (sign * np.outer(a, b) * (1.0 + 0.5 * (t - 1))).astype(np.float32).reshape(-1)
        gsq = g.astype(np.float64) ** 2
        # the fp32 rounding of g breaks exact rank one by parts in 1e-7 only
        _, vt = oracle.adamw4_factor_step(w, g, st, hp, t, want_moments=True)
        oracle.adamw32_step(w32, g, m32, v32, hp, t)
        np.testing.assert_allclose(vt, v32, rtol=2e-6)
        if t == 1:      # from the zero state the first moment is precise on both sides as well
            np.testing.assert_allclose(w, w32, rtol=1e-6, atol=1e-8)
    # a transposed reconstruction (row statistic used for columns) cannot pass the above: a and b differ


def test_marginals_of_the_reconstruction():
    # row sums of v_t give back R_t, column sums give back C_t (sum R = sum C), and R_t, C_t are the moving
    # averages of numpy's row / column sums of g^2
    rng = np.random.default_rng(4)
    rows, cols = 50, 384
    hp = oracle.Hyper(beta2=0.9)
    w = rng.standard_normal(rows * cols).astype(np.float32)
    st = oracle.state_zero_factor(rows, cols)
    R = np.zeros(rows)
    C = np.zeros(cols)
    for t in (1, 2, 3, 4):
        g = (rng.standard_normal((rows, cols)) * rng.lognormal(0, 1, (1, cols))).astype(np.float32)
        sq = g.astype(np.float64) ** 2
        R = float(np.float32(0.9)) * R + (1 - float(np.float32(0.9))) * sq.sum(axis=1)
        C = float(np.float32(0.9)) * C + (1 - float(np.float32(0.9))) * sq.sum(axis=0)
        _, vt = oracle.adamw4_factor_step(w, g.reshape(-1), st, hp, t, want_moments=True)
        np.testing.assert_allclose(st.v_row, R, rtol=1e-6)
        np.testing.assert_allclose(st.v_col, C, rtol=1e-6)
        v = vt.reshape(rows, cols).astype(np.float64)
        np.testing.assert_allclose(v.sum(axis=1), st.v_row, rtol=1e-5)
        np.testing.assert_allclose(v.sum(axis=0), st.v_col, rtol=1e-5)
        assert (v > 0).all()


def test_constant_gradient_closed_form():
    # g = k everywhere: v_hat = k^2 and m_hat = k at step 1, so w1 = w0 - lr (k / (|k| + eps) + wd w0)
    rows, cols, k = 6, 256, -0.25
    hp = oracle.Hyper(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-3, weight_decay=0.05)
    rng = np.random.default_rng(5)
    w0 = rng.standard_normal(rows * cols).astype(np.float32)
    w, st = w0.copy(), oracle.state_zero_factor(rows, cols)
    oracle.adamw4_factor_step(w, np.full(rows * cols, k, np.float32), st, hp, 1)
    want = w0.astype(np.float64) - 1e-2 * (k / (abs(k) + 1e-3) + 0.05 * w0.astype(np.float64))
    np.testing.assert_allclose(w, want, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(st.v_row, (1 - float(np.float32(0.999))) * cols * k * k, rtol=1e-6)
    np.testing.assert_allclose(st.v_col, (1 - float(np.float32(0.999))) * rows * k * k, rtol=1e-6)


def test_zero_gradient_from_zero_state_only_decays():
    rows, cols = 3, 128
    hp = oracle.Hyper(lr=0.5, weight_decay=0.1)
    w0 = np.linspace(-1, 1, rows * cols).astype(np.float32)
    w, st = w0.copy(), oracle.state_zero_factor(rows, cols)
    oracle.adamw4_factor_step(w, np.zeros(rows * cols, np.float32), st, hp, 1)
    np.testing.assert_allclose(w, w0.astype(np.float64) * (1 - 0.5 * 0.1), rtol=1e-7)
    assert (st.v_row == 0).all() and (st.v_col == 0).all() and np.isfinite(w).all()


def test_first_moment_is_the_4bit_adamw_first_moment():
    rng = np.random.default_rng(6)
    rows, cols = 20, 200                       # blocks straddle rows, the last one is short
    hp = oracle.Hyper()
    w0 = rng.standard_normal(rows * cols).astype(np.float32)
    wa, sa = w0.copy(), oracle.state_zero_factor(rows, cols)
    wb, sb = w0.copy(), oracle.state_zero(rows, cols)
    for t in (1, 2, 3):
        g = rng.standard_normal(rows * cols).astype(np.float32)
        ma, _ = oracle.adamw4_factor_step(wa, g, sa, hp, t, want_moments=True)
        mb, _ = oracle.adamw4_step(wb, g, sb, hp, t, want_moments=True)
        np.testing.assert_array_equal(ma, mb)
        np.testing.assert_array_equal(sa.m_codes, sb.m_codes)
        np.testing.assert_array_equal(sa.m_scales, sb.m_scales)


def test_power_of_two_scaling_and_row_permutation():
    rng = np.random.default_rng(7)
    rows, cols = 9, 128                        # one block per row, so a row permutation permutes blocks
    hp = oracle.Hyper(weight_decay=0.0, eps=0.0)
    w0 = rng.standard_normal(rows * cols).astype(np.float32)
    g = rng.standard_normal((rows, cols)).astype(np.float32)
    w1, s1 = w0.copy(), oracle.state_zero_factor(rows, cols)
    _, v1 = oracle.adamw4_factor_step(w1, g.reshape(-1), s1, hp, 1, want_moments=True)
    # scaling g by 2^5 scales every product and sum exactly: R, C and v by 2^10; with eps = 0 the update is unchanged
    w2, s2 = w0.copy(), oracle.state_zero_factor(rows, cols)
    _, v2 = oracle.adamw4_factor_step(w2, (g * 32).reshape(-1), s2, hp, 1, want_moments=True)
    np.testing.assert_array_equal(s2.v_row, s1.v_row * 1024)
    np.testing.assert_array_equal(s2.v_col, s1.v_col * 1024)
    np.testing.assert_allclose(v2, v1 * 1024, rtol=2e-7)
    np.testing.assert_allclose(w2, w1, rtol=1e-6, atol=1e-9)
    # permuting rows permutes R, the parameters and the first-moment blocks; C only changes by summation order
    perm = rng.permutation(rows)
    w3, s3 = w0.reshape(rows, cols)[perm].reshape(-1).copy(), oracle.state_zero_factor(rows, cols)
    oracle.adamw4_factor_step(w3, g[perm].reshape(-1), s3, hp, 1)
    np.testing.assert_array_equal(s3.v_row, s1.v_row[perm])
    np.testing.assert_allclose(s3.v_col, s1.v_col, rtol=1e-6)
    np.testing.assert_allclose(w3, w1.reshape(rows, cols)[perm].reshape(-1), rtol=1e-6, atol=1e-9)
    np.testing.assert_array_equal(s3.m_scales, s1.m_scales[perm])
