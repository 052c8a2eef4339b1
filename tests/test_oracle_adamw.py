"""Pins for the oracle's optimizer rule and for the composed 4-bit step (CPU only).

Eq. 1 and Alg. 3 of the paper, AdamW's decoupled decay.  Pins: an fp64 library AdamW
(torch.optim.AdamW on the CPU), the closed form of the first step, and consistency of the
composed step with its parts (decompress -> rule -> compress, in that order).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads

HP = oracle.Hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def _torch_adamw_f64(w0, grads, hp):
    # the step takes its hyper-parameters as fp32 numbers; give the library the same values
    f = lambda x: float(np.float32(x))
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=f(hp.lr), betas=(f(hp.beta1), f(hp.beta2)), eps=f(hp.eps),
                            weight_decay=f(hp.weight_decay))
    outs = []
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        outs.append(p.detach().numpy().copy())
    st = opt.state[p]
    return outs, st["exp_avg"].numpy(), st["exp_avg_sq"].numpy()


def test_identity_quantizer_equals_library_adamw():
    """With compress = decompress = identity, Alg. 3 is plain AdamW."""
    rng = np.random.default_rng(0)
    P, steps = 5000, 25
    w0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    grads = [(rng.standard_normal(P) * 1e-3).astype(np.float32) for _ in range(steps)]
    ref_w, ref_m, ref_v = _torch_adamw_f64(w0, grads, HP)
    w, m, v = w0.copy(), np.zeros(P, np.float32), np.zeros(P, np.float32)
    for t, g in enumerate(grads, 1):
        oracle.adamw32_step(w, g, m, v, HP, t)
        # parameters are stored in fp32 (one rounding per step); moments are fp32 arithmetic
        np.testing.assert_allclose(w, ref_w[t - 1], rtol=3e-6, atol=5e-8)
    np.testing.assert_allclose(m, ref_m, rtol=2e-6, atol=1e-9)
    np.testing.assert_allclose(v, ref_v, rtol=2e-6, atol=1e-15)


@pytest.mark.parametrize("hp", [oracle.Hyper(3e-4, 0.8, 0.95, 1e-6, 0.1),
                                oracle.Hyper(1e-2, 0.0, 0.5, 1e-3, 0.0)])
def test_identity_quantizer_other_hyperparameters(hp):
    """Different beta1/beta2 catch a swapped coefficient (Alg. 3 prints beta1 in the v line)."""
    rng = np.random.default_rng(1)
    P = 1000
    w0 = rng.standard_normal(P).astype(np.float32)
    grads = [rng.standard_normal(P).astype(np.float32) for _ in range(7)]
    ref_w, ref_m, ref_v = _torch_adamw_f64(w0, grads, hp)
    w, m, v = w0.copy(), np.zeros(P, np.float32), np.zeros(P, np.float32)
    for t, g in enumerate(grads, 1):
        oracle.adamw32_step(w, g, m, v, hp, t)
    np.testing.assert_allclose(w, ref_w[-1], rtol=3e-6, atol=3e-7)
    np.testing.assert_allclose(m, ref_m, rtol=3e-6, atol=3e-7)
    np.testing.assert_allclose(v, ref_v, rtol=3e-6, atol=3e-7)


def test_first_step_closed_form():
    """From m0 = v0 = 0: m^ = g and v^ = g^2, so w1 = w0 - lr*( g/(|g|+eps) + wd*w0 )."""
    rng = np.random.default_rng(2)
    P = 4096
    w0 = (rng.standard_normal(P) * 0.02).astype(np.float32)
    g = (rng.standard_normal(P) * 1e-3).astype(np.float32)
    g[:10] = 0.0
    w, m, v = w0.copy(), np.zeros(P, np.float32), np.zeros(P, np.float32)
    oracle.adamw32_step(w, g, m, v, HP, 1)
    g64, w64 = g.astype(np.float64), w0.astype(np.float64)
    want = w64 - HP.lr * (g64 / (np.abs(g64) + HP.eps) + HP.weight_decay * w64)
    np.testing.assert_allclose(w, want, rtol=1e-6, atol=1e-9)
    b1, b2 = float(np.float32(HP.beta1)), float(np.float32(HP.beta2))   # hyper-parameters are fp32
    np.testing.assert_allclose(m, (1 - b1) * g64, rtol=1e-6)
    np.testing.assert_allclose(v, (1 - b2) * g64 ** 2, rtol=1e-6)


def test_zero_state_dequantizes_to_zero():
    st = oracle.state_zero(5, 130)
    assert np.all(oracle.unpack_codes(st.m_codes, 650) == 7) and np.all(st.m_scales == 0)
    assert np.all(st.v_r == 0) and np.all(st.v_c == 0)
    assert np.all(oracle.dequant_m(st.m_codes, st.m_scales, 650) == 0)
    assert np.all(oracle.dequant_v(st.v_codes, st.v_r, st.v_c) == 0)


def test_quantized_first_step_updates_params_like_fp32_adamw():
    """The parameter update uses the precise m_t, v_t (compress is Alg. 3's last line), so the
    first step from the zero state moves the parameters exactly as uncompressed AdamW does."""
    rows, cols = 48, 160
    w0 = workloads.weights(11, 0, rows, cols).reshape(-1)
    g = workloads.grads(11, 0, 1, rows, cols).reshape(-1)
    w4, st = w0.copy(), oracle.state_zero(rows, cols)
    oracle.adamw4_step(w4, g, st, HP, 1)
    w32, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    oracle.adamw32_step(w32, g, m, v, HP, 1)
    np.testing.assert_array_equal(w4, w32)
    ref_w, _, _ = _torch_adamw_f64(w0, [g], HP)
    np.testing.assert_allclose(w4, ref_w[0], rtol=3e-6, atol=1e-9)


def test_composed_step_is_decompress_rule_compress():
    rows, cols = 64, 256
    hp = HP
    w = workloads.weights(5, 0, rows, cols).reshape(-1)
    st = oracle.state_zero(rows, cols)
    for t in range(1, 6):
        g = workloads.grads(5, 0, t, rows, cols, "col_lognormal").reshape(-1)
        w_before, st_before = w.copy(), st.copy()
        mt, vt = oracle.adamw4_step(w, g, st, hp, t, want_moments=True)
        # decompress
        m_prev = oracle.dequant_m(st_before.m_codes, st_before.m_scales, w.size).astype(np.float64)
        v_prev = oracle.dequant_v(st_before.v_codes, st_before.v_r, st_before.v_c).reshape(-1)
        g64 = g.astype(np.float64)
        # Eq. 1 in fp64 on the decompressed states; the oracle's fp32 moments sit within an ulp or two
        b1, b2 = float(np.float32(hp.beta1)), float(np.float32(hp.beta2))   # fp32 hyper-parameters
        ta, tb = b1 * m_prev, (1 - b1) * g64       # the two terms may cancel: bound by their size
        assert np.all(np.abs(mt - (ta + tb)) <= 2.0 ** -23 * (np.abs(ta) + np.abs(tb)) + 1e-40)
        ta, tb = b2 * v_prev.astype(np.float64), (1 - b2) * g64 ** 2
        assert np.all(np.abs(vt - (ta + tb)) <= 2.0 ** -22 * (ta + tb) + 1e-40)
        # parameter update from the precise moments, in fp64, rounded once
        bc1, bc2 = 1 - np.float64(np.float32(hp.beta1)) ** t, 1 - np.float64(np.float32(hp.beta2)) ** t
        w64 = w_before.astype(np.float64)
        lr, eps, wd = (np.float64(np.float32(x)) for x in (hp.lr, hp.eps, hp.weight_decay))
        want = w64 - lr * ((mt / bc1) / (np.sqrt(vt / bc2) + eps) + wd * w64)
        np.testing.assert_allclose(w, want.astype(np.float32), rtol=2e-7, atol=0)
        # compress: the new state is the quantization of exactly those moments
        mc, ms = oracle.quant_m(mt)
        vc, vr, vcmax = oracle.quant_v(vt.reshape(rows, cols))
        np.testing.assert_array_equal(st.m_codes, mc)
        np.testing.assert_array_equal(st.m_scales, ms)
        np.testing.assert_array_equal(st.v_codes, vc)
        np.testing.assert_array_equal(st.v_r, vr)
        np.testing.assert_array_equal(st.v_c, vcmax)


def test_rows_without_gradient_keep_zero_state():
    rows, cols = 40, 128
    w = workloads.weights(9, 0, rows, cols).reshape(-1)
    st = oracle.state_zero(rows, cols)
    for t in range(1, 4):
        g = workloads.grads(9, 0, t, rows, cols).copy()
        g[::4, :] = 0.0
        oracle.adamw4_step(w, g.reshape(-1), st, HP, t)
    assert np.all(st.v_r[::4] == 0) and np.all(st.v_r[1::4] > 0)
    assert np.all(oracle.unpack_codes(st.v_codes, w.size).reshape(rows, cols)[::4] == 0)
    assert np.all(oracle.dequant_v(st.v_codes, st.v_r, st.v_c)[::4] == 0)
    assert np.all(oracle.unpack_codes(st.m_codes, w.size).reshape(rows, cols)[::4] == 7)


def test_quantized_run_tracks_fp32_adamw():
    """Sanity of the whole method (its premise, Sec. 5): after a few steps on smooth gradients
    the 4-bit parameters stay close to uncompressed AdamW's."""
    rows, cols = 64, 256
    w0 = workloads.weights(3, 0, rows, cols).reshape(-1)
    w4, st = w0.copy(), oracle.state_zero(rows, cols)
    w32, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t in range(1, 11):
        g = workloads.grads(3, 0, t, rows, cols).reshape(-1)
        oracle.adamw4_step(w4, g, st, HP, t)
        oracle.adamw32_step(w32, g, m, v, HP, t)
    moved = np.abs(w32 - w0).mean()
    assert np.abs(w4 - w32).mean() < 0.35 * moved
