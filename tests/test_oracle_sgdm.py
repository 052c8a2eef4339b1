"""Pins of the oracle's SGD with momentum and 4-bit momentum (App. E Alg. 2).

What fixes the expected values: torch.optim.SGD in fp64 (momentum, no dampening, no decay: the same rule) for the
rule with an uncompressed buffer; the geometric-series closed form for a constant gradient; a short example
worked by hand; and the composition decompress -> rule -> compress from the separately pinned first-moment
quantizer.
"""
import numpy as np
import torch

import oracle


def test_rule_against_fp64_library_sgd():
    rng = np.random.default_rng(21)
    P, lr, beta = 1000, 0.05, 0.9
    w0 = rng.standard_normal(P).astype(np.float32)
    w, m = w0.copy(), np.zeros(P, np.float32)
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=lr, momentum=float(np.float32(beta)))
    for t in range(6):
        g = rng.standard_normal(P).astype(np.float32)
        oracle.sgdm32_step(w, g, m, lr, beta)
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
        # the momentum is kept in fp32 (one rounding per step, 6e-8 relative to its largest recent term)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=2e-6, atol=1e-6)
        np.testing.assert_allclose(m, opt.state[p]["momentum_buffer"].numpy(), rtol=1e-6, atol=2e-6)


def test_constant_gradient_closed_form():
    # m_t = g (1 - beta^t) / (1 - beta);  theta_t = theta_0 - lr g sum_{s<=t} (1 - beta^s) / (1 - beta)
    P, lr, beta, gval = 64, 0.1, 0.5, 0.25            # everything exactly representable
    w, m = np.ones(P, np.float32), np.zeros(P, np.float32)
    g = np.full(P, gval, np.float32)
    acc = 0.0
    for t in range(1, 6):
        oracle.sgdm32_step(w, g, m, lr, beta)
        mt = gval * (1 - beta ** t) / (1 - beta)
        acc += mt
        np.testing.assert_array_equal(m, np.float32(mt))
        np.testing.assert_allclose(w, 1.0 - lr * acc, rtol=1e-7)


def test_hand_example_with_compressed_momentum():
    # one block, momentum 0.5, lr 1.  Step 1 from the zero state: m_1 = g = (1, -0.4375, 0.2, 0, ...): scale 1,
    # normalized values 1 -> code 15 (+1), -0.4375 is a table entry -> its code, 0.2 lies between 0.0775 and
    # 0.2125 and nearer to 0.2125, 0 -> code 7.  theta_1 = theta_0 - m_1 uses the precise m_1.
    # Step 2 with g = 0: m_2 = 0.5 * dequantized m_1 = (0.5, -0.21875, 0.10625, 0, ...), theta_2 = theta_1 - m_2.
    T = oracle.step_table("de")
    P = 128
    g = np.zeros(P, np.float32)
    g[:3] = [1.0, -0.4375, 0.2]
    w, st = np.zeros(P, np.float32), oracle.state_zero_sgdm(P)
    oracle.sgdm4_step(w, g, st, 1.0, 0.5)
    q = oracle.unpack_codes(st.m_codes, P)
    assert st.m_scales[0] == 1.0
    assert q[0] == 15 and T[q[1]] == np.float32(-0.4375) and T[q[2]] == np.float32(0.2125) and (q[3:] == 7).all()
    np.testing.assert_array_equal(w[:4], np.array([-1.0, 0.4375, -0.2, 0.0], np.float32))
    oracle.sgdm4_step(w, np.zeros(P, np.float32), st, 1.0, 0.5)
    np.testing.assert_allclose(w[:4], [-1.5, 0.4375 + 0.21875, -0.2 - 0.10625, 0.0], rtol=1e-6)
    assert st.m_scales[0] == 0.5


def test_step_is_decompress_rule_compress():
    rng = np.random.default_rng(22)
    P, lr, beta = 128 * 7 + 53, 0.01, 0.9
    w, st = rng.standard_normal(P).astype(np.float32), oracle.state_zero_sgdm(P)
    w2, st2 = w.copy(), st.copy()
    for t in range(4):
        g = (rng.standard_normal(P) * rng.lognormal(0, 2, P)).astype(np.float32)
        mt = oracle.sgdm4_step(w, g, st, lr, beta, want_moment=True)
        m = oracle.dequant_m(st2.m_codes, st2.m_scales, P)
        oracle.sgdm32_step(w2, g, m, lr, beta)
        np.testing.assert_array_equal(mt, m)
        st2.m_codes, st2.m_scales = oracle.quant_m(m)
        np.testing.assert_array_equal(w, w2)
        np.testing.assert_array_equal(st.m_codes, st2.m_codes)
        np.testing.assert_array_equal(st.m_scales, st2.m_scales)
