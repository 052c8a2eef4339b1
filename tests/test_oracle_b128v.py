"""Pins of the oracle's block-wise (B128/Linear) second moment and of the step that uses it.

What fixes the expected values: a worked example (tests/golden/b128_linear_by_hand.txt), the closed
form of the Linear map's nearest-entry search, the already pinned rank-1 quantizer on a matrix built so
that its rank-1 scales ARE the block maxima, the already pinned first-moment quantizer, and an fp64
AdamW for the first step from the zero state.
"""
import numpy as np
import pytest

import oracle
from conftest import golden

HAND = golden("b128_linear_by_hand.txt")


def _hand_tensor():
    n = int(HAND["n"][0])
    x = np.zeros(n, np.float32)
    idx = np.array(HAND["idx"], np.int64)
    x[idx] = np.array(HAND["val"], np.float64).astype(np.float32)
    return x, idx


def test_hand_example():
    x, idx = _hand_tensor()
    codes, scales = oracle.quant_v_block(x)
    np.testing.assert_array_equal(scales, np.array(HAND["scales"], np.float64).astype(np.float32))
    q = oracle.unpack_codes(codes, x.size)
    np.testing.assert_array_equal(q[idx], np.array(HAND["codes_at_idx"], np.uint8))
    rest = np.ones(x.size, bool)
    rest[idx] = False
    assert (q[rest] == int(HAND["code_elsewhere"][0])).all()
    d = oracle.dequant_v_block(codes, scales, x.size)
    np.testing.assert_array_equal(d[idx], np.array(HAND["dequant_at_idx"], np.float64).astype(np.float32))
    # block 1 holds only the two listed elements; every unlisted element lies in block 0
    assert (d[rest] == np.float32(HAND["dequant_elsewhere"][0])).all()


def test_codes_follow_the_closed_form_of_the_linear_map():
    # nearest (k+1)/16 with ties to the lower index is clamp(ceil(16 n - 1.5), 0, 15); n is the fp32
    # quotient by the block maximum, computed here with numpy
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(128 * 9 + 50).astype(np.float32)) ** 2
    x[300:428] = 0.0                                          # an all-zero stretch covering block 3 partly
    x[384:512] = 0.0                                          # block 3 entirely zero
    codes, scales = oracle.quant_v_block(x)
    nb = oracle.n_blocks(x.size)
    pad = np.zeros(nb * 128, np.float32)
    pad[:x.size] = x
    smax = pad.reshape(nb, 128).max(axis=1)
    np.testing.assert_array_equal(scales, smax)
    assert scales[3] == 0.0
    s_el = np.repeat(smax, 128)[:x.size]
    with np.errstate(divide="ignore", invalid="ignore"):
        n = np.where(s_el == 0, np.float32(0), x / s_el).astype(np.float32)
    want = np.clip(np.ceil(16.0 * n.astype(np.float64) - 1.5), 0, 15).astype(np.uint8)
    np.testing.assert_array_equal(oracle.unpack_codes(codes, x.size), want)


def test_equals_rank1_when_the_rank1_scales_are_the_block_maxima():
    # A k x 128 matrix plus one extra row of huge values: every column maximum is huge, so
    # min(r_i, c_j) = r_i, and row i is exactly block i of the flattened matrix.  The rank-1 quantizer
    # (pinned on its own) must then give the codes of the block-wise one for the first k rows.
    rng = np.random.default_rng(2)
    k = 11
    x = (rng.standard_normal((k, 128)).astype(np.float32)) ** 2
    x[4] = 0.0                                                # a zero row = a zero block
    big = np.full((1, 128), 1e6, np.float32)
    codes_r1, r, c = oracle.quant_v(np.concatenate([x, big], axis=0))
    codes_b, scales = oracle.quant_v_block(x.reshape(-1))
    np.testing.assert_array_equal(scales, r[:k])
    q_r1 = oracle.unpack_codes(codes_r1, (k + 1) * 128)[: k * 128]
    np.testing.assert_array_equal(oracle.unpack_codes(codes_b, k * 128), q_r1)


def test_invariants():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(128 * 40 + 77).astype(np.float32) * np.float32(3e-4)) ** 2
    x[1000] = 5.0                                             # an outlier only hurts its own block
    codes, scales = oracle.quant_v_block(x)
    d = oracle.dequant_v_block(codes, scales, x.size)
    nb = oracle.n_blocks(x.size)
    s_el = np.repeat(scales, 128)[:x.size]
    # zero point absent (Sec. 4.1): a non-zero block never dequantizes to 0, smallest value is scale/16
    assert (d[s_el > 0] >= s_el[s_el > 0] / 16).all()
    # the block maximum has n = 1, code 15, and comes back exactly
    pad = np.zeros(nb * 128, np.float32)
    pad[:x.size] = d
    np.testing.assert_array_equal(pad.reshape(nb, 128).max(axis=1), scales)
    # error: half a step (scale/32) above the lowest entry, at most scale/16 below it
    err = np.abs(d.astype(np.float64) - x)
    hi = x >= s_el / 16
    assert (err[hi] <= s_el[hi] / 32 * (1 + 1e-6)).all()
    assert (err[~hi] <= s_el[~hi] / 16 * (1 + 1e-6)).all()
    # compress o decompress o compress == compress
    codes2, scales2 = oracle.quant_v_block(d)
    np.testing.assert_array_equal(codes2, codes)
    np.testing.assert_array_equal(scales2, scales)
    # the outlier's block: everything else collapses to the lowest code, other blocks are untouched
    q = oracle.unpack_codes(codes, x.size)
    blk = 1000 // 128
    others = np.r_[blk * 128:1000, 1001:(blk + 1) * 128]
    assert (q[others] == 0).all() and q[1000] == 15
    x2 = x.copy()
    x2[1000] = x[1001]
    q2 = oracle.unpack_codes(oracle.quant_v_block(x2)[0], x.size)
    keep = np.ones(x.size, bool)
    keep[blk * 128:(blk + 1) * 128] = False
    np.testing.assert_array_equal(q[keep], q2[keep])


def test_zero_state():
    st = oracle.state_zero_b128(300)
    assert (st.m_codes == 0x77).all() and (st.m_scales == 0).all()
    assert (st.v_codes == 0).all() and (st.v_scales == 0).all()
    assert (oracle.dequant_v_block(st.v_codes, st.v_scales, 300) == 0).all()


def _fp64_adamw_first_step(w, g, hp):
    # closed form of step 1 from m = v = 0 (Eq. 1): m^ = g, v^ = g^2 up to the fp32 rounding of the
    # moments, so w' = w - lr (g / (|g| + eps) + wd w); evaluated here from the fp32 moments in fp64
    b1, b2 = np.float32(hp.beta1), np.float32(hp.beta2)
    m = (np.float32(1) - b1) * g
    v = ((np.float32(1) - b2) * g) * g
    mh = m.astype(np.float64) / (1.0 - float(b1))
    vh = v.astype(np.float64) / (1.0 - float(b2))
    w64 = w.astype(np.float64)
    lr, eps, wd = (float(np.float32(z)) for z in (hp.lr, hp.eps, hp.weight_decay))
    return m, v, w64 - lr * (mh / (np.sqrt(vh) + eps) + wd * w64)


def test_first_step_equals_plain_adamw_and_compresses_its_moments():
    # the parameter update uses the precise moments (compress is the last line of Alg. 3), so step 1
    # from the zero state is plain AdamW; the stored state is the compressed (m_1, v_1)
    rng = np.random.default_rng(4)
    P = 128 * 5 + 64
    w = (rng.standard_normal(P) * 0.02).astype(np.float32)
    g = (rng.standard_normal(P) * 1e-3).astype(np.float32)
    hp = oracle.Hyper()
    m1, v1, w_ref = _fp64_adamw_first_step(w, g, hp)
    st = oracle.state_zero_b128(P)
    w4 = w.copy()
    mt, vt = oracle.adamw4_b128_step(w4, g, st, hp, 1, want_moments=True)
    np.testing.assert_array_equal(mt, m1)
    np.testing.assert_array_equal(vt, v1)
    np.testing.assert_allclose(w4, w_ref, rtol=2e-7, atol=1e-12)
    mc, ms = oracle.quant_m(m1)
    vc, vs = oracle.quant_v_block(v1)
    for got, want in ((st.m_codes, mc), (st.m_scales, ms), (st.v_codes, vc), (st.v_scales, vs)):
        np.testing.assert_array_equal(got, want)


def test_step_is_decompress_rule_compress():
    # Alg. 3 written out with the separately pinned pieces, over several steps
    rng = np.random.default_rng(5)
    P = 128 * 3 + 2
    w = (rng.standard_normal(P) * 0.02).astype(np.float32)
    hp = oracle.Hyper(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)
    st = oracle.state_zero_b128(P)
    w_a, w_b = w.copy(), w.copy()
    mc, ms, vc, vs = st.m_codes.copy(), st.m_scales.copy(), st.v_codes.copy(), st.v_scales.copy()
    for t in range(1, 6):
        g = (rng.standard_normal(P) * 1e-2).astype(np.float32)
        oracle.adamw4_b128_step(w_a, g, st, hp, t)
        m = oracle.dequant_m(mc, ms, P)
        v = oracle.dequant_v_block(vc, vs, P)
        oracle.adamw32_step(w_b, g, m, v, hp, t)               # the rule on the decompressed states
        mc, ms = oracle.quant_m(m)
        vc, vs = oracle.quant_v_block(v)
        np.testing.assert_array_equal(w_a, w_b)
        for got, want in ((st.m_codes, mc), (st.m_scales, ms), (st.v_codes, vc), (st.v_scales, vs)):
            np.testing.assert_array_equal(got, want)


def test_first_moment_path_is_shared_with_the_rank1_step_on_step_one():
    # both optimizers treat m identically; on step 1 (precise moments) params agree too
    rng = np.random.default_rng(6)
    rows, cols = 6, 192
    w = (rng.standard_normal(rows * cols) * 0.02).astype(np.float32)
    g = (rng.standard_normal(rows * cols) * 1e-3).astype(np.float32)
    hp = oracle.Hyper()
    sa, sb = oracle.state_zero(rows, cols), oracle.state_zero_b128(rows * cols)
    wa, wb = w.copy(), w.copy()
    oracle.adamw4_step(wa, g, sa, hp, 1)
    oracle.adamw4_b128_step(wb, g, sb, hp, 1)
    np.testing.assert_array_equal(wa, wb)
    np.testing.assert_array_equal(sa.m_codes, sb.m_codes)
    np.testing.assert_array_equal(sa.m_scales, sb.m_scales)
