"""Every fp32 value of the normalized range through the GPU's nearest-entry search, against the oracle.

Both mappings are step functions of n.  The oracle's steps are located by bisection over the ordered fp32 values
with its brute-force argmin (15 steps each); the GPU quantizes ALL fp32 values in [-1, 1] (first moment, signed
dynamic-exponent map, 2.13e9 values) and in [0, 1] (second moment, Linear map) -- each block of 128 holds one
element equal to 1, so that the block scale is 1 and n is the value itself -- and every code must equal the number
of oracle steps below the value."""
import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _ordered_to_float(k: np.ndarray) -> np.ndarray:
    """k in [-0x3F800000, 0x3F800000] enumerates the fp32 values of [-1, 1] in increasing order (k = 0: +0)."""
    k = np.asarray(k, np.int64)
    bits = np.where(k >= 0, k, (-k) | 0x80000000).astype(np.uint32)
    return bits.view(np.float32)


def _oracle_steps(table: np.ndarray, lo: int, hi: int):
    """For c = 0..14: the largest ordered index whose oracle code is <= c."""
    code = lambda k: int(oracle.nearest_codes(table, _ordered_to_float(np.array([k])))[0])
    assert code(hi) == 15
    out = []
    for c in range(code(lo), 15):
        a, b = lo, hi                      # code(a) <= c < code(b)
        while b - a > 1:
            mid = (a + b) // 2
            if code(mid) <= c:
                a = mid
            else:
                b = mid
        out.append(a)
    return out


def _sweep(which: int, table: np.ndarray, lo: int, hi: int):
    steps = _oracle_steps(table, lo, hi)
    first_code = int(oracle.nearest_codes(table, _ordered_to_float(np.array([lo])))[0])
    bounds = torch.from_numpy(_ordered_to_float(np.array(steps))).to(DEV)
    lpmm.ensure_init(4096)
    n_blocks = 1 << 20                                         # 127 values per block, 133 M values per chunk
    per_chunk = n_blocks * 127
    x = torch.empty(n_blocks, 128, device=DEV)
    codes = torch.empty(n_blocks * 64, dtype=torch.uint8, device=DEV)
    scales = torch.empty(n_blocks, device=DEV)
    total = 0
    seen = torch.zeros(16, dtype=torch.bool, device=DEV)
    for start in range(lo, hi + 1, per_chunk):
        k = torch.arange(start, start + per_chunk, device=DEV, dtype=torch.int64).clamp_(max=hi)
        bits = torch.where(k >= 0, k, (-k) - 0x80000000).to(torch.int32)      # int32 with the sign bit set
        x[:, 0] = 1.0
        x[:, 1:] = bits.view(torch.float32).view(n_blocks, 127)
        lpmm.lpmm_quant_state(which, x.view(-1), 1, n_blocks * 128, codes, scales, None)
        got = torch.stack([codes & 15, codes >> 4], dim=1).view(n_blocks, 128)[:, 1:]
        want = first_code + torch.bucketize(x[:, 1:].contiguous(), bounds, right=False)
        assert bool((scales == 1.0).all())
        bad = got != want.to(torch.uint8)
        assert not bool(bad.any()), f"first mismatch at value {float(x[:, 1:][bad][0])!r}"
        seen |= torch.bincount(got.reshape(-1).to(torch.int64), minlength=16) > 0
        total += per_chunk
        print(f"[gpu-test] exhaustive map {which}: {min(total, hi - lo + 1)} values", flush=True)
    torch.cuda.synchronize()
    assert int(seen.sum()) == 16 - first_code            # every code occurred: the comparison above was not vacuous


def test_every_fp32_in_minus_one_to_one_through_the_dynamic_exponent_map():
    _sweep(0, oracle.step_table("de"), -0x3F800000, 0x3F800000)


def test_every_fp32_in_zero_to_one_through_the_linear_map():
    _sweep(2, oracle.step_table("linear"), 0, 0x3F800000)


def test_every_fp32_through_the_step_kernels_compress_path():
    """The step kernels do not divide: they multiply by an approximate reciprocal and fall back to the exact
    route near a decision boundary.  From the zero state one SGD-with-momentum step has m_t = g exactly, so
    feeding every fp32 value of [-1, 1] as the gradient (block scale 1 as above) sends every value through that
    path."""
    table = oracle.step_table("de")
    lo, hi = -0x3F800000, 0x3F800000
    steps = _oracle_steps(table, lo, hi)
    bounds = torch.from_numpy(_ordered_to_float(np.array(steps))).to(DEV)
    lpmm.ensure_init(4096)
    n_blocks = 1 << 20
    per_chunk = n_blocks * 127
    g = torch.empty(n_blocks, 128, device=DEV)
    w = torch.zeros(n_blocks * 128, device=DEV)
    seen = torch.zeros(16, dtype=torch.bool, device=DEV)
    for start in range(lo, hi + 1, per_chunk):
        k = torch.arange(start, start + per_chunk, device=DEV, dtype=torch.int64).clamp_(max=hi)
        bits = torch.where(k >= 0, k, (-k) - 0x80000000).to(torch.int32)
        g[:, 0] = 1.0
        g[:, 1:] = bits.view(torch.float32).view(n_blocks, 127)
        st = lpmm.new_state_sgdm(n_blocks * 128, DEV)
        lpmm.lpmm_sgdm4_step(w, g.view(-1), st, 0.0, 0.5)
        codes = st.m_codes
        got = torch.stack([codes & 15, codes >> 4], dim=1).view(n_blocks, 128)[:, 1:]
        want = torch.bucketize(g[:, 1:].contiguous(), bounds, right=False)
        assert bool((st.m_blockscale == 1.0).all())
        bad = got != want.to(torch.uint8)
        assert not bool(bad.any()), f"first mismatch at value {float(g[:, 1:][bad][0])!r}"
        seen |= torch.bincount(got.reshape(-1).to(torch.int64), minlength=16) > 0
    torch.cuda.synchronize()
    assert int(seen.sum()) == 16
    print("[gpu-test] exhaustive: step compress path done", flush=True)


# ---- block scales that are not powers of two: the reciprocal is inexact, the guard has to work ------------------
#
# With a block scale of exactly 1 the approximate reciprocal is exact, so the sweeps above never see the error that
# the step kernels' guard (distance of the approximate normalized value to the nearest decision boundary, exact
# fallback when it is small) exists for.  Below, every block holds one element that fixes the block's scale at a
# value s with a full mantissa, and the other 127 elements sweep every fp32 value that normalizes into the map's
# range.  The oracle's code is still a non-decreasing step function of the swept value (a correctly rounded
# quotient by a positive constant is monotone), so its 15 steps are found by bisection with the oracle's own
# quantizer, which divides.

M_SCALES = [0.37, 3.1e-7, 1.9999999, 2.0 ** -99.5, 1.7e29]


def _float_to_ordered(x: float) -> int:
    b = int(np.float32(x).view(np.uint32))
    return b if b < 0x80000000 else -(b & 0x7FFFFFFF)


def _bisect_steps(code, lo, hi, top):
    """Largest ordered index with code <= c, for c = code(lo) .. top - 1."""
    assert code(hi) == top
    out = []
    for c in range(code(lo), top):
        a, b = lo, hi
        while b - a > 1:
            mid = (a + b) // 2
            if code(mid) <= c:
                a = mid
            else:
                b = mid
        out.append(a)
    return out


def _chunks(lo, hi, per_chunk):
    for start in range(lo, hi + 1, per_chunk):
        k = torch.arange(start, start + per_chunk, device=DEV, dtype=torch.int64).clamp_(max=hi)
        yield torch.where(k >= 0, k, (-k) - 0x80000000).to(torch.int32).view(torch.float32)


@pytest.mark.parametrize("scale", M_SCALES)
def test_first_moment_compress_path_at_block_scales_with_full_mantissas(scale):
    """One SGD-with-momentum step from the zero state has m_t = g exactly: every fp32 value of [-s, s] goes through
    the step kernel's multiply-by-reciprocal route (and its exact fallback) under the block scale s."""
    from conftest import progress
    s = np.float32(scale)
    hi = _float_to_ordered(float(s))
    lo = -hi

    def code(k):
        blk = np.zeros(128, np.float32)
        blk[0], blk[1] = s, _ordered_to_float(np.array([k]))[0]
        return int(oracle.unpack_codes(oracle.quant_m(blk)[0], 128)[1])

    first = code(lo)
    bounds = torch.from_numpy(_ordered_to_float(np.array(_bisect_steps(code, lo, hi, 15)))).to(DEV)
    assert bounds.numel() == 15 - first
    lpmm.ensure_init(4096)
    n_blocks = 1 << 20
    g = torch.empty(n_blocks, 128, device=DEV)
    w = torch.zeros(n_blocks * 128, device=DEV)
    seen = torch.zeros(16, dtype=torch.bool, device=DEV)
    for vals in _chunks(lo, hi, n_blocks * 127):
        g[:, 0] = float(s)
        g[:, 1:] = vals.view(n_blocks, 127)
        st = lpmm.new_state_sgdm(n_blocks * 128, DEV)
        lpmm.lpmm_sgdm4_step(w, g.view(-1), st, 0.0, 0.5)
        codes = st.m_codes
        got = torch.stack([codes & 15, codes >> 4], dim=1).view(n_blocks, 128)[:, 1:]
        want = first + torch.bucketize(g[:, 1:].contiguous(), bounds, right=False)
        assert bool((st.m_blockscale == float(s)).all())
        bad = got != want.to(torch.uint8)
        assert not bool(bad.any()), f"scale {float(s)!r}: first mismatch at value {float(g[:, 1:][bad][0])!r}"
        seen |= torch.bincount(got.reshape(-1).to(torch.int64), minlength=16) > 0
    torch.cuda.synchronize()
    assert int(seen.sum()) == 16 - first
    progress(f"exhaustive: first-moment compress path at block scale {float(s)!r}: {hi - lo + 1} values, no flip")


V_SCALES = [0.37, 3.1e-7, 1.9999999, 2.0 ** -99.5, 7.3e28]


def _sweep_second_moment(scale, step_fn, layout):
    """beta1 = beta2 = 0 from the zero state: v_t = fl(g * g) and m_t = g.  Every fp32 g >= 0 with fl(g * g) <= s
    is swept; one element per block (`layout` says where) holds g0 with fl(g0 * g0) = s' close to `scale`.
    step_fn(w, g, n_blocks) runs one step and returns (m code bytes, v code bytes, the scales that must equal s')."""
    from conftest import progress
    g0 = np.float32(np.sqrt(np.float64(scale)))
    s = np.float32(g0 * g0)                                     # the block's maximum, one fp32 rounding
    assert np.frexp(s)[0] not in (0.5, 1.0)                    # not a power of two: its reciprocal is inexact
    hp0 = oracle.Hyper(lr=0.0, beta1=0.0, beta2=0.0, eps=1e-8, weight_decay=0.0)

    def codes_of(k):
        gb = np.zeros(128, np.float32)
        gb[0], gb[1] = g0, _ordered_to_float(np.array([k]))[0]
        st = oracle.state_zero_b128(128)
        oracle.adamw4_b128_step(np.zeros(128, np.float32), gb, st, hp0, 1)
        assert st.v_scales[0] == s and st.m_scales[0] == g0
        return int(oracle.unpack_codes(st.m_codes, 128)[1]), int(oracle.unpack_codes(st.v_codes, 128)[1])

    lo, hi = 0, _float_to_ordered(float(g0))
    v_first, m_first = codes_of(lo)[1], codes_of(lo)[0]
    v_bounds = torch.from_numpy(_ordered_to_float(np.array(_bisect_steps(lambda k: codes_of(k)[1], lo, hi, 15)))).to(DEV)
    m_bounds = torch.from_numpy(_ordered_to_float(np.array(_bisect_steps(lambda k: codes_of(k)[0], lo, hi, 15)))).to(DEV)
    assert v_first == 0 and m_first == 7
    n_blocks = 1 << 20
    lpmm.ensure_init(n_blocks + 4096)               # the rank-1 form sees n_blocks rows
    g = torch.empty(n_blocks, 128, device=DEV)
    w = torch.zeros(n_blocks * 128, device=DEV)
    seen = torch.zeros(16, dtype=torch.bool, device=DEV)
    for vals in _chunks(lo, hi, n_blocks * 127):
        g[:, 0] = float(g0)
        g[:, 1:] = vals.view(n_blocks, 127)
        layout(g, float(g0))
        mq, vq, scales = step_fn(w, g.view(-1), n_blocks)
        assert bool((scales == float(s)).all())
        for q, first, bounds, what in ((vq, v_first, v_bounds, "v"), (mq, m_first, m_bounds, "m")):
            got = torch.stack([q & 15, q >> 4], dim=1).view(n_blocks, 128)[:, 1:]
            want = first + torch.bucketize(g[:, 1:].contiguous(), bounds, right=False)
            bad = got != want.to(torch.uint8)
            assert not bool(bad.any()), f"scale {float(s)!r}: first {what} mismatch at g = {float(g[:, 1:][bad][0])!r}"
            if what == "v":
                seen |= torch.bincount(got.reshape(-1).to(torch.int64), minlength=16) > 0
    torch.cuda.synchronize()
    assert int(seen.sum()) == 16
    progress(f"exhaustive: second-moment compress path at scale {float(s)!r}: {hi - lo + 1} values, no flip")


@pytest.mark.parametrize("scale", V_SCALES)
def test_second_moment_compress_path_of_the_block_wise_step(scale):
    """Through lpmm_adamw4_b128_step: the block-wise second moment's reciprocal-and-guard route (and, with
    beta1 = 0, the AdamW kernels' first-moment route) at a block maximum with a full mantissa."""
    def step(w, g, n_blocks):
        st = lpmm.new_state_b128(n_blocks * 128, DEV)
        lpmm.lpmm_adamw4_b128_step(w, g, st, 0.0, 0.0, 0.0, 1e-8, 0.0, 1)
        return st.m_codes, st.v_codes, st.v_blockscale
    _sweep_second_moment(scale, step, lambda g, g0: None)


@pytest.mark.parametrize("scale", V_SCALES[:3])
def test_second_moment_compress_path_of_the_rank1_step(scale):
    """Through lpmm_adamw4_step (pass 1 + pass 2) on a matrix of 128 columns: column 0 holds g0 in every row and row 0
    holds g0 in every column, so every row maximum and every column maximum of v_t is s and every element is
    normalized by min(r'_i, c'_j) = s; pass 2 multiplies by max(rcp r', rcp c')."""
    def layout(g, g0):
        g[0, :] = g0

    def step(w, g, n_blocks):
        st = lpmm.new_state(n_blocks, 128, DEV)
        lpmm.lpmm_adamw4_step(w, g, st, 0.0, 0.0, 0.0, 1e-8, 0.0, 1)
        assert bool((st.v_colmax == st.v_rowmax[0]).all())
        return st.m_codes, st.v_codes, st.v_rowmax
    _sweep_second_moment(scale, step, layout)
