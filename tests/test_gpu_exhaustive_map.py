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
