"""The ablation quantizers of the second moment on the GPU (lpmm_quant_ablation / lpmm_dequant_ablation: Sec. 4.1,
Tab. 1, stochastic rounding of App. D.3) against the oracle: codes, scales and decompressed values bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu

NORM = {"b128": lpmm.NORM_B128, "b2048": lpmm.NORM_B2048, "rank1": lpmm.NORM_RANK1}
MAP = {"de": lpmm.MAP_DE, "de0": lpmm.MAP_DE0, "linear": lpmm.MAP_LINEAR}
# every quantizer of Tab. 1 (second moment), the signed ones of its first line (first moment), and the rest of the grid
COMBOS = [(n, m, False) for n in ("b2048", "b128", "rank1") for m in ("de", "de0", "linear")] + \
         [("b2048", "de", True), ("b128", "de", True)]


def _input(rows, cols, signed, seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, cols)) * np.exp(2 * rng.standard_normal((rows, cols)))).astype(np.float32)
    if not signed:
        x = (x * x).astype(np.float32)
    if rows > 4:
        x[3, :] = 0.0                                 # a zero row
    flat = x.reshape(-1)
    if flat.size > 4096:
        flat[2048:4096] = 0.0                         # a zero block of 2048 (and 16 of 128)
    return x


def _gpu_quant(x, norm, map_name, signed, stochastic, seed):
    rows, cols = x.shape
    na, nb = lpmm.ablation_scale_sizes(NORM[norm], rows, cols)
    codes = torch.full((((x.size + 1) // 2 + 3) // 4 * 4,), 0xEE, dtype=torch.uint8, device=DEV)[:(x.size + 1) // 2]
    sa = torch.full((na,), -1.0, device=DEV)
    sb = torch.full((max(nb, 1),), -1.0, device=DEV)
    lpmm.lpmm_quant_ablation(NORM[norm], MAP[map_name], signed, int(stochastic), seed, to_dev(x.reshape(-1)), rows, cols,
                             codes, sa, sb if nb else None)
    return codes, sa, sb


@pytest.mark.parametrize("norm,map_name,signed", COMBOS)
@pytest.mark.parametrize("shape", [(21, 300), (64, 2048), (1, 130), (257, 1031)])
@pytest.mark.parametrize("stochastic", [False, True])
def test_ablation_quantizers_match_the_oracle(norm, map_name, signed, shape, stochastic):
    rows, cols = shape
    print(f"[gpu-test] ablation {norm}/{map_name} signed={signed} sr={stochastic} {rows}x{cols}", flush=True)
    lpmm.ensure_init(4096)
    x = _input(rows, cols, signed, seed=rows * 7 + cols)
    seed = 1234567 + rows
    want_codes, want_sa, want_sb = oracle.quant_ablation(x, norm, map_name, signed, stochastic, seed)
    codes, sa, sb = _gpu_quant(x, norm, map_name, signed, stochastic, seed)
    torch.cuda.synchronize()
    P = x.size
    got = oracle.unpack_codes(codes.cpu().numpy(), P)
    np.testing.assert_array_equal(sa.cpu().numpy(), want_sa, err_msg="scale_a")
    if norm == "rank1":
        np.testing.assert_array_equal(sb.cpu().numpy(), want_sb, err_msg="scale_b")
    np.testing.assert_array_equal(got, oracle.unpack_codes(want_codes, P), err_msg="codes")
    if P % 2:
        assert int(codes[-1]) >> 4 == 0                               # the unused nibble of an odd tail stays 0
    out = torch.full((P,), -7.0, device=DEV)
    lpmm.lpmm_dequant_ablation(NORM[norm], MAP[map_name], signed, codes, sa, sb if norm == "rank1" else None, rows, cols, out)
    want = oracle.dequant_ablation(want_codes, want_sa, want_sb, rows, cols, norm, map_name, signed)
    np.testing.assert_array_equal(out.cpu().numpy().reshape(rows, cols), want)


def test_stochastic_rounding_depends_on_the_seed_only():
    """Same seed, same codes, whatever was launched before; another seed, other codes; each code is the nearest
    entry or its neighbour."""
    lpmm.ensure_init(4096)
    x = _input(300, 1024, False, seed=5)
    a = _gpu_quant(x, "b128", "de", False, True, 11)[0].clone()
    _gpu_quant(_input(64, 256, False, seed=6), "rank1", "de0", False, True, 12)
    b = _gpu_quant(x, "b128", "de", False, True, 11)[0]
    c = _gpu_quant(x, "b128", "de", False, True, 13)[0]
    near = _gpu_quant(x, "b128", "de", False, False, 0)[0]
    assert torch.equal(a, b) and not torch.equal(a, c)
    ua, un = oracle.unpack_codes(a.cpu().numpy(), x.size).astype(int), oracle.unpack_codes(near.cpu().numpy(), x.size).astype(int)
    assert np.abs(ua - un).max() == 1


def test_bad_arguments_are_refused():
    import ctypes
    lpmm.ensure_init(4096)
    L = lpmm.lib()
    t = torch.zeros(4096, device=DEV)
    p = t.data_ptr()
    shape = (ctypes.c_int64 * 2)(4, 128)
    q = lambda *a: L.lpmm_quant_ablation(*a, 0, p, ctypes.addressof(shape), p, p, p, None)
    assert q(2, 0, 1, 0) == -1          # rank-1 of signed input
    assert q(0, 1, 1, 0) == -1          # signed DE-0
    assert q(3, 0, 0, 0) == -1          # no such normalization
    assert q(0, 0, 0, 2) == -1          # no such rounding
    assert L.lpmm_quant_ablation(2, 0, 0, 0, 0, p, ctypes.addressof(shape), p, p, None, None) == -1     # rank-1 without column maxima
    assert L.lpmm_dequant_ablation(0, 5, 0, p, p, None, ctypes.addressof(shape), p, None) == -1
    torch.cuda.synchronize()
