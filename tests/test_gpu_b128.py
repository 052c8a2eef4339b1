"""GPU parity tests of the single-pass step with the block-wise (B128/Linear) second moment, for
1-dimensional and flattened tensors, against the CPU oracle element by element."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, PARAM_ATOL, PARAM_RTOL, assert_codes_match, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-test] {request.node.name}", flush=True)
    yield
    torch.cuda.synchronize()


def upload(st: oracle.StateB128) -> lpmm.StateB128:
    return lpmm.StateB128(st.P, to_dev(st.m_codes), to_dev(st.m_scales), to_dev(st.v_codes), to_dev(st.v_scales))


def download(st: lpmm.StateB128) -> oracle.StateB128:
    f = lambda t: t.cpu().numpy().copy()
    return oracle.StateB128(st.numel, f(st.m_codes), f(st.m_blockscale), f(st.v_codes), f(st.v_blockscale))


def compare(got: oracle.StateB128, ref: oracle.StateB128, w_gpu, w_ref, mt, vt, tag):
    """Scales bit-exact; codes bit-exact up to flips within 2 ulp of a boundary (<= 1e-6 of the
    elements); parameters within 1e-5 relative / 1e-7 absolute."""
    np.testing.assert_array_equal(got.m_scales, ref.m_scales, err_msg=f"{tag}: m block scales")
    np.testing.assert_array_equal(got.v_scales, ref.v_scales, err_msg=f"{tag}: v block scales")
    P = mt.size
    sm = np.repeat(ref.m_scales, 128)[:P]
    sv = np.repeat(ref.v_scales, 128)[:P]
    with np.errstate(invalid="ignore", divide="ignore"):
        n_m = np.where(sm > 0, mt / sm, np.float32(0)).astype(np.float32)
        n_v = np.where(sv > 0, vt / sv, np.float32(0)).astype(np.float32)
    flips = assert_codes_match(got.m_codes, ref.m_codes, n_m, oracle.step_table("de"), f"{tag}: m codes")
    flips += assert_codes_match(got.v_codes, ref.v_codes, n_v, oracle.step_table("linear"), f"{tag}: v codes")
    if P & 1:   # the unused high nibble of the last byte stays 0
        assert got.m_codes[-1] >> 4 == 0 and got.v_codes[-1] >> 4 == 0, f"{tag}: padding nibble"
    np.testing.assert_allclose(w_gpu, w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=f"{tag}: parameters")
    return flips


def run(rows, cols, steps, recipe="iid", bf16=False, seed=21, hp=None, tid=0, mutate_grad=None):
    """The tensor is rows x cols taken flat (the shape only shapes the synthetic gradient)."""
    hp = hp or oracle.Hyper()
    P = rows * cols
    lpmm.ensure_init(4096)
    w_ref = workloads.weights(seed, tid, rows, cols).reshape(-1)
    st_ref = oracle.state_zero_b128(P)
    w = to_dev(w_ref.copy())
    st = lpmm.new_state_b128(P, DEV)
    fn = lpmm.lpmm_adamw4_b128_step_bf16g if bf16 else lpmm.lpmm_adamw4_b128_step
    total = 0
    for t in range(1, steps + 1):
        g = workloads.grads(seed, tid, t, rows, cols, recipe, bf16).reshape(-1)
        if mutate_grad is not None:
            g = mutate_grad(g, t)
        mt, vt = oracle.adamw4_b128_step(w_ref, g, st_ref, hp, t, want_moments=True)
        fn(w, to_dev(g, bf16), st, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)
        torch.cuda.synchronize()
        flips = compare(download(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, f"P={P} {recipe} step {t}")
        total += flips
        if flips:
            st = upload(st_ref)       # a tolerated flip must not spread
    return total


def test_zero_state_matches_oracle():
    for P in (2, 130, 4096, 999):
        got, ref = download(lpmm.new_state_b128(P, DEV)), oracle.state_zero_b128(P)
        for a, b in ((got.m_codes, ref.m_codes), (got.m_scales, ref.m_scales), (got.v_codes, ref.v_codes),
                     (got.v_scales, ref.v_scales)):
            np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("rows,cols", [(1, 128), (1, 4096), (1, 2), (1, 130), (1, 1000), (1, 127), (1, 999),
                                       (3, 128 * 8 * 16), (1, 128 * 8 * 16 + 128 * 5), (7, 4099), (64, 1024)])
def test_step_parity_small(rows, cols):
    # one block, one tile, less than a block, ragged tails (even and odd sizes), several tiles with a
    # partial last tile, a size that is nothing in particular
    assert run(rows, cols, steps=4) == 0


def test_bf16_gradients_and_column_structure():
    assert run(256, 1536, steps=4, recipe="col_lognormal", bf16=True) == 0


def test_long_run_stays_in_step():
    """200 steps with a gradient mean that persists and then dies away: growing, then shrinking block scales."""
    assert run(96, 256, steps=200, recipe="drift") == 0
    assert run(7, 333, steps=100, recipe="drift") == 0           # ragged last block


def test_outliers_and_zero_stretches():
    # config-3 style gradient: most rows zero in a step (whole blocks keep scale 0 or decay), a few
    # rows and columns 1000x larger
    assert run(1200, 512, steps=6, recipe="outlier_sparse") == 0


@pytest.mark.parametrize("hp", [oracle.Hyper(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1),
                                oracle.Hyper(lr=1e-4, beta1=0.0, beta2=0.5, eps=1e-12, weight_decay=0.0)])
def test_other_hyperparameters(hp):
    assert run(5, 128 * 40 + 64, steps=4, hp=hp) == 0


def test_extreme_scales_take_the_exact_route():
    # gradients so small / large that block scales leave [2^-100, 2^100] for some blocks
    def mut(g, t):
        g = g.copy()
        g[: 128 * 4] *= np.float32(1e-22)       # v ~ 1e-50 underflows towards denormals / zero
        g[128 * 4: 128 * 8] *= np.float32(1e18)  # v ~ 1e30 * ...: large but finite
        return g
    assert run(1, 128 * 64, steps=3, mutate_grad=mut) == 0


def test_launch_geometry_does_not_change_results():
    outs = []
    for rounds in ("1", "3", "16", "64"):
        os.environ["LPMM_B128_ROUNDS"] = rounds
        try:
            P = 128 * 8 * 20 + 128 * 3 + 50
            lpmm.ensure_init(4096)
            w = to_dev(workloads.weights(5, 0, 1, P).reshape(-1))
            st = lpmm.new_state_b128(P, DEV)
            for t in (1, 2, 3):
                g = to_dev(workloads.grads(5, 0, t, 1, P, "iid", False).reshape(-1))
                lpmm.lpmm_adamw4_b128_step(w, g, st, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
            torch.cuda.synchronize()
            d = download(st)
            outs.append((w.cpu().numpy(), d.m_codes, d.m_scales, d.v_codes, d.v_scales))
        finally:
            os.environ.pop("LPMM_B128_ROUNDS", None)
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            np.testing.assert_array_equal(a, b)


def test_dequant_matches_oracle():
    rng = np.random.default_rng(7)
    P = 128 * 9 + 70
    x = (rng.standard_normal(P).astype(np.float32) * np.float32(1e-3)) ** 2
    codes, scales = oracle.quant_v_block(x)
    out = torch.empty(P, device=DEV)
    lpmm.ensure_init(4096)
    lpmm.lpmm_dequant_state(2, to_dev(np.concatenate([codes, np.zeros((-codes.size) % 4, np.uint8)])), to_dev(scales),
                            None, 1, P, out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), oracle.dequant_v_block(codes, scales, P))


def test_quant_matches_oracle():
    rng = np.random.default_rng(8)
    P = 128 * 11 + 30
    x = (rng.standard_normal(P).astype(np.float32) * np.float32(2e-3)) ** 2
    x[256:384] = 0.0                                   # a zero block
    x[500] = 7.0                                       # an outlier
    want_codes, want_scales = oracle.quant_v_block(x)
    lpmm.ensure_init(4096)
    codes = torch.zeros((want_codes.size + 3) // 4 * 4, dtype=torch.uint8, device=DEV)
    scales = torch.empty(want_scales.size, device=DEV)
    lpmm.lpmm_quant_state(2, to_dev(x), 1, P, codes, scales, None)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(scales.cpu().numpy(), want_scales)
    np.testing.assert_array_equal(codes.cpu().numpy()[:want_codes.size], want_codes)


def test_plan_with_mixed_kinds():
    """One plan holding rank-1 tensors, block-wise tensors and fp32-state tensors."""
    from test_gpu_multi import HP
    from gpu_util import compare_step, download_state
    lpmm.ensure_init(4096)
    seed = 31
    shapes = [("r1", 256, 384, "rank1"), ("flat_a", 1, 128 * 300 + 20, "b128"), ("ln", 1, 512, "fp32"),
              ("flat_b", 96, 1024, "b128"), ("r2", 300, 256, "rank1")]
    dev, ref, descs = [], [], []
    for tid, (name, rows, cols, kind) in enumerate(shapes):
        P = rows * cols
        w_ref = workloads.weights(seed, tid, rows, cols).reshape(-1)
        w = to_dev(w_ref.copy())
        g = torch.empty(P, dtype=torch.float32, device=DEV)
        if kind == "rank1":
            st, st_ref = lpmm.new_state(rows, cols, DEV), oracle.state_zero(rows, cols)
            descs.append(lpmm.make_desc(w, g, st))
        elif kind == "b128":
            st, st_ref = lpmm.new_state_b128(P, DEV), oracle.state_zero_b128(P)
            descs.append(lpmm.make_desc(w, g, st))
        else:
            st = (torch.zeros(P, device=DEV), torch.zeros(P, device=DEV))
            st_ref = (np.zeros(P, np.float32), np.zeros(P, np.float32))
            descs.append(lpmm.make_desc(w, g, st, rows, cols))
        dev.append((w, g, st))
        ref.append((w_ref, st_ref))
    plan = lpmm.new_plan(descs, 0, DEV)
    for t in range(1, 4):
        grads = [workloads.grads(seed, tid, t, rows, cols, "col_lognormal", False).reshape(-1)
                 for tid, (_, rows, cols, _) in enumerate(shapes)]
        for (w, g, st), gn in zip(dev, grads):
            g.copy_(to_dev(gn))
        lpmm.lpmm_adamw4_step_multi(plan, HP.lr, HP.beta1, HP.beta2, HP.eps, HP.weight_decay, t)
        torch.cuda.synchronize()
        for (name, rows, cols, kind), (w, g, st), (w_ref, st_ref), gn in zip(shapes, dev, ref, grads):
            tag = f"{name} step {t}"
            if kind == "rank1":
                mt, vt = oracle.adamw4_step(w_ref, gn, st_ref, HP, t, want_moments=True)
                assert compare_step(download_state(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, tag) == 0
            elif kind == "b128":
                mt, vt = oracle.adamw4_b128_step(w_ref, gn, st_ref, HP, t, want_moments=True)
                assert compare(download(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, tag) == 0
            else:
                oracle.adamw32_step(w_ref, gn, st_ref[0], st_ref[1], HP, t)
                np.testing.assert_array_equal(st[0].cpu().numpy(), st_ref[0], err_msg=tag)
                np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=tag)
    lpmm.lpmm_adamw4_plan_release(plan)


def test_argument_errors():
    lpmm.ensure_init(4096)
    st = lpmm.new_state_b128(256, DEV)
    w = torch.zeros(256, device=DEV)
    g = torch.zeros(256, device=DEV)
    with pytest.raises(lpmm.LpmmError):
        lpmm.lpmm_adamw4_b128_step(w, g, st, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0)         # step < 1
    with pytest.raises(lpmm.LpmmError):
        lpmm.lpmm_adamw4_b128_step(w, g, st, 1e-3, 1.0, 0.999, 1e-8, 0.0, 1)         # beta1 = 1
    with pytest.raises(lpmm.LpmmError):
        lpmm.lpmm_adamw4_b128_step(w[1:], g, st, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1)     # misaligned param
    with pytest.raises(lpmm.LpmmError):
        lpmm.lpmm_adamw4_b128_state_sizes(0)
