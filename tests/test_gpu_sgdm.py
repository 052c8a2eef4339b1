"""GPU parity tests of SGD with momentum and 4-bit momentum (App. E Alg. 2) against the CPU oracle, element by
element: momentum codes and block scales bit-exact (flips only within 2 ulp of a decision boundary, at most 1e-6
of the elements), parameters within 1e-5 relative / 1e-7 absolute."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, PARAM_ATOL, PARAM_RTOL, assert_codes_match, to_dev

pytestmark = pytest.mark.gpu
LR, BETA = 0.05, 0.9


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-test] {request.node.name}", flush=True)
    yield
    torch.cuda.synchronize()


def download(st: lpmm.StateSgdm) -> oracle.StateSgdm:
    return oracle.StateSgdm(st.numel, st.m_codes.cpu().numpy().copy(), st.m_blockscale.cpu().numpy().copy())


def compare(got, ref, w_gpu, w_ref, mt, tag):
    np.testing.assert_array_equal(got.m_scales, ref.m_scales, err_msg=f"{tag}: block scales")
    P = mt.size
    sm = np.repeat(ref.m_scales, 128)[:P]
    with np.errstate(invalid="ignore", divide="ignore"):
        n_m = np.where(sm > 0, mt / sm, np.float32(0)).astype(np.float32)
    flips = assert_codes_match(got.m_codes, ref.m_codes, n_m, oracle.step_table("de"), f"{tag}: m codes")
    if P & 1:
        assert got.m_codes[-1] >> 4 == 0, f"{tag}: padding nibble"
    np.testing.assert_allclose(w_gpu, w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=f"{tag}: parameters")
    return flips


def run(rows, cols, steps, recipe="iid", bf16=False, seed=71, lr=LR, beta=BETA):
    P = rows * cols
    lpmm.ensure_init(4096)
    w_ref, st_ref = workloads.weights(seed, 0, rows, cols).reshape(-1), oracle.state_zero_sgdm(P)
    w, st = to_dev(w_ref.copy()), lpmm.new_state_sgdm(P, DEV)
    fn = lpmm.lpmm_sgdm4_step_bf16g if bf16 else lpmm.lpmm_sgdm4_step
    total = 0
    for t in range(1, steps + 1):
        g = workloads.grads(seed, 0, t, rows, cols, recipe, bf16).reshape(-1)
        mt = oracle.sgdm4_step(w_ref, g, st_ref, lr, beta, want_moment=True)
        fn(w, to_dev(g, bf16), st, lr, beta)
        torch.cuda.synchronize()
        total += compare(download(st), st_ref, w.cpu().numpy(), w_ref, mt, f"P={P} {recipe} step {t}")
    return total


def test_zero_state_matches_oracle():
    for P in (2, 130, 4096, 999):
        got, ref = download(lpmm.new_state_sgdm(P, DEV)), oracle.state_zero_sgdm(P)
        np.testing.assert_array_equal(got.m_codes, ref.m_codes)
        np.testing.assert_array_equal(got.m_scales, ref.m_scales)


@pytest.mark.parametrize("rows,cols", [(1, 128), (1, 4096), (1, 2), (1, 130), (1, 999), (3, 128 * 8 * 16),
                                       (1, 128 * 8 * 16 + 128 * 5), (7, 4099), (64, 1024)])
def test_step_parity(rows, cols):
    assert run(rows, cols, steps=4) == 0


def test_bf16_gradients_outliers_and_other_hyperparameters():
    assert run(256, 1536, steps=4, recipe="col_lognormal", bf16=True) == 0
    assert run(1200, 512, steps=5, recipe="outlier_sparse") == 0
    assert run(5, 128 * 40 + 64, steps=4, lr=1e-3, beta=0.0) == 0
    assert run(5, 128 * 40 + 64, steps=4, lr=0.5, beta=0.99) == 0


def test_long_run_stays_in_step():
    """200 steps with a gradient mean that persists and then dies away: a momentum buffer with a stable sign."""
    assert run(96, 256, steps=200, recipe="drift") == 0
    assert run(7, 333, steps=100, recipe="drift") == 0           # ragged last block


def test_fp32_momentum_step():
    rng = np.random.default_rng(72)
    P = 5000
    w_ref, m_ref = rng.standard_normal(P).astype(np.float32), np.zeros(P, np.float32)
    w, m = to_dev(w_ref.copy()), torch.zeros(P, device=DEV)
    for t in range(3):
        g = rng.standard_normal(P).astype(np.float32)
        oracle.sgdm32_step(w_ref, g, m_ref, LR, BETA)
        lpmm.lpmm_sgdm32_step(w, to_dev(g), m, P, 0, LR, BETA)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(m.cpu().numpy(), m_ref)
    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL)


@pytest.mark.parametrize("env", [{}, {"LPMM_PHASE_MPARAMS": "1"}], ids=["one-group", "many-groups"])
def test_plan_of_sgdm_tensors(env):
    seed = 73
    shapes = [(256, 384, True), (1, 128 * 300 + 20, True), (1, 512, False), (300, 1024, True), (37, 200, True)]
    os.environ.pop("LPMM_PHASE_MPARAMS", None)
    os.environ.update(env)
    try:
        lpmm.ensure_init(4096)
        dev, ref, descs = [], [], []
        for tid, (rows, cols, quant) in enumerate(shapes):
            P = rows * cols
            w_ref = workloads.weights(seed, tid, rows, cols).reshape(-1)
            w, g = to_dev(w_ref.copy()), torch.empty(P, device=DEV)
            if quant:
                st, st_ref = lpmm.new_state_sgdm(P, DEV), oracle.state_zero_sgdm(P)
                descs.append(lpmm.make_desc_sgdm(w, g, st))
            else:
                st, st_ref = torch.zeros(P, device=DEV), np.zeros(P, np.float32)
                descs.append(lpmm.make_desc_sgdm(w, g, st, P))
            dev.append((w, g, st))
            ref.append((w_ref, st_ref))
        plan = lpmm.new_plan(descs, 0, DEV)
        with pytest.raises(lpmm.LpmmError):           # an SGDM plan is not an AdamW plan
            lpmm.lpmm_adamw4_step_multi(plan, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1)
        for t in (1, 2, 3):
            grads = [workloads.grads(seed, tid, t, rows, cols, "col_lognormal").reshape(-1)
                     for tid, (rows, cols, _) in enumerate(shapes)]
            for (w, g, st), gn in zip(dev, grads):
                g.copy_(to_dev(gn))
            lpmm.lpmm_sgdm4_step_multi(plan, LR, BETA)
            torch.cuda.synchronize()
            for (rows, cols, quant), (w, g, st), (w_ref, st_ref), gn in zip(shapes, dev, ref, grads):
                tag = f"{rows}x{cols} step {t}"
                if quant:
                    mt = oracle.sgdm4_step(w_ref, gn, st_ref, LR, BETA, want_moment=True)
                    assert compare(download(st), st_ref, w.cpu().numpy(), w_ref, mt, tag) == 0
                else:
                    oracle.sgdm32_step(w_ref, gn, st_ref, LR, BETA)
                    np.testing.assert_array_equal(st.cpu().numpy(), st_ref, err_msg=tag)
                    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=tag)
        lpmm.lpmm_adamw4_plan_release(plan)
    finally:
        for k in env:
            os.environ.pop(k, None)


def test_plans_do_not_mix_optimizers_and_bad_arguments():
    lpmm.ensure_init(4096)
    w, g = torch.zeros(64 * 128, device=DEV), torch.zeros(64 * 128, device=DEV)
    d_sgdm = lpmm.make_desc_sgdm(w, g, lpmm.new_state_sgdm(64 * 128, DEV))
    d_adam = lpmm.make_desc(w, g, lpmm.new_state(64, 128, DEV))
    assert lpmm.lpmm_adamw4_plan_bytes([d_sgdm, d_adam]) == 0
    assert lpmm.lpmm_adamw4_plan_bytes([d_sgdm]) > 0
    plan = lpmm.new_plan([d_adam], 0, DEV)
    with pytest.raises(lpmm.LpmmError):
        lpmm.lpmm_sgdm4_step_multi(plan, LR, BETA)
    lpmm.lpmm_adamw4_plan_release(plan)
    st = lpmm.new_state_sgdm(1024, DEV)
    for lr, beta in ((-1.0, 0.9), (0.1, 1.0), (float("nan"), 0.5), (0.1, -0.1)):
        with pytest.raises(lpmm.LpmmError):
            lpmm.lpmm_sgdm4_step(w, g, st, lr, beta)
