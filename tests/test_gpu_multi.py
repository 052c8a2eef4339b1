"""GPU parity tests of the multi-tensor step (one plan, a few launches for the whole parameter set)
against the CPU oracle run tensor by tensor."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, PARAM_ATOL, PARAM_RTOL, compare_step, download_state, to_dev

pytestmark = pytest.mark.gpu
HP = oracle.Hyper()


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-test] {request.node.name}", flush=True)
    yield
    torch.cuda.synchronize()


def _run_set(specs, recipe, bf16, steps, seed, env=None):
    """specs: list of workloads.TensorSpec.  Runs `steps` multi-tensor steps and the oracle side by side."""
    for k in ("LPMM_PHASE_MPARAMS", "LPMM_MULTI_RW", "LPMM_FLAT"):
        os.environ.pop(k, None)
    os.environ.update(env or {})
    try:
        lpmm.ensure_init(4096)
        dev_t, ref_t, descs = [], [], []
        for tid, sp in enumerate(specs):
            w_ref = workloads.weights(seed, tid, sp.rows, sp.cols).reshape(-1)
            w = to_dev(w_ref.copy())
            g = torch.empty(sp.numel, dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
            if sp.quantized:
                st, st_ref = lpmm.new_state(sp.rows, sp.cols, DEV), oracle.state_zero(sp.rows, sp.cols)
                descs.append(lpmm.make_desc(w, g, st))
            else:
                st = (torch.zeros(sp.numel, device=DEV), torch.zeros(sp.numel, device=DEV))
                st_ref = (np.zeros(sp.numel, np.float32), np.zeros(sp.numel, np.float32))
                descs.append(lpmm.make_desc(w, g, st, sp.rows, sp.cols))
            dev_t.append((w, g, st))
            ref_t.append((w_ref, st_ref))
        plan = lpmm.new_plan(descs, 1 if bf16 else 0, DEV)
        for t in range(1, steps + 1):
            grads = [workloads.grads(seed, tid, t, sp.rows, sp.cols, recipe, bf16).reshape(-1)
                     for tid, sp in enumerate(specs)]
            for (w, g, st), gn in zip(dev_t, grads):
                g.copy_(to_dev(gn, bf16))
            lpmm.lpmm_adamw4_step_multi(plan, HP.lr, HP.beta1, HP.beta2, HP.eps, HP.weight_decay, t)
            torch.cuda.synchronize()
            for sp, (w, g, st), (w_ref, st_ref), gn in zip(specs, dev_t, ref_t, grads):
                tag = f"{sp.name} {sp.rows}x{sp.cols} step {t}"
                if sp.quantized:
                    mt, vt = oracle.adamw4_step(w_ref, gn, st_ref, HP, t, want_moments=True)
                    assert compare_step(download_state(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, tag) == 0
                else:
                    oracle.adamw32_step(w_ref, gn, st_ref[0], st_ref[1], HP, t)
                    np.testing.assert_array_equal(st[0].cpu().numpy(), st_ref[0], err_msg=tag)
                    np.testing.assert_array_equal(st[1].cpu().numpy(), st_ref[1], err_msg=tag)
                    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=tag)
        lpmm.lpmm_adamw4_plan_release(plan)
    finally:
        for k in (env or {}):
            os.environ.pop(k, None)


def _mini_transformer():
    T = workloads.TensorSpec
    out = [T("embed", 1000, 256)]
    for l in range(3):
        out += [T(f"l{l}.qkv", 256, 768), T(f"l{l}.out", 256, 256), T(f"l{l}.fc1", 256, 1024),
                T(f"l{l}.fc2", 1024, 256), T(f"l{l}.b1", 1, 768, 1), T(f"l{l}.ln", 1, 256, 1)]
    out += [T("odd", 37, 200), T("head", 300, 384)]       # one tensor that takes the general path
    return out


@pytest.mark.parametrize("env", [{}, {"LPMM_PHASE_MPARAMS": "1"}, {"LPMM_PHASE_MPARAMS": "1", "LPMM_MULTI_RW": "8"},
                                 {"LPMM_PHASE_MPARAMS": "1", "LPMM_FLAT": "1"}, {"LPMM_FLAT": "1", "LPMM_MULTI_RW": "24"},
                                 {"LPMM_PHASE_MPARAMS": "1", "LPMM_MULTI_STREAMS": "1"},
                                 {"LPMM_PHASE_MPARAMS": "1", "LPMM_MULTI_STREAMS": "0"},
                                 {"LPMM_PHASE_MPARAMS": "1", "LPMM_MULTI_STREAMS": "3"}])
def test_multi_matches_oracle_fp32_grads(env):
    """Default grouping (everything in one group), and tiny groups so that many phases overlap
    pass 1 of one group with pass 2 of the previous one; the last three: both passes of a phase in one launch,
    every pass a launch of its own on the caller's stream, and pass 1 alternating between two streams."""
    _run_set(_mini_transformer(), "col_lognormal", False, steps=4, seed=11, env=env)


def test_multi_matches_oracle_bf16_grads():
    _run_set(_mini_transformer(), "col_lognormal", True, steps=4, seed=12, env={"LPMM_PHASE_MPARAMS": "1"})


def test_multi_single_tensor_plan():
    _run_set([workloads.TensorSpec("w", 512, 512)], "iid", False, steps=3, seed=13)


def test_multi_rejects_bad_lists():
    assert lpmm.lpmm_adamw4_plan_bytes([]) == 0
    bad = lpmm.TensorDesc(1, 1, 1, 1, 1, 1, 1, 0, 128, 0, 0)
    assert lpmm.lpmm_adamw4_plan_bytes([bad]) == 0
    with pytest.raises(lpmm.LpmmError):
        lpmm.lpmm_adamw4_step_multi(torch.zeros(256, dtype=torch.uint8, device=DEV), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1)


@pytest.mark.parametrize("second", ["rank1", "factor"])
def test_per_tensor_no_decay_flag(second):
    """Tensors flagged LPMM_FLAG_NO_DECAY (biases, normalization weights, here also one matrix) are stepped with
    weight decay 0, the others with the plan's."""
    import dataclasses
    from test_gpu_factor import compare as compare_factor, download as download_factor
    hp = oracle.Hyper(lr=1e-2, weight_decay=0.2)                  # large enough for a missing decay to show
    hp0 = dataclasses.replace(hp, weight_decay=0.0)
    T = workloads.TensorSpec
    specs = [(T("w1", 256, 384), False), (T("b1", 1, 384, 1), True), (T("w2", 300, 256), True),
             (T("ln", 1, 256, 1), True), (T("odd", 37, 200), False), (T("b2", 1, 300, 1), False)]
    lpmm.ensure_init(4096)
    seed = 17
    dev_t, ref_t, descs = [], [], []
    for tid, (sp, nd) in enumerate(specs):
        w_ref = workloads.weights(seed, tid, sp.rows, sp.cols).reshape(-1)
        w, g = to_dev(w_ref.copy()), torch.empty(sp.numel, device=DEV)
        if sp.quantized and second == "factor":
            st, st_ref = lpmm.new_state_factor(sp.rows, sp.cols, DEV), oracle.state_zero_factor(sp.rows, sp.cols)
            descs.append(lpmm.make_desc(w, g, st, no_decay=nd))
        elif sp.quantized:
            st, st_ref = lpmm.new_state(sp.rows, sp.cols, DEV), oracle.state_zero(sp.rows, sp.cols)
            descs.append(lpmm.make_desc(w, g, st, no_decay=nd))
        else:
            st = (torch.zeros(sp.numel, device=DEV), torch.zeros(sp.numel, device=DEV))
            st_ref = (np.zeros(sp.numel, np.float32), np.zeros(sp.numel, np.float32))
            descs.append(lpmm.make_desc(w, g, st, sp.rows, sp.cols, no_decay=nd))
        dev_t.append((w, g, st))
        ref_t.append((w_ref, st_ref))
    plan = lpmm.new_plan(descs, 0, DEV)
    for t in (1, 2, 3):
        grads = [workloads.grads(seed, tid, t, sp.rows, sp.cols, "col_lognormal").reshape(-1)
                 for tid, (sp, _) in enumerate(specs)]
        for (w, g, st), gn in zip(dev_t, grads):
            g.copy_(to_dev(gn))
        lpmm.lpmm_adamw4_step_multi(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)
        torch.cuda.synchronize()
        for (sp, nd), (w, g, st), (w_ref, st_ref), gn in zip(specs, dev_t, ref_t, grads):
            h = hp0 if nd else hp
            tag = f"{sp.name} step {t}"
            if sp.quantized and second == "factor":
                mt, _ = oracle.adamw4_factor_step(w_ref, gn, st_ref, h, t, want_moments=True)
                assert compare_factor(download_factor(st), st_ref, w.cpu().numpy(), w_ref, mt, tag) == 0
                st.v_row.copy_(to_dev(st_ref.v_row)); st.v_col.copy_(to_dev(st_ref.v_col)); w.copy_(to_dev(w_ref))
            elif sp.quantized:
                mt, vt = oracle.adamw4_step(w_ref, gn, st_ref, h, t, want_moments=True)
                assert compare_step(download_state(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, tag) == 0
            else:
                oracle.adamw32_step(w_ref, gn, st_ref[0], st_ref[1], h, t)
                np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=tag)
    lpmm.lpmm_adamw4_plan_release(plan)
    bad = lpmm.make_desc(dev_t[0][0], dev_t[0][1], dev_t[0][2])
    bad.flags = 6
    with pytest.raises(lpmm.LpmmError):
        lpmm.new_plan([bad], 0, DEV)


def test_plan_with_more_tensors_than_one_group_holds():
    """450 small tensors: more than the segment tables of one group hold, so the plan is cut by parameters into three
    groups of unequal tensor counts (the large tensors sit at the front); quantized and fp32-state tensors mixed."""
    T = workloads.TensorSpec
    rng = np.random.default_rng(77)
    specs = [T("big0", 300, 512), T("big1", 256, 640)]
    for k in range(448):
        if k % 3 == 2:
            specs.append(T(f"v{k}", 1, int(rng.integers(1, 9)) * 128, 1))
        else:
            specs.append(T(f"w{k}", int(rng.integers(33, 90)), 128 * int(rng.integers(1, 4))))
    _run_set(specs, "col_lognormal", True, steps=3, seed=77)
    _run_set(specs, "col_lognormal", False, steps=2, seed=78, env={"LPMM_MULTI_STREAMS": "0"})
