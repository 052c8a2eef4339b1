"""GPU parity tests of the step with a factorized second moment ("4-bit Factor", Sec. 4.3) against the
CPU oracle, element by element.

The first moment is integer work: block scales bit-exact, codes bit-exact up to flips within 2 ulp of a
decision boundary.  The row / column statistics are fp32 sums on the GPU (lane partial sums, LDS, float
atomics) against fp64 sums in the oracle: a sum of n non-negative terms taken in k levels of partial sums
is off by about sqrt(k) * 2^-24 relative; the test allows 2e-5.  A relative error e of the statistics moves
the update by e / 2 of lr * m_hat / sqrt(v_hat), far inside the parameter tolerance (1e-5 relative, 1e-7
absolute)."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, PARAM_ATOL, PARAM_RTOL, assert_codes_match, to_dev

pytestmark = pytest.mark.gpu
STAT_RTOL = 2e-5
KNOBS = ("LPMM_GX", "LPMM_RW", "LPMM_RW2", "LPMM_RS", "LPMM_RS2", "LPMM_FORCE_GENERAL", "LPMM_GEN_CHUNKS")


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-test] {request.node.name}", flush=True)
    yield
    torch.cuda.synchronize()


def upload(st: oracle.StateFactor) -> lpmm.StateFactor:
    return lpmm.StateFactor(st.rows, st.cols, to_dev(st.m_codes), to_dev(st.m_scales), to_dev(st.v_row),
                            to_dev(st.v_col))


def download(st: lpmm.StateFactor) -> oracle.StateFactor:
    f = lambda t: t.cpu().numpy().copy()
    return oracle.StateFactor(st.rows, st.cols, f(st.m_codes), f(st.m_blockscale), f(st.v_row), f(st.v_col))


def compare(got, ref, w_gpu, w_ref, mt, tag):
    np.testing.assert_array_equal(got.m_scales, ref.m_scales, err_msg=f"{tag}: m block scales")
    P = mt.size
    sm = np.repeat(ref.m_scales, 128)[:P]
    with np.errstate(invalid="ignore", divide="ignore"):
        n_m = np.where(sm > 0, mt / sm, np.float32(0)).astype(np.float32)
    flips = assert_codes_match(got.m_codes, ref.m_codes, n_m, oracle.step_table("de"), f"{tag}: m codes")
    if P & 1:
        assert got.m_codes[-1] >> 4 == 0, f"{tag}: padding nibble"
    np.testing.assert_allclose(got.v_row, ref.v_row, rtol=STAT_RTOL, atol=0, err_msg=f"{tag}: row statistics")
    np.testing.assert_allclose(got.v_col, ref.v_col, rtol=STAT_RTOL, atol=0, err_msg=f"{tag}: column statistics")
    np.testing.assert_allclose(w_gpu, w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=f"{tag}: parameters")
    return flips


def run(rows, cols, steps, recipe="col_lognormal", bf16=False, seed=51, hp=None, mutate_grad=None, env=None):
    hp = hp or oracle.Hyper()
    for k in KNOBS:
        os.environ.pop(k, None)
    os.environ.update(env or {})
    try:
        lpmm.ensure_init(max(rows + cols, 4096))
        w_ref = workloads.weights(seed, 0, rows, cols).reshape(-1)
        st_ref = oracle.state_zero_factor(rows, cols)
        w = to_dev(w_ref.copy())
        st = lpmm.new_state_factor(rows, cols, DEV)
        fn = lpmm.lpmm_adamw4_factor_step_bf16g if bf16 else lpmm.lpmm_adamw4_factor_step
        total = 0
        for t in range(1, steps + 1):
            g = workloads.grads(seed, 0, t, rows, cols, recipe, bf16).reshape(-1)
            if mutate_grad is not None:
                g = mutate_grad(g, t)
            mt, _ = oracle.adamw4_factor_step(w_ref, g, st_ref, hp, t, want_moments=True)
            fn(w, to_dev(g, bf16), st, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)
            torch.cuda.synchronize()
            flips = compare(download(st), st_ref, w.cpu().numpy(), w_ref, mt, f"{rows}x{cols} {recipe} step {t}")
            total += flips
            # carry the oracle's state forward on both sides, so that rounding differences of the statistics
            # (and a tolerated flip) do not compound over the steps
            st = upload(st_ref)
            w = to_dev(w_ref.copy())
        return total
    finally:
        for k in (env or {}):
            os.environ.pop(k, None)


def test_zero_state_matches_oracle():
    for rows, cols in ((1, 2), (3, 43), (32, 128), (7, 1000)):
        got, ref = download(lpmm.new_state_factor(rows, cols, DEV)), oracle.state_zero_factor(rows, cols)
        for a, b in ((got.m_codes, ref.m_codes), (got.m_scales, ref.m_scales), (got.v_row, ref.v_row),
                     (got.v_col, ref.v_col)):
            np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("rows,cols", [(64, 128), (300, 1024), (257, 384), (1, 4096), (3, 128), (5000, 128),
                                       (2, 1280), (150, 4096), (72, 2048), (100, 1024), (130, 11008)])
def test_step_parity_fast_path(rows, cols):
    # one tile, several tiles with ragged last tiles in both passes, an odd number of column blocks (the
    # statistics pass works on strips of two), single and few rows, tall and narrow, the row spacings
    assert run(rows, cols, steps=3) == 0


@pytest.mark.parametrize("rows,cols", [(37, 200), (5, 7), (1, 999), (1000, 3), (129, 127), (2, 4100), (700, 192),
                                       (9, 2100), (40000, 3), (2000, 9)])
def test_step_parity_general_path(rows, cols):
    assert run(rows, cols, steps=3) == 0


def test_bf16_gradients():
    assert run(256, 1536, steps=4, bf16=True) == 0
    assert run(50, 333, steps=3, bf16=True) == 0


def test_long_run_stays_in_step():
    """150 steps with a gradient mean that persists and then dies away, fast and general path."""
    assert run(192, 256, steps=150, recipe="drift") == 0
    assert run(37, 200, steps=100, recipe="drift") == 0


def test_outliers_and_zero_rows():
    # most rows zero in a step (their statistic only decays), a few rows and columns 1000x larger
    assert run(1200, 512, steps=5, recipe="outlier_sparse") == 0


@pytest.mark.parametrize("hp", [oracle.Hyper(lr=3e-3, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1),
                                oracle.Hyper(lr=1e-4, beta1=0.0, beta2=0.5, eps=1e-12, weight_decay=0.0)])
def test_other_hyperparameters(hp):
    assert run(96, 640, steps=4, hp=hp) == 0


def test_zero_gradient_from_the_zero_state():
    # all statistics stay 0: the reconstruction is defined as 0 there, nothing may turn into NaN
    assert run(40, 256, steps=2, mutate_grad=lambda g, t: np.zeros_like(g)) == 0
    assert run(9, 50, steps=2, mutate_grad=lambda g, t: np.zeros_like(g)) == 0


@pytest.mark.parametrize("env", [{"LPMM_GX": "8", "LPMM_RW": "16"}, {"LPMM_GX": "2", "LPMM_RW": "300", "LPMM_RW2": "7"},
                                 {"LPMM_RS": "0", "LPMM_RS2": "0", "LPMM_RW2": "1000"},
                                 {"LPMM_RW": "64", "LPMM_RS": "3", "LPMM_RW2": "32", "LPMM_RS2": "3"},
                                 {"LPMM_RW": "40", "LPMM_RS": "2", "LPMM_RW2": "24", "LPMM_RS2": "1"},
                                 {"LPMM_FORCE_GENERAL": "1"}, {"LPMM_FORCE_GENERAL": "1", "LPMM_GEN_CHUNKS": "1"},
                                 {"LPMM_FORCE_GENERAL": "1", "LPMM_GEN_CHUNKS": "16"}])
def test_other_launch_geometries(env):
    assert run(300, 1024, steps=3, env=env) == 0


def test_first_moment_does_not_depend_on_the_launch_geometry():
    """The sums' order changes with the tiling, the first moment's bits must not."""
    rows, cols = 300, 1024
    lpmm.ensure_init(4096)
    w0 = workloads.weights(52, 0, rows, cols).reshape(-1)
    grads = [workloads.grads(52, 0, t, rows, cols, "col_lognormal").reshape(-1) for t in (1, 2, 3)]
    outs = []
    try:
        for env in ({}, {"LPMM_GX": "4", "LPMM_RW": "24", "LPMM_RW2": "12"}, {"LPMM_FORCE_GENERAL": "1"}):
            for k in KNOBS:
                os.environ.pop(k, None)
            os.environ.update(env)
            w, st = to_dev(w0.copy()), lpmm.new_state_factor(rows, cols, DEV)
            for t, g in enumerate(grads, 1):
                lpmm.lpmm_adamw4_factor_step(w, to_dev(g), st, 1e-3, 0.9, 0.999, 1e-8, 0.01, t)
            torch.cuda.synchronize()
            outs.append((download(st), w.cpu().numpy()))
    finally:
        for k in KNOBS:
            os.environ.pop(k, None)
    for st, w in outs[1:]:
        np.testing.assert_array_equal(st.m_codes, outs[0][0].m_codes)
        np.testing.assert_array_equal(st.m_scales, outs[0][0].m_scales)
        np.testing.assert_allclose(st.v_row, outs[0][0].v_row, rtol=STAT_RTOL)
        np.testing.assert_allclose(st.v_col, outs[0][0].v_col, rtol=STAT_RTOL)
        np.testing.assert_allclose(w, outs[0][1], rtol=PARAM_RTOL, atol=PARAM_ATOL)


def test_workspace_is_left_clean_for_the_other_steps():
    """The factorized step and the rank-1 step share the device workspace; each must leave it zeroed."""
    from gpu_util import compare_step, download_state, gpu_step
    rows, cols = 200, 512
    hp = oracle.Hyper()
    lpmm.ensure_init(4096)
    wf_ref, sf_ref = workloads.weights(53, 0, rows, cols).reshape(-1), oracle.state_zero_factor(rows, cols)
    wr_ref, sr_ref = workloads.weights(53, 1, rows, cols).reshape(-1), oracle.state_zero(rows, cols)
    wf, sf = to_dev(wf_ref.copy()), lpmm.new_state_factor(rows, cols, DEV)
    wr, sr = to_dev(wr_ref.copy()), lpmm.new_state(rows, cols, DEV)
    for t in (1, 2, 3):
        g = workloads.grads(53, 0, t, rows, cols, "col_lognormal").reshape(-1)
        mt, _ = oracle.adamw4_factor_step(wf_ref, g, sf_ref, hp, t, want_moments=True)
        lpmm.lpmm_adamw4_factor_step(wf, to_dev(g), sf, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)
        mt2, vt2 = oracle.adamw4_step(wr_ref, g, sr_ref, hp, t, want_moments=True)
        gpu_step(wr, to_dev(g), sr, hp, t)
        torch.cuda.synchronize()
        assert compare(download(sf), sf_ref, wf.cpu().numpy(), wf_ref, mt, f"factor step {t}") == 0
        assert compare_step(download_state(sr), sr_ref, wr.cpu().numpy(), wr_ref, mt2, vt2, f"rank-1 step {t}") == 0
        sf, wf = upload(sf_ref), to_dev(wf_ref.copy())


def test_bad_arguments_are_rejected():
    rows, cols = 8, 128
    lpmm.ensure_init(4096)
    w, g = torch.zeros(rows * cols, device=DEV), torch.zeros(rows * cols, device=DEV)
    st = lpmm.new_state_factor(rows, cols, DEV)
    L = lpmm.lib()
    import ctypes
    shape = (ctypes.c_int64 * 2)(rows, cols)
    args = lambda **kw: [kw.get("p", w.data_ptr()), kw.get("g", g.data_ptr()), st.m_codes.data_ptr(),
                         st.m_blockscale.data_ptr(), kw.get("r", st.v_row.data_ptr()), st.v_col.data_ptr(),
                         ctypes.addressof(kw.get("shape", shape)), kw.get("lr", 1e-3), 0.9, kw.get("b2", 0.999), 1e-8,
                         0.0, kw.get("t", 1), None]
    assert L.lpmm_adamw4_factor_step(*args()) == 0
    assert L.lpmm_adamw4_factor_step(*args(p=None)) != 0
    assert L.lpmm_adamw4_factor_step(*args(r=None)) != 0
    assert L.lpmm_adamw4_factor_step(*args(g=g.data_ptr() + 4)) != 0
    assert L.lpmm_adamw4_factor_step(*args(t=0)) != 0
    assert L.lpmm_adamw4_factor_step(*args(b2=1.0)) != 0
    assert L.lpmm_adamw4_factor_step(*args(shape=(ctypes.c_int64 * 2)(0, cols))) != 0
    big = (ctypes.c_int64 * 2)(1 << 31, 128)          # rows + cols beyond any registered workspace
    assert L.lpmm_adamw4_factor_step(*args(shape=big)) != 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("env", [{}, {"LPMM_PHASE_MPARAMS": "1", "LPMM_MULTI_STREAMS": "2"},
                                 {"LPMM_PHASE_MPARAMS": "1", "LPMM_MULTI_STREAMS": "1"}, {"LPMM_PHASE_MPARAMS": "1"}],
                         ids=["one-group", "two-streams", "fused-launches", "serial-launches"])
def test_plan_with_factorized_block_wise_and_fp32_tensors(env):
    """A "4-bit Factor" parameter set in one plan: matrices factorized, a large 1-dimensional tensor
    block-wise, small ones with fp32 states."""
    from test_gpu_b128 import compare as compare_b128, download as download_b128
    hp = oracle.Hyper()
    seed = 54
    shapes = [("w1", 256, 384, "factor"), ("flat", 1, 128 * 300 + 20, "b128"), ("ln", 1, 512, "fp32"),
              ("w2", 300, 1024, "factor"), ("odd", 37, 200, "factor"), ("w3", 1024, 256, "factor")]
    for k in ("LPMM_PHASE_MPARAMS", "LPMM_MULTI_STREAMS"):
        os.environ.pop(k, None)
    os.environ.update(env)
    try:
        lpmm.ensure_init(4096)
        dev, ref, descs = [], [], []
        for tid, (name, rows, cols, kind) in enumerate(shapes):
            P = rows * cols
            w_ref = workloads.weights(seed, tid, rows, cols).reshape(-1)
            w, g = to_dev(w_ref.copy()), torch.empty(P, dtype=torch.float32, device=DEV)
            if kind == "factor":
                st, st_ref = lpmm.new_state_factor(rows, cols, DEV), oracle.state_zero_factor(rows, cols)
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
        for t in (1, 2, 3):
            grads = [workloads.grads(seed, tid, t, rows, cols, "col_lognormal").reshape(-1)
                     for tid, (_, rows, cols, _) in enumerate(shapes)]
            for (w, g, st), gn in zip(dev, grads):
                g.copy_(to_dev(gn))
            lpmm.lpmm_adamw4_step_multi(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)
            torch.cuda.synchronize()
            for (name, rows, cols, kind), (w, g, st), (w_ref, st_ref), gn in zip(shapes, dev, ref, grads):
                tag = f"{name} step {t}"
                if kind == "factor":
                    mt, _ = oracle.adamw4_factor_step(w_ref, gn, st_ref, hp, t, want_moments=True)
                    assert compare(download(st), st_ref, w.cpu().numpy(), w_ref, mt, tag) == 0
                    # carry the oracle's values forward (in place: the plan refers to these buffers)
                    st.v_row.copy_(to_dev(st_ref.v_row))
                    st.v_col.copy_(to_dev(st_ref.v_col))
                    w.copy_(to_dev(w_ref))
                elif kind == "b128":
                    mt, vt = oracle.adamw4_b128_step(w_ref, gn, st_ref, hp, t, want_moments=True)
                    assert compare_b128(download_b128(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, tag) == 0
                else:
                    oracle.adamw32_step(w_ref, gn, st_ref[0], st_ref[1], hp, t)
                    np.testing.assert_array_equal(st[0].cpu().numpy(), st_ref[0], err_msg=tag)
                    np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=tag)
        lpmm.lpmm_adamw4_plan_release(plan)
    finally:
        for k in env:
            os.environ.pop(k, None)


def test_plan_rejects_rank1_and_factorized_tensors_together():
    lpmm.ensure_init(4096)
    w, g = torch.zeros(64 * 128, device=DEV), torch.zeros(64 * 128, device=DEV)
    d1 = lpmm.make_desc(w, g, lpmm.new_state(64, 128, DEV))
    d2 = lpmm.make_desc(w, g, lpmm.new_state_factor(64, 128, DEV))
    assert lpmm.lpmm_adamw4_plan_bytes([d1, d2]) == 0
    assert lpmm.lpmm_adamw4_plan_bytes([d2]) > 0


DET_STAT_RTOL = 2e-6      # fixed-order fp32 sums against fp64: about sqrt(levels) * 2^-24, observed below 1e-6


@pytest.mark.parametrize("bf16", [False, True])
def test_deterministic_sums_are_reproducible_and_match_the_oracle(bf16):
    """LPMM_FLAG_DETERMINISTIC: the same plan step on the same inputs twice gives identical bits in R, C and the
    parameters (float atomics do not), on all three launch routes, and stays within 2e-6 of the oracle's fp64
    statistics over several free-running steps.  Shapes: several row tiles of 128 with a ragged last one, an odd
    number of column blocks, a single row tile, 11008 columns."""
    hp = oracle.Hyper()
    shapes = [(300, 1024), (257, 384), (64, 128), (130, 11008), (1000, 4096)]
    for streams, mparams in (("2", "1"), ("1", "1"), ("2", "2048")):
        os.environ["LPMM_MULTI_STREAMS"], os.environ["LPMM_PHASE_MPARAMS"] = streams, mparams
        try:
            runs = []
            for rep in range(2):
                lpmm.ensure_init(4096)
                keep, descs, refs = [], [], []
                for tid, (rows, cols) in enumerate(shapes):
                    w_ref = workloads.weights(61, tid, rows, cols).reshape(-1)
                    w = to_dev(w_ref.copy())
                    g = torch.empty(rows * cols, dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)
                    st = lpmm.new_state_factor(rows, cols, DEV)
                    descs.append(lpmm.make_desc(w, g, st, deterministic=True))
                    keep.append((w, g, st))
                    refs.append((w_ref, oracle.state_zero_factor(rows, cols)))
                if rep == 0:
                    refs0 = refs                     # the oracle runs once, beside the first repetition
                plan = lpmm.new_plan(descs, 1 if bf16 else 0, DEV)
                out = []
                for t in range(1, 5):
                    for tid, ((rows, cols), (w, g, st), (w_ref, st_ref)) in enumerate(zip(shapes, keep, refs)):
                        gn = workloads.grads(61, tid, t, rows, cols, "col_lognormal", bf16).reshape(-1)
                        g.copy_(to_dev(gn, bf16))
                        if rep == 0:
                            oracle.adamw4_factor_step(w_ref, gn, st_ref, hp, t)
                    lpmm.lpmm_adamw4_step_multi(plan, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)
                    torch.cuda.synchronize()
                    out.append([(w.clone(), st.v_row.clone(), st.v_col.clone(), st.m_codes.clone()) for w, g, st in keep])
                lpmm.lpmm_adamw4_plan_release(plan)
                runs.append(out)
            for t, (a, b) in enumerate(zip(*runs), start=1):
                for (shape, xa, xb) in zip(shapes, a, b):
                    for name, ta, tb in zip(("parameters", "R", "C", "m codes"), xa, xb):
                        assert torch.equal(ta, tb), f"{shape} step {t}: {name} differ between two identical runs"
            # free-running against the oracle (the statistics' rounding compounds through beta2 only)
            for (rows, cols), (w, R, C, mq), (w_ref, st_ref) in zip(shapes, runs[0][-1], refs0):
                np.testing.assert_allclose(R.cpu().numpy(), st_ref.v_row, rtol=DET_STAT_RTOL, atol=0, err_msg=f"{rows}x{cols}: R")
                np.testing.assert_allclose(C.cpu().numpy(), st_ref.v_col, rtol=DET_STAT_RTOL, atol=0, err_msg=f"{rows}x{cols}: C")
                np.testing.assert_allclose(w.cpu().numpy(), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=f"{rows}x{cols}: parameters")
        finally:
            os.environ.pop("LPMM_MULTI_STREAMS", None)
            os.environ.pop("LPMM_PHASE_MPARAMS", None)


def test_deterministic_flag_is_refused_where_it_does_not_apply():
    lpmm.ensure_init(4096)
    w = torch.zeros(64 * 100, device=DEV)
    g = torch.zeros_like(w)
    with pytest.raises(lpmm.LpmmError):          # general path (cols % 128 != 0)
        lpmm.new_plan([lpmm.make_desc(w, g, lpmm.new_state_factor(64, 100, DEV), deterministic=True)], 0, DEV)
    w = torch.zeros(64 * 128, device=DEV)
    g = torch.zeros_like(w)
    with pytest.raises(lpmm.LpmmError):          # rank-1 tensor
        lpmm.new_plan([lpmm.make_desc(w, g, lpmm.new_state(64, 128, DEV), deterministic=True)], 0, DEV)
