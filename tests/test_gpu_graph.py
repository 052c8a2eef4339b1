"""The step entry points enqueue kernels only (no allocation, no memset, no synchronization), so a caller
can capture them into a HIP graph.  Each replay must equal the eager step bit for bit."""
import numpy as np
import pytest
import torch

import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu
H = (1e-3, 0.9, 0.999, 1e-8, 0.01)


def _states_equal(a, b):
    for name in vars(a):
        x, y = getattr(a, name), getattr(b, name)
        if torch.is_tensor(x):
            assert torch.equal(x, y), name


@pytest.mark.parametrize("kind", ["rank1", "b128", "sgdm", "nd"])
def test_single_tensor_step_replays_from_a_graph(kind):
    print(f"\n[gpu-test] graph capture {kind}", flush=True)
    rows, cols = 200, 512
    P = rows * cols
    lpmm.ensure_init(rows + cols)
    w0 = to_dev(workloads.weights(41, 0, rows, cols).reshape(-1))
    grads = [to_dev(workloads.grads(41, 0, t, rows, cols, "col_lognormal").reshape(-1)) for t in (1, 2, 3, 4)]

    def fresh():
        return {"rank1": lambda: lpmm.new_state(rows, cols, DEV), "b128": lambda: lpmm.new_state_b128(P, DEV),
                "sgdm": lambda: lpmm.new_state_sgdm(P, DEV), "nd": lambda: lpmm.new_state_nd((rows, 4, cols // 4), DEV)}[kind]()

    def step(w, g, st, t):
        if kind == "rank1":
            lpmm.lpmm_adamw4_step(w, g, st, *H, t)
        elif kind == "b128":
            lpmm.lpmm_adamw4_b128_step(w, g, st, *H, t)
        elif kind == "sgdm":
            lpmm.lpmm_sgdm4_step(w, g, st, 0.05, 0.9)
        else:
            lpmm.lpmm_adamw4_nd_step(w, g, st, *H, t)

    # eager reference; the captured call has its step number baked in, so the reference uses the same one
    w_ref, st_ref = w0.clone(), fresh()
    snaps = []
    for t, g in enumerate(grads, 1):
        step(w_ref, g, st_ref, 1)
        torch.cuda.synchronize()
        snaps.append(w_ref.clone())

    # capture one step reading a static gradient buffer, replay it with fresh gradients
    w, st = w0.clone(), fresh()
    g_static = torch.empty_like(grads[0])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            step(w, g_static, st, 1)
    torch.cuda.synchronize()
    for t, g in enumerate(grads, 1):
        g_static.copy_(g)
        torch.cuda.synchronize()            # eager work and synchronization between the replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(w, snaps[t - 1]), f"replay {t}"
    _states_equal(st, st_ref)


@pytest.mark.parametrize("env", [{}, {"LPMM_PHASE_MPARAMS": "1"}], ids=["one-stream", "two-streams"])
def test_plan_step_replays_from_a_graph(env):
    """The plan step too: with one group it is a few launches on the caller's stream, with several groups it
    forks to the plan's own stream and joins again before it returns, which a capture records as a fork/join."""
    import os
    print(f"\n[gpu-test] graph capture plan {env}", flush=True)
    T = workloads.TensorSpec
    specs = [T("a", 256, 768), T("b", 1024, 256), T("bias", 1, 768, 1), T("odd", 37, 200), T("c", 300, 384)]
    os.environ.update(env)
    try:
        lpmm.ensure_init(4096)

        def build():
            ts, descs = [], []
            for tid, sp in enumerate(specs):
                w = to_dev(workloads.weights(43, tid, sp.rows, sp.cols).reshape(-1))
                g = torch.zeros(sp.numel, device=DEV)
                if sp.quantized:
                    st = lpmm.new_state(sp.rows, sp.cols, DEV)
                    descs.append(lpmm.make_desc(w, g, st))
                    bufs = [getattr(st, n) for n in vars(st) if torch.is_tensor(getattr(st, n))]
                else:
                    st = (torch.zeros(sp.numel, device=DEV), torch.zeros(sp.numel, device=DEV))
                    descs.append(lpmm.make_desc(w, g, st, sp.rows, sp.cols))
                    bufs = list(st)
                ts.append((w, g, bufs, st))
            return ts, lpmm.new_plan(descs, 0, DEV)

        grads = [[to_dev(workloads.grads(43, tid, t, sp.rows, sp.cols, "col_lognormal").reshape(-1))
                  for tid, sp in enumerate(specs)] for t in (1, 2, 3)]
        ref, plan_ref = build()
        cap, plan_cap = build()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            with torch.cuda.graph(graph, stream=s):
                lpmm.lpmm_adamw4_step_multi(plan_cap, *H, 1)
        torch.cuda.synchronize()
        for gs in grads:
            for (w, g, _, _), (w2, g2, _, _), gn in zip(ref, cap, gs):
                g.copy_(gn)
                g2.copy_(gn)
            torch.cuda.synchronize()
            lpmm.lpmm_adamw4_step_multi(plan_ref, *H, 1)
            graph.replay()
            torch.cuda.synchronize()
            for sp, (w, _, bufs, _), (w2, _, bufs2, _) in zip(specs, ref, cap):
                assert torch.equal(w, w2), sp.name
                for x, y in zip(bufs, bufs2):
                    assert torch.equal(x, y), sp.name
        lpmm.lpmm_adamw4_plan_release(plan_ref)
        lpmm.lpmm_adamw4_plan_release(plan_cap)
    finally:
        for k in env:
            os.environ.pop(k, None)


@pytest.mark.parametrize("env", [{}, {"LPMM_PHASE_MPARAMS": "1"}], ids=["one-stream", "two-streams"])
def test_capturable_plan_step_follows_lr_and_step_on_the_device(env):
    """The capturable entry point reads the learning rate and the step number from device memory: one captured
    step, replayed while both change, must follow the eager steps with the same values (moments and their codes
    bit for bit; parameters to rounding: the bias corrections are evaluated on the device)."""
    import os
    print(f"\n[gpu-test] capturable plan step {env}", flush=True)
    T = workloads.TensorSpec
    specs = [T("a", 256, 768), T("b", 1024, 256), T("bias", 1, 768, 1), T("odd", 37, 200)]
    os.environ.update(env)
    try:
        lpmm.ensure_init(4096)

        def build():
            ts, descs = [], []
            for tid, sp in enumerate(specs):
                w = to_dev(workloads.weights(44, tid, sp.rows, sp.cols).reshape(-1))
                g = torch.zeros(sp.numel, device=DEV)
                if sp.quantized:
                    st = lpmm.new_state(sp.rows, sp.cols, DEV)
                    descs.append(lpmm.make_desc(w, g, st))
                    bufs = [getattr(st, n) for n in vars(st) if torch.is_tensor(getattr(st, n))]
                else:
                    st = (torch.zeros(sp.numel, device=DEV), torch.zeros(sp.numel, device=DEV))
                    descs.append(lpmm.make_desc(w, g, st, sp.rows, sp.cols))
                    bufs = list(st)
                ts.append((w, g, bufs))
            return ts, lpmm.new_plan(descs, 0, DEV)

        ref, plan_ref = build()
        cap, plan_cap = build()
        lr_dev = torch.zeros(1, device=DEV)
        step_dev = torch.zeros(1, dtype=torch.int64, device=DEV)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            with torch.cuda.graph(graph, stream=s):
                lpmm.lpmm_adamw4_step_multi_capturable(plan_cap, lr_dev, step_dev, 0.9, 0.999, 1e-8, 0.01)
        torch.cuda.synchronize()
        for t in (1, 2, 3, 4):
            lr = 1e-3 * (1.0 - 0.1 * t)                       # a schedule
            for tid, sp in enumerate(specs):
                gn = to_dev(workloads.grads(44, tid, t, sp.rows, sp.cols, "col_lognormal").reshape(-1))
                ref[tid][1].copy_(gn)
                cap[tid][1].copy_(gn)
            lr_dev.fill_(lr)
            step_dev.fill_(t)
            torch.cuda.synchronize()
            lpmm.lpmm_adamw4_step_multi(plan_ref, lr, 0.9, 0.999, 1e-8, 0.01, t)
            graph.replay()
            torch.cuda.synchronize()
            for sp, (w, _, bufs), (w2, _, bufs2) in zip(specs, ref, cap):
                torch.testing.assert_close(w2, w, rtol=1e-6, atol=1e-9, msg=f"{sp.name} step {t}")
                for x, y in zip(bufs, bufs2):
                    assert torch.equal(x, y), f"{sp.name} step {t}"
                w2.copy_(w)                                   # keep the two sides on identical parameters
        lpmm.lpmm_adamw4_plan_release(plan_ref)
        lpmm.lpmm_adamw4_plan_release(plan_cap)
    finally:
        for k in env:
            os.environ.pop(k, None)
