"""The torch.optim-style front ends drive the same C ABI: their results must equal the oracle's, tensor by tensor,
and the first step of 4-bit AdamW must equal torch's fp32 AdamW (the update uses the precise moments)."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
from gpu_util import DEV, PARAM_ATOL, PARAM_RTOL, compare_step, download_state
from test_gpu_sgdm import compare as compare_sgdm, download as download_sgdm

pytestmark = pytest.mark.gpu


def _model(seed):
    torch.manual_seed(seed)
    m = torch.nn.Sequential(torch.nn.Linear(256, 384), torch.nn.LayerNorm(384), torch.nn.GELU(),
                            torch.nn.Linear(384, 130), torch.nn.Linear(130, 8))
    return m.to(DEV)


def _loss(m, step):
    g = torch.Generator(device="cpu").manual_seed(1000 + step)
    x = torch.randn(32, 256, generator=g).to(DEV)
    return (m(x) ** 2).mean()


def test_adamw4bit_matches_the_oracle_and_survives_moving_gradients():
    print("\n[gpu-test] AdamW4bit front end", flush=True)
    hp = oracle.Hyper(lr=1e-3, weight_decay=0.1)
    m = _model(1)
    opt = lpmm.AdamW4bit(m.parameters(), lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps, weight_decay=hp.weight_decay)
    ref = []
    for p in m.parameters():
        w = p.detach().cpu().numpy().reshape(-1).copy()
        if p.numel() > 4096 and p.ndim == 2:
            ref.append((w, oracle.state_zero(p.shape[0], p.shape[1])))
        else:
            ref.append((w, (np.zeros(p.numel(), np.float32), np.zeros(p.numel(), np.float32))))
    for t in (1, 2, 3, 4):
        _loss(m, t).backward()
        grads = [p.grad.detach().cpu().numpy().reshape(-1).copy() for p in m.parameters()]
        opt.step()
        torch.cuda.synchronize()
        for p, st, (w_ref, st_ref), g in zip(m.parameters(), opt.state_buffers(), ref, grads):
            h = dataclasses.replace(hp, weight_decay=0.0) if p.ndim <= 1 else hp
            if isinstance(st_ref, tuple):
                oracle.adamw32_step(w_ref, g, st_ref[0], st_ref[1], h, t)
                np.testing.assert_allclose(p.detach().cpu().numpy().reshape(-1), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL)
            else:
                mt, vt = oracle.adamw4_step(w_ref, g, st_ref, h, t, want_moments=True)
                assert compare_step(download_state(st), st_ref, p.detach().cpu().numpy().reshape(-1), w_ref, mt, vt,
                                    f"{tuple(p.shape)} step {t}") == 0
            # both sides continue from the oracle's parameters: the next gradient must be the same on both
            p.data.copy_(torch.from_numpy(w_ref).view_as(p))
        opt.zero_grad(set_to_none=(t % 2 == 0))           # every other step the gradients get new addresses


def test_first_step_equals_fp32_adamw():
    print("\n[gpu-test] AdamW4bit step 1 vs torch.optim.AdamW", flush=True)
    a, b = _model(2), _model(2)
    decay = [p for p in b.parameters() if p.ndim > 1]
    no_decay = [p for p in b.parameters() if p.ndim <= 1]
    ref = torch.optim.AdamW([{"params": decay, "weight_decay": 0.05}, {"params": no_decay, "weight_decay": 0.0}],
                            lr=2e-3, betas=(0.9, 0.98), eps=1e-6)
    for second in ("rank1", "factor", "b128"):
        a.load_state_dict(_model(2).state_dict())
        opt = lpmm.AdamW4bit(a.parameters(), lr=2e-3, betas=(0.9, 0.98), eps=1e-6, weight_decay=0.05, second_moment=second)
        _loss(a, 7).backward()
        opt.step()
        if second == "rank1":
            _loss(b, 7).backward()
            ref.step()
        torch.cuda.synchronize()
        for pa, pb in zip(a.parameters(), b.parameters()):
            if second == "factor" and pa.ndim == 2 and pa.numel() > 4096:
                continue                                   # the factorized second moment is an approximation
            torch.testing.assert_close(pa, pb, rtol=2e-5, atol=2e-7)
        opt.zero_grad(set_to_none=True)


def test_sgdm4bit_matches_the_oracle():
    print("\n[gpu-test] SGDM4bit front end", flush=True)
    lr, beta = 0.05, 0.9
    m = _model(3)
    opt = lpmm.SGDM4bit(m.parameters(), lr=lr, momentum=beta)
    ref = [(p.detach().cpu().numpy().reshape(-1).copy(),
            oracle.state_zero_sgdm(p.numel()) if p.numel() > 4096 else np.zeros(p.numel(), np.float32))
           for p in m.parameters()]
    for t in (1, 2, 3):
        _loss(m, t).backward()
        grads = [p.grad.detach().cpu().numpy().reshape(-1).copy() for p in m.parameters()]
        opt.step()
        torch.cuda.synchronize()
        for p, st, (w_ref, st_ref), g in zip(m.parameters(), opt.state_buffers(), ref, grads):
            if isinstance(st_ref, np.ndarray):
                oracle.sgdm32_step(w_ref, g, st_ref, lr, beta)
                np.testing.assert_allclose(p.detach().cpu().numpy().reshape(-1), w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL)
            else:
                mt = oracle.sgdm4_step(w_ref, g, st_ref, lr, beta, want_moment=True)
                assert compare_sgdm(download_sgdm(st), st_ref, p.detach().cpu().numpy().reshape(-1), w_ref, mt,
                                    f"{tuple(p.shape)} step {t}") == 0
            p.data.copy_(torch.from_numpy(w_ref).view_as(p))
        opt.zero_grad()


def test_bad_parameters_are_rejected():
    with pytest.raises(ValueError):
        lpmm.AdamW4bit([torch.zeros(4, 4, device=DEV, dtype=torch.float16, requires_grad=True)])
    with pytest.raises(ValueError):
        lpmm.AdamW4bit([torch.zeros(4, 4, requires_grad=True)])          # not on the GPU
    opt = lpmm.AdamW4bit([torch.zeros(64, 128, device=DEV, requires_grad=True)])
    with pytest.raises(ValueError):
        opt.step()                                                       # no gradient yet


def test_adamw4bit_with_a_convolution_weight():
    """A 4-dimensional parameter takes the rank-1 second moment over all its dimensions (App. F Alg. 4)."""
    import test_gpu_rank1_nd as tn
    print("\n[gpu-test] AdamW4bit with a conv weight", flush=True)
    hp = oracle.Hyper(lr=1e-3, weight_decay=0.05)
    torch.manual_seed(5)
    conv = torch.nn.Conv2d(16, 64, 3).to(DEV)
    opt = lpmm.AdamW4bit(conv.parameters(), lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps, weight_decay=hp.weight_decay)
    shape = tuple(conv.weight.shape)
    w_ref = conv.weight.detach().cpu().numpy().reshape(-1).copy()
    st_ref = oracle.state_zero_nd(shape)
    for t in (1, 2, 3):
        g = torch.Generator(device="cpu").manual_seed(2000 + t)
        x = torch.randn(4, 16, 12, 12, generator=g).to(DEV)
        (conv(x) ** 2).mean().backward()
        gw = conv.weight.grad.detach().cpu().numpy().reshape(-1).copy()
        opt.step()
        torch.cuda.synchronize()
        mt, vt = oracle.adamw4_nd_step(w_ref, gw, st_ref, hp, t, want_moments=True)
        st = opt.state_buffers()[0]
        assert isinstance(st, lpmm.StateND)
        got, inner = tn.download(st)
        np.testing.assert_array_equal(inner, st_ref.v_stats[shape[0]:])
        assert compare_step(got, tn.as_matrix_state(st_ref), conv.weight.detach().cpu().numpy().reshape(-1), w_ref, mt, vt,
                            f"conv step {t}") == 0
        conv.weight.data.copy_(torch.from_numpy(w_ref).view_as(conv.weight))
        opt.zero_grad()


def test_capturable_optimizer_step_in_a_graph():
    """opt.step() of a capturable AdamW4bit captured once and replayed equals the eager optimizer step for step."""
    print("\n[gpu-test] capturable AdamW4bit in a graph", flush=True)
    a, b = _model(6), _model(6)
    oa = lpmm.AdamW4bit(a.parameters(), lr=1e-3, weight_decay=0.05, capturable=True)
    ob = lpmm.AdamW4bit(b.parameters(), lr=1e-3, weight_decay=0.05)
    for m, o in ((a, oa), (b, ob)):                      # one eager step each: builds the plans, gradients stay in place
        _loss(m, 0).backward()
        o.step()
        o.zero_grad()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            oa.step()
    torch.cuda.synchronize()
    oa.t -= 1                                             # the capture ran nothing on the device; undo the host-side count
    for t in (1, 2, 3):
        lr = 1e-3 / (1 + t)
        oa.set_lr(lr)
        ob.set_lr(lr)
        for m in (a, b):
            for p in m.parameters():
                p.grad.zero_()
            _loss(m, t).backward()
        torch.cuda.synchronize()
        graph.replay()
        ob.step()
        torch.cuda.synchronize()
        for pa, pb in zip(a.parameters(), b.parameters()):
            torch.testing.assert_close(pa, pb, rtol=1e-6, atol=1e-9)
            pa.data.copy_(pb.data)
    # the replays advanced the step count on the device only: a checkpoint must carry that count
    assert oa.state_dict()["t"] == ob.state_dict()["t"] == 4
    c = _model(7)
    c.load_state_dict({k: v.clone() for k, v in a.state_dict().items()})
    oc = lpmm.AdamW4bit(c.parameters(), lr=1e-3, weight_decay=0.05, capturable=True)
    oc.load_state_dict(oa.state_dict())
    oc.set_lr(2e-4)
    ob.set_lr(2e-4)
    for m, o in ((c, oc), (b, ob)):                      # step 5 in both: same bias corrections, same result
        for p in m.parameters():
            p.grad = None
        _loss(m, 4).backward()
        o.step()
    torch.cuda.synchronize()
    assert int(oc.step_dev.item()) == 5
    for pc, pb in zip(c.parameters(), b.parameters()):
        torch.testing.assert_close(pc, pb, rtol=1e-6, atol=1e-9)


def test_state_dict_round_trip_resumes_bit_for_bit():
    """6 steps == 3 steps, state_dict into a fresh optimizer, 3 more steps."""
    print("\n[gpu-test] AdamW4bit state_dict", flush=True)

    def run(m, opt, steps):
        for t in steps:
            _loss(m, t).backward()
            opt.step()
            opt.zero_grad()

    a = _model(8)
    oa = lpmm.AdamW4bit(a.parameters(), lr=1e-3)
    run(a, oa, range(1, 7))
    b = _model(8)
    ob = lpmm.AdamW4bit(b.parameters(), lr=1e-3)
    run(b, ob, range(1, 4))
    sd, weights = ob.state_dict(), {k: v.clone() for k, v in b.state_dict().items()}
    c = _model(9)                                         # other initial weights: everything must come from the checkpoint
    c.load_state_dict(weights)
    oc = lpmm.AdamW4bit(c.parameters(), lr=1e-3)
    oc.load_state_dict(sd)
    run(c, oc, range(4, 7))
    torch.cuda.synchronize()
    for pa, pc in zip(a.parameters(), c.parameters()):
        assert torch.equal(pa, pc)
    with pytest.raises(ValueError):
        lpmm.AdamW4bit(_model(8).parameters(), second_moment="b128").load_state_dict(sd)
