"""lpmm_adamw4_step_ws (the rank-1 step with a workspace of the caller's) through the C ABI: two tensors stepped on
two streams at the same time, each with its own workspace, against lpmm_adamw4_step / _step_bf16g run one after the
other on the same inputs.  The entry points run the same kernels, so every output must be identical bit for bit;
the reference entry point is the one the parity tests compare with the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu
HP = oracle.Hyper()
CASES = [(1536, 1024, True, 51), (640, 384, False, 52), (77, 100, True, 53)]      # fast path x2, general path


def _state_arrays(st):
    return [t.cpu().numpy().copy() for t in (st.m_codes, st.m_blockscale, st.v_codes, st.v_rowmax, st.v_colmax)]


def test_steps_on_two_streams_with_their_own_workspaces_equal_the_serial_steps():
    lpmm.ensure_init(4096)
    steps = 4
    tens = []
    for rows, cols, bf16, seed in CASES:
        w0 = workloads.weights(seed, 0, rows, cols).reshape(-1)
        gs = [to_dev(workloads.grads(seed, 0, t, rows, cols, "col_lognormal", bf16).reshape(-1), bf16)
              for t in range(1, steps + 1)]
        ws = torch.zeros(lpmm.lpmm_adamw4_workspace_bytes(rows + cols), dtype=torch.uint8, device=DEV)
        tens.append(dict(rows=rows, cols=cols, bf16=bf16, gs=gs, ws=ws,
                         w_ref=to_dev(w0.copy()), w=to_dev(w0.copy()),
                         st_ref=lpmm.new_state(rows, cols, DEV), st=lpmm.new_state(rows, cols, DEV)))
    # reference: one tensor after the other on the current stream, through the workspace of init
    lpmm.ensure_init(max(r + c for r, c, _, _ in CASES))
    for x in tens:
        ref = lpmm.lpmm_adamw4_step_bf16g if x["bf16"] else lpmm.lpmm_adamw4_step
        for t in range(1, steps + 1):
            ref(x["w_ref"], x["gs"][t - 1], x["st_ref"], HP.lr, HP.beta1, HP.beta2, HP.eps, HP.weight_decay, t)
    torch.cuda.synchronize()
    # the same steps, every tensor on a stream of its own with a workspace of its own, all in flight together
    streams = [torch.cuda.Stream(device=DEV) for _ in tens]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    print("[gpu-test] step_ws: %d tensors on %d streams, %d steps" % (len(tens), len(streams), steps), flush=True)
    for t in range(1, steps + 1):
        for x, s in zip(tens, streams):
            lpmm.lpmm_adamw4_step_ws(x["w"], x["gs"][t - 1], lpmm.GRAD_BF16 if x["bf16"] else lpmm.GRAD_F32, x["st"],
                                     HP.lr, HP.beta1, HP.beta2, HP.eps, HP.weight_decay, t, x["ws"], stream=s.cuda_stream)
    torch.cuda.synchronize()
    for x in tens:
        tag = "%dx%d" % (x["rows"], x["cols"])
        for name, a, b in zip(("m codes", "m block scales", "v codes", "row maxima", "column maxima"),
                              _state_arrays(x["st_ref"]), _state_arrays(x["st"])):
            np.testing.assert_array_equal(b, a, err_msg=f"{tag}: {name}")
        np.testing.assert_array_equal(x["w"].cpu().numpy(), x["w_ref"].cpu().numpy(), err_msg=f"{tag}: parameters")
        assert not bool(x["ws"].any())                                  # a completed step leaves its workspace zero-filled
        assert bool((x["st"].v_rowmax > 0).any()) and bool((x["st"].m_blockscale > 0).any())     # not vacuous


def test_step_ws_rejects_bad_workspaces():
    lpmm.ensure_init(4096)
    L = lpmm.lib()
    shape = (ctypes.c_int64 * 2)(4096, 4096)
    dummy = torch.zeros(16384, device=DEV)
    p = dummy.data_ptr()

    def call(ws, nbytes, dtype=0):
        return L.lpmm_adamw4_step_ws(p, p, dtype, p, p, p, p, p, ctypes.addressof(shape), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1,
                                     ws, nbytes, None)
    assert call(None, 1 << 20) == -1                                    # LPMM_EINVAL: no workspace
    assert call(p + 4, 1 << 20) == -1                                   # misaligned
    assert call(p, 4096) == -1                                          # smaller than the counters
    assert call(p, 8192 + 4096) == -4                                   # LPMM_EWORKSPACE: too small for 4096 + 4096
    assert call(p, 1 << 20, dtype=5) == -1                              # unknown gradient type
    torch.cuda.synchronize()
