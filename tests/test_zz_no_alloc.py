"""The entry point that allocates nothing (lpmm_adamw4_step_noalloc) against lpmm_adamw4_step / _step_bf16g on the
same inputs, through the C ABI: two calls in a row, the second on a smaller tensor, then the error path for a
tensor beyond the library's own scratch array.  The two entry points run the same kernels, so every output must
be identical bit for bit (integer state and parameters alike)."""
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


def _state_arrays(st):
    return [t.cpu().numpy().copy() for t in (st.m_codes, st.m_blockscale, st.v_codes, st.v_rowmax, st.v_colmax)]


def _run_pair(rows, cols, bf16, seed, steps):
    """The same steps through both entry points from the same start; returns nothing, asserts identity."""
    lpmm.ensure_init(rows + cols)
    w0 = workloads.weights(seed, 0, rows, cols).reshape(-1)
    w_a, w_b = to_dev(w0.copy()), to_dev(w0.copy())
    st_a, st_b = lpmm.new_state(rows, cols, DEV), lpmm.new_state(rows, cols, DEV)
    ref = lpmm.lpmm_adamw4_step_bf16g if bf16 else lpmm.lpmm_adamw4_step
    for t in range(1, steps + 1):
        g = to_dev(workloads.grads(seed, 0, t, rows, cols, "col_lognormal", bf16).reshape(-1), bf16)
        print(f"[gpu-test] noalloc {rows}x{cols} bf16={bf16} step {t}", flush=True)
        ref(w_a, g, st_a, HP.lr, HP.beta1, HP.beta2, HP.eps, HP.weight_decay, t)
        lpmm.lpmm_adamw4_step_noalloc(w_b, g, lpmm.GRAD_BF16 if bf16 else lpmm.GRAD_F32, st_b, HP.lr, HP.beta1,
                                      HP.beta2, HP.eps, HP.weight_decay, t)
        torch.cuda.synchronize()
        for name, a, b in zip(("m codes", "m block scales", "v codes", "row maxima", "column maxima"),
                              _state_arrays(st_a), _state_arrays(st_b)):
            np.testing.assert_array_equal(b, a, err_msg=f"{rows}x{cols} step {t}: {name}")
        np.testing.assert_array_equal(w_b.cpu().numpy(), w_a.cpu().numpy(), err_msg=f"{rows}x{cols} step {t}: parameters")
    assert bool((st_b.v_rowmax > 0).any()) and bool((st_b.m_blockscale > 0).any())     # not vacuous


def test_noalloc_step_equals_the_workspace_step_twice_in_a_row_second_call_smaller():
    _run_pair(1536, 1024, bf16=True, seed=41, steps=3)       # fast path, several tiles
    _run_pair(200, 384, bf16=False, seed=42, steps=3)        # smaller, fp32 gradients: the array holds the first call's leftovers
    _run_pair(77, 100, bf16=True, seed=43, steps=2)          # smaller again, general path (cols % 128 != 0)


def test_noalloc_step_rejects_sizes_beyond_its_array():
    lpmm.ensure_init(4096)
    L = lpmm.lib()
    shape = (ctypes.c_int64 * 2)(200000, 128)                # rows + cols beyond LPMM_NOALLOC_MAX_ROWS_PLUS_COLS
    dummy = torch.zeros(64, device=DEV)
    p = dummy.data_ptr()
    rc = L.lpmm_adamw4_step_noalloc(p, p, 0, p, p, p, p, p, ctypes.addressof(shape), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None)
    assert rc == -4                                          # LPMM_EWORKSPACE; nothing was enqueued
    assert b"workspace" in L.lpmm_strerror(rc)
    rc = L.lpmm_adamw4_step_noalloc(p, p, 7, p, p, p, p, p, ctypes.addressof(shape), 1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None)
    assert rc == -1                                          # unknown gradient type
    torch.cuda.synchronize()
