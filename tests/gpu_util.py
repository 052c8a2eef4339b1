"""Helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same seeded inputs and
compare state element by element."""
import numpy as np
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads

DEV = "cuda:0"

# Tolerances of the parity bar: integer state bit-exact (flips tolerated only within 2 ulp of a
# decision boundary, at most 1e-6 of the elements); parameters 1e-5 relative / 1e-7 absolute per step.
PARAM_RTOL, PARAM_ATOL = 1e-5, 1e-7
MAX_FLIP_FRACTION = 1e-6


def to_dev(a: np.ndarray, bf16: bool = False):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    if bf16:
        t = t.to(torch.bfloat16)       # values were already rounded to bf16: this cast is exact
    return t


def upload_state(st: oracle.State4) -> lpmm.State4:
    return lpmm.State4(st.rows, st.cols, to_dev(st.m_codes), to_dev(st.m_scales), to_dev(st.v_codes),
                       to_dev(st.v_r), to_dev(st.v_c))


def download_state(st: lpmm.State4) -> oracle.State4:
    f = lambda t: t.cpu().numpy().copy()
    return oracle.State4(st.rows, st.cols, f(st.m_codes), f(st.m_blockscale), f(st.v_codes),
                         f(st.v_rowmax), f(st.v_colmax))


def gpu_step(w, g, st: lpmm.State4, hp: oracle.Hyper, t: int, bf16: bool = False):
    fn = lpmm.lpmm_adamw4_step_bf16g if bf16 else lpmm.lpmm_adamw4_step
    fn(w, g, st, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, t)


def _ulp_distance_to_boundary(n: np.ndarray, T: np.ndarray) -> np.ndarray:
    """Distance of each fp32 n to the nearest decision boundary (midpoint of neighbouring table
    entries), in units of ulp(n)."""
    mids = (T[:-1].astype(np.float64) + T[1:].astype(np.float64)) / 2
    d = np.abs(n.astype(np.float64)[:, None] - mids[None, :]).min(axis=1)
    return d / np.spacing(np.abs(n).astype(np.float32)).astype(np.float64)


def assert_codes_match(got: np.ndarray, want: np.ndarray, n_values: np.ndarray, T: np.ndarray, what: str):
    """Codes must be identical; a differing code is tolerated only if the normalized value the oracle
    quantized lies within 2 ulp of a decision boundary, and such flips stay below 1e-6 of all."""
    P = n_values.size
    a, b = oracle.unpack_codes(got, P), oracle.unpack_codes(want, P)
    bad = np.nonzero(a != b)[0]
    if bad.size == 0:
        return 0
    dist = _ulp_distance_to_boundary(n_values[bad], T)
    assert np.all(dist <= 2.0), f"{what}: {np.sum(dist > 2.0)} code mismatches away from any boundary " \
                                f"(first at {bad[np.argmax(dist > 2.0)]})"
    assert np.all(np.abs(a[bad].astype(int) - b[bad].astype(int)) == 1), f"{what}: flip by more than one code"
    assert bad.size <= MAX_FLIP_FRACTION * P, f"{what}: {bad.size} boundary flips in {P} elements"
    return bad.size


def compare_step(gpu_st: oracle.State4, ref_st: oracle.State4, w_gpu: np.ndarray, w_ref: np.ndarray,
                 mt: np.ndarray, vt: np.ndarray, tag: str):
    """Compare one step's outputs.  mt, vt are the oracle's precise moments before compression."""
    np.testing.assert_array_equal(gpu_st.m_scales, ref_st.m_scales, err_msg=f"{tag}: block scales")
    np.testing.assert_array_equal(gpu_st.v_r, ref_st.v_r, err_msg=f"{tag}: row maxima")
    np.testing.assert_array_equal(gpu_st.v_c, ref_st.v_c, err_msg=f"{tag}: column maxima")
    P = mt.size
    s = np.repeat(ref_st.m_scales, 128)[:P]
    with np.errstate(invalid="ignore", divide="ignore"):
        n_m = np.where(s > 0, mt / s, np.float32(0)).astype(np.float32)
        sc = np.minimum(ref_st.v_r[:, None], ref_st.v_c[None, :]).reshape(-1)
        n_v = np.where(sc > 0, vt / sc, np.float32(0)).astype(np.float32)
    flips = assert_codes_match(gpu_st.m_codes, ref_st.m_codes, n_m, oracle.step_table("de"), f"{tag}: m codes")
    flips += assert_codes_match(gpu_st.v_codes, ref_st.v_codes, n_v, oracle.step_table("linear"), f"{tag}: v codes")
    np.testing.assert_allclose(w_gpu, w_ref, rtol=PARAM_RTOL, atol=PARAM_ATOL, err_msg=f"{tag}: parameters")
    return flips


def run_parity(rows, cols, steps, recipe="iid", bf16=False, seed=1, hp=None, teacher_forced=True,
               tensor_id=0, w_std=0.02):
    """Free-running (and, per step, teacher-forced) comparison of the HIP path with the oracle.

    Each step the GPU starts from its own previous state.  With teacher_forced=True, a state that
    differs from the oracle's only by tolerated boundary flips is replaced by the oracle's before the
    next step, so that one tolerated flip cannot spread; any other difference fails at once."""
    hp = hp or oracle.Hyper()
    lpmm.ensure_init(rows + cols)
    w_ref = workloads.weights(seed, tensor_id, rows, cols, w_std).reshape(-1)
    st_ref = oracle.state_zero(rows, cols)
    w = to_dev(w_ref.copy())
    st = lpmm.new_state(rows, cols, DEV)
    total_flips = 0
    for t in range(1, steps + 1):
        g = workloads.grads(seed, tensor_id, t, rows, cols, recipe, bf16).reshape(-1)
        mt, vt = oracle.adamw4_step(w_ref, g, st_ref, hp, t, want_moments=True)
        gpu_step(w, to_dev(g, bf16), st, hp, t, bf16)
        torch.cuda.synchronize()
        got = download_state(st)
        w_got = w.cpu().numpy()
        # both sides run free from their own parameters; nothing the GPU produced enters the oracle
        flips = compare_step(got, st_ref, w_got, w_ref, mt, vt, f"{rows}x{cols} {recipe} step {t}")
        total_flips += flips
        if flips and teacher_forced:
            st = upload_state(st_ref)
    return total_flips
