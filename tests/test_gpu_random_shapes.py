"""Seeded random shapes through every single-tensor entry point, two steps each, against the CPU oracle: a net for
indexing mistakes in geometry combinations that the hand-picked cases miss (ragged tiles, odd column-block counts,
blocks straddling rows, unit dimensions)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2309_01507_amd as lpmm
import workloads
from gpu_util import DEV, compare_step, download_state, gpu_step, to_dev
import test_gpu_b128 as tb
import test_gpu_factor as tf
import test_gpu_rank1_nd as tn
import test_gpu_sgdm as ts

pytestmark = pytest.mark.gpu
HP = oracle.Hyper()


def _shapes(seed, n, fast_share=0.5):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        rows = int(rng.integers(1, 400))
        if rng.random() < fast_share:
            cols = 128 * int(rng.integers(1, 24))
        else:
            cols = int(rng.integers(1, 900))
        out.append((rows, cols))
    return out


def test_rank1_random_shapes():
    print("\n[gpu-test] rank-1 random shapes", flush=True)
    for k, (rows, cols) in enumerate(_shapes(101, 36)):
        lpmm.ensure_init(4096)
        w_ref, st_ref = workloads.weights(101, k, rows, cols).reshape(-1), oracle.state_zero(rows, cols)
        w, st = to_dev(w_ref.copy()), lpmm.new_state(rows, cols, DEV)
        for t in (1, 2):
            g = workloads.grads(101, k, t, rows, cols, "col_lognormal").reshape(-1)
            mt, vt = oracle.adamw4_step(w_ref, g, st_ref, HP, t, want_moments=True)
            gpu_step(w, to_dev(g), st, HP, t)
            torch.cuda.synchronize()
            assert compare_step(download_state(st), st_ref, w.cpu().numpy(), w_ref, mt, vt, f"{rows}x{cols} step {t}") == 0


def test_factor_random_shapes():
    print("\n[gpu-test] factor random shapes", flush=True)
    for k, (rows, cols) in enumerate(_shapes(102, 30)):
        assert tf.run(rows, cols, steps=2, seed=200 + k) == 0


def test_b128_and_sgdm_random_sizes():
    print("\n[gpu-test] flat random sizes", flush=True)
    rng = np.random.default_rng(103)
    for k in range(24):
        P = int(rng.integers(1, 300000))
        assert tb.run(1, P, steps=2, seed=300 + k) == 0
        assert ts.run(1, P, steps=2, seed=400 + k) == 0


def test_nd_random_shapes():
    print("\n[gpu-test] n-dimensional random shapes", flush=True)
    rng = np.random.default_rng(104)
    for k in range(24):
        p = int(rng.integers(3, 6))
        shape = tuple(int(rng.integers(1, 9)) for _ in range(p - 2)) + (int(rng.choice([2, 4, 8, 16, 3, 5])),
                                                                       int(rng.choice([16, 32, 64, 7, 12])))
        shape = (int(rng.integers(1, 200)),) + shape[1:] if p > 2 else shape
        assert tn.run(shape, steps=2, seed=500 + k) == 0


@pytest.mark.parametrize("env", [{}, {"LPMM_PHASE_MPARAMS": "1"}, {"LPMM_PHASE_MPARAMS": "1", "LPMM_FLAT": "1"}],
                         ids=["one-group", "many-groups", "many-groups-flat"])
def test_random_plans(env):
    from test_gpu_multi import _run_set
    T = workloads.TensorSpec
    for seed in (111, 112):
        specs = [T(f"t{k}", r, c) for k, (r, c) in enumerate(_shapes(seed, 14, fast_share=0.7))]      # small ones keep fp32 states
        _run_set(specs, "col_lognormal", seed == 112, steps=2, seed=seed, env=env)
