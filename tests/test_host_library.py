"""CPU-only checks of lpmm4.so: it loads, exports what include/lpmm4.h declares, and its host-built
tables and search structure agree with the oracle's definitions.  No GPU call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2309_01507_amd as lpmm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "lpmm4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lpmm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 12
    L = lpmm.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in include/lpmm4.h but not exported"


def test_tables_equal_the_oracles():
    np.testing.assert_array_equal(lpmm.lpmm_table(0), oracle.step_table("de"))
    np.testing.assert_array_equal(lpmm.lpmm_table(1), oracle.step_table("linear"))


def _probe_values(T):
    rng = np.random.default_rng(0)
    mids = ((T[:-1].astype(np.float64) + T[1:].astype(np.float64)) / 2).astype(np.float32)
    near = [mids]
    for k in range(1, 4):
        up, dn = mids.copy(), mids.copy()
        for _ in range(k):
            up, dn = np.nextafter(up, np.float32(4)), np.nextafter(dn, np.float32(-4))
        near += [up, dn]
    # bucket edges of the search table: every multiple of 2^e/4 in the binades that matter
    edges = np.array([s * (1 + q / 4) * 2.0 ** e for s in (-1, 1) for e in range(-12, 1) for q in range(4)],
                     np.float32)
    edges = np.concatenate([edges, np.nextafter(edges, np.float32(4)), np.nextafter(edges, np.float32(-4))])
    rnd = rng.uniform(-1.2, 1.2, 400000).astype(np.float32)
    small = (rng.uniform(-1, 1, 200000) * 10.0 ** rng.uniform(-8, 0, 200000)).astype(np.float32)
    bits = rng.integers(0, 2 ** 32, 400000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    bits = bits[np.isfinite(bits) & (np.abs(bits) <= 4)]   # normalized values lie in [-1, 1]
    special = np.array([0.0, -0.0, 1.0, -1.0, 1e-45, -1e-45, 1e-38, 3.0, -3.0], np.float32)
    return np.concatenate([T, *near, edges, rnd, small, bits, special]).astype(np.float32)


def test_host_search_matches_bruteforce_de():
    T = oracle.step_table("de")
    n = _probe_values(T)
    np.testing.assert_array_equal(lpmm.lpmm_host_nearest_codes(0, n), oracle.nearest_codes(T, n))


def test_host_search_matches_bruteforce_linear():
    T = oracle.step_table("linear")
    n = _probe_values(T)
    np.testing.assert_array_equal(lpmm.lpmm_host_nearest_codes(1, n), oracle.nearest_codes(T, n))


def test_state_sizes():
    assert lpmm.lpmm_adamw4_state_sizes(1024, 1024) == [524288, 32768, 524288, 4096, 4096]
    assert lpmm.lpmm_adamw4_state_sizes(3, 43) == [65, 8, 65, 12, 172]       # P = 129: odd, 2 blocks
    assert lpmm.lpmm_adamw4_workspace_bytes(8192) >= 4 * 8192


def test_argument_errors_are_reported_before_any_gpu_work():
    L = lpmm.lib()
    shape = (ctypes.c_int64 * 2)(16, 128)
    bad_shape = (ctypes.c_int64 * 2)(0, 128)
    sizes = (ctypes.c_size_t * 5)()
    assert L.lpmm_adamw4_state_sizes(ctypes.addressof(bad_shape), ctypes.addressof(sizes)) == -1
    assert L.lpmm_adamw4_state_sizes(None, ctypes.addressof(sizes)) == -1
    buf = ctypes.create_string_buffer(4096 + 256)
    p = (ctypes.addressof(buf) + 255) // 256 * 256             # an aligned, non-null fake pointer
    args = [p] * 7 + [ctypes.addressof(shape)]
    ok_h = [1e-3, 0.9, 0.999, 1e-8, 0.01]

    def call(ptrs=args, h=ok_h, step=1):
        return L.lpmm_adamw4_step(*ptrs, *[ctypes.c_float(x) for x in h], step, None)

    assert call(step=0) == -1                                   # t starts at 1
    assert call(h=[1e-3, 1.0, 0.999, 1e-8, 0.01]) == -1          # beta1 must be < 1
    assert call(h=[1e-3, 0.9, -0.1, 1e-8, 0.01]) == -1
    assert call(h=[float("nan"), 0.9, 0.999, 1e-8, 0.01]) == -1
    assert call(h=[1e-3, 0.9, 0.999, -1.0, 0.01]) == -1
    assert call(ptrs=[None] + args[1:]) == -1                   # null parameter pointer
    assert call(ptrs=[p + 4] + args[1:]) == -1                  # misaligned parameter pointer
    assert call(ptrs=args[:7] + [ctypes.addressof(bad_shape)]) == -1
    assert L.lpmm_table(2, p) == -1
    assert b"invalid" in L.lpmm_strerror(-1) and b"workspace" in L.lpmm_strerror(-4)
    # a well-formed call before init (or without a GPU) is refused, not executed
    assert call() in (-2, -3)


def test_block_wise_state_sizes_and_argument_errors():
    assert lpmm.lpmm_adamw4_b128_state_sizes(4096) == [2048, 128, 2048, 128]
    assert lpmm.lpmm_adamw4_b128_state_sizes(129) == [65, 8, 65, 8]          # odd size, 2 blocks
    L = lpmm.lib()
    sizes = (ctypes.c_size_t * 4)()
    assert L.lpmm_adamw4_b128_state_sizes(0, ctypes.addressof(sizes)) == -1
    assert L.lpmm_adamw4_b128_state_sizes(16, None) == -1
    buf = ctypes.create_string_buffer(4096 + 256)
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    ok_h = [1e-3, 0.9, 0.999, 1e-8, 0.01]

    def call(ptrs=None, numel=256, h=ok_h, step=1):
        ptrs = ptrs or [p] * 6
        return L.lpmm_adamw4_b128_step(*ptrs, numel, *[ctypes.c_float(x) for x in h], step, None)

    assert call(step=0) == -1
    assert call(numel=0) == -1
    assert call(h=[1e-3, 0.9, 1.0, 1e-8, 0.01]) == -1
    assert call(ptrs=[p] * 5 + [None]) == -1                    # null block-scale pointer
    assert call(ptrs=[p + 8] + [p] * 5) == -1                   # parameters must be 16-byte aligned
    assert call() in (-2, -3)                                   # well-formed, but no initialized GPU here


def test_factorized_state_sizes_and_argument_errors():
    assert lpmm.lpmm_adamw4_factor_state_sizes(32, 128) == [2048, 128, 128, 512]
    assert lpmm.lpmm_adamw4_factor_state_sizes(3, 43) == [65, 8, 12, 172]      # 129 elements: odd, 2 blocks
    L = lpmm.lib()
    sizes = (ctypes.c_size_t * 4)()
    bad = (ctypes.c_int64 * 2)(0, 5)
    ok = (ctypes.c_int64 * 2)(2, 128)
    assert L.lpmm_adamw4_factor_state_sizes(ctypes.addressof(bad), ctypes.addressof(sizes)) == -1
    assert L.lpmm_adamw4_factor_state_sizes(ctypes.addressof(ok), None) == -1
    assert L.lpmm_adamw4_factor_state_sizes(None, ctypes.addressof(sizes)) == -1
    buf = ctypes.create_string_buffer(4096 + 256)
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    ok_h = [1e-3, 0.9, 0.999, 1e-8, 0.01]

    def call(ptrs=None, shape=ok, h=ok_h, step=1):
        ptrs = ptrs or [p] * 6
        return L.lpmm_adamw4_factor_step(*ptrs, ctypes.addressof(shape) if shape is not None else None,
                                         *[ctypes.c_float(x) for x in h], step, None)

    assert call(step=0) == -1
    assert call(shape=bad) == -1
    assert call(shape=None) == -1
    assert call(h=[1e-3, 1.0, 0.999, 1e-8, 0.01]) == -1
    assert call(h=[-1e-3, 0.9, 0.999, 1e-8, 0.01]) == -1
    assert call(ptrs=[p] * 4 + [None, p]) == -1                 # null row statistics
    assert call(ptrs=[p, p + 8] + [p] * 4) == -1                # the gradient must be 16-byte aligned
    assert call() in (-2, -3)                                   # well-formed, but no initialized GPU here
    d = lpmm.TensorDesc(p, p, p, p, None, p, p, 2, 128, lpmm.KIND_4BIT_FACTOR, 0)
    r1 = lpmm.TensorDesc(p, p, p, p, p, p, p, 2, 128, lpmm.KIND_4BIT, 0)
    assert lpmm.lpmm_adamw4_plan_bytes([d]) > 0
    assert lpmm.lpmm_adamw4_plan_bytes([d, r1]) == 0            # two optimizers in one plan


def test_nd_state_sizes_and_argument_errors():
    assert lpmm.lpmm_adamw4_nd_state_sizes((4, 3, 5)) == [30, 4, 30, 16, (15 + 8) * 4]
    assert lpmm.lpmm_adamw4_nd_state_sizes((32, 128)) == [2048, 128, 2048, 128, (128 + 128) * 4]
    L = lpmm.lib()
    sizes = (ctypes.c_size_t * 5)()
    for bad in ((5,), (0, 3, 4), (2,) * 9, (4, -1, 2), (1 << 31, 1 << 31, 4)):
        dims = (ctypes.c_int64 * len(bad))(*bad)
        assert L.lpmm_adamw4_nd_state_sizes(ctypes.addressof(dims), len(bad), ctypes.addressof(sizes)) == -1
    dims = (ctypes.c_int64 * 3)(2, 4, 32)
    assert L.lpmm_adamw4_nd_state_sizes(ctypes.addressof(dims), 3, None) == -1
    assert L.lpmm_adamw4_nd_state_sizes(None, 3, ctypes.addressof(sizes)) == -1
    buf = ctypes.create_string_buffer(4096 + 256)
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    h = [ctypes.c_float(x) for x in (1e-3, 0.9, 0.999, 1e-8, 0.01)]
    assert L.lpmm_adamw4_nd_step(*([p] * 7), ctypes.addressof(dims), 3, *h, 0, None) == -1       # step 0
    assert L.lpmm_adamw4_nd_step(*([p] * 6 + [None]), ctypes.addressof(dims), 3, *h, 1, None) == -1
    assert L.lpmm_adamw4_nd_step(*([p] * 7), ctypes.addressof(dims), 1, *h, 1, None) == -1       # one dimension
    assert L.lpmm_adamw4_nd_step(*([p] * 7), ctypes.addressof(dims), 3, *h, 1, None) in (-2, -3) # no GPU here


def test_sgdm_state_sizes_and_argument_errors():
    assert lpmm.lpmm_sgdm4_state_sizes(4096) == [2048, 128]
    assert lpmm.lpmm_sgdm4_state_sizes(129) == [65, 8]
    L = lpmm.lib()
    sizes = (ctypes.c_size_t * 2)()
    assert L.lpmm_sgdm4_state_sizes(0, ctypes.addressof(sizes)) == -1
    assert L.lpmm_sgdm4_state_sizes(16, None) == -1
    buf = ctypes.create_string_buffer(4096 + 256)
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    f = ctypes.c_float
    assert L.lpmm_sgdm4_step(p, p, p, p, 256, f(0.1), f(1.0), None) == -1          # momentum must stay below 1
    assert L.lpmm_sgdm4_step(p, p, p, p, 256, f(-0.1), f(0.9), None) == -1
    assert L.lpmm_sgdm4_step(p, p, p, None, 256, f(0.1), f(0.9), None) == -1
    assert L.lpmm_sgdm4_step(p + 4, p, p, p, 256, f(0.1), f(0.9), None) == -1
    assert L.lpmm_sgdm4_step(p, p, p, p, 0, f(0.1), f(0.9), None) == -1
    assert L.lpmm_sgdm4_step(p, p, p, p, 256, f(0.1), f(0.9), None) in (-2, -3)    # well-formed, but no GPU here
    assert L.lpmm_sgdm32_step(p, p, p, 256, 7, f(0.1), f(0.9), None) == -1         # unknown gradient type
    assert L.lpmm_sgdm4_step_multi(p, f(0.1), f(0.9), None) == -1                  # not a plan
    d = lpmm.TensorDesc(p, p, p, p, None, None, None, 1, 256, lpmm.KIND_SGDM_4BIT, 0)
    a = lpmm.TensorDesc(p, p, p, p, p, p, p, 2, 128, lpmm.KIND_4BIT, 0)
    assert lpmm.lpmm_adamw4_plan_bytes([d]) > 0 and lpmm.lpmm_adamw4_plan_bytes([d, a]) == 0


def test_plan_bytes_with_inner_dimension_tables():
    buf = ctypes.create_string_buffer(4096 + 256)
    p = (ctypes.addressof(buf) + 255) // 256 * 256
    d = lpmm.TensorDesc(p, p, p, p, p, p, p, 8, 128, lpmm.KIND_4BIT_ND, 0)
    assert lpmm.lpmm_adamw4_plan_bytes([d]) == 0                       # no inner sizes given
    d.inner = (4, 32)
    with_nd = lpmm.lpmm_adamw4_plan_bytes([d])
    plain = lpmm.lpmm_adamw4_plan_bytes([lpmm.TensorDesc(p, p, p, p, p, p, p, 8, 128, lpmm.KIND_4BIT, 0)])
    assert with_nd > plain > 0                                         # the statistics of the inner dimensions
    d.inner = (4, 31)
    assert lpmm.lpmm_adamw4_plan_bytes([d]) == 0                       # product differs from cols
    d.inner = (2,) * 8
    assert lpmm.lpmm_adamw4_plan_bytes([d]) == 0                       # too many dimensions
    f = lpmm.TensorDesc(p, p, p, p, None, p, p, 8, 128, lpmm.KIND_4BIT_FACTOR, 0)
    d.inner = (4, 32)
    assert lpmm.lpmm_adamw4_plan_bytes([d, f]) == 0                    # rank-1 and factorized tensors do not mix


def test_ablation_maps_equal_the_oracles():
    """The maps of the ablation quantizers (Sec. 4.1, Tab. 1) as the library builds them (per-decade bin midpoints)
    against the oracle's (bit-pattern decode and sort), entry for entry; combinations that do not exist are
    refused."""
    import ctypes
    for name, code, signed in (("de", 0, False), ("de", 0, True), ("de0", 1, False), ("linear", 2, False)):
        np.testing.assert_array_equal(lpmm.lpmm_ablation_table(code, signed), oracle.ablation_table(name, signed))
    out = (ctypes.c_float * 16)()
    L = lpmm.lib()
    for code, signed in ((1, 1), (2, 1), (3, 0), (-1, 0)):
        assert L.lpmm_ablation_table(code, signed, ctypes.addressof(out)) == -1
    assert L.lpmm_ablation_table(0, 0, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching any device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
