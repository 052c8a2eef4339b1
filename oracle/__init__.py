"""ctypes front end of the CPU oracle (test infrastructure, see lpmm_oracle.cpp).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package.
It never imports the GPU package and the GPU package never imports it.
Arrays are numpy, C-contiguous; state buffers are modified in place.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lpmm_oracle.cpp")
_LIB = os.path.join(_HERE, "liblpmm_oracle.so")

BLOCK = 128


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        i64 = ctypes.c_int64
        cf = ctypes.c_float
        L.oracle_table_linear.argtypes = [ctypes.c_int, f32p]
        L.oracle_table_de.argtypes = [ctypes.c_int, ctypes.c_int, f32p]
        L.oracle_table_de_f64.argtypes = [ctypes.c_int, ctypes.c_int, f64p]
        L.oracle_step_table.argtypes = [ctypes.c_int, f32p]
        L.oracle_nearest_code.argtypes = [f32p, ctypes.c_int, cf]
        L.oracle_nearest_code.restype = ctypes.c_int
        L.oracle_nearest_codes.argtypes = [f32p, ctypes.c_int, f32p, i64, u8p]
        L.oracle_quant_m.argtypes = [f32p, i64, u8p, f32p]
        L.oracle_dequant_m.argtypes = [u8p, f32p, i64, f32p]
        L.oracle_quant_v.argtypes = [f32p, i64, i64, u8p, f32p, f32p]
        L.oracle_dequant_v.argtypes = [u8p, f32p, f32p, i64, i64, f32p]
        L.oracle_adamw32_step.argtypes = [f32p, f32p, f32p, f32p, i64, cf, cf, cf, cf, cf, i64]
        L.oracle_adamw4_step.argtypes = [f32p, f32p, u8p, f32p, u8p, f32p, f32p, i64, i64,
                                         cf, cf, cf, cf, cf, i64, f32p, f32p]
        L.oracle_state_zero.argtypes = [u8p, f32p, u8p, f32p, f32p, i64, i64]
        L.oracle_quant_v_block.argtypes = [f32p, i64, u8p, f32p]
        L.oracle_dequant_v_block.argtypes = [u8p, f32p, i64, f32p]
        L.oracle_adamw4_b128_step.argtypes = [f32p, f32p, u8p, f32p, u8p, f32p, i64,
                                              cf, cf, cf, cf, cf, i64, f32p, f32p]
        L.oracle_state_zero_b128.argtypes = [u8p, f32p, u8p, f32p, i64]
        i64p = ctypes.POINTER(ctypes.c_int64)
        L.oracle_quant_v_nd.argtypes = [f32p, i64p, ctypes.c_int, u8p, f32p]
        L.oracle_dequant_v_nd.argtypes = [u8p, f32p, i64p, ctypes.c_int, f32p]
        L.oracle_adamw4_nd_step.argtypes = [f32p, f32p, u8p, f32p, u8p, f32p, i64p, ctypes.c_int,
                                            cf, cf, cf, cf, cf, i64, f32p, f32p]
        L.oracle_state_zero_nd.argtypes = [u8p, f32p, u8p, f32p, i64p, ctypes.c_int]
        L.oracle_sgdm32_step.argtypes = [f32p, f32p, f32p, i64, cf, cf]
        L.oracle_sgdm4_step.argtypes = [f32p, f32p, u8p, f32p, i64, cf, cf, f32p]
        L.oracle_adamw4_factor_step.argtypes = [f32p, f32p, u8p, f32p, f32p, f32p, i64, i64,
                                                cf, cf, cf, cf, cf, i64, f32p, f32p]
        L.oracle_state_zero_factor.argtypes = [u8p, f32p, f32p, f32p, i64, i64]
        u64 = ctypes.c_uint64
        L.oracle_ablation_table.argtypes = [ctypes.c_int, ctypes.c_int, f32p]
        L.oracle_ablation_table.restype = ctypes.c_int
        L.oracle_splitmix64_at.argtypes = [u64, u64]
        L.oracle_splitmix64_at.restype = u64
        L.oracle_uniform_at.argtypes = [u64, u64]
        L.oracle_uniform_at.restype = cf
        L.oracle_round_stochastic.argtypes = [f32p, ctypes.c_int, cf, cf]
        L.oracle_round_stochastic.restype = ctypes.c_int
        L.oracle_quant_ablation.argtypes = [ctypes.c_int] * 4 + [u64, f32p, i64, i64, u8p, f32p, f32p]
        L.oracle_quant_ablation.restype = ctypes.c_int
        L.oracle_dequant_ablation.argtypes = [ctypes.c_int] * 3 + [u8p, f32p, f32p, i64, i64, f32p]
        L.oracle_dequant_ablation.restype = ctypes.c_int
        for name in ("oracle_table_linear", "oracle_table_de", "oracle_table_de_f64",
                     "oracle_step_table", "oracle_nearest_codes", "oracle_quant_m",
                     "oracle_dequant_m", "oracle_quant_v", "oracle_dequant_v",
                     "oracle_adamw32_step", "oracle_adamw4_step", "oracle_state_zero",
                     "oracle_quant_v_block", "oracle_dequant_v_block", "oracle_adamw4_b128_step",
                     "oracle_state_zero_b128", "oracle_adamw4_factor_step", "oracle_state_zero_factor",
                     "oracle_quant_v_nd", "oracle_dequant_v_nd", "oracle_adamw4_nd_step", "oracle_state_zero_nd",
                     "oracle_sgdm32_step", "oracle_sgdm4_step"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _u8(a: np.ndarray):
    assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


# ---- tables and mapping ----------------------------------------------------------------------

def table_linear(bits: int = 4) -> np.ndarray:
    out = np.empty(1 << bits, np.float32)
    lib().oracle_table_linear(bits, _f32(out))
    return out


def table_de(bits: int = 4, signed: bool = True) -> np.ndarray:
    out = np.empty(1 << bits, np.float32)
    lib().oracle_table_de(bits, int(signed), _f32(out))
    return out


def table_de_f64(bits: int = 4, signed: bool = True) -> np.ndarray:
    out = np.empty(1 << bits, np.float64)
    lib().oracle_table_de_f64(bits, int(signed), out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out


def step_table(what: str) -> np.ndarray:
    out = np.empty(16, np.float32)
    lib().oracle_step_table({"de": 0, "linear": 1}[what], _f32(out))
    return out


def nearest_codes(table: np.ndarray, n: np.ndarray) -> np.ndarray:
    table = np.ascontiguousarray(table, np.float32)
    n = np.ascontiguousarray(n, np.float32)
    out = np.empty(n.size, np.uint8)
    lib().oracle_nearest_codes(_f32(table), table.size, _f32(n), n.size, _u8(out))
    return out.reshape(n.shape)


# ---- quantizers ------------------------------------------------------------------------------

def codes_bytes(P: int) -> int:
    return (P + 1) // 2


def n_blocks(P: int) -> int:
    return (P + BLOCK - 1) // BLOCK


def quant_m(x: np.ndarray):
    x = np.ascontiguousarray(x, np.float32).reshape(-1)
    codes = np.zeros(codes_bytes(x.size), np.uint8)
    scales = np.zeros(n_blocks(x.size), np.float32)
    lib().oracle_quant_m(_f32(x), x.size, _u8(codes), _f32(scales))
    return codes, scales


def dequant_m(codes: np.ndarray, scales: np.ndarray, P: int) -> np.ndarray:
    out = np.empty(P, np.float32)
    lib().oracle_dequant_m(_u8(codes), _f32(scales), P, _f32(out))
    return out


def quant_v(x: np.ndarray):
    x = np.ascontiguousarray(x, np.float32)
    rows, cols = x.shape
    codes = np.zeros(codes_bytes(x.size), np.uint8)
    r = np.zeros(rows, np.float32)
    c = np.zeros(cols, np.float32)
    lib().oracle_quant_v(_f32(x), rows, cols, _u8(codes), _f32(r), _f32(c))
    return codes, r, c


def dequant_v(codes: np.ndarray, r: np.ndarray, c: np.ndarray) -> np.ndarray:
    rows, cols = r.size, c.size
    out = np.empty((rows, cols), np.float32)
    lib().oracle_dequant_v(_u8(codes), _f32(r), _f32(c), rows, cols, _f32(out))
    return out


def quant_v_block(x: np.ndarray):
    """B128/Linear compress of a non-negative flat tensor (second moment of 1-D / flattened tensors)."""
    x = np.ascontiguousarray(x, np.float32).reshape(-1)
    codes = np.zeros(codes_bytes(x.size), np.uint8)
    scales = np.zeros(n_blocks(x.size), np.float32)
    lib().oracle_quant_v_block(_f32(x), x.size, _u8(codes), _f32(scales))
    return codes, scales


def dequant_v_block(codes: np.ndarray, scales: np.ndarray, P: int) -> np.ndarray:
    out = np.empty(P, np.float32)
    lib().oracle_dequant_v_block(_u8(codes), _f32(scales), P, _f32(out))
    return out


def unpack_codes(codes: np.ndarray, P: int) -> np.ndarray:
    """Byte k holds element 2k in its low nibble and element 2k+1 in its high nibble."""
    out = np.empty(codes.size * 2, np.uint8)
    out[0::2] = codes & 0x0F
    out[1::2] = codes >> 4
    return out[:P]


# ---- optimizer -------------------------------------------------------------------------------

@dataclass
class Hyper:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.01


@dataclass
class State4:
    """Compressed state of one rows x cols tensor."""
    rows: int
    cols: int
    m_codes: np.ndarray
    m_scales: np.ndarray
    v_codes: np.ndarray
    v_r: np.ndarray
    v_c: np.ndarray

    def copy(self) -> "State4":
        return State4(self.rows, self.cols, self.m_codes.copy(), self.m_scales.copy(),
                      self.v_codes.copy(), self.v_r.copy(), self.v_c.copy())


def state_zero(rows: int, cols: int) -> State4:
    P = rows * cols
    st = State4(rows, cols, np.zeros(codes_bytes(P), np.uint8), np.zeros(n_blocks(P), np.float32),
                np.zeros(codes_bytes(P), np.uint8), np.zeros(rows, np.float32),
                np.zeros(cols, np.float32))
    lib().oracle_state_zero(_u8(st.m_codes), _f32(st.m_scales), _u8(st.v_codes), _f32(st.v_r),
                            _f32(st.v_c), rows, cols)
    return st


def adamw4_step(w: np.ndarray, g: np.ndarray, st: State4, hp: Hyper, t: int, want_moments=False):
    """In place on w (float32, rows*cols) and st.  g is float32 (a bf16 gradient is passed upcast)."""
    assert w.size == st.rows * st.cols == g.size
    mt = vt = None
    null = ctypes.POINTER(ctypes.c_float)()
    if want_moments:
        mt = np.empty(w.size, np.float32)
        vt = np.empty(w.size, np.float32)
    lib().oracle_adamw4_step(_f32(w), _f32(g), _u8(st.m_codes), _f32(st.m_scales), _u8(st.v_codes),
                             _f32(st.v_r), _f32(st.v_c), st.rows, st.cols, hp.lr, hp.beta1,
                             hp.beta2, hp.eps, hp.weight_decay, t,
                             _f32(mt) if want_moments else null, _f32(vt) if want_moments else null)
    return mt, vt


def adamw32_step(w: np.ndarray, g: np.ndarray, m: np.ndarray, v: np.ndarray, hp: Hyper, t: int):
    lib().oracle_adamw32_step(_f32(w), _f32(g), _f32(m), _f32(v), w.size, hp.lr, hp.beta1, hp.beta2,
                              hp.eps, hp.weight_decay, t)


@dataclass
class StateB128:
    """Compressed state of a flat tensor of P elements, both moments block-wise (B128)."""
    P: int
    m_codes: np.ndarray
    m_scales: np.ndarray
    v_codes: np.ndarray
    v_scales: np.ndarray

    def copy(self) -> "StateB128":
        return StateB128(self.P, self.m_codes.copy(), self.m_scales.copy(), self.v_codes.copy(),
                         self.v_scales.copy())


def state_zero_b128(P: int) -> StateB128:
    st = StateB128(P, np.zeros(codes_bytes(P), np.uint8), np.zeros(n_blocks(P), np.float32),
                   np.zeros(codes_bytes(P), np.uint8), np.zeros(n_blocks(P), np.float32))
    lib().oracle_state_zero_b128(_u8(st.m_codes), _f32(st.m_scales), _u8(st.v_codes), _f32(st.v_scales), P)
    return st


def adamw4_b128_step(w: np.ndarray, g: np.ndarray, st: StateB128, hp: Hyper, t: int, want_moments=False):
    """In place on w (float32, P) and st; second moment compressed block-wise."""
    assert w.size == st.P == g.size
    mt = vt = None
    null = ctypes.POINTER(ctypes.c_float)()
    if want_moments:
        mt = np.empty(w.size, np.float32)
        vt = np.empty(w.size, np.float32)
    lib().oracle_adamw4_b128_step(_f32(w), _f32(g), _u8(st.m_codes), _f32(st.m_scales), _u8(st.v_codes),
                                  _f32(st.v_scales), st.P, hp.lr, hp.beta1, hp.beta2, hp.eps,
                                  hp.weight_decay, t, _f32(mt) if want_moments else null,
                                  _f32(vt) if want_moments else null)
    return mt, vt


@dataclass
class StateFactor:
    """State of one rows x cols tensor under "4-bit Factor": compressed first moment, row and column
    statistics of the second."""
    rows: int
    cols: int
    m_codes: np.ndarray
    m_scales: np.ndarray
    v_row: np.ndarray
    v_col: np.ndarray

    def copy(self) -> "StateFactor":
        return StateFactor(self.rows, self.cols, self.m_codes.copy(), self.m_scales.copy(),
                           self.v_row.copy(), self.v_col.copy())


def state_zero_factor(rows: int, cols: int) -> StateFactor:
    P = rows * cols
    st = StateFactor(rows, cols, np.zeros(codes_bytes(P), np.uint8), np.zeros(n_blocks(P), np.float32),
                     np.ones(rows, np.float32), np.ones(cols, np.float32))
    lib().oracle_state_zero_factor(_u8(st.m_codes), _f32(st.m_scales), _f32(st.v_row), _f32(st.v_col),
                                   rows, cols)
    return st


def adamw4_factor_step(w: np.ndarray, g: np.ndarray, st: StateFactor, hp: Hyper, t: int, want_moments=False):
    """In place on w (float32, rows*cols) and st; second moment factorized (Sec. 4.3)."""
    assert w.size == st.rows * st.cols == g.size
    mt = vt = None
    null = ctypes.POINTER(ctypes.c_float)()
    if want_moments:
        mt = np.empty(w.size, np.float32)
        vt = np.empty(w.size, np.float32)
    lib().oracle_adamw4_factor_step(_f32(w), _f32(g), _u8(st.m_codes), _f32(st.m_scales), _f32(st.v_row),
                                    _f32(st.v_col), st.rows, st.cols, hp.lr, hp.beta1, hp.beta2, hp.eps,
                                    hp.weight_decay, t, _f32(mt) if want_moments else null,
                                    _f32(vt) if want_moments else null)
    return mt, vt


# ---- rank-1 normalization of tensors with any number of dimensions (App. F Alg. 4) ----------------------

def _dims(shape):
    return (ctypes.c_int64 * len(shape))(*[int(d) for d in shape])


def quant_v_nd(x: np.ndarray):
    """x: float32 array with p >= 1 dimensions, >= 0.  Returns (codes, stats); stats = the p statistics vectors
    one after the other."""
    x = np.ascontiguousarray(x, np.float32)
    codes = np.zeros(codes_bytes(x.size), np.uint8)
    stats = np.zeros(sum(x.shape), np.float32)
    lib().oracle_quant_v_nd(_f32(x), _dims(x.shape), x.ndim, _u8(codes), _f32(stats))
    return codes, stats


def dequant_v_nd(codes: np.ndarray, stats: np.ndarray, shape) -> np.ndarray:
    out = np.empty(int(np.prod(shape)), np.float32)
    lib().oracle_dequant_v_nd(_u8(codes), _f32(stats), _dims(shape), len(shape), _f32(out))
    return out.reshape(shape)


@dataclass
class StateND:
    """Compressed state of a tensor with p dimensions (rank-1 second moment in its general form)."""
    shape: tuple
    m_codes: np.ndarray
    m_scales: np.ndarray
    v_codes: np.ndarray
    v_stats: np.ndarray

    def copy(self) -> "StateND":
        return StateND(self.shape, self.m_codes.copy(), self.m_scales.copy(), self.v_codes.copy(),
                       self.v_stats.copy())


def state_zero_nd(shape) -> StateND:
    shape = tuple(int(d) for d in shape)
    P = int(np.prod(shape))
    st = StateND(shape, np.zeros(codes_bytes(P), np.uint8), np.zeros(n_blocks(P), np.float32),
                 np.zeros(codes_bytes(P), np.uint8), np.ones(sum(shape), np.float32))
    lib().oracle_state_zero_nd(_u8(st.m_codes), _f32(st.m_scales), _u8(st.v_codes), _f32(st.v_stats),
                               _dims(shape), len(shape))
    return st


def adamw4_nd_step(w: np.ndarray, g: np.ndarray, st: StateND, hp: Hyper, t: int, want_moments=False):
    P = int(np.prod(st.shape))
    assert w.size == P == g.size
    mt = vt = None
    null = ctypes.POINTER(ctypes.c_float)()
    if want_moments:
        mt = np.empty(P, np.float32)
        vt = np.empty(P, np.float32)
    lib().oracle_adamw4_nd_step(_f32(w), _f32(g), _u8(st.m_codes), _f32(st.m_scales), _u8(st.v_codes),
                                _f32(st.v_stats), _dims(st.shape), len(st.shape), hp.lr, hp.beta1, hp.beta2,
                                hp.eps, hp.weight_decay, t, _f32(mt) if want_moments else null,
                                _f32(vt) if want_moments else null)
    return mt, vt


# ---- SGD with momentum, momentum compressed to 4 bits (App. E Alg. 2) ---------------------------------------

@dataclass
class StateSgdm:
    """Compressed momentum of a flat tensor of P elements."""
    P: int
    m_codes: np.ndarray
    m_scales: np.ndarray

    def copy(self) -> "StateSgdm":
        return StateSgdm(self.P, self.m_codes.copy(), self.m_scales.copy())


def state_zero_sgdm(P: int) -> StateSgdm:
    codes, scales = quant_m(np.zeros(P, np.float32))
    return StateSgdm(P, codes, scales)


def sgdm4_step(w: np.ndarray, g: np.ndarray, st: StateSgdm, lr: float, beta: float, want_moment=False):
    assert w.size == st.P == g.size
    mt = np.empty(w.size, np.float32) if want_moment else None
    null = ctypes.POINTER(ctypes.c_float)()
    lib().oracle_sgdm4_step(_f32(w), _f32(g), _u8(st.m_codes), _f32(st.m_scales), st.P, lr, beta,
                            _f32(mt) if want_moment else null)
    return mt


def sgdm32_step(w: np.ndarray, g: np.ndarray, m: np.ndarray, lr: float, beta: float):
    lib().oracle_sgdm32_step(_f32(w), _f32(g), _f32(m), w.size, lr, beta)


# ---- ablation quantizers of the second moment (Sec. 4.1, Tab. 1) and stochastic rounding (App. D.3) --------------

NORMS = {"b128": 0, "b2048": 1, "rank1": 2}
MAPS = {"de": 0, "de0": 1, "linear": 2}
NORM_BLOCK = {"b128": 128, "b2048": 2048}


def ablation_table(map_name: str, signed: bool = False) -> np.ndarray:
    """Entries of a 4-bit map: de (16 points; the signed or the unsigned variant), de0 (unsigned DE without its
    zero, 15 points), linear (16 points)."""
    out = np.zeros(16, np.float32)
    n = lib().oracle_ablation_table(MAPS[map_name], int(signed), _f32(out))
    if n == 0:
        raise ValueError(f"no such map: {map_name}, signed={signed}")
    return out[:n].copy()


def splitmix64_at(seed: int, idx: int) -> int:
    return int(lib().oracle_splitmix64_at(seed, idx))


def uniform_at(seed: int, idx: int) -> float:
    return float(lib().oracle_uniform_at(seed, idx))


def round_stochastic(table: np.ndarray, n: float, u: float) -> int:
    table = np.ascontiguousarray(table, np.float32)
    return int(lib().oracle_round_stochastic(_f32(table), table.size, float(n), float(u)))


def _ablation_scale_sizes(norm: str, rows: int, cols: int):
    if norm == "rank1":
        return rows, cols
    B = NORM_BLOCK[norm]
    return (rows * cols + B - 1) // B, 1


def quant_ablation(x: np.ndarray, norm: str, map_name: str, signed: bool = False, stochastic: bool = False,
                   seed: int = 0):
    """x: float32 (rows, cols).  Returns (codes, scale_a, scale_b): block scales or row maxima, column maxima
    (rank-1 only, else one unused float)."""
    x = np.ascontiguousarray(x, np.float32)
    rows, cols = x.shape
    na, nb = _ablation_scale_sizes(norm, rows, cols)
    codes = np.zeros(codes_bytes(x.size), np.uint8)
    sa, sb = np.zeros(na, np.float32), np.zeros(nb, np.float32)
    rc = lib().oracle_quant_ablation(NORMS[norm], MAPS[map_name], int(signed), int(stochastic), seed, _f32(x),
                                     rows, cols, _u8(codes), _f32(sa), _f32(sb))
    if rc != 0:
        raise ValueError(f"no such quantizer: {norm}/{map_name}, signed={signed}")
    return codes, sa, sb


def dequant_ablation(codes: np.ndarray, sa: np.ndarray, sb: np.ndarray, rows: int, cols: int, norm: str,
                     map_name: str, signed: bool = False) -> np.ndarray:
    out = np.empty((rows, cols), np.float32)
    rc = lib().oracle_dequant_ablation(NORMS[norm], MAPS[map_name], int(signed), _u8(codes), _f32(sa), _f32(sb),
                                       rows, cols, _f32(out))
    if rc != 0:
        raise ValueError(f"no such quantizer: {norm}/{map_name}, signed={signed}")
    return out
