"""ctypes binding of lpmm4.so (see include/lpmm4.h for the contract of every call).

Argument marshalling only: tensors are torch CUDA tensors used as device memory, the stream is
torch's current stream.  If the shared library is missing the import of a symbol fails loudly;
there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SRC_DIR = os.path.join(_HERE, "csrc")
_LIB = os.path.join(_HERE, "lpmm4.so")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

GRAD_F32, GRAD_BF16 = 0, 1


class LpmmError(RuntimeError):
    pass


def lib_path() -> str:
    return _LIB


def build_library(verbose: bool = False) -> str:
    """Cross-compile lpmm4.so for gfx950 with hipcc (works without a GPU)."""
    cmd = ["hipcc", *HIPCC_FLAGS, os.path.join(_SRC_DIR, "lpmm4.hip"), "-o", _LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise LpmmError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return _LIB


_lib = None

_F = ctypes.c_float
_I64 = ctypes.c_int64
_VP = ctypes.c_void_p
_SHAPE = ctypes.c_int64 * 2


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise LpmmError(f"{_LIB} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                            "(there is no CPU fallback)")
        L = ctypes.CDLL(_LIB)
        L.lpmm_strerror.argtypes = [ctypes.c_int]
        L.lpmm_strerror.restype = ctypes.c_char_p
        L.lpmm_last_hip_error.restype = ctypes.c_int
        L.lpmm_table.argtypes = [ctypes.c_int, _VP]
        L.lpmm_host_nearest_codes.argtypes = [ctypes.c_int, _VP, _I64, _VP]
        L.lpmm_adamw4_workspace_bytes.argtypes = [_I64]
        L.lpmm_adamw4_workspace_bytes.restype = ctypes.c_size_t
        L.lpmm_adamw4_init.argtypes = [ctypes.c_int, _VP, ctypes.c_size_t, _VP]
        L.lpmm_adamw4_state_sizes.argtypes = [_VP, _VP]
        L.lpmm_adamw4_state_zero.argtypes = [_VP] * 5 + [_VP, _VP]
        step_args = [_VP] * 7 + [_VP] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_step.argtypes = step_args
        L.lpmm_adamw4_step_bf16g.argtypes = step_args
        L.lpmm_adamw4_step_noalloc.argtypes = [_VP, _VP, ctypes.c_int] + [_VP] * 5 + [_VP] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_step_ws.argtypes = ([_VP, _VP, ctypes.c_int] + [_VP] * 5 + [_VP] + [_F] * 5 +
                                          [_I64, _VP, ctypes.c_size_t, _VP])
        L.lpmm_adamw32_step.argtypes = [_VP] * 4 + [_I64, ctypes.c_int] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_b128_state_sizes.argtypes = [_I64, _VP]
        L.lpmm_adamw4_b128_state_zero.argtypes = [_VP] * 4 + [_I64, _VP]
        b128_args = [_VP] * 6 + [_I64] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_b128_step.argtypes = b128_args
        L.lpmm_adamw4_b128_step_bf16g.argtypes = b128_args
        L.lpmm_adamw4_nd_state_sizes.argtypes = [_VP, ctypes.c_int, _VP]
        L.lpmm_adamw4_nd_state_zero.argtypes = [_VP] * 5 + [_VP, ctypes.c_int, _VP]
        nd_args = [_VP] * 7 + [_VP, ctypes.c_int] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_nd_step.argtypes = nd_args
        L.lpmm_adamw4_nd_step_bf16g.argtypes = nd_args
        L.lpmm_adamw4_plan_bytes_nd.argtypes = [_VP, _I64, _VP, _VP]
        L.lpmm_adamw4_plan_bytes_nd.restype = ctypes.c_size_t
        L.lpmm_adamw4_plan_build_nd.argtypes = [_VP, _I64, _VP, _VP, ctypes.c_int, _VP, ctypes.c_size_t, _VP]
        L.lpmm_sgdm4_state_sizes.argtypes = [_I64, _VP]
        L.lpmm_sgdm4_state_zero.argtypes = [_VP, _VP, _I64, _VP]
        L.lpmm_sgdm4_step.argtypes = [_VP] * 4 + [_I64, _F, _F, _VP]
        L.lpmm_sgdm4_step_bf16g.argtypes = [_VP] * 4 + [_I64, _F, _F, _VP]
        L.lpmm_sgdm32_step.argtypes = [_VP] * 3 + [_I64, ctypes.c_int, _F, _F, _VP]
        L.lpmm_sgdm4_step_multi.argtypes = [_VP, _F, _F, _VP]
        L.lpmm_adamw4_step_multi_capturable.argtypes = [_VP, _VP, _VP, _F, _F, _F, _F, _VP]
        L.lpmm_sgdm4_step_multi_capturable.argtypes = [_VP, _VP, _F, _VP]
        L.lpmm_adamw4_factor_state_sizes.argtypes = [_VP, _VP]
        L.lpmm_adamw4_factor_state_zero.argtypes = [_VP] * 4 + [_VP, _VP]
        factor_args = [_VP] * 6 + [_VP] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_factor_step.argtypes = factor_args
        L.lpmm_adamw4_factor_step_bf16g.argtypes = factor_args
        L.lpmm_dequant_state.argtypes = [ctypes.c_int, _VP, _VP, _VP, _VP, _VP, _VP]
        L.lpmm_quant_state.argtypes = [ctypes.c_int, _VP, _VP, _VP, _VP, _VP, _VP]
        L.lpmm_ablation_table.argtypes = [ctypes.c_int, ctypes.c_int, _VP]
        L.lpmm_quant_ablation.argtypes = [ctypes.c_int] * 4 + [ctypes.c_uint64, _VP, _VP, _VP, _VP, _VP, _VP]
        L.lpmm_dequant_ablation.argtypes = [ctypes.c_int] * 3 + [_VP, _VP, _VP, _VP, _VP, _VP]
        L.lpmm_adamw4_plan_bytes.argtypes = [_VP, _I64]
        L.lpmm_adamw4_plan_bytes.restype = ctypes.c_size_t
        L.lpmm_adamw4_plan_build.argtypes = [_VP, _I64, ctypes.c_int, _VP, ctypes.c_size_t, _VP]
        L.lpmm_adamw4_step_multi.argtypes = [_VP] + [_F] * 5 + [_I64, _VP]
        L.lpmm_adamw4_plan_release.argtypes = [_VP]
        L.lpmm_profile_begin.argtypes = [_I64]
        L.lpmm_profile_end.argtypes = [_VP, _VP]
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        L = lib()
        msg = L.lpmm_strerror(rc).decode()
        if rc == -3:
            msg += f" [hipError {L.lpmm_last_hip_error()}]"
        raise LpmmError(f"{what}: {msg} (code {rc})")


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _shape(rows: int, cols: int):
    return _SHAPE(int(rows), int(cols))


# ---- host-only calls ---------------------------------------------------------------------------------

def lpmm_table(which: int):
    import numpy as np
    out = np.empty(16, np.float32)
    _check(lib().lpmm_table(which, out.ctypes.data), "lpmm_table")
    return out


def lpmm_host_nearest_codes(which: int, n):
    import numpy as np
    n = np.ascontiguousarray(n, np.float32)
    out = np.empty(n.size, np.uint8)
    _check(lib().lpmm_host_nearest_codes(which, n.ctypes.data, n.size, out.ctypes.data),
           "lpmm_host_nearest_codes")
    return out.reshape(n.shape)


def lpmm_adamw4_workspace_bytes(max_rows_plus_cols: int) -> int:
    return int(lib().lpmm_adamw4_workspace_bytes(int(max_rows_plus_cols)))


def lpmm_adamw4_state_sizes(rows: int, cols: int):
    sizes = (ctypes.c_size_t * 5)()
    shape = _shape(rows, cols)
    _check(lib().lpmm_adamw4_state_sizes(ctypes.addressof(shape), ctypes.addressof(sizes)),
           "lpmm_adamw4_state_sizes")
    return [int(s) for s in sizes]


# ---- device calls ------------------------------------------------------------------------------------

_workspaces = {}   # device index -> (tensor kept alive, capacity in rows+cols)


def lpmm_adamw4_init(device: int, workspace, stream=None) -> None:
    nbytes = workspace.numel() * workspace.element_size()
    _check(lib().lpmm_adamw4_init(int(device), _ptr(workspace), nbytes, _stream(stream)),
           "lpmm_adamw4_init")


def ensure_init(max_rows_plus_cols: int, device=None) -> None:
    """Allocate (with torch) and register a workspace large enough for rows + cols, once per device."""
    import torch
    dev = torch.cuda.current_device() if device is None else int(device)
    have = _workspaces.get(dev)
    if have is not None and have[1] >= max_rows_plus_cols:
        return
    torch.cuda.synchronize(dev)   # steps that use the old workspace must have finished
    cap = max(int(max_rows_plus_cols), 1 << 16)
    nbytes = lpmm_adamw4_workspace_bytes(cap)
    ws = torch.zeros((nbytes + 255) // 256 * 256, dtype=torch.uint8, device=f"cuda:{dev}")
    with torch.cuda.device(dev):
        lpmm_adamw4_init(dev, ws)
        torch.cuda.synchronize(dev)
    _workspaces[dev] = (ws, cap)


@dataclass
class State4:
    """The five device buffers of one quantized tensor's optimizer state."""
    rows: int
    cols: int
    m_codes: "object"
    m_blockscale: "object"
    v_codes: "object"
    v_rowmax: "object"
    v_colmax: "object"


def new_state(rows: int, cols: int, device="cuda") -> State4:
    """Allocate (torch) and zero (library) the state of a rows x cols tensor."""
    import torch
    sz = lpmm_adamw4_state_sizes(rows, cols)
    pad4 = lambda n: (n + 3) // 4 * 4
    st = State4(rows, cols,
                torch.empty(pad4(sz[0]), dtype=torch.uint8, device=device)[:sz[0]],
                torch.empty(sz[1] // 4, dtype=torch.float32, device=device),
                torch.empty(pad4(sz[2]), dtype=torch.uint8, device=device)[:sz[2]],
                torch.empty(sz[3] // 4, dtype=torch.float32, device=device),
                torch.empty(sz[4] // 4, dtype=torch.float32, device=device))
    lpmm_adamw4_state_zero(st)
    return st


def lpmm_adamw4_state_zero(st: State4, stream=None) -> None:
    shape = _shape(st.rows, st.cols)
    _check(lib().lpmm_adamw4_state_zero(_ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_codes),
                                        _ptr(st.v_rowmax), _ptr(st.v_colmax),
                                        ctypes.addressof(shape), _stream(stream)),
           "lpmm_adamw4_state_zero")


def _step(fn_name, param, grad, st: State4, lr, beta1, beta2, eps, weight_decay, step, stream):
    shape = _shape(st.rows, st.cols)
    fn = getattr(lib(), fn_name)
    _check(fn(_ptr(param), _ptr(grad), _ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_codes),
              _ptr(st.v_rowmax), _ptr(st.v_colmax), ctypes.addressof(shape), lr, beta1, beta2, eps,
              weight_decay, int(step), _stream(stream)), fn_name)


def lpmm_adamw4_step(param, grad, st: State4, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _step("lpmm_adamw4_step", param, grad, st, lr, beta1, beta2, eps, weight_decay, step, stream)


def lpmm_adamw4_step_bf16g(param, grad, st: State4, lr, beta1, beta2, eps, weight_decay, step,
                           stream=None):
    _step("lpmm_adamw4_step_bf16g", param, grad, st, lr, beta1, beta2, eps, weight_decay, step, stream)


def lpmm_adamw4_step_noalloc(param, grad, grad_dtype: int, st: State4, lr, beta1, beta2, eps, weight_decay, step,
                             stream=None):
    shape = _shape(st.rows, st.cols)
    _check(lib().lpmm_adamw4_step_noalloc(_ptr(param), _ptr(grad), int(grad_dtype), _ptr(st.m_codes),
                                          _ptr(st.m_blockscale), _ptr(st.v_codes), _ptr(st.v_rowmax),
                                          _ptr(st.v_colmax), ctypes.addressof(shape), lr, beta1, beta2, eps,
                                          weight_decay, int(step), _stream(stream)), "lpmm_adamw4_step_noalloc")


def lpmm_adamw4_step_ws(param, grad, grad_dtype: int, st: State4, lr, beta1, beta2, eps, weight_decay, step,
                        workspace, stream=None):
    """workspace: a zero-filled uint8 / float32 device tensor of at least lpmm_adamw4_workspace_bytes(rows + cols)
    bytes that no other call in flight uses."""
    shape = _shape(st.rows, st.cols)
    _check(lib().lpmm_adamw4_step_ws(_ptr(param), _ptr(grad), int(grad_dtype), _ptr(st.m_codes),
                                     _ptr(st.m_blockscale), _ptr(st.v_codes), _ptr(st.v_rowmax),
                                     _ptr(st.v_colmax), ctypes.addressof(shape), lr, beta1, beta2, eps,
                                     weight_decay, int(step), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream(stream)),
           "lpmm_adamw4_step_ws")


# ---- block-wise second moment (1-D / flattened tensors) ------------------------------------------------

@dataclass
class StateB128:
    """The four device buffers of a flat tensor's optimizer state, both moments block-wise."""
    numel: int
    m_codes: "object"
    m_blockscale: "object"
    v_codes: "object"
    v_blockscale: "object"


def lpmm_adamw4_b128_state_sizes(numel: int):
    sizes = (ctypes.c_size_t * 4)()
    _check(lib().lpmm_adamw4_b128_state_sizes(int(numel), ctypes.addressof(sizes)),
           "lpmm_adamw4_b128_state_sizes")
    return [int(s) for s in sizes]


def lpmm_adamw4_b128_state_zero(st: StateB128, stream=None) -> None:
    _check(lib().lpmm_adamw4_b128_state_zero(_ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_codes),
                                             _ptr(st.v_blockscale), int(st.numel), _stream(stream)),
           "lpmm_adamw4_b128_state_zero")


def new_state_b128(numel: int, device="cuda") -> StateB128:
    """Allocate (torch) and zero (library) the block-wise state of a flat tensor."""
    import torch
    sz = lpmm_adamw4_b128_state_sizes(numel)
    pad4 = lambda n: (n + 3) // 4 * 4
    st = StateB128(numel,
                   torch.empty(pad4(sz[0]), dtype=torch.uint8, device=device)[:sz[0]],
                   torch.empty(sz[1] // 4, dtype=torch.float32, device=device),
                   torch.empty(pad4(sz[2]), dtype=torch.uint8, device=device)[:sz[2]],
                   torch.empty(sz[3] // 4, dtype=torch.float32, device=device))
    lpmm_adamw4_b128_state_zero(st)
    return st


def _b128_step(fn_name, param, grad, st: StateB128, lr, beta1, beta2, eps, weight_decay, step, stream):
    fn = getattr(lib(), fn_name)
    _check(fn(_ptr(param), _ptr(grad), _ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_codes),
              _ptr(st.v_blockscale), int(st.numel), lr, beta1, beta2, eps, weight_decay, int(step),
              _stream(stream)), fn_name)


def lpmm_adamw4_b128_step(param, grad, st: StateB128, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _b128_step("lpmm_adamw4_b128_step", param, grad, st, lr, beta1, beta2, eps, weight_decay, step, stream)


def lpmm_adamw4_b128_step_bf16g(param, grad, st: StateB128, lr, beta1, beta2, eps, weight_decay, step,
                                stream=None):
    _b128_step("lpmm_adamw4_b128_step_bf16g", param, grad, st, lr, beta1, beta2, eps, weight_decay, step,
               stream)


# ---- factorized second moment ("4-bit Factor") ------------------------------------------------------------

@dataclass
class StateFactor:
    """The four device buffers of one rows x cols tensor's state with a factorized second moment."""
    rows: int
    cols: int
    m_codes: "object"
    m_blockscale: "object"
    v_row: "object"
    v_col: "object"


def lpmm_adamw4_factor_state_sizes(rows: int, cols: int):
    sizes = (ctypes.c_size_t * 4)()
    shape = _SHAPE(int(rows), int(cols))
    _check(lib().lpmm_adamw4_factor_state_sizes(ctypes.addressof(shape), ctypes.addressof(sizes)),
           "lpmm_adamw4_factor_state_sizes")
    return [int(s) for s in sizes]


def lpmm_adamw4_factor_state_zero(st: StateFactor, stream=None) -> None:
    shape = _SHAPE(st.rows, st.cols)
    _check(lib().lpmm_adamw4_factor_state_zero(_ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_row),
                                               _ptr(st.v_col), ctypes.addressof(shape), _stream(stream)),
           "lpmm_adamw4_factor_state_zero")


def new_state_factor(rows: int, cols: int, device="cuda") -> StateFactor:
    """Allocate (torch) and zero (library) the state of a rows x cols tensor, second moment factorized."""
    import torch
    sz = lpmm_adamw4_factor_state_sizes(rows, cols)
    pad4 = lambda n: (n + 3) // 4 * 4
    st = StateFactor(rows, cols,
                     torch.empty(pad4(sz[0]), dtype=torch.uint8, device=device)[:sz[0]],
                     torch.empty(sz[1] // 4, dtype=torch.float32, device=device),
                     torch.empty(sz[2] // 4, dtype=torch.float32, device=device),
                     torch.empty(sz[3] // 4, dtype=torch.float32, device=device))
    lpmm_adamw4_factor_state_zero(st)
    return st


def _factor_step(fn_name, param, grad, st: StateFactor, lr, beta1, beta2, eps, weight_decay, step, stream):
    fn = getattr(lib(), fn_name)
    shape = _SHAPE(st.rows, st.cols)
    _check(fn(_ptr(param), _ptr(grad), _ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_row), _ptr(st.v_col),
              ctypes.addressof(shape), lr, beta1, beta2, eps, weight_decay, int(step), _stream(stream)), fn_name)


def lpmm_adamw4_factor_step(param, grad, st: StateFactor, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _factor_step("lpmm_adamw4_factor_step", param, grad, st, lr, beta1, beta2, eps, weight_decay, step, stream)


def lpmm_adamw4_factor_step_bf16g(param, grad, st: StateFactor, lr, beta1, beta2, eps, weight_decay, step,
                                  stream=None):
    _factor_step("lpmm_adamw4_factor_step_bf16g", param, grad, st, lr, beta1, beta2, eps, weight_decay, step,
                 stream)


# ---- rank-1 second moment of tensors with more than two dimensions ----------------------------------------

@dataclass
class StateND:
    """The five device buffers of the state of a tensor with 2..8 dimensions (see lpmm4.h for v_col's layout)."""
    shape: tuple
    m_codes: "object"
    m_blockscale: "object"
    v_codes: "object"
    v_row: "object"
    v_col: "object"


def _dims(shape):
    return (ctypes.c_int64 * len(shape))(*[int(d) for d in shape])


def lpmm_adamw4_nd_state_sizes(shape):
    sizes = (ctypes.c_size_t * 5)()
    dims = _dims(shape)
    _check(lib().lpmm_adamw4_nd_state_sizes(ctypes.addressof(dims), len(shape), ctypes.addressof(sizes)),
           "lpmm_adamw4_nd_state_sizes")
    return [int(s) for s in sizes]


def lpmm_adamw4_nd_state_zero(st: StateND, stream=None) -> None:
    dims = _dims(st.shape)
    _check(lib().lpmm_adamw4_nd_state_zero(_ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_codes), _ptr(st.v_row),
                                           _ptr(st.v_col), ctypes.addressof(dims), len(st.shape), _stream(stream)),
           "lpmm_adamw4_nd_state_zero")


def new_state_nd(shape, device="cuda") -> StateND:
    """Allocate (torch) and zero (library) the state of a tensor with 2..8 dimensions."""
    import torch
    shape = tuple(int(d) for d in shape)
    sz = lpmm_adamw4_nd_state_sizes(shape)
    pad4 = lambda n: (n + 3) // 4 * 4
    st = StateND(shape,
                 torch.empty(pad4(sz[0]), dtype=torch.uint8, device=device)[:sz[0]],
                 torch.empty(sz[1] // 4, dtype=torch.float32, device=device),
                 torch.empty(pad4(sz[2]), dtype=torch.uint8, device=device)[:sz[2]],
                 torch.empty(sz[3] // 4, dtype=torch.float32, device=device),
                 torch.empty(sz[4] // 4, dtype=torch.float32, device=device))
    lpmm_adamw4_nd_state_zero(st)
    return st


def _nd_step(fn_name, param, grad, st: StateND, lr, beta1, beta2, eps, weight_decay, step, stream):
    fn = getattr(lib(), fn_name)
    dims = _dims(st.shape)
    _check(fn(_ptr(param), _ptr(grad), _ptr(st.m_codes), _ptr(st.m_blockscale), _ptr(st.v_codes), _ptr(st.v_row),
              _ptr(st.v_col), ctypes.addressof(dims), len(st.shape), lr, beta1, beta2, eps, weight_decay, int(step),
              _stream(stream)), fn_name)


def lpmm_adamw4_nd_step(param, grad, st: StateND, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _nd_step("lpmm_adamw4_nd_step", param, grad, st, lr, beta1, beta2, eps, weight_decay, step, stream)


def lpmm_adamw4_nd_step_bf16g(param, grad, st: StateND, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _nd_step("lpmm_adamw4_nd_step_bf16g", param, grad, st, lr, beta1, beta2, eps, weight_decay, step, stream)


# ---- SGD with momentum, 4-bit momentum ------------------------------------------------------------------------

@dataclass
class StateSgdm:
    """The two device buffers of a flat tensor's compressed momentum."""
    numel: int
    m_codes: "object"
    m_blockscale: "object"


def lpmm_sgdm4_state_sizes(numel: int):
    sizes = (ctypes.c_size_t * 2)()
    _check(lib().lpmm_sgdm4_state_sizes(int(numel), ctypes.addressof(sizes)), "lpmm_sgdm4_state_sizes")
    return [int(s) for s in sizes]


def lpmm_sgdm4_state_zero(st: StateSgdm, stream=None) -> None:
    _check(lib().lpmm_sgdm4_state_zero(_ptr(st.m_codes), _ptr(st.m_blockscale), int(st.numel), _stream(stream)),
           "lpmm_sgdm4_state_zero")


def new_state_sgdm(numel: int, device="cuda") -> StateSgdm:
    import torch
    sz = lpmm_sgdm4_state_sizes(numel)
    st = StateSgdm(numel, torch.empty((sz[0] + 3) // 4 * 4, dtype=torch.uint8, device=device)[:sz[0]],
                   torch.empty(sz[1] // 4, dtype=torch.float32, device=device))
    lpmm_sgdm4_state_zero(st)
    return st


def lpmm_sgdm4_step(param, grad, st: StateSgdm, lr, momentum, stream=None):
    _check(lib().lpmm_sgdm4_step(_ptr(param), _ptr(grad), _ptr(st.m_codes), _ptr(st.m_blockscale), int(st.numel),
                                 lr, momentum, _stream(stream)), "lpmm_sgdm4_step")


def lpmm_sgdm4_step_bf16g(param, grad, st: StateSgdm, lr, momentum, stream=None):
    _check(lib().lpmm_sgdm4_step_bf16g(_ptr(param), _ptr(grad), _ptr(st.m_codes), _ptr(st.m_blockscale),
                                       int(st.numel), lr, momentum, _stream(stream)), "lpmm_sgdm4_step_bf16g")


def lpmm_sgdm32_step(param, grad, m, numel, grad_dtype, lr, momentum, stream=None):
    _check(lib().lpmm_sgdm32_step(_ptr(param), _ptr(grad), _ptr(m), int(numel), int(grad_dtype), lr, momentum,
                                  _stream(stream)), "lpmm_sgdm32_step")


def lpmm_sgdm4_step_multi(plan, lr, momentum, stream=None) -> None:
    _check(lib().lpmm_sgdm4_step_multi(_ptr(plan), lr, momentum, _stream(stream)), "lpmm_sgdm4_step_multi")


def make_desc_sgdm(param, grad, state, numel=None) -> "TensorDesc":
    """state: a StateSgdm (4-bit momentum) or one fp32 momentum tensor (then numel must be given)."""
    if isinstance(state, StateSgdm):
        return TensorDesc(_ptr(param), _ptr(grad), _ptr(state.m_codes), _ptr(state.m_blockscale), None, None, None,
                          1, state.numel, KIND_SGDM_4BIT, 0)
    return TensorDesc(_ptr(param), _ptr(grad), _ptr(state), None, None, None, None, 1, int(numel), KIND_SGDM_FP32, 0)


def lpmm_adamw32_step(param, grad, m, v, numel, grad_dtype, lr, beta1, beta2, eps, weight_decay, step,
                      stream=None):
    _check(lib().lpmm_adamw32_step(_ptr(param), _ptr(grad), _ptr(m), _ptr(v), int(numel),
                                   int(grad_dtype), lr, beta1, beta2, eps, weight_decay, int(step),
                                   _stream(stream)), "lpmm_adamw32_step")


def lpmm_dequant_state(which: int, codes, scale_a, scale_b, rows, cols, out, stream=None):
    shape = _shape(rows, cols)
    _check(lib().lpmm_dequant_state(int(which), _ptr(codes), _ptr(scale_a), _ptr(scale_b),
                                    ctypes.addressof(shape), _ptr(out), _stream(stream)),
           "lpmm_dequant_state")


def lpmm_quant_state(which: int, x, rows, cols, codes, scale_a, scale_b, stream=None):
    shape = _shape(rows, cols)
    _check(lib().lpmm_quant_state(int(which), _ptr(x), ctypes.addressof(shape), _ptr(codes),
                                  _ptr(scale_a), _ptr(scale_b), _stream(stream)),
           "lpmm_quant_state")


# ---- the ablation quantizers of the second moment ---------------------------------------------------------

NORM_B128, NORM_B2048, NORM_RANK1 = 0, 1, 2
MAP_DE, MAP_DE0, MAP_LINEAR = 0, 1, 2
ROUND_NEAREST, ROUND_STOCHASTIC = 0, 1


def lpmm_ablation_table(map_: int, is_signed: bool = False):
    import numpy as np
    out = np.zeros(16, np.float32)
    n = lib().lpmm_ablation_table(int(map_), int(is_signed), out.ctypes.data)
    _check(min(n, 0), "lpmm_ablation_table")
    return out[:n].copy()


def ablation_scale_sizes(norm: int, rows: int, cols: int):
    """Number of floats of scale_a and scale_b."""
    if norm == NORM_RANK1:
        return rows, cols
    B = 128 if norm == NORM_B128 else 2048
    return (rows * cols + B - 1) // B, 0


def lpmm_quant_ablation(norm, map_, is_signed, rounding, seed, x, rows, cols, codes, scale_a, scale_b, stream=None):
    shape = _shape(rows, cols)
    _check(lib().lpmm_quant_ablation(int(norm), int(map_), int(is_signed), int(rounding), int(seed), _ptr(x),
                                     ctypes.addressof(shape), _ptr(codes), _ptr(scale_a), _ptr(scale_b),
                                     _stream(stream)), "lpmm_quant_ablation")


def lpmm_dequant_ablation(norm, map_, is_signed, codes, scale_a, scale_b, rows, cols, out, stream=None):
    shape = _shape(rows, cols)
    _check(lib().lpmm_dequant_ablation(int(norm), int(map_), int(is_signed), _ptr(codes), _ptr(scale_a),
                                       _ptr(scale_b), ctypes.addressof(shape), _ptr(out), _stream(stream)),
           "lpmm_dequant_ablation")


# ---- many tensors in one call ------------------------------------------------------------------------

KIND_4BIT, KIND_FP32, KIND_4BIT_B128, KIND_4BIT_FACTOR, KIND_SGDM_4BIT, KIND_SGDM_FP32, KIND_4BIT_ND = 0, 1, 2, 3, 4, 5, 6
FLAG_NO_DECAY = 1
FLAG_DETERMINISTIC = 2


class TensorDesc(ctypes.Structure):
    """Mirror of lpmm_tensor_desc."""
    _fields_ = [("param", _VP), ("grad", _VP), ("m_state", _VP), ("m_blockscale", _VP), ("v_state", _VP),
                ("v_rowmax", _VP), ("v_colmax", _VP), ("rows", _I64), ("cols", _I64),
                ("kind", ctypes.c_int32), ("flags", ctypes.c_int32)]


def make_desc(param, grad, state, rows=None, cols=None, no_decay=False, deterministic=False) -> TensorDesc:
    """state: a State4 (4-bit, rank-1 second moment), a StateB128 (4-bit, block-wise second moment), a StateFactor
    (factorized second moment) or a (m, v) pair of fp32 tensors (then rows, cols must be given).
    no_decay: the plan's weight decay does not apply to this tensor."""
    flags = FLAG_NO_DECAY if no_decay else 0
    if deterministic:
        flags |= FLAG_DETERMINISTIC          # factorized tensors only: sums in a fixed order
    if isinstance(state, StateFactor):
        return TensorDesc(_ptr(param), _ptr(grad), _ptr(state.m_codes), _ptr(state.m_blockscale), None,
                          _ptr(state.v_row), _ptr(state.v_col), state.rows, state.cols, KIND_4BIT_FACTOR, flags)
    if isinstance(state, StateND):
        cols = 1
        for v in state.shape[1:]:
            cols *= int(v)
        d = TensorDesc(_ptr(param), _ptr(grad), _ptr(state.m_codes), _ptr(state.m_blockscale), _ptr(state.v_codes),
                       _ptr(state.v_row), _ptr(state.v_col), int(state.shape[0]), cols, KIND_4BIT_ND, flags)
        d.inner = tuple(int(v) for v in state.shape[1:])
        return d
    if isinstance(state, StateB128):
        return TensorDesc(_ptr(param), _ptr(grad), _ptr(state.m_codes), _ptr(state.m_blockscale),
                          _ptr(state.v_codes), _ptr(state.v_blockscale), None, 1, state.numel,
                          KIND_4BIT_B128, flags)
    if isinstance(state, State4):
        return TensorDesc(_ptr(param), _ptr(grad), _ptr(state.m_codes), _ptr(state.m_blockscale),
                          _ptr(state.v_codes), _ptr(state.v_rowmax), _ptr(state.v_colmax), state.rows,
                          state.cols, KIND_4BIT, flags)
    m, v = state
    return TensorDesc(_ptr(param), _ptr(grad), _ptr(m), None, _ptr(v), None, None, int(rows), int(cols),
                      KIND_FP32, flags)


def _inner_tables(descs):
    """Side tables for LPMM_KIND_4BIT_ND descriptors (their inner sizes ride on the Python object as `.inner`)."""
    if not any(getattr(d, "inner", None) for d in descs):
        return None, None, None
    dims = (ctypes.c_int64 * (7 * len(descs)))()
    ndim = (ctypes.c_int32 * len(descs))()
    for i, d in enumerate(descs):
        inner = getattr(d, "inner", None) or ()
        ndim[i] = len(inner)
        for r, v in enumerate(inner[:7]):       # more than 7 inner sizes: the count alone makes the library refuse
            dims[7 * i + r] = int(v)
    return dims, ndim, (ctypes.addressof(dims), ctypes.addressof(ndim))


def lpmm_adamw4_plan_bytes(descs) -> int:
    arr = (TensorDesc * len(descs))(*descs)
    dims, ndim, ptrs = _inner_tables(descs)
    if ptrs is None:
        return int(lib().lpmm_adamw4_plan_bytes(ctypes.addressof(arr), len(descs)))
    return int(lib().lpmm_adamw4_plan_bytes_nd(ctypes.addressof(arr), len(descs), *ptrs))


def lpmm_adamw4_plan_build(descs, grad_dtype: int, plan, stream=None) -> None:
    arr = (TensorDesc * len(descs))(*descs)
    nbytes = plan.numel() * plan.element_size()
    dims, ndim, ptrs = _inner_tables(descs)
    if ptrs is None:
        _check(lib().lpmm_adamw4_plan_build(ctypes.addressof(arr), len(descs), int(grad_dtype), _ptr(plan), nbytes,
                                            _stream(stream)), "lpmm_adamw4_plan_build")
    else:
        _check(lib().lpmm_adamw4_plan_build_nd(ctypes.addressof(arr), len(descs), *ptrs, int(grad_dtype), _ptr(plan),
                                               nbytes, _stream(stream)), "lpmm_adamw4_plan_build_nd")


def lpmm_adamw4_step_multi(plan, lr, beta1, beta2, eps, weight_decay, step, stream=None) -> None:
    _check(lib().lpmm_adamw4_step_multi(_ptr(plan), lr, beta1, beta2, eps, weight_decay, int(step),
                                        _stream(stream)), "lpmm_adamw4_step_multi")


def lpmm_adamw4_step_multi_capturable(plan, lr_dev, step_dev, beta1, beta2, eps, weight_decay, stream=None) -> None:
    """lr_dev: float32 tensor of one element on the device, step_dev: int64 tensor of one element on the device."""
    _check(lib().lpmm_adamw4_step_multi_capturable(_ptr(plan), _ptr(lr_dev), _ptr(step_dev), beta1, beta2, eps,
                                                   weight_decay, _stream(stream)), "lpmm_adamw4_step_multi_capturable")


def lpmm_sgdm4_step_multi_capturable(plan, lr_dev, momentum, stream=None) -> None:
    _check(lib().lpmm_sgdm4_step_multi_capturable(_ptr(plan), _ptr(lr_dev), momentum, _stream(stream)),
           "lpmm_sgdm4_step_multi_capturable")


def lpmm_adamw4_plan_release(plan) -> None:
    _check(lib().lpmm_adamw4_plan_release(_ptr(plan)), "lpmm_adamw4_plan_release")


def new_plan(descs, grad_dtype: int, device="cuda"):
    """Allocate (torch) and build a plan; returns the device buffer that is the plan."""
    import torch
    nbytes = lpmm_adamw4_plan_bytes(descs)
    if nbytes == 0:
        raise LpmmError("lpmm_adamw4_plan_bytes: invalid tensor list")
    plan = torch.zeros(nbytes, dtype=torch.uint8, device=device)
    lpmm_adamw4_plan_build(descs, grad_dtype, plan)
    torch.cuda.synchronize()
    return plan


def lpmm_profile_begin(max_calls: int) -> None:
    _check(lib().lpmm_profile_begin(int(max_calls)), "lpmm_profile_begin")


def lpmm_profile_end():
    """Returns (sum of pass-1 ms, sum of pass-2 ms, recorded calls)."""
    ms = (ctypes.c_double * 2)()
    n = ctypes.c_int64()
    _check(lib().lpmm_profile_end(ctypes.addressof(ms), ctypes.addressof(n)), "lpmm_profile_end")
    return float(ms[0]), float(ms[1]), int(n.value)
