"""Seeded synthetic inputs for the 4-bit AdamW step: shapes, weights and gradients.

This module serves both the CPU oracle's tests and the GPU path's tests and benchmark, and for
that reason holds none of the optimizer's or the quantizers' arithmetic: only shapes, random
numbers and the bf16 storage format.  Every array is a pure function of
(run seed, purpose, tensor id, step), drawn from numpy's counter-based Philox generator.

The parameter sets imitate the transformer workloads the paper fine-tunes (its Tab. 4 models);
the gradient recipes imitate the outlier structure its Sec. 3 and App. B report for real moments
(outliers in fixed rows for some tensors and in fixed columns for others).  They stand in for the
paper's datasets and checkpoints, none of which is available here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

QUANT_MIN_NUMEL = 4096  # App. C.1 of the paper: tensors of size <= 4096 keep fp32 states

_PURPOSE = {"weight": 1, "grad": 2, "col_sigma": 3, "row_outlier": 4, "col_outlier": 5,
            "row_zero": 6, "grad_mean": 7}


def rng(seed: int, purpose: str, tensor_id: int = 0, step: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([int(seed), _PURPOSE[purpose], int(tensor_id), int(step)])
    return np.random.Generator(np.random.Philox(ss))


# ---- bf16 storage format (round-to-nearest-even on the fp32 bit pattern) ------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- parameter sets --------------------------------------------------------------------------

@dataclass(frozen=True)
class TensorSpec:
    name: str
    rows: int      # 1-D tensors have rows == 1
    cols: int
    ndim: int = 2

    @property
    def numel(self) -> int:
        return self.rows * self.cols

    @property
    def quantized(self) -> bool:
        """Paper's rule (App. C.1) as applied to the benchmark configurations: 2-D tensors above 4096 elements are
        quantized; 1-D biases / norm vectors keep fp32 states."""
        return self.ndim >= 2 and self.numel > QUANT_MIN_NUMEL


def _vec(name, n):
    return TensorSpec(name, 1, n, 1)


def param_set(config: str) -> List[TensorSpec]:
    """Tensor lists of the five workloads.  Matrices are (rows, cols) row-major."""
    out: List[TensorSpec] = []
    if config == "c1_single_1024":
        out.append(TensorSpec("w", 1024, 1024))
    elif config == "c2_bert_base":
        out.append(TensorSpec("embed", 30522, 768))
        for l in range(12):
            out += [TensorSpec(f"l{l}.qkv", 768, 2304), TensorSpec(f"l{l}.out", 768, 768),
                    TensorSpec(f"l{l}.fc1", 768, 3072), TensorSpec(f"l{l}.fc2", 3072, 768),
                    _vec(f"l{l}.qkv_b", 2304), _vec(f"l{l}.out_b", 768), _vec(f"l{l}.fc1_b", 3072),
                    _vec(f"l{l}.fc2_b", 768), _vec(f"l{l}.ln1_w", 768), _vec(f"l{l}.ln1_b", 768),
                    _vec(f"l{l}.ln2_w", 768), _vec(f"l{l}.ln2_b", 768)]
    elif config == "c3_outlier_32000x4096":
        out.append(TensorSpec("embed", 32000, 4096))
    elif config == "c4_gpt2_medium":
        out.append(TensorSpec("wte", 50257, 1024))
        for l in range(24):
            out += [TensorSpec(f"h{l}.qkv", 1024, 3072), TensorSpec(f"h{l}.proj", 1024, 1024),
                    TensorSpec(f"h{l}.fc", 1024, 4096), TensorSpec(f"h{l}.fc_proj", 4096, 1024),
                    _vec(f"h{l}.qkv_b", 3072), _vec(f"h{l}.proj_b", 1024), _vec(f"h{l}.fc_b", 4096),
                    _vec(f"h{l}.fc_proj_b", 1024), _vec(f"h{l}.ln1_w", 1024),
                    _vec(f"h{l}.ln1_b", 1024), _vec(f"h{l}.ln2_w", 1024), _vec(f"h{l}.ln2_b", 1024)]
        out += [_vec("ln_f_w", 1024), _vec("ln_f_b", 1024)]
    elif config == "c5_llama_7b":
        out.append(TensorSpec("embed", 32000, 4096))
        for l in range(32):
            out += [TensorSpec(f"l{l}.q", 4096, 4096), TensorSpec(f"l{l}.k", 4096, 4096),
                    TensorSpec(f"l{l}.v", 4096, 4096), TensorSpec(f"l{l}.o", 4096, 4096),
                    TensorSpec(f"l{l}.gate", 4096, 11008), TensorSpec(f"l{l}.up", 4096, 11008),
                    TensorSpec(f"l{l}.down", 11008, 4096),
                    _vec(f"l{l}.norm1", 4096), _vec(f"l{l}.norm2", 4096)]
        out += [_vec("norm_f", 4096), TensorSpec("lm_head", 32000, 4096)]
    else:
        raise KeyError(config)
    return out


CONFIGS = ("c1_single_1024", "c2_bert_base", "c3_outlier_32000x4096", "c4_gpt2_medium",
           "c5_llama_7b")
GRAD_RECIPE = {"c1_single_1024": "iid", "c2_bert_base": "col_lognormal",
               "c3_outlier_32000x4096": "outlier_sparse", "c4_gpt2_medium": "col_lognormal",
               "c5_llama_7b": "col_lognormal"}
GRAD_BF16 = {"c1_single_1024": False, "c2_bert_base": False, "c3_outlier_32000x4096": False,
             "c4_gpt2_medium": True, "c5_llama_7b": True}


# ---- weights and gradients -------------------------------------------------------------------

def weights(seed: int, tensor_id: int, rows: int, cols: int, std: float = 0.02) -> np.ndarray:
    g = rng(seed, "weight", tensor_id)
    return (g.standard_normal((rows, cols), dtype=np.float32) * np.float32(std)).astype(np.float32)


def col_sigma(seed: int, tensor_id: int, cols: int, median: float = 1e-3, s: float = 1.0):
    """Per-column gradient scale, lognormal(ln median, s), fixed for the whole run."""
    g = rng(seed, "col_sigma", tensor_id)
    return (np.float32(median) * np.exp(np.float32(s) * g.standard_normal(cols, dtype=np.float32))
            ).astype(np.float32)


def grads(seed: int, tensor_id: int, step: int, rows: int, cols: int, recipe: str = "iid",
          bf16: bool = False) -> np.ndarray:
    """Gradient of one tensor at one step, float32 (rows, cols).  With bf16=True the values are
    rounded to bf16 and returned upcast, i.e. exactly what a bf16 gradient buffer holds."""
    z = rng(seed, "grad", tensor_id, step).standard_normal((rows, cols), dtype=np.float32)
    if recipe == "iid":                      # config 1: N(0, 1e-3)
        out = z * np.float32(1e-3)
    elif recipe == "col_lognormal":          # configs 2, 4, 5: N(0, sigma_j), fixed-column outliers
        out = z * col_sigma(seed, tensor_id, cols)[None, :]
    elif recipe == "outlier_sparse":         # config 3
        out = z * np.float32(1e-4)
        n_r = max(1, rows // 100)            # 1 % of rows, fixed for the run
        n_c = max(1, cols // 200)            # 0.5 % of columns, fixed for the run
        hot_r = rng(seed, "row_outlier", tensor_id).choice(rows, n_r, replace=False)
        hot_c = rng(seed, "col_outlier", tensor_id).choice(cols, n_c, replace=False)
        out[hot_r, :] *= np.float32(1e3)
        out[:, hot_c] *= np.float32(1e3)
        # sparse-token pattern: a fresh 90 % of the rows is zero each step, on top of a fixed
        # 0.5 % of rows that never receive a gradient (they keep an all-zero state)
        never = rng(seed, "row_zero", tensor_id, 0).choice(rows, max(1, rows // 200), replace=False)
        zero = rng(seed, "row_zero", tensor_id, step + 1).random(rows) < 0.9
        zero[never] = True
        out[zero, :] = 0.0
    elif recipe == "drift":                  # long runs: a persistent mean that dies away under the column noise
        sig = col_sigma(seed, tensor_id, cols)[None, :]
        mean = rng(seed, "grad_mean", tensor_id).standard_normal((rows, cols), dtype=np.float32)
        out = (z + mean * np.float32(3.0 * np.exp(-step / 40.0))) * sig
    else:
        raise KeyError(recipe)
    out = np.ascontiguousarray(out, np.float32)
    if bf16:
        out = bf16_bits_to_f32(f32_to_bf16_bits(out)).reshape(rows, cols)
    return out
