"""A synthetic quantization-error study of the second-moment quantizers that the paper ablates (Sec. 4.1, Tab. 1):
normalization (B2048, B128, rank-1) x mapping (DE with zero, DE-0, Linear) x rounding (nearest, stochastic as in
App. D.3), on the CPU with the oracle's quantizers (oracle_quant_ablation / oracle_dequant_ablation).  Test
infrastructure like the rest of this directory; the GPU library has the same quantizers behind
lpmm_quant_ablation, and its own study script.

What is measured, per quantizer, on a synthetic second moment: the share of entries that decompress to exactly 0,
and the error of h(v) = 1 / (sqrt(v) + 1e-6), the factor by which Adam's update direction scales (Sec. 4.1 "zero-point
problem").  Run as a script for the table:  python -m oracle.quant_error_study
"""
from __future__ import annotations

import numpy as np

from . import dequant_ablation, quant_ablation


def roundtrip(x: np.ndarray, norm: str, map_name: str, stochastic: bool = False, seed: int = 0) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float32)
    codes, sa, sb = quant_ablation(x, norm, map_name, False, stochastic, seed)
    return dequant_ablation(codes, sa, sb, x.shape[0], x.shape[1], norm, map_name)


def synthetic_second_moment(rows=512, cols=1024, seed=0) -> np.ndarray:
    """EMA of g^2 over 50 steps for g_ij ~ N(0, sigma_j), sigma_j log-normal (spread 0.5) with 1 % of the columns
    10x larger: outliers that persist in fixed columns, one of the patterns Sec. 3 / App. B report for optimizer
    states."""
    rng = np.random.default_rng(seed)
    sigma = 1e-3 * np.exp(0.5 * rng.standard_normal(cols))
    sigma[rng.choice(cols, cols // 100, replace=False)] *= 10.0
    v = np.zeros((rows, cols))
    for _ in range(50):
        g = rng.standard_normal((rows, cols)) * sigma[None, :]
        v = 0.999 * v + 0.001 * g * g
    return v.astype(np.float32)


def h(v):
    return 1.0 / (np.sqrt(v.astype(np.float64)) + 1e-6)


def study(v: np.ndarray, seed=1):
    rows = []
    v64 = v.astype(np.float64)
    for norm in ("b2048", "b128", "rank1"):
        for map_name in ("de", "de0", "linear"):
            for sr in (False, True):
                d = roundtrip(v, norm, map_name, sr, seed)
                ratio = h(d) / h(v)
                rows.append({"norm": norm, "map": map_name, "rounding": "stochastic" if sr else "nearest",
                             "zero_share": float((d == 0).mean()),
                             "median_h_factor": float(10 ** np.median(np.abs(np.log10(ratio)))),
                             "share_h_off_2x": float((np.abs(np.log10(ratio)) > np.log10(2.0)).mean()),
                             "rel_err_v": float(np.sqrt(((d.astype(np.float64) - v64) ** 2).sum() / (v64 ** 2).sum()))})
    return rows


if __name__ == "__main__":
    v = synthetic_second_moment()
    print("| normalization | map | rounding | entries -> 0 | median factor by which h is off | entries with h off by > 2x | rel. error of v |")
    print("|---|---|---|---|---|---|---|")
    for r in study(v):
        print(f"| {r['norm']} | {r['map']} | {r['rounding']} | {100 * r['zero_share']:.1f} % | "
              f"{r['median_h_factor']:.2f} | {100 * r['share_h_off_2x']:.1f} % | {r['rel_err_v']:.3f} |")
