"""A synthetic quantization-error study of the second-moment quantizers that the paper ablates (Sec. 4.1, Tab. 1):
normalization (per tensor, B2048, B128, rank-1) x mapping (DE with zero, DE-0, Linear) x rounding (nearest,
stochastic as in App. D.3).  CPU only, numpy in fp64 on top of the oracle's tables; test infrastructure like the rest
of this directory (there is no GPU counterpart: none of these variants is on a step's path except Rank-1/Linear and
B128/Linear, which the oracle proper and the kernels implement).

What is measured, per quantizer, on a synthetic second moment: the share of entries that decompress to exactly 0,
and the error of h(v) = 1 / (sqrt(v) + 1e-6), the factor by which Adam's update direction scales (Sec. 4.1 "zero-point
problem").  Run as a script for the table:  python -m oracle.quant_error_study
"""
from __future__ import annotations

import numpy as np

from . import table_de, table_linear


def mapping(name: str) -> np.ndarray:
    """de: unsigned 4-bit dynamic-exponent map (contains 0); de0: the same without its zero (15 points, Sec. 4.1);
    linear: (i+1)/16."""
    if name == "de":
        return table_de(4, signed=False).astype(np.float64)
    if name == "de0":
        t = table_de(4, signed=False).astype(np.float64)
        return t[t > 0]
    if name == "linear":
        return table_linear(4).astype(np.float64)
    raise ValueError(name)


def scales(x: np.ndarray, norm: str) -> np.ndarray:
    """Per-element normalization scale of a non-negative matrix (Sec. 2.2 per-tensor and block-wise over the
    row-major flattening, Sec. 4.2 rank-1)."""
    if norm == "tensor":
        return np.full(x.shape, x.max())
    if norm.startswith("b"):
        B = int(norm[1:])
        flat = x.reshape(-1)
        nb = -(-flat.size // B)
        pad = np.zeros(nb * B)
        pad[:flat.size] = flat
        return np.repeat(pad.reshape(nb, B).max(axis=1), B)[:flat.size].reshape(x.shape)
    if norm == "rank1":
        return np.minimum(x.max(axis=1)[:, None], x.max(axis=0)[None, :])
    raise ValueError(norm)


def quantize(n: np.ndarray, T: np.ndarray, u: np.ndarray | None = None) -> np.ndarray:
    """Codes of normalized values n in [0, 1].  u is None: nearest entry, ties to the lower index (Sec. 2.2).
    u given (uniform numbers in [0, 1), one per element): stochastic rounding between the two neighbouring entries
    (App. D.3): the upper one with probability (n - T[q1]) / (T[q2] - T[q1]); values outside the table's range
    or on an entry have a single candidate."""
    hi = np.clip(np.searchsorted(T, n, side="left"), 0, T.size - 1)       # first entry >= n
    lo = np.clip(hi - 1, 0, T.size - 1)
    lo = np.where(T[hi] == n, hi, lo)                                      # n is an entry: one candidate
    lo = np.where(n < T[0], 0, lo)
    hi = np.where(n < T[0], 0, hi)
    hi = np.where(n > T[-1], T.size - 1, hi)
    lo = np.where(n > T[-1], T.size - 1, lo)
    if u is None:
        return np.where(np.abs(n - T[lo]) <= np.abs(T[hi] - n), lo, hi)
    gap = T[hi] - T[lo]
    p_up = np.where(gap > 0, (n - T[lo]) / np.where(gap > 0, gap, 1.0), 0.0)
    return np.where(u < p_up, hi, lo)


def roundtrip(x: np.ndarray, norm: str, map_name: str, u: np.ndarray | None = None) -> np.ndarray:
    T = mapping(map_name)
    s = scales(x, norm)
    n = np.divide(x, s, out=np.zeros_like(x), where=s > 0)
    return T[quantize(n, T, u)] * s


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
    return v


def h(v):
    return 1.0 / (np.sqrt(v) + 1e-6)


def study(v: np.ndarray, seed=1):
    rng = np.random.default_rng(seed)
    u = rng.random(v.shape)
    rows = []
    for norm in ("tensor", "b2048", "b128", "rank1"):
        for map_name in ("de", "de0", "linear"):
            for sr in (False, True):
                d = roundtrip(v, norm, map_name, u if sr else None)
                ratio = h(d) / h(v)
                rows.append({"norm": norm, "map": map_name, "rounding": "stochastic" if sr else "nearest",
                             "zero_share": float((d == 0).mean()),
                             "median_h_factor": float(10 ** np.median(np.abs(np.log10(ratio)))),
                             "share_h_off_2x": float((np.abs(np.log10(ratio)) > np.log10(2.0)).mean()),
                             "rel_err_v": float(np.sqrt(((d - v) ** 2).sum() / (v ** 2).sum()))})
    return rows


if __name__ == "__main__":
    v = synthetic_second_moment()
    print("| normalization | map | rounding | entries -> 0 | median factor by which h is off | entries with h off by > 2x | rel. error of v |")
    print("|---|---|---|---|---|---|---|")
    for r in study(v):
        print(f"| {r['norm']} | {r['map']} | {r['rounding']} | {100 * r['zero_share']:.1f} % | "
              f"{r['median_h_factor']:.2f} | {100 * r['share_h_off_2x']:.1f} % | {r['rel_err_v']:.3f} |")
