"""Quantization-error study of the second-moment quantizers that the paper ablates (Sec. 4.1, Tab. 1), on the GPU with
the library's own kernels (lpmm_quant_ablation / lpmm_dequant_ablation): normalization (B2048, B128, rank-1) x map
(DE with zero, DE-0, Linear) x rounding (nearest, stochastic as in App. D.3).

The input is a synthetic second moment built on the device: the moving average (beta2 = 0.999, 50 steps) of g^2 for
g_ij ~ N(0, sigma_j), sigma_j log-normal with 1 % of the columns ten times larger, i.e. outliers that persist in fixed
columns as the paper reports for real optimizer states (Sec. 3, App. B).  Reported per quantizer: the share of
entries that decompress to exactly zero, and how far h(v) = 1 / (sqrt(v) + 1e-6), the factor that scales Adam's
update (Sec. 4.1, "zero-point problem"), is off after the round trip.

    python -m paper_2309_01507_amd.quant_error_study [rows cols]
"""
from __future__ import annotations

import sys

from . import binding as B


def synthetic_second_moment(rows: int, cols: int, seed: int = 0, device="cuda:0"):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    sigma = 1e-3 * torch.exp(0.5 * torch.randn(cols, generator=gen, device=device))
    hot = torch.randperm(cols, generator=gen, device=device)[:max(1, cols // 100)]
    sigma[hot] *= 10.0
    v = torch.zeros(rows, cols, device=device)
    for _ in range(50):
        g = torch.randn(rows, cols, generator=gen, device=device) * sigma[None, :]
        v.mul_(0.999).addcmul_(g, g, value=0.001)
    return v


def roundtrip(v, norm: int, map_: int, stochastic: bool, seed: int = 1):
    import torch
    rows, cols = v.shape
    na, nb = B.ablation_scale_sizes(norm, rows, cols)
    codes = torch.empty(((v.numel() + 1) // 2 + 3) // 4 * 4, dtype=torch.uint8, device=v.device)
    sa = torch.empty(na, device=v.device)
    sb = torch.empty(max(nb, 1), device=v.device)
    out = torch.empty_like(v)
    B.lpmm_quant_ablation(norm, map_, False, B.ROUND_STOCHASTIC if stochastic else B.ROUND_NEAREST, seed,
                          v.reshape(-1), rows, cols, codes, sa, sb if nb else None)
    B.lpmm_dequant_ablation(norm, map_, False, codes, sa, sb if nb else None, rows, cols, out.reshape(-1))
    return out


def study(v):
    import torch
    h = lambda t: 1.0 / (torch.sqrt(t.double()) + 1e-6)
    rows = []
    for norm_name, norm in (("b2048", B.NORM_B2048), ("b128", B.NORM_B128), ("rank1", B.NORM_RANK1)):
        for map_name, map_ in (("de", B.MAP_DE), ("de0", B.MAP_DE0), ("linear", B.MAP_LINEAR)):
            for sr in (False, True):
                d = roundtrip(v, norm, map_, sr)
                off = torch.abs(torch.log10(h(d) / h(v)))
                rows.append({"norm": norm_name, "map": map_name, "rounding": "stochastic" if sr else "nearest",
                             "zero_share": float((d == 0).double().mean()),
                             "median_h_factor": float(10 ** off.reshape(-1).median()),
                             "share_h_off_2x": float((off > 0.30102999566).double().mean()),
                             "rel_err_v": float(torch.sqrt(((d.double() - v.double()) ** 2).sum() / (v.double() ** 2).sum()))})
    return rows


def main(argv):
    import torch
    rows, cols = (int(argv[1]), int(argv[2])) if len(argv) >= 3 else (4096, 4096)
    torch.cuda.set_device(0)
    B.ensure_init(rows + cols)
    v = synthetic_second_moment(rows, cols)
    print(f"synthetic second moment {rows} x {cols}")
    print("| normalization | map | rounding | entries -> 0 | median factor by which h is off | entries with h off by > 2x | rel. error of v |")
    print("|---|---|---|---|---|---|---|")
    for r in study(v):
        print(f"| {r['norm']} | {r['map']} | {r['rounding']} | {100 * r['zero_share']:.1f} % | "
              f"{r['median_h_factor']:.2f} | {100 * r['share_h_off_2x']:.1f} % | {r['rel_err_v']:.3f} |")


if __name__ == "__main__":
    main(sys.argv)
