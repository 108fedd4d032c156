"""Accuracy / OOB evaluation of compiled LUT layers on the GPU, in the shape of the paper's Tables 1 and 5.

    python -m paper_2601_03332_amd.evaluate [--seeds 5] [--batch 4096]

For the paper's controlled-sweep layer shape (Sec. 6.2 Case A: 10 -> 8, grid 8, cubic, value_repr =
spline_component, inputs N(0,1) clipped to the knot domain) it prints
  * in-range MAE / MaxAbs of the LUT layer against the fp32 B-spline layer for L in {16,32,64,128} and both
    quantisation schemes (Sec. 7.1, Table 1's protocol: closed + clip_x), and
  * the 2x2 boundary_mode x oob_policy matrix at L = 64 symmetric int8 (Sec. 7.4, Table 5's protocol): fraction
    of rows with any out-of-domain input, error on those rows, error on the in-range rows.
Both layers run as the library's HIP kernels; only the error statistics are taken with torch.  The layers are
randomly initialised here, so the absolute numbers are not the paper's; the trends are (error halves per
doubling of L; in-range error independent of the contract; half_open counts inputs clipped onto t_K as OOB).
"""
from __future__ import annotations

import argparse

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seeds", type=int, default=5)
    ap.add_argument("--batch", type=int, default=4096)
    args = ap.parse_args()
    import torch

    import paper_2601_03332_amd as lk
    from lutkan_inputs import ASYM_UINT8, CLIP_X, CLOSED, HALF_OPEN, SYM_INT8, ZERO_SPLINE, case_a

    dev = "cuda:0"

    def run(seed, L, scheme, boundary, oob):
        w = case_a(seed=seed, L=L, scheme=scheme, boundary=boundary, oob=oob, B=args.batch)
        s = w.layers[0]
        art = lk.lutkan_compile(s.d, s.m, s.G, s.p, s.ext_knots, s.coef, s.L, s.scheme, s.boundary, s.oob,
                                edge_scales=s.edge_scales)
        x = torch.from_numpy(w.x).to(dev)
        stats = torch.zeros(2, dtype=torch.int64, device=dev)
        y_lut = lk.lutkan_forward(art.to_device(dev), x, stats=stats)
        # reference: the un-quantised spline layer under closed + clip_x (every clipped input is in its domain)
        y_ref = lk.bspline_kan_forward(art.bspline_to_device(dev).with_contract(CLOSED, CLIP_X), x)
        lo, hi = float(art.knots[0]), float(art.knots[-1])
        inside = (x >= lo) & ((x <= hi) if boundary == CLOSED else (x < hi))
        row_in = inside.all(dim=1)
        err = (y_lut - y_ref).abs()
        e_in = err[row_in]
        e_out = err[~row_in]
        return dict(mae_in=float(e_in.mean()) if e_in.numel() else float("nan"),
                    max_in=float(e_in.max()) if e_in.numel() else float("nan"),
                    mae_oob=float(e_out.mean()) if e_out.numel() else float("nan"),
                    max_oob=float(e_out.max()) if e_out.numel() else float("nan"),
                    oob_any_frac=float(stats[1].item()) / x.shape[0])

    def agg(rows, key):
        v = np.array([r[key] for r in rows], dtype=np.float64)
        return f"{np.nanmean(v):.6f} +- {np.nanstd(v):.6f}" if np.isfinite(v).any() else "N/A"

    print(f"In-range error vs L (closed + clip_x, {args.seeds} seeds, batch {args.batch}) -- protocol of Table 1")
    print(f"{'L':>4} {'scheme':>10} {'MAE (in-range)':>24} {'MaxAbs (in-range)':>24}")
    for scheme, name in ((ASYM_UINT8, "asymmetric"), (SYM_INT8, "symmetric")):
        for L in (16, 32, 64, 128):
            rows = [run(seed, L, scheme, CLOSED, CLIP_X) for seed in range(args.seeds)]
            print(f"{L:>4} {name:>10} {agg(rows, 'mae_in'):>24} {agg(rows, 'max_in'):>24}")
    print()
    print("OOB matrix at L = 64 symmetric int8 -- protocol of Table 5 (rows with any out-of-domain input)")
    print(f"{'boundary':>10} {'policy':>12} {'OOB frac':>20} {'MAE (OOB rows)':>24} {'MaxAbs (OOB rows)':>24} {'MAE (in-range rows)':>24}")
    for boundary, bn in ((CLOSED, "closed"), (HALF_OPEN, "half_open")):
        for oob, on in ((CLIP_X, "clip_x"), (ZERO_SPLINE, "zero_spline")):
            rows = [run(seed, 64, SYM_INT8, boundary, oob) for seed in range(args.seeds)]
            print(f"{bn:>10} {on:>12} {agg(rows, 'oob_any_frac'):>20} {agg(rows, 'mae_oob'):>24} {agg(rows, 'max_oob'):>24} {agg(rows, 'mae_in'):>24}")


if __name__ == "__main__":
    main()
