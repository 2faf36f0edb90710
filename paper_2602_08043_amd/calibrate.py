#!/usr/bin/env python3
"""e_max calibration on the device, following the paper's "Practical calibration protocol"
(section 3.6): positive matrices with |N(1,1)| elements, the relative verification difference
max_i |E_i| / |checksum_i| over many trials at representative sizes, and e_max = that maximum
plus a 20 % safety margin.

The matrices are drawn on the device with torch's seeded generator (inputs only); E and the
checksum come from the library's own kernels (vabft_encode + vabft_gemm_verified_fused), so the
result reflects the accumulation order of these kernels on this GPU.

    python -m paper_2602_08043_amd.calibrate --dtype bf16 --sizes 256 1024 4096 --trials 200
"""
from __future__ import annotations

import argparse
import json
import math
import time

import torch

from . import binding as vb
from .session import VerifiedGemm

_TDT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32, "f64": torch.float64,
        "f8": torch.float8_e4m3fn}


def calibrate_one(dtype: str, M: int, N: int, K: int, transB: int, trials: int, seed: int = 0, dist: str = "abs_n_1_1",
                  max_seconds: float = 60.0):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    vg = VerifiedGemm(M, N, K, dtype, transB)
    e_default = vb.vabft_default_emax(dtype, K, N)
    worst_rel = 0.0
    worst_over_T = 0.0
    flagged = 0
    t0 = time.time()
    done = 0
    bshape = (N, K) if transB else (K, N)
    for _ in range(trials):
        if dist == "abs_n_1_1":
            A = (torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32) + 1.0).abs_().to(_TDT[dtype])
            B = (torch.randn(bshape, generator=g, device="cuda", dtype=torch.float32) + 1.0).abs_().to(_TDT[dtype])
        elif dist == "n_0_1":
            A = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32).to(_TDT[dtype])
            B = torch.randn(bshape, generator=g, device="cuda", dtype=torch.float32).to(_TDT[dtype])
        else:
            raise KeyError(dist)
        vg.run_fused(A, B, e_default)
        E = vg.E.double().abs()
        worst_rel = max(worst_rel, float((E / vg.expected.double().abs()).max()))
        worst_over_T = max(worst_over_T, float((E / vg.T.double()).max()))
        flagged += int(vg.nflag.item())
        done += 1
        if time.time() - t0 > max_seconds:
            break
    u = 2.0 ** -53 if dtype == "f64" else 2.0 ** -24
    return {"dtype": dtype, "M": M, "N": N, "K": K, "transB": transB, "dist": dist, "trials": done,
            "max_rel_E": worst_rel, "max_rel_E_over_u": worst_rel / u, "e_max_with_margin": 1.2 * worst_rel,
            "default_e_max": e_default, "max_E_over_T_at_default": worst_over_T, "flagged_rows_at_default": flagged}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="bf16", choices=sorted(_TDT))
    ap.add_argument("--sizes", type=int, nargs="+", default=[256, 512, 1024, 2048, 4096])
    ap.add_argument("--trials", type=int, default=100)
    ap.add_argument("--transB", type=int, default=0)
    ap.add_argument("--dist", default="abs_n_1_1")
    ap.add_argument("--max-seconds", type=float, default=40.0)
    args = ap.parse_args()
    rows = []
    for n in args.sizes:
        r = calibrate_one(args.dtype, n, n, n, args.transB, args.trials, seed=n, dist=args.dist,
                          max_seconds=args.max_seconds)
        rows.append(r)
        print(json.dumps(r), flush=True)
    # least-squares fit e = a*sqrt(n) + b of the margin-inclusive values (the paper's GPU law)
    if len(rows) >= 2:
        xs = [math.sqrt(r["K"]) for r in rows]
        ys = [r["e_max_with_margin"] for r in rows]
        mx, my = sum(xs) / len(xs), sum(ys) / len(ys)
        a = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
        print(json.dumps({"fit": "e_max = a*sqrt(n) + b", "a": a, "b": my - a * mx}))


if __name__ == "__main__":
    main()
