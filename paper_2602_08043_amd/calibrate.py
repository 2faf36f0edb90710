#!/usr/bin/env python3
"""e_max calibration on the device, following the paper's "Practical calibration protocol"
(section 3.6): positive matrices with |N(1,1)| elements, the relative verification difference
max_i |E_i| / |checksum_i| over many trials at representative sizes, and e_max = that maximum
plus a 20 % safety margin.

The matrices are drawn on the device with torch's seeded generator (inputs only); E and the
checksum come from the library's own kernels (vabft_encode + vabft_gemm_verified_fused), so the
result reflects the accumulation order of these kernels on this GPU.

    python -m paper_2602_08043_amd.calibrate --dtype bf16 --sizes 256 1024 4096 --trials 100000 >> run.jsonl
    python -m paper_2602_08043_amd.calibrate --merge run1.jsonl run2.jsonl      # markdown table of the runs

One JSON line per (dtype, size, layout); lines of several runs with different --seed-offset values are merged
by --merge (trials add up, maxima combine).
"""
from __future__ import annotations

import argparse
import json
import math
import sys
import time

_U = {"f64": 2.0 ** -53}


def calibrate_one(dtype: str, M: int, N: int, K: int, transB: int, trials: int, seed: int = 0, dist: str = "abs_n_1_1",
                  max_seconds: float = 60.0):
    import torch

    from . import binding as vb
    from .session import VerifiedGemm

    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32, "f64": torch.float64,
           "f8": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}[dtype]
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    vg = VerifiedGemm(M, N, K, dtype, transB)
    e_default = vb.vabft_default_emax(dtype, K, N)
    # running maxima and the flag count stay on the device; the host looks at them every 64 trials
    worst_rel = torch.zeros((), dtype=torch.float64, device="cuda")
    worst_over_T = torch.zeros((), dtype=torch.float64, device="cuda")
    flagged = torch.zeros((), dtype=torch.int64, device="cuda")
    t0 = time.time()
    t_said = t0
    done = 0
    bshape = (N, K) if transB else (K, N)
    gen_dt = torch.float64 if dtype == "f64" else torch.float32
    while done < trials:
        if dist == "abs_n_1_1":
            A = torch.randn((M, K), generator=g, device="cuda", dtype=gen_dt).add_(1.0).abs_().to(tdt)
            B = torch.randn(bshape, generator=g, device="cuda", dtype=gen_dt).add_(1.0).abs_().to(tdt)
        elif dist == "n_0_1":
            A = torch.randn((M, K), generator=g, device="cuda", dtype=gen_dt).to(tdt)
            B = torch.randn(bshape, generator=g, device="cuda", dtype=gen_dt).to(tdt)
        else:
            raise KeyError(dist)
        vg.run_fused(A, B, e_default)
        E = vg.E.double().abs_()
        worst_rel = torch.maximum(worst_rel, (E / vg.expected.double().abs_()).max())
        worst_over_T = torch.maximum(worst_over_T, (E / vg.T.double()).max())
        flagged += vg.nflag[0]
        done += 1
        if done % 64 == 0:
            torch.cuda.synchronize()
            now = time.time()
            if now - t_said > 30.0:  # a progress line of the work itself, for whoever watches a long run
                print(f"calibrate: {dtype} n={K} transB={transB}: {done} trials, {now - t0:.0f} s", file=sys.stderr,
                      flush=True)
                t_said = now
            if now - t0 > max_seconds:
                break
    u = _U.get(dtype, 2.0 ** -24)
    wr = float(worst_rel.item())
    return {"dtype": dtype, "M": M, "N": N, "K": K, "transB": transB, "dist": dist, "trials": done, "seed": seed,
            "max_rel_E": wr, "max_rel_E_over_u": wr / u, "e_max_with_margin": 1.2 * wr,
            "default_e_max": e_default, "max_E_over_T_at_default": float(worst_over_T.item()),
            "flagged_rows_at_default": int(flagged.item()), "seconds": time.time() - t0}


def paper_law(dtype: str, n: int) -> float:
    """The paper's recommended GPU law (table "Recommended e_max across platforms", H100 rows)."""
    return 1.0e-17 * math.sqrt(n) + 2.5e-16 if dtype == "f64" else 5.0e-9 * math.sqrt(n) + 1.2e-7


def merge(paths):
    """Markdown table of the JSON lines of one or more runs: per (dtype, layout, n) the trials add up and the
    maxima combine."""
    acc = {}
    for path in paths:
        with open(path) as f:
            for line in f:
                line = line.strip()
                if not line.startswith("{"):
                    continue
                r = json.loads(line)
                if "dtype" not in r:
                    continue
                key = (r["dtype"], r["transB"], r["K"])
                a = acc.setdefault(key, {"trials": 0, "max_rel_E": 0.0, "flagged": 0, "over_T": 0.0, "default": None})
                a["trials"] += r["trials"]
                a["max_rel_E"] = max(a["max_rel_E"], r["max_rel_E"])
                a["flagged"] += r["flagged_rows_at_default"]
                a["over_T"] = max(a["over_T"], r["max_E_over_T_at_default"])
                a["default"] = r["default_e_max"]
    try:  # the default as the library computes it now (runs made before a change of the law recorded the old one)
        from . import binding as vb
        vb.load()
        current_default = vb.vabft_default_emax
    except (ImportError, OSError):
        current_default = None
    order = {"bf16": 0, "f16": 1, "f32": 2, "f64": 3, "f8": 4, "f8e5m2": 5}
    print("| dtype | B stored | n | trials | max rel. difference | in units of u | +20 % | paper law | library default "
          "| default / (+20 %) | flagged rows | max abs(E)/T during the run |")
    print("|---|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|")
    for (dt, tb, n) in sorted(acc, key=lambda k: (order.get(k[0], 9), k[1], k[2])):
        a = acc[(dt, tb, n)]
        u = _U.get(dt, 2.0 ** -24)
        m20 = 1.2 * a["max_rel_E"]
        if current_default is not None:
            a["default"] = current_default(dt, n, n)
        print(f"| {dt} | {'N x K' if tb else 'K x N'} | {n} | {a['trials']} | {a['max_rel_E']:.3e} | "
              f"{a['max_rel_E'] / u:.2f} | {m20:.3e} | {paper_law(dt, n):.3e} | {a['default']:.3e} | "
              f"{a['default'] / m20:.3f} | {a['flagged']} | {a['over_T']:.2f} |")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16", "f32", "f64", "f8", "f8e5m2"])
    ap.add_argument("--sizes", type=int, nargs="+", default=[256, 512, 1024, 2048, 4096])
    ap.add_argument("--trials", type=int, default=100)
    ap.add_argument("--transB", type=int, default=0)
    ap.add_argument("--dist", default="abs_n_1_1")
    ap.add_argument("--max-seconds", type=float, default=40.0, help="time cap per size")
    ap.add_argument("--seed-offset", type=int, default=0, help="added to the per-size seed n (a second run "
                    "of the same size draws fresh matrices)")
    ap.add_argument("--merge", nargs="+", help="JSON-lines files of earlier runs: print their merged table")
    args = ap.parse_args()
    if args.merge:
        merge(args.merge)
        return
    rows = []
    for n in args.sizes:
        r = calibrate_one(args.dtype, n, n, n, args.transB, args.trials, seed=n + args.seed_offset, dist=args.dist,
                          max_seconds=args.max_seconds)
        rows.append(r)
        print(json.dumps(r), flush=True)
    # least-squares fit e = a*sqrt(n) + b of the margin-inclusive values (the paper's GPU law)
    if len(rows) >= 2:
        xs = [math.sqrt(r["K"]) for r in rows]
        ys = [r["e_max_with_margin"] for r in rows]
        mx, my = sum(xs) / len(xs), sum(ys) / len(ys)
        a = sum((x - mx) * (y - my) for x, y in zip(xs, ys)) / sum((x - mx) ** 2 for x in xs)
        print(json.dumps({"fit": "e_max = a*sqrt(n) + b", "a": a, "b": my - a * mx}), file=sys.stderr)


if __name__ == "__main__":
    main()
