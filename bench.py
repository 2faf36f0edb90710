#!/usr/bin/env python3
"""Benchmark of the V-ABFT verified-GEMM hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: checksum encode of B (+ statistics), A-side statistics /
expected checksum / threshold, and the MFMA GEMM with the fused row-sum check.

Prints ONE JSON line: verified-GEMM TFLOP/s (whole path), with the roofline of the
dominant kernel (the GEMM, MFMA-bound), the CPU oracle timed on the host cores, and
the method's quality figures (ABFT overhead, false-positive rate, detection rate by
flipped bit, threshold / actual-difference ratio).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2516.6, "f16": 2516.6, "f8": 5033.2, "f32": 157.3, "f64": 78.6}  # MI355X dense matrix peaks
HBM_PEAK_GBPS = 8000.0
ELEM_BYTES = {"bf16": 2, "f16": 2, "f8": 1, "f32": 4, "f64": 8}
# HBM-side bytes per launch of the verified GEMM kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# scaled by the same counters on 1 GiB device copies (profiles/gemm16_fast_bf16_c2_4096_hbm_traffic.md).
# A counter figure cannot be taken live inside this script; workloads without a profile report null.
PROFILED_TRAFFIC_BYTES = {"c2_bf16_4096": (2.0 * 99887 + 1.0 * 35209) * 1024}

WORKLOAD_TEXT = {
    "c1_f32_256": "FP32 GEMM M=N=K=256, A,B ~ N(0,1), row-checksum V-ABFT check",
    "c2_bf16_4096": "BF16 GEMM M=N=K=4096, FP32 accumulation, A,B ~ N(0,1), B stored K x N, "
                    "fused check before output quantisation",
    "c3_bf16_ffn": "BF16 FFN GEMM M=4096 K=4096 N=11008, weights N(0,0.02) truncated 2 sigma in N x K layout, "
                   "activations N(0,1) with 1% outlier columns x20",
    "c4_f16_8192": "FP16 GEMM M=N=K=8192, A,B ~ U(-1,1), FP32 accumulation",
    "c5_f64_2048": "FP64 GEMM M=N=K=2048, A ~ N(0,1), B ~ N(0,1) truncated 3 sigma",
    "c6_f8_4096": "FP8 E4M3 GEMM M=N=K=4096, FP32 accumulation, FP16 output, A,B ~ N(0,1), B stored N x K "
                  "(not one of the five benchmark configurations)",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c2_bf16_4096", choices=sorted(WORKLOAD_TEXT))
    ap.add_argument("--quality-trials", type=int, default=40, help="fault-free trials for FPR / tightness")
    ap.add_argument("--flips-per-bit", type=int, default=16, help="single-bit-flip trials per bit position")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-quality", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of known size (reference for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path is built and measured on ONE GPU; run with --gpus 1 "
              "(the path shards without an exchange step -- by rows, by column blocks or by K -- but no multi-GPU figure exists)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    from paper_2602_08043_amd import binding as vb
    from paper_2602_08043_amd.session import VerifiedGemm, to_device

    vb.load()  # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = wl.make_config(args.config, seed=0)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    flops = 2.0 * M * N * K
    A, B = to_device(cfg["A"], dt), to_device(cfg["B"], dt)
    vg = VerifiedGemm(M, N, K, dt, tb)
    e_max = vb.vabft_default_emax(dt, K, N)

    def step():
        # S1..S3 travel as per-workgroup partials through the workspace; the fused call folds them
        vg.encode(B, defer_S=True)
        vg.gemm_fused(A, B, e_max, deferred_S=True)

    def timed(fn, steps, warmup, inner_events=None):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = torch.cuda.Event(enable_timing=True)
        t1 = torch.cuda.Event(enable_timing=True)
        t0.record()
        for i in range(steps):
            fn() if inner_events is None else fn(inner_events[i])
        t1.record()
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) / steps  # ms per step

    if args.copy_calibration:
        # 5 copies of 1 GiB (read 1 GiB + write 1 GiB each): the counters of these dispatches
        # (the runtime's device-to-device copy kernel) give the KiB-per-count factor
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- bring the GPU to its sustained clocks first (untimed, ~0.3 s of the same steps): the
    #      first milliseconds after idle run at different clocks than a long job does
    t_spin = time.time()
    while time.time() - t_spin < 0.3:
        for _ in range(20):
            step()
        torch.cuda.synchronize()

    # ---- the timed region: W untimed warm-up steps, then exactly K whole-path steps between
    #      two synchronisations
    ms_step = timed(step, args.steps, args.warmup)
    nflag_timed = int(vg.nflag.item())

    # ---- the dominant kernel's launch duration: the same K steps again with the GEMM launch
    #      bracketed by its own pair of events on the launch stream (kept out of the loop above
    #      because every event record costs a ~6 us bubble on this stack)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]

    def step_ev(pair):
        vg.encode(B, defer_S=True)
        pair[0].record()
        vg.gemm_fused(A, B, e_max, deferred_S=True)
        pair[1].record()

    ms_step_with_events = timed(step_ev, args.steps, 0, ev)
    gemm_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))

    # ---- same kernel without verification, and the steady-state (B pre-encoded) path
    ms_plain = timed(lambda: vg.gemm(A, B, 0), args.steps, args.warmup)

    ms_steady = timed(lambda: vg.gemm_fused(A, B, e_max, deferred_S=True), args.steps, args.warmup)

    vg.encode(B)  # the three-call route reads S1..S3 from their own buffer

    def three_call():
        vg.threshold(A, e_max)
        vg.gemm(A, B, 1)

    ms_three_call = timed(three_call, args.steps, args.warmup)
    ms_gemm_verified_only = timed(lambda: vg.gemm(A, B, 1), args.steps, args.warmup)

    # ---- position-weighted checksum route (detect + locate + correct): the same GEMM with the
    #      weighted row sums, and the small locate / correct pass
    vg.encode_weighted(B)
    vg.threshold_weighted(A, e_max)
    ms_gemm_weighted = timed(lambda: vg.gemm_weighted(A, B), args.steps, args.warmup)
    ms_locate = timed(lambda: vg.locate_correct(1), args.steps, args.warmup)
    ms_enc_w = timed(lambda: vg.encode_weighted(B), args.steps, args.warmup)
    ms_thr_w = timed(lambda: vg.threshold_weighted(A, e_max), args.steps, args.warmup)
    # ---- block-wise check (per block of W columns): the GEMM leaves partials, a small kernel compares
    vg.encode_blocks(B)
    vg.threshold_blocks(A)
    ms_gemm_blocks = timed(lambda: vg.gemm_blocks(A, B), args.steps, args.warmup)
    nblk_timed = int(vg.nblockflag.item())
    ms_enc_blocks = timed(lambda: vg.encode_blocks(B), args.steps, args.warmup)
    ms_thr_blocks = timed(lambda: vg.threshold_blocks(A), args.steps, args.warmup)

    # ---- row + column check in one launch
    vg.encode(B)
    vg.threshold(A, e_max)
    vg.encode_a(A)
    vg.threshold_cols(B)
    ms_gemm_rc = timed(lambda: vg.gemm_rc(A, B), args.steps, args.warmup)
    ncol_timed = int(vg.ncolflag.item())
    ms_enc_a = timed(lambda: vg.encode_a(A), args.steps, args.warmup)
    ms_thr_cols = timed(lambda: vg.threshold_cols(B), args.steps, args.warmup)
    vg.encode(B)
    vg.threshold(A, e_max)

    # ---- HBM-bound passes on rotating buffers (> 512 MB in total, so the 256 MB
    #      Infinity Cache cannot serve them)
    eb = ELEM_BYTES[dt]
    nrot = max(3, int(np.ceil(600e6 / (K * N * eb))) + 1)
    Bs = [B] + [B.clone() for _ in range(nrot - 1)]
    nrotA = max(3, int(np.ceil(600e6 / (M * K * eb))) + 1)
    As = [A] + [A.clone() for _ in range(nrotA - 1)]
    ctr = [0]

    def enc_rot():
        vg.encode(Bs[ctr[0] % nrot])
        ctr[0] += 1

    def thr_rot():
        vg.threshold(As[ctr[0] % nrotA], e_max)
        ctr[0] += 1

    def enc_def_rot():
        vg.encode(Bs[ctr[0] % nrot], defer_S=True)
        ctr[0] += 1

    ms_enc_def = timed(enc_def_rot, max(args.steps, 3 * nrot), nrot)
    ms_enc = timed(enc_rot, max(args.steps, 3 * nrot), nrot)
    ms_thr = timed(thr_rot, max(args.steps, 3 * nrotA), nrotA)
    del Bs, As
    vg.encode(B)
    vg.threshold(A, e_max)

    out = {
        "metric": "verified_gemm_tflops",
        "value": flops / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dt,
        "data": "synthetic",
        "config": {"workload": f"{args.config}: {WORKLOAD_TEXT[args.config]}", "M": M, "N": N, "K": K, "transB": tb,
                   "e_max": e_max, "c_sigma": 2.5,
                   "step": "vabft_encode(B, d_S=NULL) + vabft_gemm_verified_fused(A, B, d_S=NULL) [B-side checksum and "
                           "statistics; A-side statistics, fold of S1..S3, threshold, GEMM, row sums, compare/flag]"},
    }
    peak = PEAK_TFLOPS[dt]
    # average launch duration of the dominant kernel: K back-to-back launches of the fused call between two
    # HIP events on the launch stream (ms_steady).  Bracketing every single launch with its own event pair
    # (gemm_ms) adds the event records' own bubbles to each figure and reads 3 - 5 % longer than rocprofv3's
    # kernel trace; it is reported beside it.
    single_launch = ((dt in ("bf16", "f16") and M % 256 == 0 and N % 256 == 0 and K % 128 == 0) or
                     (dt in ("f32", "f64") and M % 128 == 0 and N % 128 == 0 and K % 16 == 0) or
                     (dt == "f8" and tb == 1 and M % 256 == 0 and N % 256 == 0 and N >= 512 and K % 256 == 0 and
                      (K // 256) // (N // 256) + 2 <= 8))
    # other cases (ragged shapes) run the A-side pass (and the compare) as launches of their own inside the
    # fused call: for them the dominant kernel is timed through the call that takes the threshold as an input
    ms_dom = ms_steady if single_launch else ms_gemm_verified_only
    achieved = flops / (ms_dom * 1e-3) / 1e12
    out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                       "traffic": PROFILED_TRAFFIC_BYTES.get(args.config),
                       "kernel": ("vabft_gemm_verified_fused launch (verified GEMM kernel)" if single_launch else
                                  "vabft_gemm_verified launch (verified GEMM kernel, threshold given)"),
                       "avg_launch_ms": ms_dom, "avg_launch_ms_single_event_pairs": gemm_ms}
    out["frac_of_peak_whole_path"] = out["value"] / peak
    out["plain_gemm_tflops"] = flops / (ms_plain * 1e-3) / 1e12
    out["overhead_pct"] = {"cold_encode_included": 100.0 * (ms_step / ms_plain - 1.0),
                           "steady_state_B_preencoded": 100.0 * (ms_steady / ms_plain - 1.0),
                           "three_call_route_B_preencoded": 100.0 * (ms_three_call / ms_plain - 1.0),
                           "check_with_given_threshold": 100.0 * (ms_gemm_verified_only / ms_plain - 1.0)}
    out["ms"] = {"plain_gemm": ms_plain, "verified_gemm_given_threshold": ms_gemm_verified_only,
                 "fused_call": ms_steady, "threshold_plus_gemm_calls": ms_three_call,
                 "encode_cold": ms_enc, "threshold_cold": ms_thr}
    out["hbm_passes"] = {
        "encode": {"GBps": K * N * eb / (ms_enc * 1e-3) / 1e9, "frac": K * N * eb / (ms_enc * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "encode_fold_deferred": {"GBps": K * N * eb / (ms_enc_def * 1e-3) / 1e9,
                                 "frac": K * N * eb / (ms_enc_def * 1e-3) / 1e9 / HBM_PEAK_GBPS, "ms": ms_enc_def},
        "threshold": {"GBps": M * K * eb / (ms_thr * 1e-3) / 1e9, "frac": M * K * eb / (ms_thr * 1e-3) / 1e9 / HBM_PEAK_GBPS},
    }
    out["weighted_route"] = {"ms_gemm_with_weighted_rowsums": ms_gemm_weighted, "ms_locate_correct": ms_locate,
                             "ms_encode_weighted_warm": ms_enc_w, "ms_threshold_weighted_warm": ms_thr_w,
                             "gemm_overhead_pct_vs_plain": 100.0 * (ms_gemm_weighted / ms_plain - 1.0)}
    out["row_column_route"] = {"ms_gemm_with_row_and_column_check": ms_gemm_rc, "ms_encode_a_warm": ms_enc_a,
                               "ms_threshold_cols_warm": ms_thr_cols,
                               "gemm_overhead_pct_vs_plain": 100.0 * (ms_gemm_rc / ms_plain - 1.0),
                               "column_flags_in_timed_region": ncol_timed}
    out["block_route"] = {"block_width": vg.W, "ms_gemm_with_block_check": ms_gemm_blocks,
                          "ms_encode_blocks_warm": ms_enc_blocks, "ms_threshold_blocks_warm": ms_thr_blocks,
                          "gemm_overhead_pct_vs_plain": 100.0 * (ms_gemm_blocks / ms_plain - 1.0),
                          "block_flags_in_timed_region": nblk_timed}
    out["flags_in_timed_region"] = nflag_timed
    out["ms"]["step_with_inner_events"] = ms_step_with_events

    # ---- method quality: FPR, tightness, detection rate by bit ------------------
    if not args.no_quality:
        t_q = time.time()
        g = torch.Generator(device="cuda")
        g.manual_seed(1234)
        tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32, "f64": torch.float64,
               "f8": torch.float8_e4m3fn}[dt]
        fp_rows = fp_trials = 0
        sumT = sumE = 0.0
        worst = 0.0
        n_ff = args.quality_trials
        for t in range(n_ff):
            if args.config == "c4_f16_8192":
                At = (torch.rand((M, K), generator=g, device="cuda", dtype=torch.float32) * 2 - 1).to(tdt)
                Bt = (torch.rand(B.shape, generator=g, device="cuda", dtype=torch.float32) * 2 - 1).to(tdt)
            else:
                At = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32).to(tdt)
                Bt = torch.randn(B.shape, generator=g, device="cuda", dtype=torch.float32).to(tdt)
                if args.config == "c3_bf16_ffn":
                    Bt = (Bt.float().clamp_(-2, 2) * 0.02).to(tdt)
            vg.run_fused(At, Bt, e_max)
            nf = int(vg.nflag.item())
            fp_rows += nf
            fp_trials += int(nf > 0)
            Tm, Em = vg.T.double(), vg.E.double().abs()
            sumT += float(Tm.mean())
            sumE += float(Em.mean())
            worst = max(worst, float((Em / Tm).max()))
            if time.time() - t_q > 60:
                n_ff = t + 1
                break
        out["quality"] = {"fault_free_trials": n_ff, "false_positive_trials": fp_trials,
                          "false_positive_rows": fp_rows, "fpr": fp_trials / n_ff,
                          "threshold_over_actual_mean": sumT / max(sumE, 1e-300),
                          "worst_row_E_over_T": worst,
                          "inputs": "fresh seeded device-generated matrices of the configuration's distribution"}
        # detection rate by bit: single flips at seeded (i, j) on the configuration's own inputs
        # (through the weighted route, so the same runs also give the localisation rate: a flip counts
        # as located when the reported column is the injected one)
        vg.encode_weighted(B)
        vg.threshold_weighted(A, e_max)
        rng = np.random.Generator(np.random.Philox(key=[2024, 7]))
        bits = list(range(52, 64)) if dt == "f64" else list(range(16, 32))
        dr, lr = {}, {}
        for bit in bits:
            det = located = tot = 0
            for _ in range(args.flips_per_bit):
                i, j = int(rng.integers(0, M)), int(rng.integers(0, N))
                inj = vg.make_inject(mode=1, faults=[(i, j, bit)])
                vg.gemm_weighted(A, B, inj)
                vg.locate_correct(1)
                fl = int(vg.flags[i].item())
                det += fl
                located += int(fl and int(vg.loc[i].item()) == j)
                tot += 1
            dr[str(bit)] = det / tot
            lr[str(bit)] = located / tot
            if time.time() - t_q > 150:
                break
        out["quality"]["detection_rate_by_acc_bit"] = dr
        out["quality"]["localisation_rate_by_acc_bit"] = lr
        out["quality"]["flips_per_bit"] = args.flips_per_bit
        vg.encode(B)
        vg.threshold(A, e_max)

    # ---- offline (post-quantisation) mode on the paper's BF16 tightness-table workloads: U(0,1),
    #      n x n x n, e_max = 2 u_output, plain GEMM followed by the post-hoc check of the stored C
    if not args.no_quality and dt == "bf16":
        g2 = torch.Generator(device="cuda")
        g2.manual_seed(4321)
        table = {}
        for n in (128, 256, 512, 1024, 2048):
            vo = VerifiedGemm(n, n, n, "bf16", 0)
            e_off = vb.vabft_default_emax_offline("bf16", n, n)
            sT = sE = 0.0
            fp = 0
            trials = 50
            for _ in range(trials):
                Ao = torch.rand((n, n), generator=g2, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                Bo = torch.rand((n, n), generator=g2, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                vo.run_offline(Ao, Bo, e_off)
                fp += int(vo.nflag.item() > 0)
                sT += float(vo.T.double().mean())
                sE += float(vo.E.double().abs().mean())
            table[str(n)] = {"threshold_mean": sT / trials, "actual_diff_mean": sE / trials,
                             "tightness": sT / max(sE, 1e-300), "false_positive_trials": fp, "trials": trials}
        out["quality"]["offline_bf16_uniform01"] = {"e_max": vb.vabft_default_emax_offline("bf16", 128, 128),
                                                    "by_size": table}

    # ---- the CPU oracle timed on the host cores (bounded: one full trial of the workload)
    if not args.no_cpu_baseline:
        from oracle import vabft_oracle as orc
        rows = None
        sample = "one full trial (all rows) of the workload"
        if flops > 3e11:  # keep the default run short: product on a row sample, everything else complete
            nrows = max(64, int(M * 3e11 / flops))
            rows = np.arange(nrows)
            sample = f"first {nrows} of {M} rows of the product (statistics, checksums, thresholds for all rows)"
        # repeat whole oracle passes until about 10 s of host time have been spent
        t0 = time.time()
        n_pass = 0
        while True:
            o = orc.verify(cfg["A"], cfg["B"], dt, tb, e_max=e_max, rows=rows)
            n_pass += 1
            t_cpu = time.time() - t0
            if t_cpu >= 10.0 or n_pass >= 100000:
                break
        done_flops = (flops if rows is None else flops * len(rows) / M) * n_pass
        sample = f"{n_pass} x " + sample
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": done_flops / t_cpu / 1e12, "unit": "TFLOP/s", "cores": int(cores),
                               "kind": "oracle", "sample": sample, "seconds": t_cpu,
                               "oracle_flags": int(o["flags"].sum())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
