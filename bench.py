#!/usr/bin/env python3
"""Benchmark of the V-ABFT verified-GEMM hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: checksum encode of B (+ statistics), A-side statistics /
expected checksum / threshold, and the MFMA GEMM with the fused row-sum check.

Prints ONE JSON line.  Its top level is the headline workload (benchmark configuration 2,
BF16 4096^3): verified-GEMM TFLOP/s of the whole path, the roofline of the dominant kernel
(the GEMM, MFMA-bound), the CPU oracle timed on the host cores, and the method's quality
figures.  `configs` holds the same report for each of the five benchmark configurations
(configuration 5 with both of its B matrices): TFLOP/s and fraction of the dtype's dense peak,
ABFT overhead against the same kernel without verification (cold / steady state / check
only), false-positive rate, detection rate by flipped accumulator bit, threshold / actual
difference ratio, and the oracle's time on a bounded sample.
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

PEAK_TFLOPS = {"bf16": 2516.6, "f16": 2516.6, "f8": 5033.2, "f8e5m2": 5033.2, "f32": 157.3, "f64": 78.6}  # MI355X dense matrix peaks
HBM_PEAK_GBPS = 8000.0
ELEM_BYTES = {"bf16": 2, "f16": 2, "f8": 1, "f8e5m2": 1, "f32": 4, "f64": 8}
# Bytes per launch of the verified GEMM kernel that crossed the L2 boundary, from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE scaled by the same counters on 1 GiB device copies (profiles/verified_gemm_c1_to_c5_hbm_traffic.md, one
# table per workload; the bytes are served by the Infinity Cache or by HBM, the counter does not tell which).  A counter figure cannot be taken live inside this script; workloads without a profile report null.
PROFILED_TRAFFIC_BYTES = {"c1_f32_256": 2062399, "c2_bf16_4096": 239404586, "c3_bf16_ffn": 688285063,
                          "c4_f16_8192": 1762836180, "c5_f64_2048": 238568149}

HEADLINE = "c2_bf16_4096"
WORKLOAD_TEXT = {
    "c1_f32_256": "FP32 GEMM M=N=K=256, A,B ~ N(0,1), row-checksum V-ABFT check",
    "c2_bf16_4096": "BF16 GEMM M=N=K=4096, FP32 accumulation, A,B ~ N(0,1), B stored K x N, "
                    "fused check before output quantisation",
    "c3_bf16_ffn": "BF16 FFN GEMM M=4096 K=4096 N=11008, weights N(0,0.02) truncated 2 sigma in N x K layout, "
                   "activations N(0,1) with 1% outlier columns x20",
    "c4_f16_8192": "FP16 GEMM M=N=K=8192, A,B ~ U(-1,1), FP32 accumulation, Bernoulli accumulator flips 1e-6",
    "c5_f64_2048": "FP64 GEMM M=N=K=2048, A ~ N(0,1), B ~ N(0,1) truncated 3 sigma (variant 0) or U(0,1) (variant 1)",
    "c6_f8_4096": "FP8 E4M3 GEMM M=N=K=4096, FP32 accumulation, FP16 output, A,B ~ N(0,1), B stored N x K "
                  "(not one of the five benchmark configurations)",
    "c8_f8e5m2_4096": "FP8 E5M2 GEMM M=N=K=4096, FP32 accumulation, FP16 output, A,B ~ N(0,1), B stored N x K "
                      "(not one of the five benchmark configurations)",
    "c7_f32_4096": "FP32 GEMM M=N=K=4096, A,B ~ N(0,1) (not one of the five benchmark configurations: the FP32 kernel "
                   "at a size bound by the matrix instruction)",
}
# trials of the quality statistics (the benchmark configurations' own counts; configuration 1 names one fault-free
# run and 8 flips, more are run because they are free at that size)
FAULT_FREE_TRIALS = {"c1_f32_256": 200, "c2_bf16_4096": 1000, "c3_bf16_ffn": 100, "c4_f16_8192": 20,
                     "c5_f64_2048": 500, "c6_f8_4096": 40, "c7_f32_4096": 40, "c8_f8e5m2_4096": 40}
FLIP_TRIALS = {"c1_f32_256": 176, "c2_bf16_4096": 1008, "c3_bf16_ffn": 112, "c4_f16_8192": 32,
               "c5_f64_2048": 132, "c6_f8_4096": 64, "c7_f32_4096": 64, "c8_f8e5m2_4096": 64}


def timed(torch, fn, steps, warmup):
    """ms per call: `warmup` untimed calls, then exactly `steps` calls between two events and a synchronisation."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(steps):
        fn()
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / steps


def spin_up(torch, fn, seconds=0.3):
    """Bring the GPU to its sustained clocks first (untimed): the first milliseconds after idle run at different
    clocks than a long job does."""
    t = time.time()
    while time.time() - t < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()


def mfma_probe_tflops(torch, vb, dt, cache={}):
    """Sustained rate of a register-only loop of the GEMM's matrix instruction on random operands."""
    if dt in cache or dt in ("f8", "f8e5m2"):
        return cache.get(dt)
    out = torch.empty(65536, dtype=torch.float32, device="cuda")
    iters = {"bf16": 2000, "f16": 2000, "f32": 1000, "f64": 500}[dt]
    flops = [0.0]

    def launch():
        flops[0] = vb.vabft_probe_mfma(dt, iters, out.data_ptr(), torch.cuda.current_stream().cuda_stream)

    spin_up(torch, launch, 0.25)
    ms = timed(torch, launch, 30, 5)
    cache[dt] = flops[0] / (ms * 1e-3) / 1e12
    return cache[dt]


def quality(torch, np, wl, vb, vg, name, variant, A, B, e_max, n_ff, n_flip, budget_s):
    """False-positive rate and tightness on fresh matrices of the configuration's distribution; detection and
    localisation rate by flipped accumulator bit on the configuration's own inputs."""
    dt, M, N = vg.dtype, vg.M, vg.N
    t_q = time.time()
    g = torch.Generator(device="cuda")
    g.manual_seed(1234 + 17 * variant)
    fp_trials = torch.zeros((), dtype=torch.int64, device="cuda")
    fp_rows = torch.zeros((), dtype=torch.int64, device="cuda")
    sumT = torch.zeros((), dtype=torch.float64, device="cuda")
    sumE = torch.zeros((), dtype=torch.float64, device="cuda")
    worst = torch.zeros((), dtype=torch.float64, device="cuda")
    done = 0
    for t in range(n_ff):
        At, Bt = wl.device_trial(name, g, variant)
        vg.run_fused(At, Bt, e_max)
        nf = vg.nflag[0].to(torch.int64)
        fp_rows += nf
        fp_trials += (nf > 0).to(torch.int64)
        Tm, Em = vg.T.double(), vg.E.double().abs_()
        sumT += Tm.mean()
        sumE += Em.mean()
        worst = torch.maximum(worst, (Em / Tm).max())
        done += 1
        if done % 16 == 0:
            torch.cuda.synchronize()
            if time.time() - t_q > budget_s:
                break
    q = {"fault_free_trials": done, "false_positive_trials": int(fp_trials.item()),
         "false_positive_rows": int(fp_rows.item()), "fpr": float(fp_trials.item()) / max(done, 1),
         "threshold_over_actual_mean": float(sumT.item()) / max(float(sumE.item()), 1e-300),
         "worst_row_E_over_T": float(worst.item()),
         "inputs": "fresh seeded device-generated matrices of the configuration's distribution (workloads.device_trial)"}
    # ---- single flips at seeded (i, j), stratified over the accumulator bits, through the weighted route (so the
    #      same runs give the localisation rate: a flip counts as located when the reported column is the injected one)
    vg.encode_weighted(B)
    vg.threshold_weighted(A, e_max)
    rng = np.random.Generator(np.random.Philox(key=[2024, 7 + variant]))
    if name == "c1_f32_256":
        bits = list(range(20, 31))      # "exponent or high mantissa"
    elif dt == "f64":
        bits = list(range(52, 63))
    else:
        bits = list(range(16, 32))
    per_bit = max(1, n_flip // len(bits))
    det = torch.zeros(len(bits), dtype=torch.int64, device="cuda")
    loc = torch.zeros(len(bits), dtype=torch.int64, device="cuda")
    tot = [0] * len(bits)
    t_f = time.time()
    for r in range(per_bit):
        for b, bit in enumerate(bits):
            i, j = int(rng.integers(0, M)), int(rng.integers(0, N))
            inj = vg.make_inject(mode=1, faults=[(i, j, bit)])
            vg.gemm_weighted(A, B, inj)
            vg.locate_correct(1)
            fl = vg.flags[i].to(torch.int64)
            det[b] += fl
            loc[b] += fl * (vg.loc[i] == j).to(torch.int64)
            tot[b] += 1
        torch.cuda.synchronize()
        if time.time() - t_f > budget_s:
            break
    det_h, loc_h = det.tolist(), loc.tolist()
    q["single_flip_trials"] = int(sum(tot))
    q["flips_per_bit"] = tot[0]
    q["detection_rate_by_acc_bit"] = {str(bit): det_h[b] / max(tot[b], 1) for b, bit in enumerate(bits)}
    q["localisation_rate_by_acc_bit"] = {str(bit): loc_h[b] / max(tot[b], 1) for b, bit in enumerate(bits)}
    q["detection_rate_all_bits"] = sum(det_h) / max(sum(tot), 1)
    if name == "c4_f16_8192":
        # the configuration's own fault model: Bernoulli flips at 1e-6 per element on accumulator bits 16..31
        vg.encode(B)
        hit = miss = big = big_det = 0
        n_trials = 0
        for t in range(n_ff):
            inj = vg.make_inject(mode=2, seed=777 + t, rate=1e-6, bit_lo=16, bit_hi=31)
            vg.gemm_fused(A, B, e_max, inj=inj)
            r_flags = vg.flags.cpu().numpy()
            T_h = vg.T.cpu().numpy()
            n, recs = vg.inject_records()
            rows = {}
            for (i, _j, _b, before, after) in recs:
                rows.setdefault(i, []).append(abs(after - before))
            for i, ds in rows.items():
                d = max(ds)
                f = int(r_flags[i])
                hit += f
                miss += 1 - f
                if not (d < 10 * T_h[i]):
                    big += 1
                    big_det += f
            n_trials += 1
            if time.time() - t_f > 2 * budget_s:
                break
        q["bernoulli_1e-6"] = {"trials": n_trials, "rows_with_flips": hit + miss, "rows_flagged": hit,
                               "rows_with_a_flip_of_at_least_10T": big, "of_those_flagged": big_det}
    vg.encode(B)
    vg.threshold(A, e_max)
    return q


def oracle_time(np, wl, cfg, e_max, seconds):
    """The CPU oracle on the host cores, on a bounded sample of the workload (whole oracle passes are repeated
    until `seconds` of host time are spent)."""
    from oracle import vabft_oracle as orc
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    flops = 2.0 * M * N * K
    rows = None
    sample = "one full trial (all rows) of the workload"
    if flops > 3e11:  # keep the run short: product on a row sample, everything else complete
        nrows = max(64, int(M * 3e11 / flops))
        rows = np.arange(nrows)
        sample = f"first {nrows} of {M} rows of the product (statistics, checksums, thresholds for all rows)"
    t0 = time.time()
    n_pass = 0
    while True:
        o = orc.verify(cfg["A"], cfg["B"], dt, tb, e_max=e_max, rows=rows)
        n_pass += 1
        t_cpu = time.time() - t0
        if t_cpu >= seconds or n_pass >= 100000:
            break
    done_flops = (flops if rows is None else flops * len(rows) / M) * n_pass
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": done_flops / t_cpu / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_pass} x " + sample, "seconds": t_cpu, "oracle_flags": int(o["flags"].sum())}


def bench_config(mods, name, variant, steps, warmup, args, headline):
    torch, np, wl, vb, VerifiedGemm, to_device = mods
    cfg = wl.make_config(name, seed=0, variant=variant)
    dt, M, N, K, tb = cfg["dtype"], cfg["M"], cfg["N"], cfg["K"], cfg["transB"]
    flops = 2.0 * M * N * K
    A, B = to_device(cfg["A"], dt), to_device(cfg["B"], dt)
    vg = VerifiedGemm(M, N, K, dt, tb)
    e_max = vb.vabft_default_emax(dt, K, N)
    peak = PEAK_TFLOPS[dt]

    def step():
        # S1..S3 travel as per-workgroup partials through the workspace; the fused call folds them
        vg.encode(B, defer_S=True)
        vg.gemm_fused(A, B, e_max, deferred_S=True)

    spin_up(torch, step)
    # keep every timed loop of the larger workloads to a fraction of a second
    probe_ms = timed(torch, step, 5, 2)
    if not headline:
        steps = int(min(steps, max(10, 0.25e3 / probe_ms)))
        warmup = int(min(warmup, max(3, steps // 5)))
    # ---- the timed region: W untimed warm-up steps, then exactly K whole-path steps between two synchronisations
    ms_step = timed(torch, step, steps, warmup)
    nflag_timed = int(vg.nflag.item())
    # ... and K back-to-back launches of the fused call alone (the roofline's launch duration)
    ms_steady = timed(torch, lambda: vg.gemm_fused(A, B, e_max, deferred_S=True), steps, warmup)

    # ---- the overhead figures.  The chip's clock under matrix load follows its power draw with a lag of many
    # launches, so two loops timed one after the other sit in different states and their ratio drifts by several
    # percent either way.  The routes are therefore timed in interleaved rounds (every route sees the same state)
    # and compared by their medians.  Both forms of S1..S3 are in place at once: folded in vg.S for the calls that
    # read it, as partials in the workspace for the fused call.
    vg.encode(B)
    vg.threshold(A, e_max)
    vg.encode(B, defer_S=True)

    def three_call():
        vg.threshold(A, e_max)
        vg.gemm(A, B, 1)

    routes = {"step": step, "plain": lambda: vg.gemm(A, B, 0),
              "fused": lambda: vg.gemm_fused(A, B, e_max, deferred_S=True), "check": lambda: vg.gemm(A, B, 1),
              "three_call": three_call}
    rounds = 9
    per_round = max(5, steps // rounds)
    samples = {k: [] for k in routes}
    for _ in range(rounds):
        for k, fn in routes.items():
            samples[k].append(timed(torch, fn, per_round, 2))
    med = {k: float(np.median(v)) for k, v in samples.items()}
    ms_plain, ms_check, ms_three_call = med["plain"], med["check"], med["three_call"]
    ms_fused_il, ms_step_il = med["fused"], med["step"]
    # The other fair comparison: every route brought to its own sustained state first (a quarter of a second of
    # nothing but that route), then timed; the plain GEMM at both ends.  A route whose launches contain waits
    # draws less power and holds a higher clock in its matrix phases, so these ratios come out below the
    # interleaved ones: this is what a job that runs one route all day sees.
    own = {}
    for k in ("plain", "check", "fused", "three_call", "step", "plain_again"):
        fn = routes["plain" if k == "plain_again" else k]
        spin_up(torch, fn, 0.25)
        own[k] = timed(torch, fn, steps, warmup)
    own_plain = 0.5 * (own["plain"] + own["plain_again"])
    vg.encode(B)
    vg.threshold(A, e_max)

    single_launch = ((dt in ("bf16", "f16") and M % 256 == 0 and N % 256 == 0 and K % 128 == 0) or
                     (dt in ("f32", "f64") and M % 128 == 0 and N % 128 == 0 and K % 16 == 0) or
                     (dt in ("f8", "f8e5m2") and tb == 1 and M % 256 == 0 and N % 256 == 0 and N >= 512 and K % 256 == 0 and
                      (K // 256) // (N // 256) + 2 <= 8))
    ms_dom = ms_steady if single_launch else ms_check
    achieved = flops / (ms_dom * 1e-3) / 1e12
    probe = mfma_probe_tflops(torch, vb, dt)
    tag = name if name != "c5_f64_2048" else f"{name}_v{variant}"
    out = {
        "name": tag,
        "workload": f"{name}: {WORKLOAD_TEXT[name]}" + (f" [B variant {variant}]" if name == "c5_f64_2048" else ""),
        "dtype": dt, "M": M, "N": N, "K": K, "transB": tb, "e_max": e_max, "c_sigma": 2.5,
        "value": flops / (ms_step * 1e-3) / 1e12, "unit": "TFLOP/s", "steps": steps, "warmup": warmup,
        "ms_per_step": ms_step, "frac_of_peak_whole_path": flops / (ms_step * 1e-3) / 1e12 / peak,
        # average launch duration of the dominant kernel: K back-to-back launches of the fused call between two
        # HIP events on the launch stream (an event pair around every single launch adds the records' own bubbles)
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": PROFILED_TRAFFIC_BYTES.get(name),
                     "kernel": ("vabft_gemm_verified_fused launch (verified GEMM kernel)" if single_launch else
                                "vabft_gemm_verified launch (verified GEMM kernel, threshold given)"),
                     "avg_launch_ms": ms_dom,
                     "measured_mfma_loop_tflops": probe,
                     "frac_of_measured_mfma_loop": (achieved / probe) if probe else None},
        "plain_gemm_tflops": flops / (own_plain * 1e-3) / 1e12,
        "plain_gemm_frac_of_peak": flops / (own_plain * 1e-3) / 1e12 / peak,
        # every route in its own sustained state (see above), against the plain GEMM in its own
        "overhead_pct": {"cold_encode_included": 100.0 * (own["step"] / own_plain - 1.0),
                         "steady_state_B_preencoded": 100.0 * (own["fused"] / own_plain - 1.0),
                         "three_call_route_B_preencoded": 100.0 * (own["three_call"] / own_plain - 1.0),
                         "check_with_given_threshold": 100.0 * (own["check"] / own_plain - 1.0),
                         "method": "each route timed after a quarter of a second of nothing but that route; the plain "
                                   "GEMM at both ends"},
        # ratios of medians over interleaved rounds of all routes: every route in the same (mixed) state, in which
        # the plain GEMM runs faster than it does on its own
        "overhead_pct_interleaved_rounds": {
            "cold_encode_included": 100.0 * (ms_step_il / ms_plain - 1.0),
            "steady_state_B_preencoded": 100.0 * (ms_fused_il / ms_plain - 1.0),
            "three_call_route_B_preencoded": 100.0 * (ms_three_call / ms_plain - 1.0),
            "check_with_given_threshold": 100.0 * (ms_check / ms_plain - 1.0),
            "plain_gemm_ms": ms_plain,
            "method": f"medians of {rounds} interleaved rounds of {per_round} launches per route"},
        "ms": {"plain_gemm": own_plain, "verified_gemm_given_threshold": own["check"], "fused_call": own["fused"],
               "whole_path_step": own["step"], "threshold_plus_gemm_calls": own["three_call"],
               "fused_call_timed_region": ms_steady},
        "flags_in_timed_region": nflag_timed,
    }

    # ---- HBM-bound passes on rotating buffers (> 512 MB in total, so the 256 MB Infinity Cache cannot serve them)
    eb = ELEM_BYTES[dt]
    if variant == 0:
        # (at most 64 buffers: a matrix of the smallest configuration is 256 KiB, its passes are bound by launch
        # latency whatever serves them)
        nrot = min(64, max(3, int(np.ceil(600e6 / (K * N * eb))) + 1))
        Bs = [B] + [B.clone() for _ in range(nrot - 1)]
        nrotA = min(64, max(3, int(np.ceil(600e6 / (M * K * eb))) + 1))
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

        hs = max(steps // 2, 3 * nrot)
        ms_enc_def = timed(torch, enc_def_rot, hs, nrot)
        ms_enc = timed(torch, enc_rot, hs, nrot)
        ms_thr = timed(torch, thr_rot, max(steps // 2, 3 * nrotA), nrotA)
        # what a kernel that only reads B reaches on this chip, and what an empty launch costs, in the same loop
        probe_out = torch.zeros(4, dtype=torch.float32, device="cuda")

        def read_rot():
            t = Bs[ctr[0] % nrot]
            vb.vabft_probe_read(t.data_ptr(), t.numel() * t.element_size(), probe_out.data_ptr())
            ctr[0] += 1

        ms_read = timed(torch, read_rot, hs, nrot)
        ms_empty = timed(torch, lambda: vb.vabft_probe_read(None, 0, probe_out.data_ptr()), 200, 20)
        del Bs, As
        vg.encode(B)
        vg.threshold(A, e_max)
        out["ms"].update({"encode_cold": ms_enc, "threshold_cold": ms_thr, "encode_cold_fold_deferred": ms_enc_def})
        bB, bA = K * N * eb, M * K * eb
        out["hbm_passes"] = {
            "encode": {"GBps": bB / (ms_enc * 1e-3) / 1e9, "frac": bB / (ms_enc * 1e-3) / 1e9 / HBM_PEAK_GBPS},
            "encode_fold_deferred": {"GBps": bB / (ms_enc_def * 1e-3) / 1e9,
                                     "frac": bB / (ms_enc_def * 1e-3) / 1e9 / HBM_PEAK_GBPS},
            "threshold": {"GBps": bA / (ms_thr * 1e-3) / 1e9, "frac": bA / (ms_thr * 1e-3) / 1e9 / HBM_PEAK_GBPS},
            "read_only_kernel_over_B": {"GBps": bB / (ms_read * 1e-3) / 1e9,
                                        "frac": bB / (ms_read * 1e-3) / 1e9 / HBM_PEAK_GBPS, "ms": ms_read},
            "empty_kernel_launch_ms": ms_empty,
        }

    if headline:
        # ---- the other routes, on the headline workload only: prepared once (each keeps its vectors in buffers of
        # its own), then each timed in its own sustained state against the plain GEMM, like the figures above
        vg.encode_weighted(B)
        vg.threshold_weighted(A, e_max)
        vg.encode_blocks(B)
        vg.threshold_blocks(A)
        vg.encode_a(A)
        vg.threshold_cols(B)
        vg.encode(B)
        vg.threshold(A, e_max)
        routes2 = {"plain": lambda: vg.gemm(A, B, 0), "w": lambda: vg.gemm_weighted(A, B),
                   "blocks": lambda: vg.gemm_blocks(A, B), "rc": lambda: vg.gemm_rc(A, B)}
        kb_ok = dt in ("bf16", "f16") and M % 256 == 0 and N % 256 == 0 and K % 128 == 0 and K > 1024
        if kb_ok:  # block-wise with K split as well, K-blocks of 1024 (the section's tile depth)
            from paper_2602_08043_amd.session import KBlockedGemm
            kg = KBlockedGemm(M, N, K, dt, tb, 1024)
            kg.run(A, B)
            routes2["blocks_k1024"] = lambda: kg.gemm(A, B)
        own2 = {}
        for k in ("plain", "w", "blocks", "rc") + (("blocks_k1024",) if kb_ok else ()) + ("plain_again",):
            fn = routes2["plain" if k == "plain_again" else k]
            spin_up(torch, fn, 0.25)
            own2[k] = timed(torch, fn, steps, warmup)
        ms_w, ms_blocks, ms_rc = own2["w"], own2["blocks"], own2["rc"]
        ms_plain2 = 0.5 * (own2["plain"] + own2["plain_again"])
        ms_locate = timed(torch, lambda: vg.locate_correct(1), steps, warmup)
        vg.encode(B)
        vg.threshold(A, e_max)
        out["other_routes_gemm_overhead_pct_vs_plain"] = {
            "with_position_weighted_row_sums": 100.0 * (ms_w / ms_plain2 - 1.0),
            "with_row_and_column_check": 100.0 * (ms_rc / ms_plain2 - 1.0),
            "block_wise_check": 100.0 * (ms_blocks / ms_plain2 - 1.0),
            "block_wise_check_k_blocks_of_1024": (100.0 * (own2["blocks_k1024"] / ms_plain2 - 1.0)) if kb_ok else None,
            "k_blocked_flagged_pieces_fault_free": int(kg.nblockflag.item()) if kb_ok else None,
            "ms_locate_correct": ms_locate}

    if not args.no_quality:
        n_ff = FAULT_FREE_TRIALS[name] if args.quality_trials is None else args.quality_trials
        n_flip = FLIP_TRIALS[name] if args.flip_trials is None else args.flip_trials
        out["quality"] = quality(torch, np, wl, vb, vg, name, variant, A, B, e_max, n_ff, n_flip, args.quality_seconds)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = oracle_time(np, wl, cfg, e_max, 10.0 if headline else 2.5)
    del vg, A, B
    torch.cuda.empty_cache()
    return out


def offline_bf16_table(torch, vb, VerifiedGemm):
    """Offline (post-quantisation) mode on the paper's BF16 tightness-table workloads: U(0,1), n x n x n,
    e_max = 2 u_output, plain GEMM followed by the post-hoc check of the stored C."""
    g2 = torch.Generator(device="cuda")
    g2.manual_seed(4321)
    table = {}
    for n in (128, 256, 512, 1024, 2048):
        vo = VerifiedGemm(n, n, n, "bf16", 0)
        e_off = vb.vabft_default_emax_offline("bf16", n, n)
        sT = torch.zeros((), dtype=torch.float64, device="cuda")
        sE = torch.zeros((), dtype=torch.float64, device="cuda")
        fp = torch.zeros((), dtype=torch.int64, device="cuda")
        trials = 50
        for _ in range(trials):
            Ao = torch.rand((n, n), generator=g2, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            Bo = torch.rand((n, n), generator=g2, device="cuda", dtype=torch.float32).to(torch.bfloat16)
            vo.run_offline(Ao, Bo, e_off)
            fp += (vo.nflag[0] > 0).to(torch.int64)
            sT += vo.T.double().mean()
            sE += vo.E.double().abs().mean()
        table[str(n)] = {"threshold_mean": float(sT.item()) / trials, "actual_diff_mean": float(sE.item()) / trials,
                         "tightness": float(sT.item()) / max(float(sE.item()), 1e-300),
                         "false_positive_trials": int(fp.item()), "trials": trials}
    return {"e_max": vb.vabft_default_emax_offline("bf16", 128, 128), "by_size": table}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="all", choices=["all"] + sorted(WORKLOAD_TEXT),
                    help="'all' (default): the headline workload plus every benchmark configuration in `configs`; "
                         "a name: that workload alone (its report becomes the top level)")
    ap.add_argument("--quality-trials", type=int, default=None, help="fault-free trials (default: the configurations' counts)")
    ap.add_argument("--flip-trials", type=int, default=None, help="single-bit-flip trials (default: the configurations' counts)")
    ap.add_argument("--quality-seconds", type=float, default=12.0, help="time cap of each quality loop of a configuration")
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
    mods = (torch, np, wl, vb, VerifiedGemm, to_device)

    if args.copy_calibration:
        # 5 copies of 1 GiB (read 1 GiB + write 1 GiB each): the counters of these dispatches
        # (the runtime's device-to-device copy kernel) give the KiB-per-count factor
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    head_name = HEADLINE if args.config == "all" else args.config
    head = bench_config(mods, head_name, 0, args.steps, args.warmup, args, headline=True)
    out = {
        "metric": "verified_gemm_tflops",
        "value": head["value"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": head["steps"],
        "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": head["workload"], "M": head["M"], "N": head["N"], "K": head["K"],
                   "transB": head["transB"], "e_max": head["e_max"], "c_sigma": 2.5,
                   "step": "vabft_encode(B, d_S=NULL) + vabft_gemm_verified_fused(A, B, d_S=NULL) [B-side checksum and "
                           "statistics; A-side statistics, fold of S1..S3, threshold, GEMM, row sums, compare/flag]"},
    }
    for k in ("roofline", "frac_of_peak_whole_path", "plain_gemm_tflops", "plain_gemm_frac_of_peak", "overhead_pct",
              "overhead_pct_interleaved_rounds", "ms",
              "hbm_passes", "other_routes_gemm_overhead_pct_vs_plain", "flags_in_timed_region", "quality",
              "cpu_baseline"):
        if k in head:
            out[k] = head[k]
    if not args.no_quality and head["dtype"] == "bf16":
        out["quality"]["offline_bf16_uniform01"] = offline_bf16_table(torch, vb, VerifiedGemm)
    if args.config == "all":
        reports = []
        for name, variant in (("c1_f32_256", 0), (HEADLINE, 0), ("c3_bf16_ffn", 0), ("c4_f16_8192", 0),
                              ("c5_f64_2048", 0), ("c5_f64_2048", 1)):
            if name == HEADLINE:
                reports.append({k: v for k, v in head.items() if k != "other_routes_gemm_overhead_pct_vs_plain"})
                continue
            print(f"bench.py: {name} variant {variant}", file=sys.stderr, flush=True)
            reports.append(bench_config(mods, name, variant, args.steps, args.warmup, args, headline=False))
        out["configs"] = reports
    print(json.dumps(out))


if __name__ == "__main__":
    main()
