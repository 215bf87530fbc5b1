#!/usr/bin/env python3
"""Throughput of fault-injection campaigns on one MI355X.

One step = one pass of the whole hot path over one batch of trials: every trial runs the
complete GEMM with its fault, the fused detector / corrector / counters, then the batch is
classified (fi_gemm_inject_batch + fi_classify).  Inputs, the fault list and the plan
(fault-free result, magnitude maxima) are resident in HBM before the timed region; plan
construction is timed separately and reported in `config`.

Prints ONE JSON line.  `value` counts only flops the matrix cores executed: 2*M*N*K per
trial, every trial recomputing the whole product.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2516.6     # 256 CUs x 4096 flop/clk/CU x 2.4 GHz, dense FP16/BF16

# HBM bytes of one campaign launch of the default workload and kernel choice, from two
# `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch) scaled by what the same
# counters read for a plain 1 GiB copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0); profiles/ holds the
# commands.  They describe the kernel sources whose digest is recorded with them and are not
# reported for any other.
TRAFFIC = {
    "sources_sha256": "73bf5516d50982b097438602074423d6b613f3abc0ac6b78b8916481b0b3c584",
    "fetch_bytes": 2.16782e6 * 2.0 * 1024,
    "write_bytes": 151.375 * 1.0 * 1024,
}


def kernel_sources_digest():
    from paper_2311_05782_amd import build
    return build.sources_digest()


def mfma_loop_peak(torch, fi, fmt, n_cus, random_data, iters=150000, reps=3):
    """What the matrix cores sustain on this machine when waves only issue MFMAs (fi_probe_mfma_loop):
    the campaign kernel's occupancy, register-resident operands.  Returns TFLOP/s (median of
    `reps` launches of about 80 ms) and the shader clock the last launch sustained."""
    sink = torch.empty(n_cus * 512, dtype=torch.float32, device="cuda")
    clk = torch.zeros(4, dtype=torch.int64, device="cuda")
    fi.fi_probe_mfma_loop(fmt, random_data, iters // 10, n_cus, sink, clk)
    torch.cuda.synchronize()
    ms = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fi.fi_probe_mfma_loop(fmt, random_data, iters, n_cus, sink, clk)
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    flops = float(n_cus) * 8 * 2 * 8 * iters * 32768.0
    return flops / (sorted(ms)[len(ms) // 2] * 1e-3) / 1e12, clock_ghz(clk.cpu().numpy())


def clock_ghz(c):
    """{cycles, 100 MHz ticks, cycles, ticks} of one launch -> sustained shader clock in GHz."""
    ticks = int(c[3]) - int(c[1])
    return round((int(c[2]) - int(c[0])) / (ticks / 1e8) / 1e9, 3) if ticks > 0 else None


def cpu_baseline(w, budget_s=15.0):
    """The CPU oracle as it stands, timed on a row slab of one fault-free pass of the same GEMM
    (a trial of the oracle in `full` mode is exactly such a pass), scaled to the whole matrix."""
    import numpy as np
    from oracle import pyoracle as orc
    cores = orc.threads()

    def slab_time(rows):
        p = orc.problem(rows, w.N, w.K, w.kb, w.fmt)
        t0 = time.perf_counter()
        orc.gemm(p, np.ascontiguousarray(w.A[:rows]), w.B)
        return time.perf_counter() - t0

    probe_rows = min(w.M, 4 * cores)
    t_probe = slab_time(probe_rows)
    rows = int(min(w.M, max(probe_rows, probe_rows * budget_s / max(t_probe, 1e-6))))
    rows = max(cores, rows // cores * cores)
    t = slab_time(rows) if rows > probe_rows else t_probe
    reps = 1
    if rows == w.M and t < 0.7 * budget_s:          # a whole pass is quick: time several
        reps = int(budget_s / t)
        t0 = time.perf_counter()
        for _ in range(reps):
            slab_time(rows)
        t = (time.perf_counter() - t0) / reps
    flops = 2.0 * rows * w.N * w.K
    t_trial = t * w.M / rows
    return {"value": flops / t / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "trials_per_s": 1.0 / t_trial,
            "sample": "rows 0..%d of a fault-free %dx%dx%d pass, %d time(s), %.1f s each, scaled by M/%d to a whole trial"
                      % (rows - 1, w.M, w.N, w.K, reps, t, rows)}


def two_layer(torch, n_trials=256, policy=1):
    import numpy as np
    from paper_2311_05782_amd import fi, workloads as wl
    M, D, H, fmt = 512, 768, 3072, wl.BF16
    Xw, W1w, W2w = wl.two_layer_mlp(M, D, H, fmt)
    plan1 = fi.Plan(fi.plan_desc(M, H, D, 32, fmt), fi.words_to_device(Xw), fi.words_to_device(W1w))
    d_h = torch.empty((n_trials, M, H), dtype=torch.int16, device="cuda")
    d_hstar = torch.empty((M, H), dtype=torch.int16, device="cuda")
    fi.fi_activation_round(fmt, plan1.buffer_ptr(fi.BUF_C_STAR), M * H, d_hstar)
    torch.cuda.synchronize()
    plan2 = fi.Plan(fi.plan_desc(M, D, H, 32, fmt), d_hstar, fi.words_to_device(W2w))
    d_c1 = torch.empty((n_trials, M, H), dtype=torch.float32, device="cuda")
    r1, r2 = fi.empty_results(n_trials), fi.empty_results(n_trials)
    res = {"shape": "%dx%d -> %d -> %d bf16, k-block 32" % (M, D, H, D), "trials": n_trials,
           "policy": {0: "none", 1: "zero", 2: "recompute"}[policy]}
    for label, mode, nbits in (("acc_1bit", fi.KIND_ALL_ACC, 1), ("product_4bit", fi.KIND_ALL_PRODUCT, 4)):
        ff = fi.to_device(fi.fi_sample_faults(11, 0, n_trials, plan1.desc, mode, nbits))

        def chain():
            plan1.fi_gemm_inject_batch(ff, n_trials, policy, r1, d_c1)
            fi.fi_activation_round(fmt, d_c1, n_trials * M * H, d_h)
            plan2.fi_gemm_propagate_batch(d_h, M * H, n_trials, wl.CORRECT_NONE, r2)
        # about 30 ms of warm-up chains (the device idles during the host-side set-up above), then
        # the median per-call time over 9 chains
        for _ in range(12):
            chain()
        torch.cuda.synchronize()
        runs = []
        for _ in range(9):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record(); plan1.fi_gemm_inject_batch(ff, n_trials, policy, r1, d_c1)
            ev[1].record(); fi.fi_activation_round(fmt, d_c1, n_trials * M * H, d_h)
            ev[2].record(); plan2.fi_gemm_propagate_batch(d_h, M * H, n_trials, wl.CORRECT_NONE, r2)
            ev[3].record(); torch.cuda.synchronize()
            runs.append([ev[i].elapsed_time(ev[i + 1]) for i in range(3)])
        ms = [sorted(r[i] for r in runs)[len(runs) // 2] for i in range(3)]
        h_unfused = d_h.clone()
        # the same chain with the hand-over fused into the campaign's epilogue (two calls)
        runs = []
        for k in range(12):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            ev[0].record(); plan1.fi_gemm_inject_batch_act(ff, n_trials, policy, r1, d_h)
            ev[1].record(); plan2.fi_gemm_propagate_batch(d_h, M * H, n_trials, wl.CORRECT_NONE, r2)
            ev[2].record(); torch.cuda.synchronize()
            if k >= 3:
                runs.append([ev[i].elapsed_time(ev[i + 1]) for i in range(2)])
        msf = [sorted(r[i] for r in runs)[len(runs) // 2] for i in range(2)]
        assert torch.equal(h_unfused, d_h), "the fused hand-over differs from the two-call form"
        del h_unfused
        a, b = fi.results_to_host(r1), fi.results_to_host(r2)
        c1 = np.where(a["n_flagged"] > 0, 2, np.where(a["n_dev_pre"] > 0, 1, 0))
        out_masked = b["n_dev_pre"] == 0
        res[label] = {
            "layer1_masked_sdc_detected": [int((c1 == k).sum()) for k in range(3)],
            "output_masked": int(out_masked.sum()),
            "layer1_sdc_masked_at_output": int(((c1 == 1) & out_masked).sum()),
            "layer1_detected_masked_at_output_after_correction": int(((c1 == 2) & out_masked).sum()),
            "ms_layer1_activation_layer2": [round(x, 3) for x in ms],
            "ms_fused_layer1_layer2": [round(x, 3) for x in msf],
            "chain_trials_per_s": round(n_trials / (sum(msf) * 1e-3), 1),
            "chain_trials_per_s_three_calls": round(n_trials / (sum(ms) * 1e-3), 1),
            "layer2_tflops": round(2.0 * M * D * H * n_trials / (ms[2] * 1e-3) / 1e12, 1),
            "activation_GBps": round(n_trials * M * H * 6 / (ms[1] * 1e-3) / 1e9, 1),
        }
    plan1.destroy(); plan2.destroy()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="square4096")
    ap.add_argument("--trials", type=int, default=0, help="trials per batch (default: the workload's)")
    ap.add_argument("--tile", type=int, default=-1)
    ap.add_argument("--group", type=int, default=-1)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="headline measurement only: no CPU baseline, detector or other-campaign timings")
    ap.add_argument("--sources-digest", action="store_true", help="print the kernel sources' digest and exit")
    ap.add_argument("--campaigns", action="store_true", help="also time the four other campaigns")
    ap.add_argument("--detector", action="store_true", help="also time the standalone detector kernel")
    ap.add_argument("--two-layer", action="store_true", help="also time the two-layer chain")
    ap.add_argument("--no-loop-peak", action="store_true", help="skip the MFMA-loop probe (achievable peak)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference row for HBM byte counters)")
    args = ap.parse_args()
    if args.sources_digest:
        print(kernel_sources_digest())
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: campaigns shard by trial with no exchange, and this library "
              "runs on a single MI355X.  Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2311_05782_amd import fi, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs an MI355X; no device is visible.", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    w = wl.ALL[args.workload]()
    n_trials = args.trials or w.n_trials
    policy = w.policies[0]

    d_A, d_B = fi.words_to_device(w.A), fi.words_to_device(w.B)
    desc = fi.plan_desc(w.M, w.N, w.K, w.kb, w.fmt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    plan = fi.Plan(desc, d_A, d_B)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    if args.tile >= 0 or args.group > 0:
        plan.tune(args.tile, args.group if args.group > 0 else -1)
    faults = fi.fi_sample_faults(w.fault_seed, 0, n_trials, desc, w.kind_mode, w.nbits)
    d_f = fi.to_device(faults)
    d_r = fi.empty_results(n_trials)
    d_cls = torch.empty(n_trials, dtype=torch.uint8, device="cuda")
    d_cnt = torch.empty(3, dtype=torch.int64, device="cuda")
    d_clk = torch.zeros(12, dtype=torch.int64, device="cuda")
    plan.set_clock_sink(d_clk)

    def step():
        plan.fi_gemm_inject_batch(d_f, n_trials, policy, d_r)
        plan.fi_classify(d_r, n_trials, d_cls, d_cnt)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)           # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # HIP events on the launching stream bracket the campaign launch of every step: the GEMM
    # kernel(s) plus the record fill and the trial partition, a few microseconds each.
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record()
        plan.fi_gemm_inject_batch(d_f, n_trials, policy, d_r)
        ev[k][1].record()
        plan.fi_classify(d_r, n_trials, d_cls, d_cnt)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    kern_ms = [a.elapsed_time(b) for a, b in ev]
    clocks = d_clk.cpu().numpy()
    plan.set_clock_sink(None)
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    loop_peak = loop_clock = loop_peak_const = loop_clock_const = None
    if not args.no_loop_peak:
        loop_peak, loop_clock = mfma_loop_peak(torch, fi, w.fmt, n_cus, 1)
        loop_peak_const, loop_clock_const = mfma_loop_peak(torch, fi, w.fmt, n_cus, 0)
    flops_per_launch = w.flops_per_trial * n_trials
    ms_per_step = wall * 1e3 / args.steps
    tflops = flops_per_launch * args.steps / wall / 1e12
    achieved = flops_per_launch / (sum(kern_ms) / len(kern_ms) * 1e-3) / 1e12
    counts = d_cnt.cpu().numpy().tolist()
    default_run = (args.workload == "square4096" and not args.trials and args.tile < 0 and args.group <= 0)
    traffic = None
    if default_run and TRAFFIC["sources_sha256"] == kernel_sources_digest():
        traffic = round(TRAFFIC["fetch_bytes"] + TRAFFIC["write_bytes"])

    out = {
        "metric": "fault-injected GEMM TFLOP/s and trials/sec on 1 MI355X; % of MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s",
        "trials_per_s": round(n_trials * args.steps / wall, 1),
        "frac_of_mfma_peak": round(tflops / MFMA_PEAK_TFLOPS, 4),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.fmt == wl.BF16 else "fp16", "data": "synthetic",
        "config": {"workload": "%s: M=%d N=%d K=%d %s operands, FP32 accumulate, k-block %d, %d trials/batch, "
                               "%d-bit faults (kind mode %d), fused detect + %s"
                               % (w.name, w.M, w.N, w.K, "BF16" if w.fmt == wl.BF16 else "FP16", w.kb, n_trials,
                                  w.nbits, w.kind_mode, {0: "no correction", 1: "zero-correct", 2: "recompute-correct"}[policy]),
                   "trials_per_batch": n_trials, "plan_create_ms": round(plan_ms, 2),
                   "outcomes_masked_sdc_detected": counts},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                     "traffic_unit": "HBM bytes per launch (fetch + write)", "kernel": plan.describe(),
                     "flops_per_launch": flops_per_launch, "kernel_ms_avg": round(sum(kern_ms) / len(kern_ms), 3),
                     "kernel_ms_median": round(sorted(kern_ms)[len(kern_ms) // 2], 3),
                     "kernel_ms_min": round(min(kern_ms), 3),
                     # the shader clock the last timed campaign launch sustained (the kernel's own counters)
                     "sustained_clock_ghz": clock_ghz(clocks[0:4]), "nominal_clock_ghz": 2.4,
                     # what an MFMA-only loop reaches on this machine, in the same occupancy: on random
                     # operands of the campaign's format (the achievable peak: the part lowers its clock
                     # under matrix load) and on constant operands
                     "mfma_loop_peak": None if loop_peak is None else round(loop_peak, 1),
                     "mfma_loop_clock_ghz": loop_clock,
                     "mfma_loop_peak_constant_data": None if loop_peak_const is None else round(loop_peak_const, 1),
                     "mfma_loop_clock_constant_data_ghz": loop_clock_const,
                     "frac_of_mfma_loop_peak": None if not loop_peak else round(achieved / loop_peak, 4)},
    }
    # The standalone detector / corrector (fi_detect_correct) on materialised outputs of the same
    # problem: an HBM-bound kernel, 4 bytes read per element, priced against the 8 TB/s roof.
    extras = default_run and not args.no_cpu_baseline      # the full default run; profiles use the bare one
    if extras or args.detector:
        batch = 16
        c = torch.empty((batch, w.M, w.N), dtype=torch.float32, device="cuda").uniform_(-1.0, 1.0)
        nfl = torch.zeros(batch, dtype=torch.int32, device="cuda")
        for _ in range(2):
            plan.fi_detect_correct(c, batch, policy, None, nfl)
        dev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for a, b in dev:
            a.record()
            plan.fi_detect_correct(c, batch, policy, None, nfl)
            b.record()
        torch.cuda.synchronize()
        dms = [a.elapsed_time(b) for a, b in dev]
        dbytes = float(batch) * w.M * w.N * 4
        dgbs = dbytes / (sum(dms) / len(dms) * 1e-3) / 1e9
        out["detector_roofline"] = {"kernel": "detect_correct_kernel<4> (+ a 1-block counter fill)", "bound": "hbm",
                                    "achieved": round(dgbs, 1), "peak": 8000.0, "unit": "GB/s",
                                    "frac": round(dgbs / 8000.0, 4), "bytes_per_launch": dbytes,
                                    "kernel_ms_avg": round(sum(dms) / len(dms), 4), "batch": batch,
                                    "flagged": int(nfl.sum().item())}
        del c
    # The affected-tiles-only campaign on the same batch: a different product (only what a fault can
    # reach is computed), reported as trials per second and never against the MFMA roof.
    if extras or args.campaigns:
        for _ in range(2):
            plan.fi_gemm_inject_batch_affected(d_f, n_trials, policy, d_r)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(10):
            plan.fi_gemm_inject_batch_affected(d_f, n_trials, policy, d_r)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t1) / 10
        out["affected_only"] = {"entry_point": "fi_gemm_inject_batch_affected", "trials_per_s": round(n_trials / dt, 1),
                                "ms_per_batch": round(dt * 1e3, 4)}
    # The other campaigns (parity-test configurations), a few launches each: context, not the metric.
    if extras or args.campaigns:
        others = {}
        for name in ("tiny128", "bert_linear", "resnet_conv", "detector_stress"):
            ww = wl.ALL[name]()
            pl = fi.Plan(fi.plan_desc(ww.M, ww.N, ww.K, ww.kb, ww.fmt), fi.words_to_device(ww.A), fi.words_to_device(ww.B))
            ff = fi.to_device(fi.fi_sample_faults(ww.fault_seed, 0, ww.n_trials, pl.desc, ww.kind_mode, ww.nbits))
            rr = fi.empty_results(ww.n_trials)
            # Host-side set-up (plan, fault list) leaves the device idle; launches of a millisecond
            # or two then run below the steady-state clock.  Warm up for about 30 ms of launches and
            # time at least 60 ms (at least 5 launches).
            t1 = time.perf_counter()
            for _ in range(2):
                pl.fi_gemm_inject_batch(ff, ww.n_trials, ww.policies[0], rr)
            torch.cuda.synchronize()
            one = max((time.perf_counter() - t1) / 2, 1e-5)
            for _ in range(min(200, int(0.03 / one))):
                pl.fi_gemm_inject_batch(ff, ww.n_trials, ww.policies[0], rr)
            reps = max(5, min(400, int(0.06 / one) + 1))
            cls_buf = d_cls[:1].new_empty(ww.n_trials)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(reps):
                pl.fi_gemm_inject_batch(ff, ww.n_trials, ww.policies[0], rr)
                pl.fi_classify(rr, ww.n_trials, cls_buf, d_cnt)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t1) / reps
            others[name] = {"shape": "%dx%dx%d %s kb %d" % (ww.M, ww.N, ww.K, "bf16" if ww.fmt == wl.BF16 else "fp16", ww.kb),
                            "trials": ww.n_trials, "launches_timed": reps, "ms_per_batch": round(dt * 1e3, 3),
                            "trials_per_s": round(ww.n_trials / dt, 1),
                            "tflops": round(ww.flops_per_trial * ww.n_trials / dt / 1e12, 2)}
            for _ in range(2):
                pl.fi_gemm_inject_batch_affected(ff, ww.n_trials, ww.policies[0], rr)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(5):
                pl.fi_gemm_inject_batch_affected(ff, ww.n_trials, ww.policies[0], rr)
            torch.cuda.synchronize()
            others[name]["affected_only_trials_per_s"] = round(5 * ww.n_trials / (time.perf_counter() - t1), 1)
            if name == "bert_linear":
                # The same batch size with every trial of ONE fault kind (Sec. IV-A's sites): what the
                # operand-fault path costs against accumulator flips.
                by_kind = {}
                for label, km in (("acc", fi.KIND_ALL_ACC), ("a_operand", fi.KIND_ALL_A), ("b_operand", fi.KIND_ALL_B),
                                  ("product", fi.KIND_ALL_PRODUCT)):
                    fk = fi.to_device(fi.fi_sample_faults(ww.fault_seed, 0, ww.n_trials, pl.desc, km, 1))
                    for _ in range(3):
                        pl.fi_gemm_inject_batch(fk, ww.n_trials, ww.policies[0], rr)
                    torch.cuda.synchronize()
                    t1 = time.perf_counter()
                    for _ in range(8):
                        pl.fi_gemm_inject_batch(fk, ww.n_trials, ww.policies[0], rr)
                    torch.cuda.synchronize()
                    by_kind[label] = round(ww.flops_per_trial * ww.n_trials * 8 / (time.perf_counter() - t1) / 1e12, 1)
                others[name]["tflops_by_fault_kind"] = by_kind
            pl.destroy()
            if name == "detector_stress":
                # Coverage of the three output-side detectors on the same fault list (Sec. VI-A's
                # exponent-only bound check against the operand-derived magnitude bounds).
                cov = {}
                for label, mode in (("rowcol", fi.BOUND_ROWCOL), ("global", fi.BOUND_GLOBAL), ("exponent", fi.BOUND_EXPONENT)):
                    pb = fi.Plan(fi.plan_desc(ww.M, ww.N, ww.K, ww.kb, ww.fmt, bound_mode=mode),
                                 fi.words_to_device(ww.A), fi.words_to_device(ww.B))
                    pb.fi_gemm_inject_batch_affected(ff, ww.n_trials, ww.policies[0], rr)
                    pb.fi_classify(rr, ww.n_trials, d_cls[:1].new_empty(ww.n_trials), d_cnt)
                    torch.cuda.synchronize()
                    cov[label] = [int(x) for x in d_cnt.cpu().tolist()]
                    pb.destroy()
                others[name]["masked_sdc_detected_by_detector"] = cov
        out["other_campaigns"] = others
    # Two layers, Y = relu(X W1) W2 with a transformer feed-forward block's shapes: a fault in the
    # first GEMM, detector + corrector, ReLU and rounding to the operand format, then the second GEMM
    # of every trial in full; how many of the faults layer 1 does not mask still show at the output.
    if extras or args.campaigns or args.two_layer:
        out["two_layer"] = two_layer(torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
        out["cpu_baseline"]["value"] = float("%.4g" % out["cpu_baseline"]["value"])
        out["cpu_baseline"]["trials_per_s"] = float("%.4g" % out["cpu_baseline"]["trials_per_s"])
    plan.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
