#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A "step" is one pass of the whole path (plan upload, operand images, the single sweep over
the vocabulary that yields the row statistics and the gradient factors, merge, combine,
gradient contraction, scatter and window reductions) over one batch of seeded synthetic
rollouts already resident in HBM.  Prints ONE JSON line:

* `value`: distilled tokens/s of the fused configuration the metric names, from the wall clock
  around exactly `--steps` calls (synchronised on both sides); next to it the median of the
  per-call durations taken with HIP events on the launch stream.
* `roofline`: the dominant kernel (the vocabulary sweep) against the bf16 MFMA peak, its launch
  duration from HIP events on the launch stream (the library's profiling entry point).
* `parity`: the timed call's own outputs compared with the fp64 oracle on the sampled rows the
  CPU baseline computes anyway.
* `logits_given`: the bandwidth-bound configuration timed in the same run (HIP-event median of
  >= 10 calls), with its own roofline object against the HBM peak and its own parity block.
* `cpu_baseline`: the oracle timed on the host cores on a bounded sample.
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
KL_REL, KL_ABS, DH_REL = 1e-3, 1e-6, 2e-3      # the parity bars of the test-suite


def _cpu_threads() -> int:
    try:
        from threadpoolctl import threadpool_info
        n = [i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"]
        if n:
            return int(max(n))
    except Exception:
        pass
    return len(os.sched_getaffinity(0))


def _event_times(run, n):
    """Milliseconds of n calls of run(), each bracketed by HIP events on the current stream."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in ev:
        a.record()
        st = run()
        b.record()
        assert st == 0
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in ev]


def _oracle_fused_baseline(w, prob, k_rows):
    """fp64 oracle on a seeded sample of computed rows of the same workload."""
    import torch
    from oracle import adwin_oracle as O
    from paper_2605_28396_amd import synth
    rows = synth.sample_rows(w, k_rows)
    idx = torch.from_numpy(rows).to(prob["h_s"].device)
    Hs = synth.to_f64(prob["h_s"][idx])
    Ht = synth.to_f64(prob["h_t"][idx])
    Ws = synth.to_f64(prob["W_s"])
    Wt = synth.to_f64(prob["W_t"])
    ids = prob["ids"][idx].cpu().numpy()
    t0 = time.perf_counter()
    kl, c, g = O.rows_terms(Hs, Ht, Ws, Wt, ids)
    dt = time.perf_counter() - t0
    return {"value": len(rows) / dt, "unit": "tokens/s", "cores": _cpu_threads(), "kind": "oracle",
            "sample": f"{len(rows)} seeded computed rows of this workload (full vocabulary, fp64, "
                      f"numpy/BLAS inner products), {dt:.1f} s"}, (rows, kl, c, g)


def _oracle_logits_baseline(w, prob, k_rows):
    import numpy as np
    import torch
    from oracle import adwin_oracle as O
    from paper_2605_28396_amd import synth
    rows = synth.sample_rows(w, k_rows)
    ids = prob["ids"].cpu().numpy()
    dt = 0.0
    kl = np.zeros(len(rows))
    dz = []
    for lo in range(0, len(rows), 256):                   # fp64 copies of 256 rows at a time
        part = rows[lo:lo + 256]
        idx = torch.from_numpy(part).to(prob["z_s"].device)
        zs = synth.to_f64(prob["z_s"][idx])
        zt = synth.to_f64(prob["z_t"][idx])
        t0 = time.perf_counter()
        for r in range(len(part)):
            kl[lo + r] = O.token_kl(zs[r], zt[r])
            O.token_cost(zs[r], zt[r], int(ids[part[r]]))
            d = O.token_dz(zs[r], zt[r])
            if lo + r < 64:
                dz.append(d)
        dt += time.perf_counter() - t0
    return {"value": len(rows) / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(rows)} seeded admitted rows of this workload (fp64, numpy), {dt:.1f} s"}, (rows, kl, dz)


def _measured_traffic(summary: str, kernel: str):
    """HBM bytes per launch of `kernel` from a committed rocprofv3 counter summary under
    profiles/ (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each scaled by what the same
    counter reads for the 1 GiB copy kernel in the same run), or None.  Not a measurement of
    this run: counters need rocprofv3 around the process."""
    path = os.path.join(ROOT, "profiles", summary)
    try:
        vals = {}
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[1] in ("FETCH_SIZE", "WRITE_SIZE"):
                vals[(f[0], f[1])] = float(f[3])
        gib = 1048576.0
        rd = vals[(kernel, "FETCH_SIZE")] * gib / vals[("adwin::copy_kernel", "FETCH_SIZE")]
        wr = vals[(kernel, "WRITE_SIZE")] * gib / vals[("adwin::copy_kernel", "WRITE_SIZE")]
        return (rd + wr) * 1024.0
    except Exception:
        return None


def _row_alpha_p(w, rows):
    """alpha^p of the sequence-mean reduction for the given packed rows (0 outside the windows)."""
    import numpy as np
    lens = np.diff(w.offsets)
    n = np.minimum(w.window.astype(np.int64), lens)
    i = np.searchsorted(w.offsets, rows, side="right") - 1
    j = rows - w.offsets[i]
    return np.where(j < n[i], 1.0 / (w.B * np.maximum(n[i], 1)), 0.0)


def _bench_logits(B, synth, dev, steps, cpu_rows, estimator):
    """The bandwidth-bound configuration: HIP-event median of `steps` calls, roofline, parity."""
    import numpy as np
    import torch
    w = synth.workload("logits_given")
    lens = np.diff(w.offsets)
    n_adm = int(np.minimum(w.window.astype(np.int64), lens).sum())
    prob = synth.logits_problem(w, dev)
    call = B.LogitsCall(prob["z_s"], prob["z_t"], prob["ids"], w.offsets, w.window,
                        reduction=B.ADWIN_RED_SEQ_MEAN, estimator=estimator)
    for _ in range(3):
        assert call.run() == 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    times = _event_times(call.run, steps)
    wall_ms = (time.perf_counter() - t0) / steps * 1e3
    assert int(call.out["status_dev"][0]) == 0
    ms = float(np.median(times))
    phases = [B.adwin_opd_from_logits_profile(call) for _ in range(5)]
    kernel_ms = float(np.median([p["stats"] for p in phases]))
    V = w.V
    alg_bytes = 6.0 * V * n_adm + 2.0 * V * (w.T - n_adm)      # read z_s, z_t + write dz; zero rows
    ach = alg_bytes / (kernel_ms * 1e-3) / 1e9
    out = {
        "workload": "logits_given", "rollouts": w.B, "packed_rows": w.T, "computed_rows": n_adm, "V": V,
        "value": n_adm / (ms * 1e-3), "unit": "tokens/s", "ms_per_call_median": ms, "ms_per_call_wall": wall_ms,
        "calls_timed": steps, "timing": "HIP events on the launch stream around each call; median",
        "roofline": {"bound": "hbm", "kernel": "logits_row_resident_kernel + zero-fill of the rows outside the windows",
                     "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": ach / PEAK_HBM_GBS,
                     "traffic": _measured_traffic("logits_given_hbm_counters.txt", "adwin::logits_row_resident_kernel"),
                     "traffic_source": "profiles/logits_given_hbm_counters.txt (rocprofv3 --pmc, separate run)",
                     "launch_ms": kernel_ms, "alg_bytes_per_launch": alg_bytes,
                     "whole_call_frac": alg_bytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }
    if cpu_rows > 0:
        cpu, (rows, kl, dz) = _oracle_logits_baseline(w, prob, cpu_rows)
        idx = torch.from_numpy(rows).to(dev)
        got_kl = call.out["kl"][idx].double().cpu().numpy()
        kl_err = np.abs(got_kl - kl) / (KL_REL * np.abs(kl) + KL_ABS)
        a = _row_alpha_p(w, rows[:len(dz)])
        ref_dz = np.stack(dz) * a[:, None]
        got_dz = call.out["dz"][idx[:len(dz)]].double().cpu().numpy()
        scale = np.abs(ref_dz).max()
        dz_err = np.abs(got_dz - ref_dz) - 2.0 ** -8 * np.abs(ref_dz)       # one bf16 storage ulp
        out["cpu_baseline"] = cpu
        out["parity"] = {"rows": int(len(rows)), "kl_rel_max": float((np.abs(got_kl - kl) / np.abs(kl)).max()),
                         "dz_rows": len(dz), "dz_err_over_max": float(dz_err.max() / scale),
                         "ok": bool(kl_err.max() <= 1.0 and dz_err.max() <= DH_REL * scale)}
    del call, prob
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="strong_to_weak",
                    choices=["tiny", "logits_given", "strong_to_weak", "same_family", "probe_alignment"])
    ap.add_argument("--cpu-rows", type=int, default=-1,
                    help="rows of the oracle sample (0 = skip; default: about 15 s of host work)")
    ap.add_argument("--dh-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--estimator", default="expected", choices=["expected", "sampled"],
                    help="expected: gradient of the full-vocabulary KL (default, the metric's path); "
                         "sampled: Eq. 4 on the sampled token (one gradient contraction)")
    ap.add_argument("--head-grad", action="store_true",
                    help="also emit the gradient with respect to the student LM-head weights "
                         "(dW_s, one more contraction per objective; not part of the headline metric)")
    ap.add_argument("--no-logits-given", action="store_true",
                    help="skip the bandwidth-bound configuration (profiling runs of the fused path)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2605_28396_amd import binding as B, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    est = B.ADWIN_EST_SAMPLED if args.estimator == "sampled" else B.ADWIN_EST_EXPECTED
    cpu_rows_logits = 1024 if args.cpu_rows < 0 else args.cpu_rows

    if args.workload == "logits_given":
        # the bandwidth-bound configuration as the headline of this run
        lg = _bench_logits(B, synth, dev, max(args.steps, 10), cpu_rows_logits, est)
        line = {
            "metric": "distilled tokens/sec (fused fwd+bwd reverse-KL, V=151936) + % roofline",
            "value": lg["value"], "unit": "tokens/s", "n_gpus": 1, "steps": lg["calls_timed"], "warmup": 3,
            "ms_per_step": lg["ms_per_call_wall"], "ms_per_step_median": lg["ms_per_call_median"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "logits_given", "rollouts": lg["rollouts"], "packed_rows": lg["packed_rows"],
                       "computed_rows": lg["computed_rows"], "V": lg["V"], "estimator": args.estimator},
            "roofline": lg["roofline"], "cpu_baseline": lg.get("cpu_baseline"), "parity": lg.get("parity"),
            "ceilings": {"copy_GBps": B.adwin_opd_ceiling_copy(),
                         "note": "measured on this box: the library's streaming copy of 1 GiB (read+write bytes); "
                                 "it also calibrates the HBM counters of a profiling run"},
        }
        print(json.dumps(line))
        return 0

    w = synth.workload(args.workload)
    lens = np.diff(w.offsets)
    n = np.minimum(w.window.astype(np.int64), lens)
    n_adm = int(n.sum())
    prob = synth.hidden_problem(w, dev)
    call = B.FusedCall(prob["h_s"], prob["h_t"], prob["W_s"], prob["W_t"], prob["ids"],
                       w.offsets, w.window, mode=w.mode, reduction=B.ADWIN_RED_SEQ_MEAN,
                       dh_dtype=B.ADWIN_DT_BF16 if args.dh_dtype == "bf16" else B.ADWIN_DT_F32,
                       estimator=est,
                       want=B.FusedCall.DEFAULT_OUTPUTS + (("dW_prefix", "dW_full") if args.head_grad else ()))
    tokens = w.T if w.mode == synth.MODE_PREFIX_AND_FULL else n_adm
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        st = call.run()
        assert st == 0, B.adwin_opd_strerror(st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    times = _event_times(call.run, args.steps)              # records events, synchronises at the end
    dt = time.perf_counter() - t0
    assert int(call.out["status_dev"][0]) == 0 or os.environ.get("ADWIN_BENCH_NOCHECK")
    ms_per_step = dt / args.steps * 1e3
    value = tokens / (dt / args.steps)
    ms_median = float(np.median(times))

    # per-kernel durations from HIP events on the launch stream (same launches, profiled)
    phases = [B.adwin_opd_fused_profile(call) for _ in range(5)]
    ph = {k: float(np.median([p[k] for p in phases])) for k in phases[0]}

    V, Hs, Ht = w.V, w.H_s, w.H_t
    # the sweep kernel is launched once per slab of computed rows; figures are per launch
    launches = max(1, B.adwin_opd_fused_launch_info(call.p)["slabs"])
    f_stats = 2.0 * V * (Hs + Ht) * tokens / launches   # one full-vocabulary sweep of both heads
    launch_ms = ph["stats"] / launches
    ach = f_stats / (launch_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "logit_pass_dma_kernel", "achieved": ach,
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                "traffic": _measured_traffic(f"fused_{w.name}_hbm_counters.txt",
                                             "adwin::logit_pass_dma_kernel<2>"),
                "traffic_source": f"profiles/fused_{w.name}_hbm_counters.txt (rocprofv3 --pmc, separate run)",
                "launch_ms": launch_ms, "launches_per_call": launches,
                "alg_flops_per_launch": f_stats}
    f_alg = 2.0 * V * (2 * Hs + Ht) * tokens            # student fwd + teacher fwd + dz W_s
    if args.head_grad:                                  # + dz^T h_s per objective
        f_alg += 2.0 * V * Hs * tokens * (2 if w.mode == synth.MODE_PREFIX_AND_FULL else 1)
    # executed = algorithmic on the single-sweep scheme: logits once, one gradient contraction
    f_exec = f_alg
    f_grad = 2.0 * V * Hs * tokens
    t_s = ms_median * 1e-3
    extra = {"roofline_call": {
        "scheme": "single_sweep",
        "alg_tflops": f_alg / t_s / 1e12, "alg_frac": f_alg / t_s / 1e12 / PEAK_BF16_TFLOPS,
        "exec_tflops": f_exec / t_s / 1e12, "exec_frac": f_exec / t_s / 1e12 / PEAK_BF16_TFLOPS,
        "combine_GBps": None if ph["dz"] == 0.0 else 6.0 * V * tokens / (ph["dz"] * 1e-3) / 1e9,
        "grad_gemm_tflops": f_grad / (ph["grad"] * 1e-3) / 1e12}}

    cpu, parity = None, None
    if args.cpu_rows < 0:
        args.cpu_rows = 2048
    if args.cpu_rows > 0:
        cpu, (rows, kl, c, g) = _oracle_fused_baseline(w, prob, args.cpu_rows)
        # the timed call's own outputs on those rows
        idx = torch.from_numpy(rows).to(dev)
        got_kl = call.out["kl"][idx].double().cpu().numpy()
        got_c = call.out["c"][idx].double().cpu().numpy()
        probe = w.mode == synth.MODE_PREFIX_AND_FULL
        key = "dh_full" if probe else "dh_prefix"
        got_dh = call.out[key][idx].double().cpu().numpy()
        if probe:
            i = np.searchsorted(w.offsets, rows, side="right") - 1
            alpha = 1.0 / (w.B * np.maximum(lens[i], 1))
        else:
            alpha = _row_alpha_p(w, rows)
        ref_dh = g * alpha[:, None]
        scale = np.abs(ref_dh).max()
        tol_dh = DH_REL * scale + (2.0 ** -8 * np.abs(ref_dh) if args.dh_dtype == "bf16" else 0.0)
        kl_err = np.abs(got_kl - kl) / (KL_REL * np.abs(kl) + KL_ABS)
        parity = {"rows": int(len(rows)), "against": "fp64 oracle on the cpu_baseline sample",
                  "kl_rel_max": float((np.abs(got_kl - kl) / np.abs(kl)).max()),
                  "c_abs_max": float(np.abs(got_c - c).max()),
                  "dh_rel_max": float(np.abs(got_dh - ref_dh).max() / scale),
                  "bars": {"kl_rel": KL_REL, "dh_rel_of_max": DH_REL},
                  "ok": bool(kl_err.max() <= 1.0 and (np.abs(got_dh - ref_dh) <= tol_dh).all()
                             and (np.abs(got_c - c) <= 1e-3 * np.maximum(1.0, np.abs(c))).all())}

    line = {
        "metric": "distilled tokens/sec (fused fwd+bwd reverse-KL, V=151936) + % roofline",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": ms_median,
        "timing": "value and ms_per_step: wall clock around exactly `steps` calls, synchronised on both "
                  "sides; ms_per_step_median: HIP events on the launch stream around each of those calls",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "rollouts": w.B, "packed_rows": w.T, "computed_rows": tokens,
                   "V": w.V, "H_s": w.H_s, "H_t": w.H_t,
                   "mode": "prefix_and_full" if w.mode else "prefix_only", "estimator": args.estimator, "head_grad": bool(args.head_grad)},
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity, "phase_ms": ph,
    }
    line.update(extra)
    del call, prob
    torch.cuda.empty_cache()
    if not args.no_logits_given:
        line["logits_given"] = _bench_logits(B, synth, dev, max(args.steps, 10), cpu_rows_logits, est)
    line["ceilings"] = {"copy_GBps": B.adwin_opd_ceiling_copy(), "mfma_bf16_TFLOPs": B.adwin_opd_ceiling_mfma(),
                        "mfma_bf16_random_operands_TFLOPs": B.adwin_opd_ceiling_mfma_random(),
                        "note": "measured on this box: streaming copy (read+write bytes); "
                                "register-resident 32x32x16 bf16 MFMA loop with constant operands and "
                                "with pseudo-random operands (the rate the power limit sustains on "
                                "real data)"}
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
