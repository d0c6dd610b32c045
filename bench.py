#!/usr/bin/env python3
"""Benchmark of the calibration hot path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic activation batch:
conqur_step_batch (rotate + normalise + corner + accumulate), conqur_quant_error
(int4 score of the rotated batch) and conqur_update_rotation (Procrustes / polar).
Headline workload: c3 of the benchmark's configs -- d = 4096, bf16 activations, 2048 tokens
per batch, one update per batch, prox_lambda = 0.1 (the cross-covariance of a
2048-token batch is rank deficient at d = 4096).  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line.

  value            tokens/s of rotate+corner+accumulate alone (the metric's first
                   half): tokens per batch / device time of conqur_step_batch, from
                   one HIP event pair around the call's kernels, over the K timed steps
  roofline         the whole conqur_step_batch against the bf16 MFMA peak:
                   frac = value * 4 d^2 / 2.5e15; the two GEMM launches alone as gemm_pair
  stage_ms         from a second pass over the same K steps with an event pair
                   around every kernel (per-kernel durations) and in-kernel clock probes
  ms_per_procrustes  the metric's second half: device ms per conqur_update_rotation, in the
                   workload's configuration (prox_lambda as listed); procrustes_lambda_to_zero
                   is the same update with prox_lambda = 0 (the limit lambda -> 0+)
  ms_per_step      wall-clock per whole step (step_batch + quant_error + update)
  workloads        the other four configurations, compact: the same quantities each
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16/fp16 MFMA
PEAK_HBM_GBS = 8000.0


def measured_traffic(name):
    """HBM bytes per conqur_step_batch from the committed rocprofv3 --pmc summary of this workload (FETCH_SIZE and
    WRITE_SIZE passes scaled by a copy kernel of known size), or None if there is none.  The summary carries the
    figure on a line `traffic_bytes_per_step: N`."""
    path = os.path.join(ROOT, "profiles", f"step_{name}_pmc_traffic.txt")
    try:
        m = re.search(r"^traffic_bytes_per_step:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(w, X0, R0, sample_tokens):
    """The oracle, as it stands, on a bounded sample: one step_batch on `sample_tokens` rows of a batch, and one Procrustes
    at a width its Jacobi SVD finishes in seconds (extrapolated by its O(d^3) cost per sweep when that is below dh)."""
    from oracle import oracle as O
    import numpy as np
    oc = O.OracleCalibrator(w.d, w.heads, w.dtype, R0, w.prox_lambda)
    Xs = X0[:sample_tokens]
    t0 = time.perf_counter()
    oc.step_batch(Xs)
    dt = time.perf_counter() - t0
    ds = min(w.dh, 2048)
    A = np.random.Generator(np.random.Philox(key=1)).standard_normal((ds, ds))
    t1 = time.perf_counter()
    O.procrustes(A)
    dp = time.perf_counter() - t1
    scale = (w.dh / ds) ** 3 * w.heads
    how = (f"timed at d={ds}: {dp:.2f} s, x ({w.dh}/{ds})^3 = {dp * scale:.0f} s extrapolated" if ds < w.dh else
           f"at d={ds}: {dp:.2f} s per head, x {w.heads} heads = {dp * scale:.2f} s")
    return {
        "value": len(Xs) / dt, "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
        "sample": f"oracle step_batch (rotate+corner+accumulate, fp64 naive loops) on the first {len(Xs)} tokens of "
                  f"batch 0 of {w.name} (d={w.d}, heads={w.heads}), {dt:.2f} s; oracle Procrustes (one-sided Jacobi SVD) {how}",
        "procrustes_s": dp * scale,
    }


def run_workload(B, I, w, T, K, W, full, lam_zero_updates):
    """K timed steps (after W warm-up steps) of workload w with T tokens per batch.  full: also the second pass with
    per-kernel events, the clock probes and the extra score / emit kernels.  Returns the result dict."""
    import torch
    d, dh = w.d, w.dh
    n_distinct = min(K + W, 8 if d <= 4096 else 3)
    host = [I.batch(w, b, T) for b in range(n_distinct)]
    R0 = I.initial_rotation(w)
    dev = [B.to_device(x, w.dtype) for x in host]
    cal = B.Calibrator(d, w.heads, w.dtype, R0, max_tokens=T, prox_lambda=w.prox_lambda)
    res = {}
    if full:
        res["pr_start"] = float(cal.row_diagnostics(dev[0])[0].mean())   # mean PR/d of batch 0 under the initial rotation
    cal.set_timing(1)               # one event pair around each whole call

    def one_step(i):
        X = dev[i % n_distinct]
        cal.step_batch(X)
        sse, en = cal.quant_error(X, 4)
        _, st = cal.update_rotation()
        return sse / en, st

    for i in range(W):
        one_step(i)
    torch.cuda.synchronize()
    whole = {k: 0.0 for k in ("step", "quant", "update")}
    iters = 0
    issued = 0.0
    rel = []
    t0 = time.perf_counter()
    for i in range(W, W + K):
        r, st = one_step(i)
        tm = cal.timing()           # stream is already synchronised by update_rotation
        for k in whole:
            whole[k] += tm[k]
        iters += st[0]["iters"]
        issued += st[0]["mfma_flop"]
        rel.append(r)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for k in whole:
        whole[k] /= K
    # Second pass over the same K steps with an event pair around every kernel stage and the in-kernel clock
    # probes: the per-kernel durations.  (The extra event records serialise kernel launches, so these stages
    # sum to slightly more than the whole-call times of the first pass.)
    cal.set_timing(2)
    acc = {k: 0.0 for k in ("prep", "rotate", "accumulate", "stats", "update", "quant_rotate", "quant_error")}
    for i in range(W, W + K):
        one_step(i)
        tm = cal.timing()
        for k in acc:
            acc[k] += tm[k]
    probe = cal.clock_probe()       # of the last step's two GEMM launches
    for k in acc:
        acc[k] /= K
    step_ms = whole["step"]
    gemm_ms = acc["rotate"] + acc["accumulate"]
    step_flops = 4.0 * T * dh * dh * w.heads            # rotate + accumulate, per batch
    polar_flops = 4.0 * dh ** 3 * w.heads * (iters / K)  # one Gram + one apply per Newton-Schulz iteration
    y_bytes = T * d * (2 if w.dtype == "bf16" else 4)
    res.update(
        tokens_per_s=T / (step_ms * 1e-3), ms_per_step_batch=step_ms, ms_per_procrustes=whole["update"],
        ms_per_quant_error=whole["quant"], polar_iters=iters / K, wall_ms_per_step=wall * 1e3 / K,
        end_to_end_tokens_per_s=T * K / wall, stage_ms=acc, rel_first_last=[rel[0], rel[-1]], probe=probe,
        step_flops=step_flops, gemm_ms=gemm_ms, polar_flops=polar_flops, y_bytes=y_bytes,
        step_frac=step_flops / (step_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        polar_frac=polar_flops / (whole["update"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        polar_flops_issued=issued / K,
        polar_frac_issued=(issued / K) / (whole["update"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
    )
    if w.dh == 128 and w.dtype == "bf16":
        # heads of width 128 take the fused step kernel: bound by reading X once (256 bytes per token and head)
        res["step_hbm_gbs"] = T * d * 2 / (step_ms * 1e-3) / 1e9
    if full:
        # the zero-point (asymmetric) quantiser score at the paper's evaluation clipping ratio: same rotate GEMM, the
        # error kernel tracks min and max instead of max |y|
        zp_ms, zp_rel = 0.0, 0.0
        for i in range(K):
            s_zp, e_zp = cal.quant_error_zp(dev[i % n_distinct], 4, 0.9)
            zp_ms += cal.timing()["quant_error"]
            zp_rel = s_zp / e_zp
        res["zp_ms"], res["zp_rel"] = zp_ms / K, zp_rel
        # the same quantiser emitting the fake-quantised rotated rows (the input of a quantised layer): reads Y, writes Yq
        Yq = torch.empty((T, d), dtype=dev[0].dtype, device=dev[0].device)
        emit_ms = 0.0
        for i in range(K):
            cal.rotate_quant(dev[i % n_distinct], 4, True, 0.9, Yq)
            emit_ms += cal.timing()["quant_error"]
        res["emit_ms"] = emit_ms / K
        res["pr_end"] = float(cal.row_diagnostics(dev[0])[0].mean())
    cal.close()
    if lam_zero_updates and w.prox_lambda > 0.0:
        # the same update at prox_lambda = 0, i.e. the limit lambda -> 0+ (the library's floor 2^-20): R <- U V^T on the
        # range of M, the completion nearest R_prev on its null space; about twice the main steps
        c0 = B.Calibrator(d, w.heads, w.dtype, R0, max_tokens=T, prox_lambda=0.0)
        ms, it, orth = 0.0, 0, 0.0
        for i in range(lam_zero_updates + 1):
            c0.step_batch(dev[i % n_distinct])
            _, st = c0.update_rotation()
            if i:                                    # the first one warms up
                ms += st[0]["ms"]; it += st[0]["iters"]; orth = max(orth, st[0]["orth_err"])
        c0.close()
        res["lam0"] = {"ms_per_procrustes": ms / lam_zero_updates, "polar_iters": it / lam_zero_updates,
                       "device_orth_err_max": orth, "prox_lambda": 0.0,
                       "note": "prox_lambda = 0 is taken as lambda -> 0+ (floor 2^-20)"}
    res["host0"], res["R0"] = host[0], R0
    return res


def describe(w, T):
    return (f"{w.name}: d={w.d}, heads={w.heads}, {w.dtype} activations, {T} tokens/batch, one Procrustes update per "
            f"batch, prox_lambda={w.prox_lambda}, fp32 M and R")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--tokens", type=int, default=0,
                    help="tokens per batch instead of the workload's own (exploration only: the line's config then says so)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the compact runs of the other four configurations")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="0 = one whole batch")
    ap.add_argument("--pmc-copy", action="store_true",
                    help="also run three 256 MiB device-to-device copies (the known-size kernel that scales "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the path is single-device; sharded, every GPU would accumulate "
              "its own M over its tokens and all-reduce it before the update); --gpus N with N > 1 is not supported",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_10793_amd import binding as B
    from paper_2605_10793_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no HIP device", file=sys.stderr)
        sys.exit(1)
    w = I.WORKLOADS[args.workload]
    T, d = args.tokens or w.tokens_per_batch, w.d
    K, W = args.steps, args.warmup

    if args.pmc_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    r = run_workload(B, I, w, T, K, W, full=True, lam_zero_updates=3)
    acc = r["stage_ms"]
    out = {
        "metric": "calibration tokens/sec (rotate+corner+accumulate) at d=4096; ms per Procrustes",
        "value": r["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": r["wall_ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": describe(w, T), "tokens_per_batch": T, "d": d, "heads": w.heads},
        "ms_per_procrustes": r["ms_per_procrustes"],
        "ms_per_procrustes_note": f"the workload's own configuration, prox_lambda={w.prox_lambda}",
        "ms_per_quant_error": r["ms_per_quant_error"],
        "polar_iters_per_update": r["polar_iters"],
        "end_to_end_tokens_per_s": r["end_to_end_tokens_per_s"],
        "stage_ms": acc,
        "stage_ms_note": "second pass of the same steps with an event pair around every kernel stage",
        "int4_rel_err_first_last": r["rel_first_last"],
        "mean_participation_ratio_first_last": [r["pr_start"], r["pr_end"]],
        "roofline": {
            "bound": "mfma", "kernel": "conqur_step_batch (row norms, scaled transpose, rotate+corner GEMM, accumulate GEMM)",
            "achieved": r["step_flops"] / (r["ms_per_step_batch"] * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": r["step_frac"],
            "traffic": measured_traffic(w.name) if T == w.tokens_per_batch else None,
            "traffic_source": f"profiles/step_{w.name}_pmc_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes)",
            "flops_per_step": r["step_flops"], "ms_per_step_batch": r["ms_per_step_batch"],
            "measured_over": "one HIP event pair on the library's stream around each conqur_step_batch, the K timed steps",
            "gemm_pair": {
                "kernel": "gemm_nt_kernel (rotate+corner launch and accumulate launch of step_batch)",
                "achieved": r["step_flops"] / (r["gemm_ms"] * 1e-3) / 1e12,
                "frac": r["step_flops"] / (r["gemm_ms"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "ms": r["gemm_ms"],
                "measured_over": "per-kernel HIP events, second pass of the same steps",
            },
            # in-kernel probe: the shader clock the chip sustains while these kernels' MFMAs run (the published peak
            # assumes 2400 MHz) and where each launch's time goes
            "clock_probe": r["probe"],
        },
        "roofline_polar": {
            "bound": "mfma", "achieved": r["polar_flops"] / (r["ms_per_procrustes"] * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": r["polar_frac"],
            "issued": {"achieved": r["polar_flops_issued"] / (r["ms_per_procrustes"] * 1e-3) / 1e12, "frac": r["polar_frac_issued"],
                       "flop_per_update": r["polar_flops_issued"]},
            "note": "achieved / frac: algorithmic 4*d^3 per polar iteration (one Gram matrix, one apply) over the whole "
                    "update; issued: the MFMA work the update's launches really ran, as the library counts it "
                    "(conqur_update_stats.mfma_flop: symmetric products run on the tiles on and above the diagonal only, "
                    "the closing step adds the D^2 and two-plane correction products)",
        },
        "roofline_quant_error": {
            "bound": "hbm", "achieved": r["y_bytes"] / (acc["quant_error"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": r["y_bytes"] / (acc["quant_error"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
        },
        "roofline_quant_error_zp": {
            "bound": "hbm", "achieved": r["y_bytes"] / (r["zp_ms"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": r["y_bytes"] / (r["zp_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, "ms": r["zp_ms"], "clip_ratio": 0.9,
            "int4_rel_err": r["zp_rel"],
        },
        "roofline_rotate_quant_emit": {
            "bound": "hbm", "achieved": 2 * r["y_bytes"] / (r["emit_ms"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": 2 * r["y_bytes"] / (r["emit_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, "ms": r["emit_ms"], "clip_ratio": 0.9,
        },
    }
    if "lam0" in r:
        out["procrustes_lambda_to_zero"] = r["lam0"]
    if w.dh == 128 and w.dtype == "bf16":
        x_bytes = T * d * 2
        out["roofline"] = {
            "bound": "hbm", "kernel": "conqur_step_batch (k_head_step128 and the reduction of the token shares)",
            "achieved": r["step_hbm_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": r["step_hbm_gbs"] / PEAK_HBM_GBS,
            "traffic": measured_traffic(w.name), "bytes_per_step": x_bytes, "ms_per_step_batch": r["ms_per_step_batch"],
            "measured_over": "one HIP event pair on the library's stream around each conqur_step_batch",
        }
    host0, R0 = r["host0"], r["R0"]
    if not args.no_other_workloads and not args.tokens:
        # the other four configurations, compact (fewer steps; the same timing as above)
        others = []
        for name in ("c1", "c2", "c3", "c4", "c5"):
            if name == w.name:
                continue
            wo = I.WORKLOADS[name]
            Ko = max(2, min(K, 8 if wo.d <= 4096 else 3))
            ro = run_workload(B, I, wo, wo.tokens_per_batch, Ko, 2, full=False, lam_zero_updates=2)
            e = {"workload": describe(wo, wo.tokens_per_batch), "steps": Ko, "tokens_per_s": ro["tokens_per_s"],
                 "ms_per_step_batch": ro["ms_per_step_batch"], "ms_per_procrustes": ro["ms_per_procrustes"],
                 "polar_iters_per_update": ro["polar_iters"], "end_to_end_tokens_per_s": ro["end_to_end_tokens_per_s"],
                 "ms_per_quant_error": ro["ms_per_quant_error"]}
            if "step_hbm_gbs" in ro:
                e["roofline"] = {"bound": "hbm", "achieved": ro["step_hbm_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                 "frac": ro["step_hbm_gbs"] / PEAK_HBM_GBS,
                                 "note": "fused per-head step: bound by reading X once (256 bytes per token and head)"}
            else:
                e["roofline"] = {"bound": "mfma", "achieved": ro["step_frac"] * PEAK_BF16_TFLOPS, "peak": PEAK_BF16_TFLOPS,
                                 "unit": "TFLOP/s", "frac": ro["step_frac"],
                                 "note": "whole conqur_step_batch, 4 dh^2 heads FLOP per token"}
            e["roofline_polar_frac"] = ro["polar_frac"]
            e["roofline_polar_frac_issued"] = ro["polar_frac_issued"]
            if "lam0" in ro:
                e["procrustes_lambda_to_zero"] = ro["lam0"]
            others.append(e)
            del ro
        out["workloads"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, host0, R0, args.cpu_sample_tokens or T)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
