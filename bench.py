#!/usr/bin/env python3
"""Benchmark of the calibration hot path on one MI355X.

One "step" = one pass of the whole hot path over one synthetic activation batch:
conqur_step_batch (rotate + normalise + corner + accumulate), conqur_quant_error
(int4 score of the rotated batch) and conqur_update_rotation (Procrustes / polar).
Workload: c3 of the benchmark's configs -- d = 4096, bf16 activations, 2048 tokens per
batch, one update per batch, prox_lambda = 0.1 (the cross-covariance of a 2048-token
batch is rank deficient at d = 4096).  Inputs are resident in HBM before the timed
region.  Prints ONE JSON line.

  value            tokens/s of rotate+corner+accumulate alone (the metric's first
                   half): tokens per batch / device time of conqur_step_batch, from
                   one HIP event pair around the call's kernels, over the K timed steps
  stage_ms, roofline  from a second pass over the same K steps with an event pair
                   around every kernel (per-kernel durations) and in-kernel clock probes
  ms_per_procrustes  the metric's second half: device ms per conqur_update_rotation
  ms_per_step      wall-clock per whole step (step_batch + quant_error + update)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16/fp16 MFMA
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per step_batch GEMM launch pair on c3, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes scaled by a
# 256 MiB copy (profiles/bench_c3_pmc_traffic_mfma.txt): fetch 224.4 MiB + write 80.0 MiB.
MEASURED_TRAFFIC_BYTES = {"c3": 3.19e8}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--tokens", type=int, default=0,
                    help="tokens per batch instead of the workload's own (exploration only: the line's config then says so)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    import numpy as np
    import torch
    from paper_2605_10793_amd import binding as B
    from paper_2605_10793_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no HIP device", file=sys.stderr)
        sys.exit(1)
    w = I.WORKLOADS[args.workload]
    T, d = args.tokens or w.tokens_per_batch, w.d
    K, W = args.steps, args.warmup
    n_distinct = min(K + W, 8)
    host = [I.batch(w, b, T) for b in range(n_distinct)]
    R0 = I.initial_rotation(w)
    dev = [B.to_device(x, w.dtype) for x in host]
    cal = B.Calibrator(d, w.heads, w.dtype, R0, max_tokens=T, prox_lambda=w.prox_lambda)
    pr_start = float(cal.row_diagnostics(dev[0])[0].mean())      # mean PR/d of batch 0 under the initial rotation
    cal.set_timing(1)               # one event pair around each whole call

    def one_step(i):
        X = dev[i % n_distinct]
        cal.step_batch(X)
        sse, en = cal.quant_error(X, 4)
        _, st = cal.update_rotation()
        return sse / en, st

    if args.pmc_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    for i in range(W):
        one_step(i)
    torch.cuda.synchronize()
    whole = {k: 0.0 for k in ("step", "quant", "update")}
    iters = 0
    rel = []
    t0 = time.perf_counter()
    for i in range(W, W + K):
        r, st = one_step(i)
        tm = cal.timing()           # stream is already synchronised by update_rotation
        for k in whole:
            whole[k] += tm[k]
        iters += st[0]["iters"]
        rel.append(r)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for k in whole:
        whole[k] /= K
    # Second pass over the same K steps with an event pair around every kernel stage and the in-kernel clock
    # probes: the per-kernel durations the rooflines use.  (The extra event records serialise kernel launches,
    # so these stages sum to slightly more than the whole-call times of the first pass.)
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
    # the zero-point (asymmetric) quantiser score at the paper's evaluation clipping ratio: same rotate GEMM, the
    # error kernel tracks min and max instead of max |y|
    zp_ms, zp_rel = 0.0, 0.0
    for i in range(K):
        s_zp, e_zp = cal.quant_error_zp(dev[i % n_distinct], 4, 0.9)
        zp_ms += cal.timing()["quant_error"]
        zp_rel = s_zp / e_zp
    zp_ms /= K
    # the same quantiser emitting the fake-quantised rotated rows (the input of a quantised layer): reads Y, writes Yq
    import torch
    Yq = torch.empty((T, d), dtype=dev[0].dtype, device=dev[0].device)
    emit_ms = 0.0
    for i in range(K):
        cal.rotate_quant(dev[i % n_distinct], 4, True, 0.9, Yq)
        emit_ms += cal.timing()["quant_error"]
    emit_ms /= K
    step_ms = whole["step"]
    gemm_ms = acc["rotate"] + acc["accumulate"]
    dh = w.dh
    step_flops = 4.0 * T * dh * dh * w.heads            # rotate + accumulate, per batch
    polar_flops = 4.0 * dh ** 3 * w.heads * (iters / K)  # one Gram + one apply per Newton-Schulz iteration
    y_bytes = T * d * (2 if w.dtype == "bf16" else 4)
    out = {
        "metric": "calibration tokens/sec (rotate+corner+accumulate) at d=4096; ms per Procrustes",
        "value": T / (step_ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall * 1e3 / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: d={d}, heads={w.heads}, {w.dtype} activations, {T} tokens/batch, one "
                               f"Procrustes update per batch, prox_lambda={w.prox_lambda}, fp32 M and R",
                   "tokens_per_batch": T, "d": d, "heads": w.heads},
        "ms_per_procrustes": whole["update"],
        "ms_per_quant_error": whole["quant"],
        "polar_iters_per_update": iters / K,
        "end_to_end_tokens_per_s": T * K / wall,
        "stage_ms": acc,
        "stage_ms_note": "second pass of the same steps with an event pair around every kernel stage",
        "int4_rel_err_first_last": [rel[0], rel[-1]],
        "mean_participation_ratio_first_last": [pr_start, float(cal.row_diagnostics(dev[0])[0].mean())],
        "roofline": {
            "bound": "mfma", "kernel": "gemm_nt_kernel (rotate+corner launch and accumulate launch of step_batch)",
            "achieved": step_flops / (gemm_ms * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": step_flops / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(w.name) if T == w.tokens_per_batch else None,
            "flops_per_launch_pair": step_flops, "ms_per_launch_pair": gemm_ms,
            "measured_over": "per-kernel HIP events on the library's stream, second pass of the same steps",
            # in-kernel probe: the shader clock the chip sustains while these kernels' MFMAs run (the published peak
            # assumes 2400 MHz) and where each launch's time goes
            "clock_probe": probe,
        },
        "roofline_polar": {
            "bound": "mfma", "achieved": polar_flops / (acc["update"] * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": polar_flops / (acc["update"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "note": "algorithmic 4*d^3 per polar iteration (one Gram matrix, one apply) over the whole update; the "
                    "MFMA work actually issued differs: symmetric products run on the tiles on and above the "
                    "diagonal only, the closing step adds the D^2, ||D^3|| and two-plane correction products",
        },
        "roofline_quant_error": {
            "bound": "hbm", "achieved": y_bytes / (acc["quant_error"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": y_bytes / (acc["quant_error"] * 1e-3) / 1e9 / PEAK_HBM_GBS,
        },
    }
    out["roofline_quant_error_zp"] = {
        "bound": "hbm", "achieved": y_bytes / (zp_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": y_bytes / (zp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "ms": zp_ms, "clip_ratio": 0.9, "int4_rel_err": zp_rel,
    }
    out["roofline_rotate_quant_emit"] = {
        "bound": "hbm", "achieved": 2 * y_bytes / (emit_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": 2 * y_bytes / (emit_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "ms": emit_ms, "clip_ratio": 0.9,
    }
    if w.dh == 128 and w.dtype == "bf16":
        # heads of width 128 take the fused step kernel: bound by reading X once (256 bytes per token and head)
        x_bytes = T * d * 2
        out["roofline"] = {
            "bound": "hbm", "kernel": "k_head_step128 + k_head_reduce (the whole step_batch)",
            "achieved": x_bytes / (gemm_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": x_bytes / (gemm_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None,
            "bytes_per_launch_pair": x_bytes, "ms_per_launch_pair": gemm_ms,
            "measured_over": "per-kernel HIP events on the library's stream, second pass of the same steps",
        }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, host[0], R0, args.cpu_sample_tokens or T)
    cal.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
