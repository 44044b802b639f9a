#!/usr/bin/env python3
"""Benchmark of the fused LM-head + cross-entropy hot path on one MI355X.

A step is one cce_forward + cce_backward over one batch of the Qwen2.5-0.5B LM-head
shape (N = 8192 tokens, D = 896, V = 151936; seeded synthetic inputs, already resident in
HBM).  Prints ONE JSON line: tokens/s (the headline metric of this build), the MFMA roofline
of the dominant kernel family measured with HIP events inside the timed steps, and the
fp64 CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload qwen05b] [--no-cpu-baseline]
                    [--no-other-configs] [--calibrate-matmul] [--calibrate-copy] [--all-rows]

After the headline region the other full-size configurations (1b, 7b, smallv) are timed as well
(3 steps each, inputs generated on the box from the seed) and reported under `other_configs`;
`value` stays the headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
METRIC = "fused linear-CE fwd+bwd tokens/s at N=8192,D=896,V=151936; % bf16 MFMA peak"


def stored_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc summary kept under profiles/
    (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel calibration), or None.  Counters cannot
    be read from inside this process, so the figure comes from that separate, committed run."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}.txt")
    try:
        for line in open(path):
            t = line.split()
            if len(t) >= 3 and t[0] == "traffic_bytes_per_launch" and t[1] == kernel:
                return float(t[2])
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="qwen05b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-rows", action="store_true",
                    help="time cce_forward + cce_backward (every row goes through the kernels) as the headline "
                         "instead of the row-skipping entry points")
    ap.add_argument("--cpu-sample-rows", type=int, default=8192)
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the timing of the other full-size configurations (1b, 7b, smallv)")
    ap.add_argument("--calibrate-matmul", action="store_true",
                    help="also time the vendor GEMM (torch.matmul, bf16) at 8192^3 and at the forward's own shape, on "
                         "random and on constant data: the calibration of what a plain GEMM sustains on this device")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size reference that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this script")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path would shard over tokens or over the "
              "vocabulary, but no multi-GPU code is part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2601_02609_amd import binding as B, build, inputs as I

    if not build.is_built():
        build.build(verbose=False)
    B.lib()                                   # raises if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    w = I.make_config(args.workload)
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    dev = torch.device("cuda:0")
    H = torch.from_numpy(w.hidden.view(np.int16)).to(dev).view(torch.bfloat16)
    W = torch.from_numpy(w.weight.view(np.int16)).to(dev).view(torch.bfloat16)
    y = torch.from_numpy(w.labels).to(dev)
    dl = torch.from_numpy(w.dloss_mean).to(dev)
    ws = B.alloc_workspace(N, D, V)
    loss = torch.empty(N, dtype=torch.float32, device=dev)
    lse = torch.empty(N, dtype=torch.float32, device=dev)
    dH = torch.empty(N, D, dtype=torch.bfloat16, device=dev)
    dW = torch.empty(V, D, dtype=torch.float32, device=dev)

    def all_rows_step():
        B.cce_forward(H, W, y, w.spec.ignore_index, workspace=ws, loss=loss, lse=lse)
        B.cce_backward(H, W, y, lse, dl, w.spec.ignore_index, workspace=ws, d_hidden=dH, d_weight=dW)

    # Row skipping (include/cce_compact.h): rows whose label is ignore_index take no part in the
    # loss, so the entry points that are told how many rows are valid leave them out of every
    # product.  The count comes from the host copy of the labels, as a data loader has it.
    n_valid_host = int(((w.labels != w.spec.ignore_index) & (w.labels >= 0) & (w.labels < V)).sum())
    skipping = (not args.all_rows) and B.get_row_skipping(N, D, V, n_valid_host)
    wc = B.alloc_compact_workspace(N, D, V, n_valid_host)

    def skip_step():
        B.cce_forward_compact(H, W, y, n_valid_host, w.spec.ignore_index, workspace=wc, loss=loss, lse=lse)
        B.cce_backward_compact(H, W, y, lse, dl, n_valid_host, w.spec.ignore_index, workspace=wc, d_hidden=dH, d_weight=dW)

    step = skip_step if skipping else all_rows_step
    ws_used = wc if skipping else ws
    rows_run = n_valid_host if skipping else N          # rows whose products are computed

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: exactly K steps, bracketed by synchronisation
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    total_ms = e0.elapsed_time(e1)
    ms_per_step = total_ms / args.steps
    tok_s = N * args.steps / (total_ms * 1e-3)

    # the same K steps once more with the library's HIP events around every kernel launch
    # (same stream): per-family launch durations for the roofline.  Kept out of the region
    # above because ~150 event pairs per step add a few percent of gaps between launches.
    B.profile_begin()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    profiled_ms_per_step = e0.elapsed_time(e1) / args.steps
    fam = B.profile_end()

    # sanity on the outputs of the last step (finite loss, non-zero gradient, bad labels none)
    n_valid = w.n_valid
    mean_loss = float(loss.sum().item()) / max(n_valid, 1)
    grad_norm = float(dW.double().pow(2).sum().sqrt().item())
    assert np.isfinite(mean_loss) and grad_norm > 0.0 and B.read_status(ws_used) == 0

    nvd = float(rows_run) * V * D
    # algorithmic MFMA flops per step of each family, over the rows that are computed (all N, or
    # the valid ones when rows are skipped: flops that are not run are not counted)
    fam_flops = {"lse_partial_kernel": 2 * nvd, "grad_tile_kernel": 2 * nvd, "grad_gemm_kernel": 4 * nvd}
    dom = max(fam, key=lambda k: fam[k][0])
    dom_ms, dom_launches = fam[dom]
    achieved = fam_flops[dom] * args.steps / (dom_ms * 1e-3) / 1e12
    executed_tflops = 8 * nvd / (ms_per_step * 1e-3) / 1e12
    roofline = {
        "bound": "mfma", "kernel": dom, "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
        "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
        "traffic": stored_traffic(args.workload, dom + ("/row_skipping" if skipping else "")),
        "avg_launch_us": round(dom_ms * 1e3 / max(dom_launches, 1), 2),
        "launches_per_step": dom_launches // max(args.steps, 1),
        "flops_per_launch": fam_flops[dom] * args.steps / max(dom_launches, 1),
        "timed": f"second pass of the same {args.steps} steps with HIP events around every launch "
                 f"({profiled_ms_per_step:.3f} ms/step with events)",
        "families_ms_per_step": {k: round(v[0] / args.steps, 4) for k, v in fam.items()},
        "families_tflops": {k: round(fam_flops[k] * args.steps / (v[0] * 1e-3) / 1e12, 1) if v[0] > 0 else None
                            for k, v in fam.items()},
    }

    # The steps around the path (not part of a timed step): one-pass HBM-bound kernels, timed
    # with events on the stream they run on, reported as achieved bytes/s of their algorithmic
    # traffic against the 8 TB/s HBM peak.
    def timed_us(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    def timed_us_graph(fn, reps=20):
        """Launches of a few microseconds: the host cannot enqueue them as fast as they run (a call
        through the binding costs ~20 us), so `reps` calls are captured in one HIP graph and the
        replay is timed -- device time per call, launch gaps between the nodes included."""
        fn()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for _ in range(reps):
                    fn()
        g.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        g.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / reps

    gam = torch.ones(D, dtype=torch.bfloat16, device=dev)
    yn, dxn = torch.empty_like(H), torch.empty_like(H)
    _, rstd = B.cce_rmsnorm_forward(H, gam, 1e-6, y=yn)
    dgam = torch.empty(D, dtype=torch.float32, device=dev)
    nws = torch.empty(B.lib().cce_rmsnorm_workspace_bytes(N, D), dtype=torch.uint8, device=dev)
    sws = torch.empty(B.lib().cce_sumsq_workspace_bytes(), dtype=torch.uint8, device=dev)
    ssq = torch.empty(1, dtype=torch.float64, device=dev)
    master = W.float().view(-1)
    mom, var = torch.zeros_like(master), torch.zeros_like(master)
    Wcopy = torch.empty_like(W)
    aux_us = {
        "rmsnorm_forward": timed_us_graph(lambda: B.cce_rmsnorm_forward(H, gam, 1e-6, y=yn, rstd=rstd)),
        "rmsnorm_backward": timed_us_graph(lambda: B.cce_rmsnorm_backward(H, gam, rstd, dH, dx=dxn, dgamma=dgam, workspace=nws)),
        "grad_sumsq": timed_us_graph(lambda: B.cce_grad_sumsq(dW.view(-1), sumsq=ssq, workspace=sws)),
        "adamw_step": timed_us(lambda: B.cce_adamw_step(master, dW.view(-1), mom, var, 1, lr=0.0, param_bf16=Wcopy.view(-1))),
    }
    aux_bytes = {"rmsnorm_forward": 4.0 * N * D, "rmsnorm_backward": 6.0 * N * D,
                 "grad_sumsq": 4.0 * V * D, "adamw_step": 30.0 * V * D}
    aux = {k: {"us": round(aux_us[k], 1), "GB_per_s": round(aux_bytes[k] / aux_us[k] * 1e-3, 0),
               "frac_of_8TBps": round(aux_bytes[k] / aux_us[k] * 1e-3 / 8000.0, 3)} for k in aux_us}
    del master, mom, var, Wcopy

    # The FP8 variant of the same step (logit products in E4M3 on the block-scaled MFMA, gradient
    # contractions in bf16), next to the headline: not `value`, which stays the bf16 path.
    fp8 = None
    nvd_all = float(N) * V * D              # the FP8 variant runs all rows
    if D % 128 == 0:
        hq, hsc = B.cce_quantize_e4m3(H)
        wq, wsc = B.cce_quantize_e4m3(W)
        q_us = timed_us(lambda: (B.cce_quantize_e4m3(H, q=hq, scales=hsc), B.cce_quantize_e4m3(W, q=wq, scales=wsc)))
        f_us = timed_us(lambda: B.cce_fp8_forward(hq, hsc, wq, wsc, y, w.spec.ignore_index, workspace=ws, loss=loss, lse=lse))
        b_us = timed_us(lambda: B.cce_fp8_backward(hq, hsc, wq, wsc, H, W, y, lse, dl, w.spec.ignore_index,
                                                   workspace=ws, d_hidden=dH, d_weight=dW), reps=10)
        step_us = q_us + f_us + b_us
        fp8 = {"ms_per_step_with_quantisation": round(step_us * 1e-3, 4), "tokens_per_s": round(N / (step_us * 1e-6), 1),
               "quantise_us": round(q_us, 1), "quantise_GB_per_s": round(3.0 * (N + V) * D / q_us * 1e-3, 0),
               "forward_us": round(f_us, 1), "forward_tflops": round(2 * nvd_all / (f_us * 1e-6) / 1e12, 1),
               "forward_frac_of_fp8_mfma_peak": round(2 * nvd_all / (f_us * 1e-6) / 1e12 / 5000.0, 3),
               "backward_us": round(b_us, 1)}
        del hq, hsc, wq, wsc

    # The other path of the two (all rows / row skipping), same buffers, for comparison.
    other = all_rows_step if skipping else skip_step
    o_us = timed_us(other, reps=10)
    o_rows = N if skipping else n_valid_host
    other_path = {"entry_points": "cce_forward + cce_backward (all rows)" if skipping
                  else "cce_forward_compact + cce_backward_compact",
                  "rows_skipped": (not skipping) and bool(B.get_row_skipping(N, D, V, n_valid_host)),
                  "ms_per_step": round(o_us * 1e-3, 4), "tokens_per_s": round(N / (o_us * 1e-6), 1),
                  "rows_computed": int(o_rows),
                  "tflops_executed": round(8.0 * o_rows * V * D / (o_us * 1e-6) / 1e12, 1),
                  "pct_bf16_mfma_peak": round(100 * 8.0 * o_rows * V * D / (o_us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2),
                  "workspace_bytes": int((ws if skipping else wc).numel())}

    # what the peak is divided by: the nominal figure, the one the device properties give
    # (compute units x 4096 flop/clock x clock), and a register-only MFMA loop on this device
    cus, khz = B.device_info()
    # register-only loop on operands loaded once from memory: the same instruction stream on random
    # normal values and on constants -- the difference is the device's response to operand activity
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    probe_rand = torch.randn(512 * 48, device=dev, generator=gen).bfloat16()
    B.mfma_probe_data_tflops(probe_rand, iters=4000)          # clocks up
    peak_info = {
        "nominal_tflops": MFMA_BF16_PEAK_TFLOPS,
        "from_device_properties_tflops": round(cus * 4096 * khz * 1e3 / 1e12, 1),
        "compute_units": cus, "clock_mhz": khz // 1000,
        "register_only_mfma_loop_tflops": round(B.mfma_probe_tflops(iters=20000), 1),
        "register_only_random_operands_tflops": round(B.mfma_probe_data_tflops(probe_rand, iters=20000), 1),
        "register_only_constant_operands_tflops": round(B.mfma_probe_data_tflops(torch.full_like(probe_rand, 0.5), iters=20000), 1),
        "register_only_zero_operands_tflops": round(B.mfma_probe_data_tflops(torch.zeros_like(probe_rand), iters=20000), 1),
    }
    roofline["practical_peak"] = {
        "register_only_random_operands_tflops": peak_info["register_only_random_operands_tflops"],
        "note": "rate of a register-only MFMA loop on random bf16 operands on this device (no LDS, no memory): what the "
                "matrix cores sustain at the clock the device holds under operand activity; `frac` stays against the nominal peak"}

    matmul_cal = None
    if args.calibrate_matmul:
        def mm_tflops(M, Nn, K, kind, reps=10):
            if kind == "random":
                a = torch.randn(M, K, device=dev).bfloat16()
                b = torch.randn(Nn, K, device=dev).bfloat16()
            else:
                a = torch.full((M, K), 0.5, device=dev).bfloat16()
                b = torch.full((Nn, K), 0.25, device=dev).bfloat16()
            c = a @ b.T
            torch.cuda.synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record()
            for _ in range(reps):
                c = a @ b.T
            t1.record()
            torch.cuda.synchronize()
            del a, b, c
            return round(2.0 * M * Nn * K * reps / (t0.elapsed_time(t1) * 1e-3) / 1e12, 1)
        matmul_cal = {f"{m}x{n}x{k}_{kind}": mm_tflops(m, n, k, kind)
                      for (m, n, k) in ((8192, 8192, 8192), (8192, 151936, 896), (16384, 8192, 4096))
                      for kind in ("random", "constant")}
        matmul_cal["what"] = "torch.matmul (vendor GEMM) bf16 TFLOP/s, M x N x K, random normal vs constant operands"

    # The other full-size configurations, through the entry points the library itself would pick
    # (row skipping where its planner rates it faster, else all rows): 3 timed steps each after one
    # warm-up step.  Inputs are generated here from the seed; the headline tensors are freed first.
    other_configs = None
    if not args.no_other_configs and args.workload == "qwen05b":
        del H, W, y, dl, ws, wc, loss, lse, dH, dW, gam, yn, dxn, rstd, dgam, nws, sws, ssq
        torch.cuda.empty_cache()
        other_configs = {}
        for name in ("1b", "7b", "smallv"):
            wo = I.make_config(name)
            No, Do, Vo = wo.spec.N, wo.spec.D, wo.spec.V
            Ho = torch.from_numpy(wo.hidden.view(np.int16)).to(dev).view(torch.bfloat16)
            Wo = torch.from_numpy(wo.weight.view(np.int16)).to(dev).view(torch.bfloat16)
            yo = torch.from_numpy(wo.labels).to(dev)
            dlo = torch.from_numpy(wo.dloss_mean).to(dev)
            nv = int(((wo.labels != wo.spec.ignore_index) & (wo.labels >= 0) & (wo.labels < Vo)).sum())
            skip_o = bool(B.get_row_skipping(No, Do, Vo, nv))
            wso = B.alloc_compact_workspace(No, Do, Vo, nv) if skip_o else B.alloc_workspace(No, Do, Vo)
            lo = torch.empty(No, dtype=torch.float32, device=dev)
            so = torch.empty(No, dtype=torch.float32, device=dev)
            dHo = torch.empty(No, Do, dtype=torch.bfloat16, device=dev)
            dWo = torch.empty(Vo, Do, dtype=torch.float32, device=dev)

            def step_o():
                if skip_o:
                    B.cce_forward_compact(Ho, Wo, yo, nv, wo.spec.ignore_index, workspace=wso, loss=lo, lse=so)
                    B.cce_backward_compact(Ho, Wo, yo, so, dlo, nv, wo.spec.ignore_index, workspace=wso, d_hidden=dHo, d_weight=dWo)
                else:
                    B.cce_forward(Ho, Wo, yo, wo.spec.ignore_index, workspace=wso, loss=lo, lse=so)
                    B.cce_backward(Ho, Wo, yo, so, dlo, wo.spec.ignore_index, workspace=wso, d_hidden=dHo, d_weight=dWo)
            us = timed_us(step_o, reps=3)
            assert B.read_status(wso) == 0 and bool(torch.isfinite(lo).all())
            rows_o = nv if skip_o else No
            tf = 8.0 * rows_o * Vo * Do / (us * 1e-6) / 1e12
            other_configs[name] = {
                "N": No, "D": Do, "V": Vo, "n_valid": nv, "ms_per_step": round(us * 1e-3, 3),
                "tokens_per_s": round(No / (us * 1e-6), 1),
                "rows_computed": int(rows_o), "tflops_executed": round(tf, 1),
                "pct_bf16_mfma_peak": round(100 * tf / MFMA_BF16_PEAK_TFLOPS, 2),
                "workspace_bytes": int(wso.numel()),
                "workspace_pct_of_logits": round(100.0 * wso.numel() / B.materialised_logit_bytes(No, Vo), 3),
                "entry_points": "cce_forward_compact + cce_backward_compact" if skip_o else "cce_forward + cce_backward",
                "backward_tiling_256": list(B.get_compact_tiling(No, Do, Vo, nv) if skip_o else B.get_backward_tiling(No, Do, Vo)),
                "backward_gemm_tile": list(B.get_backward_gemm_tile(nv if skip_o else No, Do, Vo)),
                "steps": 3, "mean_loss": round(float(lo.sum().item()) / max(nv, 1), 5)}
            del wo, Ho, Wo, yo, dlo, wso, lo, so, dHo, dWo
            torch.cuda.empty_cache()

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import cce_oracle as O     # baseline leg only; never on the product path
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
        except Exception:
            cores = os.cpu_count() or 1
        rows = min(args.cpu_sample_rows, N)
        t0 = time.perf_counter()
        O.forward(w.hidden[:rows], w.weight, w.labels[:rows], w.spec.ignore_index)
        O.backward(w.hidden[:rows], w.weight, w.labels[:rows], w.dloss_mean[:rows], w.spec.ignore_index)
        dt = time.perf_counter() - t0
        cpu = {"value": round(rows / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "fp64_gflops_6NVD": round(6.0 * rows * V * D / dt / 1e9, 1),
               "sample": f"fp64 oracle forward+backward on the first {rows} of {N} rows with the full "
                         f"V={V} vocabulary ({dt:.1f} s wall)"}

    out = {
        "metric": METRIC, "value": round(tok_s, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={N} D={D} V={V}, {w.spec.ignore_frac:.0%} ignore_index, "
                               f"seed {w.spec.seed}", "n_valid": n_valid,
                   "entry_points": "cce_forward_compact + cce_backward_compact (rows with ignore_index are left out of "
                                   "every product; the count of valid rows is taken from the host copy of the labels)"
                                   if skipping else "cce_forward + cce_backward (all rows)"},
        "valid_tokens_per_s": round(n_valid / (ms_per_step * 1e-3), 1),
        "tflops_executed_8NVD": round(executed_tflops, 1),
        "tflops_model_6NVD": round(6 * nvd / (ms_per_step * 1e-3) / 1e12, 1),
        "pct_bf16_mfma_peak": round(100 * executed_tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "rows_computed": int(rows_run),
        "workspace_bytes": int(ws_used.numel()),
        "workspace_pct_of_logits": round(100.0 * ws_used.numel() / B.materialised_logit_bytes(N, V), 3),
        "backward_tiling_256": list(B.get_compact_tiling(N, D, V, n_valid) if skipping else B.get_backward_tiling(N, D, V)),
        "mean_loss": round(mean_loss, 5),
        "roofline": roofline, "cpu_baseline": cpu, "other_configs": other_configs, "around_the_path_hbm": aux,
        "fp8_variant": fp8, "other_path": other_path, "mfma_peak": peak_info, "matmul_calibration": matmul_cal,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
