#!/usr/bin/env python3
"""Benchmark of the KurTail rotation-learning step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic calibration
activations resident in HBM: kt_kurtosis_loss_grad (forward GEMM + row moments, which also keeps
Y in fp32 scratch; row finalisation; dL/dY from the kept Y; X^T G GEMM) followed by kt_cayley_step.
With --recompute the library gets its smaller workspace and recomputes Y with a second GEMM instead.
Prints ONE JSON line: tokens/s for the whole step, the roofline figures of the dominant
kernel measured with HIP events inside the timed region, and the fp64 CPU oracle timed on
a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 matrix
KERNEL_NAMES = {0: "gemm_nt_kernel<bf16 256x256, EpiMoments> (forward + row moments)",
                1: "gemm_nt_kernel<bf16 256x256, EpiGrad> (recompute + dL/dY)",
                2: "gemm_nt_kernel<bf16 256x256, EpiStore> (dR = X^T G)"}
KERNEL_NAMES_KEEP = {0: "gemm_nt_kernel<bf16 256x256, EpiMomentsKeep> (forward + row moments + Y kept in fp32)",
                     2: "gemm_nt_kernel<bf16 256x256, EpiStore> (dR = X^T G)"}
# Fabric-side bytes per launch (rocprofv3 --pmc FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, calibrated on a 1 GiB
# device copy; see profiles/c3_gemm_counters.md).  Counters need a profiler run of their own, so the
# figures measured for the default workload are carried here as constants; other workloads report null.
MEASURED_TRAFFIC_BYTES = {"C3": {"recompute": {0: (6.00 + 0.0625) * 2**30, 1: (6.01 + 1.0) * 2**30, 2: (6.00 + 0.0625) * 2**30},
                                 "keep": {0: (6.05 + 2.14) * 2**30, 2: (6.00 + 0.0625) * 2**30}}}
CPU_SAMPLE_ROWS = {"C1": 2048, "C2": 32768, "C3": 16384, "C4": 131072, "C5": 4096}


class ClockSampler:
    """Shader clock and board power WHILE the timed steps run: a host thread reads the driver's sysfs files
    (pp_dpm_sclk: the level marked '*' is the current clock; hwmon power1_input, microwatts) every couple of
    milliseconds between start() and stop().  The roofline peak is quoted at 2.4 GHz; this says what clock the
    chip actually held under the load.  Returns None where the files are not readable."""

    def __init__(self):
        import glob
        self.sclk = next(iter(sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))), None)
        self.power = next(iter(sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))), None)
        self.samples, self._stop, self._thread = [], False, None

    def _read(self):
        mhz = watts = None
        try:
            with open(self.sclk) as f:
                for line in f:
                    if "*" in line:
                        mhz = float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
            with open(self.power) as f:
                watts = float(f.read()) / 1e6
        except Exception:
            pass
        return mhz, watts

    def _run(self):
        while not self._stop:
            self.samples.append(self._read())
            time.sleep(0.002)

    def start(self):
        if self.sclk is None or self.power is None:
            return
        import threading
        self._thread = threading.Thread(target=self._run, daemon=True)
        self._thread.start()

    def stop(self):
        if self._thread is None:
            return None
        self._stop = True
        self._thread.join()
        mhz = sorted(m for m, _ in self.samples if m is not None)
        w = sorted(p for _, p in self.samples if p is not None)
        if not mhz or not w:
            return None
        mid = lambda v: v[len(v) // 2]
        return {"samples": len(self.samples), "sclk_mhz_median": mid(mhz), "sclk_mhz_min": mhz[0], "sclk_mhz_max": mhz[-1],
                "power_w_median": round(mid(w), 1), "power_w_max": round(w[-1], 1),
                "source": "sysfs pp_dpm_sclk / hwmon power1_input polled by a host thread during the timed steps"}


def phase_stamps(kt, step, d, n, recompute):
    """One step with the GEMM kernel's own time stamps (wave 0 of every workgroup: shader-clock counter at entry,
    after the prologue, after the main loop, after the epilogue; the 100 MHz counter at entry and exit)."""
    import ctypes
    import numpy as np
    L = kt.lib()
    if not hasattr(L, "kt_debug_stamps_arm"):
        sys.exit("bench.py --phase-stamps: the library was not built with -DKT_PHASE_STAMPS")
    slots, wgs, words = 8, 16384, 8
    buf = np.zeros(slots * wgs * words, dtype=np.uint64)
    L.kt_debug_stamps_arm()
    step()
    L.kt_debug_stamps_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
    assert L.kt_debug_stamps_read(buf.ctypes.data_as(ctypes.c_void_p), buf.nbytes) == 0
    r_all = buf.reshape(slots, wgs, words).astype(np.int64)
    cay = ["Cayley: M = dR R^T"] + [f"Cayley iteration {i}" for i in range(1, 7)]
    names = (["forward + row moments", "recompute + dL/dY", "dR = X^T G"] if recompute else
             ["forward + row moments + Y kept", "dR = X^T G"]) + cay   # the GEMM launches of a step, in order
    k_of = ([d, d, n] if recompute else [d, n])                          # contraction length of the big ones
    out = []
    for s in range(slots):
        r = r_all[s][r_all[s][:, 3] > 0]
        if not len(r):
            continue
        pro, loop, epi, tot = r[:, 1] - r[:, 0], r[:, 2] - r[:, 1], r[:, 3] - r[:, 2], r[:, 3] - r[:, 0]
        wall_us = (r[:, 5] - r[:, 4]) / 100.0
        span_us = (r[:, 5].max() - r[:, 4].min()) / 100.0
        rec = {"launch": names[s], "workgroups": int(len(r)), "span_us": round(float(span_us), 1),
               "share_prologue": round(float(pro.sum() / tot.sum()), 4), "share_main_loop": round(float(loop.sum() / tot.sum()), 4),
               "share_epilogue": round(float(epi.sum() / tot.sum()), 4),
               "cycles_per_workgroup_median": {"prologue": int(np.median(pro)), "main_loop": int(np.median(loop)), "epilogue": int(np.median(epi))},
               "shader_clock_mhz_median": round(float(np.median(tot / np.maximum(wall_us, 1e-9))), 0),
               "cu_occupancy_of_span": round(float(wall_us.sum() / (span_us * 256)), 4)}
        if s < len(k_of):  # K slabs x 64 matrix instructions per wave x 32 cycles each, back to back
            k = k_of[s]
            rec["main_loop_efficiency"] = round(float((k / 64) * 64 * 32 / np.median(loop)), 4)
        out.append(rec)
    print(json.dumps({"phase_stamps": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C3", help="workload: C1..C5 (default C3: d=4096, n=131072)")
    ap.add_argument("--n", type=int, default=None, help="override the token count (debugging)")
    ap.add_argument("--batch", type=int, default=None, help="override the problem count (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cayley", action="store_true", help="time loss+grad only")
    ap.add_argument("--op", choices=["step", "fakequant", "quant-metrics", "hadamard", "sensitivity"], default="step",
                    help="what a 'step' is: the training step (default, the headline metric) or one call of "
                         "kt_rotate_quant_metrics (evaluation-side figures) on the same activations")
    ap.add_argument("--hadamard-d", type=int, default=None,
                    help="--op hadamard: row length m 2^k to use instead of the config's d (same number of bytes)")
    ap.add_argument("--loss", choices=["row", "pooled"], default="row",
                    help="per-token-row kurtosis (default, the headline step) or the paper-literal pooled loss "
                         "with RMSNorm (kappa_target 1.8)")
    ap.add_argument("--optimizer", choices=["sgd", "adam"], default="sgd",
                    help="retraction timed inside the step: Cayley SGD (default, the headline step) or Cayley Adam")
    ap.add_argument("--recompute", action="store_true",
                    help="hand kt_kurtosis_loss_grad only its smaller workspace: Y is then recomputed by a second GEMM in "
                         "the backward pass instead of being kept in fp32 by the forward pass (same result)")
    ap.add_argument("--phase-stamps", action="store_true",
                    help="developer builds only (KT_HIPCC_EXTRA=-DKT_PHASE_STAMPS python -m paper_2503_01483_amd.build): "
                         "after the warm-up run ONE step with the in-kernel time stamps armed and print, per GEMM "
                         "launch, the share of prologue / main loop / epilogue and the shader clock the stamps imply")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="after timing, copy X once with a plain device copy (a kernel of known traffic, "
                         "2 x bytes(X), against which rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (token rows would shard over "
              "GPUs with one all-reduce of dR per step)", file=sys.stderr)
        sys.exit(2)

    import torch
    import ktgen
    import paper_2503_01483_amd as kt

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda"
    t0 = time.time()
    X, R, cfg = ktgen.make_problem(args.config, seed=0, device=dev, n=args.n, batch=args.batch)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    batch, n, d = X.shape
    lr = cfg["lr"]
    bf16 = cfg["dtype"] == "bf16"

    ws = kt.Workspace(dev)
    pooled = args.loss == "pooled"
    ws.get(max(kt.kt_workspace_bytes(kt.KT_OP_POOLED_LOSS_GRAD if pooled else kt.KT_OP_LOSS_GRAD, batch, n, d,
                                     kt.KT_BF16 if bf16 else kt.KT_F32),
               kt.kt_workspace_bytes(kt.KT_OP_CAYLEY, batch, 0, d, kt.KT_F32)))
    loss = torch.zeros(batch, device=dev)
    dR = torch.empty((batch, d, d), device=dev)
    info = torch.zeros(batch, dtype=torch.int32, device=dev)
    Rw = R.clone()
    adam = args.optimizer == "adam"
    Mom = torch.zeros_like(dR) if adam else None
    vmom = torch.ones(batch, device=dev) if adam else None
    counter = [0]

    def step():
        if pooled:
            kt.kt_pooled_kurtosis_loss_grad(X, Rw, loss=loss, dR=dR, workspace=ws, recompute=args.recompute)
        else:
            kt.kt_kurtosis_loss_grad(X, Rw, loss=loss, dR=dR, workspace=ws, recompute=args.recompute)
        if args.no_cayley:
            return
        if adam:
            counter[0] += 1
            kt.kt_cayley_adam_step(Rw, dR, Mom, vmom, counter[0], lr, info=info, workspace=ws)
        else:
            kt.kt_cayley_step(Rw, dR, lr, info=info, workspace=ws)

    if args.op == "quant-metrics":
        ws.get(kt.kt_workspace_bytes(kt.KT_OP_QUANT_METRICS, batch, n, d, kt.KT_BF16 if bf16 else kt.KT_F32))
        q_amax = torch.empty((batch, n, 2), device=dev)
        q_es = torch.empty((batch, n, 2), device=dev)
        q_ea = torch.empty((batch, n, 2), device=dev)
        q_succ = torch.zeros(batch, dtype=torch.int64, device=dev)

        def step():  # noqa: F811
            kt.kt_rotate_quant_metrics(X, Rw, quantile=0.98, amax=q_amax, err_sym=q_es, err_asym=q_ea,
                                       success=q_succ, workspace=ws)

    if args.op == "fakequant":
        ws.get(kt.kt_workspace_bytes(kt.KT_OP_FAKEQUANT, batch, n, d, kt.KT_BF16 if bf16 else kt.KT_F32))
        fq_codes = torch.empty((batch, n, d), dtype=torch.int8, device=dev)
        fq_scales = torch.empty((batch, n), device=dev)
        fq_err = torch.empty((batch, n, 2), device=dev)

        def step():  # noqa: F811
            kt.kt_rotate_fakequant_int4(X, Rw, clip_ratio=1.0, scales_out=fq_scales, codes=fq_codes, err=fq_err,
                                        workspace=ws)

    if args.op == "sensitivity":
        ws.get(kt.kt_workspace_bytes(kt.KT_OP_QUANT_METRICS, 1, n, d, kt.KT_BF16 if bf16 else kt.KT_F32))
        Ys = torch.empty((1, n, d), device=dev)
        kt.kt_rotate_quant_metrics(X[0:1], Rw[0:1], quantile=1.0, Y=Ys, workspace=ws)
        s_alphas = torch.tensor([0.05, 0.1, 0.2], device=dev)
        s_out = [None, None]

        def step():  # noqa: F811
            s_out[0], s_out[1] = kt.kt_quant_sensitivity(Ys, s_alphas, bits=4, workspace=ws)

    if args.op == "hadamard":
        h_d = args.hadamard_d or d
        h_rows = batch * n * d // h_d
        Xh = X.reshape(-1)[:h_rows * h_d].reshape(h_rows, h_d)
        Yh = torch.empty_like(Xh)

        def step():  # noqa: F811
            kt.kt_hadamard_rows(Xh, out=Yh)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.phase_stamps:
        phase_stamps(kt, step, d, n, args.recompute)
        return
    loss_first = loss.clone()
    kt.kt_profile_enable(8 * args.steps + 8)
    kt.kt_profile_reset()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    sampler = ClockSampler()
    sampler.start()
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        step()
    marks[args.steps].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    state = sampler.stop()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    prof = {k: kt.kt_profile_read(k) for k in range(6)}
    kt.kt_profile_enable(0)
    if args.op == "sensitivity":
        ms = 1e3 * elapsed / args.steps
        evals = float(n) * d * (3 * 32 + 4)      # three sweeps of 32 candidate steps, one of 1 + 3 fractions
        lane_ops = evals * 5                     # per candidate: mul, rint, clamp (med3), fma, fma
        # 256 CUs x 4 SIMDs x 32 fp32 lanes x 2.4 GHz, one operation per lane and cycle (the published 157.3 TFLOP/s
        # counts a fused multiply-add as two; measured: a wave64 instruction every 2.4-2.6 cycles per SIMD)
        peak = 256 * 4 * 32 * 2.4e9 / 1e12
        print(json.dumps({
            "metric": "elements/sec through kt_quant_sensitivity (optimal int4 step + sensitivity of one tensor)",
            "value": round(float(n) * d * args.steps / elapsed, 1), "unit": "elements/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"{args.config}: Y = X R of problem 0, {n * d} fp32 entries, 3 fractions"},
            "roofline": {"bound": "alu", "kernel": "sens_sweep_kernel (4 launches per call)",
                         "achieved": round(lane_ops / (ms * 1e-3) / 1e12, 2), "peak": round(peak, 1), "unit": "Tlane-op/s",
                         "frac": round(lane_ops / (ms * 1e-3) / 1e12 / peak, 4), "traffic": None},
            "s_opt": float(s_out[0][0]), "mse_opt": float(s_out[0][1]), "gamma": s_out[1].cpu().tolist(),
            "cpu_baseline": None}))
        return
    if args.op == "fakequant":
        ms = 1e3 * elapsed / args.steps
        flops_call = 2.0 * batch * n * d * d      # one GEMM pass: Y staged in fp32, then one row kernel
        fq_bytes = float(batch) * n * (d * 3 + 12)  # d = 128: x read once (bf16), codes, scale and error pair written
        peak_call = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
        print(json.dumps({
            "metric": "tokens/sec through kt_rotate_fakequant_int4 (rotate + per-token symmetric int4 codes, scales, error)",
            "value": round(batch * n * args.steps / elapsed, 1), "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
            "config": {"workload": f"{args.config}: n={n} tokens x d={d}, batch={batch}, clip 1.0, codes + scales + error"},
            "roofline": ({"bound": "hbm", "kernel": "quant_d128_kernel (single pass: rotate, row maximum, codes, error)",
                          "achieved": round(fq_bytes / (ms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                          "frac": round(fq_bytes / (ms * 1e-3) / 1e9 / 8000.0, 4), "bytes_per_launch": fq_bytes,
                          "traffic": None} if (bf16 and d == 128) else
                         {"bound": "mfma", "kernel": "whole call (gemm_nt_kernel<EpiStore> into the fp32 staging buffer + quant_rows_kernel)",
                          "achieved": round(flops_call / (ms * 1e-3) / 1e12, 1), "peak": peak_call, "unit": "TFLOP/s",
                          "frac": round(flops_call / (ms * 1e-3) / 1e12 / peak_call, 4), "flops_per_launch": flops_call,
                          "traffic": None}),
            "rel_err_int4": float(fq_err[0, :, 0].double().sum() / fq_err[0, :, 1].double().sum()),
            "cpu_baseline": None}))
        return
    if args.op == "hadamard":
        ms = 1e3 * elapsed / args.steps
        nbytes = 2.0 * h_rows * h_d * (2 if bf16 else 4)     # rows read once, written once (algorithmic)
        print(json.dumps({
            "metric": "tokens/sec through kt_hadamard_rows (online Hadamard rotation of token rows)",
            "value": round(h_rows * args.steps / elapsed, 1), "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
            "config": {"workload": f"{args.config}: {h_rows} token rows x d={h_d}"},
            "roofline": {"bound": "hbm", "kernel": "hadamard_rows_kernel" + (" + hadamard_cross_kernel" if (h_d & (h_d - 1)) or h_d > 4096 else ""), "achieved": round(nbytes / (ms * 1e-3) / 1e9, 1),
                         "peak": 8000.0, "unit": "GB/s", "frac": round(nbytes / (ms * 1e-3) / 1e9 / 8000.0, 4),
                         "bytes_per_launch": nbytes, "traffic": None},
            "cpu_baseline": None}))
        return
    if args.op == "quant-metrics":
        ms = 1e3 * elapsed / args.steps
        esz = 2 if bf16 else 4
        alg_bytes = batch * n * d * esz                 # the activations once: what the figures need
        hw_bytes = batch * n * d * (2 * esz + 8)        # X twice (GEMM, baseline max), Y written and read (fp32)
        flops_call = 2.0 * batch * n * d * d
        peak_call = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
        print(json.dumps({
            "metric": "tokens/sec through kt_rotate_quant_metrics (rotation GEMM + per-token row kernel)",
            "value": round(batch * n * args.steps / elapsed, 1), "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
            "config": {"workload": f"{args.config}: n={n} tokens x d={d}, batch={batch}, quantile 0.98"},
            # d >= 2048: the rotation GEMM (2 n d^2 flop) bounds the call; below, the row kernel's HBM traffic
            "roofline": ({"bound": "mfma", "kernel": "whole call (gemm_nt_kernel<EpiStore> + quant_metrics_row_kernel)",
                          "achieved": round(flops_call / (ms * 1e-3) / 1e12, 1), "peak": peak_call, "unit": "TFLOP/s",
                          "frac": round(flops_call / (ms * 1e-3) / 1e12 / peak_call, 4), "flops_per_launch": flops_call,
                          "traffic": None} if d >= 2048 else
                         {"bound": "hbm", "kernel": "whole call (gemm_nt_kernel<EpiStore> + quant_metrics_row_kernel)",
                          "achieved": round(alg_bytes / (ms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                          "frac": round(alg_bytes / (ms * 1e-3) / 1e9 / 8000.0, 4), "bytes_per_launch": alg_bytes,
                          "hardware_bytes": hw_bytes, "traffic": None}),
            "success_rate": [float(x) / n for x in q_succ.cpu().tolist()[:4]],
            "rel_err_sym_int4_q98": float(q_es[0, :, 0].double().sum() / q_es[0, :, 1].double().sum()),
            "rel_err_asym_int4": float(q_ea[0, :, 0].double().sum() / q_ea[0, :, 1].double().sum()),
            "cpu_baseline": None}))
        return

    if args.pmc_calibration:
        Xc = torch.empty_like(X)
        Xc.copy_(X)
        torch.cuda.synchronize()
        del Xc

    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = batch * n * args.steps / elapsed
    flops_launch = 2.0 * batch * n * d * d           # one GEMM launch: 2 n d^2 per problem
    peak = PEAK_BF16_TFLOPS if bf16 else PEAK_F32_TFLOPS
    kern = {}
    for k in (0, 1, 2):
        tot, cnt = prof[k]
        if cnt:
            kern[k] = {"avg_ms": tot / cnt, "launches": cnt, "tflops": flops_launch / (tot / cnt * 1e-3) / 1e12}
    fused = bf16 and d == 128 and not pooled   # single-pass kernel: reads X once, bound by HBM rather than by the matrix pipe
    # Y kept (the default while 4 n d bytes fit the library's limit) or recomputed: which launches are GEMMs
    keep = not fused and not args.recompute and kt.kt_workspace_bytes(
        kt.KT_OP_POOLED_LOSS_GRAD if pooled else kt.KT_OP_LOSS_GRAD, batch, n, d, kt.KT_BF16 if bf16 else kt.KT_F32) > \
        kt.kt_workspace_bytes(kt.KT_OP_POOLED_LOSS_GRAD_RECOMPUTE if pooled else kt.KT_OP_LOSS_GRAD_RECOMPUTE, batch, n, d,
                              kt.KT_BF16 if bf16 else kt.KT_F32)
    gemms = [k for k in kern if not (keep and k == 1)]
    dom = max(gemms, key=lambda k: kern[k]["avg_ms"])
    hw_mult = 4.0 if keep else 6.0   # GEMM flop the step executes, in units of n d^2
    if fused:
        x_bytes = 2.0 * batch * n * d
        gbs = x_bytes / (kern[0]["avg_ms"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "fused_d128_kernel (rotate + moments + dL/dY + X^T G in one pass over X)",
                    "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s", "frac": round(gbs / 8000.0, 4),
                    "avg_launch_ms": round(kern[0]["avg_ms"], 4), "bytes_per_launch": x_bytes,
                    "mfma_tflops_4nd2": round(2 * flops_launch / (kern[0]["avg_ms"] * 1e-3) / 1e12, 1), "traffic": None}
    else:
        roofline = {"bound": "mfma", "kernel": ((KERNEL_NAMES_KEEP if keep else KERNEL_NAMES)[dom]) if bf16 else "gemm_nt_kernel<f32 128x128>",
                    "achieved": round(kern[dom]["tflops"], 2), "peak": peak, "unit": "TFLOP/s",
                    "frac": round(kern[dom]["tflops"] / peak, 4), "avg_launch_ms": round(kern[dom]["avg_ms"], 4),
                    "flops_per_launch": flops_launch,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(args.config, {}).get("keep" if keep else "recompute", {}).get(dom)
                    if args.n is None and not pooled else None,
                    "traffic_source": "carried from profiles/c3_gemm_counters.md (rocprofv3 --pmc runs of this command); "
                                      "not measured in this run"}
    names = {0: "fused_pass_ms" if fused else ("fwd_moments_keep_y_ms" if keep else "fwd_moments_ms"),
             1: "grad_from_kept_y_ms" if keep else "bwd_recompute_ms", 2: "grad_xtg_ms"}
    breakdown = {names[k]: round(kern[k]["avg_ms"], 4) for k in kern}
    if keep and 1 in kern:  # the entry-by-entry kernel: reads Y (fp32), writes dL/dY in the GEMM dtype
        gy_bytes = batch * n * d * (4.0 + (2.0 if bf16 else 4.0))
        breakdown["grad_from_kept_y_gbs"] = round(gy_bytes / (kern[1]["avg_ms"] * 1e-3) / 1e9, 1)
    if prof[3][1]:
        breakdown["x_transpose_ms"] = round(prof[3][0] / prof[3][1], 4)
    breakdown["cayley_ms"] = round(prof[4][0] / max(prof[4][1], 1), 4)
    iters = info.cpu().tolist()
    breakdown["cayley_iters_last"] = iters[:4]
    # a retraction that did not converge is rejected by the library (R unchanged): such a run did not do the step
    cayley_ok = args.no_cayley or all(i > 0 for i in iters)
    alg_tflops = 4.0 * batch * n * d * d * args.steps / elapsed / 1e12
    hw_tflops = hw_mult * batch * n * d * d * args.steps / elapsed / 1e12

    # The form of the step in which Y never reaches HBM (recomputed by a second GEMM in the backward pass; the
    # library takes it when handed its smaller workspace), timed beside the default on the same box and state of R.
    recomputed = None
    loss_last = float(loss[0])
    if keep and args.op == "step":
        def step_recompute():
            if pooled:
                kt.kt_pooled_kurtosis_loss_grad(X, Rw, loss=loss, dR=dR, workspace=ws, recompute=True)
            else:
                kt.kt_kurtosis_loss_grad(X, Rw, loss=loss, dR=dR, workspace=ws, recompute=True)
            if args.no_cayley:
                return
            if adam:
                counter[0] += 1
                kt.kt_cayley_adam_step(Rw, dR, Mom, vmom, counter[0], lr, info=info, workspace=ws)
            else:
                kt.kt_cayley_step(Rw, dR, lr, info=info, workspace=ws)
        for _ in range(min(args.warmup, 2)):
            step_recompute()
        torch.cuda.synchronize()
        tr = time.perf_counter()
        for _ in range(args.steps):
            step_recompute()
        torch.cuda.synchronize()
        el = time.perf_counter() - tr
        recomputed = {"what": "same step with Y recomputed by a second GEMM instead of kept in fp32 scratch "
                              "(bit-identical loss and gradient); bench.py --recompute times this form alone",
                      "ms_per_step": round(1e3 * el / args.steps, 4), "value": round(batch * n * args.steps / el, 1),
                      "unit": "tokens/s",
                      "frac_of_bf16_peak_algorithmic_4nd2": round(4.0 * batch * n * d * d * args.steps / el / 1e12 / peak, 4),
                      "frac_of_bf16_peak_hardware_6nd2": round(6.0 * batch * n * d * d * args.steps / el / 1e12 / peak, 4)}

    cpu = None
    if not args.no_cpu_baseline and not pooled:
        import numpy as np
        import oracle
        rows = min(n, CPU_SAMPLE_ROWS[args.config])
        Xs = ktgen.to_f64(X[0, :rows])
        Rs = ktgen.to_f64(ktgen.bf16_round(R[0]) if bf16 else R[0])
        t0 = time.perf_counter()
        o = oracle.loss_grad(Xs, Rs)
        cpu_s = time.perf_counter() - t0
        # the oracle's Cayley step (fp64 LU) on its own gradient: at the config's d up to 2048, above that timed at
        # d = 2048 on the leading block of R and dR and scaled by (d/2048)^3 (every part of it is cubic in d)
        dc = min(d, 2048)
        Rc = np.ascontiguousarray(ktgen.to_f64(R[0])[:dc, :dc])
        Gc = np.ascontiguousarray(o["dR"][:dc, :dc])
        t0 = time.perf_counter()
        oracle.cayley_step(Rc, Gc, lr)
        cay_meas = time.perf_counter() - t0
        cay_s = cay_meas * (d / dc) ** 3
        lg_rate = rows / cpu_s
        step_rate = n / (n / lg_rate + (0.0 if args.no_cayley else cay_s))
        cpu = {"value": round(step_rate, 2), "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"plain fp64 oracle, one problem of the same workload: loss+grad on the first {rows} token rows "
                         f"at d={d} ({cpu_s:.1f} s, {lg_rate:.1f} tokens/s, linear in rows) + its Cayley step (LU) "
                         + (f"timed at d={dc} ({cay_meas:.1f} s) and scaled by (d/{dc})^3 to {cay_s:.1f} s"
                            if dc != d else f"at d={d} ({cay_s:.2f} s)")
                         + f"; value = n / (n / loss+grad rate + Cayley time) for n={n}; not a tuned CPU baseline",
               "loss_grad_tokens_per_s": round(lg_rate, 2), "cayley_step_s": round(cay_s, 2)}
        # while the oracle result is here: the same rows through the GPU path must agree
        l2 = torch.zeros(1, device=dev)
        d2 = torch.empty((1, d, d), device=dev)
        kt.kt_kurtosis_loss_grad(X[0:1, :rows], R[0:1], loss=l2, dR=d2, workspace=ws)
        torch.cuda.synchronize()
        rel = float(np.linalg.norm(d2[0].cpu().numpy() - o["dR"]) / np.linalg.norm(o["dR"]))
        cpu["gpu_vs_oracle_on_sample"] = {"loss_rel": abs(l2.item() - o["loss"]) / o["loss"], "dR_rel": rel}

    out = {
        "metric": "calibration tokens/sec through kurtosis loss+grad step; % of bf16 MFMA peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(per_step[len(per_step) // 2], 4), "ms_per_step_min": round(per_step[0], 4),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.config}: n={n} tokens x d={d}, batch={batch}, "
                               f"{'pooled ' if pooled else ''}loss+grad{'' if args.no_cayley else ('+Cayley Adam' if adam else '+Cayley')} step, lr={lr}",
                   "global_batch": batch * n, "hidden": d},
        "tflops_algorithmic_4nd2": round(alg_tflops, 2),
        "tflops_hardware": None if fused else round(hw_tflops, 2),
        "hardware_flop_count": None if fused else ("4 n d^2: Y kept in fp32 scratch by the forward GEMM" if keep else
                                                   "6 n d^2: Y recomputed by a second GEMM in the backward pass"),
        "frac_of_bf16_peak_algorithmic": round(alg_tflops / peak, 4),
        "frac_of_bf16_peak_hardware": None if fused else round(hw_tflops / peak, 4),
        # the stated goal is the WHOLE step at >= 50 % of the matrix peak; roofline.frac below is one launch
        "step_target": {"frac_goal": 0.5, "met_algorithmic_4nd2": bool(alg_tflops / peak >= 0.5),
                        "met_hardware_count": None if fused else bool(hw_tflops / peak >= 0.5)},
        "roofline": roofline, "kernels_ms": breakdown, "y_never_in_hbm_form": recomputed, "cpu_baseline": cpu,
        "loss_first_last": [float(loss_first[0]), loss_last], "input_gen_s": round(gen_s, 1),
        "gpu_state_during_timed_region": state,
        "context": "paper: SpinQuant needs >= 4x H100 80GB for Llama3-70B rotations, KurTail a single GPU",
    }
    if not cayley_ok:
        out["value"] = None
        out["invalid"] = f"the Cayley fixed point did not converge (info = {iters[:4]}): the steps timed did not update R"
    print(json.dumps(out))
    if not cayley_ok:
        sys.exit(3)


if __name__ == "__main__":
    main()
