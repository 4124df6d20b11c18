#!/usr/bin/env python3
"""Benchmark of the MXFP8 linear-layer hot path on one MI355X.

One step = the whole path for one 8B-class MLP up-projection layer (T = 8192 tokens,
H = 4096 -> O = 14336), forward and backward, on seeded synthetic tensors resident in HBM:

    quantize X  [T x H] BF16, both axes      quantize W [O x H] BF16, both axes
    fprop  Y  = X_row  . W_row^T   (BF16 out)
    quantize dY [T x O] FP32, both axes
    dgrad  dX = dY_row . W_colT^T  (BF16 out)
    wgrad  dW = dY_colT . X_colT^T (FP32 out)
    dequantize X_row -> BF16

Prints ONE JSON line. `value` is the GEMM work of a step (3 x 2*T*H*O flop) divided by the whole
step time, quantize and dequantize passes included. `roofline` describes the GEMM (fprop launch),
`roofline_quantize` the quantizer (X, both axes), both timed live with events on the launch
stream inside the timed region. `cpu_baseline` times the CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

T, H, O = 8192, 4096, 14336
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_FP8_PEAK_TFLOPS = 5000.0  # dense FP8 / MX-FP8 matrix peak
MFMA_SUSTAINED_TFLOPS = 4970.0  # what a register-only loop of the scaled MFMA instruction reached on an MI355X


def _ensure_built():
    from paper_2506_08027_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_08027_amd.build import build_library
        build_library()


def cpu_baseline():
    """The oracle as it stands on the host cores, on a bounded sample of the same workload."""
    import oracle
    from paper_2506_08027_amd import synth_inputs as si
    rows_q, rows_g, cols_g = 4096, 4096, 4096   # about 20 s of oracle time on 8 to 16 cores
    x = si.activations(rows_q, H, seed=2)
    w = si.weights(cols_g, H, seed=4)
    t0 = time.perf_counter()
    xq, xs = oracle.quantize_rowwise(x)
    oracle.quantize_colwise(x)
    tq = time.perf_counter() - t0
    wq, ws = oracle.quantize_rowwise(w)              # operands for the GEMM sample
    t0 = time.perf_counter()
    oracle.gemm_rows(xq, xs, wq, ws, np.arange(rows_g))
    tg = time.perf_counter() - t0
    gemm_flops = 2.0 * rows_g * cols_g * H
    quant_bytes = rows_q * H * 4.0625
    return {
        "value": gemm_flops / tg / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(), "kind": "oracle",
        "sample": f"GEMM: {rows_g} output rows x {cols_g} columns at K={H} of the fprop product "
                  f"({tg:.2f} s, decode of the operands included); quantize: X[{rows_q}x{H}] BF16 both axes "
                  f"({tq:.2f} s = {quant_bytes / tq / 1e9:.4f} GB/s)",
        "quantize_gbs": quant_bytes / tq / 1e9,
    }


def traffic_from_profile(row_prefix):
    """HBM-side bytes per launch (fetched + written) measured with rocprofv3 PMC counters and kept in
    profiles/hbm_traffic_pmc.txt (the counters cannot be read from inside this process)."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")) as f:
            for line in f:
                if line.startswith(row_prefix):
                    cells = [c.strip() for c in line.split("|")]
                    return (float(cells[1]) + float(cells[2])) * 1e6
    except (OSError, ValueError, IndexError):
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--opt-in", action="store_true",
                    help="also time the opt-in paths (tiled scale layout, persistent GEMM kernel) after the step "
                         "loop and report them as `opt_in_paths`; the headline numbers are not affected")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known HBM traffic, used to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (there is no CPU fallback of the product path)")
    _ensure_built()
    import paper_2506_08027_amd as mx
    from paper_2506_08027_amd import synth_inputs as si

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    bf = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    X = bf(si.activations(T, H, seed=2))
    W = bf(si.weights(O, H, seed=4))
    dY = torch.from_numpy(si.gradients(T, O, seed=5, spikes=True)).to(dev)
    u8 = dict(dtype=torch.uint8, device=dev)

    def qbufs(r, c):
        return dict(q_row=torch.empty((r, c), **u8), s_row=torch.empty((r, c // 32), **u8),
                    q_colT=torch.empty((c, r), **u8), s_colT=torch.empty((c, r // 32), **u8))
    Xq, Wq, dYq = qbufs(T, H), qbufs(O, H), qbufs(T, O)
    Y = torch.empty((T, O), dtype=torch.bfloat16, device=dev)
    dX = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    dW = torch.empty((O, H), dtype=torch.float32, device=dev)
    Xd = torch.empty((T, H), dtype=torch.bfloat16, device=dev)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    gemm_ev, quant_ev = [], []

    def step(timed):
        e = (ev(), ev(), ev(), ev()) if timed else None
        if timed:
            e[0].record()
        mx.mxfp8_quantize(X, mx.BOTH, **Xq)
        if timed:
            e[1].record()
        mx.mxfp8_quantize(W, mx.BOTH, **Wq)
        if timed:
            e[2].record()
        mx.mxfp8_gemm(mx.FPROP, Xq["q_row"], Xq["s_row"], Wq["q_row"], Wq["s_row"], Y)
        if timed:
            e[3].record()
            quant_ev.append((e[0], e[1]))
            gemm_ev.append((e[2], e[3]))
        mx.mxfp8_quantize(dY, mx.BOTH, **dYq)
        mx.mxfp8_gemm(mx.DGRAD, dYq["q_row"], dYq["s_row"], Wq["q_colT"], Wq["s_colT"], dX)
        mx.mxfp8_gemm(mx.WGRAD, dYq["q_colT"], dYq["s_colT"], Xq["q_colT"], Xq["s_colT"], dW)
        mx.mxfp8_dequantize(Xq["q_row"], Xq["s_row"], Xd)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    def timed_ms(fn, reps=10):
        for _ in range(3):
            fn()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def tiled_scale_variants():
        """The opt-in paths (tiled scale layout, persistent GEMM kernel), timed outside the step and
        reported next to the headline numbers, which stay on the default entry points."""
        lay = mx.SCALES_TILED

        def tbufs(r, c):
            return dict(q_row=torch.empty((r, c), **u8), s_row=torch.empty(mx.mxfp8_scale_bytes(r, c, lay), **u8),
                        q_colT=torch.empty((c, r), **u8), s_colT=torch.empty(mx.mxfp8_scale_bytes(c, r, lay), **u8))
        Xt, Wt, dYt = tbufs(T, H), tbufs(O, H), tbufs(T, O)
        q_x = timed_ms(lambda: mx.mxfp8_quantize_ex(X, mx.BOTH, **Xt, scale_layout=lay))
        mx.mxfp8_quantize_ex(W, mx.BOTH, **Wt, scale_layout=lay)
        q_dy = timed_ms(lambda: mx.mxfp8_quantize_ex(dY, mx.BOTH, **dYt, scale_layout=lay))
        # the three products of the layer: default kernel / tiled scales / persistent kernel on either layout
        calls = {
            "fprop": (lambda q, lay_: (mx.FPROP, q[0]["q_row"], q[0]["s_row"], q[1]["q_row"], q[1]["s_row"], Y, lay_),
                      (Xq, Wq), (Xt, Wt)),
            "dgrad": (lambda q, lay_: (mx.DGRAD, q[0]["q_row"], q[0]["s_row"], q[1]["q_colT"], q[1]["s_colT"], dX, lay_),
                      (dYq, Wq), (dYt, Wt)),
            "wgrad": (lambda q, lay_: (mx.WGRAD, q[0]["q_colT"], q[0]["s_colT"], q[1]["q_colT"], q[1]["s_colT"], dW, lay_),
                      (dYq, Xq), (dYt, Xt)),
        }
        tf = lambda ms: 2.0 * T * H * O / (ms * 1e-3) / 1e12
        out = {"quantize_x_bf16_both_gbs_tiled": T * H * 4.0625 / (q_x * 1e-3) / 1e9, "quantize_x_ms_tiled": q_x,
               "quantize_dy_f32_both_gbs_tiled": T * O * 6.0625 / (q_dy * 1e-3) / 1e9, "quantize_dy_ms_tiled": q_dy}
        for name, (mk, rowmajor, tiled_ops) in calls.items():
            out[name + "_tflops_default"] = tf(timed_ms(lambda: mx.mxfp8_gemm_ex(*mk(rowmajor, mx.SCALES_ROWMAJOR))))
            out[name + "_tflops_tiled"] = tf(timed_ms(lambda: mx.mxfp8_gemm_ex(*mk(tiled_ops, lay))))
            os.environ["MXFP8_GEMM_PERSISTENT"] = "256"
            try:
                out[name + "_tflops_persistent"] = tf(timed_ms(lambda: mx.mxfp8_gemm_ex(*mk(rowmajor, mx.SCALES_ROWMAJOR))))
                out[name + "_tflops_tiled_persistent"] = tf(timed_ms(lambda: mx.mxfp8_gemm_ex(*mk(tiled_ops, lay))))
                for tune in (1, 2, 3, 4, 5, 6):          # schedule variants of the persistent K step
                    os.environ["MXFP8_GEMM_TUNE"] = str(tune)
                    out[f"{name}_tflops_tiled_persistent_tune{tune}"] = tf(timed_ms(
                        lambda: mx.mxfp8_gemm_ex(*mk(tiled_ops, lay))))
            finally:
                os.environ.pop("MXFP8_GEMM_PERSISTENT", None)
                os.environ.pop("MXFP8_GEMM_TUNE", None)
        # forward product that also emits the MXFP8 copies of its BF16 output (the next layer's operands)
        Yt = tbufs(T, O)
        for axis, key in ((mx.ROWWISE, "row"), (mx.BOTH, "both")):
            out[f"fprop_tflops_fused_output_quantize_{key}"] = tf(timed_ms(lambda: mx.mxfp8_gemm_quantize_ex(
                mx.FPROP, Xt["q_row"], Xt["s_row"], Wt["q_row"], Wt["s_row"], Y, axis, Yt["q_row"], Yt["s_row"],
                Yt["q_colT"], Yt["s_colT"], lay)))
        out["quantize_y_bf16_both_ms_tiled"] = timed_ms(lambda: mx.mxfp8_quantize_ex(Y, mx.BOTH, **Yt, scale_layout=lay))
        return out

    tiled = None
    if args.opt_in:
        try:
            tiled = tiled_scale_variants()
        except Exception as exc:  # the headline measurement above must survive a problem in the extra one
            tiled = {"error": repr(exc)}

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = dt / args.steps * 1e3
    step_flops = 3 * 2.0 * T * H * O
    gemm_ms = float(np.mean([a.elapsed_time(b) for a, b in gemm_ev]))
    quant_ms = float(np.mean([a.elapsed_time(b) for a, b in quant_ev]))
    gemm_tflops = 2.0 * T * H * O / (gemm_ms * 1e-3) / 1e12
    quant_bytes = T * H * 4.0625            # 2 B read + 2 x (1 + 1/32) B written per element
    quant_gbs = quant_bytes / (quant_ms * 1e-3) / 1e9

    out = {
        "metric": "MXFP8 GEMM TFLOP/s (% MFMA peak) + quantize GB/s (% HBM), 8B-class, 1 GPU",
        "value": step_flops / (dt / args.steps) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp8-e4m3 x ue8m0, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"8B-class MLP up-projection linear layer, fwd+bwd: T={T} tokens, H={H} -> O={O}; "
                               "quantize X,W (BF16) and dY (FP32) along both axes, fprop+dgrad+wgrad, dequantize X",
                   "T": T, "H": H, "O": O},
        "gemm_tflops_fprop": gemm_tflops, "quantize_gbs_bf16_both": quant_gbs,
        "roofline": {"bound": "mfma", "achieved": gemm_tflops, "peak": MFMA_FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gemm_tflops / MFMA_FP8_PEAK_TFLOPS,
                     "peak_sustained": MFMA_SUSTAINED_TFLOPS, "frac_sustained": gemm_tflops / MFMA_SUSTAINED_TFLOPS,
                     "traffic": traffic_from_profile("fprop 8192x14336x4096"),
                     "kernel": "gemm_kernel (fprop 8192x14336x4096, BF16 out)", "avg_ms": gemm_ms},
        "roofline_quantize": {"bound": "hbm", "achieved": quant_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                              "frac": quant_gbs / HBM_PEAK_GBS, "traffic": traffic_from_profile("quantize X BF16"),
                              "kernel": "quantize_kernel<BF16, row+col> (X 8192x4096)", "avg_ms": quant_ms},
    }
    if tiled is not None:
        out["opt_in_paths"] = tiled
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
