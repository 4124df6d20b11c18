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

through the `_ex` entry points with the tiled scale layout (the layout both kernels are fastest with).

Prints ONE JSON line. `value` is the GEMM work of a step (3 x 2*T*H*O flop) divided by the whole
step time, quantize and dequantize passes included. `roofline` describes the forward GEMM launch and
`roofline_dgrad` / `roofline_wgrad` the two backward products, each timed with events on the launch
stream inside the timed region. `roofline_quantize` (X, BF16, both axes) and `roofline_quantize_f32`
(dY, FP32, both axes) are timed after the step loop over >= 100 launches that rotate over more than
512 MB of distinct sources and destinations, so that the 256 MB memory-side cache cannot serve them.
Two measured ceilings of the box stand beside the published peaks: `peak_sustained` in the GEMM rooflines is
the rate a register-only loop of the matrix instruction sustains in this very run (mxfp8_mfma_rate_probe),
`plain_copy_gbs` in the quantize rooflines is the library's plain copy kernel (mxfp8_copy_rate_probe, one workgroup
per compute unit) on the same tensor under the same rotation, `torch_copy_gbs` torch's copy_ of it.
`fused_output_quantization` times the forward product with the MXFP8 copies of Y emitted from its epilogue
against the product followed by a stand-alone quantize of Y; `simulated_path` times the BF16 product of the
round-tripped operands (Section 3.1) against the BF16 matrix peak; `grouped_moe` times the grouped forward
product of a mixture-of-experts layer (Appendix A.4); `mxfp4_path` times the MXFP4 conversion of X and the forward
product on MXFP4 operands (Table 1) against the 4-bit matrix peak; `mxfp6_path` the MXFP6 conversion, the exact
expansion to E4M3 bytes and the product of the expanded operands.
`layer_set_16384` times the three products of each linear layer of an 8B-class transformer block at
16384 tokens. `cpu_baseline` times the CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import hashlib
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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense BF16 matrix peak
MFMA_FP4_PEAK_TFLOPS = 10100.0  # dense FP4 / FP6 matrix peak


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


def kernel_sources_digest():
    """Identifies the kernel sources a profile was taken with."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2506_08027_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def traffic_from_profile(row_prefix):
    """HBM-side bytes per launch (fetched + written) measured with rocprofv3 PMC counters and kept in
    profiles/hbm_traffic_pmc.txt (the counters cannot be read from inside this process). Only a profile
    taken with the kernel sources of this very tree counts; otherwise the traffic is unknown (None)."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_pmc.txt")) as f:
            lines = f.read().splitlines()
        if not any(l.startswith("# kernel sources:") and kernel_sources_digest() in l for l in lines):
            return None
        for line in lines:
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
    ap.add_argument("--no-extras", action="store_true",
                    help="only the step loop (for profiler runs): no rotating quantize timing, no 16384-token layer set")
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
    lay = mx.SCALES_TILED
    bf = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    X = bf(si.activations(T, H, seed=2))
    W = bf(si.weights(O, H, seed=4))
    dY = torch.from_numpy(si.gradients(T, O, seed=5, spikes=True)).to(dev)
    u8 = dict(dtype=torch.uint8, device=dev)

    def qbufs(r, c):
        return dict(q_row=torch.empty((r, c), **u8), s_row=torch.empty(mx.mxfp8_scale_bytes(r, c, lay), **u8),
                    q_colT=torch.empty((c, r), **u8), s_colT=torch.empty(mx.mxfp8_scale_bytes(c, r, lay), **u8))
    Xq, Wq, dYq = qbufs(T, H), qbufs(O, H), qbufs(T, O)
    Y = torch.empty((T, O), dtype=torch.bfloat16, device=dev)
    dX = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    dW = torch.empty((O, H), dtype=torch.float32, device=dev)
    Xd = torch.empty((T, H), dtype=torch.bfloat16, device=dev)

    ev = lambda: torch.cuda.Event(enable_timing=True)   # recorded on torch's current stream, where the launches go
    marks = {"fprop": [], "dgrad": [], "wgrad": []}

    def timed(name, on, fn):
        if not on:
            return fn()
        a, b = ev(), ev()
        a.record()
        fn()
        b.record()
        marks[name].append((a, b))

    def step(on):
        mx.mxfp8_quantize_ex(X, mx.BOTH, **Xq, scale_layout=lay)
        mx.mxfp8_quantize_ex(W, mx.BOTH, **Wq, scale_layout=lay)
        timed("fprop", on, lambda: mx.mxfp8_gemm_ex(mx.FPROP, Xq["q_row"], Xq["s_row"], Wq["q_row"], Wq["s_row"], Y, lay))
        mx.mxfp8_quantize_ex(dY, mx.BOTH, **dYq, scale_layout=lay)
        timed("dgrad", on, lambda: mx.mxfp8_gemm_ex(mx.DGRAD, dYq["q_row"], dYq["s_row"], Wq["q_colT"], Wq["s_colT"], dX, lay))
        timed("wgrad", on, lambda: mx.mxfp8_gemm_ex(mx.WGRAD, dYq["q_colT"], dYq["s_colT"], Xq["q_colT"], Xq["s_colT"], dW, lay))
        mx.mxfp8_dequantize_ex(Xq["q_row"], Xq["s_row"], Xd, lay)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    def rotating_quantize(src, sets, launches):
        """Average time of one both-axes quantize launch over `launches` launches that walk through `sets`
        distinct source tensors and as many distinct output sets (bracketed by one pair of events)."""
        r, c = src.shape
        srcs = [src] + [src.clone() for _ in range(sets - 1)]
        outs = [qbufs(r, c) for _ in range(sets)]
        for i in range(min(sets, 4)):
            mx.mxfp8_quantize_ex(srcs[i], mx.BOTH, **outs[i], scale_layout=lay)
        a, b = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for i in range(launches):
            mx.mxfp8_quantize_ex(srcs[i % sets], mx.BOTH, **outs[i % sets], scale_layout=lay)
        b.record()
        torch.cuda.synchronize()
        footprint = sets * (src.numel() * src.element_size() + 2 * r * c)
        return a.elapsed_time(b) / launches, footprint

    def rotating_dequantize(sets, launches):
        """Average time of one decode of X's row copy to BF16 over `launches` launches that walk through `sets`
        distinct quantized tensors and as many outputs (one pair of events around the lot)."""
        qs = [Xq["q_row"]] + [Xq["q_row"].clone() for _ in range(sets - 1)]
        ss = [Xq["s_row"]] + [Xq["s_row"].clone() for _ in range(sets - 1)]
        ds = [torch.empty((T, H), dtype=torch.bfloat16, device=dev) for _ in range(sets)]
        for i in range(min(sets, 4)):
            mx.mxfp8_dequantize_ex(qs[i], ss[i], ds[i], lay)
        a, b = ev(), ev()
        torch.cuda.synchronize()
        a.record()
        for i in range(launches):
            mx.mxfp8_dequantize_ex(qs[i % sets], ss[i % sets], ds[i % sets], lay)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / launches, sets * T * H * 3

    def layer_set():
        """The four linear layers of an 8B-class transformer block at 16384 tokens: every product timed on
        operands quantized on the GPU from tensors drawn on the GPU (torch generator, seed 16384)."""
        T5 = 16384
        g = torch.Generator(device=dev)
        g.manual_seed(16384)
        out, total_flop, total_ms = {}, 0.0, 0.0

        def ms_of(fn, reps=5):
            fn()
            a, b = ev(), ev()
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        for name, h, o in (("qkv", 4096, 6144), ("attn_out", 4096, 4096), ("gate_up", 4096, 28672), ("down", 14336, 4096)):
            x = torch.randn((T5, h), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
            w = (0.02 * torch.randn((o, h), generator=g, device=dev, dtype=torch.float32)).to(torch.bfloat16)
            dy = (1e-3 * torch.randn((T5, o), generator=g, device=dev, dtype=torch.float32)).to(torch.bfloat16)
            xq, wq, dyq = (mx.quantize(t, "both", scale_layout=lay) for t in (x, w, dy))
            del x, w, dy
            y = torch.empty((T5, o), dtype=torch.bfloat16, device=dev)
            dx = torch.empty((T5, h), dtype=torch.bfloat16, device=dev)
            dw = torch.empty((o, h), dtype=torch.float32, device=dev)
            flop = 2.0 * T5 * h * o
            times = {
                "fprop": ms_of(lambda: mx.mxfp8_gemm_ex(mx.FPROP, xq["q_row"], xq["s_row"], wq["q_row"], wq["s_row"], y, lay)),
                "dgrad": ms_of(lambda: mx.mxfp8_gemm_ex(mx.DGRAD, dyq["q_row"], dyq["s_row"], wq["q_colT"], wq["s_colT"], dx, lay)),
                "wgrad": ms_of(lambda: mx.mxfp8_gemm_ex(mx.WGRAD, dyq["q_colT"], dyq["s_colT"], xq["q_colT"], xq["s_colT"], dw, lay)),
            }
            out[name] = {"H": h, "O": o, **{k + "_tflops": flop / (v * 1e-3) / 1e12 for k, v in times.items()}}
            total_flop += 3 * flop
            total_ms += sum(times.values())
            del xq, wq, dyq, y, dx, dw
        out["layer_tflop"] = total_flop / 1e12
        out["layer_gemm_ms"] = total_ms
        out["layer_tflops"] = total_flop / (total_ms * 1e-3) / 1e12
        out["frac_of_peak"] = out["layer_tflops"] / MFMA_FP8_PEAK_TFLOPS
        return out

    def ms_avg(fn, reps=20, warm=3):
        for _ in range(warm):
            fn()
        a, b = ev(), ev()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    def fused_output_quantization():
        """fprop that also emits the MXFP8 copies of Y from its epilogue, against fprop followed by a
        stand-alone quantize of Y (same outputs, one more pass over Y)."""
        Yq = qbufs(T, O)
        args_ = (Xq["q_row"], Xq["s_row"], Wq["q_row"], Wq["s_row"], Y)
        res = {}
        for axis, name in ((mx.ROWWISE, "rowwise"), (mx.BOTH, "both")):
            sel = {k: v for k, v in Yq.items() if axis == mx.BOTH or k.endswith("row")}
            fused = ms_avg(lambda: mx.mxfp8_gemm_quantize_ex(mx.FPROP, *args_, axis, **{"c" + k: v for k, v in sel.items()},
                                                             scale_layout=lay))
            separate = ms_avg(lambda: (mx.mxfp8_gemm_ex(mx.FPROP, *args_, lay),
                                       mx.mxfp8_quantize_ex(Y, axis, **sel, scale_layout=lay)))
            res[name] = {"fused_ms": fused, "gemm_then_quantize_ms": separate}
        return res

    def simulated_path():
        """Section 3.1's simulated MX path for the forward product: the BF16 GEMM of the round-tripped operands
        (bound: BF16 matrix peak), and the round trip itself (quantize + dequantize of X)."""
        a16, b16 = torch.empty_like(X), torch.empty_like(W)
        mx.mxfp8_dequantize_ex(Xq["q_row"], Xq["s_row"], a16, lay)
        mx.mxfp8_dequantize_ex(Wq["q_row"], Wq["s_row"], b16, lay)
        ms = ms_avg(lambda: mx.mxfp8_gemm_bf16(a16, b16, Y))
        rt = ms_avg(lambda: (mx.mxfp8_quantize_ex(X, mx.ROWWISE, q_row=Xq["q_row"], s_row=Xq["s_row"], scale_layout=lay),
                             mx.mxfp8_dequantize_ex(Xq["q_row"], Xq["s_row"], a16, lay)))
        tf = gemm_flop / (ms * 1e-3) / 1e12
        return {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "kernel": f"gemm_persistent_kernel, BF16 operands (fprop {T}x{O}x{H}, BF16 out)",
                "avg_ms": ms, "launches": 20, "round_trip_X_ms": rt,
                "round_trip_X_gbs": T * H * (2 + 1.03125 + 1.03125 + 2) / (rt * 1e-3) / 1e9}

    def grouped_moe():
        """Mixture-of-experts forward product (Appendix A.4): 16384 routed tokens sorted by expert, 8 experts of
        the benchmark's shape (4096 -> 14336), uneven expert loads with one empty expert, group ends on the GPU."""
        T5, E = 16384, 8
        g = torch.Generator(device=dev)
        g.manual_seed(8)
        x = torch.randn((T5, H), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
        xq = mx.quantize(x, "rowwise", scale_layout=lay)
        wq, ws = [], []
        for _ in range(E):
            w = (0.02 * torch.randn((O, H), generator=g, device=dev, dtype=torch.float32)).to(torch.bfloat16)
            q = mx.quantize(w, "rowwise", scale_layout=lay)
            wq.append(q["q_row"]); ws.append(q["s_row"])
            del w, q
        b_q, b_s = torch.stack(wq), torch.cat(ws)
        del wq, ws
        ends = torch.tensor([1536, 4096, 4096, 7808, 9984, 12032, 14976, 16384], dtype=torch.int32, device=dev)
        y = torch.empty((T5, O), dtype=torch.bfloat16, device=dev)
        ms = ms_avg(lambda: mx.mxfp8_gemm_grouped_ex(mx.FPROP, xq["q_row"], xq["s_row"], b_q, b_s, ends, y, lay), reps=10)
        tf = 2.0 * T5 * H * O / (ms * 1e-3) / 1e12
        res = {"bound": "mfma", "achieved": tf, "peak": MFMA_FP8_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_FP8_PEAK_TFLOPS,
               "kernel": f"gemm_persistent_kernel, grouped (fprop, {T5} tokens over {E} experts {H}->{O}, BF16 out)",
               "avg_ms": ms, "launches": 10}
        del b_q, b_s, xq
        # weight gradient of the same layer: dW_e [O x H] for every expert, FP32
        dy = (1e-3 * torch.randn((T5, O), generator=g, device=dev, dtype=torch.float32)).to(torch.bfloat16)
        dyq, xcq = mx.quantize(dy, "colwise", scale_layout=lay), mx.quantize(x, "colwise", scale_layout=lay)
        del dy, x, y
        dw = torch.empty((E, O, H), dtype=torch.float32, device=dev)
        ms_w = ms_avg(lambda: mx.mxfp8_gemm_grouped_ex(mx.WGRAD, dyq["q_colT"], dyq["s_colT"], xcq["q_colT"], xcq["s_colT"], ends,
                                                       dw, lay), reps=10)
        res["wgrad_tflops"] = 2.0 * T5 * H * O / (ms_w * 1e-3) / 1e12
        res["wgrad_ms"] = ms_w
        res["wgrad_kernel"] = "gemm_kernel, reduction axis grouped (one workgroup per expert and tile, FP32 out)"
        return res

    def single_copy():
        """Section 5: the column copy of X derived from its row copy when the backward pass needs it, against
        what it replaces (keeping q_colT of X from the forward pass costs its bytes; making it again from the
        BF16 source costs that pass)."""
        ms = ms_avg(lambda: mx.mxfp8_requantize_colwise_ex(Xq["q_row"], Xq["s_row"], Xq["q_colT"], Xq["s_colT"], lay))
        ms_src = ms_avg(lambda: mx.mxfp8_quantize_ex(X, mx.COLWISE, q_colT=Xq["q_colT"], s_colT=Xq["s_colT"], scale_layout=lay))
        return {"requantize_ms": ms, "requantize_gbs": T * H * 2 * (1 + 1 / 32) / (ms * 1e-3) / 1e9,
                "colwise_quantize_from_bf16_ms": ms_src}

    def mxfp4_path():
        """Table 1's narrower format on the same layer: X and W converted to MXFP4 (row copies; X also timed with both
        copies) and the forward product on the 4-bit form of the scaled matrix instruction (dense peak 10.1 PFLOP/s)."""
        xq = mx.fp4_quantize(X, "both", lay)
        wq = mx.fp4_quantize(W, "rowwise", lay)
        ms = ms_avg(lambda: mx.mxfp8_fp4_gemm_ex(mx.FPROP, xq["q_row"], xq["s_row"], wq["q_row"], wq["s_row"], Y, lay))
        q_ms = ms_avg(lambda: mx.mxfp8_fp4_quantize_ex(X, mx.BOTH, xq["q_row"], xq["s_row"], xq["q_colT"], xq["s_colT"], lay))
        d_ms = ms_avg(lambda: mx.mxfp8_fp4_dequantize_ex(xq["q_row"], xq["s_row"], Xd, lay))
        tf = gemm_flop / (ms * 1e-3) / 1e12
        sustained = sustained_mfma_tflops(4)
        return {"bound": "mfma", "achieved": tf, "peak": MFMA_FP4_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_FP4_PEAK_TFLOPS,
                "peak_sustained": sustained, "frac_sustained": tf / sustained,
                "kernel": f"gemm_persistent_kernel, MXFP4 operands (fprop {T}x{O}x{H}, BF16 out)", "avg_ms": ms, "launches": 20,
                "quantize_X_both_ms": q_ms, "quantize_X_both_gbs": T * H * (2 + 2 * (0.5 + 1 / 32)) / (q_ms * 1e-3) / 1e9,
                "dequantize_X_bf16_ms": d_ms, "dequantize_X_bf16_gbs": T * H * (0.5 + 1 / 32 + 2) / (d_ms * 1e-3) / 1e9}

    def mxfp6_path():
        """Table 1's 6-bit formats on the same layer: X and W converted to MXFP6-E2M3, expanded exactly to E4M3 bytes
        and multiplied by the MXFP8 product kernel; the rate counts expansion of both operands plus the product."""
        xq = mx.fp6_quantize(X, mx.E2M3, "both", lay)
        wq = mx.fp6_quantize(W, mx.E2M3, "rowwise", lay)
        x8, w8 = torch.empty((T, H), dtype=torch.uint8, device=dev), torch.empty((O, H), dtype=torch.uint8, device=dev)
        q_ms = ms_avg(lambda: mx.mxfp8_fp6_quantize_ex(X, mx.BOTH, mx.E2M3, xq["q_row"], xq["s_row"], xq["q_colT"], xq["s_colT"], lay))
        e_ms = ms_avg(lambda: (mx.mxfp8_fp6_expand_ex(xq["q_row"], mx.E2M3, x8), mx.mxfp8_fp6_expand_ex(wq["q_row"], mx.E2M3, w8)))
        g_ms = ms_avg(lambda: mx.mxfp8_gemm_ex(mx.FPROP, x8, xq["s_row"], w8, wq["s_row"], Y, lay))
        d_ms = ms_avg(lambda: mx.mxfp8_fp6_dequantize_ex(xq["q_row"], xq["s_row"], mx.E2M3, Xd, lay))
        tf = gemm_flop / ((e_ms + g_ms) * 1e-3) / 1e12
        return {"bound": "mfma", "achieved": tf, "peak": MFMA_FP8_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_FP8_PEAK_TFLOPS,
                "kernel": f"expand_fp6_kernel x2 + gemm_persistent_kernel (fprop {T}x{O}x{H}, BF16 out, E2M3 operands as E4M3)",
                "expand_ms": e_ms, "gemm_ms": g_ms, "quantize_X_both_ms": q_ms,
                "quantize_X_both_gbs": T * H * (2 + 2 * (0.75 + 1 / 32)) / (q_ms * 1e-3) / 1e9,
                "dequantize_X_bf16_ms": d_ms, "dequantize_X_bf16_gbs": T * H * (0.75 + 1 / 32 + 2) / (d_ms * 1e-3) / 1e9}

    def sustained_mfma_tflops(element_bits=8):
        """What the matrix pipes of this GPU sustain on the scaled matrix instruction alone (E4M3 or E2M1 operands in
        registers, pseudo-random bits, no memory traffic), at the clock the power management settles on: the ceiling
        a GEMM could reach on this machine if moving data were free. About 0.3 s of launches, the last two thirds timed."""
        sink = torch.empty(512 * 256, dtype=torch.float32, device=dev)
        for _ in range(40):
            mx.mxfp8_mfma_rate_probe_ex(512, 1000, element_bits, sink)
        a, b = ev(), ev()
        a.record()
        flop = 0.0
        for _ in range(80):
            flop += mx.mxfp8_mfma_rate_probe_ex(512, 1000, element_bits, sink)
        b.record()
        torch.cuda.synchronize()
        return flop / (a.elapsed_time(b) * 1e-3) / 1e12

    def rotating_copy_gbs(src, sets, launches):
        """A plain device-to-device copy of the same source with the same rotation: what the memory system of
        this box gives the simplest possible stream (read + write bytes per second). Two copies: the library's own
        copy kernel in the configuration that measured fastest (one workgroup per compute unit, grid-stride,
        128-bit streaming loads and stores), and torch's copy_."""
        srcs = [src] + [src.clone() for _ in range(sets - 1)]
        dsts = [torch.empty_like(t) for t in srcs]
        cus = torch.cuda.get_device_properties(dev).multi_processor_count
        res = []
        for fn in (lambda i: mx.mxfp8_copy_rate_probe(srcs[i % sets], dsts[i % sets], cus, 0),
                   lambda i: dsts[i % sets].copy_(srcs[i % sets])):
            for i in range(sets):
                fn(i)
            a, b = ev(), ev()
            torch.cuda.synchronize()
            a.record()
            for i in range(launches):
                fn(i)
            b.record()
            torch.cuda.synchronize()
            res.append(2.0 * src.numel() * src.element_size() / (a.elapsed_time(b) / launches * 1e-3) / 1e9)
        return res

    gemm_flop = 2.0 * T * H * O
    extras = {}
    mfma_sustained = sustained_mfma_tflops()
    if not args.no_extras:
        q_ms, q_fp = rotating_quantize(X, 8, 160)
        f_ms, f_fp = rotating_quantize(dY, 2, 100)
        extras["quant_bf16"] = (q_ms, q_fp, 160, rotating_copy_gbs(X, 8, 160))
        extras["quant_f32"] = (f_ms, f_fp, 100, rotating_copy_gbs(dY, 2, 100))
        extras["dequant_bf16"] = rotating_dequantize(11, 165) + (165,)
        for key, fn in (("fused_output_quantization", fused_output_quantization), ("simulated_path", simulated_path),
                        ("grouped_moe", grouped_moe), ("single_copy", single_copy), ("mxfp4_path", mxfp4_path), ("mxfp6_path", mxfp6_path),
                        ("layer_set", layer_set)):
            try:
                extras[key] = fn()
            except Exception as exc:   # the headline measurement must survive a problem in an extra one
                extras[key] = {"error": repr(exc)}

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = dt / args.steps * 1e3
    step_flops = 3 * gemm_flop
    gemm_bytes = {"fprop": (T + O) * H * (1 + 1 / 32) + T * O * 2, "dgrad": (T + H) * O * (1 + 1 / 32) + T * H * 2,
                  "wgrad": (O + H) * T * (1 + 1 / 32) + O * H * 4}
    shapes = {"fprop": f"{T}x{O}x{H}, BF16 out", "dgrad": f"{T}x{H}x{O}, BF16 out", "wgrad": f"{O}x{H}x{T}, FP32 out"}

    def gemm_roofline(name):
        ms = float(np.mean([a.elapsed_time(b) for a, b in marks[name]]))
        tf = gemm_flop / (ms * 1e-3) / 1e12
        return {"bound": "mfma", "achieved": tf, "peak": MFMA_FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / MFMA_FP8_PEAK_TFLOPS, "peak_sustained": mfma_sustained,
                "frac_sustained": tf / mfma_sustained, "traffic": traffic_from_profile(name + " "),
                "algorithmic_bytes": gemm_bytes[name], "kernel": f"gemm_persistent_kernel ({name} {shapes[name]})",
                "avg_ms": ms, "launches": len(marks[name])}

    out = {
        "metric": "MXFP8 GEMM TFLOP/s (% MFMA peak) + quantize GB/s (% HBM), 8B-class, 1 GPU",
        "value": step_flops / (dt / args.steps) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp8-e4m3 x ue8m0, fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"8B-class MLP up-projection linear layer, fwd+bwd: T={T} tokens, H={H} -> O={O}; "
                               "quantize X,W (BF16) and dY (FP32) along both axes, fprop+dgrad+wgrad, dequantize X; "
                               "tiled scale layout",
                   "T": T, "H": H, "O": O},
        "roofline": gemm_roofline("fprop"),
        "roofline_dgrad": gemm_roofline("dgrad"),
        "roofline_wgrad": gemm_roofline("wgrad"),
    }
    out["gemm_tflops_fprop"] = out["roofline"]["achieved"]
    for key, name, elems, bpe, prof in (("roofline_quantize", "quant_bf16", T * H, 4.0625, "quantize X BF16"),
                                        ("roofline_quantize_f32", "quant_f32", T * O, 6.0625, "quantize dY FP32")):
        if name in extras:
            ms, footprint, launches, copy_gbs = extras[name]
            gbs = elems * bpe / (ms * 1e-3) / 1e9
            out[key] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                        "traffic": traffic_from_profile(prof), "algorithmic_bytes": elems * bpe,
                        "kernel": f"quantize_kernel ({'BF16 X 8192x4096' if name == 'quant_bf16' else 'FP32 dY 8192x14336'}, both axes)",
                        "avg_ms": ms, "launches": launches, "rotating_footprint_mb": footprint / 1e6,
                        "plain_copy_gbs": copy_gbs[0], "frac_of_plain_copy": gbs / copy_gbs[0], "torch_copy_gbs": copy_gbs[1]}
    if "dequant_bf16" in extras:
        ms, footprint, launches = extras["dequant_bf16"]
        nbytes = T * H * (1 + 1 / 32 + 2)
        gbs = nbytes / (ms * 1e-3) / 1e9
        out["roofline_dequantize"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                                      "traffic": traffic_from_profile("dequantize X"), "algorithmic_bytes": nbytes,
                                      "kernel": f"dequantize_kernel (X {T}x{H} row copy -> BF16)", "avg_ms": ms, "launches": launches,
                                      "rotating_footprint_mb": footprint / 1e6}
    if "roofline_quantize" in out:
        out["quantize_gbs_bf16_both"] = out["roofline_quantize"]["achieved"]
    for key in ("fused_output_quantization", "simulated_path", "grouped_moe", "single_copy", "mxfp4_path", "mxfp6_path"):
        if key in extras:
            out[key] = extras[key]
    if "layer_set" in extras:
        out["layer_set_16384"] = extras["layer_set"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
