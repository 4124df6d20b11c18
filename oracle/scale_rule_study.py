"""Synthetic-data stand-in for the paper's comparison of scale rounding rules (Section 3.3, the figure
that contrasts the OCP v1 rule with Algorithm 1) and of element formats (Section 3.1): how many elements
saturate, and the quantization error, when the seeded LLM-shaped tensors of this repository are
quantized row-wise under each (format, rule). CPU only, oracle only; run by hand:
    python oracle/scale_rule_study.py
The paper's own evidence is training curves on its data; this only shows the mechanism on tensors
with the same shape of distribution."""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import oracle  # noqa: E402
from paper_2506_08027_amd import synth_inputs as si  # noqa: E402


def study(name, x):
    rows = []
    for fmt, top in (("e4m3", 448.0), ("e5m2", 57344.0)):
        for rule in ("up", "ocp"):
            q, s = oracle.quantize_rowwise_mode(x, fmt, rule)
            back = oracle.dequantize_mode(q, s, fmt)
            scaled = np.abs(x.astype(np.float64)).reshape(x.shape[0], -1, 32) / np.exp2(s.astype(np.float64) - 127)[..., None]
            over = scaled > top
            err = back - x
            rows.append((name, fmt, rule, over.any(-1).mean(), over.mean(), float((err ** 2).sum() / (x.astype(np.float64) ** 2).sum()),
                         float(np.abs(err).max() / np.abs(x).max())))
    return rows


def main():
    tensors = [
        ("activations", si.bf16_bits_to_f32(si.activations(2048, 4096, seed=2))),
        ("weights", si.bf16_bits_to_f32(si.weights(2048, 4096, seed=4))),
        ("gradients+spikes", np.asarray(si.gradients(2048, 4096, seed=5, spikes=True), np.float32)),
    ]
    print(f"{'tensor':18s} {'fmt':5s} {'rule':4s} {'blocks w/ overflow':>19s} {'elements clipped':>17s} {'rel. MSE':>10s} {'max err / max':>14s}")
    for name, x in tensors:
        for r in study(name, np.ascontiguousarray(x, np.float32)):
            print(f"{r[0]:18s} {r[1]:5s} {r[2]:4s} {r[3]:19.4f} {r[4]:17.6f} {r[5]:10.3e} {r[6]:14.3e}")


if __name__ == "__main__":
    main()
