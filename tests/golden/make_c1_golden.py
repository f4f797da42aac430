"""Writes tests/golden/c1_oracle_values.txt: sampled values of the CPU oracle's outputs for
configuration C1 (Tiny).  Calls only the oracle and the shared seeded input generator; it is a
regression pin for the oracle (the paper prints no numeric example to compare with).

    python tests/golden/make_c1_golden.py
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2603_06664_amd import workloads as W  # noqa: E402


def c1_outputs():
    cfg = W.CONFIGS["C1"]
    inp = W.make_inputs(cfg)
    f64 = lambda b: W.bf16_bits_to_f32(b).astype(np.float64)
    H, D = cfg.n_heads, cfg.head_dim
    k_rot = np.empty((cfg.n_keys, H, D))
    for (s, nf, row0, n, off, is_cur) in W.chunk_schedule(cfg):
        k_rot[row0:row0 + n] = oracle.qk_norm_rotate(f64(inp.k)[row0:row0 + n], inp.gain_k, cfg.eps, H * D,
                                                     cfg.dims, cfg.theta, cfg.grid_h, cfg.grid_w, s, off)
    q_rot = oracle.qk_norm_rotate(f64(inp.q), inp.gain_q, cfg.eps, H * D, cfg.dims, cfg.theta, cfg.grid_h,
                                  cfg.grid_w, cfg.start_frame, 0)
    o, lse = oracle.attention(q_rot, k_rot, f64(inp.v), D ** -0.5)
    return q_rot, k_rot, o, lse


SAMPLES = [("q_rot", (0, 0, 0)), ("q_rot", (23, 1, 127)), ("q_rot", (7, 0, 45)), ("q_rot", (11, 1, 90)),
           ("k_rot", (0, 0, 1)), ("k_rot", (71, 1, 126)), ("k_rot", (30, 0, 44)), ("k_rot", (50, 1, 87)),
           ("o", (0, 0, 0)), ("o", (23, 1, 127)), ("o", (12, 0, 64)), ("o", (5, 1, 3)),
           ("lse", (0, 0)), ("lse", (1, 23)), ("lse", (0, 12))]

if __name__ == "__main__":
    q_rot, k_rot, o, lse = c1_outputs()
    arrays = dict(q_rot=q_rot, k_rot=k_rot, o=o, lse=lse)
    with open(os.path.join(HERE, "c1_oracle_values.txt"), "w") as f:
        f.write("# CPU-oracle outputs for configuration C1 (seed 0), written by make_c1_golden.py.\n")
        f.write("# Regression pin of the oracle only: the paper prints no numeric example.\n")
        f.write("# columns: array, index..., value\n")
        for name, idx in SAMPLES:
            f.write("%s %s %.17g\n" % (name, " ".join(str(i) for i in idx), arrays[name][idx]))
    print("written")
