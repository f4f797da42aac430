#!/usr/bin/env python3
"""Benchmark of the per-chunk hot path on one MI355X.

One step = crope_qk_norm_rotate_append + chunk_attention for one 480P chunk (one layer,
one denoising pass) on synthetic Wan-shaped bf16 tensors already resident in HBM.  The
default workload is the final chunk of a 21-latent-frame video (4680 queries x 32760
keys, 12 heads).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
# HBM bytes per launch at workload C4 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled
# by what the same counter reads for a 1 GiB copy (x2.000 and x1.000); the summary with the
# commands is profiles/chunk_attention_and_rope_C4_pmc.md.  Other workloads report null.
MEASURED_TRAFFIC_BYTES = {
    "C4": {"chunk_attention": (162809.3 * 2.000 + 14046.1 * 1.000) * 1024,
           "crope_qk_norm_rotate_append": (21204.7 * 2.000 + 42120.0 * 1.000) * 1024,
           # profiles/qkv_project_C4_kernel_trace_and_pmc.md (per-head norm variant)
           "crope_qkv_project_norm_rotate_append": (76935.5 * 2.000 + 42120.0 * 1.000) * 1024},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5", "R288", "R960", "C5P", "C4R"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-projection", action="store_true",
                    help="skip the separate timing of the fused QKV projection entry point")
    ap.add_argument("--cpu-rows", type=int, default=1024,
                    help="query rows of the workload the CPU oracle is timed on")
    ap.add_argument("--input-sets", type=int, default=8,
                    help="disjoint q/k/v input sets rotated between steps so the append kernel "
                         "reads from HBM, not from the 256 MB last-level cache")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives on the hot path); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2603_06664_amd as P
    from paper_2603_06664_amd import binding, workloads as W
    binding._load()   # no fallback: raises if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    import harness as Hn

    cfg = W.CONFIGS[args.workload]
    H, D = cfg.n_heads, cfg.head_dim
    inp = W.make_inputs(cfg)
    desc, tab = Hn.make_table()
    cap = cfg.capacity_frames * cfg.hw
    k_cache = torch.zeros((cap, H, D), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros_like(k_cache)
    k_all, v_all = Hn.to_dev_bf16(inp.k), Hn.to_dev_bf16(inp.v)
    gq, gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()
    group = H * D

    # fill the cache the way generation would (history blocks and other shards), untimed
    cur = None
    scratch = torch.empty((cfg.chunk_tokens, H, D), dtype=torch.bfloat16, device="cuda")
    for (s, nf, row0, n, off, is_cur) in W.chunk_schedule(cfg):
        if is_cur:
            cur = (s, row0, n, off)
        P.crope_qk_norm_rotate_append(desc, tab, k_all[row0:row0 + n], k_all[row0:row0 + n],
                                      v_all[row0:row0 + n], gq, gk, cfg.eps, group, n, H, cfg.grid_h,
                                      cfg.grid_w, s, off, scratch[:n], k_cache, v_cache, cap,
                                      Hn.dst_row(cfg, s, off))
    s, row0, n, off = cur
    dst = Hn.dst_row(cfg, s, off)
    # rotating input sets for the timed append (set 0 = the real inputs; others are copies
    # at different addresses so every step streams from HBM)
    q0 = Hn.to_dev_bf16(inp.q)
    sets = [(q0, k_all[row0:row0 + n], v_all[row0:row0 + n])]
    for _ in range(max(0, args.input_sets - 1)):
        sets.append(tuple(t.clone() for t in sets[0]))
    q_rot = torch.empty_like(q0)
    out = torch.empty_like(q0)
    lse = torch.empty((H, cfg.n_q), dtype=torch.float32, device="cuda")
    segs = Hn.visible_segments(cfg)
    n_keys = sum(m for _, m in segs)
    ws_bytes = P.chunk_attention_workspace_bytes(cfg.n_q, H, n_keys)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")

    def step(i, ev=None):
        q, k, v = sets[i % len(sets)]
        if ev: ev[0].record()
        P.crope_qk_norm_rotate_append(desc, tab, q, k, v, gq, gk, cfg.eps, group, n, H, cfg.grid_h,
                                      cfg.grid_w, s, off, q_rot, k_cache, v_cache, cap, dst)
        if ev: ev[1].record()
        P.chunk_attention(q_rot, cfg.n_q, H, k_cache, v_cache, cap, segs, Hn.SCALE, out, lse, ws,
                          ws_bytes)
        if ev: ev[2].record()

    # setup: the first launches upload the code objects and ramp the clocks; not part of the
    # W warm-up steps the caller asked for
    for i in range(15):
        step(i)
    torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # timed region: exactly K steps, wall clock between synchronisations
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    # per-kernel average launch duration with events on the launch stream: K back-to-back
    # launches of one kernel between two events (an event pair around a single 20 us kernel
    # would add its own few microseconds), same work as the timed steps
    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(args.steps):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    def rope_only(i):
        q, k, v = sets[i % len(sets)]
        P.crope_qk_norm_rotate_append(desc, tab, q, k, v, gq, gk, cfg.eps, group, n, H, cfg.grid_h,
                                      cfg.grid_w, s, off, q_rot, k_cache, v_cache, cap, dst)

    def attn_only(i):
        P.chunk_attention(q_rot, cfg.n_q, H, k_cache, v_cache, cap, segs, Hn.SCALE, out, lse, ws,
                          ws_bytes)

    rope_runs = [timed(rope_only) for _ in range(3)]
    attn_runs = [timed(attn_only) for _ in range(3)]
    rope_ms, attn_ms = float(np.mean(rope_runs)), float(np.mean(attn_runs))
    t_rope, t_attn = np.array(rope_runs), np.array(attn_runs)
    step(0)   # leave out/lse holding the result of a whole step for the parity sample
    torch.cuda.synchronize()

    flops = cfg.attention_flops
    rope_bytes = cfg.rope_bytes
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12
    rope_gbps = rope_bytes / (rope_ms * 1e-3) / 1e9
    value = flops / (ms_per_step * 1e-3) / 1e12

    result = {
        "metric": "chunk attention TFLOP/s + fused RoPE GB/s; ms per 480P chunk (1 GPU)",
        "value": round(value, 3), "unit": "TFLOP/s (attention FLOPs / whole-step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d heads, %d queries x %d keys, d=128, grid %dx%d, start_frame %d"
                               % (cfg.name, H, cfg.n_q, n_keys, cfg.grid_h, cfg.grid_w, cfg.start_frame),
                   "input_sets": len(sets)},
        "attention_ms": round(attn_ms, 5), "attention_ms_min": round(float(t_attn.min()), 5),
        "attention_tflops": round(attn_tflops, 2),
        "rope_ms": round(rope_ms, 5), "rope_ms_min": round(float(t_rope.min()), 5),
        "rope_gbps": round(rope_gbps, 1),
        "roofline": {"kernel": "chunk_attention", "bound": "mfma", "achieved": round(attn_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("chunk_attention"),
                     "algorithmic_flops_per_launch": flops},
        "roofline_rope": {"kernel": "crope_qk_norm_rotate_append", "bound": "hbm",
                          "achieved": round(rope_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                          "frac": round(rope_gbps / PEAK_HBM_GBPS, 4),
                          "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get("crope_qk_norm_rotate_append"),
                          "algorithmic_bytes_per_launch": rope_bytes},
    }

    # Beside the step: the local QKV projection fused with norm + RoPE + cache update (the
    # next row of the path, Algorithm 3 step 1 folded in), timed on its own at the same token
    # count with model width c_in = H*128, against the same work done as a vendor GEMM followed
    # by crope_qk_norm_rotate_append.  Both norm readings; inputs rotate over 4 sets.
    if not args.no_projection:
        c_in = H * D
        pin = W.make_projection_inputs(cfg)
        w_qkv = Hn.to_dev_bf16(pin.w)
        bias = torch.from_numpy(pin.bias).cuda()
        xs = [Hn.to_dev_bf16(pin.x)]
        for _ in range(3):
            xs.append(xs[0].clone())
        proj_flops = 2.0 * n * c_in * 3 * H * D
        y_buf = torch.empty((n, 3 * H * D), dtype=torch.bfloat16, device="cuda")
        bias_bf16 = bias.to(torch.bfloat16)
        fused = {}
        for label, grp in (("norm_per_head", D), ("norm_row_wide", H * D)):
            pws_bytes = P.crope_qkv_project_workspace_bytes(n, H, grp)
            pws = torch.empty(max(pws_bytes, 16), dtype=torch.uint8, device="cuda")

            def fused_call(i, grp=grp, pws=pws, pws_bytes=pws_bytes):
                P.crope_qkv_project_norm_rotate_append(desc, tab, xs[i % 4], w_qkv, bias, c_in, gq, gk,
                                                       cfg.eps, grp, n, H, cfg.grid_h, cfg.grid_w, s, off,
                                                       q_rot, k_cache, v_cache, cap, dst, pws, pws_bytes)

            def unfused_call(i, grp=grp):
                torch.addmm(bias_bf16, xs[i % 4], w_qkv.t(), out=y_buf)
                y = y_buf.view(n, 3, H, D)
                P.crope_qk_norm_rotate_append(desc, tab, y[:, 0], y[:, 1], y[:, 2], gq, gk, cfg.eps, grp,
                                              n, H, cfg.grid_h, cfg.grid_w, s, off, q_rot, k_cache,
                                              v_cache, cap, dst)

            for i in range(20):
                fused_call(i)
                unfused_call(i)
            t_f = min(timed(fused_call) for _ in range(3))
            t_u = min(timed(unfused_call) for _ in range(3))
            fused[label] = {"ms": round(t_f, 5), "tflops": round(proj_flops / (t_f * 1e-3) / 1e12, 1),
                            "vendor_gemm_then_append_ms": round(t_u, 5)}
        best = fused["norm_per_head"]
        result["fused_projection"] = {
            "kernel": "crope_qkv_project_norm_rotate_append", "c_in": c_in, "tokens": n,
            "algorithmic_flops_per_launch": proj_flops, **fused,
            "roofline": {"bound": "mfma", "achieved": best["tflops"], "peak": PEAK_BF16_TFLOPS,
                         "unit": "TFLOP/s", "frac": round(best["tflops"] / PEAK_BF16_TFLOPS, 4),
                         "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get(
                             "crope_qkv_project_norm_rotate_append")}}
        # the timed calls above overwrote the chunk's cache rows and q_rot with projected data:
        # restore the step's own result for the parity sample
        step(0)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        import oracle
        rows = min(args.cpu_rows, cfg.n_q)
        ridx = np.linspace(0, cfg.n_q - 1, rows).astype(np.int64)
        t0 = time.perf_counter()
        kf = Hn.bits_to_f64(inp.k)
        vf = Hn.bits_to_f64(inp.v)
        t_conv = time.perf_counter() - t0
        t0 = time.perf_counter()
        # rotated keys of every visible frame (what the cache holds), then the sampled rows
        k_rot = np.empty_like(kf)
        for (cs, nf, r0, cn, coff, _) in W.chunk_schedule(cfg):
            k_rot[r0:r0 + cn] = oracle.qk_norm_rotate(kf[r0:r0 + cn], inp.gain_k, cfg.eps, group,
                                                     cfg.dims, cfg.theta, cfg.grid_h, cfg.grid_w, cs, coff)
        q_rot_o = oracle.qk_norm_rotate(Hn.bits_to_f64(inp.q), inp.gain_q, cfg.eps, group, cfg.dims,
                                        cfg.theta, cfg.grid_h, cfg.grid_w, s, off)
        t_rot = time.perf_counter() - t0
        t0 = time.perf_counter()
        o_ref, _ = oracle.attention(q_rot_o[ridx], k_rot, vf, Hn.SCALE)
        t_att = time.perf_counter() - t0
        cpu_flops = 4.0 * rows * n_keys * D * H
        result["cpu_baseline"] = {
            "value": round(cpu_flops / t_att / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "fp64 oracle attention on %d of %d query rows (all heads, all %d keys): %.2f s; "
                      "oracle norm+rotate of all visible keys and the chunk's queries: %.2f s"
                      % (rows, cfg.n_q, n_keys, t_att, t_rot),
            "attention_seconds_full_extrapolated": round(t_att * cfg.n_q / rows, 1),
            "gpu_over_oracle": round(attn_tflops / (cpu_flops / t_att / 1e12), 0),
        }
        got = Hn.bits_to_f64(Hn.dev_bits(out))[ridx]
        mx, rl, _ = Hn.errors(got, o_ref)
        result["parity_sample"] = {"rows": rows, "max_abs": float("%.3e" % mx), "rel_l2": float("%.3e" % rl)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
