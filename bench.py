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
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
# HBM bytes per launch at workload C4 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch,
# mean of the last 20 dispatches of the benchmark's own step), each scaled by what the same counter
# reads for a 1 GiB copy (x2.000 and x1.000); the summary with the commands is
# profiles/chunk_attention_and_append_C4_counters.md.  Other workloads report null.
MEASURED_TRAFFIC_BYTES = {
    "C4": {"chunk_attention": (247622.1 * 2.000 + 14286.7 * 1.000) * 1024,
           "crope_qk_norm_rotate_append": (21209.0 * 2.000 + 42175.3 * 1.000) * 1024,
           # profiles/qkv_project_C4_kernel_trace_and_counters.md (per-head norm variant)
           "crope_qkv_project_norm_rotate_append": (76838.2 * 2.000 + 42120.0 * 1.000) * 1024},
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
    ap.add_argument("--cpu-rows", type=int, default=0,
                    help="query rows of the workload the CPU oracle is timed on (0 = all of them)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the MFMA-only loop and the plain copy that measure this GPU's own ceilings")
    ap.add_argument("--input-sets", type=int, default=0,
                    help="disjoint q/k/v input sets rotated between steps so the append kernel "
                         "reads from HBM, not from the 256 MB last-level cache (0 = as many as "
                         "it takes to hold 512 MB of inputs, at least 8)")
    return ap.parse_args()


def _ceilings_lib():
    import ctypes
    from paper_2603_06664_amd import build
    lib = ctypes.CDLL(build.CEILINGS_LIB)
    lib.ceiling_mfma_operand_bytes.restype = ctypes.c_size_t
    lib.ceiling_mfma_flops.restype = ctypes.c_double
    lib.ceiling_mfma_flops.argtypes = [ctypes.c_int]
    lib.ceiling_mfma_launch.restype = ctypes.c_int
    lib.ceiling_mfma_launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    lib.ceiling_copy_launch.restype = ctypes.c_int
    lib.ceiling_copy_launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    return lib


def _events_ms(torch, fn, reps):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _graph_ms(torch, fn, reps):
    """Average duration of fn(i), i < reps, captured once into a HIP graph and replayed between
    two events on the capture stream."""
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        fn(0)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(reps):
                fn(i)
        graph.replay()   # untimed
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def measure_mfma_ceiling(torch, attn_tflops):
    """What the matrix pipes of THIS GPU sustain with nothing else going on: 8 waves per CU
    issuing only bf16 MFMAs on random operands for about the duration of one attention launch."""
    lib = _ceilings_lib()
    ops = torch.randn(lib.ceiling_mfma_operand_bytes() // 2, device="cuda").to(torch.bfloat16)
    sink = torch.zeros(512 * 256, dtype=torch.float32, device="cuda")
    iters = 6000   # ~0.9 ms per launch at 1.6 PFLOP/s

    def run(i):
        rc = lib.ceiling_mfma_launch(ops.data_ptr(), sink.data_ptr(), iters, torch.cuda.current_stream().cuda_stream)
        assert rc == 0, "ceiling_mfma_launch: hipError %d" % rc
    for i in range(5):
        run(i)
    ms = min(_graph_ms(torch, run, 20) for _ in range(3))
    tf = lib.ceiling_mfma_flops(iters) / (ms * 1e-3) / 1e12
    return {"ceiling_mfma": {"what": "MFMA-only loop (v_mfma_f32_32x32x16_bf16, random bf16 operands in "
                                     "registers, 8 waves on each of the 256 CUs), measured in this run",
                             "tflops": round(tf, 1), "frac_of_datasheet_peak": round(tf / PEAK_BF16_TFLOPS, 4)},
            "frac_of_ceiling_mfma": round(attn_tflops / tf, 4)}


def measure_copy_ceiling(torch, sb, rope_bytes, rope_gbps, steps):
    """A plain 16-byte-per-lane copy that moves as many bytes as the append kernel (half read,
    half written), sources rotating over as many disjoint buffers as the append's inputs."""
    lib = _ceilings_lib()
    half = (int(rope_bytes) // 2 + 15) // 16 * 16
    srcs = [torch.empty(half, dtype=torch.uint8, device="cuda").random_(0, 255) for _ in range(len(sb.sets))]
    dstb = torch.empty(half, dtype=torch.uint8, device="cuda")

    def run(i):
        rc = lib.ceiling_copy_launch(dstb.data_ptr(), srcs[i % len(srcs)].data_ptr(), half,
                                     torch.cuda.current_stream().cuda_stream)
        assert rc == 0, "ceiling_copy_launch: hipError %d" % rc
    for i in range(10):
        run(i)
    ms = min(_graph_ms(torch, run, steps) for _ in range(3))
    gbps = 2.0 * half / (ms * 1e-3) / 1e9
    return {"ceiling_copy": {"what": "plain device copy, 16 B per lane, %d bytes read + %d written per launch, "
                                     "sources rotating over %d buffers, measured in this run" % (half, half, len(srcs)),
                             "gbps": round(gbps, 1), "us": round(ms * 1e3, 2),
                             "frac_of_datasheet_peak": round(gbps / PEAK_HBM_GBPS, 4)},
            "frac_of_ceiling_copy": round(rope_gbps / gbps, 4)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives on the hot path); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2603_06664_amd as P
    from paper_2603_06664_amd import binding, devutil, workloads as W
    binding._load()   # no fallback: raises if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    cfg = W.CONFIGS[args.workload]
    H, D = cfg.n_heads, cfg.head_dim
    inp = W.make_inputs(cfg)
    # tables, gains, the cache filled the way generation would have (untimed), and
    # args.input_sets copies of the call's inputs at different addresses
    n_sets = args.input_sets if args.input_sets > 0 else max(8, -(-(512 << 20) // (int(cfg.rope_bytes) // 2)))
    sb = devutil.StepBuffers(cfg, inp, input_sets=n_sets)
    desc, tab, gq, gk, group = sb.desc, sb.tab, sb.gq, sb.gk, sb.group
    k_cache, v_cache, cap = sb.k_cache, sb.v_cache, sb.cap
    s, n, off, dst = sb.s, sb.n, sb.off, sb.dst
    sets, q_rot, out, lse = sb.sets, sb.q_rot, sb.out, sb.lse
    segs, n_keys, ws, ws_bytes = sb.segs, sb.n_keys, sb.ws, sb.ws_bytes
    SETUP_STEPS = 15

    def step(i):
        sb.append(i)
        sb.attention()

    # setup: the first launches upload the code objects and ramp the clocks; not part of the
    # W warm-up steps the caller asked for
    for i in range(SETUP_STEPS):
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

    # per-kernel average launch duration: K back-to-back launches of one kernel (same work as
    # the timed steps, inputs rotating) captured once into a HIP graph on the launch stream and
    # replayed between two events, so that no host time per launch enters the figure (a Python
    # call through the binding costs ~15 us, about as much as one append kernel runs)
    def timed(fn):
        return _graph_ms(torch, fn, args.steps)

    def timed_eager(fn):   # for calls that include a library GEMM (not captured)
        return _events_ms(torch, fn, args.steps)

    def rope_only(i):
        sb.append(i)

    def attn_only(i):
        sb.attention()

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
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "setup_launches_before_warmup": SETUP_STEPS,
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
        w_qkv = devutil.to_dev_bf16(pin.w)
        bias = torch.from_numpy(pin.bias).cuda()
        xs = [devutil.to_dev_bf16(pin.x)]
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
            t_f = min(timed_eager(fused_call) for _ in range(3))
            t_u = min(timed_eager(unfused_call) for _ in range(3))
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

    if not args.no_ceilings:
        result["roofline"].update(measure_mfma_ceiling(torch, attn_tflops))
        result["roofline_rope"].update(measure_copy_ceiling(torch, sb, rope_bytes, rope_gbps, args.steps))

    if not args.no_cpu_baseline:
        import oracle
        rows = cfg.n_q if args.cpu_rows <= 0 else min(args.cpu_rows, cfg.n_q)
        ridx = np.arange(cfg.n_q) if rows == cfg.n_q else np.linspace(0, cfg.n_q - 1, rows).astype(np.int64)
        kf = devutil.bits_to_f64(inp.k)
        vf = devutil.bits_to_f64(inp.v)
        t0 = time.perf_counter()
        # what the cache holds: rotated keys of every visible frame, written block by block at the
        # rows the schedule gives them, then gathered in the order of the visible segments
        cache = oracle.Cache(cap, H, D)
        for (cs, nf, r0, cn, coff, _) in W.chunk_schedule(cfg):
            k_rot = oracle.qk_norm_rotate(kf[r0:r0 + cn], inp.gain_k, cfg.eps, group, cfg.dims, cfg.theta,
                                          cfg.grid_h, cfg.grid_w, cs, coff)
            cache.write(devutil.dst_row(cfg, cs, coff), k_rot, vf[r0:r0 + cn])
        kk, vv = cache.gather(segs)
        q_rot_o = oracle.qk_norm_rotate(devutil.bits_to_f64(inp.q), inp.gain_q, cfg.eps, group, cfg.dims,
                                        cfg.theta, cfg.grid_h, cfg.grid_w, s, off)
        t_rot = time.perf_counter() - t0
        t0 = time.perf_counter()
        o_ref, lse_ref = oracle.attention(q_rot_o[ridx], kk, vv, devutil.SCALE)
        t_att = time.perf_counter() - t0
        cpu_flops = 4.0 * rows * n_keys * D * H
        result["cpu_baseline"] = {
            "value": round(cpu_flops / t_att / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": "fp64 oracle attention on %s query rows (all heads, all %d keys): %.2f s; "
                      "oracle norm+rotate of all visible keys and the chunk's queries: %.2f s"
                      % ("all %d" % rows if rows == cfg.n_q else "%d of %d" % (rows, cfg.n_q), n_keys, t_att, t_rot),
            "attention_seconds": round(t_att, 2), "rows": rows,
            "gpu_over_oracle": round(attn_tflops / (cpu_flops / t_att / 1e12), 0),
        }
        # parity of the timed step's own output against the oracle, same rows
        got = devutil.bits_to_f64(devutil.dev_bits(out))[ridx]
        diff = np.abs(got - o_ref)
        lse_got = lse.cpu().numpy().astype(np.float64)[:, ridx]
        result["parity"] = {"rows": rows, "of": cfg.n_q,
                            "o_max_abs": float("%.3e" % diff.max()),
                            "o_rel_l2": float("%.3e" % (np.sqrt((diff ** 2).sum() / (o_ref ** 2).sum()))),
                            "lse_max_abs": float("%.3e" % np.abs(lse_got - lse_ref).max()),
                            "within_tolerance": bool(diff.max() <= 2e-2 and
                                                     np.sqrt((diff ** 2).sum() / (o_ref ** 2).sum()) <= 1e-2)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
