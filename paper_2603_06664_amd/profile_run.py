"""Workload for rocprofv3: a few launches of each hot-path kernel at a benchmark shape, plus
one plain device copy of known size that calibrates the HBM byte counters.

  rocprofv3 --kernel-trace --stats --output-format csv -d OUT -- python3 -m paper_2603_06664_amd.profile_run
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT -- python3 -m paper_2603_06664_amd.profile_run
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT -- python3 -m paper_2603_06664_amd.profile_run

Inputs are random bf16 tensors of the workload's shape (values do not matter for byte or
duration counters); the append kernel rotates over disjoint input sets so that its reads
come from HBM rather than from the last-level cache.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as P
from .workloads import CONFIGS

COPY_BYTES = 1 << 30


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--iters", type=int, default=8)
    ap.add_argument("--input-sets", type=int, default=8)
    args = ap.parse_args()
    cfg = CONFIGS[args.workload]
    H, D, n, nk = cfg.n_heads, cfg.head_dim, cfg.n_q, cfg.n_keys
    dev = "cuda"
    desc = P.TableDesc()
    tab = torch.empty(P.crope_table_bytes(desc) // 4, dtype=torch.float32, device=dev)
    P.crope_build_table(desc, tab)
    # calibration copy: reads COPY_BYTES and writes COPY_BYTES
    src = torch.empty(COPY_BYTES, dtype=torch.uint8, device=dev).random_(0, 255)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    sets = [tuple(torch.randn(n, H, D, device=dev, dtype=torch.bfloat16) for _ in range(3))
            for _ in range(args.input_sets)]
    gq = torch.ones(H * D, device=dev)
    gk = torch.ones(H * D, device=dev)
    cap = nk
    k_cache = torch.randn(cap, H, D, device=dev, dtype=torch.bfloat16)
    v_cache = torch.randn(cap, H, D, device=dev, dtype=torch.bfloat16)
    q_rot = torch.empty(n, H, D, device=dev, dtype=torch.bfloat16)
    out = torch.empty_like(q_rot)
    ws_bytes = P.chunk_attention_workspace_bytes(n, H, nk)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    dst_row = (cfg.start_frame - cfg.first_kv_frame) * cfg.hw + cfg.token_offset
    torch.cuda.synchronize()
    for i in range(args.iters):
        q, k, v = sets[i % len(sets)]
        P.crope_qk_norm_rotate_append(desc, tab, q, k, v, gq, gk, cfg.eps, H * D, n, H, cfg.grid_h,
                                      cfg.grid_w, cfg.start_frame, cfg.token_offset, q_rot, k_cache,
                                      v_cache, cap, dst_row)
        P.chunk_attention(q_rot, n, H, k_cache, v_cache, cap, [(0, nk)], D ** -0.5, out, None, ws,
                          ws_bytes)
    # the fused projection entry point (both norm readings), model width c_in = H*128
    c_in = H * D
    xs = [torch.randn(n, c_in, device=dev, dtype=torch.bfloat16) for _ in range(4)]
    w_qkv = (torch.randn(3 * H * D, c_in, device=dev) * c_in ** -0.5).to(torch.bfloat16)
    bias = 0.1 * torch.randn(3 * H * D, device=dev)
    pws_bytes = P.crope_qkv_project_workspace_bytes(n, H, H * D)
    pws = torch.empty(max(pws_bytes, 16), dtype=torch.uint8, device=dev)
    for i in range(args.iters):
        grp = D if i % 2 == 0 else H * D
        P.crope_qkv_project_norm_rotate_append(desc, tab, xs[i % 4], w_qkv, bias, c_in, gq, gk, cfg.eps, grp,
                                               n, H, cfg.grid_h, cfg.grid_w, cfg.start_frame,
                                               cfg.token_offset, q_rot, k_cache, v_cache, cap, dst_row, pws,
                                               pws_bytes)
    torch.cuda.synchronize()
    print("profile_run done: %s, %d iterations, copy %d bytes" % (cfg.name, args.iters, COPY_BYTES))


if __name__ == "__main__":
    main()
