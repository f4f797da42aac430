"""Device-side plumbing shared by the benchmark, the profiling workload, smoke() and the tests:
moving bf16 bit patterns to and from the GPU, building the rotary tables through the C ABI,
and the cache-row bookkeeping of a workload (which ring slot a frame occupies, which row
ranges are visible).  No arithmetic of the method and no reference implementation lives here.
"""
from __future__ import annotations

import numpy as np

from . import workloads as W

SCALE = 128 ** -0.5   # softmax scale 1/sqrt(head_dim)


def bits_to_f64(b: np.ndarray) -> np.ndarray:
    return W.bf16_bits_to_f32(b).astype(np.float64)


def to_dev_bf16(bits: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev_bits(t) -> np.ndarray:
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def make_table(desc=None):
    import torch
    from . import binding as P
    desc = desc or P.TableDesc()
    tab = torch.empty(P.crope_table_bytes(desc) // 4, dtype=torch.float32, device="cuda")
    P.crope_build_table(desc, tab)
    return desc, tab


def dst_row(cfg: W.ChunkConfig, start_frame: int, token_offset: int) -> int:
    """Cache row where the call for (start_frame, token_offset) writes its first token."""
    return W.cache_slot(cfg, start_frame) * cfg.hw + token_offset


def visible_segments(cfg: W.ChunkConfig):
    """Row segments holding frames first_kv_frame .. start_frame+n_frames-1, oldest first,
    merged where slots are consecutive."""
    segs = []
    for f in range(cfg.first_kv_frame, cfg.start_frame + cfg.n_frames):
        start = W.cache_slot(cfg, f) * cfg.hw
        if segs and segs[-1][0] + segs[-1][1] == start:
            segs[-1] = (segs[-1][0], segs[-1][1] + cfg.hw)
        else:
            segs.append((start, cfg.hw))
    return segs


class StepBuffers:
    """Everything one hot-path step of a workload needs, resident on the GPU: tables, gains,
    caches filled the way generation would have filled them (every earlier block and, for a
    sharded workload, the other ranks' rows of the current block, all through
    crope_qk_norm_rotate_append), the current call's raw q, k, v and its outputs."""

    def __init__(self, cfg: W.ChunkConfig, inp: W.ChunkInputs, norm_group=None, input_sets: int = 1,
                 folded: bool = True):
        """folded: the step's append writes q times scale*log2(e) and its attention runs with
        CROPE_SCALE_FOLDED (the faster pairing); otherwise plain q and an explicit scale."""
        import torch
        from . import binding as P
        self.cfg, self.P = cfg, P
        self.folded = folded
        self.q_scale = P.crope_folded_q_scale(SCALE) if folded else 1.0
        H, D = cfg.n_heads, cfg.head_dim
        self.H, self.D = H, D
        self.group = H * D if norm_group is None else norm_group
        self.desc, self.tab = make_table(P.TableDesc(dim_t=cfg.dims[0], dim_h=cfg.dims[1], dim_w=cfg.dims[2],
                                                     theta=cfg.theta))
        self.cap = cfg.capacity_frames * cfg.hw
        self.k_cache = torch.zeros((self.cap, H, D), dtype=torch.bfloat16, device="cuda")
        self.v_cache = torch.zeros_like(self.k_cache)
        k_all, v_all = to_dev_bf16(inp.k), to_dev_bf16(inp.v)
        self.gq, self.gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()
        cur = None
        stand_in = torch.empty((cfg.chunk_tokens, H, D), dtype=torch.bfloat16, device="cuda")
        for (s, nf, row0, n, off, is_cur) in W.chunk_schedule(cfg):
            if is_cur:
                cur = (s, row0, n, off)
            # history / other ranks' calls: only their k, v matter; k stands in for q
            P.crope_qk_norm_rotate_append(self.desc, self.tab, k_all[row0:row0 + n], k_all[row0:row0 + n],
                                          v_all[row0:row0 + n], self.gq, self.gk, cfg.eps, self.group, n, H,
                                          cfg.grid_h, cfg.grid_w, s, off, stand_in[:n], self.k_cache,
                                          self.v_cache, self.cap, dst_row(cfg, s, off))
        self.s, row0, self.n, self.off = cur
        self.dst = dst_row(cfg, self.s, self.off)
        q0 = to_dev_bf16(inp.q)
        # set 0 = the real inputs; the others are copies at different addresses, so that a loop
        # over the sets streams every step's inputs from HBM rather than from the last-level cache
        self.sets = [(q0, k_all[row0:row0 + self.n], v_all[row0:row0 + self.n])]
        for _ in range(max(0, input_sets - 1)):
            self.sets.append(tuple(t.clone() for t in self.sets[0]))
        self.q_rot = torch.empty_like(q0)
        self.out = torch.empty_like(q0)
        self.lse = torch.empty((H, cfg.n_q), dtype=torch.float32, device="cuda")
        self.segs = visible_segments(cfg)
        self.n_keys = sum(m for _, m in self.segs)
        self.ws_bytes = P.chunk_attention_workspace_bytes(cfg.n_q, H, self.n_keys)
        self.ws = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()

    def append(self, i: int = 0):
        cfg, P = self.cfg, self.P
        q, k, v = self.sets[i % len(self.sets)]
        if self.folded:
            P.crope_qk_norm_rotate_append_qscaled(self.desc, self.tab, q, k, v, self.gq, self.gk, cfg.eps,
                                                  self.group, self.n, self.H, cfg.grid_h, cfg.grid_w, self.s,
                                                  self.off, self.q_scale, self.q_rot, self.k_cache, self.v_cache,
                                                  self.cap, self.dst)
        else:
            P.crope_qk_norm_rotate_append(self.desc, self.tab, q, k, v, self.gq, self.gk, cfg.eps, self.group,
                                          self.n, self.H, cfg.grid_h, cfg.grid_w, self.s, self.off, self.q_rot,
                                          self.k_cache, self.v_cache, self.cap, self.dst)

    def attention(self):
        self.P.chunk_attention(self.q_rot, self.cfg.n_q, self.H, self.k_cache, self.v_cache, self.cap,
                               self.segs, self.P.CROPE_SCALE_FOLDED if self.folded else SCALE, self.out,
                               self.lse, self.ws, self.ws_bytes)

    def step(self, i: int = 0):
        self.append(i)
        self.attention()
