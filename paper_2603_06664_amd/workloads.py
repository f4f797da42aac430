"""Seeded synthetic inputs and the registry of the five benchmark configurations.

This module serves both the CPU oracle's tests and the HIP path's tests/bench.  It
holds NONE of the method's arithmetic (no norm, no rotation, no softmax): only shapes,
seeds, random draws and the fp32<->bf16 bit conversion needed to hand both sides the
very same bf16-representable values.

Shapes follow the paper's workload (Experimental Setup: 5 s of 832x480 video at 16 FPS
=> 21 latent frames of 30x52 tokens; chunk-wise generation with three latent frames per
block, start_frame = 0, 3, 6, ... — Section 3.3.2 item 1).  Values are synthetic:
N(0,1) activations, N(1,0.1) RMSNorm gains.

Draw order for a config with generator ``numpy.random.default_rng(seed)`` (float32
draws, then round-to-nearest-even to bf16):
  1. raw q   [Lq, H, D]                    (current chunk / local shard only)
  2. raw k   [n_kv_frames*HW, H, D]        (every frame the cache will ever hold)
  3. raw v   [n_kv_frames*HW, H, D]
  4. gain_q  [H*D]   N(1, 0.1), rounded to bf16-representable fp32
  5. gain_k  [H*D]   same
  6. (k_head_scale only) sigma_h ~ U(0.5, 2) [H], multiplied into gain_k per head
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

HEAD_DIM = 128
DIM_T, DIM_H, DIM_W = 44, 42, 42
THETA = 10000.0
EPS = 1e-6
TAU = 3  # latent frames per generation block


# --------------------------------------------------------------------------- bf16 bits
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # NaN stays NaN (quiet); everything else: add 0x7FFF + lsb, then truncate.
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 values that are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class ChunkConfig:
    name: str
    seed: int
    n_heads: int
    grid_h: int
    grid_w: int
    start_frame: int          # s: global index of the chunk's first frame
    n_frames: int             # F: frames in the current chunk
    first_kv_frame: int       # oldest frame the cache holds when the chunk attends
    token_offset: int = 0     # Delta: global token index of the local shard's row 0
    n_local: Optional[int] = None   # local query/key rows of this call (None = whole chunk)
    cache_frames: Optional[int] = None  # ring capacity in frames (None = all kv frames)
    k_head_scale: bool = False
    head_dim: int = HEAD_DIM
    dims: tuple = (DIM_T, DIM_H, DIM_W)
    theta: float = THETA
    eps: float = EPS

    @property
    def hw(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def chunk_tokens(self) -> int:
        return self.n_frames * self.hw

    @property
    def n_q(self) -> int:
        return self.chunk_tokens if self.n_local is None else self.n_local

    @property
    def n_kv_frames(self) -> int:
        return self.start_frame + self.n_frames - self.first_kv_frame

    @property
    def n_keys(self) -> int:
        return self.n_kv_frames * self.hw

    @property
    def capacity_frames(self) -> int:
        return self.n_kv_frames if self.cache_frames is None else self.cache_frames

    @property
    def attention_flops(self) -> float:
        return 4.0 * self.n_q * self.n_keys * self.head_dim * self.n_heads

    @property
    def rope_bytes(self) -> float:
        # read q,k,v + write q~,k~,v, bf16
        return 6.0 * self.n_q * self.n_heads * self.head_dim * 2


CONFIGS: Dict[str, ChunkConfig] = {
    # Tiny: 2 heads, 4x6 grid, one-frame chunk at frame 5, cache = frames 3..5 in a 3-frame ring.
    "C1": ChunkConfig("C1", 0, 2, 4, 6, start_frame=5, n_frames=1, first_kv_frame=3, cache_frames=3),
    # Wan-1.3B-shaped 480P chunks: 12 heads, 30x52 tokens/frame, 3-frame chunks.
    "C2": ChunkConfig("C2", 1, 12, 30, 52, start_frame=0, n_frames=3, first_kv_frame=0),
    "C3": ChunkConfig("C3", 2, 12, 30, 52, start_frame=6, n_frames=3, first_kv_frame=0),
    "C4": ChunkConfig("C4", 3, 12, 30, 52, start_frame=18, n_frames=3, first_kv_frame=0,
                      k_head_scale=True),
    # One sequence-parallel rank's share (rank 2 of 8) at 40 heads: rows 1170..1754 of the chunk.
    "C5": ChunkConfig("C5", 4, 40, 30, 52, start_frame=18, n_frames=3, first_kv_frame=0,
                      token_offset=2 * 585, n_local=585),
    # --- further shapes of the paper's evaluation (Section 4.2.1: 288x512 and 960x1664 next to
    # 480x832) and the paper's own attention layout after the fused all-to-all (Algorithm 3
    # step 4: all 4680 queries of the chunk, H/P = 40/8 = 5 heads per rank)
    "R288": ChunkConfig("R288", 5, 12, 18, 32, start_frame=18, n_frames=3, first_kv_frame=0),
    "R960": ChunkConfig("R960", 6, 12, 60, 104, start_frame=18, n_frames=3, first_kv_frame=0),
    "C5P": ChunkConfig("C5P", 7, 5, 30, 52, start_frame=18, n_frames=3, first_kv_frame=0),
    # rolling window at full size: a ring of 9 frames (14040 rows) that has wrapped; the final
    # chunk sees frames 12..20, which sit in slots 3..8, 0, 1, 2 -> two row segments
    "C4R": ChunkConfig("C4R", 8, 12, 30, 52, start_frame=18, n_frames=3, first_kv_frame=12, cache_frames=9),
}


@dataclass
class ChunkInputs:
    """bf16 bit patterns (uint16) plus fp32 gains for one config."""
    cfg: ChunkConfig
    q: np.ndarray        # [n_q, H, D] uint16
    k: np.ndarray        # [n_kv_frames*HW, H, D] uint16, frame-major from first_kv_frame
    v: np.ndarray        # same shape
    gain_q: np.ndarray   # [H*D] float32
    gain_k: np.ndarray   # [H*D] float32
    extra: dict = field(default_factory=dict)


def make_inputs(cfg: ChunkConfig) -> ChunkInputs:
    rng = np.random.default_rng(cfg.seed)
    H, D = cfg.n_heads, cfg.head_dim
    q = f32_to_bf16_bits(rng.standard_normal((cfg.n_q, H, D), dtype=np.float32))
    k = f32_to_bf16_bits(rng.standard_normal((cfg.n_keys, H, D), dtype=np.float32))
    v = f32_to_bf16_bits(rng.standard_normal((cfg.n_keys, H, D), dtype=np.float32))
    gq = round_to_bf16((1.0 + 0.1 * rng.standard_normal(H * D, dtype=np.float32)).astype(np.float32))
    gk = round_to_bf16((1.0 + 0.1 * rng.standard_normal(H * D, dtype=np.float32)).astype(np.float32))
    extra = {}
    if cfg.k_head_scale:
        sigma = rng.uniform(0.5, 2.0, size=H).astype(np.float32)
        gk = (gk.reshape(H, D) * sigma[:, None]).astype(np.float32).reshape(-1)
        extra["sigma_h"] = sigma
    return ChunkInputs(cfg, q, k, v, gq, gk, extra)


def chunk_schedule(cfg: ChunkConfig):
    """The append calls that fill the cache the way block-wise generation would.

    Yields (start_frame, n_frames, src_row0, n_rows, token_offset, is_current) for each
    generation block from ``first_kv_frame`` up to and including the current chunk.
    ``src_row0`` indexes ChunkInputs.k / .v.  For a sharded config the current chunk is
    yielded shard by shard (the other ranks' rows stand in for what a collective would
    have delivered); ``is_current`` marks the one call that belongs to this rank.
    """
    hw = cfg.hw
    f = cfg.first_kv_frame
    end = cfg.start_frame + cfg.n_frames
    while f < end:
        blk = cfg.n_frames
        nf = min(blk, end - f) if f >= cfg.start_frame else min(blk, cfg.start_frame - f)
        row0 = (f - cfg.first_kv_frame) * hw
        if f == cfg.start_frame and cfg.n_local is not None:
            n = cfg.n_local
            total = nf * hw
            for off in range(0, total, n):
                rows = min(n, total - off)
                yield (f, nf, row0 + off, rows, off, off == cfg.token_offset)
        else:
            yield (f, nf, row0, nf * hw, 0, f == cfg.start_frame)
        f += nf


def cache_slot(cfg: ChunkConfig, frame: int) -> int:
    """Ring slot (in frames) that holds global frame ``frame``."""
    return (frame - cfg.first_kv_frame) % cfg.capacity_frames if cfg.cache_frames is None \
        else frame % cfg.capacity_frames


# --------------------------------------------------------------------------- projection
@dataclass
class ProjectionInputs:
    """Inputs of the local QKV projection (Algorithm 3 step 1) for one call's token rows."""
    x: np.ndarray      # [n_tokens, c_in] uint16 (bf16 bits): hidden states
    w: np.ndarray      # [3*H*D, c_in] uint16 (bf16 bits): rows 0..HD-1 W_q, then W_k, then W_v
    bias: np.ndarray   # [3*H*D] float32, bf16-representable


def make_projection_inputs(cfg: ChunkConfig, n_tokens: Optional[int] = None,
                           c_in: Optional[int] = None) -> ProjectionInputs:
    """Draw order with ``default_rng(cfg.seed + 1000)``: x ~ N(0,1) [n, c_in]; w ~ N(0, 1/c_in)
    [3HD, c_in] (so that the projected q, k, v are ~N(0,1) like the unfused path's inputs);
    bias ~ N(0, 0.1) [3HD].  c_in defaults to the model width H*D."""
    rng = np.random.default_rng(cfg.seed + 1000)
    hd = cfg.n_heads * cfg.head_dim
    c_in = hd if c_in is None else c_in
    n = cfg.n_q if n_tokens is None else n_tokens
    x = f32_to_bf16_bits(rng.standard_normal((n, c_in), dtype=np.float32))
    w = f32_to_bf16_bits(rng.standard_normal((3 * hd, c_in), dtype=np.float32) * np.float32(c_in ** -0.5))
    bias = round_to_bf16((0.1 * rng.standard_normal(3 * hd, dtype=np.float32)).astype(np.float32))
    return ProjectionInputs(x, w, bias)
