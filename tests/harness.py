"""Shared test plumbing: runs one configuration through the HIP path (via the C-ABI
binding) and through the CPU oracle on the same seeded inputs, and compares.

Tolerances (bf16 outputs): relative L2 <= 1e-2 over a tensor and, per element,
|got - oracle| <= 2e-2 wherever |oracle| < 8.  A bf16 number of magnitude >= 8 has a half-ulp
of 2^-5 > 2e-2, so no single rounding of the oracle value can meet 2e-2 there; for those
elements (rotated keys under a per-head gain scale) the bound is bf16's own half-ulp at the
oracle value's binade, 2^(floor(log2|oracle|) - 8), plus 2^-18 * |oracle| for the fp32
arithmetic in front of the rounding.
"""
from __future__ import annotations

import numpy as np

from paper_2603_06664_amd import workloads as W
from paper_2603_06664_amd.devutil import (  # noqa: F401  (re-exported for the tests)
    SCALE, bits_to_f64, dev_bits, dst_row, make_table, to_dev_bf16, visible_segments)

MAX_ABS = 2e-2
REL_L2 = 1e-2
LARGE = 8.0   # below this magnitude the flat 2e-2 bound applies


def element_bound(ref: np.ndarray) -> np.ndarray:
    a = np.abs(np.asarray(ref, dtype=np.float64))
    big = a >= LARGE
    half_ulp = np.exp2(np.floor(np.log2(np.where(big, a, LARGE))) - 8.0)
    return np.where(big, half_ulp + 2.0 ** -18 * a, MAX_ABS)


def errors(got: np.ndarray, ref: np.ndarray):
    """max-abs difference, relative L2, and the largest excess over the per-element bound
    (<= 0 when every element is inside it)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    max_abs = float(diff.max()) if diff.size else 0.0
    denom = float(np.sqrt((ref ** 2).sum()))
    rel_l2 = float(np.sqrt((diff ** 2).sum()) / denom) if denom > 0 else 0.0
    excess = float((diff - element_bound(ref)).max()) if diff.size else -1.0
    return max_abs, rel_l2, excess


def assert_close(name, got, ref):
    max_abs, rel_l2, excess = errors(got, ref)
    msg = "%s: max_abs=%.3e rel_l2=%.3e" % (name, max_abs, rel_l2)
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), msg + " (non-finite)"
    assert rel_l2 <= REL_L2, msg
    assert excess <= 0.0, msg + " (an element is %.3e beyond its bound: 2e-2 below |ref| = 8, bf16 half-ulp above)" % excess
    return max_abs, rel_l2


# ------------------------------------------------------------------ oracle side
def oracle_chain(cfg: W.ChunkConfig, inp: W.ChunkInputs, norm_group=None, q_rows=None):
    """Returns dict with q_rot [n_q,H,D], k_cache/v_cache [cap,H,D] (fp64), segs, o, lse.
    ``q_rows``: optional indices of query rows for which attention is evaluated."""
    import oracle
    H, D = cfg.n_heads, cfg.head_dim
    group = H * D if norm_group is None else norm_group
    cap_tokens = cfg.capacity_frames * cfg.hw
    cache = oracle.Cache(cap_tokens, H, D)
    kf, vf = bits_to_f64(inp.k), bits_to_f64(inp.v)
    q_rot = None
    for (s, nf, row0, n, off, is_cur) in W.chunk_schedule(cfg):
        k_rot = oracle.qk_norm_rotate(kf[row0:row0 + n], inp.gain_k, cfg.eps, group, cfg.dims,
                                      cfg.theta, cfg.grid_h, cfg.grid_w, s, off)
        cache.write(dst_row(cfg, s, off), k_rot, vf[row0:row0 + n])
        if is_cur:
            q_rot = oracle.qk_norm_rotate(bits_to_f64(inp.q), inp.gain_q, cfg.eps, group, cfg.dims,
                                          cfg.theta, cfg.grid_h, cfg.grid_w, s, off)
    segs = visible_segments(cfg)
    kk, vv = cache.gather(segs)
    qs = q_rot if q_rows is None else q_rot[np.asarray(q_rows)]
    o, lse = oracle.attention(qs, kk, vv, SCALE)
    return dict(q_rot=q_rot, k_cache=cache.k, v_cache=cache.v, segs=segs, o=o, lse=lse)


# ------------------------------------------------------------------ HIP side
def hip_chain(cfg: W.ChunkConfig, inp: W.ChunkInputs, norm_group=None, want_lse=True, folded=False):
    """Runs table build, every append call of the schedule, then attention, through the
    C ABI.  Returns numpy results (bf16 bits widened to fp64 where noted).
    folded: the current call writes q multiplied by scale*log2(e) (…_append_qscaled) and attention
    runs with CROPE_SCALE_FOLDED; the returned q_rot has the factor divided out again."""
    import torch
    import paper_2603_06664_amd as P
    H, D = cfg.n_heads, cfg.head_dim
    group = H * D if norm_group is None else norm_group
    desc, tab = make_table(P.TableDesc(dim_t=cfg.dims[0], dim_h=cfg.dims[1], dim_w=cfg.dims[2],
                                       theta=cfg.theta))
    cap = cfg.capacity_frames * cfg.hw
    k_cache = torch.zeros((cap, H, D), dtype=torch.bfloat16, device="cuda")
    v_cache = torch.zeros_like(k_cache)
    q = to_dev_bf16(inp.q)
    k = to_dev_bf16(inp.k)
    v = to_dev_bf16(inp.v)
    gq = torch.from_numpy(inp.gain_q).cuda()
    gk = torch.from_numpy(inp.gain_k).cuda()
    q_out = torch.empty_like(q)
    scratch_q = None
    for (s, nf, row0, n, off, is_cur) in W.chunk_schedule(cfg):
        if is_cur:
            qi, qo = q, q_out
        else:
            # history / other ranks' calls: only their k, v matter; feed k as a stand-in q
            if scratch_q is None or scratch_q.shape[0] < n:
                scratch_q = torch.empty((n, H, D), dtype=torch.bfloat16, device="cuda")
            qi, qo = k[row0:row0 + n], scratch_q[:n]
        if folded and is_cur:
            P.crope_qk_norm_rotate_append_qscaled(desc, tab, qi, k[row0:row0 + n], v[row0:row0 + n], gq, gk,
                                                  cfg.eps, group, n, H, cfg.grid_h, cfg.grid_w, s, off,
                                                  P.crope_folded_q_scale(SCALE), qo, k_cache, v_cache, cap,
                                                  dst_row(cfg, s, off))
        else:
            P.crope_qk_norm_rotate_append(desc, tab, qi, k[row0:row0 + n], v[row0:row0 + n], gq, gk,
                                          cfg.eps, group, n, H, cfg.grid_h, cfg.grid_w, s, off, qo,
                                          k_cache, v_cache, cap, dst_row(cfg, s, off))
    segs = visible_segments(cfg)
    out = torch.empty_like(q_out)
    lse = torch.empty((H, cfg.n_q), dtype=torch.float32, device="cuda") if want_lse else None
    n_keys = sum(n for _, n in segs)
    ws_bytes = P.chunk_attention_workspace_bytes(cfg.n_q, H, n_keys)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    P.chunk_attention(q_out, cfg.n_q, H, k_cache, v_cache, cap, segs, P.CROPE_SCALE_FOLDED if folded else SCALE,
                      out, lse, ws, ws_bytes)
    torch.cuda.synchronize()
    q_unit = P.crope_folded_q_scale(SCALE) if folded else 1.0
    return dict(q_rot=bits_to_f64(dev_bits(q_out)) / q_unit, k_cache=bits_to_f64(dev_bits(k_cache)),
                v_cache_bits=dev_bits(v_cache), o=bits_to_f64(dev_bits(out)),
                lse=lse.cpu().numpy().astype(np.float64) if want_lse else None, segs=segs)


# ------------------------------------------------------------------ fused projection
def oracle_projected(cfg: W.ChunkConfig, pin: W.ProjectionInputs, inp: W.ChunkInputs, norm_group=None,
                     use_bias=True):
    """fp64 chain of Algorithm 3 steps 1-3 for the current call's rows: (q~, k~, v)."""
    import oracle
    H, D = cfg.n_heads, cfg.head_dim
    group = H * D if norm_group is None else norm_group
    return oracle.qkv_project_norm_rotate(
        bits_to_f64(pin.x), bits_to_f64(pin.w), pin.bias if use_bias else None, inp.gain_q, inp.gain_k,
        cfg.eps, group, H, cfg.dims, cfg.theta, cfg.grid_h, cfg.grid_w, cfg.start_frame, cfg.token_offset)


def hip_projected(cfg: W.ChunkConfig, pin: W.ProjectionInputs, inp: W.ChunkInputs, norm_group=None,
                  use_bias=True, cap_extra=5, dst=3, x_pad=0):
    """Runs crope_qkv_project_norm_rotate_append once.  Returns q~ [n,H,D] (fp64 from bf16),
    the written k rows, the written v rows, and the untouched remainder of the caches (bits)."""
    import torch
    import paper_2603_06664_amd as P
    H, D = cfg.n_heads, cfg.head_dim
    group = H * D if norm_group is None else norm_group
    n, c_in = pin.x.shape
    desc, tab = make_table(P.TableDesc(dim_t=cfg.dims[0], dim_h=cfg.dims[1], dim_w=cfg.dims[2],
                                       theta=cfg.theta))
    cap = n + cap_extra
    canary = 0x7FC1   # a NaN pattern no kernel writes
    k_cache = torch.full((cap, H, D), 0, dtype=torch.int16, device="cuda").fill_(canary).view(torch.bfloat16)
    v_cache = k_cache.clone()
    xs = to_dev_bf16(pin.x)
    if x_pad:
        buf = torch.zeros((n, c_in + x_pad), dtype=torch.bfloat16, device="cuda")
        buf[:, :c_in] = xs
        xs = buf[:, :c_in]
    w = to_dev_bf16(pin.w)
    bias = torch.from_numpy(pin.bias).cuda() if use_bias else None
    gq = torch.from_numpy(inp.gain_q).cuda()
    gk = torch.from_numpy(inp.gain_k).cuda()
    q_out = torch.empty((n, H, D), dtype=torch.bfloat16, device="cuda")
    ws_bytes = P.crope_qkv_project_workspace_bytes(n, H, group)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    P.crope_qkv_project_norm_rotate_append(desc, tab, xs, w, bias, c_in, gq, gk, cfg.eps, group, n, H,
                                           cfg.grid_h, cfg.grid_w, cfg.start_frame, cfg.token_offset,
                                           q_out, k_cache, v_cache, cap, dst, ws, ws_bytes)
    torch.cuda.synchronize()
    kb, vb = dev_bits(k_cache), dev_bits(v_cache)
    untouched = np.concatenate([kb[:dst].ravel(), kb[dst + n:].ravel(), vb[:dst].ravel(), vb[dst + n:].ravel()])
    return dict(q=bits_to_f64(dev_bits(q_out)), k=bits_to_f64(kb[dst:dst + n]), v=bits_to_f64(vb[dst:dst + n]),
                untouched_ok=bool(np.all(untouched == canary)))
