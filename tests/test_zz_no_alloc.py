"""chunk_attention_static, the entry point that allocates nothing (its scratch is a buffer
built into the library), against chunk_attention with a caller-provided workspace: same
kernels and work division, so the outputs must be bit-identical; both are also held to the
oracle.  Two calls in a row share the built-in buffer, the second with a smaller input."""
import numpy as np
import pytest

from paper_2603_06664_amd import workloads as W

import harness as Hn

pytestmark = pytest.mark.gpu


def _case(P, n_q, H, n_keys, seed, expect_split, folded=False):
    import torch
    import oracle
    rng = np.random.default_rng(seed)
    bits = lambda shape: W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    qb, kb, vb = bits((n_q, H, 128)), bits((n_keys, H, 128)), bits((n_keys, H, 128))
    q_ref = Hn.bits_to_f64(qb)
    scale = Hn.SCALE
    if folded:   # q as the q-scaling append call would have written it
        c = np.float32(P.crope_folded_q_scale(Hn.SCALE))
        qb = W.f32_to_bf16_bits(W.bf16_bits_to_f32(qb) * c)
        q_ref = Hn.bits_to_f64(qb) / float(c)
        scale = P.CROPE_SCALE_FOLDED
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    segs = [(0, n_keys)]
    wsb = P.chunk_attention_workspace_bytes(n_q, H, n_keys)
    assert (wsb > 0) == expect_split, "workspace %d" % wsb
    assert wsb <= P.chunk_attention_static_capacity()
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    out_ref, out_new = torch.empty_like(q), torch.empty_like(q)
    lse_ref = torch.empty((H, n_q), dtype=torch.float32, device="cuda")
    lse_new = torch.empty_like(lse_ref)
    P.chunk_attention(q, n_q, H, k, v, n_keys, segs, scale, out_ref, lse_ref, ws, wsb)
    torch.cuda.synchronize()
    print("static call: n_q=%d heads=%d keys=%d scratch=%d" % (n_q, H, n_keys, wsb), flush=True)
    P.chunk_attention_static(q, n_q, H, k, v, n_keys, segs, scale, out_new, lse_new)
    torch.cuda.synchronize()
    assert np.array_equal(Hn.dev_bits(out_new), Hn.dev_bits(out_ref))
    assert np.array_equal(lse_new.cpu().numpy(), lse_ref.cpu().numpy())
    o, lse = oracle.attention(q_ref, Hn.bits_to_f64(kb), Hn.bits_to_f64(vb), Hn.SCALE)
    Hn.assert_close("o", Hn.bits_to_f64(Hn.dev_bits(out_new)), o)
    assert np.max(np.abs(lse_new.cpu().numpy().astype(np.float64) - lse)) <= 2e-2


def test_static_scratch_matches_workspace_entry_point():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    import paper_2603_06664_amd as P
    from paper_2603_06664_amd import binding
    binding._load()
    assert P.chunk_attention_static_capacity() == 64 << 20
    # few queries against many keys: the key range is split and the partials go through the scratch
    _case(P, 300, 6, 9000, seed=501, expect_split=True)
    # second call on the same buffer with a smaller input (fewer queries, heads and keys)
    _case(P, 70, 2, 5000, seed=502, expect_split=True)
    # a shape that is not split uses no scratch at all
    _case(P, 2100, 16, 400, seed=503, expect_split=False)
    # and once more through the scratch with the softmax factor folded into q
    _case(P, 150, 3, 7000, seed=504, expect_split=True, folded=True)


def test_static_scratch_rejects_oversized_problem():
    import paper_2603_06664_amd as P
    from paper_2603_06664_amd import binding
    binding._load()

    class Fake:   # validation fails before any memory is touched
        def __init__(self, shape): self.shape = shape
        def data_ptr(self): return 0x10000
        def dim(self): return 3
        def stride(self, i): return [self.shape[1] * 128, 128, 1][i]
    n_q, H, n_keys = 300, 64, 60000
    assert P.chunk_attention_workspace_bytes(n_q, H, n_keys) > P.chunk_attention_static_capacity()
    q, c = Fake((n_q, H, 128)), Fake((n_keys, H, 128))
    with pytest.raises(P.CropeError) as ei:
        P.chunk_attention_static(q, n_q, H, c, c, n_keys, [(0, n_keys)], Hn.SCALE, q, None)
    assert ei.value.code == -5 and "built-in" in ei.value.message
