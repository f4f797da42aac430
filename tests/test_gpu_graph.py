"""The step under HIP graph capture: crope_qk_norm_rotate_append_qscaled + chunk_attention_static
(the entry point that allocates nothing) recorded once and replayed several times, with eager
work and synchronisations between the replays and new inputs each time.  Every replay must equal
the eager result of the same inputs bit for bit, and the first one the oracle."""
import numpy as np
import pytest

from paper_2603_06664_amd import workloads as W

import harness as Hn

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("split", [True, False], ids=["split_keys", "one_pass"])
def test_graph_replays_match_eager(split):
    import torch
    import paper_2603_06664_amd as P
    from paper_2603_06664_amd.devutil import StepBuffers
    if split:    # one frame of queries against 25 frames of keys: the key range is split, partials in the scratch
        cfg = W.ChunkConfig("GR1", 61, 3, 9, 11, start_frame=24, n_frames=1, first_kv_frame=0)
    else:        # the first block of 16 heads: one pass over the keys, no scratch
        cfg = W.ChunkConfig("GR2", 62, 16, 9, 11, start_frame=0, n_frames=3, first_kv_frame=0)
    inp = W.make_inputs(cfg)
    sb = StepBuffers(cfg, inp, folded=True)
    assert (sb.ws_bytes > 0) == split
    q_in = sb.sets[0][0]
    rng = np.random.default_rng(5)
    variants = [Hn.dev_bits(q_in)] + [W.f32_to_bf16_bits(rng.standard_normal(q_in.shape).astype(np.float32))
                                      for _ in range(3)]

    def step_static():
        sb.append(0)
        P.chunk_attention_static(sb.q_rot, cfg.n_q, sb.H, sb.k_cache, sb.v_cache, sb.cap, sb.segs,
                                 P.CROPE_SCALE_FOLDED, sb.out, sb.lse)

    # eager results of every input variant, through the workspace entry point
    eager = []
    for bits in variants:
        q_in.copy_(Hn.to_dev_bf16(bits))
        sb.step(0)
        torch.cuda.synchronize()
        eager.append((Hn.dev_bits(sb.out).copy(), sb.lse.cpu().numpy().copy()))
    ref = Hn.oracle_chain(cfg, inp)
    Hn.assert_close("o (eager)", Hn.bits_to_f64(eager[0][0]), ref["o"])

    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        step_static()            # warm-up outside the capture (the library looks up its scratch here)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            step_static()
    torch.cuda.synchronize()
    for r, bits in enumerate(variants + variants[:1]):
        print("replay", r, flush=True)
        q_in.copy_(Hn.to_dev_bf16(bits))      # eager work between the replays
        sb.out.zero_()
        sb.lse.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want_o, want_lse = eager[r % len(variants)]
        assert np.array_equal(Hn.dev_bits(sb.out), want_o), "replay %d differs from the eager result" % r
        assert np.array_equal(sb.lse.cpu().numpy(), want_lse)
