"""The calls only enqueue and read nothing on the host, so a step can be captured into a HIP graph: every
replay must give what the eager calls give (replayed several times, with eager work and synchronisations in
between)."""
import numpy as np
import pytest
import torch

from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
SMALL = synth.ModelShape(2, 512, 8, 2, 128, 1408, 5000, 4999, dtype="bf16", lm_head_scale=8.0, name="small-gqa")


@pytest.mark.parametrize("ms", [synth.TINY, SMALL], ids=["tiny-f32", "small-bf16"])
def test_graph_replay_equals_eager(ms):
    P, Q = 64, 32
    w = synth.Weights(ms, 11)
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=8, n_pages=8, max_batch=1, max_q=Q, max_tokens=P)
    table = eng.i32(H.identity_table(eng, 1))
    prompt = synth.random_tokens(ms, 11, P)
    eng.prefill_kv(eng.i32(prompt), eng.i32([0, P]), table, None, total_tokens=P, max_seqlen=P)
    prefix = eng.i32([P])
    qt = eng.i32(np.full((1, Q), ms.mask_id))
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    nrem = torch.zeros(1, 1, dtype=torch.int32, device=eng.device)

    def eager_from(tokens):
        t = tokens.clone()
        c, f, e = torch.zeros_like(cand), torch.zeros_like(conf), torch.zeros_like(ent)
        r = torch.zeros_like(nrem)
        eng.denoise_step(t, prefix, table, c, f, e, max_prefix_len=P)
        eng.unmask(t, c, f, 0.9, 2, n_remaining=r)
        torch.cuda.synchronize()
        return t.cpu(), c.cpu(), f.cpu(), e.cpu(), r.cpu()

    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        eng.denoise_step(qt, prefix, table, cand, conf, ent, max_prefix_len=P)
        eng.unmask(qt, cand, conf, 0.9, 2, n_remaining=nrem)
    torch.cuda.synchronize()
    qt.copy_(eng.i32(np.full((1, Q), ms.mask_id)))          # the capture itself does not run the step
    for replay in range(4):
        want = eager_from(qt)                                # eager work on the same state, between replays
        graph.replay()
        torch.cuda.synchronize()
        got = (qt.cpu(), cand.cpu(), conf.cpu(), ent.cpu(), nrem.cpu())
        for g, wv in zip(got, want):
            assert torch.equal(g, wv), replay
        assert int(nrem) == Q - 2 * (replay + 1)
    assert eng.read_status() == 0
    eng.close()
