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


@pytest.mark.parametrize("ms", [synth.TINY, SMALL], ids=["tiny-f32", "small-bf16"])
def test_cached_multiblock_round_as_one_graph(ms):
    """A whole cached round of multi-block decoding for a batch - windows built on the device, the step with padding
    rows, the selection with a floor per block, the write-back and the state transitions - captured once and replayed
    round after round: every replay must leave the tokens, states and counters the eager calls leave."""
    Bn, NB, BL, Wn = 3, 3, 32, 2
    lens = [48, 33, 64]
    thr = 100.0 if ms is SMALL else 5.46            # an entropy threshold that lets a few positions through per round
    w = synth.Weights(ms, 12)
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=12, n_pages=12 * Bn, max_batch=Bn, max_q=Wn * BL,
                        max_tokens=sum(lens) + Bn * Wn * BL)
    dev = eng.device
    table = eng.i32(H.identity_table(eng, Bn))
    prompts = [synth.random_tokens(ms, 70 + b, lens[b]) for b in range(Bn)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(prompts)), eng.i32(cu), table, None, total_tokens=int(cu[-1]), max_seqlen=max(lens))
    Q = Wn * BL
    base = eng.i32(lens)
    max_prefix = max(lens) + NB * BL

    def buffers():
        return dict(win=torch.zeros(Bn, Q, dtype=torch.int32, device=dev), wfl=torch.zeros(Bn, Wn, dtype=torch.int32, device=dev),
                    pre=torch.zeros(Bn, dtype=torch.int32, device=dev), qv=torch.zeros(Bn, dtype=torch.int32, device=dev),
                    wlo=torch.zeros(Bn, dtype=torch.int32, device=dev), cand=torch.zeros(Bn, Q, dtype=torch.int32, device=dev),
                    conf=torch.zeros(Bn, Q, dtype=torch.float32, device=dev), ent=torch.zeros(Bn, Q, dtype=torch.float32, device=dev))

    def one_round(gen, state, counter, b):
        eng.fsm_window(gen, state, base, BL, Wn, 0, b["win"], b["wfl"], b["pre"], b["qv"], b["wlo"])
        eng.denoise_step_var(b["win"], b["pre"], b["qv"], table, b["cand"], b["conf"], b["ent"], max_prefix_len=max_prefix)
        eng.unmask_blocks(b["win"], b["cand"], b["ent"], thr, b["wfl"], True, BL)
        eng.fsm_scatter(b["win"], b["wlo"], b["qv"], gen, NB, BL, Wn)
        eng.fsm_update(gen, state, counter, BL, 0.1, 0.95, 1, None, None, None)

    def fresh():
        gen = torch.full((Bn, NB * BL), ms.mask_id, dtype=torch.int32, device=dev)
        state = torch.zeros(Bn, NB, dtype=torch.int32, device=dev)
        state[:, 0] = 2
        return gen, state, torch.zeros(Bn, NB, dtype=torch.int32, device=dev)

    gen, state, counter = fresh()
    gb = buffers()
    one_round(*[t.clone() for t in (gen, state, counter)], buffers())          # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_round(gen, state, counter, gb)
    torch.cuda.synchronize()
    g0, s0, c0 = fresh()
    gen.copy_(g0); state.copy_(s0); counter.copy_(c0)
    progressed = 0
    for replay in range(6):
        eg, es, ec = gen.clone(), state.clone(), counter.clone()
        one_round(eg, es, ec, buffers())                                       # eager, on a copy of the same state
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(gen, eg) and torch.equal(state, es) and torch.equal(counter, ec), replay
        progressed += int((gen != ms.mask_id).sum())
    assert progressed > 0 and eng.read_status() == 0
    eng.close()


@pytest.mark.parametrize("ms", [synth.TINY, SMALL], ids=["tiny-f32", "small-bf16"])
def test_whole_decode_round_as_one_graph(ms):
    """The round that needs no host read - plan-driven windows, cached step, packed forward without cache with a
    device-resident total, selection, write-back, transitions, next plan - captured once and replayed until the batch
    is decoded: after every replay the tokens, states and plan equal those of the same rounds run eagerly."""
    from tests.test_gpu_fsm import BL, RoundBuffers, device_round
    NB, Wn, delay, refresh_every = 3, 3, 1, 4
    lens = [48, 33, 64]
    Bn = len(lens)
    thr = 100.0 if ms is SMALL else 5.46
    cap = sum(lens) + Bn * NB * BL
    w = synth.Weights(ms, 12)
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=12, n_pages=12 * Bn, max_batch=Bn, max_q=Wn * BL,
                        max_tokens=cap)
    table = eng.i32(H.identity_table(eng, Bn))
    prompts = [synth.random_tokens(ms, 70 + b, lens[b]) for b in range(Bn)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)

    def prefill():
        eng.prefill_kv(eng.i32(np.concatenate(prompts)), eng.i32(cu), table, None, total_tokens=int(cu[-1]),
                       max_seqlen=max(lens))

    n_rounds = 14
    prefill()
    rb = RoundBuffers(eng, ms, prompts, NB, Wn, cap)
    eager = []
    for _ in range(n_rounds):
        device_round(eng, rb, table, thr, delay, refresh_every)
        eager.append([t.clone() for t in (rb.gen, rb.state, rb.counter, rb.nocache, rb.plan_commit, rb.cu)])
    torch.cuda.synchronize()
    assert any(int(e[5][-1]) > 0 for e in eager) and any(int(e[5][-1]) == 0 for e in eager)   # both kinds of round
    assert int((eager[-1][0] == ms.mask_id).sum()) < int((eager[0][0] == ms.mask_id).sum())

    prefill()
    rg = RoundBuffers(eng, ms, prompts, NB, Wn, cap)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        device_round(eng, rg, table, thr, delay, refresh_every)
    torch.cuda.synchronize()
    fresh = RoundBuffers(eng, ms, prompts, NB, Wn, cap)        # the capture itself runs nothing, but start clean anyway
    for name in ("gen", "state", "counter", "since", "nocache", "plan_commit"):
        getattr(rg, name).copy_(getattr(fresh, name))
    prefill()
    for rnd in range(n_rounds):
        graph.replay()
        torch.cuda.synchronize()
        got = [rg.gen, rg.state, rg.counter, rg.nocache, rg.plan_commit, rg.cu]
        for g, e in zip(got, eager[rnd]):
            assert torch.equal(g, e), rnd
        _ = (rg.gen + 1).sum().item()                          # eager work and a synchronisation between replays
    assert eng.read_status() == 0
    eng.close()
