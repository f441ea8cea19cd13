"""Dream-7B / Qwen2.5-7B-shaped layer (d 3584, 28 query / 4 KV heads x 128, MLP 18944, vocab 152064) at
full width, on slices the oracle can compute:
  * long-context step: prefix KV of 8192 tokens drawn directly (N(0,1), bf16), 2 sequences, block of 32
    with 16 masked -- the shape of the batch-32 / 8192-prefix workload, one layer, two of its sequences;
  * the same step at batch 4 (128 rows), which takes the large-M kernels;
  * two blocks in flight (Q = 64, threshold 0.85, floor 1 per block) on prefilled prompts of 2048 and
    1500 tokens -- the shape of the batch-16 workload, one layer, two of its sequences."""
import numpy as np
import pytest
import torch

from oracle import dllm_oracle as O
from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
W = synth.as_float
ST = synth.round_bf16
MS = synth.DREAM_7B.with_layers(1)


@pytest.fixture(scope="module")
def weights():
    w = synth.Weights(MS, 4)
    w.layer(0), w.globals()
    return w


def fill_pool(eng, table_row, layer, k_bits, v_bits):
    """Writes K/V [n, Hkv, dh] (bf16 bit patterns) of one sequence into its pages."""
    n = k_bits.shape[0]
    pt = eng.cfg.page_tokens
    for which, bits in ((0, k_bits), (1, v_bits)):
        slab = eng.kv_slab(layer, which)                          # [pages, Hkv, pt, dh] view
        t = torch.from_numpy(bits.astype(np.int16)).view(torch.bfloat16).to(eng.device)
        for p0 in range(0, n, pt):
            m = min(pt, n - p0)
            slab[int(table_row[p0 // pt]), :, :m, :] = t[p0:p0 + m].permute(1, 0, 2)


def check_step(eng, w, Bn, Q, blks, caches, prefix, table, tau, m, block_len):
    qt = eng.i32(np.stack(blks))
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(Bn, Q, dtype=torch.float32, device=eng.device)
    eng.denoise_step(qt, eng.i32(prefix), eng.i32(table), cand, conf, ent, max_prefix_len=max(prefix))
    logits = eng.debug_logits(qt, eng.i32(prefix), eng.i32(table), max_prefix_len=max(prefix)).cpu().numpy()
    nb = Q // block_len
    nun = torch.zeros(Bn, nb, dtype=torch.int32, device=eng.device)
    eng.unmask(qt, cand, conf, tau, m, block_len=block_len, n_unmasked=nun)
    after = qt.cpu().numpy()
    for b in range(Bn):
        ck, cv = caches[b]
        exact, _ = O.forward_cached(w, blks[b], [W(ck)], [W(cv)], widen=W)
        err = H.rel_err_rows(logits[b], exact).max()
        r = O.denoise_step(w, blks[b], [W(ck)], [W(cv)], tau, m, block_len=block_len, widen=W, store=ST)
        print(f"seq {b}: logit rel err vs exact oracle {err:.3e}, vs bf16-storage oracle "
              f"{H.rel_err_rows(logits[b], r['logits']).max():.3e}")
        assert err <= H.logit_tol("bf16", 1)
        masked = blks[b] == MS.mask_id
        n_gap, n_rows, _, _ = H.check_exact_decisions(MS, exact, masked, cand.cpu().numpy()[b], H.logit_tol("bf16", 1))
        print(f"  {n_gap} of {n_rows} masked rows decided against the exact oracle")
        H.check_step_outputs(MS, r, masked, cand.cpu().numpy()[b], conf.cpu().numpy()[b], ent.cpu().numpy()[b],
                             "bf16", gpu_logits=logits[b])
        decided = all(H.selection_is_decided(r["conf"][s0:s0 + block_len], masked[s0:s0 + block_len], tau, m)
                      for s0 in range(0, Q, block_len))
        if decided:
            assert np.nonzero(after[b] != blks[b])[0].tolist() == r["chosen"]
        assert int(nun[b].sum()) >= sum(min(m, int(masked[s0:s0 + block_len].sum())) for s0 in range(0, Q, block_len))
    assert eng.read_status() == 0


@pytest.mark.parametrize("Bn", [2, 4])
def test_long_prefix_step_with_drawn_kv(weights, Bn):
    w = weights
    P, Q, pt = 8192, 32, 64
    mp = (P + Q + pt - 1) // pt
    eng = H.make_engine(MS, w, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q)
    if Bn > 2:
        eng.set_kernel_mode(0)
    rng = np.random.default_rng(3)
    table = rng.permutation(Bn * mp).astype(np.int32).reshape(Bn, mp)      # scattered physical pages
    prefix = [P, P - 1000][:2] + [P - 37 * i for i in range(2, Bn)]
    caches, blks = [], []
    for b in range(Bn):
        k, v = synth.random_kv(MS, 4, 0, b, prefix[b])
        fill_pool(eng, table[b], 0, k, v)
        caches.append((k, v))
        blks.append(synth.masked_block(MS, 40 + b, Q, 16))
    check_step(eng, w, Bn, Q, blks, caches, prefix, table, 0.9, 1, Q)
    eng.close()


def test_two_blocks_in_flight_on_prefilled_prompts(weights):
    w = weights
    lens, Q, pt = [2048, 1500], 64, 64
    mp = (max(lens) + Q + pt - 1) // pt
    eng = H.make_engine(MS, w, page_tokens=pt, max_pages_per_seq=mp, n_pages=2 * mp, max_batch=2, max_q=Q,
                        max_tokens=sum(lens))
    table = H.identity_table(eng, 2)
    seqs = [synth.random_tokens(MS, 50 + i, n) for i, n in enumerate(lens)]
    toks = np.concatenate(seqs).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(toks), eng.i32(cu), eng.i32(table), None, total_tokens=len(toks), max_seqlen=max(lens))
    caches, blks = [], []
    for b in range(2):
        ck, cv = O.prefill(w, seqs[b], widen=W, store=ST)
        got = H.gather_cache(eng, table[b], lens[b], 0, 0)
        assert np.abs(got - ck[0]).max() <= 2e-2 * np.abs(ck[0]).max()
        got = H.gather_cache(eng, table[b], lens[b], 0, 1)
        assert np.abs(got - cv[0]).max() <= 2e-2 * np.abs(cv[0]).max()
        # the step is checked against the oracle's own (storage-precision) cache, as bf16 bit patterns
        caches.append((synth.f32_to_bf16_bits(ck[0].astype(np.float32)), synth.f32_to_bf16_bits(cv[0].astype(np.float32))))
        blks.append(synth.masked_block(MS, 60 + b, Q, 40))
    check_step(eng, w, 2, Q, blks, caches, lens, table, 0.85, 1, 32)
    eng.close()


def test_full_depth_batch_32_prefix_8192_sampled_sequences():
    """The long-context large-batch workload in the launch configuration bench.py times (Dream-7B-shaped, 28 layers,
    batch 32, prefix KV of 8192 tokens per sequence drawn on the device, one block of 32 with 16 masked): the
    library runs the whole batch, the oracle recomputes two of its sequences layer by layer from host copies of
    the device-drawn weights and of those sequences' cache pages."""
    from paper_2601_07568_amd.binding import Engine
    ms = synth.DREAM_7B
    Bn, P, Q, pt = 32, 8192, 32, 64
    dev = torch.device("cuda:0")
    mp = (P + Q + pt - 1) // pt
    g, layers = synth.device_weights(ms, torch, dev, 5)
    eng = Engine(ms, None, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q, max_tokens=0,
                 device_weights=(g, layers), pack=False)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    pool = eng.kv_pool.view(torch.bfloat16)
    for i in range(0, pool.numel(), 1 << 28):
        n = min(1 << 28, pool.numel() - i)
        pool[i:i + n] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    table_np = np.arange(Bn * mp).reshape(Bn, mp)
    table = eng.i32(table_np)
    blks = np.stack([synth.masked_block(ms, 5, Q, 16, stream=b) for b in range(Bn)])
    sample = [3, 29]
    # host copies of the sampled sequences' caches, taken before the step writes its own rows behind them
    caches = {b: [(H.gather_cache_rows(eng, table_np[b], P, l, 0).astype(np.float64),
                   H.gather_cache_rows(eng, table_np[b], P, l, 1).astype(np.float64)) for l in range(ms.n_layers)]
              for b in sample}
    qt = eng.i32(blks)
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=dev)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)
    ent = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)
    prefix = eng.i32([P] * Bn)
    eng.denoise_step(qt, prefix, table, cand, conf, ent, max_prefix_len=P)
    assert eng.read_status() == 0
    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    ident = lambda a: a
    pos = np.arange(Q) + P
    xs = {(b, w): host(g["tok_emb"][torch.from_numpy(blks[b]).to(dev)]) for b in sample for w in (0, 1)}
    for l in range(ms.n_layers):
        lw = {n: host(t) for n, t in layers[l].items()}
        for b in sample:
            ck, cv = caches[b][l]
            for w in (0, 1):
                st = ST if w else None
                x = xs[(b, w)]
                q, k, v = O.layer_qkv(ms, lw, x, pos, ident, st)
                xs[(b, w)] = O.layer_finish(ms, lw, x, O.attention(q, np.concatenate([ck, k]), np.concatenate([cv, v])),
                                            ident, st)
        del lw

    class Head:
        pass
    head = Head()
    head.ms = ms
    hw = {"final_norm": host(g["final_norm"]), "lm_head": host(g["lm_head"])}
    Head.__getitem__ = lambda self, k: hw[k]
    for b in sample:
        stored = O.head_logits(head, xs[(b, 1)], ident, ST)
        exact = O.head_logits(head, xs[(b, 0)], ident)
        masked = blks[b] == ms.mask_id
        n_gap, n_rows, _, _ = H.check_exact_decisions(ms, exact, masked, cand.cpu().numpy()[b],
                                                      H.logit_tol("bf16", ms.n_layers))
        print(f"seq {b}: {n_gap} of {n_rows} masked rows decided against the exact oracle; bf16-storage oracle vs exact "
              f"{H.rel_err_rows(stored, exact).max():.3e}")
        ocand, oconf, oent, _ = O.confidence(stored, ms.mask_id)
        r = {"logits": stored, "cand": ocand, "conf": oconf, "entropy": oent}
        # outputs only (the batch's logits are never materialised): decisions and statistics of the masked rows, with
        # the fixed full-depth tolerance against the oracle with bfloat16 storage
        n_exact = H.check_step_outputs(ms, r, masked, cand.cpu().numpy()[b], conf.cpu().numpy()[b],
                                       ent.cpu().numpy()[b], "bf16", eps=H.logit_tol("bf16", ms.n_layers, "storage"))
        print(f"seq {b}: {n_exact} of {int(masked.sum())} masked rows decided by margin and equal")
        assert (cand.cpu().numpy()[b][~masked] == blks[b][~masked]).all()
    eng.close()


def test_full_depth_batch_16_prefill_and_two_blocks_in_flight_sampled_sequence():
    """The batch-16 workload at its own size and in the launch configuration bench.py times (Dream-7B-shaped, 28
    layers, 16 prompts prefilled in ONE dllm_prefill_kv call, then a step with two blocks of 32 in flight per sequence,
    threshold 0.85, floor 1 per block): fifteen prompts have the workload's 2048 tokens, one has 192 so that the
    oracle can recompute it at full depth (prefill and step chained, layer by layer from host copies of the
    device-drawn weights; 28 layers of a 2048-token prompt in float64 are out of reach in a test).  Checked for that
    sequence: the deepest cached K, the logits (materialised by the debug call for the whole batch), candidates,
    confidences, entropies and the per-block unmask sets."""
    from paper_2601_07568_amd.binding import Engine
    ms = synth.DREAM_7B
    Bn, S, Q, bl, pt = 16, 2048, 64, 32, 64
    sample, S_short = 5, 192
    lens = [S] * Bn
    lens[sample] = S_short
    dev = torch.device("cuda:0")
    mp = (S + Q + pt - 1) // pt
    g, layers = synth.device_weights(ms, torch, dev, 4)
    eng = Engine(ms, None, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q,
                 max_tokens=sum(lens), device_weights=(g, layers), pack=False)
    table_np = np.arange(Bn * mp).reshape(Bn, mp)
    table = eng.i32(table_np)
    prompts = [synth.random_tokens(ms, 40 + b, lens[b]) for b in range(Bn)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(prompts)), eng.i32(cu), table, None, total_tokens=int(cu[-1]), max_seqlen=S)
    blks = np.stack([np.concatenate([synth.masked_block(ms, 5, bl, 24, stream=2 * b),
                                     synth.masked_block(ms, 5, bl, 32, stream=2 * b + 1)]) for b in range(Bn)])
    qt = eng.i32(blks)
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=dev)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)
    ent = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)
    prefix = eng.i32(lens)
    eng.denoise_step(qt, prefix, table, cand, conf, ent, max_prefix_len=S)
    logits = eng.debug_logits(qt, prefix, table, max_prefix_len=S)[sample].cpu().numpy()
    nun = torch.zeros(Bn, 2, dtype=torch.int32, device=dev)
    eng.unmask(qt, cand, conf, 0.85, 1, block_len=bl, n_unmasked=nun)
    assert eng.read_status() == 0
    ref = H.layerwise_oracle_step(ms, g, layers, prompts[sample], blks[sample])
    exact, stored = ref["exact"], ref["stored"]
    got_k = H.gather_cache_rows(eng, table_np[sample], S_short, ms.n_layers - 1, 0)
    assert np.abs(got_k - ref["k_last"]).max() <= H.logit_tol("bf16", ms.n_layers, "storage") * np.abs(ref["k_last"]).max()
    err_exact, err_store = H.rel_err_rows(logits, exact).max(), H.rel_err_rows(logits, stored).max()
    print(f"28 layers, batch 16: logit rel err vs exact oracle {err_exact:.3e}, vs bf16-storage oracle {err_store:.3e}; "
          f"bf16-storage oracle vs exact oracle {H.rel_err_rows(stored, exact).max():.3e}")
    eps_exact, eps_store = H.logit_tol("bf16", ms.n_layers), H.logit_tol("bf16", ms.n_layers, "storage")
    assert err_store <= eps_store and err_exact <= eps_exact
    masked = blks[sample] == ms.mask_id
    c, f, e = cand.cpu().numpy()[sample], conf.cpu().numpy()[sample], ent.cpu().numpy()[sample]
    n_gap, n_rows, _, _ = H.check_exact_decisions(ms, exact, masked, c, eps_exact)
    ocand, oconf, oent, _ = O.confidence(stored, ms.mask_id)
    r = {"logits": stored, "cand": ocand, "conf": oconf, "entropy": oent}
    n_exact = H.check_step_outputs(ms, r, masked, c, f, e, "bf16", gpu_logits=logits, eps=eps_store)
    print(f"{n_gap} of {n_rows} masked rows decided against the exact oracle, {n_exact} against the oracle with "
          f"bfloat16 storage")
    # the per-block selection (threshold cannot fire at this vocabulary size: the floor of each block)
    after = qt.cpu().numpy()[sample]
    for k in range(2):
        sl = slice(k * bl, (k + 1) * bl)
        _, ch = O.unmask(blks[sample][sl], ocand[sl], oconf[sl], ms.mask_id, 0.85, 1)
        assert int(nun[sample, k]) == len(ch) == 1
        if H.selection_is_decided(oconf[sl], masked[sl], 0.85, 1):
            assert np.nonzero(after[sl] != blks[sample][sl])[0].tolist() == ch
    # every other sequence: outputs well-formed
    call = cand.cpu().numpy()
    mall = blks == ms.mask_id
    assert ((call[mall] >= 0) & (call[mall] < ms.vocab) & (call[mall] != ms.mask_id)).all()
    assert (call[~mall] == blks[~mall]).all() and (nun.cpu().numpy() == 1).all()
    eng.close()
