"""GPU parity at the tiny float32 configuration (2 layers, d 256, 4 heads x 64, MLP 688, vocab
4096, prompt 64, one block of 32): every call of the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import dllm_oracle as O
from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
TINY = synth.TINY
P, Q = 64, 32


@pytest.fixture(scope="module")
def world():
    w = synth.Weights(TINY, 0)
    eng = H.make_engine(TINY, w, page_tokens=16, max_pages_per_seq=16, n_pages=48, max_batch=3, max_q=64,
                        max_tokens=512)
    prompt = synth.random_tokens(TINY, 0, P)
    ck, cv = O.prefill(w, prompt)
    return dict(w=w, eng=eng, prompt=prompt, ck=ck, cv=cv)


def gpu_prefill(eng, seqs, table, n_cache=None):
    toks = np.concatenate(seqs).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum([len(s) for s in seqs])]).astype(np.int32)
    eng.prefill_kv(eng.i32(toks), eng.i32(cu), eng.i32(table), None if n_cache is None else eng.i32(n_cache),
                   total_tokens=len(toks), max_seqlen=max(len(s) for s in seqs))


def test_prefill_cache_matches_oracle(world):
    eng, w = world["eng"], world["w"]
    table = H.identity_table(eng, 1)
    gpu_prefill(eng, [world["prompt"]], table)
    assert eng.read_status() == 0
    for l in range(TINY.n_layers):
        for which, ref in ((0, world["ck"][l]), (1, world["cv"][l])):
            got = H.gather_cache(eng, table[0], P, l, which)
            assert np.abs(got - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())


def test_teacher_forced_steps_logits_conf_and_unmask(world):
    eng, w = world["eng"], world["w"]
    table = H.identity_table(eng, 1)
    gpu_prefill(eng, [world["prompt"]], table)
    rec = []
    O.decode(w, world["prompt"], 1, Q, 0.9, 1, record=rec)
    assert len(rec) == 32
    prefix = eng.i32([P]); tab = eng.i32(table)
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    n_exact = 0
    for step, r in enumerate(rec):
        qt = eng.i32(r["before"][None, :])
        if step % 8 == 0:
            logits = eng.debug_logits(qt, prefix, tab, max_prefix_len=P).cpu().numpy()[0]
            assert H.rel_err_rows(logits, r["logits"]).max() <= H.LOGIT_TOL["f32"]
        eng.denoise_step(qt, prefix, tab, cand, conf, ent, max_prefix_len=P)
        masked = r["before"] == TINY.mask_id
        c, cf, en = cand.cpu().numpy()[0], conf.cpu().numpy()[0], ent.cpu().numpy()[0]
        n_exact += H.check_step_outputs(TINY, r, masked, c, cf, en, "f32")
        # rows that are not masked report their own token with confidence 1
        assert (c[~masked] == r["before"][~masked]).all() and (cf[~masked] == 1).all()
        nun = torch.zeros(1, 1, dtype=torch.int32, device=eng.device)
        nrem = torch.zeros(1, 1, dtype=torch.int32, device=eng.device)
        eng.unmask(qt, cand, conf, 0.9, 1, n_unmasked=nun, n_remaining=nrem)
        if H.selection_is_decided(r["conf"], masked, 0.9, 1):
            after = qt.cpu().numpy()[0]
            chosen = np.nonzero(after != r["before"])[0].tolist()
            assert chosen == r["chosen"]
            assert int(nun) == len(chosen) and int(nrem) == masked.sum() - len(chosen)
    assert n_exact > 400
    assert eng.read_status() == 0


def test_teacher_forced_steps_entropy_rule(world):
    """The paper's own selection rule (entropy <= theta, floor by lowest entropy) through dllm_unmask_entropy,
    on the oracle's trajectory under that rule.  Entropies agree to ~1e-5 here, so a step is exempt only if the
    oracle's own selection is within 1e-3 nats of changing."""
    eng, w = world["eng"], world["w"]
    table = H.identity_table(eng, 1)
    gpu_prefill(eng, [world["prompt"]], table)
    prefix = eng.i32([P]); tab = eng.i32(table)
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    # the tiny random model is far from peaked (entropies 5.44 .. 5.47 nats on the first step): theta = 2 leaves
    # the floor to decide every step, theta = 5.443 sits in a gap of the first step's entropies and passes several rows
    for theta, need in ((2.0, 16), (5.443, 1)):
      rec = []
      O.decode(w, world["prompt"], 1, Q, theta, 1, record=rec, rule="entropy")
      assert 1 <= len(rec) <= 32
      checked = multi = 0
      for r in rec:
        qt = eng.i32(r["before"][None, :])
        eng.denoise_step(qt, prefix, tab, cand, conf, ent, max_prefix_len=P)
        masked = r["before"] == TINY.mask_id
        np.testing.assert_allclose(ent.cpu().numpy()[0][masked], r["entropy"][masked], rtol=0, atol=2e-4)
        eng.unmask_entropy(qt, cand, ent, theta, 1)
        # decided: no masked entropy within the margin of theta, floor boundary not a near-tie
        if H.selection_is_decided(-np.asarray(r["entropy"]), masked, -theta, 1):
            after = qt.cpu().numpy()[0]
            assert np.nonzero(after != r["before"])[0].tolist() == r["chosen"]
            assert (after[r["chosen"]] == r["cand"][r["chosen"]]).all()
            checked += 1
            multi += len(r["chosen"]) > 1
      assert checked >= need
      if theta > 5:
          assert multi >= 1
    assert eng.read_status() == 0


def test_free_running_decode_matches_oracle(world):
    """The GPU carries its own state from step to step; it is put back on the oracle's trajectory
    only after a step whose selection the oracle itself leaves within 1e-3 of a tie."""
    eng, w = world["eng"], world["w"]
    table = H.identity_table(eng, 1)
    gpu_prefill(eng, [world["prompt"]], table)
    rec = []
    seq, steps = O.decode(w, world["prompt"], 1, Q, 0.9, 1, record=rec)
    qt = eng.i32(np.full((1, Q), TINY.mask_id))
    prefix = eng.i32([P]); tab = eng.i32(table)
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    nrem = torch.ones(1, 1, dtype=torch.int32, device=eng.device)
    free = 0
    for n, r in enumerate(rec):
        before = qt.cpu().numpy()[0]
        assert (before == r["before"]).all()
        eng.denoise_step(qt, prefix, tab, cand, conf, max_prefix_len=P)
        eng.unmask(qt, cand, conf, 0.9, 1, n_remaining=nrem)
        after = qt.cpu().numpy()[0]
        masked = before == TINY.mask_id
        assert (after[~masked] == before[~masked]).all() and (after != before).sum() >= 1
        assert int(nrem) == (after == TINY.mask_id).sum()
        _, _, _, p = O.confidence(r["logits"], TINY.mask_id)
        sure_ids = (H.top2_margin(p) > H.MARGIN)[r["chosen"]].all()
        if H.selection_is_decided(r["conf"], masked, 0.9, 1) and sure_ids:
            assert (after == r["tokens"]).all()
            free += 1
        else:
            qt = eng.i32(r["tokens"][None])
    assert free >= 4            # the masked rows of this model are nearly alike: most steps are near-ties
    assert int((qt.cpu().numpy()[0] == TINY.mask_id).sum()) == 0


def test_refresh_rewrites_cache_and_cached_step_equals_recompute(world):
    eng, w = world["eng"], world["w"]
    table = H.identity_table(eng, 1)
    blk = synth.masked_block(TINY, 5, Q, 20)
    seq = np.concatenate([world["prompt"], blk])
    full, Ks, Vs, _ = O.forward_full(w, seq)
    # refresh over prompt + in-flight block, committing only the prompt; step outputs for the block
    n_tok = len(seq)
    cand = torch.full((n_tok,), -7, dtype=torch.int32, device=eng.device)
    conf = torch.full((n_tok,), -7.0, dtype=torch.float32, device=eng.device)
    ent = torch.full((n_tok,), -7.0, dtype=torch.float32, device=eng.device)
    eng.refresh_cache(eng.i32(seq), eng.i32([0, n_tok]), eng.i32(table), eng.i32([P]), cand, conf, ent,
                      total_tokens=n_tok, max_seqlen=n_tok)
    for l in range(TINY.n_layers):
        got = H.gather_cache(eng, table[0], P, l, 0)
        assert np.abs(got - Ks[l][:P]).max() <= 1e-5 * max(1.0, np.abs(Ks[l]).max())
        got = H.gather_cache(eng, table[0], P, l, 1)
        assert np.abs(got - Vs[l][:P]).max() <= 1e-5 * max(1.0, np.abs(Vs[l]).max())
    c, cf, en = cand.cpu().numpy(), conf.cpu().numpy(), ent.cpu().numpy()
    assert (c[:P] == -7).all() and (cf[:P] == -7).all()             # committed rows untouched
    r = {"logits": full[P:], "cand": O.confidence(full[P:], TINY.mask_id)[0]}
    H.check_step_outputs(TINY, r, blk == TINY.mask_id, c[P:], cf[P:], en[P:], "f32")
    # now a cached step over the same block sees the same K/V: logits equal the no-cache rows
    logits = eng.debug_logits(eng.i32(blk[None]), eng.i32([P]), eng.i32(table), max_prefix_len=P).cpu().numpy()[0]
    assert H.rel_err_rows(logits, full[P:]).max() <= H.LOGIT_TOL["f32"]
    assert eng.read_status() == 0


def test_batch_of_ragged_sequences_and_page_permutation(world):
    eng, w = world["eng"], world["w"]
    lens = [64, 37, 50]
    seqs = [synth.random_tokens(TINY, 10 + i, n) for i, n in enumerate(lens)]
    blks = [synth.masked_block(TINY, 20 + i, Q, 12 + 4 * i) for i in range(3)]
    rng = np.random.default_rng(0)
    outs = []
    for perm in (None, rng.permutation(eng.cfg.n_pages)):
        table = H.identity_table(eng, 3, perm)
        eng.kv_pool.zero_()
        gpu_prefill(eng, seqs, table)
        lg = eng.debug_logits(eng.i32(np.stack(blks)), eng.i32(lens), eng.i32(table), max_prefix_len=max(lens))
        outs.append(lg.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])                        # physical page order is invisible
    for b in range(3):
        ck, cv = O.prefill(w, seqs[b])
        ref, _ = O.forward_cached(w, blks[b], ck, cv)
        assert H.rel_err_rows(outs[0][b], ref).max() <= H.LOGIT_TOL["f32"]
    assert eng.read_status() == 0


def test_two_blocks_in_flight_with_per_block_floor(world):
    eng, w = world["eng"], world["w"]
    table = H.identity_table(eng, 1)
    gpu_prefill(eng, [world["prompt"]], table)
    blk = synth.masked_block(TINY, 31, 64, 40)
    r = O.denoise_step(w, blk, world["ck"], world["cv"], tau=0.15, m=2, block_len=32)
    qt = eng.i32(blk[None])
    cand = torch.zeros(1, 64, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, 64, dtype=torch.float32, device=eng.device)
    eng.denoise_step(qt, eng.i32([P]), eng.i32(table), cand, conf, max_prefix_len=P)
    masked = blk == TINY.mask_id
    H.check_step_outputs(TINY, r, masked, cand.cpu().numpy()[0], conf.cpu().numpy()[0], None, "f32")
    nun = torch.zeros(1, 2, dtype=torch.int32, device=eng.device)
    eng.unmask(qt, cand, conf, 0.15, 2, block_len=32, n_unmasked=nun)
    decided = all(H.selection_is_decided(r["conf"][s], masked[s], 0.15, 2) for s in (slice(0, 32), slice(32, 64)))
    if decided:
        after = qt.cpu().numpy()[0]
        assert np.nonzero(after != blk)[0].tolist() == r["chosen"]
        assert (after == r["tokens"]).all()
        assert nun.cpu().numpy().sum() == len(r["chosen"])


def test_device_side_bounds_checks_set_status_instead_of_faulting(world):
    eng = world["eng"]
    table = H.identity_table(eng, 1)
    gpu_prefill(eng, [world["prompt"]], table)
    blk = synth.masked_block(TINY, 5, Q, 20)
    bad = blk.copy(); bad[3] = TINY.vocab + 5; bad[4] = -2
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    eng.denoise_step(eng.i32(bad[None]), eng.i32([P]), eng.i32(table), cand, conf, max_prefix_len=P)
    assert eng.read_status() & 1
    eng.reset_status()
    t2 = table.copy(); t2[0, 1] = eng.cfg.n_pages + 3; t2[0, 2] = -1
    eng.denoise_step(eng.i32(blk[None]), eng.i32([P]), eng.i32(t2), cand, conf, max_prefix_len=P)
    assert eng.read_status() & 2
    eng.reset_status()
    assert eng.read_status() == 0


def test_device_side_lengths_are_checked_against_the_host_values(world):
    """Lengths that live in device memory and disagree with the host values that sized the launch (a prefix longer
    than max_prefix_len or negative, a packed sequence longer than max_seqlen, cu_seqlens that do not add up to
    total_tokens or go backwards) are clamped on the device and reported as a status bit; nothing faults, and a
    consistent call afterwards is clean and correct."""
    from paper_2601_07568_amd.binding import STATUS_BAD_LENGTH
    eng = world["eng"]
    table = H.identity_table(eng, 2)
    tab = eng.i32(table)
    seqs = [world["prompt"], synth.random_tokens(TINY, 9, 40)]
    gpu_prefill(eng, seqs, table)
    assert eng.read_status() == 0
    blk = np.stack([synth.masked_block(TINY, 5, Q, 20), synth.masked_block(TINY, 6, Q, 20)])
    cand = torch.zeros(2, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(2, Q, dtype=torch.float32, device=eng.device)
    for bad_prefix in ([P, 1000], [P, -3], [P + 1, 40]):
        eng.denoise_step(eng.i32(blk), eng.i32(bad_prefix), tab, cand, conf, max_prefix_len=max(P, 40))
        assert eng.read_status() & STATUS_BAD_LENGTH, bad_prefix
        eng.reset_status()
    toks = eng.i32(np.concatenate(seqs))
    n = P + 40
    for bad_cu, max_seqlen in (([0, P, n], P - 1),          # a sequence longer than max_seqlen
                               ([0, P, n - 5], P),           # does not add up to total_tokens
                               ([0, P, n + 7], P),           # beyond total_tokens
                               ([0, 70, 50], 70),            # goes backwards
                               ([3, P, n], P)):              # does not start at 0
        eng.prefill_kv(toks, eng.i32(bad_cu), tab, None, total_tokens=n, max_seqlen=max_seqlen)
        assert eng.read_status() & STATUS_BAD_LENGTH, bad_cu
        eng.reset_status()
    # a consistent call afterwards: clean status, cache as the oracle's
    gpu_prefill(eng, seqs, table)
    assert eng.read_status() == 0
    got = H.gather_cache(eng, table[0], P, TINY.n_layers - 1, 0)
    assert np.abs(got - world["ck"][-1]).max() <= 1e-5 * max(1.0, np.abs(world["ck"][-1]).max())


def test_peaked_model_threshold_fires_on_model_confidences():
    """The tiny model with its LM head scaled by 48 instead of 8: the distributions are peaked, so the threshold 0.9
    selects rows on confidences the model itself produced (twelve in the first step, more later) and the floor only
    carries the steps in between.  Two blocks with a refresh at the boundary, teacher-forced (every step from the
    oracle's state: logits, candidates, confidences, the unmask set with its threshold part) and free-running (the GPU
    carries its own state; it is put back on the oracle's trajectory only after a step the oracle leaves within 1e-3
    of a tie)."""
    import dataclasses
    ms = dataclasses.replace(TINY, lm_head_scale=48.0, name="tiny-peaked")
    w = synth.Weights(ms, 0)
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=16, n_pages=16, max_batch=1, max_q=Q, max_tokens=256)
    prompt = synth.random_tokens(ms, 0, P)
    table = H.identity_table(eng, 1)
    tab = eng.i32(table)
    rec = []
    seq, steps = O.decode(w, prompt, 2, Q, 0.9, 1, record=rec)
    by_threshold = [sum(1 for i in r["chosen"] if r["conf"][i] >= 0.9) for r in rec]
    assert sum(1 for n in by_threshold if n >= 2) >= 3 and steps < 2 * Q // 2      # the threshold really drives it
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    nun = torch.zeros(1, 1, dtype=torch.int32, device=eng.device)
    for mode in ("teacher-forced", "free-running"):
        cur = P
        eng.prefill_kv(eng.i32(prompt), eng.i32([0, P]), tab, None, total_tokens=P, max_seqlen=P)
        qt = eng.i32(np.full((1, Q), ms.mask_id))
        decided = thresholded = thr_rows = 0
        n_exact = 0
        for n, r in enumerate(rec):
            if mode == "teacher-forced":
                qt = eng.i32(r["before"][None])
            before = qt.cpu().numpy()[0]
            assert (before == r["before"]).all()
            masked = before == ms.mask_id
            eng.denoise_step(qt, eng.i32([cur]), tab, cand, conf, ent, max_prefix_len=cur)
            c, cf, en = cand.cpu().numpy()[0], conf.cpu().numpy()[0], ent.cpu().numpy()[0]
            if mode == "teacher-forced":
                logits = eng.debug_logits(qt, eng.i32([cur]), tab, max_prefix_len=cur).cpu().numpy()[0]
                assert H.rel_err_rows(logits, r["logits"]).max() <= H.logit_tol("f32", ms.n_layers)
                n_exact += H.check_step_outputs(ms, r, masked, c, cf, en, "f32")
            eng.unmask(qt, cand, conf, 0.9, 1, n_unmasked=nun)
            after = qt.cpu().numpy()[0]
            _, _, _, p = O.confidence(r["logits"], ms.mask_id)
            sure_ids = (H.top2_margin(p) > H.MARGIN)[r["chosen"]].all()
            if mode == "teacher-forced":
                # row by row, whatever the rest of the step: a row clearly above the threshold is decoded to the
                # oracle's token, a row clearly below it is decoded only if the floor could pick it
                top = max(r["conf"][masked]) if masked.any() else 0.0
                for i in np.nonzero(masked)[0]:
                    if r["conf"][i] >= 0.9 + H.MARGIN and H.top2_margin(p)[i] > H.MARGIN:
                        assert after[i] == r["cand"][i], (n, i)
                        thr_rows += 1
                    elif r["conf"][i] <= 0.9 - H.MARGIN and r["conf"][i] < top - H.MARGIN:
                        assert after[i] == ms.mask_id, (n, i)
            if H.selection_is_decided(r["conf"], masked, 0.9, 1) and sure_ids:
                assert (after == r["tokens"]).all(), (mode, n)
                assert int(nun) == len(r["chosen"])
                decided += 1
                thresholded += by_threshold[n] >= 2
            elif mode == "free-running":
                qt = eng.i32(r["tokens"][None])
            if not (r["tokens"] == ms.mask_id).any():                          # block boundary: refresh, next block
                cur += Q
                full = eng.i32(np.concatenate([prompt, seq[P:cur]]))
                eng.refresh_cache(full, eng.i32([0, cur]), tab, None, total_tokens=cur, max_seqlen=cur)
                qt = eng.i32(np.full((1, Q), ms.mask_id))
        print(f"{mode}: {decided} of {len(rec)} steps decided and equal, {thresholded} of them with two or more rows "
              f"taken by the threshold" + (f", {n_exact} rows' candidates decided, {thr_rows} rows decoded by the "
                                           f"threshold alone" if mode == "teacher-forced" else ""))
        assert decided >= (2 * len(rec)) // 3 and thresholded >= 1
        assert mode != "teacher-forced" or thr_rows >= 30
    assert eng.read_status() == 0
    eng.close()
