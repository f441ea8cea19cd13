"""Multi-block decoding (Section 3.2): the device-side block state machine and the per-block selection against
the oracle on synthetic inputs (bit-exact), and whole multi-block decodes of the tiny workload round by round."""
import numpy as np
import pytest
import torch

from oracle import dllm_oracle as O
from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
TINY = synth.TINY
P, BL = 64, 32


@pytest.fixture(scope="module")
def eng():
    return H.make_engine(TINY, synth.Weights(TINY, 0), page_tokens=16, max_pages_per_seq=16, n_pages=32, max_batch=2,
                         max_q=128, max_tokens=512)


@pytest.mark.parametrize("block_len,n_blocks", [(32, 4), (4, 9), (7, 3), (100, 2)])
def test_fsm_update_matches_oracle_on_random_states(eng, block_len, n_blocks):
    rng = np.random.default_rng(block_len * 100 + n_blocks)
    mask = TINY.mask_id
    for trial in range(40):
        Bn = 3
        add_at, full_at = [(0.1, 0.95), (0.25, 0.75), (1.0, 1.0), (0.5, 0.5), (0.0, 0.3)][trial % 5]
        delay, nocache = int(rng.integers(0, 3)), bool(rng.integers(0, 2))
        state = rng.integers(0, 5, (Bn, n_blocks)).astype(np.int32)
        counter = rng.integers(0, 3, (Bn, n_blocks)).astype(np.int32)
        gen = rng.integers(0, 4000, (Bn, n_blocks * block_len)).astype(np.int32)
        for b in range(Bn):
            for k in range(n_blocks):
                # fill levels around the thresholds, plus empty and full blocks
                n_filled = int(rng.choice([0, 1, int(0.1 * block_len), int(np.ceil(0.1 * block_len)),
                                           int(0.95 * block_len), int(np.ceil(0.95 * block_len)), block_len - 1,
                                           block_len, int(rng.integers(0, block_len + 1))]))
                idx = rng.permutation(block_len)[:block_len - n_filled]
                gen[b, k * block_len + idx] = mask
        d_state, d_counter = eng.i32(state), eng.i32(counter)
        floor = torch.zeros(Bn, n_blocks, dtype=torch.int32, device=eng.device)
        summ = torch.zeros(Bn, 4, dtype=torch.int32, device=eng.device)
        eng.fsm_update(eng.i32(gen), d_state, d_counter, block_len, add_at, full_at, delay, nocache, floor, summ)
        gs, gc, gf, gsum = (t.cpu().numpy() for t in (d_state, d_counter, floor, summ))
        for b in range(Bn):
            filled = [int((gen[b, k * block_len:(k + 1) * block_len] != mask).sum()) for k in range(n_blocks)]
            rs, rc = O.fsm_update(state[b].tolist(), counter[b].tolist(), filled, block_len, add_at, full_at, delay,
                                  nocache)
            assert gs[b].tolist() == rs and gc[b].tolist() == rc
            act = [k for k, s in enumerate(rs) if s in (O.ACTIVATED, O.FULLY_ACTIVATED)]
            assert gf[b].tolist() == [1 if s == O.FULLY_ACTIVATED else 0 if s == O.ACTIVATED else -1 for s in rs]
            assert gsum[b].tolist() == [act[0] if act else -1, act[-1] if act else -1, int(O.STABILIZING in rs),
                                        sum(s == O.COMPLETED for s in rs)]


@pytest.mark.parametrize("by_entropy", [False, True])
def test_unmask_blocks_floor_per_block(eng, by_entropy):
    ms = eng.ms
    rng = np.random.default_rng(31 + by_entropy)
    Bn, nblk, bl = 2, 4, 32
    for trial in range(8):
        tokens = np.where(rng.random((Bn, nblk * bl)) < 0.6, ms.mask_id, rng.integers(0, 4000, (Bn, nblk * bl))).astype(np.int32)
        stat = (rng.choice([0.0, 0.2, 0.45, 0.5, 0.9, 3.0], size=tokens.shape) if trial % 2 else rng.random(tokens.shape) * 2).astype(np.float32)
        cand = rng.integers(0, 4000, tokens.shape).astype(np.int32)
        floor = rng.choice([-1, 0, 1, 3], size=(Bn, nblk)).astype(np.int32)
        thr = float(rng.choice([0.45, 0.9, -1.0, 5.0]))
        qt = eng.i32(tokens)
        nun = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
        nrem = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
        eng.unmask_blocks(qt, eng.i32(cand), torch.from_numpy(stat).to(eng.device), thr, eng.i32(floor), by_entropy, bl,
                          nun, nrem)
        got = qt.cpu().numpy()
        for b in range(Bn):
            for k in range(nblk):
                sl = slice(k * bl, (k + 1) * bl)
                n_masked = int((tokens[b, sl] == ms.mask_id).sum())
                if floor[b, k] < 0:
                    assert (got[b, sl] == tokens[b, sl]).all() and int(nun[b, k]) == 0 and int(nrem[b, k]) == n_masked
                    continue
                f = O.unmask_entropy if by_entropy else O.unmask
                ref, ch = f(tokens[b, sl], cand[b, sl], stat[b, sl], ms.mask_id, np.float32(thr), int(floor[b, k]))
                assert (got[b, sl] == ref).all()
                assert int(nun[b, k]) == len(ch) and int(nrem[b, k]) == n_masked - len(ch)


def decided(rec_round, thr, rule, block_len):
    """The oracle's selection of this round is not within the margin of changing, in any active block."""
    st = rec_round["state"]
    for b, s in enumerate(st):
        if s not in (O.ACTIVATED, O.FULLY_ACTIVATED):
            continue
        off = (b - rec_round["lo"]) * block_len
        sl = slice(b * block_len, (b + 1) * block_len)
        masked = rec_round["before"][sl] == TINY.mask_id
        floor = 1 if s == O.FULLY_ACTIVATED else 0
        stat = rec_round["entropy" if rule == "entropy" else "conf"][off:off + block_len]
        sgn = -1.0 if rule == "entropy" else 1.0
        c = (sgn * np.asarray(stat))[masked]
        if len(c) == 0:
            continue
        if (np.abs(c - sgn * thr) <= H.MARGIN).any():
            return False
        srt = np.sort(c)[::-1]
        if 0 < floor < len(c) and srt[floor - 1] - srt[floor] <= H.MARGIN:
            return False
    return True


@pytest.mark.parametrize("thr,rule,delay,n_blocks,refresh_every",
                         [(5.443, "entropy", 1, 3, 0), (2.0, "entropy", 2, 2, 0), (0.9, "prob", 1, 2, 0),
                          (5.443, "entropy", 1, 2, 3)])
def test_multiblock_decode_round_by_round(eng, thr, rule, delay, n_blocks, refresh_every):
    """Every round of the oracle's multi-block decode is replayed on the GPU from the oracle's state: the forward the
    state machine asks for (cached step over the window, or a forward without cache that also rewrites it), the
    per-block selection with the floors of the block states, and the transitions."""
    w = synth.Weights(TINY, 0)
    prompt = synth.random_tokens(TINY, 0, P)
    rec = []
    seq, rounds = O.decode_multiblock(w, prompt, n_blocks, BL, thr, rule, delay=delay, record=rec,
                                      refresh_every=refresh_every)
    assert rounds == len(rec) and any(r["nocache"] for r in rec) and any(r["hi"] > r["lo"] for r in rec)
    if refresh_every:                  # the periodic refresh fires on rounds that have no stabilizing block
        assert any(r["nocache"] and O.STABILIZING not in r["state"] for r in rec)
    # the plan of every next round on the device (dllm_fsm_plan), driven by the oracle's states
    d_since = torch.zeros(1, dtype=torch.int32, device=eng.device)
    d_nocache = torch.zeros(1, dtype=torch.int32, device=eng.device)
    d_commit = torch.zeros(1, dtype=torch.int32, device=eng.device)
    table = H.identity_table(eng, 1)
    tab = eng.i32(table)
    # the cache the GPU holds follows the same schedule: prompt first, then rewritten by each no-cache round
    eng.prefill_kv(eng.i32(prompt), eng.i32([0, P]), tab, None, total_tokens=P, max_seqlen=P)
    checked = 0
    for ri, r in enumerate(rec):
        lo, hi, st = r["lo"], r["hi"], r["state"]
        nw = hi - lo + 1
        gen = r["before"]
        window = gen[lo * BL:(hi + 1) * BL]
        Q = nw * BL
        cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
        conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
        ent = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
        if r["nocache"]:
            n_tok = P + (hi + 1) * BL
            full = np.concatenate([prompt, gen[:(hi + 1) * BL]])
            done_after = sum(s == O.COMPLETED for s in r["state_after"])
            assert P + done_after * BL == r["n_cached"]
            if ri:
                assert int(d_commit) == r["n_cached"]             # what the device planned for this round
            c2 = torch.zeros(n_tok, dtype=torch.int32, device=eng.device)
            f2 = torch.zeros(n_tok, dtype=torch.float32, device=eng.device)
            e2 = torch.zeros(n_tok, dtype=torch.float32, device=eng.device)
            eng.refresh_cache(eng.i32(full), eng.i32([0, n_tok]), tab, eng.i32([P + done_after * BL]), c2, f2, e2,
                              total_tokens=n_tok, max_seqlen=n_tok)
            s0 = P + lo * BL
            cand[0], conf[0], ent[0] = c2[s0:], f2[s0:], e2[s0:]
        else:
            assert all(s == O.COMPLETED for s in st[:lo])
            eng.denoise_step(eng.i32(window[None, :]), eng.i32([P + lo * BL]), tab, cand, conf, ent,
                             max_prefix_len=P + lo * BL)
        # plan of the next round from this round's outcome (the oracle's states, so that no near-tie exempts it)
        eng.fsm_plan(eng.i32(np.array([r["state_after"]], dtype=np.int32)), eng.i32(np.array([r["counter_after"]], dtype=np.int32)),
                     eng.i32([P]), BL, refresh_every, d_since, d_nocache, d_commit)
        if ri + 1 < len(rec):
            assert bool(int(d_nocache)) == rec[ri + 1]["nocache"], (ri, int(d_nocache), int(d_since))
        masked = window == TINY.mask_id
        np.testing.assert_allclose(ent.cpu().numpy()[0][masked], r["entropy"][masked], rtol=0, atol=5e-4)
        # floors from the device state machine's own output for this state (a zero-effect update: no tokens changed)
        d_state = eng.i32(np.array([st], dtype=np.int32))
        floors = eng.i32(np.array([[1 if s == O.FULLY_ACTIVATED else 0 if s == O.ACTIVATED else -1 for s in st[lo:hi + 1]]],
                                  dtype=np.int32))
        qt = eng.i32(window[None, :])
        eng.unmask_blocks(qt, cand, ent if rule == "entropy" else conf, thr, floors, rule == "entropy", BL)
        if not decided(r, thr, rule, BL):
            continue
        after = qt.cpu().numpy()[0]
        chosen = [lo * BL + int(i) for i in np.nonzero(after != window)[0]]
        assert chosen == r["chosen"]
        new_gen = gen.copy()
        new_gen[lo * BL:(hi + 1) * BL] = after
        d_counter = eng.i32(np.array([rec[ri - 1]["counter_after"] if ri else [0] * n_blocks], dtype=np.int32))
        summ = torch.zeros(1, 4, dtype=torch.int32, device=eng.device)
        eng.fsm_update(eng.i32(new_gen[None, :]), d_state, d_counter, BL, 0.1, 0.95, delay, r["nocache"], None, summ)
        assert d_state.cpu().numpy()[0].tolist() == r["state_after"]
        assert d_counter.cpu().numpy()[0].tolist() == r["counter_after"]
        checked += 1
    # the tiny random model's confidences sit within 1e-3 of each other far more often than its entropies
    assert checked >= max(1, len(rec) // (3 if rule == "entropy" else 8))
    assert eng.read_status() == 0


def test_unmask_traced_records_the_teacher_order(eng):
    """One token per step through dllm_unmask_traced on synthetic confidences: the recorded order equals the oracle's
    replay of the same selections, and noisy sequences built from it on the device equal the oracle's."""
    ms = eng.ms
    rng = np.random.default_rng(77)
    Bn, nblk, bl = 2, 3, 8
    n = nblk * bl
    order = torch.zeros(Bn, n, dtype=torch.int32, device=eng.device)
    ref_order = np.zeros((Bn, n), dtype=np.int64)
    tokens = np.full((Bn, n), ms.mask_id, dtype=np.int32)
    qt = eng.i32(tokens)
    step = 0
    for blk in range(nblk):                                     # blocks in sequence, one position per step
        for _ in range(bl):
            step += 1
            conf = rng.random((Bn, n)).astype(np.float32)
            cand = rng.integers(0, 4000, (Bn, n)).astype(np.int32)
            sl = slice(blk * bl, (blk + 1) * bl)
            view = qt[:, sl].contiguous()
            ov = order[:, sl].contiguous()
            eng.unmask_traced(view, eng.i32(cand[:, sl]), torch.from_numpy(conf[:, sl].copy()).to(eng.device), 2.0, 1,
                              step, ov)
            qt[:, sl] = view
            order[:, sl] = ov
            for b in range(Bn):
                new, ch = O.unmask(tokens[b, sl], cand[b, sl], conf[b, sl], ms.mask_id, np.float32(2.0), 1)
                tokens[b, sl] = new
                (i,) = ch
                ref_order[b, blk * bl + i] = step
    assert (qt.cpu().numpy() == tokens).all()
    got_order = order.cpu().numpy()
    assert (got_order == ref_order).all()
    for b in range(Bn):
        assert sorted(got_order[b].tolist()) == list(range(1, n + 1))
    y = rng.integers(0, 4000, (Bn, n)).astype(np.int32)
    out = torch.zeros(Bn, n, dtype=torch.int32, device=eng.device)
    for s_list, k, t in (([4, 9], 8, 0.5), ([0, 0], n, 0.25), ([8, 16], 8, 1.0), ([3, 20], 5, 0.0), ([0, 23], 1, 0.7)):
        eng.noisy_sequence(eng.i32(y), order, eng.i32(s_list), k, t, out)
        got = out.cpu().numpy()
        for b in range(Bn):
            assert (got[b] == O.noisy_sequence(y[b], ref_order[b], s_list[b], k, t, ms.mask_id)).all()


def test_eos_scan_and_active_list(eng):
    ms = eng.ms
    rng = np.random.default_rng(5)
    eos = 17
    for Bn, n in ((1, 32), (7, 100), (130, 64), (64, 1)):
        gen = rng.integers(0, 40, (Bn, n)).astype(np.int32)          # small alphabet: EOS shows up often
        gen[rng.random((Bn, n)) < 0.1] = ms.mask_id
        if Bn > 3:
            gen[2, :] = 3                                             # no EOS, no mask
            gen[3, 0] = eos
        fin = torch.zeros(Bn, dtype=torch.int32, device=eng.device)
        first = torch.zeros(Bn, dtype=torch.int32, device=eng.device)
        act = torch.zeros(Bn, dtype=torch.int32, device=eng.device)
        nact = torch.zeros(1, dtype=torch.int32, device=eng.device)
        eng.eos_scan(eng.i32(gen), eos, fin, first, act, nact)
        ref = [O.eos_state(gen[b].tolist(), eos, ms.mask_id) for b in range(Bn)]
        assert fin.cpu().numpy().tolist() == [int(f) for f, _ in ref]
        assert first.cpu().numpy().tolist() == [p for _, p in ref]
        alive = [b for b in range(Bn) if not ref[b][0]]
        assert int(nact) == len(alive)
        assert act.cpu().numpy().tolist() == alive + [-1] * (Bn - len(alive))


def test_batched_multiblock_rounds_with_ragged_windows():
    """Three sequences (different prompts and prompt lengths) decoded with the state machine at once: every cached
    round is ONE dllm_denoise_step_var call over per-sequence windows built on the device (dllm_fsm_window), one
    dllm_unmask_blocks, one dllm_fsm_scatter and one dllm_fsm_update (forward type derived per sequence); sequences
    whose round must not use the cache get an empty window there and their own refresh call.  Every round starts from
    the oracle's per-sequence state and is compared with it."""
    ms = TINY
    w = synth.Weights(ms, 0)
    NB, Wn, thr, delay = 3, 3, 5.443, 1
    lens = [64, 40, 57]
    Bn = len(lens)
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=12, n_pages=12 * Bn, max_batch=Bn, max_q=Wn * BL,
                        max_tokens=512)
    prompts = [synth.random_tokens(ms, 50 + b, lens[b]) for b in range(Bn)]
    recs = []
    for b in range(Bn):
        rec = []
        O.decode_multiblock(w, prompts[b], NB, BL, thr, "entropy", delay=delay, record=rec)
        recs.append(rec)
    table = H.identity_table(eng, Bn)
    tab = eng.i32(table)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(prompts)), eng.i32(cu), tab, None, total_tokens=int(cu[-1]), max_seqlen=max(lens))
    dev = eng.device
    Q = Wn * BL
    win = torch.zeros(Bn, Q, dtype=torch.int32, device=dev)
    wfl = torch.zeros(Bn, Wn, dtype=torch.int32, device=dev)
    pre = torch.zeros(Bn, dtype=torch.int32, device=dev)
    qv = torch.zeros(Bn, dtype=torch.int32, device=dev)
    wlo = torch.zeros(Bn, dtype=torch.int32, device=dev)
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=dev)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)
    ent = torch.zeros(Bn, Q, dtype=torch.float32, device=dev)
    base = eng.i32(lens)
    done_state = [O.COMPLETED] * NB
    checked = batched_wide = 0
    for rnd in range(max(len(r) for r in recs)):
        live = [b for b in range(Bn) if rnd < len(recs[b])]
        gen_np = np.zeros((Bn, NB * BL), dtype=np.int32)
        st_np = np.zeros((Bn, NB), dtype=np.int32)
        ct_np = np.zeros((Bn, NB), dtype=np.int32)
        for b in range(Bn):
            if b in live:
                r = recs[b][rnd]
                gen_np[b], st_np[b] = r["before"], r["state"]
                ct_np[b] = recs[b][rnd - 1]["counter_after"] if rnd else [0] * NB
            else:                                               # finished: whatever it ended with, all blocks done
                gen_np[b], st_np[b] = recs[b][-1]["before"], done_state
        gen, state, counter = eng.i32(gen_np), eng.i32(st_np), eng.i32(ct_np)
        eng.fsm_window(gen, state, base, BL, Wn, 0, win, wfl, pre, qv, wlo)
        qv_np, pre_np, lo_np = qv.cpu().numpy(), pre.cpu().numpy(), wlo.cpu().numpy()
        for b in range(Bn):
            cached = b in live and not recs[b][rnd]["nocache"]
            if cached:
                r = recs[b][rnd]
                assert qv_np[b] == (r["hi"] - r["lo"] + 1) * BL and lo_np[b] == r["lo"] and pre_np[b] == lens[b] + r["lo"] * BL
            else:
                assert qv_np[b] == 0 and (wfl.cpu().numpy()[b] == -1).all()
        # sequences whose round does not use the cache: their own forward (keeps their caches on the oracle's schedule)
        for b in live:
            r = recs[b][rnd]
            if not r["nocache"]:
                continue
            n_tok = lens[b] + (r["hi"] + 1) * BL
            full = np.concatenate([prompts[b], r["before"][:(r["hi"] + 1) * BL]])
            done_after = sum(s == O.COMPLETED for s in r["state_after"])
            eng.refresh_cache(eng.i32(full), eng.i32([0, n_tok]), eng.i32(table[b:b + 1]),
                              eng.i32([lens[b] + done_after * BL]), None, None, None, total_tokens=n_tok, max_seqlen=n_tok)
        if int(qv_np.max()) > 0:
            eng.denoise_step_var(win, pre, qv, tab, cand, conf, ent, max_prefix_len=int(pre_np.max()))
            eng.unmask_blocks(win, cand, ent, thr, wfl, True, BL)
            eng.fsm_scatter(win, wlo, qv, gen, NB, BL, Wn)
            batched_wide += int((qv_np > 0).sum()) > 1
        eng.fsm_update(gen, state, counter, BL, 0.1, 0.95, delay, None, None, None)
        got_gen, got_state, got_ct = gen.cpu().numpy(), state.cpu().numpy(), counter.cpu().numpy()
        for b in range(Bn):
            if b not in live:
                assert (got_gen[b] == gen_np[b]).all() and got_state[b].tolist() == done_state
                continue
            r = recs[b][rnd]
            if r["nocache"]:
                assert (got_gen[b] == gen_np[b]).all()          # untouched by the batched calls
                continue
            masked = r["before"][r["lo"] * BL:(r["hi"] + 1) * BL] == ms.mask_id
            np.testing.assert_allclose(ent.cpu().numpy()[b][:len(masked)][masked], r["entropy"][masked], rtol=0, atol=5e-4,
                                       err_msg=f"round {rnd} seq {b} window {r['lo']}..{r['hi']} qv {qv_np.tolist()} pre {pre_np.tolist()}")
            if not decided(r, thr, "entropy", BL):
                continue
            assert np.nonzero(got_gen[b] != gen_np[b])[0].tolist() == r["chosen"]
            assert got_state[b].tolist() == r["state_after"] and got_ct[b].tolist() == r["counter_after"]
            checked += 1
    assert checked >= 6 and batched_wide >= 2
    assert eng.read_status() == 0
    eng.close()


@pytest.mark.parametrize("ms_name,Bn,Q", [("tiny", 3, 16), ("small", 2, 32), ("small", 4, 32), ("small", 10, 32)])
def test_early_stop_compaction_and_step_over_the_live_sequences(ms_name, Bn, Q):
    """Section 3.2, early stopping: dllm_eos_scan lists the live sequences, dllm_gather_rows brings their tokens,
    prefix lengths and block-table rows to the front, dllm_denoise_step_live runs the step over the live count (a
    device value; B stays the launch size), dllm_scatter_rows puts the results back.  Against the oracle: the live
    list and the compacted arrays bit for bit, the step of every live sequence as its own oracle step, and for the
    finished ones nothing: own tokens reported, nothing written to their cache.  Batches of 2 (at most 64 rows), 4
    (128 rows) and 10 sequences (320 rows) take the three GEMM forms of a bfloat16 step."""
    from tests.test_gpu_bf16 import SMALL
    ms = TINY if ms_name == "tiny" else SMALL
    dtype = "f32" if ms_name == "tiny" else "bf16"
    W, ST = (None, None) if dtype == "f32" else (synth.as_float, synth.round_bf16)
    w = synth.Weights(ms, 3)
    rng = np.random.default_rng(11)
    lens = [int(x) for x in rng.integers(20, 60, Bn)]
    mp, pt = 8, 16
    eng = H.make_engine(ms, w, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q,
                        max_tokens=sum(lens))
    prompts = [synth.random_tokens(ms, 70 + b, lens[b]) for b in range(Bn)]
    table = H.identity_table(eng, Bn)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(prompts)), eng.i32(cu), eng.i32(table), None, total_tokens=int(cu[-1]),
                   max_seqlen=max(lens))
    eos = 5
    gen = np.stack([synth.masked_block(ms, 80 + b, Q, Q // 2) for b in range(Bn)]).astype(np.int32)
    gen[gen == eos] = 6
    finished_want = [b for b in range(Bn) if b % 3 == 1]
    for b in finished_want:                              # an EOS with nothing masked before it
        gen[b, :3] = [11, 12, eos]
    live = O.live_sequences(gen, eos, ms.mask_id)
    assert live == [b for b in range(Bn) if b not in finished_want] and 0 < len(live) < Bn
    dev = eng.device
    fin = torch.zeros(Bn, dtype=torch.int32, device=dev)
    act = torch.zeros(Bn, dtype=torch.int32, device=dev)
    nact = torch.zeros(1, dtype=torch.int32, device=dev)
    eng.eos_scan(eng.i32(gen), eos, fin, None, act, nact)
    assert int(nact) == len(live) and act.cpu().numpy()[:len(live)].tolist() == live
    # compaction on the device == the oracle's
    g_gen, g_len, g_tab = eng.i32(gen), eng.i32(np.array(lens)[:, None]), eng.i32(table)
    c_gen, c_len, c_tab = torch.zeros_like(g_gen), torch.zeros_like(g_len), torch.zeros_like(g_tab)
    eng.gather_rows(act, nact, g_gen, c_gen, 7)
    eng.gather_rows(act, nact, g_len, c_len, 0)
    eng.gather_rows(act, nact, g_tab, c_tab, -1)
    assert (c_gen.cpu().numpy() == O.gather_rows(gen, live, 7)).all()
    assert (c_len.cpu().numpy() == O.gather_rows(np.array(lens)[:, None], live, 0)).all()
    assert (c_tab.cpu().numpy() == O.gather_rows(table, live, -1)).all()
    # sentinel K/V in the in-flight positions of every sequence: only live ones may be overwritten
    for l in range(ms.n_layers):
        for which in (0, 1):
            slab = eng.kv_slab(l, which)
            for b in range(Bn):
                for p in range(lens[b], lens[b] + Q):
                    slab[int(table[b][p // pt]), :, p % pt, :] = 3.0
    cand = torch.full((Bn, Q), -5, dtype=torch.int32, device=dev)
    conf = torch.full((Bn, Q), -5.0, dtype=torch.float32, device=dev)
    ent = torch.full((Bn, Q), -5.0, dtype=torch.float32, device=dev)
    eng.denoise_step_live(c_gen, c_len.view(-1), None, nact, c_tab, cand, conf, ent, max_prefix_len=max(lens))
    assert eng.read_status() == 0
    c, f, e = cand.cpu().numpy(), conf.cpu().numpy(), ent.cpu().numpy()
    n_dec = 0
    for i, b in enumerate(live):
        ck, cv = O.prefill(w, prompts[b], widen=W, store=ST)
        r = O.denoise_step(w, gen[b], ck, cv, 0.9, 1, widen=W, store=ST)
        n_dec += H.check_step_outputs(ms, r, gen[b] == ms.mask_id, c[i], f[i], e[i], dtype)
        got = H.gather_cache(eng, table[b], lens[b] + Q, ms.n_layers - 1, 0)
        assert not (got[lens[b]:] == 3.0).all()                      # the live sequence's rows were cached
    assert n_dec >= len(live) * Q // 8
    for i in range(len(live), Bn):                                     # rows past the live count: filled tokens reported
        assert (c[i] == 7).all() and (f[i] == 1).all()
    for b in finished_want:
        for l in range(ms.n_layers):
            for which in (0, 1):
                got = H.gather_cache(eng, table[b], lens[b] + Q, l, which)
                assert (got[lens[b]:] == 3.0).all()                    # nothing of a finished sequence was touched
    # unmask on the compacted batch, then back to the original order
    eng.unmask(c_gen, cand, conf, 0.9, 1)
    back = eng.i32(gen)
    eng.scatter_rows(act, nact, c_gen, back)
    want = gen.copy()
    for i, b in enumerate(live):
        want[b] = c_gen.cpu().numpy()[i]
    assert (back.cpu().numpy() == want).all()
    for b in finished_want:
        assert (back.cpu().numpy()[b] == gen[b]).all()
    eng.close()


class RoundBuffers:
    """Device state of a batch under multi-block decoding and the scratch of one round; nothing in here is read by the
    host while rounds run."""

    def __init__(self, eng, ms, prompts, NB, Wn, cap):
        dev = eng.device
        Bn = len(prompts)
        lens = [len(p) for p in prompts]
        self.Bn, self.NB, self.Wn, self.Q, self.cap = Bn, NB, Wn, Wn * BL, cap
        self.max_seqlen = max(lens) + NB * BL
        pt = np.zeros((Bn, max(lens)), dtype=np.int32)
        for b, p in enumerate(prompts):
            pt[b, :lens[b]] = p
        self.prompts = eng.i32(pt)
        self.base = eng.i32(lens)
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        self.gen = torch.full((Bn, NB * BL), ms.mask_id, **i32)
        self.state = torch.zeros(Bn, NB, **i32)
        self.state[:, 0] = O.FULLY_ACTIVATED
        self.counter = torch.zeros(Bn, NB, **i32)
        self.since, self.nocache, self.plan_commit = (torch.zeros(Bn, **i32) for _ in range(3))
        self.win, self.wfl = torch.zeros(Bn, self.Q, **i32), torch.zeros(Bn, Wn, **i32)
        self.pre, self.qv, self.qvc, self.wlo = (torch.zeros(Bn, **i32) for _ in range(4))
        self.cand, self.conf, self.ent = torch.zeros(Bn, self.Q, **i32), torch.zeros(Bn, self.Q, **f32), torch.zeros(Bn, self.Q, **f32)
        self.ptok, self.cu, self.ncommit = torch.zeros(cap, **i32), torch.zeros(Bn + 1, **i32), torch.zeros(Bn, **i32)
        self.c2, self.f2, self.e2 = torch.zeros(cap, **i32), torch.zeros(cap, **f32), torch.zeros(cap, **f32)


def device_round(eng, rb, table, thr, delay, refresh_every):
    """One round of multi-block decoding of a batch as a fixed sequence of calls: no value comes back to the host."""
    eng.fsm_round_windows(rb.gen, rb.state, rb.base, rb.nocache, BL, rb.Wn, 0, rb.win, rb.wfl, rb.pre, rb.qv, rb.qvc, rb.wlo)
    eng.denoise_step_var(rb.win, rb.pre, rb.qvc, table, rb.cand, rb.conf, rb.ent, max_prefix_len=rb.max_seqlen)
    eng.fsm_pack(rb.prompts, rb.gen, rb.state, rb.base, rb.nocache, rb.plan_commit, BL, rb.Wn, 0, rb.ptok, rb.cu,
                 rb.ncommit, max_seqlen=rb.max_seqlen)
    eng.refresh_cache_dev(rb.ptok, rb.cu, table, rb.ncommit, rb.c2, rb.f2, rb.e2, max_seqlen=rb.max_seqlen)
    eng.fsm_unpack(rb.cu, rb.pre, rb.qv, rb.nocache, rb.c2, rb.f2, rb.e2, rb.cand, rb.conf, rb.ent)
    eng.unmask_blocks(rb.win, rb.cand, rb.ent, thr, rb.wfl, True, BL)
    eng.fsm_scatter(rb.win, rb.wlo, rb.qv, rb.gen, rb.NB, BL, rb.Wn)
    eng.fsm_update(rb.gen, rb.state, rb.counter, BL, 0.1, 0.95, delay, None, None, None)
    eng.fsm_plan(rb.state, rb.counter, rb.base, BL, refresh_every, rb.since, rb.nocache, rb.plan_commit)


@pytest.mark.parametrize("refresh_every", [0, 3])
def test_whole_multiblock_decode_of_a_batch_without_host_reads(refresh_every):
    """Three sequences decoded to the end by one fixed sequence of calls per round: the plan on the device sends each
    sequence through the cached step or through the packed forward without cache (whose total is device-resident), the
    host reads nothing until the last round is enqueued.  Snapshots taken on the device after every round are then held
    against the oracle's rounds, sequence by sequence, for as long as the two agree; they may part only on a round whose
    selection was a near-tie in the oracle."""
    ms = TINY
    w = synth.Weights(ms, 0)
    NB, Wn, thr, delay = 3, 3, 5.443, 1
    lens = [64, 40, 57]
    Bn = len(lens)
    cap = sum(lens) + Bn * NB * BL
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=12, n_pages=12 * Bn, max_batch=Bn, max_q=Wn * BL,
                        max_tokens=cap)
    prompts = [synth.random_tokens(ms, 50 + b, lens[b]) for b in range(Bn)]
    recs, finals = [], []
    for b in range(Bn):
        rec = []
        seq, _ = O.decode_multiblock(w, prompts[b], NB, BL, thr, "entropy", delay=delay, record=rec,
                                     refresh_every=refresh_every)
        recs.append(rec)
        finals.append(seq[lens[b]:])
    tab = eng.i32(H.identity_table(eng, Bn))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(prompts)), eng.i32(cu), tab, None, total_tokens=int(cu[-1]), max_seqlen=max(lens))
    rb = RoundBuffers(eng, ms, prompts, NB, Wn, cap)
    n_rounds = max(len(r) for r in recs) + 2
    snaps = []
    for _ in range(n_rounds):
        flag = rb.nocache.clone()                      # forward type of the round about to run (device copy, no read)
        device_round(eng, rb, tab, thr, delay, refresh_every)
        snaps.append((flag, rb.gen.clone(), rb.state.clone(), rb.cu.clone()))
    assert eng.read_status() == 0                      # the first host read
    snaps = [tuple(t.cpu().numpy() for t in s) for s in snaps]
    compared = mixed = nocache_seen = 0
    for b in range(Bn):
        rec = recs[b]
        for rnd, r in enumerate(rec):
            flag, gen, state, cu_d = snaps[rnd]
            assert bool(flag[b]) == r["nocache"], (b, rnd)
            n_packed = int(cu_d[b + 1] - cu_d[b])
            assert n_packed == (lens[b] + (r["hi"] + 1) * BL if r["nocache"] else 0)
            after = rec[rnd + 1]["before"] if rnd + 1 < len(rec) else finals[b]
            if not (gen[b] == after).all():
                # only a near-tie of the oracle's selection may go the other way; the trajectories part here
                assert not decided(r, thr, "entropy", BL), (b, rnd, np.nonzero(gen[b] != r["before"])[0].tolist(), r["chosen"])
                break
            assert state[b].tolist() == r["state_after"]
            compared += 1
            nocache_seen += r["nocache"]
            others = [flag[o] for o in range(Bn) if o != b and rnd < len(recs[o])]
            mixed += bool(r["nocache"] and others and not all(others))
        else:
            # in step with the oracle to the end: the same text, and the rounds after the last one changed nothing
            assert (snaps[-1][1][b] == finals[b]).all()
    assert compared >= 12 and nocache_seen >= 2 and mixed >= 1, (compared, nocache_seen, mixed)
    eng.close()
