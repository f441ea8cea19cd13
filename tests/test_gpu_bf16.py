"""GPU parity in bfloat16: a small grouped-query model with ragged shapes (several tiles and tails
in every dimension), and the LLaDA-8B-shaped single layer + LM head at its full size (prefix 512,
block of 32 with 24 masked).  Both kernel selections (automatic and forced generic) are checked."""
import numpy as np
import pytest
import torch

from oracle import dllm_oracle as O
from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
W = synth.as_float
ST = synth.round_bf16
SMALL = synth.ModelShape(2, 512, 8, 2, 128, 1408, 5000, 4999, dtype="bf16", lm_head_scale=8.0, name="small-gqa")
SMALL64 = synth.ModelShape(1, 384, 6, 3, 64, 1000, 3000, 2999, dtype="bf16", lm_head_scale=8.0, name="small-dh64")


def run_small(ms, lens, Q, n_masked, mode, seed=7, mp=8, pt=32):
    w = synth.Weights(ms, seed)
    Bn = len(lens)
    eng = H.make_engine(ms, w, page_tokens=pt, max_pages_per_seq=mp, n_pages=Bn * mp, max_batch=Bn, max_q=Q,
                        max_tokens=sum(lens) + Bn * Q)
    eng.set_kernel_mode(mode)
    seqs = [synth.random_tokens(ms, seed + i, n) for i, n in enumerate(lens)]
    blks = [synth.masked_block(ms, seed + 10 + i, Q, n_masked) for i in range(Bn)]
    table = H.identity_table(eng, Bn)
    toks = np.concatenate(seqs).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(toks), eng.i32(cu), eng.i32(table), None, total_tokens=len(toks), max_seqlen=max(lens))
    qt = eng.i32(np.stack(blks))
    logits = eng.debug_logits(qt, eng.i32(lens), eng.i32(table), max_prefix_len=max(lens)).cpu().numpy()
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(Bn, Q, dtype=torch.float32, device=eng.device)
    eng.denoise_step(qt, eng.i32(lens), eng.i32(table), cand, conf, ent, max_prefix_len=max(lens))
    n_exact = 0
    n_gap = n_rows = 0
    for b in range(Bn):
        ck, cv = O.prefill(w, seqs[b], widen=W)
        for l in range(ms.n_layers):
            for which, ref in ((0, ck[l]), (1, cv[l])):
                got = H.gather_cache(eng, table[b], lens[b], l, which)
                assert np.abs(got - ref).max() <= 2e-2 * np.abs(ref).max()
        exact, _ = O.forward_cached(w, blks[b], ck, cv, widen=W)          # no rounding anywhere
        assert H.rel_err_rows(logits[b], exact).max() <= H.logit_tol("bf16", ms.n_layers)
        # decisions against the exact oracle wherever the logit tolerance leaves no room for another arg max
        g, n, _, _ = H.check_exact_decisions(ms, exact, blks[b] == ms.mask_id, cand.cpu().numpy()[b],
                                             H.logit_tol("bf16", ms.n_layers))
        n_gap, n_rows = n_gap + g, n_rows + n
        ckq, cvq = O.prefill(w, seqs[b], widen=W, store=ST)
        r = O.denoise_step(w, blks[b], ckq, cvq, 0.9, 1, widen=W, store=ST)
        n_exact += H.check_step_outputs(ms, r, blks[b] == ms.mask_id, cand.cpu().numpy()[b],
                                        conf.cpu().numpy()[b], ent.cpu().numpy()[b], "bf16", gpu_logits=logits[b])
    assert eng.read_status() == 0
    print(f"{ms.name}: {n_gap} of {n_rows} masked rows decided against the exact oracle, {n_exact} against the "
          f"oracle with bfloat16 storage")
    assert n_exact >= Bn * n_masked // 2
    # refresh with step outputs for the in-flight rows equals the oracle's no-cache forward
    b = 0
    seq = np.concatenate([seqs[b], blks[b]])
    n_tok = len(seq)
    c2 = torch.zeros(n_tok, dtype=torch.int32, device=eng.device)
    f2 = torch.zeros(n_tok, dtype=torch.float32, device=eng.device)
    eng.refresh_cache(eng.i32(seq), eng.i32([0, n_tok]), eng.i32(table[:1]), eng.i32([lens[b]]), c2, f2,
                      total_tokens=n_tok, max_seqlen=n_tok)
    full, Ks, Vs, _ = O.forward_full(w, seq, widen=W, store=ST)
    rr = {"logits": full[lens[b]:], "cand": O.confidence(full[lens[b]:], ms.mask_id)[0]}
    H.check_step_outputs(ms, rr, blks[b] == ms.mask_id, c2.cpu().numpy()[lens[b]:], f2.cpu().numpy()[lens[b]:],
                         None, "bf16")
    got = H.gather_cache(eng, table[0], lens[b], ms.n_layers - 1, 0)
    assert np.abs(got - Ks[-1][:lens[b]]).max() <= 2e-2 * np.abs(Ks[-1]).max()
    eng.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_small_gqa_model(mode):
    run_small(SMALL, [100, 77], 32, 20, mode)


@pytest.mark.parametrize("mode", [0, 1])
def test_small_head_dim_64_model(mode):
    run_small(SMALL64, [45, 130, 64], 64, 40, mode)


def test_small_model_256_query_rows_and_long_prefill():
    """Four sequences x 64 query rows and a 539-token prefill: the 256-row tiles of the large GEMM path with
    ragged feature counts (1000 MLP features, 3000 vocabulary entries) and a ragged last row tile."""
    run_small(SMALL64, [45, 130, 64, 300], 64, 40, 0, mp=12)


@pytest.mark.parametrize("pt,mp", [(24, 8), (8, 24), (128, 2)])
def test_small_gqa_model_other_page_sizes(pt, mp):
    """Page sizes that are not a power of two (the staged attention does not take them), the smallest one (a
    64-key block spans eight pages) and one larger than a block."""
    run_small(SMALL, [100, 77], 32, 20, 0, mp=mp, pt=pt)


WIDE_MLP = synth.ModelShape(1, 320, 5, 5, 64, 8192, 2000, 1999, dtype="bf16", lm_head_scale=8.0, name="wide-mlp")


def test_wide_mlp_narrow_model_on_256_row_tiles():
    """d_model 320 with an 8192-wide MLP and a 300-token prefill: the down projection takes the 256-row tiles with a
    long K and a ragged feature count (320 = one and a quarter tiles), its K sum split and folded by the next norm."""
    run_small(WIDE_MLP, [300, 41], 32, 20, 0, mp=12)


@pytest.mark.parametrize("Q,n_masked", [(32, 24), (48, 30), (64, 40), (128, 70)])
def test_llada_shaped_layer_and_head_full_size(Q, n_masked):
    """Workload: one LLaDA-8B-shaped layer + LM head over vocab 126464, batch 1, prefix 512, block 32
    (24 masked), threshold 0.9, floor 1 -- all rows checked against the oracle.  Also with 48, 64 and 128 query
    rows (more blocks in flight): the weight-streaming kernels with three and four row tiles, and the streaming
    tiles that take over above 64 rows."""
    ms = synth.LLADA_8B.with_layers(1)
    P = 512
    w = synth.Weights(ms, 2)
    eng = H.make_engine(ms, w, page_tokens=64, max_pages_per_seq=10, n_pages=10, max_batch=1, max_q=Q, max_tokens=P)
    prompt = synth.random_tokens(ms, 2, P)
    blk = synth.masked_block(ms, 2, Q, n_masked)
    table = H.identity_table(eng, 1)
    eng.prefill_kv(eng.i32(prompt), eng.i32([0, P]), eng.i32(table), None, total_tokens=P, max_seqlen=P)
    qt = eng.i32(blk[None])
    cand = torch.zeros(1, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(1, Q, dtype=torch.float32, device=eng.device)
    eng.denoise_step(qt, eng.i32([P]), eng.i32(table), cand, conf, ent, max_prefix_len=P)
    logits = eng.debug_logits(qt, eng.i32([P]), eng.i32(table), max_prefix_len=P).cpu().numpy()[0]
    ck, cv = O.prefill(w, prompt, widen=W)
    exact, _ = O.forward_cached(w, blk, ck, cv, widen=W)
    assert H.rel_err_rows(logits, exact).max() <= H.logit_tol("bf16", 1)
    n_gap, n_rows, _, _ = H.check_exact_decisions(ms, exact, blk == ms.mask_id, cand.cpu().numpy()[0],
                                                  H.logit_tol("bf16", 1))
    print(f"{n_gap} of {n_rows} masked rows decided against the exact oracle")
    ck, cv = O.prefill(w, prompt, widen=W, store=ST)
    r = O.denoise_step(w, blk, ck, cv, 0.9, 1, widen=W, store=ST)
    print("logit rel err vs exact oracle", H.rel_err_rows(logits, exact).max(), "vs bf16-storage oracle",
          H.rel_err_rows(logits, r["logits"]).max())
    masked = blk == ms.mask_id
    H.check_step_outputs(ms, r, masked, cand.cpu().numpy()[0], conf.cpu().numpy()[0], ent.cpu().numpy()[0], "bf16",
                         gpu_logits=logits)
    eng.unmask(qt, cand, conf, 0.9, 1)
    if H.selection_is_decided(r["conf"], masked, 0.9, 1):
        assert np.nonzero(qt.cpu().numpy()[0] != blk)[0].tolist() == r["chosen"]
    assert eng.read_status() == 0
    eng.close()


@pytest.mark.parametrize("Bn,Q", [(1, 32), (4, 64)])
def test_degenerate_steps_nothing_masked_and_empty_prefix(Bn, Q):
    """A step whose block holds no [MASK] (the LM head has no rows to do) and a step over an empty prefix (the block
    attends to itself only), on the small-row and on the 256-row path."""
    ms = SMALL64
    w = synth.Weights(ms, 9)
    eng = H.make_engine(ms, w, page_tokens=32, max_pages_per_seq=4, n_pages=4 * Bn, max_batch=Bn, max_q=Q,
                        max_tokens=Bn * Q)
    table = H.identity_table(eng, Bn)
    tab = eng.i32(table)
    cand = torch.full((Bn, Q), -7, dtype=torch.int32, device=eng.device)
    conf = torch.full((Bn, Q), -7.0, dtype=torch.float32, device=eng.device)
    ent = torch.full((Bn, Q), -7.0, dtype=torch.float32, device=eng.device)
    # empty prefix, nothing masked
    blk = np.stack([synth.random_tokens(ms, 20 + b, Q) for b in range(Bn)]).astype(np.int32)
    eng.denoise_step(eng.i32(blk), eng.i32([0] * Bn), tab, cand, conf, ent, max_prefix_len=0)
    assert (cand.cpu().numpy() == blk).all() and (conf.cpu().numpy() == 1).all()
    # empty prefix, some masked: equals the oracle's no-cache forward over the block alone
    blks = np.stack([synth.masked_block(ms, 30 + b, Q, Q // 2) for b in range(Bn)]).astype(np.int32)
    eng.denoise_step(eng.i32(blks), eng.i32([0] * Bn), tab, cand, conf, ent, max_prefix_len=0)
    logits = eng.debug_logits(eng.i32(blks), eng.i32([0] * Bn), tab, max_prefix_len=0).cpu().numpy()
    for b in range(Bn):
        exact, _, _, _ = O.forward_full(w, blks[b], widen=W)
        assert H.rel_err_rows(logits[b], exact).max() <= H.logit_tol("bf16", ms.n_layers)
        H.check_exact_decisions(ms, exact, blks[b] == ms.mask_id, cand.cpu().numpy()[b], H.logit_tol("bf16", ms.n_layers))
        full, _, _, _ = O.forward_full(w, blks[b], widen=W, store=ST)
        r = {"logits": full, "cand": O.confidence(full, ms.mask_id)[0]}
        H.check_step_outputs(ms, r, blks[b] == ms.mask_id, cand.cpu().numpy()[b], conf.cpu().numpy()[b],
                             ent.cpu().numpy()[b], "bf16", gpu_logits=logits[b])
    assert eng.read_status() == 0
    eng.close()


@pytest.mark.parametrize("lens,qvalid", [([70], [32]), ([100, 77, 45, 130], [64, 32, 0, 33])])
def test_step_with_padding_rows(lens, qvalid):
    """dllm_denoise_step_var: rows past q_valid[b] are padding.  The valid rows must equal the oracle's step over the
    valid rows alone, padding rows report their own token, and nothing is written to the cache behind the valid rows
    (one sequence on the <= 64-row kernels, four on the large path)."""
    ms, Q = SMALL, 64
    w = synth.Weights(ms, 7)
    Bn = len(lens)
    eng = H.make_engine(ms, w, page_tokens=32, max_pages_per_seq=8, n_pages=8 * Bn, max_batch=Bn, max_q=Q,
                        max_tokens=sum(lens) + Bn * Q)
    seqs = [synth.random_tokens(ms, 40 + i, n) for i, n in enumerate(lens)]
    table = H.identity_table(eng, Bn)
    tab = eng.i32(table)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(seqs)), eng.i32(cu), tab, None, total_tokens=int(cu[-1]), max_seqlen=max(lens))
    blks = np.stack([synth.masked_block(ms, 60 + b, Q, 30) for b in range(Bn)]).astype(np.int32)
    for b in range(Bn):
        blks[b, qvalid[b]:] = ms.mask_id if b % 2 else 11          # padding content must not matter, masks included
    # sentinel K/V behind every sequence's valid rows
    for l in range(ms.n_layers):
        for which in (0, 1):
            slab = eng.kv_slab(l, which)
            for b in range(Bn):
                for p in range(lens[b] + qvalid[b], lens[b] + Q):
                    slab[int(table[b][p // 32]), :, p % 32, :] = 3.0
    cand = torch.zeros(Bn, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(Bn, Q, dtype=torch.float32, device=eng.device)
    ent = torch.zeros(Bn, Q, dtype=torch.float32, device=eng.device)
    eng.denoise_step_var(eng.i32(blks), eng.i32(lens), eng.i32(qvalid), tab, cand, conf, ent, max_prefix_len=max(lens))
    assert eng.read_status() == 0
    c, f, e = cand.cpu().numpy(), conf.cpu().numpy(), ent.cpu().numpy()
    for b in range(Bn):
        nv = qvalid[b]
        assert (c[b, nv:] == blks[b, nv:]).all() and (f[b, nv:] == 1).all()
        for l in range(ms.n_layers):
            for which in (0, 1):
                got = H.gather_cache(eng, table[b], lens[b] + Q, l, which)
                assert (got[lens[b] + nv:] == 3.0).all()              # nothing written behind the valid rows
        if nv == 0:
            continue
        ck, cv = O.prefill(w, seqs[b], widen=W, store=ST)
        r = O.denoise_step(w, blks[b, :nv], ck, cv, 0.9, 1, widen=W, store=ST)
        n_exact = H.check_step_outputs(ms, r, blks[b, :nv] == ms.mask_id, c[b, :nv], f[b, :nv], e[b, :nv], "bf16")
        assert n_exact >= 1
    eng.close()


@pytest.mark.parametrize("lens,extra", [([70, 0, 55], 40), ([0, 0, 0], 96), ([130, 90, 60], 17)])
def test_refresh_with_a_device_resident_total_equals_the_sized_call(lens, extra):
    """dllm_refresh_cache_dev takes a token buffer that is larger than the packed batch (its capacity sizes the
    launches, cu_seqlens[B] says where the batch ends, sequences may be empty): the cache it writes and the step
    outputs of the real rows are those of dllm_refresh_cache called with the exact sizes; an empty batch changes
    nothing.  (Capacity and total stay within the same tile class of the GEMMs, so the results are bit-identical.)"""
    ms = SMALL
    w = synth.Weights(ms, 21)
    Bn = len(lens)
    total = sum(lens)
    cap = total + extra
    eng = H.make_engine(ms, w, page_tokens=32, max_pages_per_seq=8, n_pages=Bn * 8, max_batch=Bn, max_q=64,
                        max_tokens=cap)
    table = eng.i32(H.identity_table(eng, Bn))
    seqs = [synth.random_tokens(ms, 30 + b, n) for b, n in enumerate(lens)]
    for s in seqs:                                              # the last 16 positions of a sequence are in flight
        s[-16::2] = ms.mask_id
    ncommit = eng.i32([max(n - 16, 0) for n in lens])
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    packed = np.concatenate(seqs + [np.zeros(0, dtype=np.int64)]).astype(np.int32)
    dev = eng.device
    pool0 = eng.kv_pool.clone()

    def outs(n):
        return (torch.full((n,), -7, dtype=torch.int32, device=dev), torch.full((n,), -7.0, device=dev),
                torch.full((n,), -7.0, device=dev))

    want = None
    if total > 0:
        c1, f1, e1 = outs(total)
        eng.refresh_cache(eng.i32(packed), eng.i32(cu), table, ncommit, c1, f1, e1, total_tokens=total,
                          max_seqlen=max(lens))
        want = (eng.kv_pool.clone(), c1, f1, e1)
        eng.kv_pool.copy_(pool0)
    buf = np.full(cap, 3, dtype=np.int32)                      # rows behind the batch: any valid token
    buf[:total] = packed
    c2, f2, e2 = outs(cap)
    eng.refresh_cache_dev(eng.i32(buf), eng.i32(cu), table, ncommit, c2, f2, e2, max_seqlen=max(max(lens), 1))
    torch.cuda.synchronize()
    assert eng.read_status() == 0
    if total == 0:
        assert torch.equal(eng.kv_pool, pool0)
        assert int((c2 != -7).sum()) == 0                       # no row is a sequence's: nothing reported
    else:
        assert torch.equal(eng.kv_pool, want[0])
        assert torch.equal(c2[:total], want[1]) and torch.equal(f2[:total], want[2]) and torch.equal(e2[:total], want[3])
        assert int((c2[total:] != -7).sum()) == 0 and int((c2[:total] != -7).sum()) > 0
    eng.close()


@pytest.mark.parametrize("ms,Q,pt", [(SMALL64, 32, 32), (SMALL, 32, 64), (SMALL, 64, 64), (SMALL, 64, 16)],
                         ids=["register-direct", "staged-4-waves", "staged-8-waves", "staged-small-pages"])
def test_page_ids_out_of_range_in_the_matrix_core_attention(ms, Q, pt):
    """A block table with page ids that address no page (too large, negative) in one sequence, on every bfloat16
    attention kernel: the status bit is raised, nothing faults (the kernels check every id before they address the
    pool with it), the sequence with the clean table gets bit for bit what it gets without the bad neighbour, and the
    bad sequence's outputs are finite."""
    from paper_2601_07568_amd.binding import STATUS_BAD_PAGE
    lens = [150, 200]
    mp = (max(lens) + Q + pt - 1) // pt + 1
    w = synth.Weights(ms, 9)
    eng = H.make_engine(ms, w, page_tokens=pt, max_pages_per_seq=mp, n_pages=2 * mp, max_batch=2, max_q=Q,
                        max_tokens=sum(lens) + 2 * Q)
    table = H.identity_table(eng, 2)
    seqs = [synth.random_tokens(ms, 40 + i, n) for i, n in enumerate(lens)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(seqs)), eng.i32(cu), eng.i32(table), None, total_tokens=int(cu[-1]),
                   max_seqlen=max(lens))
    qt = eng.i32(np.stack([synth.masked_block(ms, 60 + i, Q, Q // 2) for i in range(2)]))
    dev = eng.device

    def step(tab):
        c = torch.zeros(2, Q, dtype=torch.int32, device=dev)
        f = torch.zeros(2, Q, dtype=torch.float32, device=dev)
        e = torch.zeros(2, Q, dtype=torch.float32, device=dev)
        pool = eng.kv_pool.clone()                      # a step writes its rows' K/V: same starting cache for both runs
        eng.denoise_step(qt.clone(), eng.i32(lens), eng.i32(tab), c, f, e, max_prefix_len=max(lens))
        torch.cuda.synchronize()
        eng.kv_pool.copy_(pool)
        return c.cpu().numpy(), f.cpu().numpy(), e.cpu().numpy()

    clean = step(table)
    assert eng.read_status() == 0
    bad = table.copy()
    bad[1, 1] = 2 * mp + 7                               # past the pool
    bad[1, 2] = -1
    got = step(bad)
    assert eng.read_status() & STATUS_BAD_PAGE
    eng.reset_status()
    for g, c in zip(got, clean):
        assert (g[0] == c[0]).all()
        assert np.isfinite(g[1].astype(np.float64)).all()
    again = step(table)                                  # and a clean call afterwards is clean
    assert eng.read_status() == 0
    for g, c in zip(again, clean):
        assert (g == c).all()
    eng.close()
