"""dllm_unmask alone against the oracle's selection on synthetic confidences (exact ties; NaN values in a test of
their own), single and multiple blocks, all thresholds and floors."""
import numpy as np
import pytest
import torch

from oracle import dllm_oracle as O
from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def eng():
    ms = synth.TINY.with_layers(0)
    return H.make_engine(ms, synth.Weights(ms, 0), max_batch=4, max_q=64)


@pytest.mark.parametrize("block_len,nblk", [(32, 1), (32, 2), (64, 1), (16, 4), (7, 3), (200, 2)])
def test_unmask_matches_oracle(eng, block_len, nblk):
    ms = eng.ms
    rng = np.random.default_rng(block_len * 10 + nblk)
    Bn, Qn = 3, block_len * nblk
    for trial in range(6):
        tokens = np.where(rng.random((Bn, Qn)) < 0.6, ms.mask_id, rng.integers(0, 4000, (Bn, Qn))).astype(np.int32)
        if trial == 0:
            tokens[0, :block_len] = 5                                     # a block with nothing masked
        conf = (rng.choice([0.1, 0.5, 0.85, 0.9, 0.95], size=(Bn, Qn)) if trial % 2
                else rng.random((Bn, Qn))).astype(np.float32)
        cand = rng.integers(0, 4000, (Bn, Qn)).astype(np.int32)
        for tau, m in ((0.9, 1), (0.85, 2), (1.5, 1), (0.0, 1), (0.5, 5), (0.95, 300)):
            qt = eng.i32(tokens)
            nun = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
            nrem = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
            eng.unmask(qt, eng.i32(cand), torch.from_numpy(conf).to(eng.device), tau, m, block_len=block_len,
                       n_unmasked=nun, n_remaining=nrem)
            got = qt.cpu().numpy()
            for b in range(Bn):
                for k in range(nblk):
                    sl = slice(k * block_len, (k + 1) * block_len)
                    ref, ch = O.unmask(tokens[b, sl], cand[b, sl], conf[b, sl], ms.mask_id, np.float32(tau), m)
                    assert (got[b, sl] == ref).all()
                    assert int(nun[b, k]) == len(ch)
                    assert int(nrem[b, k]) == int((tokens[b, sl] == ms.mask_id).sum()) - len(ch)


@pytest.mark.parametrize("block_len,nblk", [(32, 1), (32, 2), (16, 4), (7, 3), (200, 2)])
def test_unmask_entropy_matches_oracle(eng, block_len, nblk):
    """dllm_unmask_entropy against the oracle's entropy-threshold selection, exact ties included, floors from 0
    (threshold only) up to more than the block holds."""
    ms = eng.ms
    rng = np.random.default_rng(7000 + block_len * 10 + nblk)
    Bn, Qn = 3, block_len * nblk
    for trial in range(6):
        tokens = np.where(rng.random((Bn, Qn)) < 0.6, ms.mask_id, rng.integers(0, 4000, (Bn, Qn))).astype(np.int32)
        if trial == 0:
            tokens[0, :block_len] = 5
        ent = (rng.choice([0.0, 0.2, 0.4, 0.45, 0.5, 3.0], size=(Bn, Qn)) if trial % 2
               else rng.random((Bn, Qn)) * 2).astype(np.float32)
        cand = rng.integers(0, 4000, (Bn, Qn)).astype(np.int32)
        for theta, m in ((0.45, 1), (0.4, 0), (0.5, 2), (-1.0, 1), (100.0, 0), (0.2, 5), (0.0, 300)):
            qt = eng.i32(tokens)
            nun = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
            nrem = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
            eng.unmask_entropy(qt, eng.i32(cand), torch.from_numpy(ent).to(eng.device), theta, m, block_len=block_len,
                               n_unmasked=nun, n_remaining=nrem)
            got = qt.cpu().numpy()
            for b in range(Bn):
                for k in range(nblk):
                    sl = slice(k * block_len, (k + 1) * block_len)
                    ref, ch = O.unmask_entropy(tokens[b, sl], cand[b, sl], ent[b, sl], ms.mask_id, np.float32(theta), m)
                    assert (got[b, sl] == ref).all()
                    assert int(nun[b, k]) == len(ch)
                    assert int(nrem[b, k]) == int((tokens[b, sl] == ms.mask_id).sum()) - len(ch)


def test_threshold_only_floor_zero(eng):
    """min_unmask = 0 (the conservative strategy of a newly activated block): nothing below the threshold moves."""
    ms = eng.ms
    tokens = np.full((1, 32), ms.mask_id, dtype=np.int32)
    conf = np.linspace(0.1, 0.8, 32, dtype=np.float32)[None]
    cand = np.arange(32, dtype=np.int32)[None]
    qt = eng.i32(tokens)
    eng.unmask(qt, eng.i32(cand), torch.from_numpy(conf).to(eng.device), 0.9, 0)
    assert (qt.cpu().numpy() == tokens).all()
    ref, ch = O.unmask(tokens[0], cand[0], conf[0], ms.mask_id, np.float32(0.5), 0)
    eng.unmask(qt, eng.i32(cand), torch.from_numpy(conf).to(eng.device), 0.5, 0)
    assert (qt.cpu().numpy()[0] == ref).all() and len(ch) > 0


@pytest.mark.parametrize("by_entropy", [False, True])
def test_nan_statistics_pass_no_threshold_and_rank_last(eng, by_entropy):
    """NaN confidences / entropies: never selected by the threshold, taken by the floor only after every number
    (lowest index first) - the same sets as the oracle, on blocks where a third of the values are NaN and on a block
    that holds nothing but NaN."""
    ms = eng.ms
    rng = np.random.default_rng(99 + by_entropy)
    Bn, bl, nblk = 3, 32, 2
    Qn = bl * nblk
    for trial in range(4):
        tokens = np.where(rng.random((Bn, Qn)) < 0.7, ms.mask_id, rng.integers(0, 4000, (Bn, Qn))).astype(np.int32)
        stat = rng.random((Bn, Qn)).astype(np.float32)
        stat[rng.random((Bn, Qn)) < 0.35] = np.nan
        stat[0, :bl] = np.nan
        cand = rng.integers(0, 4000, (Bn, Qn)).astype(np.int32)
        for thr, m in ((0.5, 1), (0.5, 0), (0.2, 7), (2.0, 40), (-1.0, 3)):
            qt = eng.i32(tokens)
            nun = torch.zeros(Bn, nblk, dtype=torch.int32, device=eng.device)
            fn = eng.unmask_entropy if by_entropy else eng.unmask
            fn(qt, eng.i32(cand), torch.from_numpy(stat).to(eng.device), thr, m, block_len=bl, n_unmasked=nun)
            got = qt.cpu().numpy()
            for b in range(Bn):
                for k in range(nblk):
                    sl = slice(k * bl, (k + 1) * bl)
                    ofn = O.unmask_entropy if by_entropy else O.unmask
                    ref, ch = ofn(tokens[b, sl], cand[b, sl], stat[b, sl], ms.mask_id, np.float32(thr), m)
                    assert (got[b, sl] == ref).all(), (trial, thr, m, b, k)
                    assert int(nun[b, k]) == len(ch)
