"""dllm_unmask alone against the oracle's selection on synthetic confidences (exact ties, NaN-free),
single and multiple blocks, all thresholds and floors."""
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
