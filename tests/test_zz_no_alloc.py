"""The denoise step for callers that cannot allocate (dllm_denoise_step_static): same kernels as
dllm_denoise_step with the intermediates in the library's own device array.  Checked through the C ABI against
dllm_denoise_step itself on the same inputs, bit for bit (outputs and the K/V the step writes), on two calls in a
row of which the second is smaller, and for the status bits it merges into the context."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2601_07568_amd import binding as B
from paper_2601_07568_amd import synth
from tests import harness as H

pytestmark = pytest.mark.gpu
SMALL = synth.ModelShape(2, 512, 8, 2, 128, 1408, 5000, 4999, dtype="bf16", lm_head_scale=8.0, name="small-gqa")


def both_steps(eng, blks, lens, table):
    """(cand, conf, entropy, pool bytes) of the workspace call and of the static-scratch call on the same inputs."""
    out = []
    Bn, Q = blks.shape
    pool0 = eng.kv_pool.clone()
    for fn in (eng.denoise_step, eng.denoise_step_static):
        eng.kv_pool.copy_(pool0)
        cand = torch.full((Bn, Q), -3, dtype=torch.int32, device=eng.device)
        conf = torch.full((Bn, Q), -3.0, dtype=torch.float32, device=eng.device)
        ent = torch.full((Bn, Q), -3.0, dtype=torch.float32, device=eng.device)
        fn(eng.i32(blks), eng.i32(lens), eng.i32(table), cand, conf, ent, max_prefix_len=max(lens))
        out.append((cand.cpu().numpy(), conf.cpu().numpy(), ent.cpu().numpy(), eng.kv_pool.cpu().numpy().copy()))
    return out


@pytest.mark.parametrize("ms,seed", [(SMALL, 7), (synth.TINY, 0)])
def test_static_scratch_step_equals_workspace_step_twice_second_smaller(ms, seed):
    w = synth.Weights(ms, seed)
    lens, Q = [100, 77], 32
    eng = H.make_engine(ms, w, page_tokens=32, max_pages_per_seq=8, n_pages=16, max_batch=2, max_q=Q,
                        max_tokens=sum(lens))
    assert B.lib().dllm_workspace_bytes(C.byref(eng.cfg)) <= B.lib().dllm_static_scratch_bytes()
    table = H.identity_table(eng, 2)
    seqs = [synth.random_tokens(ms, seed + i, n) for i, n in enumerate(lens)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    eng.prefill_kv(eng.i32(np.concatenate(seqs)), eng.i32(cu), eng.i32(table), None, total_tokens=int(cu[-1]),
                   max_seqlen=max(lens))
    blks = np.stack([synth.masked_block(ms, seed + 10 + i, Q, 20) for i in range(2)]).astype(np.int32)
    # first call: two sequences of 32 rows; second call: one sequence of 16 rows (the array still holds the first's data)
    for bl, ln, tb in ((blks, lens, table), (blks[1:, :16].copy(), lens[1:], table[1:])):
        a, b = both_steps(eng, bl, ln, tb)
        masked = bl == ms.mask_id
        assert masked.any() and (a[0][masked] != -3).all() and (a[0][masked] != ms.mask_id).all()
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    assert eng.read_status() == 0
    # a token id outside the vocabulary inside the static call shows up in the context's status word
    bad = blks.copy()
    bad[0, 3] = ms.vocab + 5
    cand = torch.zeros(2, Q, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(2, Q, dtype=torch.float32, device=eng.device)
    eng.denoise_step_static(eng.i32(bad), eng.i32(lens), eng.i32(table), cand, conf, None, max_prefix_len=max(lens))
    assert eng.read_status() & B.STATUS_BAD_TOKEN
    eng.reset_status()
    # and the next good call is clean again (the array's own status word is cleared by every call)
    eng.denoise_step_static(eng.i32(blks), eng.i32(lens), eng.i32(table), cand, conf, None, max_prefix_len=max(lens))
    assert eng.read_status() == 0
    eng.close()


def test_static_scratch_step_rejects_a_context_that_does_not_fit():
    ms = synth.TINY
    w = synth.Weights(ms, 0)
    eng = H.make_engine(ms, w, page_tokens=16, max_pages_per_seq=16, n_pages=16, max_batch=1, max_q=32,
                        max_tokens=16384)
    assert B.lib().dllm_workspace_bytes(C.byref(eng.cfg)) > B.lib().dllm_static_scratch_bytes()
    qt = eng.i32(synth.masked_block(ms, 1, 32, 8)[None])
    cand = torch.zeros(1, 32, dtype=torch.int32, device=eng.device)
    conf = torch.zeros(1, 32, dtype=torch.float32, device=eng.device)
    with pytest.raises(B.DllmError) as e:
        eng.denoise_step_static(qt, eng.i32([0]), eng.i32(H.identity_table(eng, 1)), cand, conf, None, max_prefix_len=0)
    assert e.value.code == B.DLLM_ENOSPACE
    eng.close()
