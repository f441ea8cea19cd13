"""Shared helpers of the GPU parity tests: engine set-up from the seeded generator, block tables,
and the comparison rules (per-row max-norm relative error of logits; token ids and unmask sets
exact except where the oracle itself is within 1e-3 of a tie or of the threshold)."""
from __future__ import annotations

import numpy as np

from oracle import dllm_oracle as O
from paper_2601_07568_amd import synth

MARGIN = 1e-3          # top-2 probability margin below which a token id may differ
LOGIT_TOL = {"f32": 1e-4, "bf16": 2e-2}


def logit_tol(dtype, n_layers, against="exact"):
    """Per-row max-norm relative logit tolerance by model depth: fixed numbers.

    float: 1e-4 at any depth.  bfloat16: 2e-2 is the tolerance of a slice of up to two layers + head.  Every layer
    rounds five activations to bfloat16, and the logit error of a random-weight model grows like the square root
    of the depth (measured against the exact oracle: 1.0e-2 at one layer, 1.6-2.0e-2 at four, 4.6e-2 at 32;
    against the oracle that rounds where the library rounds: 0.4e-2, 0.9e-2, 2.3e-2), so deeper models get
    2.5e-2 (up to 4 layers) and 6e-2 (up to 32) against the exact oracle, and 2e-2 / 3e-2 against the oracle
    with bfloat16 storage."""
    if dtype == "f32":
        return 1e-4
    if against == "exact":
        return 2e-2 if n_layers <= 2 else (2.5e-2 if n_layers <= 4 else 6e-2)
    return 2e-2 if n_layers <= 4 else 3e-2


def make_engine(ms, weights, **kw):
    from paper_2601_07568_amd.binding import Engine
    return Engine(ms, weights, **kw)


def identity_table(eng, B, perm=None):
    """Block table [B, max_pages_per_seq]: sequence b owns pages b*mp .. (b+1)*mp-1 (optionally
    sent through a permutation of the physical pages)."""
    mp = eng.cfg.max_pages_per_seq
    t = np.arange(B * mp, dtype=np.int32).reshape(B, mp)
    assert B * mp <= eng.cfg.n_pages
    if perm is not None:
        t = np.asarray(perm, dtype=np.int32)[t]
    return t


def rel_err_rows(got, ref):
    """max_v |got - ref| / max(max_v |ref|, 1e-6), per row."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.abs(got - ref).max(axis=-1) / np.maximum(np.abs(ref).max(axis=-1), 1e-6)


def top2_margin(p):
    s = np.sort(p, axis=-1)
    return s[:, -1] - s[:, -2]


def gather_cache(eng, table_row, n, layer, which):
    """Positions 0..n-1 of one sequence out of the paged pool -> numpy [n, Hkv, dh] float32."""
    slab = eng.kv_slab(layer, which).float().cpu().numpy()      # [pages, Hkv, pt, dh] (K), V transposed
    pt = eng.cfg.page_tokens
    out = np.empty((n, slab.shape[1], slab.shape[3]), dtype=np.float32)
    for j in range(n):
        out[j] = slab[table_row[j // pt], :, j % pt, :]
    return out


def gather_cache_rows(eng, table_row, n, layer, which):
    """As gather_cache, page by page on the device (for long prefixes)."""
    import torch
    slab = eng.kv_slab(layer, which)                            # [pages, Hkv, pt, dh] view
    pt = eng.cfg.page_tokens
    n_pages = (n + pt - 1) // pt
    idx = torch.as_tensor(np.asarray(table_row[:n_pages]), device=slab.device, dtype=torch.long)
    rows = slab[idx].permute(0, 2, 1, 3).reshape(n_pages * pt, slab.shape[1], slab.shape[3])[:n]
    return rows.float().cpu().numpy()


STORE = {"f32": None, "bf16": synth.round_bf16}     # storage precision of the decisions, per dtype


def check_step_outputs(ms, r, masked, cand, conf, ent, dtype, gpu_logits=None, eps=None):
    """GPU cand/conf/entropy of the masked rows against an oracle step record r (r comes from the
    oracle run in the model's storage precision, so that both sides decide in the same precision).

    Token ids must agree wherever the oracle's top-2 logit gap exceeds twice the logit tolerance (then any
    logits within tolerance have the same arg max).  float: also wherever its top-2 probability margin exceeds
    1e-3 (with a logit tolerance of 1e-4 such a margin is always a gap far above the tolerance).  bfloat16: a
    margin of 1e-3 on a flat distribution (p_max = 0.15: a logit gap of 0.008) lies inside the logit tolerance
    itself (0.02 * max|z| = 0.2), so agreement on such rows cannot be required row by row; they are counted,
    and at least nine in ten of them must agree.

    Tolerances follow from the logit tolerance eps (relative to the row's largest |z|): with
    delta = eps * max|z|, log(conf) = z_max - lse moves by at most 2*delta, and to first order the
    entropy moves by at most delta * sum_v p_v |z_v - mean_p z| (a factor 1.5 covers the rest)."""
    z = np.asarray(r["logits"], dtype=np.float64)
    _, oconf, oent, p = O.confidence(z, ms.mask_id)
    margin = top2_margin(p)
    eps = LOGIT_TOL[dtype] if eps is None else eps
    zz = np.delete(z, ms.mask_id, axis=1)
    pp = np.delete(p, ms.mask_id, axis=1)
    delta = eps * np.abs(z).max(axis=-1)
    spread = (pp * np.abs(zz - (pp * zz).sum(-1, keepdims=True))).sum(-1)
    n_exact = n_margin = n_margin_ok = 0
    zs = np.sort(zz, axis=-1)
    gap = zs[:, -1] - zs[:, -2]
    for i in np.nonzero(masked)[0]:
        if gap[i] > 2 * delta[i] or (dtype == "f32" and margin[i] > MARGIN):
            assert cand[i] == r["cand"][i], (i, cand[i], r["cand"][i], margin[i], gap[i], delta[i])
            n_exact += 1
        elif margin[i] > MARGIN:
            n_margin += 1
            n_margin_ok += int(cand[i] == r["cand"][i])
        assert abs(np.log(conf[i] / oconf[i])) <= 2 * delta[i] + 1e-6, (i, conf[i], oconf[i], delta[i])
        if ent is not None:
            assert abs(ent[i] - oent[i]) <= 1.5 * delta[i] * spread[i] + 1e-5, (i, ent[i], oent[i])
    assert n_margin_ok * 10 >= n_margin * 9, (n_margin_ok, n_margin)
    n_exact += n_margin_ok
    if gpu_logits is not None:
        # property of the fused epilogue: its outputs are the softmax statistics of the logits the
        # same forward materialises through the debug hook
        g = np.array(gpu_logits, dtype=np.float64)
        g[:, ms.mask_id] = -np.inf
        gm = g.max(-1)
        gl = gm + np.log(np.exp(g - gm[:, None]).sum(-1))
        gconf = np.exp(gm - gl)
        srt = np.sort(g, axis=-1)
        for i in np.nonzero(masked)[0]:
            assert abs(conf[i] / gconf[i] - 1) <= 2e-3, (i, conf[i], gconf[i])
            if srt[i, -1] - srt[i, -2] > 1e-3 * max(1.0, abs(srt[i, -1])):
                assert cand[i] == int(np.argmax(g[i])), (i, cand[i], int(np.argmax(g[i])))
    return n_exact


def check_exact_decisions(ms, exact_logits, masked, cand, eps):
    """Token ids against the EXACT oracle (float64, no rounding anywhere): wherever its top-2 logit gap exceeds
    2 * eps * max|z| every set of logits within the tolerance eps has the same arg max, so the library's candidate
    must be the exact oracle's.  Returns (rows decided that way, masked rows, masked rows whose top-2 probability
    margin exceeds 1e-3 and how many of those agree) for the test to report; only the first rule is asserted, a
    margin above 1e-3 with a logit gap inside the logit tolerance does not fix the arg max."""
    z = np.array(exact_logits, dtype=np.float64, copy=True)
    ocand, _, _, p = O.confidence(z, ms.mask_id)
    delta = eps * np.abs(z).max(axis=-1)
    z[:, ms.mask_id] = -np.inf
    zs = np.sort(z, axis=-1)
    gap = zs[:, -1] - zs[:, -2]
    margin = top2_margin(p)
    rows = np.nonzero(masked)[0]
    n_gap = n_margin = n_margin_ok = 0
    for i in rows:
        if gap[i] > 2 * delta[i]:
            assert cand[i] == ocand[i], ("exact oracle", i, cand[i], ocand[i], gap[i], delta[i], margin[i])
            n_gap += 1
        if margin[i] > MARGIN:
            n_margin += 1
            n_margin_ok += int(cand[i] == ocand[i])
    return n_gap, len(rows), n_margin, n_margin_ok


def selection_is_decided(conf, masked, tau, m):
    """True if the oracle's unmask set is not within MARGIN of changing: no masked confidence within
    MARGIN of tau, and the m'-th and (m'+1)-th confidences differ by more than MARGIN."""
    c = np.asarray(conf)[np.asarray(masked)]
    if len(c) == 0:
        return True
    if (np.abs(c - tau) <= MARGIN).any():
        return False
    mm = min(m, len(c))
    s = np.sort(c)[::-1]
    if mm < len(c) and s[mm - 1] - s[mm] <= MARGIN:
        return False
    return True


def layerwise_oracle_step(ms, g, layers, prompt, blk, caches=None):
    """The oracle on a model whose weights live on the device (too large to hold on the host in float64 all at
    once): layer by layer, a layer's weights are on the host only while it is used.  Runs the no-cache forward over
    `prompt` (its K/V are the cache: what dllm_prefill_kv computes) and the denoise-step forward of the block `blk`
    against that cache, both exactly and with bfloat16 storage at the library's rounding points.  With `caches`
    (per layer (K, V) float64 arrays) the prompt pass is skipped and those are the cache.
    Returns {"exact": logits, "stored": logits, "k_last": last layer's prompt K of the storage variant}."""
    import torch
    host = lambda t: t.float().cpu().numpy().astype(np.float64)
    ident = lambda a: a
    dev = g["tok_emb"].device
    Q = len(blk)
    P = len(prompt) if caches is None else caches[0][0].shape[0]
    emb = lambda toks: host(g["tok_emb"][torch.from_numpy(np.asarray(toks, dtype=np.int64)).to(dev)])
    xb = {None: emb(blk), "st": emb(blk)}
    xp = {None: emb(prompt), "st": emb(prompt)} if caches is None else None
    k_last = None
    for l in range(ms.n_layers):
        lw = {n: host(t) for n, t in layers[l].items()}
        for key in (None, "st"):
            st = synth.round_bf16 if key else None
            if caches is None:
                q, k, v = O.layer_qkv(ms, lw, xp[key], np.arange(P), ident, st)
                xp[key] = O.layer_finish(ms, lw, xp[key], O.attention(q, k, v), ident, st)
                ck, cv = k, v
                if key and l == ms.n_layers - 1:
                    k_last = k
            else:
                ck, cv = caches[l]
            q, k, v = O.layer_qkv(ms, lw, xb[key], np.arange(Q) + P, ident, st)
            xb[key] = O.layer_finish(ms, lw, xb[key], O.attention(q, np.concatenate([ck, k]), np.concatenate([cv, v])),
                                     ident, st)
        del lw

    class Head:
        pass
    head = Head()
    head.ms = ms
    hw = {"final_norm": host(g["final_norm"]), "lm_head": host(g["lm_head"])}
    Head.__getitem__ = lambda self, k: hw[k]
    return {"exact": O.head_logits(head, xb[None], ident), "stored": O.head_logits(head, xb["st"], ident, synth.round_bf16),
            "k_last": k_last}
